"""CPU oracle for the AMS-Quant weight-only quantized Linear (arxiv 2510.16045).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow numpy/fp64
transcription of what the paper defines, written independently of the HIP
library in ``paper_2510_16045_amd``: the two share no code, no tables and no
helpers, and neither imports the other.  Only tests, the smoke check and the
``cpu_baseline`` leg of the benchmark may import this module.

Every function cites the passage of the paper it follows.  Where the paper is
silent the reading that was taken is stated in the docstring.

Conventions
-----------
* A *code* is the integer ``[S | E(2 bits) | M(m bits)]`` of one weight in the
  mini-float format e2m<m> (Sec. 2.2, Table 1): e2m3 has 6-bit codes, e2m2 has
  5-bit codes.  The *magnitude code* is the code without its sign bit.
* W is ``[N, K]`` (output channels x input channels), fp16.
* One scale per output channel (row), stored as fp16 (Sec. 3.1 "channel-wise").
* Mantissa sharing groups ``k`` consecutive weights along K (the input-channel
  dimension, Sec. 3.1 "Mantissa Sharing").

Pinned by tests/test_oracle_*.py (Table 1 values, closed forms, exhaustive
rounding against the definition, brute force over all shared-bit assignments,
round trips, k=1 reduction to plain RTN, numpy matmul; the re-rounding search
against the format with one mantissa bit less and a brute force over all code
tuples; scales per run of input channels against scalar arithmetic).  Not pinned: the bit
order inside the paper's packed words (its figures are not available); only
the word counts the paper states are asserted ("parity unpinned" for bit
order, which no result depends on).
"""

from __future__ import annotations

from dataclasses import dataclass

import numpy as np

EXP_BITS = 2
# Sec. 2.2 prints "bias = 2^e-1"; Table 1 lists bias 1 for E2M3 (and 3 for
# E3M2), so the superscript is read as 2^(e-1) - 1.
BIAS = 2 ** (EXP_BITS - 1) - 1


@dataclass(frozen=True)
class Format:
    """An FP(x-1).y format: e2m<mbits> codes, ``group`` weights share the LSB.

    Sec. 3.1: x = 1 + 2 + mbits bits per weight before sharing, y = 1/group.
    """

    name: str
    mbits: int
    group: int

    @property
    def code_bits(self) -> int:
        return 1 + EXP_BITS + self.mbits

    @property
    def n_mag(self) -> int:
        return 1 << (EXP_BITS + self.mbits)

    @property
    def bits_per_weight(self) -> float:
        return (self.code_bits - 1) + 1.0 / self.group


FP533 = Format("fp5.33-e2m3", 3, 3)  # abstract; Sec. 3.3 item 1
FP425 = Format("fp4.25-e2m2", 2, 4)  # abstract; Sec. 3.2
# plain RTN formats = group size 1 (Sec. 2.1); other shared formats of Sec. 4.1
FP6_E2M3 = Format("fp6-e2m3", 3, 1)
FP5_E2M2 = Format("fp5-e2m2", 2, 1)
FP4_E2M1 = Format("fp4-e2m1", 1, 1)
FP45 = Format("fp4.5-e2m2", 2, 2)
FP433 = Format("fp4.33-e2m2", 2, 3)

FORMATS = {f.name: f for f in (FP533, FP425, FP6_E2M3, FP5_E2M2, FP4_E2M1, FP45, FP433)}


# --------------------------------------------------------------------------
# Sec. 2.2: value of a code
# --------------------------------------------------------------------------
def magnitude_of(mag_code: int, mbits: int) -> float:
    """Value of one magnitude code, by the two-branch formula of Sec. 2.2.

    E != 0:  2^(E-bias) * (1 + sum_i d_i / 2^i)
    E == 0:  2^(1-bias) * (    sum_i d_i / 2^i)
    The all-ones exponent is an ordinary value (no inf / NaN), Sec. 2.2.
    """
    e = mag_code >> mbits
    frac = 0.0
    for i in range(1, mbits + 1):
        d_i = (mag_code >> (mbits - i)) & 1
        frac += d_i / (2.0**i)
    if e != 0:
        return 2.0 ** (e - BIAS) * (1.0 + frac)
    return 2.0 ** (1 - BIAS) * frac


def magnitude_table(fmt: Format) -> np.ndarray:
    """All magnitudes of the format, indexed by magnitude code (fp64)."""
    return np.array([magnitude_of(c, fmt.mbits) for c in range(fmt.n_mag)], dtype=np.float64)


def format_max(fmt: Format) -> float:
    """Largest representable magnitude ("M" of Eq. 1)."""
    return float(magnitude_table(fmt)[-1])


def decode(codes: np.ndarray, fmt: Format) -> np.ndarray:
    """Signed fp64 value of full codes (sign bit on top), Sec. 2.2.

    A set sign bit on a zero magnitude gives -0.0.
    """
    codes = np.asarray(codes).astype(np.int64)
    sign_bit = EXP_BITS + fmt.mbits
    mag = magnitude_table(fmt)[codes & (fmt.n_mag - 1)]
    return np.where((codes >> sign_bit) & 1 == 1, -mag, mag)


# --------------------------------------------------------------------------
# Eq. 1: scale and round-to-nearest
# --------------------------------------------------------------------------
def row_scales(W: np.ndarray, fmt: Format) -> np.ndarray:
    """Per-output-channel scale s = max|W| / M (Eq. 1), rounded to fp16.

    Reading where the paper is silent: the scale is stored as fp16 and the
    rounded scale is the one used to quantize, so encode and decode agree; a
    row whose scale would be zero (all-zero row, or absmax/M below the fp16
    range) or is not finite gets s = 1.
    """
    W = np.asarray(W)
    if W.dtype != np.float16:
        raise TypeError("W must be float16")
    if not np.all(np.isfinite(W)):
        raise ValueError("W holds inf or NaN")
    absmax = np.max(np.abs(W.astype(np.float64)), axis=1)
    s = (absmax / format_max(fmt)).astype(np.float16)
    s = np.where(s == 0, np.float16(1.0), s).astype(np.float16)
    return s


def rtn_magnitude_codes(a: np.ndarray, fmt: Format) -> np.ndarray:
    """Round(w) = argmin_alpha |w - alpha| over the format's magnitudes (Sec. 2.1).

    ``a`` holds non-negative fp64 magnitudes.  The definition is evaluated as
    written: the distance to every magnitude is formed and the smallest wins.
    Reading where the paper is silent: an exact tie between two neighbouring
    magnitudes goes to the one with the even magnitude code; inputs above the
    largest magnitude land on it (the argmin already does that).
    """
    a = np.asarray(a, dtype=np.float64)
    table = magnitude_table(fmt)
    dist = np.abs(a[..., None] - table)  # [..., n_mag]
    first = np.argmin(dist, axis=-1)
    last = (fmt.n_mag - 1) - np.argmin(dist[..., ::-1], axis=-1)
    # first != last only on an exact tie; the two are then neighbours
    return np.where(first % 2 == 0, first, last).astype(np.int64)


def rtn_codes(W: np.ndarray, s: np.ndarray, fmt: Format) -> np.ndarray:
    """Q(W) = Round(W / s) per row (Eq. 1) as full codes.

    The sign bit is 1 exactly when W < 0 (so -0.0 and +0.0 both get sign 0);
    W / s is an fp64 division of two fp16-exact numbers.
    """
    W64 = np.asarray(W).astype(np.float64)
    s64 = np.asarray(s).astype(np.float64)[:, None]
    t = W64 / s64
    mag = rtn_magnitude_codes(np.abs(t), fmt)
    sign = (W64 < 0).astype(np.int64)
    return (sign << (EXP_BITS + fmt.mbits)) | mag


# --------------------------------------------------------------------------
# Sec. 3.1: mantissa sharing + adaptive searching
# --------------------------------------------------------------------------
def set_last_bit(codes: np.ndarray, m0: int) -> np.ndarray:
    """G(FPx_i, m0): set the last mantissa bit of each code to m0 (Sec. 3.1)."""
    return (np.asarray(codes) & ~1) | m0


def reround_magnitude_codes(a: np.ndarray, fmt: Format, m0: int) -> np.ndarray:
    """Nearest magnitude among the codes whose last mantissa bit is m0.

    Not in the paper: the re-rounding variant of the search (see ams_quantize).
    The argmin of Sec. 2.1 restricted to every other code.  An exact tie goes to
    the code whose remaining bits (code >> 1) are even; inputs above the largest
    such magnitude land on it.
    """
    a = np.asarray(a, dtype=np.float64)
    table = magnitude_table(fmt)[m0::2]  # indexed by code >> 1
    dist = np.abs(a[..., None] - table)
    first = np.argmin(dist, axis=-1)
    last = (len(table) - 1) - np.argmin(dist[..., ::-1], axis=-1)
    upper = np.where(first % 2 == 0, first, last).astype(np.int64)
    return 2 * upper + m0


def tensor_scales(W: np.ndarray, fmt: Format) -> np.ndarray:
    """Per-tensor granularity (Sec. 5): Eq. 1 with the maximum taken over the whole
    matrix; returned once per row so that it can stand in for row_scales."""
    W = np.asarray(W)
    flat = row_scales(W.reshape(1, -1), fmt)
    return np.repeat(flat, W.shape[0])


def ams_quantize(W: np.ndarray, fmt: Format, chunk_rows: int = 64, search: str = "set", per_tensor: bool = False):
    """Channel-wise RTN, grouping along K, adaptive search of the shared bit.

    Follows Sec. 3.1 in order: (1) RTN of every weight to FPx with one scale
    per output channel; (2) groups of ``fmt.group`` consecutive weights along
    the input-channel dimension; (3) for every group both values of the shared
    last mantissa bit are tried, every member's last bit is set to it, and the
    value with the smaller sum of squared differences between the dequantized
    (Eq. 2) and the original weights is kept.

    Readings where the paper is silent:
    * the upper bits of each code stay those of its plain RTN code;
    * the squared errors are fp64, added in member order, and a tie keeps 0;
    * when K is not a multiple of the group size the last group is shorter:
      only its real members enter the sum (padding is never an output).

    ``per_tensor=True`` uses one scale for the whole matrix (the coarsest
    granularity Sec. 5 names) instead of one per output channel.

    ``search="reround"`` is a variant that is NOT in the paper: for each value
    of the shared bit every member is re-rounded to the nearest code that ends
    in that bit (instead of keeping the upper bits of its RTN code); the rest
    (squared errors, order, tie) is as above.  Its error can only be smaller.

    Returns (codes [N,K] int64 full codes whose LSB is the group's shared bit,
             scales [N] float16, shared [N, ceil(K/group)] uint8).
    """
    if search not in ("set", "reround"):
        raise ValueError(search)
    W = np.asarray(W)
    N, K = W.shape
    g = fmt.group
    n_groups = -(-K // g)
    s = tensor_scales(W, fmt) if per_tensor else row_scales(W, fmt)
    codes = np.empty((N, K), dtype=np.int64)
    shared = np.empty((N, n_groups), dtype=np.uint8)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        Wc = W[r0:r1]
        sc = s[r0:r1]
        c_rtn = rtn_codes(Wc, sc, fmt)
        W64 = Wc.astype(np.float64)
        s64 = sc.astype(np.float64)[:, None]
        sq, cand = [], []
        for m0 in (0, 1):
            if search == "set":
                c_m0 = set_last_bit(c_rtn, m0)  # G(FPx_i, m0)
            else:
                sign = (W64 < 0).astype(np.int64) << (EXP_BITS + fmt.mbits)
                c_m0 = sign | reround_magnitude_codes(np.abs(W64 / s64), fmt, m0)
            cand.append(c_m0)
            deq = decode(c_m0, fmt) * s64  # Eq. 2
            sq.append((deq - W64) ** 2)
        sse = [np.zeros((r1 - r0, n_groups)), np.zeros((r1 - r0, n_groups))]
        for j in range(g):  # member order; a short last group has fewer members
            cols = np.arange(j, K, g)
            for m0 in (0, 1):
                sse[m0][:, : len(cols)] = sse[m0][:, : len(cols)] + sq[m0][:, cols]
        pick = (sse[1] < sse[0]).astype(np.int64)  # tie keeps 0
        shared[r0:r1] = pick
        per_weight = np.repeat(pick, g, axis=1)[:, :K]
        codes[r0:r1] = np.where(per_weight == 1, cand[1], cand[0])
    return codes, s, shared


# --------------------------------------------------------------------------
# Sec. 3.2 / 3.3 item 1: the paper's packed words (canonical layout)
# --------------------------------------------------------------------------
def canonical_packed_bytes(fmt: Format, N: int, K: int) -> int:
    """Bytes of the paper's packing: one uint16 per 3 weights for FP5.33
    (Sec. 3.3 item 1), 17 uint16 per 64 weights for FP4.25 (Sec. 3.2)."""
    if fmt == FP533:
        return 2 * (-(-K // 3)) * N
    if fmt == FP425:
        return 2 * 17 * (-(-K // 64)) * N
    raise NotImplementedError(fmt.name)


def pack_canonical(codes: np.ndarray, fmt: Format) -> np.ndarray:
    """Pack final codes (LSB already equal within each group) into uint16 words.

    FP5.33 (Sec. 3.3 item 1): the three 5-bit remainders of a group and its
    shared bit fill one half-word.  FP4.25 (Sec. 3.2): per 64 weights, 16 words
    of 4-bit remainders followed by one word of the 16 shared bits.
    Bit order is not given by the paper (figure unavailable); taken here:
    FP5.33 word = rem0 | rem1<<5 | rem2<<10 | shared<<15; FP4.25 word g of a
    block = rem(4g+j) << 4j for j=0..3, word 16 bit g = shared bit of group g.
    Missing weights at the end of a row are stored as zero remainders.
    Returns uint16 [N, words_per_row].
    """
    codes = np.asarray(codes).astype(np.int64)
    N, K = codes.shape
    g = fmt.group
    Kp = -(-K // g) * g
    padded = np.zeros((N, Kp), dtype=np.int64)
    padded[:, :K] = codes
    grp = padded.reshape(N, Kp // g, g)
    lsb = grp & 1
    real = np.zeros((N, Kp), dtype=bool)
    real[:, :K] = True
    real = real.reshape(N, Kp // g, g)
    # all real members of a group must carry the same last bit
    first = lsb[:, :, :1]
    if np.any((lsb != first) & real):
        raise ValueError("codes of one group disagree in their shared bit")
    shared = lsb[:, :, 0]
    rem = grp >> 1
    if fmt == FP533:
        words = rem[:, :, 0] | (rem[:, :, 1] << 5) | (rem[:, :, 2] << 10) | (shared << 15)
        return words.astype(np.uint16)
    if fmt == FP425:
        n_groups = Kp // g
        n_blocks = -(-n_groups // 16)
        rem_b = np.zeros((N, n_blocks * 16, 4), dtype=np.int64)
        rem_b[:, :n_groups] = rem
        sh_b = np.zeros((N, n_blocks * 16), dtype=np.int64)
        sh_b[:, :n_groups] = shared
        nib = rem_b[:, :, 0] | (rem_b[:, :, 1] << 4) | (rem_b[:, :, 2] << 8) | (rem_b[:, :, 3] << 12)
        nib = nib.reshape(N, n_blocks, 16)
        shw = (sh_b.reshape(N, n_blocks, 16) << np.arange(16)).sum(axis=2, keepdims=True)
        return np.concatenate([nib, shw], axis=2).reshape(N, n_blocks * 17).astype(np.uint16)
    raise NotImplementedError(fmt.name)


def unpack_canonical(words: np.ndarray, fmt: Format, K: int) -> np.ndarray:
    """Inverse of :func:`pack_canonical`: uint16 words -> full codes [N,K].

    This is the bit-level restoration of Sec. 3.2 up to the code: shift and
    mask the remainder out of its word, OR the group's shared bit in as LSB.
    """
    words = np.asarray(words).astype(np.int64)
    N = words.shape[0]
    if fmt == FP533:
        n_groups = words.shape[1]
        sh = (words >> 15) & 1
        out = np.empty((N, n_groups, 3), dtype=np.int64)
        for j in range(3):
            out[:, :, j] = (((words >> (5 * j)) & 0x1F) << 1) | sh
        return out.reshape(N, n_groups * 3)[:, :K]
    if fmt == FP425:
        blocks = words.reshape(N, -1, 17)
        nib = blocks[:, :, :16]
        shw = blocks[:, :, 16]
        out = np.empty((N, blocks.shape[1], 16, 4), dtype=np.int64)
        for gidx in range(16):
            sh = (shw >> gidx) & 1
            for j in range(4):
                out[:, :, gidx, j] = (((nib[:, :, gidx] >> (4 * j)) & 0xF) << 1) | sh
        return out.reshape(N, -1)[:, :K]
    raise NotImplementedError(fmt.name)


# --------------------------------------------------------------------------
# Eq. 2: dequantization; the Linear
# --------------------------------------------------------------------------
def dequant_unscaled(codes: np.ndarray, fmt: Format) -> np.ndarray:
    """The restored FPx value of each code as fp16 (always exact), Sec. 3.2."""
    return decode(codes, fmt).astype(np.float16)


def per_weight_scales(s: np.ndarray, K: int, scale_group: int | None = None) -> np.ndarray:
    """The scale of every weight as fp64 [N, K]: one per row (s is [N]) or one per
    run of ``scale_group`` input channels of a row (s is [N, ceil(K / scale_group)])."""
    s64 = np.asarray(s).astype(np.float64)
    if s64.ndim == 1:
        return np.repeat(s64[:, None], K, axis=1)
    if scale_group is None or s64.shape[1] != -(-K // scale_group):
        raise ValueError("grouped scales need the matching scale_group")
    return np.repeat(s64, scale_group, axis=1)[:, :K]


def dequant_real(codes: np.ndarray, s: np.ndarray, fmt: Format, scale_group: int | None = None) -> np.ndarray:
    """DeQ(W) = Q(W) * s (Eq. 2) in fp64, unrounded (the product is exact)."""
    codes = np.asarray(codes)
    return decode(codes, fmt) * per_weight_scales(s, codes.shape[1], scale_group)


def dequant_scaled(codes: np.ndarray, s: np.ndarray, fmt: Format, scale_group: int | None = None) -> np.ndarray:
    """Eq. 2 rounded once to fp16 (round-to-nearest-even, subnormals kept)."""
    return dequant_real(codes, s, fmt, scale_group).astype(np.float16)


def linear(codes: np.ndarray, s: np.ndarray, X: np.ndarray, fmt: Format, scale_group: int | None = None) -> np.ndarray:
    """Y[m,n] = sum_k DeQ(W)[n,k] * X[m,k] in fp64 (Eq. 2 then a plain matmul).

    X is the fp16 activation matrix [M,K] widened to fp64.
    """
    X64 = np.asarray(X).astype(np.float64)
    return X64 @ dequant_real(codes, s, fmt, scale_group).T


def ams_quantize_grouped(W: np.ndarray, fmt: Format, scale_group: int, search: str = "set"):
    """AMS quantization with one scale per run of ``scale_group`` input channels of a row.

    Sec. 5 states that the method works at any granularity "from per-tensor and
    per-channel to per-group"; only per-channel is spelled out (Sec. 3.1).  The
    reading taken: Eq. 1 is applied to every run of ``scale_group`` consecutive
    input channels of a row by itself (its own max |W| / M, rounded to fp16), the
    sharing groups and the search stay inside a run (``scale_group`` must be a
    multiple of the sharing group size), and everything else is as ams_quantize.
    So the result is the per-channel method applied to each column block alone.

    Returns (codes [N,K], scales [N, ceil(K/scale_group)] float16).
    """
    W = np.asarray(W)
    N, K = W.shape
    if scale_group <= 0 or scale_group % fmt.group != 0:
        raise ValueError("scale_group must be a positive multiple of the sharing group size")
    codes = np.empty((N, K), dtype=np.int64)
    n_sg = -(-K // scale_group)
    scales = np.empty((N, n_sg), dtype=np.float16)
    for j in range(n_sg):
        block = slice(j * scale_group, min(K, (j + 1) * scale_group))
        c, s, _ = ams_quantize(np.ascontiguousarray(W[:, block]), fmt, search=search)
        codes[:, block] = c
        scales[:, j] = s
    return codes, scales


def fp16_linear(W: np.ndarray, X: np.ndarray) -> np.ndarray:
    """The unquantized Linear Y = X W^T in fp64 (the W16A16 baseline of Sec. 4.2)."""
    return np.asarray(X).astype(np.float64) @ np.asarray(W).astype(np.float64).T


def weight_mse(W: np.ndarray, fmt: Format) -> float:
    """Mean squared error between DeQ(Q(W)) and W (the search objective, Sec. 3.1)."""
    codes, s, _ = ams_quantize(W, fmt)
    d = dequant_real(codes, s, fmt) - np.asarray(W).astype(np.float64)
    return float(np.mean(d * d))
