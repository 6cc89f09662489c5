"""Pins for the CPU oracle: each test checks oracle/ams_oracle.py against something
other than itself -- values the paper prints (Table 1), closed forms, numpy's own
fp16 decoder and rounding, hand-worked groups, brute force over every shared-bit
assignment, round trips and invariants.  No GPU, no HIP library.
"""

import itertools
import os

import numpy as np
import pytest

from oracle import ams_oracle as O
from paper_2510_16045_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
AMS = [O.FP533, O.FP425]


def _all_finite_fp16():
    bits = np.arange(1 << 16, dtype=np.uint16)
    v = bits.view(np.float16)
    return v[np.isfinite(v)]


# ---------------------------------------------------------------- P1: decode
def test_table1_e2m3_extremes():
    want = {}
    for line in open(os.path.join(GOLDEN, "table1_e2m3.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        want[k] = float(v)
    assert O.BIAS == want["exponent_bias"]
    t = O.magnitude_table(O.FP533)
    assert t.max() == want["max_normal"]
    assert t[1 << 3] == want["min_normal"]  # E=1, M=0
    assert t[(1 << 3) - 1] == want["max_subnormal"]  # E=0, M=111
    assert t[1] == want["min_subnormal"]


def test_value_sets_closed_form():
    e2m3 = [i / 8 for i in range(16)] + [2 + i / 4 for i in range(8)] + [4 + i / 2 for i in range(8)]
    e2m2 = [i / 4 for i in range(8)] + [2 + i / 2 for i in range(4)] + [4.0 + i for i in range(4)]
    e2m1 = [0, 0.5, 1, 1.5, 2, 3, 4, 6]
    assert O.magnitude_table(O.FP533).tolist() == e2m3
    assert O.magnitude_table(O.FP425).tolist() == e2m2
    assert O.magnitude_table(O.FP4_E2M1).tolist() == e2m1
    # e2m2 is e2m3 with the last mantissa bit clear; no inf/NaN anywhere
    assert O.magnitude_table(O.FP533)[0::2].tolist() == e2m2
    for f in O.FORMATS.values():
        assert np.all(np.isfinite(O.magnitude_table(f)))
        assert np.all(np.diff(O.magnitude_table(f)) > 0)


@pytest.mark.parametrize("fmt", AMS)
def test_decode_matches_numpy_fp16_bit_view(fmt):
    # a bias-1 e2mX code placed at the top of fp16's exponent/mantissa fields is the
    # same number times 2^-14 (fp16 bias 15); numpy's fp16 decoder is the referee
    codes = np.arange(1 << fmt.code_bits)
    sign = codes >> (fmt.code_bits - 1)
    mag = codes & (fmt.n_mag - 1)
    bits = ((sign << 15) | (mag << (10 - fmt.mbits))).astype(np.uint16)
    via_fp16 = bits.view(np.float16).astype(np.float64) * 2.0**14
    got = O.decode(codes, fmt)
    assert np.array_equal(got, via_fp16)
    assert np.array_equal(np.signbit(got), sign == 1)  # -0.0 for (S=1, mag 0)


# ---------------------------------------------------------------- P2/P3: RTN
@pytest.mark.parametrize("fmt", AMS + [O.FP4_E2M1])
def test_encode_of_decode_is_identity(fmt):
    mags = O.magnitude_table(fmt)
    assert np.array_equal(O.rtn_magnitude_codes(mags, fmt), np.arange(fmt.n_mag))


def _rne_on_grid(a, mbits):
    """Textbook round-half-even onto the e2m<mbits> grid via numpy's round()."""
    a = np.asarray(a, dtype=np.float64)
    e = np.floor(np.log2(np.maximum(a, 1.0)))  # below 1 the grid is the subnormal one
    e = np.minimum(e, 2.0)
    step = 2.0**e / (1 << mbits)
    fmax = 2.0**2 * (2 - 2.0**-mbits)
    return np.minimum(np.round(a / step) * step, fmax)


@pytest.mark.parametrize("fmt", AMS)
@pytest.mark.parametrize("scale", [1.0, 0.5, 3.0, 0.0123])
def test_rtn_exhaustive_against_textbook_rounding(fmt, scale):
    v = _all_finite_fp16()
    v = np.sort(v[~np.signbit(v)].astype(np.float64))
    t = v / scale
    codes = O.rtn_magnitude_codes(t, fmt)
    got = O.magnitude_table(fmt)[codes]
    assert np.array_equal(got, _rne_on_grid(t, fmt.mbits))
    assert np.all(np.diff(codes) >= 0)  # monotone
    inside = t <= O.format_max(fmt)
    table = O.magnitude_table(fmt)
    lo = table[np.maximum(codes - 1, 0)]
    hi = table[np.minimum(codes + 1, fmt.n_mag - 1)]
    half = np.maximum(got - lo, hi - got) / 2
    assert np.all(np.abs(got - t)[inside] <= half[inside])
    assert np.all(codes[~inside] == fmt.n_mag - 1)  # saturation


@pytest.mark.parametrize("fmt", AMS)
def test_rtn_ties_go_to_even_code(fmt):
    table = O.magnitude_table(fmt)
    mids = (table[:-1] + table[1:]) / 2
    codes = O.rtn_magnitude_codes(mids, fmt)
    lower = np.arange(fmt.n_mag - 1)
    want = np.where(lower % 2 == 0, lower, lower + 1)
    assert np.array_equal(codes, want)


def test_sign_rule():
    W = np.array([[-0.0, 0.0, -1e-4, 1e-4, -7.5, 7.5]], dtype=np.float16)
    s = np.array([1.0], dtype=np.float16)
    c = O.rtn_codes(W, s, O.FP533)
    assert (c >> 5).tolist() == [[0, 0, 1, 0, 1, 0]]
    assert (c & 31).tolist() == [[0, 0, 0, 0, 31, 31]]


# ---------------------------------------------------------------- P4: scale
@pytest.mark.parametrize("fmt", AMS)
def test_scale_and_absmax(fmt):
    W = synth.gaussian_weights(64, 200, 7)
    s = O.row_scales(W, fmt)
    absmax = np.abs(W.astype(np.float64)).max(axis=1)
    assert s.dtype == np.float16
    assert np.array_equal(s, (absmax / O.format_max(fmt)).astype(np.float16))
    c = O.rtn_codes(W, s, fmt)
    j = np.abs(W.astype(np.float64)).argmax(axis=1)
    assert np.all((c[np.arange(64), j] & (fmt.n_mag - 1)) == fmt.n_mag - 1)


def test_degenerate_rows():
    W = np.zeros((3, 12), dtype=np.float16)
    W[1, 5] = np.float16(6e-8)  # absmax/7.5 underflows fp16 -> s = 1
    W[2, :] = np.float16(-3.0)
    for fmt in AMS:
        codes, s, _ = O.ams_quantize(W, fmt)
        assert s[0] == 1.0 and s[1] == 1.0
        assert np.all(codes[0] == 0)
        assert np.all(O.dequant_scaled(codes, s, fmt)[2] == np.float16(-3.0))
    with pytest.raises(ValueError):
        O.row_scales(np.array([[np.inf, 1.0]], dtype=np.float16), O.FP533)


# ---------------------------------------------------------------- P5-P7: search
def test_group_size_one_is_plain_rtn():
    W = synth.gaussian_weights(16, 96, 3)
    for fmt in (O.FP6_E2M3, O.FP5_E2M2):
        codes, s, shared = O.ams_quantize(W, fmt)
        assert np.array_equal(codes, O.rtn_codes(W, s, fmt))
        assert np.array_equal(shared, codes & 1)


@pytest.mark.parametrize("fmt", AMS + [O.FP45, O.FP433])
@pytest.mark.parametrize("K", [96, 100, 13])
def test_search_invariants(fmt, K):
    W = synth.gaussian_weights(48, K, 11 + K)
    codes, s, shared = O.ams_quantize(W, fmt)
    g = fmt.group
    rtn = O.rtn_codes(W, s, fmt)
    W64 = W.astype(np.float64)
    # sharing runs along K: every group's members end with the same last bit
    assert np.array_equal(codes & 1, np.repeat(shared, g, axis=1)[:, :K])
    assert np.array_equal(codes >> 1, rtn >> 1)  # upper bits untouched
    n_groups = -(-K // g)
    same = 0
    for n in range(W.shape[0]):
        for gi in range(n_groups):
            sl = slice(gi * g, min(K, gi * g + g))
            e = lambda c: float(np.sum((O.decode(c, fmt) * float(s[n]) - W64[n, sl]) ** 2))
            e_rtn, e_ams = e(rtn[n, sl]), e(codes[n, sl])
            e0, e1 = e(O.set_last_bit(rtn[n, sl], 0)), e(O.set_last_bit(rtn[n, sl], 1))
            assert e_rtn <= e_ams + 1e-30
            assert abs(e_ams - min(e0, e1)) <= 1e-12 * max(e_ams, 1e-30)
            if len(set((rtn[n, sl] & 1).tolist())) == 1:
                same += 1
                assert np.array_equal(codes[n, sl], rtn[n, sl])
    if K == 96:  # about 2^(1-g) of random groups already agree
        frac = same / (W.shape[0] * n_groups)
        assert 0.5 * 2.0 ** (1 - g) < frac < 2.0 * 2.0 ** (1 - g)


@pytest.mark.parametrize("fmt", AMS)
def test_search_is_globally_optimal_on_tiny_matrices(fmt):
    # enumerate every assignment of shared bits; scalar arithmetic only
    W = synth.gaussian_weights(2, 4 * fmt.group - 1, 5)  # ragged last group
    codes, s, shared = O.ams_quantize(W, fmt)
    rtn = O.rtn_codes(W, s, fmt)
    g, K = fmt.group, W.shape[1]
    n_groups = -(-K // g)
    sign_bit = fmt.code_bits - 1
    for n in range(2):
        best = None
        for assign in itertools.product((0, 1), repeat=n_groups):
            tot = 0.0
            for k in range(K):
                c = (int(rtn[n, k]) & ~1) | assign[k // g]
                v = O.magnitude_of(c & (fmt.n_mag - 1), fmt.mbits)
                v = -v if (c >> sign_bit) & 1 else v
                tot += (v * float(s[n]) - float(W[n, k])) ** 2
            if best is None or tot < best[0] - 1e-18:
                best = (tot, assign)
        mine = float(np.sum((O.dequant_real(codes, s, fmt)[n] - W[n].astype(np.float64)) ** 2))
        assert abs(mine - best[0]) <= 1e-12 * best[0]


# ---- the re-rounding variant of the search (not in the paper) ---------------------------------
@pytest.mark.parametrize("big,small", [(O.FP6_E2M3, O.FP5_E2M2), (O.FP5_E2M2, O.FP4_E2M1)])
def test_reround_to_bit_zero_is_rtn_of_the_format_with_one_bit_less(big, small):
    # the codes ending in 0 are the value set of the format with one mantissa bit less
    # (test_value_sets_closed_form), so re-rounding to them is that format's plain RTN
    a = np.abs(np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64))
    for scale in (1.0, 0.37, 3.0):
        assert np.array_equal(O.reround_magnitude_codes(a / scale, big, 0) >> 1, O.rtn_magnitude_codes(a / scale, small))


@pytest.mark.parametrize("fmt", [O.FP6_E2M3, O.FP5_E2M2])
def test_reround_to_bit_one_is_nearest_and_ties_follow_the_rule(fmt):
    odd = O.magnitude_table(fmt)[1::2]
    a = np.abs(np.arange(0, 0x4900, dtype=np.uint16).view(np.float16).astype(np.float64))  # 0 .. 10
    got = O.reround_magnitude_codes(a, fmt, 1)
    assert np.all(got & 1 == 1)
    for x, c in zip(a.tolist(), got.tolist()):  # scalar brute force, the definition
        d = [abs(x - v) for v in odd.tolist()]
        assert d[c >> 1] == min(d)
    mids = (odd[:-1] + odd[1:]) / 2  # exact ties: the even one of the two upper parts wins
    tie = O.reround_magnitude_codes(mids, fmt, 1) >> 1
    assert np.all(tie % 2 == 0) and np.all((tie == np.arange(len(mids))) | (tie == np.arange(len(mids)) + 1))
    assert O.reround_magnitude_codes(np.array([1e9]), fmt, 1)[0] == fmt.n_mag - 1  # saturates


@pytest.mark.parametrize("fmt", AMS + [O.FP45, O.FP433])
def test_reround_search_invariants(fmt):
    K = 100
    W = synth.gaussian_weights(32, K, 77)
    c_set, s, _ = O.ams_quantize(W, fmt)
    c_rr, s_rr, shared = O.ams_quantize(W, fmt, search="reround")
    assert np.array_equal(s, s_rr)
    g = fmt.group
    assert np.array_equal(c_rr & 1, np.repeat(shared, g, axis=1)[:, :K])
    sign_bit = fmt.code_bits - 1
    assert np.array_equal(c_rr >> sign_bit, (W < 0).astype(np.int64))
    W64 = W.astype(np.float64)
    one_less = O.Format("one-less", fmt.mbits - 1, 1)
    t = np.abs(W64 / s.astype(np.float64)[:, None])
    c_low = ((W < 0).astype(np.int64) << sign_bit) | (O.rtn_magnitude_codes(t, one_less) << 1)
    err = lambda c: (O.decode(c, fmt) * s.astype(np.float64)[:, None] - W64) ** 2
    e_rr, e_set, e_low = err(c_rr), err(c_set), err(c_low)
    strictly = 0
    for gi in range(-(-K // g)):
        sl = slice(gi * g, min(K, gi * g + g))
        a, b, c = e_rr[:, sl].sum(1), e_set[:, sl].sum(1), e_low[:, sl].sum(1)
        assert np.all(a <= b * (1 + 1e-12) + 1e-30)  # never worse than setting the bit
        assert np.all(a <= c * (1 + 1e-12) + 1e-30)  # never worse than plain RTN with one bit less
        strictly += int(np.sum(a < b * (1 - 1e-9)))
    assert strictly > 0  # and it does help somewhere


@pytest.mark.parametrize("fmt", AMS)
def test_reround_search_is_optimal_over_all_codes_with_a_common_last_bit(fmt):
    # brute force: every tuple of codes of a group that ends in the same bit (scalar arithmetic)
    W = synth.gaussian_weights(3, 2 * fmt.group + 1, 9)
    codes, s, _ = O.ams_quantize(W, fmt, search="reround")
    g, K = fmt.group, W.shape[1]
    mags = [O.magnitude_of(c, fmt.mbits) for c in range(fmt.n_mag)]
    for n in range(W.shape[0]):
        sc = float(s[n])
        for k0 in range(0, K, g):
            ws = [float(W[n, k]) for k in range(k0, min(K, k0 + g))]
            best = None
            for m0 in (0, 1):
                cand = [c for c in range(fmt.n_mag) if c & 1 == m0]
                for tup in itertools.product(cand, repeat=len(ws)):
                    # the sign is fixed by the weight, so only magnitudes are enumerated
                    tot = 0.0
                    for w, c in zip(ws, tup):
                        v = -mags[c] if w < 0 else mags[c]
                        tot += (v * sc - w) ** 2
                    if best is None or tot < best:
                        best = tot
            mine = 0.0
            for w, c in zip(ws, codes[n, k0 : k0 + g].tolist()):
                v = mags[c & (fmt.n_mag - 1)]
                mine += ((-v if w < 0 else v) * sc - w) ** 2
            assert abs(mine - best) <= 1e-12 * max(best, 1e-300)


# ---- one scale per run of input channels (Sec. 5: "any granularity") ---------------------------
@pytest.mark.parametrize("fmt", AMS + [O.FP45, O.FP433, O.FP6_E2M3])
def test_grouped_scales_definition(fmt):
    N, K, sg = 5, 100, 12 * fmt.group
    W = synth.heavy_tail_weights(N, K, 91)
    codes, s = O.ams_quantize_grouped(W, fmt, sg)
    n_sg = -(-K // sg)
    assert s.shape == (N, n_sg) and codes.shape == (N, K)
    W64 = W.astype(np.float64)
    fmax = O.format_max(fmt)
    for n in range(N):
        for j in range(n_sg):
            blk = W64[n, j * sg : (j + 1) * sg]
            want = np.float16(np.max(np.abs(blk)) / fmax)  # Eq. 1 on the run alone
            assert s[n, j] == (want if want != 0 else np.float16(1.0))
    # sharing groups stay inside a run and still agree in their last bit
    g = fmt.group
    for k0 in range(0, K, g):
        assert np.all((codes[:, k0 : k0 + g] & 1) == (codes[:, k0 : k0 + 1] & 1))
    # Eq. 2 with the run's scale, scalar arithmetic
    deq = O.dequant_real(codes, s, fmt, sg)
    sign_bit = fmt.code_bits - 1
    for n in range(N):
        for k in range(K):
            c = int(codes[n, k])
            v = O.magnitude_of(c & (fmt.n_mag - 1), fmt.mbits)
            v = -v if (c >> sign_bit) & 1 else v
            assert deq[n, k] == v * float(s[n, k // sg])
    # and a plain matmul on top of it
    X = synth.activations(3, K, 92)
    Y = O.linear(codes, s, X, fmt, sg)
    for m in range(3):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += deq[n, k] * float(X[m, k])
            assert abs(Y[m, n] - acc) <= 1e-12 * max(1.0, abs(acc))


@pytest.mark.parametrize("fmt", AMS)
def test_grouped_scales_reduce_to_per_channel_and_help_on_heavy_tails(fmt):
    W = synth.heavy_tail_weights(16, 768, 93)
    c_row, s_row, _ = O.ams_quantize(W, fmt)
    c_one, s_one = O.ams_quantize_grouped(W, fmt, 768)  # one run = the whole row
    assert np.array_equal(c_row, c_one) and np.array_equal(s_row, s_one[:, 0])
    c_big, s_big = O.ams_quantize_grouped(W, fmt, 1200)  # a run longer than the row
    assert np.array_equal(c_row, c_big) and np.array_equal(s_row, s_big[:, 0])
    W64 = W.astype(np.float64)
    mse = lambda c, s_, sg: float(np.mean((O.dequant_real(c, s_, fmt, sg) - W64) ** 2))
    c96, s96 = O.ams_quantize_grouped(W, fmt, 96)
    assert mse(c96, s96, 96) < mse(c_row, s_row, None)
    with pytest.raises(ValueError):
        O.ams_quantize_grouped(W, fmt, fmt.group + 1)
    with pytest.raises(ValueError):
        O.dequant_real(c96, s96, fmt, 128)


@pytest.mark.parametrize("fmt", AMS)
def test_per_tensor_scale_is_per_channel_on_the_flattened_matrix(fmt):
    # with K a multiple of the group size the groups of the flattened matrix are the same groups
    N, K = 6, 24 * fmt.group
    W = synth.heavy_tail_weights(N, K, 94)
    codes, s, shared = O.ams_quantize(W, fmt, per_tensor=True)
    c1, s1, _ = O.ams_quantize(W.reshape(1, -1), fmt)
    assert np.all(s == s1[0]) and s.shape == (N,)
    assert s1[0] == np.float16(np.max(np.abs(W.astype(np.float64))) / O.format_max(fmt))
    assert np.array_equal(codes, c1.reshape(N, K))


def test_worked_groups_fixture():
    names = {"fp4.25": O.FP425, "fp5.33": O.FP533}
    n = 0
    for line in open(os.path.join(GOLDEN, "worked_groups.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f, w, sh, dq = [p.strip() for p in line.split("|")]
        fmt = names[f]
        W = np.array([[float(x) for x in w.split()]], dtype=np.float16)
        codes, s, shared = O.ams_quantize(W, fmt)
        assert s[0] == 1.0
        assert shared[0].tolist() == [int(x) for x in sh.split()]
        assert O.dequant_scaled(codes, s, fmt)[0].astype(np.float64).tolist() == [float(x) for x in dq.split()]
        n += 1
    assert n == 5


def test_search_tie_keeps_zero():
    # +-(midpoint) members: setting the bit to 0 or 1 costs the same -> 0
    # e2m3 with s = 1: 0.0625 lies midway between 0 and 0.125
    W2 = np.array([[7.5, 7.0, 0.0625, 0.0625]], dtype=np.float16)
    codes, s, shared = O.ams_quantize(W2, O.Format("t2", 3, 2))
    assert s[0] == 1.0 and shared[0].tolist() == [0, 0] and codes[0].tolist() == [30, 30, 0, 0]


# ---------------------------------------------------------------- P8: packing
@pytest.mark.parametrize("fmt", AMS)
@pytest.mark.parametrize("K", [1, 3, 64, 100, 768, 4096])
def test_pack_roundtrip_and_sizes(fmt, K):
    rng = np.random.default_rng(K)
    N, g = 5, fmt.group
    n_groups = -(-K // g)
    rem = rng.integers(0, 1 << (fmt.code_bits - 1), size=(N, K))
    sh = rng.integers(0, 2, size=(N, n_groups))
    codes = (rem << 1) | np.repeat(sh, g, axis=1)[:, :K]
    words = O.pack_canonical(codes, fmt)
    assert words.dtype == np.uint16
    assert words.nbytes == O.canonical_packed_bytes(fmt, N, K)
    assert np.array_equal(O.unpack_canonical(words, fmt, K), codes)
    if fmt == O.FP533:
        assert words.nbytes == 2 * (-(-K // 3)) * N  # one half-word per 3 weights
    else:
        assert words.nbytes == 34 * (-(-K // 64)) * N  # 17 half-words per 64 weights


def test_pack_rejects_inconsistent_group():
    codes = np.array([[1, 0, 1]])
    with pytest.raises(ValueError):
        O.pack_canonical(codes, O.FP533)


def test_storage_claims():
    # "FP5.3 ... reducing 66.7% storage" (introduction) and the bit-widths in the names
    assert abs((1 - O.FP533.bits_per_weight / 16) - 0.667) < 5e-4
    assert abs(O.FP533.bits_per_weight - 16 / 3) < 1e-12
    assert O.FP425.bits_per_weight == 4.25
    assert O.canonical_packed_bytes(O.FP533, 4096, 4096) == 11_190_272
    assert O.canonical_packed_bytes(O.FP425, 4096, 14336) == 31_195_136


# ---------------------------------------------------------------- P9: ordering
def test_weight_mse_ordering_follows_bit_width():
    # synthetic shadow of the accuracy ordering of Table 2 / the sweet-spot figure
    W = synth.gaussian_weights(64, 1536, 9)
    order = [O.FP6_E2M3, O.FP533, O.FP5_E2M2, O.FP45, O.FP433, O.FP425, O.FP4_E2M1]
    mse = [O.weight_mse(W, f) for f in order]
    assert all(a < b for a, b in zip(mse, mse[1:])), mse


# ---------------------------------------------------------------- P10/P11: dequant, Linear
@pytest.mark.parametrize("fmt", AMS)
def test_dequant_scaled_against_fp32_product(fmt):
    W = synth.heavy_tail_weights(32, 120, 4)
    codes, s, _ = O.ams_quantize(W, fmt)
    sign = codes >> (fmt.code_bits - 1)
    bits = ((sign << 15) | ((codes & (fmt.n_mag - 1)) << (10 - fmt.mbits))).astype(np.uint16)
    v32 = bits.view(np.float16).astype(np.float32) * np.float32(2.0**14)
    want = (v32 * s.astype(np.float32)[:, None]).astype(np.float16)  # exact product, one rounding
    got = O.dequant_scaled(codes, s, fmt)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    assert np.array_equal(O.dequant_unscaled(codes, fmt).astype(np.float32), v32)


@pytest.mark.parametrize("fmt", AMS)
def test_linear_is_a_plain_matmul(fmt):
    W, X = synth.gaussian_weights(40, 130, 6), synth.activations(3, 130, 6)
    codes, s, _ = O.ams_quantize(W, fmt)
    Y = O.linear(codes, s, X, fmt)
    D = O.dequant_real(codes, s, fmt)
    ref = np.zeros((3, 40))
    for m in range(3):
        for n in range(40):
            ref[m, n] = sum(float(D[n, k]) * float(X[m, k]) for k in range(130))
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-15)
    # one-hot activation picks out a single restored weight
    E = np.zeros((1, 130), dtype=np.float16)
    E[0, 77] = 1.0
    assert np.array_equal(O.linear(codes, s, E, fmt)[0], D[:, 77])
    # transposed-operand mistake would break this shape check
    assert Y.shape == (3, 40)


def test_fp16_linear_is_a_plain_matmul():
    # the checker of the fp16 baseline kernel, pinned by a scalar triple loop over exactly decoded binary16
    # inputs (fractions: no floating point in the decode), a one-hot row and a transposed-operand trap
    from fractions import Fraction

    def half_exact(h):  # IEEE binary16 bit pattern -> exact rational
        sgn, e, m = h >> 15, (h >> 10) & 31, h & 1023
        assert e != 31
        v = Fraction(m, 1 << 24) if e == 0 else Fraction(1024 + m, 1024) * Fraction(2) ** (e - 15)
        return -v if sgn else v

    W, X = synth.gaussian_weights(7, 33, 12), synth.activations(3, 33, 12)
    Y = O.fp16_linear(W, X)
    assert Y.shape == (3, 7) and Y.dtype == np.float64  # [M, N]: a transposed operand would give 7 x 3 or fail
    Wb, Xb = W.view(np.uint16), X.view(np.uint16)
    for m in range(3):
        for n in range(7):
            exact = sum(half_exact(int(Wb[n, k])) * half_exact(int(Xb[m, k])) for k in range(33))
            assert abs(Y[m, n] - float(exact)) <= 1e-13 * max(1.0, abs(float(exact))), (m, n)
    E = np.zeros((1, 33), dtype=np.float16)
    E[0, 20] = 2.0
    assert np.array_equal(O.fp16_linear(W, E)[0], 2.0 * W[:, 20].astype(np.float64))
    # rectangular identity-like weights: Y picks columns of X
    Wi = np.zeros((4, 33), dtype=np.float16)
    for n in range(4):
        Wi[n, 5 * n + 1] = 1.0
    assert np.array_equal(O.fp16_linear(Wi, X), X[:, [1, 6, 11, 16]].astype(np.float64))


def test_quantized_linear_is_close_to_fp16_linear():
    # the quantized Linear approximates the fp16 one; coarser format -> larger error
    W, X = synth.gaussian_weights(128, 768, 8), synth.activations(4, 768, 8)
    ref = O.fp16_linear(W, X)
    errs = []
    for fmt in (O.FP533, O.FP425):
        codes, s, _ = O.ams_quantize(W, fmt)
        Y = O.linear(codes, s, X, fmt)
        errs.append(np.linalg.norm(Y - ref) / np.linalg.norm(ref))
    assert errs[0] < errs[1] < 0.2
    assert errs[0] < 0.08
