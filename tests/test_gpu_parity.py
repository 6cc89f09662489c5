"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Restored weights must match bit for bit; Linear outputs must
be within relative L2 1e-3 and max |error| <= 2e-2 of the output rms (unit-scale outputs)."""

import numpy as np
import pytest

import paper_2510_16045_amd as ams
from oracle import ams_oracle as O
from paper_2510_16045_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

PAPER_PAIRS = [(ams.FP533, O.FP533), (ams.FP425, O.FP425)]  # the two formats the paper builds kernels for
PAIRS = PAPER_PAIRS + [(ams.FP45, O.FP45), (ams.FP433, O.FP433), (ams.FP6, O.FP6_E2M3), (ams.FP5, O.FP5_E2M2), (ams.FP4, O.FP4_E2M1)]
REL_L2_TOL = 1e-3
MAX_ABS_TOL = 2e-2  # relative to rms(Y_ref)


def dev(a: np.ndarray):
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


def host16(t) -> np.ndarray:
    return t.cpu().view(torch.int16).numpy().view(np.float16)


def check_linear(y_gpu: np.ndarray, ref: np.ndarray, what=""):
    y = y_gpu.astype(np.float64)
    rel = np.linalg.norm(y - ref) / max(np.linalg.norm(ref), 1e-300)
    rms = np.sqrt(np.mean(ref * ref))
    mx = np.max(np.abs(y - ref)) / max(rms, 1e-300)
    assert rel <= REL_L2_TOL, f"{what}: rel L2 {rel}"
    assert mx <= MAX_ABS_TOL, f"{what}: max abs / rms {mx}"


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_dequant_every_code_through_the_kernel(fmt, ofmt):
    # every remainder with both shared bits in every member position, over several records
    g, nrem = ofmt.group, 1 << (ofmt.code_bits - 1)
    rows = []
    for sh in (0, 1):
        for shift in range(g):
            rem = (np.arange(nrem * g) // 1 + shift * 7) % nrem
            rows.append(((rem << 1) | sh).astype(np.uint8))
    if g == 1:  # no sharing: every full code in every position of a lane chunk
        for shift in range(0, 33, 1):
            rows.append(((np.arange(nrem) * 2 + shift * 3 + (np.arange(nrem) // 3)) % (2 * nrem)).astype(np.uint8))
    codes = np.stack(rows)
    codes = np.tile(codes, (3, 2))[:, : codes.shape[1] * 2 - 5]  # ragged tail, several strips' worth of rows
    lsb = codes[:, ::g][:, : -(-codes.shape[1] // g)] & 1
    codes = ((codes >> 1) << 1) | np.repeat(lsb, g, axis=1)[:, : codes.shape[1]]
    N, K = codes.shape
    s = (np.linspace(0.001, 9.0, N)).astype(np.float16)
    wp = dev(ams.ams_pack_codes(fmt, codes))
    got_u = host16(ams.ams_dequant(fmt, wp, None, N, K, scaled=False))
    got_s = host16(ams.ams_dequant(fmt, wp, dev(s), N, K, scaled=True))
    assert np.array_equal(got_u.view(np.uint16), O.dequant_unscaled(codes, ofmt).view(np.uint16))
    assert np.array_equal(got_s.view(np.uint16), O.dequant_scaled(codes, s, ofmt).view(np.uint16))


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
@pytest.mark.parametrize(
    "maker,N,K",
    [(synth.gaussian_weights, 256, 768), (synth.gaussian_weights, 37, 1000), (synth.heavy_tail_weights, 80, 4100), (synth.gaussian_weights, 1, 3)],
)
def test_dequant_bit_exact(fmt, ofmt, maker, N, K):
    W = maker(N, K, 31)
    packed, scales = ams.ams_pack(fmt, W)
    codes, o_scales, _ = O.ams_quantize(W, ofmt)
    got = host16(ams.ams_dequant(fmt, dev(packed), dev(scales), N, K, scaled=True))
    assert np.array_equal(got.view(np.uint16), O.dequant_scaled(codes, o_scales, ofmt).view(np.uint16))
    got = host16(ams.ams_dequant(fmt, dev(packed), None, N, K, scaled=False))
    assert np.array_equal(got.view(np.uint16), O.dequant_unscaled(codes, ofmt).view(np.uint16))


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
@pytest.mark.parametrize(
    "N,K,Ms",
    [
        (256, 768, (1, 2, 3, 4, 8, 16, 17, 32)),  # baseline config 1 (+ batch sweep)
        (37, 1000, (1, 5, 32)),  # ragged strip, ragged record, ragged group
        (48, 14336, (1, 16)),  # long K: many records per wave
        (528, 4096, (1, 4, 32)),  # M=32 needs several activation phases
        (16, 5, (1,)),
        (70000, 64, (1, 7)),  # many strips, one record each: 18 strips per workgroup
        (64, 20000, (3, 17)),  # four strips, very long rows: K in many phases at M=17
    ],
)
def test_linear_matches_oracle(fmt, ofmt, N, K, Ms):
    W = synth.gaussian_weights(N, K, 41)
    packed, scales = ams.ams_pack(fmt, W)
    codes, o_scales, _ = O.ams_quantize(W, ofmt)
    wp, sc = dev(packed), dev(scales)
    for M in Ms:
        X = synth.activations(M, K, 41 + M)
        y = host16(ams.ams_linear(wp, sc, dev(X), N, fmt))
        check_linear(y, O.linear(codes, o_scales, X, ofmt), f"N={N} K={K} M={M}")


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_reround_packed_weights_through_the_kernels(fmt, ofmt):
    # the re-rounding search only changes which codes are packed: same layout, same kernels
    N, K = 100, 1030
    W = synth.gaussian_weights(N, K, 45)
    packed, scales = ams.ams_pack_ex(fmt, ams.SEARCH_REROUND, W)
    codes, o_scales, _ = O.ams_quantize(W, ofmt, search="reround")
    got = host16(ams.ams_dequant(fmt, dev(packed), dev(scales), N, K, scaled=True))
    assert np.array_equal(got.view(np.uint16), O.dequant_scaled(codes, o_scales, ofmt).view(np.uint16))
    X = synth.activations(3, K, 46)
    y = host16(ams.ams_linear(dev(packed), dev(scales), dev(X), N, fmt))
    check_linear(y, O.linear(codes, o_scales, X, ofmt), "reround")


REC_K = {ams.FP533: 96, ams.FP425: 128, ams.FP45: 128, ams.FP433: 96, ams.FP6: 96, ams.FP5: 128, ams.FP4: 128}


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
@pytest.mark.parametrize("N,K,mult,Ms", [(100, 1030, 1, (1, 3)), (48, 14336, 2, (1, 16)), (528, 4096, 1, (4, 32)), (16, 5, 1, (1,))])
def test_grouped_scales_through_the_kernels(fmt, ofmt, N, K, mult, Ms):
    # one scale per run of input channels: restored weights bit for bit, Linear within tolerance
    sg = REC_K[fmt] * mult
    W = synth.heavy_tail_weights(N, K, 47)
    packed, scales = ams.ams_pack_grouped(fmt, W, sg)
    codes, o_scales = O.ams_quantize_grouped(W, ofmt, sg)
    wp, sc = dev(packed), dev(scales)
    got = host16(ams.ams_dequant_grouped(fmt, wp, sc, sg, N, K, scaled=True))
    assert np.array_equal(got.view(np.uint16), O.dequant_scaled(codes, o_scales, ofmt, sg).view(np.uint16))
    for M in Ms:
        X = synth.activations(M, K, 48 + M)
        y = host16(ams.ams_linear_grouped(wp, sc, sg, dev(X), N, fmt))
        check_linear(y, O.linear(codes, o_scales, X, ofmt, sg), f"grouped N={N} K={K} M={M}")


@pytest.mark.parametrize("fmt,ofmt", PAPER_PAIRS)
def test_grouped_scales_large_shape_sampled_rows(fmt, ofmt):
    # many strips per workgroup; at M=32 the strips per workgroup are capped and the grid takes several rounds
    N, K = 28672, 4096
    sg = REC_K[fmt]
    W = synth.gaussian_weights(N, K, 83)
    packed, scales = ams.ams_pack_grouped(fmt, W, sg)
    wp, sc = dev(packed), dev(scales)
    rows = np.unique(np.r_[0:16, N - 16 : N, np.arange(7, N, 131), 16 * 255 : 16 * 257 + 1])
    codes, o_scales = O.ams_quantize_grouped(W[rows], ofmt, sg)
    for M in (1, 8, 32):
        X = synth.activations(M, K, 84 + M)
        y = host16(ams.ams_linear_grouped(wp, sc, sg, dev(X), N, fmt)).astype(np.float64)
        assert np.all(np.isfinite(y))
        check_linear(y[:, rows].astype(np.float16), O.linear(codes, o_scales, X, ofmt, sg), f"grouped large M={M}")


@pytest.mark.parametrize("fmt,ofmt", PAPER_PAIRS)
def test_grouped_scales_lone_wavefronts(fmt, ofmt):
    # ten strips per workgroup: every wavefront alone on its strip finishes it from its accumulators, here with the
    # per-run scales already applied record by record (the last workgroup is ragged)
    N, K = 40100, 1024
    sg = REC_K[fmt] * 2
    W = synth.gaussian_weights(N, K, 85)
    packed, scales = ams.ams_pack_grouped(fmt, W, sg)
    wp, sc = dev(packed), dev(scales)
    rows = np.unique(np.r_[0:32, N - 40 : N, np.arange(11, N, 397)])
    codes, o_scales = O.ams_quantize_grouped(W[rows], ofmt, sg)
    for M in (1, 20):
        X = synth.activations(M, K, 86 + M)
        y = host16(ams.ams_linear_grouped(wp, sc, sg, dev(X), N, fmt)).astype(np.float64)
        assert np.all(np.isfinite(y))
        check_linear(y[:, rows].astype(np.float16), O.linear(codes, o_scales, X, ofmt, sg), f"grouped lone M={M}")


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_linear_heavy_tail_weights_and_outlier_activations(fmt, ofmt):
    N, K = 64, 8192
    W = synth.heavy_tail_weights(N, K, 51)
    X = synth.activations(8, K, 51)
    X[:, ::97] *= np.float16(30.0)  # channel-wise activation outliers
    packed, scales = ams.ams_pack(fmt, W)
    codes, o_scales, _ = O.ams_quantize(W, ofmt)
    y = host16(ams.ams_linear(dev(packed), dev(scales), dev(X), N, fmt))
    check_linear(y, O.linear(codes, o_scales, X, ofmt), "heavy tail")


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_linear_one_hot_activation_returns_the_restored_weight(fmt, ofmt):
    # a single product and a single rounding: Y[0, n] must be the scaled restored weight exactly
    N, K = 40, 1000
    W = synth.gaussian_weights(N, K, 61)
    packed, scales = ams.ams_pack(fmt, W)
    codes, o_scales, _ = O.ams_quantize(W, ofmt)
    want = O.dequant_scaled(codes, o_scales, ofmt)
    wp, sc = dev(packed), dev(scales)
    ks = list(range(0, 40)) + list(range(90, 135)) + [511, 512, 767, 768, 998, 999]
    X = np.zeros((len(ks), K), dtype=np.float16)
    for i, k in enumerate(ks):
        X[i, k] = 1.0
    for i0 in range(0, len(ks), 32):
        y = host16(ams.ams_linear(wp, sc, dev(X[i0 : i0 + 32]), N, fmt))
        for i in range(y.shape[0]):
            # compared as numbers: a sum that starts from +0 cannot return the -0 of a negative zero code
            assert np.array_equal(y[i], want[:, ks[i0 + i]]), ks[i0 + i]


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
def test_linear_full_size_sampled_rows(fmt, ofmt):
    # baseline config 2 shape (4096 x 4096, M=1) in the launch configuration the benchmark times;
    # the oracle quantizes a sample of rows (rows are independent) and checks those outputs
    W, X = synth.config2()
    N, K = W.shape
    packed, scales = ams.ams_pack(fmt, W)
    y = host16(ams.ams_linear(dev(packed), dev(scales), dev(X), N, fmt)).astype(np.float64)
    rows = np.r_[0:16, 2040:2056, 4080:4096, np.arange(5, N, 257)]
    codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
    ref = O.linear(codes, o_scales, X, ofmt)
    check_linear(y[:, rows].astype(np.float16), ref, "config 2 sample")
    assert np.all(np.isfinite(y))


@pytest.mark.parametrize("fmt,ofmt", PAPER_PAIRS + [(ams.FP433, O.FP433), (ams.FP6, O.FP6_E2M3)])
@pytest.mark.parametrize(
    "N,K,Ms",
    [
        (28672, 4096, (1, 4, 16, 32)),  # Llama-8B gate/up: 7 strips per workgroup, two wavefronts on each; M=32 walks K in phases
        (4200, 14336, (1, 8)),  # long K, workgroups with 2 strips and with 1; M=8 walks K in phases
        (8200, 1000, (1, 32)),  # ragged everything, 3 strips per workgroup, two MFMA row tiles
    ],
)
def test_linear_large_shapes_sampled_rows(fmt, ofmt, N, K, Ms):
    # shapes whose workgroups own several strips, in the launch configuration the benchmark
    # times; the oracle quantizes a sample of rows (rows are independent) and checks those outputs
    W = synth.gaussian_weights(N, K, 81)
    packed, scales = ams.ams_pack(fmt, W)
    wp, sc = dev(packed), dev(scales)
    rows = np.unique(np.r_[0:16, N - 16 : N, np.arange(7, N, 131), 16 * 255 : 16 * 257 + 1])
    rows = rows[rows < N]
    codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
    for M in Ms:
        X = synth.activations(M, K, 81 + M)
        y = host16(ams.ams_linear(wp, sc, dev(X), N, fmt)).astype(np.float64)
        assert np.all(np.isfinite(y))
        check_linear(y[:, rows].astype(np.float16), O.linear(codes, o_scales, X, ofmt), f"N={N} K={K} M={M} sample")


@pytest.mark.parametrize("fmt,ofmt", PAIRS)
@pytest.mark.parametrize(
    "N,K,Ms",
    [
        (200, 6000, (16, 17, 32)),  # one strip per workgroup, many phases
        (90, 6004, (32,)),  # activation rows not 16-byte aligned
        (4400, 3000, (24, 32)),  # two strips per workgroup, the last workgroup has one
    ],
)
def test_linear_activations_in_several_phases(fmt, ofmt, N, K, Ms):
    # batches whose activations do not fit in LDS: wavefronts that own a strip, others that stage
    # the next phase's activations beside them
    W = synth.gaussian_weights(N, K, 91)
    packed, scales = ams.ams_pack(fmt, W)
    wp, sc = dev(packed), dev(scales)
    rows = np.unique(np.r_[0:32, N - 32 : N, np.arange(5, N, 37)])
    codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
    for M in Ms:
        assert "phases=1 " not in ams.ams_linear_plan(fmt, M, N, K)
        X = synth.activations(M, K, 92 + M)
        y = host16(ams.ams_linear(wp, sc, dev(X), N, fmt)).astype(np.float64)
        assert np.all(np.isfinite(y))
        check_linear(y[:, rows].astype(np.float16), O.linear(codes, o_scales, X, ofmt), f"N={N} K={K} M={M}")


@pytest.mark.parametrize("fmt,ofmt", [(ams.FP425, O.FP425), (ams.FP45, O.FP45), (ams.FP433, O.FP433), (ams.FP6, O.FP6_E2M3)])
def test_linear_records_dealt_in_whole_side_groups(fmt, ofmt):
    # formats that keep last bits beside the chunks: where the side groups of a strip divide evenly among its
    # wavefronts they are dealt whole (one side dword per group); an odd number of groups per wavefront, a last
    # group that runs into the padding records, several phases of K at M = 32
    sg = {ams.FP425: 4, ams.FP45: 2, ams.FP433: 4, ams.FP6: 2}[fmt]
    N = 20496  # 1281 strips: 6 per workgroup, two wavefronts on each
    rows = np.unique(np.r_[0:16, N - 16 : N, np.arange(9, N, 211), 16 * 95 : 16 * 97])
    # six groups per strip (three per wavefront, the last one partly padding) in one phase; 32 / sg groups in two phases at M = 32
    for K, Ms in ((REC_K[fmt] * sg * 6 - 5, (1, 5)), (REC_K[fmt] * 32 - 5, (32,))):
        W = synth.gaussian_weights(N, K, 87)
        packed, scales = ams.ams_pack(fmt, W)
        wp, sc = dev(packed), dev(scales)
        codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
        for M in Ms:
            plan = ams.ams_linear_plan(fmt, M, N, K)
            assert "side_groups=1" in plan and "waves_per_strip=2" in plan, plan
            assert ("phases=1 " in plan) == (M < 32), plan
            X = synth.activations(M, K, 88 + M)
            y = host16(ams.ams_linear(wp, sc, dev(X), N, fmt)).astype(np.float64)
            assert np.all(np.isfinite(y))
            check_linear(y[:, rows].astype(np.float16), O.linear(codes, o_scales, X, ofmt), f"side groups fmt {ofmt.name} K={K} M={M}")


def test_linear_70b_gate_up_sampled_rows():
    # the largest benchmark shape (57344 x 8192, 14 strips per workgroup, 313 MB packed), FP5.33
    N, K = synth.LLAMA70B_LAYERS["gate_up"]
    W = synth.gaussian_weights(N, K, 85)
    packed, scales = ams.ams_pack(ams.FP533, W)
    wp, sc = dev(packed), dev(scales)
    rows = np.unique(np.r_[0:16, N - 16 : N, np.arange(11, N, 409)])
    codes, o_scales, _ = O.ams_quantize(W[rows], O.FP533)
    del W
    for M in (1, 8):
        X = synth.activations(M, K, 86 + M)
        y = host16(ams.ams_linear(wp, sc, dev(X), N, ams.FP533)).astype(np.float64)
        assert np.all(np.isfinite(y))
        check_linear(y[:, rows].astype(np.float16), O.linear(codes, o_scales, X, O.FP533), f"70B gate/up M={M}")


@pytest.mark.parametrize(
    "N,K,Ms",
    [(256, 768, (1, 2, 4, 8, 16, 32)), (37, 1000, (1, 7, 20)), (40, 14336, (1, 16)), (4200, 1000, (1, 4, 5))],  # the last: every CU busy
)
def test_fp16_baseline_matches_oracle(N, K, Ms):
    W = synth.gaussian_weights(N, K, 71)
    w = dev(W)
    for M in Ms:
        X = synth.activations(M, K, 71 + M)
        y = host16(ams.ams_fp16_linear(w, dev(X)))
        check_linear(y, O.fp16_linear(W, X), f"fp16 N={N} K={K} M={M}")


def test_linear_random_large_shapes_sampled_rows():
    # seeded random problems large enough to reach every launch plan (wave groups, several phases of K,
    # the contiguous-piece kernel, the split of K): sampled rows against the oracle, with and without a workspace
    rng = np.random.default_rng(16045)
    ws = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda")
    kinds = set()
    for case in range(15):
        fmt, ofmt = PAIRS[int(rng.integers(len(PAIRS)))]
        N = int(2 ** rng.uniform(9, 13.2))
        K = min(int(2 ** rng.uniform(9, 15)), (40 << 20) // N)
        M = int(rng.choice([1, 3, 8, 13, 16, 17, 24, 32]))
        if case == 14:  # three strips per workgroup, large tiles, five phases: the contiguous-piece kernel
            N, K, M = 8200, 8000, 32
        print(f"case {case}: fmt {ofmt.name} N={N} K={K} M={M}", flush=True)
        W = synth.gaussian_weights(N, K, 3000 + case)
        X = synth.activations(M, K, 4000 + case)
        packed, scales = ams.ams_pack(fmt, W)
        rows = np.unique(np.r_[0:16, N - 16 : N, rng.integers(0, N, 24)])
        codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
        ref = O.linear(codes, o_scales, X, ofmt)
        wp, sc, x = dev(packed), dev(scales), dev(X)
        what = f"case {case}: fmt {ofmt.name} N={N} K={K} M={M}"
        for use_ws in (False, True):
            kinds.add(ams.ams_linear_plan(fmt, M, N, K, with_workspace=use_ws).split()[0])
            y = host16(ams.ams_linear_ws(wp, sc, x, N, fmt, ws) if use_ws else ams.ams_linear(wp, sc, x, N, fmt)).astype(np.float64)
            assert np.all(np.isfinite(y)), what
            check_linear(y[:, rows].astype(np.float16), ref, what + (" (workspace)" if use_ws else ""))
    assert kinds == {"column"}  # every packed format takes the one kernel, whatever the shape


def test_linear_random_shapes_all_entry_points():
    # seeded random problems: every format, ragged N and K, any batch, the three Linear entry points
    rng = np.random.default_rng(2510_16045)
    ws = torch.zeros(8 << 20, dtype=torch.uint8, device="cuda")
    for case in range(40):
        fmt, ofmt = PAIRS[int(rng.integers(len(PAIRS)))]
        N = int(rng.integers(1, 700))
        K = int(rng.integers(1, 3000)) if case % 4 else int(rng.integers(1, 40))
        M = int(rng.integers(1, 33))
        W = synth.gaussian_weights(N, K, 1000 + case)
        X = synth.activations(M, K, 2000 + case)
        x = dev(X)
        what = f"case {case}: fmt {ofmt.name} N={N} K={K} M={M}"
        packed, scales = ams.ams_pack(fmt, W)
        codes, o_scales, _ = O.ams_quantize(W, ofmt)
        ref = O.linear(codes, o_scales, X, ofmt)
        wp, sc = dev(packed), dev(scales)
        check_linear(host16(ams.ams_linear(wp, sc, x, N, fmt)), ref, what)
        check_linear(host16(ams.ams_linear_ws(wp, sc, x, N, fmt, ws)), ref, what + " (workspace)")
        sg = REC_K[fmt] * int(rng.choice([1, 2, 8]))
        gp, gs = ams.ams_pack_grouped(fmt, W, sg)
        gcodes, g_scales = O.ams_quantize_grouped(W, ofmt, sg)
        y = host16(ams.ams_linear_grouped(dev(gp), dev(gs), sg, x, N, fmt))
        check_linear(y, O.linear(gcodes, g_scales, X, ofmt, sg), what + f" (scale runs of {sg})")
    torch.cuda.synchronize()
    assert not ws[: 4 * 16384].any()


# ---- K split over workgroups through a workspace -------------------------------------------------
@pytest.mark.parametrize("fmt,ofmt", PAPER_PAIRS + [(ams.FP433, O.FP433)])
def test_linear_with_workspace_matches_oracle(fmt, ofmt):
    # one workspace, zero-filled once, reused by every call below: each call must leave it clean
    ws = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda")
    split_seen = 0
    for N, K, Ms in [(2560, 9728, (1, 8)), (3000, 6004, (16, 32)), (4096, 14336, (8,)), (5120, 25600, (4,))]:
        W = synth.gaussian_weights(N, K, 95)
        packed, scales = ams.ams_pack(fmt, W)
        wp, sc = dev(packed), dev(scales)
        rows = np.unique(np.r_[0:16, N - 16 : N, np.arange(3, N, 97)])
        codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
        for M in Ms:
            need = ams.ams_linear_workspace_bytes(fmt, M, N, K)
            assert need <= ws.numel()
            split_seen += need > 0
            X = synth.activations(M, K, 96 + M)
            x = dev(X)
            y1 = host16(ams.ams_linear_ws(wp, sc, x, N, fmt, ws))
            y2 = host16(ams.ams_linear_ws(wp, sc, x, N, fmt, ws))  # the counters were left at zero
            assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))  # deterministic whoever arrives last
            assert np.all(np.isfinite(y1.astype(np.float64)))
            check_linear(y1[:, rows], O.linear(codes, o_scales, X, ofmt), f"workspace N={N} K={K} M={M}")
            # no workspace, or one that is too small: the plain path, bit for bit
            y0 = host16(ams.ams_linear(wp, sc, x, N, fmt))
            assert np.array_equal(host16(ams.ams_linear_ws(wp, sc, x, N, fmt, None)).view(np.uint16), y0.view(np.uint16))
            assert np.array_equal(host16(ams.ams_linear_ws(wp, sc, x, N, fmt, ws[:256])).view(np.uint16), y0.view(np.uint16))
    assert split_seen >= 4  # the cases above are meant to take the split path
    torch.cuda.synchronize()
    # partial tiles stay behind in the workspace; only the counters must be back at zero
    assert not ws[: 4 * 16384].any()


@pytest.mark.parametrize(
    "N,K",
    [(1, 8), (37, 1000), (5000, 520), (4097, 512), (9000, 24), (256, 40960), (28672, 4096)],
)
def test_fp16_baseline_small_batches_rows_dealt_to_wavefronts(N, K):
    # batches up to 4 take the GEMV form: whole rows per wavefront (more rows than the grid has wavefronts, fewer,
    # one), 512-channel segments with a ragged last one, rows as long as LDS holds activations for
    W = synth.gaussian_weights(N, K, 75)
    w = dev(W)
    rows = np.unique(np.r_[0 : min(N, 32), max(N - 32, 0) : N, np.arange(0, N, 211), 4090 : min(N, 4100)])
    for M in (1, 2, 3, 4):
        if "gemv" not in ams.ams_linear_plan(-1, M, N, K):
            assert 2 * M * K > 150 * 1024  # only activations that do not fit in LDS go elsewhere
            continue
        X = synth.activations(M, K, 75 + M)
        y = host16(ams.ams_fp16_linear(w, dev(X)))
        assert np.all(np.isfinite(y.astype(np.float32)))
        check_linear(y[:, rows], O.fp16_linear(W[rows], X), f"fp16 N={N} K={K} M={M}")


def test_fp16_baseline_keeps_subnormal_weights():
    # weights below the smallest normal binary16 must count (the restored packed weights live there too)
    rng = np.random.default_rng(5)
    N, K = 300, 1024
    W = (rng.integers(1, 1024, size=(N, K)).astype(np.uint16) | (rng.integers(0, 2, size=(N, K)).astype(np.uint16) << 15)).view(np.float16)
    X = synth.activations(2, K, 6)
    y = host16(ams.ams_fp16_linear(dev(W), dev(X)))
    check_linear(y, O.fp16_linear(W, X), "subnormal weights")
    assert np.count_nonzero(y) > y.size // 2


def test_fp16_baseline_with_workspace_matches_oracle():
    ws = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda")
    for N, K, M in [(6144, 4096, 4), (5000, 4104, 8), (3000, 6008, 32)]:
        assert 0 < ams.ams_linear_workspace_bytes(-1, M, N, K) <= ws.numel()
        W = synth.gaussian_weights(N, K, 97)
        X = synth.activations(M, K, 98)
        y = host16(ams.ams_fp16_linear_ws(dev(W), dev(X), ws))
        rows = np.unique(np.r_[0:16, N - 16 : N, np.arange(3, N, 97)])
        check_linear(y[:, rows], O.fp16_linear(W[rows], X), f"fp16 workspace N={N} K={K} M={M}")
    torch.cuda.synchronize()
    assert not ws[: 4 * 16384].any()


def test_device_entry_points_reject_bad_arguments():
    lib = ams.load_library()
    W = synth.gaussian_weights(16, 96, 1)
    packed, scales = ams.ams_pack(ams.FP533, W)
    wp, sc = dev(packed), dev(scales)
    x = dev(synth.activations(1, 96, 1))
    y = torch.empty((1, 16), dtype=torch.float16, device="cuda")
    p = lambda t: t.data_ptr()
    assert lib.ams_linear(p(wp), p(sc), p(x), p(y), 0, 16, 96, 0, None) == -2
    assert lib.ams_linear(p(wp), p(sc), p(x), p(y), 33, 16, 96, 0, None) == -2
    assert lib.ams_linear(p(wp), p(sc), p(x), p(y), 1, 16, 96, 9, None) == -1
    assert lib.ams_linear(None, p(sc), p(x), p(y), 1, 16, 96, 0, None) == -3
    assert lib.ams_linear(p(wp) + 2, p(sc), p(x), p(y), 1, 16, 96, 0, None) == -4
    assert lib.ams_dequant(9, p(wp), p(sc), p(y), 16, 96, 1, None) == -1
    assert lib.ams_fp16_linear(p(x), p(x), p(y), 1, 1, 95, None) == -2
    assert lib.ams_linear_grouped(p(wp), p(sc), 100, p(x), p(y), 1, 16, 96, 0, None) == -2
    assert lib.ams_dequant_grouped(0, p(wp), p(sc), 95, p(y), 16, 96, 1, None) == -2
    assert lib.ams_read_probe(None, 1024, None, None) == -3
    assert lib.ams_read_probe(p(wp) + 2, 1024, None, None) == -4
    torch.cuda.synchronize()


def test_read_probe_runs_on_any_size_and_changes_nothing():
    buf = torch.arange(3 * 1024 * 1024 + 700, dtype=torch.uint8, device="cuda")
    before = buf.clone()
    for nbytes in (0, 700, 1024, 17 * 1024, 1 << 20, buf.numel()):
        ams.ams_read_probe(buf, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(buf, before)
