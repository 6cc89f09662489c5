"""GPU parity on the benchmark configurations at their full sizes, in the launch configuration
bench.py times: the Llama-70B-shaped layers on heavy-tailed weights with outliers (both paper
formats, M in {1, 4, 8}), the Llama-8B qkv and down projections, the batch sweep on the Llama-8B
gate/up and down projections (M = 1 .. 32, with and without a split of K), and the Qwen down
projections of Table 3.  The oracle quantizes a sample of rows (rows are independent: first and
last strip, a workgroup boundary, a stride through the matrix) and checks those outputs; the
restored weights of the sampled strips must match bit for bit."""

import numpy as np
import pytest

import paper_2510_16045_amd as ams
from oracle import ams_oracle as O
from paper_2510_16045_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

PAPER_PAIRS = [(ams.FP533, O.FP533), (ams.FP425, O.FP425)]
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
    assert np.all(np.isfinite(y)), what
    rel = np.linalg.norm(y - ref) / max(np.linalg.norm(ref), 1e-300)
    rms = np.sqrt(np.mean(ref * ref))
    mx = np.max(np.abs(y - ref)) / max(rms, 1e-300)
    assert rel <= REL_L2_TOL, f"{what}: rel L2 {rel}"
    assert mx <= MAX_ABS_TOL, f"{what}: max abs / rms {mx}"


def sampled_strips(N: int, stride: int, extra=()) -> np.ndarray:
    """Strips of 16 rows: the first, the last, the ones around workgroup 255 / 256 (the grid has 256
    workgroups and strips are dealt round robin), and every stride-th."""
    n_strips = -(-N // 16)
    s = np.r_[0, n_strips - 1, 254:258, np.arange(3, n_strips, stride), np.asarray(extra, dtype=np.int64)]
    return np.unique(s[s < n_strips])


def check_shape_against_oracle(N, K, W, Ms, stride, with_workspace=False, with_static=False, extra_strips=()):
    strips = sampled_strips(N, stride, extra_strips)
    rows = np.concatenate([np.arange(16 * t, min(N, 16 * t + 16)) for t in strips])
    ws = torch.zeros(16 << 20, dtype=torch.uint8, device="cuda") if with_workspace else None
    for fmt, ofmt in PAPER_PAIRS:
        packed, scales = ams.ams_pack(fmt, W)
        codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
        assert np.array_equal(scales[rows].view(np.uint16), o_scales.view(np.uint16))
        wp, sc = dev(packed), dev(scales)
        # restored weights of the sampled rows, bit for bit (the whole matrix is restored on the GPU, the
        # sampled rows are gathered there and compared on the host)
        full = ams.ams_dequant(fmt, wp, sc, N, K, scaled=True)
        got = host16(full[torch.from_numpy(rows).cuda()].contiguous())
        del full
        want = O.dequant_scaled(codes, o_scales, ofmt).view(np.uint16)
        assert np.array_equal(got.view(np.uint16), want), f"{ofmt.name} N={N} K={K}: restored weights"
        for M in Ms:
            X = synth.activations(M, K, 500 + M)
            ref = O.linear(codes, o_scales, X, ofmt)
            x = dev(X)
            print(f"{ofmt.name} N={N} K={K} M={M}: {ams.ams_linear_plan(fmt, M, N, K)}", flush=True)
            y = host16(ams.ams_linear(wp, sc, x, N, fmt))
            assert np.all(np.isfinite(y.astype(np.float32)))
            check_linear(y[:, rows], ref, f"{ofmt.name} N={N} K={K} M={M}")
            if ws is not None:
                y = host16(ams.ams_linear_ws(wp, sc, x, N, fmt, ws))
                check_linear(y[:, rows], ref, f"{ofmt.name} N={N} K={K} M={M} (workspace)")
            if with_static:
                y = host16(ams.ams_linear_static_ws(wp, sc, x, N, fmt))
                check_linear(y[:, rows], ref, f"{ofmt.name} N={N} K={K} M={M} (static scratch)")
        del wp, sc


@pytest.mark.parametrize("layer,stride", [("o", 37), ("gate_up", 211), ("down", 61)])
def test_llama70b_layers_heavy_tail_weights(layer, stride):
    # Student-t(4) x 0.02 weights, 0.1 % of them x 20: rows with an outlier get a large scale and
    # mostly subnormal codes, which is what the fp32 scale x 2^14 epilogue has to survive
    N, K = synth.LLAMA70B_LAYERS[layer]
    W = synth.heavy_tail_weights(N, K, 700 + len(layer))
    assert np.abs(W.astype(np.float32)).max() > 2.0  # outliers are there
    check_shape_against_oracle(N, K, W, (1, 4, 8), stride, with_workspace=layer != "gate_up")


@pytest.mark.parametrize("layer,stride", [("qkv", 29), ("o", 23), ("down", 31)])
def test_llama8b_layers_small_batches(layer, stride):
    N, K = synth.LLAMA8B_LAYERS[layer]
    W = synth.gaussian_weights(N, K, 710 + len(layer))
    check_shape_against_oracle(N, K, W, (1, 2), stride)


@pytest.mark.parametrize("layer,stride", [("gate_up", 173), ("down", 41)])
def test_llama8b_batch_sweep(layer, stride):
    # the batch sweep the benchmark times: every batch size, through the plain entry point, the caller's
    # workspace and the library's static scratch
    N, K = synth.LLAMA8B_LAYERS[layer]
    W = synth.gaussian_weights(N, K, 730 + len(layer))
    check_shape_against_oracle(N, K, W, (1, 2, 4, 8, 16, 32), stride, with_workspace=True, with_static=True)


def test_llama8b_vocabulary_projection():
    # 128256 x 4096: 8016 strips, 16 per workgroup, 501 workgroups on 256 compute units (two rounds); sampled
    # strips include both sides of the boundary between the rounds and of a workgroup
    N, K = synth.LLAMA8B_LM_HEAD
    W = synth.gaussian_weights(N, K, 740)
    check_shape_against_oracle(N, K, W, (1, 8), 499, with_static=True, extra_strips=(15, 16, 4095, 4096, 8000, 8015))


@pytest.mark.parametrize("model,Ms", [("qwen2.5-7b", (1, 2, 16)), ("qwen3-4b", (1, 32))])
def test_qwen_down_projections(model, Ms):
    # MLP-down shapes of Table 3, with and without the split of K
    N, K = synth.QWEN_DOWN_LAYERS[model]
    W = synth.gaussian_weights(N, K, 720 + len(model))
    check_shape_against_oracle(N, K, W, Ms, 23, with_workspace=True)


@pytest.mark.parametrize("N,K,Ms", [(1_000_003, 100, (1, 5)), (20, 1_000_000, (1, 5, 32))])
def test_extreme_aspect_ratios(N, K, Ms):
    # a million rows of two records each (62501 strips: thousands of workgroups in many rounds), and two strips
    # of ten thousand records (K walked in phases from M = 5 on, split over workgroups when a workspace is given)
    W = synth.gaussian_weights(N, K, 750 + (N % 7))
    check_shape_against_oracle(N, K, W, Ms, 4999, with_workspace=N < 100, with_static=N < 100)


@pytest.mark.parametrize("N,K,Ms,ws", [(30000, 16384, (8, 32), True), (14336, 4096, (1, 2, 3), False)])
def test_lone_wavefronts_and_eight_wavefront_plans(N, K, Ms, ws):
    # 30000 x 16384 with a workspace: K in two slices and fifteen strips per workgroup, every wavefront alone on its
    # strip, so the partial tiles go to the workspace straight from the accumulators (the last workgroup is ragged);
    # 14336 x 4096: four strips per workgroup, eight wavefronts with three records ahead, two on each strip
    if ws:
        assert "k_slices=2" in ams.ams_linear_plan(ams.FP533, Ms[0], N, K, with_workspace=True)
        assert "waves_per_strip=1 " in ams.ams_linear_plan(ams.FP533, Ms[0], N, K, with_workspace=True)
    else:
        assert "waves=8 waves_per_strip=2 " in ams.ams_linear_plan(ams.FP533, Ms[0], N, K)
    W = synth.gaussian_weights(N, K, 760 + (N % 5))
    check_shape_against_oracle(N, K, W, Ms, 97, with_workspace=ws, with_static=ws)


@pytest.mark.parametrize("N,K,Ms", [(45000, 4096, (1, 3, 8)), (45000, 16384, (8,)), (45000, 1001, (2,))])
def test_wavefronts_with_two_strips_each(N, K, Ms):
    # 2813 strips: eleven per workgroup (an odd number for eight wavefronts with two strips each: one wavefront has
    # a single strip), the last workgroup has eight; 43 records per strip (an odd count), K walked in two phases, or
    # activation rows that are not 16-byte aligned (K = 1001)
    for M in Ms:
        assert "strips_per_wave=2" in ams.ams_linear_plan(ams.FP533, M, N, K)
    assert "phases=1 " not in ams.ams_linear_plan(ams.FP533, 8, 45000, 16384)
    W = synth.gaussian_weights(N, K, 770 + (K % 7))
    n_strips = -(-N // 16)
    check_shape_against_oracle(N, K, W, Ms, 211, extra_strips=tuple(range(n_strips - 12, n_strips)) + tuple(range(0, 23)))


@pytest.mark.parametrize("fmt,ofmt", [(ams.FP5, O.FP5_E2M2), (ams.FP4, O.FP4_E2M1)])
@pytest.mark.parametrize("N,K,Ms", [(45000, 4096, (1, 8)), (28672, 4096, (1, 4))])
def test_other_formats_without_side_groups_on_the_eight_wavefront_plans(fmt, ofmt, N, K, Ms):
    # FP5 (four side bytes per lane and record, no side groups) and FP4 take the same plans as FP5.33: two strips per
    # wavefront on 45000 rows, one wavefront alone on each of seven strips on 28672
    want = "strips_per_wave=2" if N == 45000 else "waves=8 waves_per_strip=1 "
    assert want in ams.ams_linear_plan(fmt, Ms[0], N, K)
    W = synth.gaussian_weights(N, K, 780)
    packed, scales = ams.ams_pack(fmt, W)
    n_strips = -(-N // 16)
    strips = sampled_strips(N, 173, tuple(range(n_strips - 12, n_strips)))
    rows = np.concatenate([np.arange(16 * t, min(N, 16 * t + 16)) for t in strips])
    codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
    wp, sc = dev(packed), dev(scales)
    for M in Ms:
        X = synth.activations(M, K, 781 + M)
        y = host16(ams.ams_linear(wp, sc, dev(X), N, fmt))
        check_linear(y[:, rows], O.linear(codes, o_scales, X, ofmt), f"{ofmt.name} N={N} K={K} M={M}")


def test_random_shapes_with_many_strips_per_workgroup():
    # seeded random problems with 7 to 16 strips per workgroup (lone wavefronts, two strips per wavefront, ragged last
    # workgroups, odd record counts, unaligned rows), any format and batch: sampled strips against the oracle
    rng = np.random.default_rng(451)
    fmts = [(ams.FP533, O.FP533), (ams.FP425, O.FP425), (ams.FP45, O.FP45), (ams.FP433, O.FP433), (ams.FP6, O.FP6_E2M3),
            (ams.FP5, O.FP5_E2M2), (ams.FP4, O.FP4_E2M1)]
    seen = set()
    for case in range(12):
        fmt, ofmt = fmts[case % len(fmts)]
        N = int(rng.integers(26000, 66000))
        K = int(rng.integers(300, 150_000_000 // N))
        if case % 3 == 0:
            K = K // 8 * 8 + int(rng.integers(1, 8))  # rows that are not 16-byte aligned
        M = int(rng.choice([1, 2, 3, 5, 8, 9, 16, 17, 32]))
        plan = ams.ams_linear_plan(fmt, M, N, K)
        print(f"case {case}: {ofmt.name} N={N} K={K} M={M}: {plan}", flush=True)
        kv = dict(x.split("=") for x in plan.split()[1:])
        seen.add((kv["waves"], kv["strips_per_wave"], kv["waves_per_strip"]))
        W = synth.gaussian_weights(N, K, 800 + case)
        packed, scales = ams.ams_pack(fmt, W)
        n_strips = -(-N // 16)
        strips = sampled_strips(N, 331, tuple(range(n_strips - 18, n_strips)) + tuple(range(0, 18)))
        rows = np.concatenate([np.arange(16 * t, min(N, 16 * t + 16)) for t in strips])
        codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
        X = synth.activations(M, K, 900 + case)
        y = host16(ams.ams_linear(dev(packed), dev(scales), dev(X), N, fmt))
        assert np.all(np.isfinite(y.astype(np.float32)))
        check_linear(y[:, rows], O.linear(codes, o_scales, X, ofmt), f"case {case}: {ofmt.name} N={N} K={K} M={M}")
    assert ("8", "2", "1") in seen and ("16", "1", "1") in seen  # two strips per wavefront; sixteen lone wavefronts
