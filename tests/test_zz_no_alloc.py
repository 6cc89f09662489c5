"""The entry point that allocates nothing (ams_linear_static_ws: the split of K through the
library's static device scratch) against ams_linear_ws with a caller's workspace: same kernels,
same launch plan, so the outputs must agree bit for bit (and with the oracle within tolerance),
on calls in a row that share the scratch, the later ones with smaller inputs."""

import ctypes

import numpy as np
import pytest

import paper_2510_16045_amd as ams
from oracle import ams_oracle as O
from paper_2510_16045_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a: np.ndarray):
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


def host16(t) -> np.ndarray:
    return t.cpu().view(torch.int16).numpy().view(np.float16)


def test_static_scratch_entry_point_matches_the_workspace_one():
    lib = ams.load_library()
    ws = torch.zeros(16 << 20, dtype=torch.uint8, device="cuda")
    # first a large problem that takes the split of K, then smaller ones on the same scratch
    cases = [(ams.FP533, O.FP533, 4096, 14336, 16), (ams.FP425, O.FP425, 2560, 9728, 8), (ams.FP533, O.FP533, 528, 4096, 4),
             (ams.FP425, O.FP425, 37, 1000, 1)]
    split_seen = 0
    for fmt, ofmt, N, K, M in cases:
        W = synth.gaussian_weights(N, K, 900 + M)
        X = synth.activations(M, K, 901 + M)
        packed, scales = ams.ams_pack(fmt, W)
        wp, sc, x = dev(packed), dev(scales), dev(X)
        split_seen += ams.ams_linear_workspace_bytes(fmt, M, N, K) > 0
        print(f"N={N} K={K} M={M}: {ams.ams_linear_plan(fmt, M, N, K, with_workspace=True)}", flush=True)
        want = host16(ams.ams_linear_ws(wp, sc, x, N, fmt, ws))
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        # straight through the C ABI
        rc = lib.ams_linear_static_ws(wp.data_ptr(), sc.data_ptr(), x.data_ptr(), y.data_ptr(), M, N, K, fmt,
                                      ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0, lib.ams_strerror(rc)
        got = host16(y)
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), f"N={N} K={K} M={M}"
        # a second call right behind it finds the counters at zero again
        got2 = host16(ams.ams_linear_static_ws(wp, sc, x, N, fmt))
        assert np.array_equal(got2.view(np.uint16), want.view(np.uint16)), f"N={N} K={K} M={M} (second call)"
        rows = np.unique(np.r_[0:16, N - 16 : N, np.arange(3, N, 97)])
        rows = rows[(rows >= 0) & (rows < N)]
        codes, o_scales, _ = O.ams_quantize(W[rows], ofmt)
        ref = O.linear(codes, o_scales, X, ofmt)
        yy = got[:, rows].astype(np.float64)
        assert np.linalg.norm(yy - ref) <= 1e-3 * np.linalg.norm(ref)
        assert np.max(np.abs(yy - ref)) <= 2e-2 * np.sqrt(np.mean(ref * ref))
    assert split_seen >= 2


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    lib = ams.load_library()
    W = synth.gaussian_weights(16, 96, 1)
    packed, scales = ams.ams_pack(ams.FP533, W)
    wp, sc = dev(packed), dev(scales)
    x = dev(synth.activations(1, 96, 1))
    y = torch.empty((1, 16), dtype=torch.float16, device="cuda")
    p = lambda t: t.data_ptr()
    # a shape whose split of K wants more than the static array holds; the size check comes before
    # anything is launched, so the pointers of a small problem are enough
    limit = (64 << 10) + (8 << 20)
    assert ams.ams_linear_workspace_bytes(ams.FP533, 32, 36000, 14336) > limit
    assert lib.ams_linear_static_ws(p(wp), p(sc), p(x), p(y), 32, 36000, 14336, 0, None) == -8  # AMS_ERR_SCRATCH
    assert ams.ams_linear_workspace_bytes(ams.FP425, 17, 36000, 28672) > limit
    assert lib.ams_linear_static_ws(p(wp), p(sc), p(x), p(y), 17, 36000, 28672, 1, None) == -8
    assert b"scratch" in lib.ams_strerror(-8)
    assert lib.ams_linear_static_ws(p(wp), p(sc), p(x), p(y), 1, 16, 96, 9, None) == -1
    assert lib.ams_linear_static_ws(None, p(sc), p(x), p(y), 1, 16, 96, 0, None) == -3
    assert lib.ams_linear_static_ws(p(wp), p(sc), p(x), p(y), 1, 16, 96, 0, None) == 0
    torch.cuda.synchronize()
