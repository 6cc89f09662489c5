"""The Linear entry points under HIP graph capture: the four Linears of a decoder layer
captured once, replayed several times with eager work between the replays; every
replay must give the eager result bit for bit (the kernels are deterministic)."""

import numpy as np
import pytest

import paper_2510_16045_amd as ams
from paper_2510_16045_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def dev(a: np.ndarray):
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


@pytest.mark.parametrize("M,use_ws", [(1, False), (8, True)])
def test_decoder_layer_linears_replay_like_eager(M, use_ws):
    # scaled-down qkv / o / gate-up / down (hidden 1024, intermediate 3584), both paper formats
    shapes = [("qkv", 1536, 1024), ("o", 1024, 1024), ("gate_up", 7168, 1024), ("down", 1024, 3584)]
    if use_ws:  # a down projection that takes the split of K (Qwen3-4B's), so the workspace exchange is replayed too
        shapes[3] = ("down", 2560, 9728)
        assert ams.ams_linear_workspace_bytes(ams.FP425, M, 2560, 9728) > 0
    ws = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda") if use_ws else None
    layers = []
    for i, (name, N, K) in enumerate(shapes):
        fmt = ams.FP533 if i % 2 == 0 else ams.FP425
        packed, scales = ams.ams_pack(fmt, synth.gaussian_weights(N, K, 300 + i))
        x = dev(synth.activations(M, K, 310 + i))
        y = torch.zeros((M, N), dtype=torch.float16, device="cuda")
        layers.append((fmt, N, dev(packed), dev(scales), x, y))

    def run():
        for fmt, N, wp, sc, x, y in layers:
            if ws is None:
                ams.ams_linear(wp, sc, x, N, fmt, out=y)
            else:
                ams.ams_linear_ws(wp, sc, x, N, fmt, ws, out=y)

    run()  # eager (also raises the kernels' LDS limits outside the capture)
    torch.cuda.synchronize()
    want = [y.clone() for *_, y in layers]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for r in range(4):
        for *_, y in layers:
            y.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for (*_, y), w in zip(layers, want):
            assert torch.equal(y.view(torch.int16), w.view(torch.int16)), f"replay {r}"
        run()  # eager work between the replays
        torch.cuda.synchronize()
        for (*_, y), w in zip(layers, want):
            assert torch.equal(y.view(torch.int16), w.view(torch.int16)), f"eager after replay {r}"
    if ws is not None:
        assert not ws[: 4 * 16384].any()

