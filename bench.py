#!/usr/bin/env python3
"""Benchmark of the MI355X AMS-Quant weight-only quantized Linear (decode path).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-sweep] [--no-70b] [--layers 8b|70b|qwen]

One *step* is one pass over the Linear set of one Llama-3-8B decoder layer at decode
time (fused qkv, o, fused gate/up, down; M = 1) in both AMS formats: eight ams_linear
launches whose packed weights all stream from HBM.  To keep every launch cold, the
step rotates through several resident copies of each packed matrix (a real decode
step touches each layer's weights once per token and the model never fits a cache).

stdout carries ONE JSON line: whole-step packed-weight GB/s as `value`, per-layer
figures (us per Linear with percentiles, cache-resident time, GB/s, fraction of the
8 TB/s HBM peak and of a bare read of the same bytes, speed-up over the in-build fp16
Linear and the library GEMM) under `layers`, a `roofline` object for the dominant kernel,
a `cpu_baseline` object (the numpy oracle timed on this host) and, unless switched off,
`batch_sweep` (M = 1..32 on the 8B gate/up and down projections, both formats, plain
ams_linear and the split of K through the library's static scratch, against the faster of
the two fp16 baselines) and `llama70b` (the Llama-70B-shaped layers on heavy-tailed weights
at M = 1, 4, 8).
"""

from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
ROTATE_BYTES = 512 << 20  # a Linear timed alone rotates over copies of its weights worth at least this (2 x the 256 MB last-level cache)
CLOCK_RAMP_S = 0.5  # untimed load before the warm-up steps, so that an idle GPU's clocks are up
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by what the same counters read for
# a device copy of known size): kept beside the profile summaries they come from, with the layout version they hold for
PROFILES_DIR = os.path.join(ROOT, "profiles")
FMT_NAMES = {0: "fp5.33-e2m3", 1: "fp4.25-e2m2", 2: "fp4.5-e2m2", 3: "fp4.33-e2m2", 4: "fp6-e2m3", 5: "fp5-e2m2", 6: "fp4-e2m1"}
SWEEP_MS = (1, 2, 4, 8, 16, 32)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--layers", default="8b", choices=["8b", "70b", "qwen"], help="layer set of the step and of the per-layer table")
    ap.add_argument("--no-sweep", action="store_true", help="skip the batch sweep M=1..32 (gate/up and down of the 8B set)")
    ap.add_argument("--sweep-all-layers", action="store_true", help="sweep every layer of the set, not only gate/up and down")
    ap.add_argument("--no-70b", action="store_true", help="skip the Llama-70B-shaped layers at M=1,4,8")
    ap.add_argument("--no-lm-head", action="store_true", help="skip the Llama-3-8B vocabulary projection (128256 x 4096) at M=1,8")
    ap.add_argument("--no-qwen", action="store_true", help="skip the Qwen MLP-down shapes of the paper's Table 3 at batch 1, 4, 16, 32")
    ap.add_argument("--out", default=None, help="also write the sweep table to this file")
    ap.add_argument("--all-formats", action="store_true", help="per-layer figures and the sweep for all seven formats (the step keeps the paper's two)")
    ap.add_argument("--group-scales", action="store_true", help="also time ams_linear_grouped (one scale per record-sized run of K) per layer")
    ap.add_argument("--workspace", action="store_true", help="the step and the per-layer table call ams_linear_ws / ams_fp16_linear_ws with a workspace")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-kernel", default=None, metavar="LAYER:FMT:M",
                    help="only launch one Linear (e.g. gate_up:fp4.25:1, down:fp16:1) a few times, for rocprofv3, and exit")
    ap.add_argument("--copies-mb", type=int, default=1024, help="rotate through at least this many MB of weights per layer set")
    return ap.parse_args()


def to_dev(a, torch):
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


class Layer:
    """One Linear: packed copies in the given formats + fp16 copies, all resident in HBM."""

    def __init__(self, name, N, K, W, ams, torch, n_copies, fp16_copies, fmts):
        self.name, self.N, self.K = name, N, K
        self.packed, self.scales, self.canon = {}, {}, {}
        for fmt in fmts:
            p, s = ams.ams_pack(fmt, W)
            base = to_dev(p, torch)
            # timed alone, a layer rotates over its own copies: at least twice the last-level cache
            n = max(n_copies, -(-ROTATE_BYTES // base.numel()))
            self.packed[fmt] = [base] + [base.clone() for _ in range(n - 1)]
            self.scales[fmt] = to_dev(s, torch)
            self.canon[fmt] = ams.ams_canonical_bytes(fmt, N, K)
        w = to_dev(W, torch)
        n16 = max(fp16_copies, -(-ROTATE_BYTES // (2 * w.numel())))
        self.w16 = [w] + [w.clone() for _ in range(n16 - 1)]
        self.W = W  # host copy, for the variants packed on demand


def build_layers(shapes, maker, seed0, fmts, copies_mb, ams, torch):
    set_bytes = sum(n * k * 16 // 3 // 8 for n, k in shapes.values())
    n_copies = max(2, -(-copies_mb * (1 << 20) // set_bytes))
    fp16_copies = max(2, -(-copies_mb * (1 << 20) // (3 * set_bytes)))
    layers = []
    for i, (name, (N, K)) in enumerate(shapes.items()):
        W = maker(N, K, seed0 + i)
        layers.append(Layer(name, N, K, W, ams, torch, n_copies, fp16_copies, fmts))
        del W
    return layers, n_copies


def time_launches(torch, fn, n_launch, warm=2, replays=5, spread=False):
    """Average GPU time per call of fn(i): n_launch back-to-back launches are captured in a HIP graph
    (so that the host's launch cost does not gate the measurement) and the graph is replayed between
    HIP events on the launch stream.  spread=True times every replay by itself and also returns the
    10th / 50th / 90th percentile of the per-replay averages."""
    g = torch.cuda.CUDAGraph()
    fn(0)
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        for i in range(n_launch):
            fn(i)
    for _ in range(warm):
        g.replay()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
    ev[0].record()
    for r in range(replays):
        g.replay()
        if spread or r == replays - 1:
            ev[r + 1].record()
    torch.cuda.synchronize()
    mean = ev[0].elapsed_time(ev[replays]) * 1e3 / (n_launch * replays)  # us
    if not spread:
        return mean
    per = sorted(ev[r].elapsed_time(ev[r + 1]) * 1e3 / n_launch for r in range(replays))
    pick = lambda q: per[min(len(per) - 1, int(q * len(per)))]
    return mean, {"p10": round(pick(0.1), 3), "p50": round(pick(0.5), 3), "p90": round(pick(0.9), 3), "replays": replays, "launches_per_replay": n_launch}


def random_codes(ofmt, N, K, seed):
    """Seeded random codes whose last bits agree inside every sharing group (input generation only:
    what the oracle's unpack / dequant / matmul cost does not depend on which codes they are)."""
    rng = np.random.default_rng(seed)
    g = ofmt.group
    rem = rng.integers(0, 1 << (ofmt.code_bits - 1), size=(N, K), dtype=np.uint8)
    shared = np.repeat(rng.integers(0, 2, size=(N, -(-K // g)), dtype=np.uint8), g, axis=1)[:, :K]
    return (rem << 1) | shared


def cpu_baseline(shapes):
    """The oracle as it stands (canonical unpack -> dequant -> fp64 matmul, M = 1) timed on this host: every Linear
    of the 8B decode step in both formats, whole, one pass (about 10 s of CPU work on 16 cores, 30 s on 8), plus
    baseline configurations 1 and 2 in full."""
    from oracle import ams_oracle as O
    from paper_2510_16045_amd import synth

    try:
        from threadpoolctl import threadpool_info

        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1

    def timed(ofmt, codes, s, X, repeats):
        words = O.pack_canonical(codes, ofmt)  # offline step, not timed
        K = codes.shape[1]
        best = None
        for _ in range(repeats):
            t0 = time.perf_counter()
            c = O.unpack_canonical(words, ofmt, K)
            y = O.linear(c, s, X, ofmt)
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
            del c, y
        return words.nbytes, best

    # the step's own workload, both formats; codes are seeded random ones (the oracle's quantizer, the
    # offline step, would take minutes at this size and is not part of what is timed)
    total_bytes, total_t, per_layer = 0, 0.0, []
    for i, (name, (N, K)) in enumerate(shapes.items()):
        X = synth.activations(1, K, 3)
        for ofmt in (O.FP533, O.FP425):
            rows = N  # the whole layer: about 10 s of CPU work for the set on 16 cores
            codes = random_codes(ofmt, rows, K, 77 + i)
            s = np.full(rows, 0.01, dtype=np.float16)
            nbytes, t = timed(ofmt, codes, s, X, 1)
            per_layer.append({"layer": name, "fmt": ofmt.name, "ms": round(t * 1e3, 1), "GBps": round(nbytes / t / 1e9, 4)})
            total_bytes += nbytes
            total_t += t
            del codes
    # baseline configurations 1 and 2 in full, quantized by the oracle itself (offline, untimed), best of 3
    configs = {}
    for label, (W, X), ofmt in (("config1_256x768_fp4.25_m1", synth.config1(), O.FP425), ("config2_4096x4096_fp5.33_m1", synth.config2(), O.FP533)):
        if W.shape[0] > 1024:  # quantizing 16.7 M weights with the oracle takes ~15 s: random codes, as above
            codes, s = random_codes(ofmt, *W.shape, 5), np.full(W.shape[0], 0.01, dtype=np.float16)
        else:
            codes, s, _ = O.ams_quantize(W, ofmt)
        nbytes, t = timed(ofmt, codes, s, X, 3)
        configs[label] = {"us_per_linear": round(t * 1e6, 1), "GBps": round(nbytes / t / 1e9, 4)}
    return {
        "value": total_bytes / total_t / 1e9,
        "unit": "GB/s",
        "cores": threads,
        "host_cores_available": len(os.sched_getaffinity(0)),
        "kind": "oracle",
        "sample": "the whole workload of `value`: the eight Linears of the Llama-3-8B decode step (4 layers x FP5.33 + FP4.25, M=1), "
                  "canonical unpack + dequant + fp64 matmul, one pass each, seeded random codes; `full_configs`: baseline configurations 1 and 2 whole, best of 3",
        "seconds": round(total_t, 2),
        "per_layer": per_layer,
        "full_configs": configs,
    }


def profile_kernel(args, shapes, torch, ams, synth):
    """Launch one Linear `--steps` times on rotating copies (plain launches, no graph) for a profiler."""
    name, fmt_s, m_s = args.profile_kernel.split(":")
    if name == "copy":  # calibration for HBM traffic counters: a device copy of a known size (fmt field = MiB)
        n = int(fmt_s) << 20
        src = [torch.full((n,), 7, dtype=torch.uint8, device="cuda") for _ in range(3)]
        dst = torch.empty(n, dtype=torch.uint8, device="cuda")
        for i in range(args.steps):
            dst.copy_(src[i % 3])
        torch.cuda.synchronize()
        print(json.dumps({"profiled": args.profile_kernel, "launches": args.steps, "bytes_read": n, "bytes_written": n}))
        return
    N, K = shapes[name]
    M = int(m_s)
    W = synth.gaussian_weights(N, K, 100)
    x = to_dev(synth.activations(M, K, 7), torch)
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    n_copies = 6
    if fmt_s == "fp16":
        ws = [to_dev(W, torch) for _ in range(3)]
        run = lambda i: ams.ams_fp16_linear(ws[i % 3], x, out=y)
    else:
        fmt = {"fp5.33": ams.FP533, "fp4.25": ams.FP425, "fp4.5": ams.FP45, "fp4.33": ams.FP433, "fp6": ams.FP6, "fp5": ams.FP5, "fp4": ams.FP4}[fmt_s]
        p, s = ams.ams_pack(fmt, W)
        ps = [to_dev(p, torch) for _ in range(n_copies)]
        sc = to_dev(s, torch)
        if args.workspace:  # the entry point that may split K over workgroups
            wsp = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda")
            run = lambda i: ams.ams_linear_ws(ps[i % n_copies], sc, x, N, fmt, wsp, out=y)
        else:
            run = lambda i: ams.ams_linear(ps[i % n_copies], sc, x, N, fmt, out=y)
    for i in range(args.steps):
        run(i)
    torch.cuda.synchronize()
    print(json.dumps({"profiled": args.profile_kernel, "launches": args.steps}))


def measured_traffic(ams, layer, fmt_name, M):
    """HBM bytes per launch from the tracked counter summaries (profiles/*hbm_traffic*.md carry one line
    `traffic-json: {...}` each), or None when there is none for this launch or it was measured with another
    packed layout (major version of the library)."""
    import glob

    for path in sorted(glob.glob(os.path.join(PROFILES_DIR, "*hbm_traffic*.md"))):
        try:
            with open(path) as f:
                lines = [ln for ln in f if ln.startswith("traffic-json:")]
            for ln in lines:
                e = json.loads(ln[len("traffic-json:"):])
                if e.get("layout_version") == ams.ams_version() // 100 and (e.get("layer"), e.get("fmt"), e.get("M")) == (layer, fmt_name, M):
                    return int(e["fetch_bytes"]) + int(e["write_bytes"])
        except (OSError, ValueError, KeyError):
            continue
    return None


def batch_sweep(layers, fmts, ams, torch, synth, n_launch, ws, batches=None):
    """Every layer x M in 1..32 x format: plain ams_linear, the split of K (static scratch), both fp16 baselines."""
    rows = []
    for l in layers:
        for Mb in batches or SWEEP_MS:
            x = to_dev(synth.activations(Mb, l.K, 9), torch)
            y = torch.empty((Mb, l.N), dtype=torch.float16, device="cuda")
            t16 = time_launches(torch, lambda i: ams.ams_fp16_linear(l.w16[i % len(l.w16)], x, out=y), n_launch)
            t16ws = time_launches(torch, lambda i: ams.ams_fp16_linear_ws(l.w16[i % len(l.w16)], x, ws, out=y), n_launch)
            tlib = time_launches(torch, lambda i: torch.matmul(x, l.w16[i % len(l.w16)].t(), out=y), n_launch)
            best16 = min(t16, t16ws, tlib)
            for fmt in fmts:
                pk, sc = l.packed[fmt], l.scales[fmt]
                t = time_launches(torch, lambda i: ams.ams_linear(pk[i % len(pk)], sc, x, l.N, fmt, out=y), n_launch)
                try:
                    tws = time_launches(torch, lambda i: ams.ams_linear_static_ws(pk[i % len(pk)], sc, x, l.N, fmt, out=y), n_launch)
                except ams.AmsError:  # shape beyond the static scratch: that entry point does not take it
                    tws = None
                tb = t if tws is None else min(t, tws)
                rows.append({"layer": l.name, "N": l.N, "K": l.K, "M": Mb, "fmt": FMT_NAMES[fmt], "us": round(t, 3),
                             "us_static_ws": None if tws is None else round(tws, 3),
                             "GBps": round(l.canon[fmt] / t / 1e3, 1), "fp16_us": round(t16, 3), "fp16_ws_us": round(t16ws, 3),
                             "library_gemm_fp16_us": round(tlib, 3), "speedup_vs_fp16": round(t16 / t, 3),
                             "speedup_vs_best_fp16": round(best16 / t, 3), "speedup_static_ws_vs_best_fp16": None if tws is None else round(best16 / tws, 3),
                             "best_speedup_vs_best_fp16": round(best16 / tb, 3)})
    return rows


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import __graft_entry__

    __graft_entry__.ensure_built()  # loads what is built; a tree with no library gets one built first
    import paper_2510_16045_amd as ams
    from paper_2510_16045_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    ams.load_library()
    torch.cuda.set_device(0)
    ams.ams_init()  # every kernel's LDS limit raised before anything is captured in a graph

    shapes = {"8b": synth.LLAMA8B_LAYERS, "70b": synth.LLAMA70B_LAYERS, "qwen": synth.QWEN_DOWN_LAYERS}[args.layers]
    if args.profile_kernel:
        profile_kernel(args, shapes, torch, ams, synth)
        return
    maker = synth.heavy_tail_weights if args.layers == "70b" else synth.gaussian_weights
    t_setup = time.perf_counter()
    fmts = (ams.FP533, ams.FP425)  # the step: the two formats the paper builds kernels for
    all_fmts = (ams.FP6, ams.FP533, ams.FP5, ams.FP45, ams.FP433, ams.FP425, ams.FP4) if args.all_formats else fmts
    layers, n_copies = build_layers(shapes, maker, 100, all_fmts, args.copies_mb, ams, torch)
    print(f"# setup {time.perf_counter() - t_setup:.1f}s, {n_copies} packed copies per layer", file=sys.stderr)

    ws = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda")

    def linear(packed, scales, x, N, fmt, out):
        if not args.workspace:
            return ams.ams_linear(packed, scales, x, N, fmt, out=out)
        return ams.ams_linear_ws(packed, scales, x, N, fmt, ws, out=out)

    def fp16_linear(w, x, out):
        return ams.ams_fp16_linear(w, x, out=out) if not args.workspace else ams.ams_fp16_linear_ws(w, x, ws, out=out)

    M = 1
    xs = {l.name: to_dev(synth.activations(M, l.K, 7), torch) for l in layers}
    ys = {l.name: torch.empty((M, l.N), dtype=torch.float16, device="cuda") for l in layers}

    def step(i):
        for l in layers:
            for fmt in fmts:
                linear(l.packed[fmt][i % n_copies], l.scales[fmt], xs[l.name], l.N, fmt, ys[l.name])

    # ---- the contract's timed region: W warm-up steps, K timed steps, sync on both sides.
    # One HIP graph per rotating copy holds the eight launches of a step; a step is one graph replay.
    graphs = []
    step(0)
    torch.cuda.synchronize()
    for c in range(n_copies):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step(c)
        graphs.append(g)
    # a box that has been idle needs a moment of load before its clocks are up (untimed, before the
    # W warm-up steps: without it the first figures of a fresh process come out up to 15 % low)
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < CLOCK_RAMP_S:
        for c in range(n_copies):
            graphs[c].replay()
        torch.cuda.synchronize()
    for i in range(args.warmup):
        graphs[i % n_copies].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        graphs[i % n_copies].replay()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    step_bytes = sum(l.canon[fmt] for l in layers for fmt in fmts)
    value = step_bytes / (wall / args.steps) / 1e9
    del graphs

    # ---- per-layer figures (each Linear alone, back to back, rotating copies)
    per_layer = []
    n_launch = 8 * n_copies
    for l in layers:
        t16 = time_launches(torch, lambda i: fp16_linear(l.w16[i % len(l.w16)], xs[l.name], ys[l.name]), n_launch)
        tlib = time_launches(torch, lambda i: torch.matmul(xs[l.name], l.w16[i % len(l.w16)].t(), out=ys[l.name]), n_launch)
        for fmt in all_fmts:
            t, pct = time_launches(torch, lambda i: linear(l.packed[fmt][i % len(l.packed[fmt])], l.scales[fmt], xs[l.name], l.N, fmt, ys[l.name]), n_launch, replays=10, spread=True)
            warm = time_launches(torch, lambda i: linear(l.packed[fmt][0], l.scales[fmt], xs[l.name], l.N, fmt, ys[l.name]), n_launch)
            # second denominator: a bare read of the same packed bytes (same rotation), nothing computed
            t_read = time_launches(torch, lambda i: ams.ams_read_probe(l.packed[fmt][i % len(l.packed[fmt])]), n_launch)
            t_grouped = None
            if args.group_scales:
                sg = 96 if fmt in (ams.FP533, ams.FP433, ams.FP6) else 128
                gp, gs = ams.ams_pack_grouped(fmt, l.W, sg)
                gpd = [to_dev(gp, torch)]
                gpd += [gpd[0].clone() for _ in range(n_copies - 1)]
                gsd = to_dev(gs.reshape(-1), torch)
                t_grouped = time_launches(torch, lambda i: ams.ams_linear_grouped(gpd[i % n_copies], gsd, sg, xs[l.name], l.N, fmt, out=ys[l.name]), n_launch)
                del gpd, gsd
            gbps = l.canon[fmt] / t / 1e3
            per_layer.append(
                {
                    "layer": l.name, "N": l.N, "K": l.K, "M": M, "fmt": FMT_NAMES[fmt],
                    "us": round(t, 3), "us_percentiles": pct, "us_cache_resident": round(warm, 3),
                    "bare_read_us": round(t_read, 3), "frac_of_bare_read": round(t_read / t, 4),
                    "us_group_scales": None if t_grouped is None else round(t_grouped, 3),
                    "packed_bytes": l.canon[fmt], "allocated_bytes": ams.ams_packed_bytes(fmt, l.N, l.K),
                    "GBps": round(gbps, 1), "hbm_frac": round(gbps / HBM_PEAK_GBPS, 4),
                    "fp16_us": round(t16, 3), "fp16_GBps": round(2 * l.N * l.K / t16 / 1e3, 1),
                    "speedup_vs_fp16": round(t16 / t, 3),
                    "library_gemm_fp16_us": round(tlib, 3),
                    "speedup_vs_best_fp16": round(min(t16, tlib) / t, 3),
                }
            )

    # ---- roofline of the dominant kernel: the launch that moves the most bytes
    dom = max((r for r in per_layer if r["fmt"] in (FMT_NAMES[0], FMT_NAMES[1])), key=lambda r: r["packed_bytes"])
    dl = next(l for l in layers if l.name == dom["layer"])
    dfmt = next(f for f, n in FMT_NAMES.items() if n == dom["fmt"])
    alg_bytes = dl.canon[dfmt] + 2 * dl.N + 2 * M * dl.K + 2 * M * dl.N
    t_dom = time_launches(torch, lambda i: linear(dl.packed[dfmt][i % len(dl.packed[dfmt])], dl.scales[dfmt], xs[dl.name], dl.N, dfmt, ys[dl.name]), n_launch, replays=20)
    achieved = alg_bytes / t_dom / 1e3
    roofline = {
        "bound": "hbm", "kernel": f"column_kernel<{dom['fmt']}> {dl.N}x{dl.K} M={M}",
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "us_per_launch": round(t_dom, 3), "algorithmic_bytes": alg_bytes,
        "traffic": measured_traffic(ams, dl.name, dom["fmt"], M) if args.layers == "8b" else None,
    }

    # launch floor: an empty launch of the Linear kernel's shape (256 workgroups x 1024 threads)
    launch_floor = time_launches(torch, lambda i: ams.ams_read_probe(layers[0].packed[fmts[0]][0], 0), n_launch)

    # ---- batch sweep (Table 3's columns): gate/up and down of the 8B set unless told otherwise
    sweep = None
    if not args.no_sweep:
        sweep_layers = layers if (args.sweep_all_layers or args.layers != "8b") else [l for l in layers if l.name in ("gate_up", "down")]
        sweep = batch_sweep(sweep_layers, all_fmts, ams, torch, synth, n_launch, ws)
        if args.out:
            with open(args.out, "w") as f:
                json.dump({"layers": args.layers, "sweep": sweep}, f, indent=1)

    # ---- larger layers, each set built, timed and freed by itself
    def measure_set(shape_set, maker, seed, batches, label):
        t_setup = time.perf_counter()
        big, _ = build_layers(shape_set, maker, seed, fmts, args.copies_mb, ams, torch)
        print(f"# {label} setup {time.perf_counter() - t_setup:.1f}s", file=sys.stderr)
        rows = []
        for l in big:
            for Mb in batches:
                x = to_dev(synth.activations(Mb, l.K, 11), torch)
                y = torch.empty((Mb, l.N), dtype=torch.float16, device="cuda")
                nl = 4 * max(len(l.w16), 2)
                t16 = time_launches(torch, lambda i: ams.ams_fp16_linear(l.w16[i % len(l.w16)], x, out=y), nl)
                tlib = time_launches(torch, lambda i: torch.matmul(x, l.w16[i % len(l.w16)].t(), out=y), nl)
                for fmt in fmts:
                    pk, sc = l.packed[fmt], l.scales[fmt]
                    nl = 4 * max(len(pk), 2)
                    t = time_launches(torch, lambda i: ams.ams_linear(pk[i % len(pk)], sc, x, l.N, fmt, out=y), nl)
                    try:
                        tws = time_launches(torch, lambda i: ams.ams_linear_static_ws(pk[i % len(pk)], sc, x, l.N, fmt, out=y), nl)
                    except ams.AmsError:
                        tws = None
                    t_read = time_launches(torch, lambda i: ams.ams_read_probe(pk[i % len(pk)]), nl) if Mb == 1 else None
                    gbps = l.canon[fmt] / t / 1e3
                    rows.append({"layer": l.name, "N": l.N, "K": l.K, "M": Mb, "fmt": FMT_NAMES[fmt], "us": round(t, 3),
                                 "us_static_ws": None if tws is None else round(tws, 3),
                                 "bare_read_us": None if t_read is None else round(t_read, 3),
                                 "GBps": round(gbps, 1), "hbm_frac": round(gbps / HBM_PEAK_GBPS, 4),
                                 "fp16_us": round(t16, 3), "library_gemm_fp16_us": round(tlib, 3),
                                 "speedup_vs_fp16": round(t16 / t, 3), "speedup_vs_best_fp16": round(min(t16, tlib) / t, 3)})
        del big
        gc.collect()
        torch.cuda.empty_cache()
        return rows

    llama70b = lm_head = qwen_down = None
    if args.layers == "8b" and not (args.no_70b and args.no_lm_head and args.no_qwen):
        del layers, dl, xs, ys
        l = None
        gc.collect()
        torch.cuda.empty_cache()
        # the Llama-70B-shaped layers (heavy-tailed weights with outliers) at M = 1, 4, 8
        if not args.no_70b:
            llama70b = measure_set(synth.LLAMA70B_LAYERS, synth.heavy_tail_weights, 200, (1, 4, 8), "70B")
        # the output projection onto the vocabulary, the largest Linear of a Llama-3-8B decode step
        if not args.no_lm_head:
            lm_head = measure_set({"lm_head": synth.LLAMA8B_LM_HEAD}, synth.gaussian_weights, 300, (1, 8), "lm_head")
        # the MLP down projections the paper's efficiency table is measured on, at its batch sizes
        if not args.no_qwen:
            t_setup = time.perf_counter()
            qw, _ = build_layers(synth.QWEN_DOWN_LAYERS, synth.gaussian_weights, 400, fmts, args.copies_mb, ams, torch)
            print(f"# qwen setup {time.perf_counter() - t_setup:.1f}s", file=sys.stderr)
            qwen_down = batch_sweep(qw, fmts, ams, torch, synth, n_launch, ws, batches=(1, 4, 16, 32))
            del qw
            gc.collect()
            torch.cuda.empty_cache()

    cpu = None if args.no_cpu_baseline else cpu_baseline(synth.LLAMA8B_LAYERS)

    line = {
        "metric": "packed_weight_GBps", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {
            "workload": f"Llama-3-8B decode-step Linear set (qkv 6144x4096, o 4096x4096, gate/up 28672x4096, down 4096x14336), M=1, "
                        f"FP5.33-e2m3 + FP4.25-e2m2, weights N(0,0.02), per-row fp16 scales, cold HBM ({n_copies} rotating copies)"
            if args.layers == "8b" else f"{args.layers} layer set, M=1, both formats",
            "linears_per_step": len(shapes) * len(fmts), "packed_bytes_per_step": step_bytes,
            "hbm_peak_GBps": HBM_PEAK_GBPS, "hbm_frac": round(value / HBM_PEAK_GBPS, 4),
            "fp16_baseline": "in-build ams_fp16_linear: a GEMV on the VALU at M <= 4 (rows dealt to wavefronts), the MFMA kernels above; "
                             "speedup_vs_best_fp16 takes the fastest of it, its workspace variant and the library GEMM",
            "launch_floor_us": round(launch_floor, 3), "clock_ramp_s": CLOCK_RAMP_S, "entry_point": "ams_linear_ws" if args.workspace else "ams_linear",
        },
        "roofline": roofline, "cpu_baseline": cpu, "layers": per_layer,
        # the single-Linear configuration of the baseline list (4096x4096, FP5.33-e2m3, M=1) is the `o` layer of this set
        "single_linear_4096x4096_fp533_m1": next(({"us": r["us"], "GBps": r["GBps"], "hbm_frac": r["hbm_frac"], "speedup_vs_fp16": r["speedup_vs_fp16"]}
                                                  for r in per_layer if (r["N"], r["K"], r["fmt"]) == (4096, 4096, FMT_NAMES[0])), None),
        # baseline configuration 4: us = plain ams_linear, us_static_ws = ams_linear_static_ws (K split over workgroups where it pays);
        # fp16 side: the in-build kernel without / with a workspace and the library GEMM, the fastest of the three is the denominator
        "batch_sweep": sweep,
        # baseline configuration 5: Student-t(4) x 0.02 weights with 0.1 % outliers x 20
        "llama70b": llama70b,
        # Llama-3-8B's vocabulary projection (128256 x 4096): a Linear large enough that the launch floor and the
        # epilogue stop mattering
        "lm_head": lm_head,
        # the shapes of the paper's Table 3 (MLP down of Qwen3-4B, Qwen2.5-7B, Qwen3-32B) at batch 1, 4, 16, 32; columns as in batch_sweep
        "qwen_down": qwen_down,
        "paper_context": "paper reports 2.8x / 3.2x decode speed-up over fp16 (FP5.33 / FP4.25) on an unnamed GPU of ~22 TFLOPS, 290 GB/s",
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
