#!/usr/bin/env python3
"""Benchmark of the 3-D linear layer's per-rank hot path on one MI355X.

A step is one pass of the hot path over one batch of synthetic input that is
already resident in HBM: the forward product P = X_il W_lj and the two backward
products Q = dY_ij W_lj^T and R = X_il^T dY_ij of one processor of the q^3 cube
(Algorithm 1 step 3, Algorithm 2 lines 1-2).  The headline workload is the
MFMA-bound configuration (q = 4, hidden 8192 MLP up-projection, one processor's
share at its real shape); the other configurations are reported beside it.

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused:
this build runs on one GPU.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "fp8_e4m3": 5000.0, "f32": 157.3}   # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0

# name -> (q, M, K, N, in dtype, out dtype of the partial products, description)
RANK_SHARE = {
    "config2": (4, 8192, 2048, 8192, "bf16", "bf16",
                "one rank's share, q=4, MLP up-proj h=2048->8192, tokens 8192: X_il [2048,512] W_lj [512,2048] "
                "dY_ij [2048,2048], bf16 in, fp32 accumulate, bf16 out"),
    "config4": (4, 32768, 8192, 32768, "bf16", "bf16",
                "one rank's share, q=4, MLP up-proj h=8192->32768, tokens 32768: X_il [8192,2048] W_lj [2048,8192] "
                "dY_ij [8192,8192], bf16 in, fp32 accumulate, bf16 out"),
    "config5": (8, 16384, 12288, 49152, "fp8_e4m3", "bf16",
                "one rank's share, q=8, MLP up-proj h=12288->49152, tokens 16384: X_il [2048,1536] W_lj [1536,6144] "
                "dY_ij [2048,6144], fp8 e4m3 in with per-tensor scales, fp32 accumulate, bf16 out"),
}
CONFIG3 = [("qkv", 2048, 6144, "y"), ("attn_out", 2048, 2048, "z"), ("mlp_up", 2048, 8192, "y"),
           ("mlp_down", 8192, 2048, "z")]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="config4", choices=sorted(RANK_SHARE))
    ap.add_argument("--dist", default="normal", choices=["normal", "uniform", "zeros"],
                    help="operand distribution of the headline workload: the configuration's own (N(0,1) activations and "
                         "gradients, N(0,0.02) weights), uniform[-1,1), or all zeros (the achieved rate depends on the data: "
                         "the shader clock under the matrix cores does)")
    ap.add_argument("--repeats", type=int, default=5, help="measurements per reported figure (the median is reported)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU time aimed at by the cpu_baseline sample")
    ap.add_argument("--config3-linear", default=None, choices=[c[0] for c in CONFIG3],
                    help="restrict the config-3 virtual cube to one linear (clean per-kernel profiler counters)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference for scaling profiler byte counters)")
    return ap.parse_args()


def csrc_digest():
    """Digest of the kernel sources: ties a stored profiler figure to the code it was measured on."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2105_14450_amd", "csrc", "*")) +
                       glob.glob(os.path.join(ROOT, "include", "*.h"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


def median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2105_14450_amd as c3
    from paper_2105_14450_amd import synth
    if not os.path.exists(c3.binding.LIB_PATH):
        from paper_2105_14450_amd import build as _b
        _b.build()
    c3.binding.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    c3.cube3d_init()
    stream = torch.cuda.current_stream()
    REP = max(1, args.repeats)

    store = {"f32": torch.float32, "bf16": torch.int16, "fp8_e4m3": torch.uint8}

    def dev(raw):
        raw = np.ascontiguousarray(raw)
        if raw.dtype == np.uint16:
            raw = raw.view(np.int16)
        return torch.from_numpy(raw).cuda()

    def timed_once(fn, iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(iters):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    def timed(fn, iters):
        """Milliseconds per call of fn(): `iters` back-to-back calls between two HIP events on the launch
        stream, median of REP such measurements."""
        fn()
        torch.cuda.synchronize()
        return median([timed_once(fn, iters) for _ in range(REP)])

    def timed_graph(fn, iters):
        """Same, with the `iters` launches replayed from one HIP graph (no host launch gaps)."""
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for _ in range(iters):
                    fn()
        g.replay()
        torch.cuda.synchronize()
        return median([timed_once(g.replay, 1) for _ in range(REP)]) / iters

    def rank_share(name, seed, dist="normal", copies=1):
        """One processor's three products of a configuration.  copies > 1: that many separate sets of
        operand and result buffers (same values), for launches that never find their data in a cache."""
        q, M, K, N, dt, odt, desc = RANK_SHARE[name]
        Mb, Kb, Nb = M // q, K // q, N // q
        if dist == "zeros":
            z = lambda shape: synth.store(np.zeros(shape, dtype=np.float32), dt, True)
            X, W, G = z((Mb, Kb)), z((Kb, Nb)), z((Mb, Nb))
        else:
            sw = 0.02 if dist == "normal" else 1.0
            X = synth.store(synth.draw((Mb, Kb), dist, seed, synth.TID_X), dt)
            W = synth.store(synth.draw((Kb, Nb), dist, seed, synth.TID_W, sw), dt)
            G = synth.store(synth.draw((Mb, Nb), dist, seed, synth.TID_DY), dt)
        d = c3.make_desc(q, M, K, N, in_dtype=c3.binding.DTYPE_CODES[dt], out_dtype=c3.binding.DTYPE_CODES[odt],
                         scale_x=X[1], scale_w=W[1], scale_dy=G[1])
        sets = []
        for _ in range(copies):
            sets.append({"X": dev(X[0]), "W": dev(W[0]), "G": dev(G[0]),
                         "P": torch.empty((Mb, Nb), dtype=store[odt], device="cuda"),
                         "Q": torch.empty((Mb, Kb), dtype=store[odt], device="cuda"),
                         "R": torch.empty((Kb, Nb), dtype=store[odt], device="cuda")})
        ws = {}
        for op in (c3.OP_FWD, c3.OP_BWD_DX, c3.OP_BWD_DW):
            n = c3.cube3d_workspace_bytes(d, op, False)
            ws[op] = torch.empty(n, dtype=torch.uint8, device="cuda") if n else None
        rank = (1, 2, 3)

        def make(t):
            return {
                "fwd": lambda: c3.cube3d_linear_fwd(d, rank, t["X"], t["W"], t["P"], ws[c3.OP_FWD]),
                "bwd_dx": lambda: c3.cube3d_linear_bwd_dx(d, rank, t["G"], t["W"], t["Q"], ws[c3.OP_BWD_DX]),
                "bwd_dw": lambda: c3.cube3d_linear_bwd_dw(d, rank, t["X"], t["G"], t["R"], ws[c3.OP_BWD_DW]),
            }
        ops = [make(t) for t in sets]
        flop = 2.0 * Mb * Kb * Nb
        host = {"X": X, "W": W, "G": G}
        set_bytes = sum(v.numel() * v.element_size() for v in sets[0].values())
        return (ops[0] if copies == 1 else ops), flop, (Mb, Kb, Nb), desc, dt, host, set_bytes

    ORDER = ("fwd", "bwd_dx", "bwd_dw")
    SEEDS = {"config2": 2, "config4": 4, "config5": 5}

    # ---- headline workload ------------------------------------------------------------------------
    ops, flop, (Mb, Kb, Nb), desc, dt, host, _ = rank_share(args.workload, SEEDS[args.workload], args.dist)

    def step():
        for k in ORDER:
            ops[k]()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # exactly `steps` steps between two events, synchronised on both sides; REP such measurements,
    # the median is reported (all of them are listed in config.ms_per_step_repeats)
    plain_ms = []
    for _ in range(REP):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(args.steps):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        plain_ms.append(e0.elapsed_time(e1) / args.steps)
    ms_per_step = median(plain_ms)
    value = 3.0 * flop / (ms_per_step * 1e-3) / 1e12

    # Per-kernel launch durations, measured live IN STEP ORDER: an event behind every launch of REP more
    # passes of `steps` steps, so each kernel finds the caches as the step leaves them (a loop over one
    # product alone keeps its whole working set in the 256 MB Infinity Cache and reads faster than it
    # runs inside the step).  Duration of a launch = time between the events around it on the launch
    # stream; reported: the median over all REP * steps launches of that kernel.
    per = {k: [] for k in ORDER}
    step_ms = []
    for _ in range(REP):
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(ORDER) + 1)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        for row in evs:
            row[0].record(stream)
            for j, k in enumerate(ORDER):
                ops[k]()
                row[j + 1].record(stream)
        torch.cuda.synchronize()
        for row in evs:
            for j, k in enumerate(ORDER):
                per[k].append(row[j].elapsed_time(row[j + 1]))
        step_ms.append(evs[0][0].elapsed_time(evs[-1][-1]) / args.steps)
    kern = {}
    for k in ORDER:
        ms = median(per[k])
        kern[k] = {"avg_us": round(ms * 1e3, 2), "tflops": round(flop / (ms * 1e-3) / 1e12, 1),
                   "frac_of_peak": round(flop / (ms * 1e-3) / 1e12 / PEAK_TFLOPS[dt], 4)}
    dom = max(kern, key=lambda k: kern[k]["avg_us"])
    # HBM traffic of the dominant kernel from the stored profiler counters, only if they were measured
    # on these very kernel sources and this operand distribution
    traffic, traffic_note = None, "no stored counters"
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % args.workload)
    if os.path.exists(tpath):
        try:
            tj = json.load(open(tpath))
            if tj.get("csrc_digest") != csrc_digest():
                traffic_note = "stored counters are from other kernel sources (digest %s)" % tj.get("csrc_digest")
            elif args.dist != "normal":
                traffic_note = "stored counters are for the configuration's own operand distribution"
            else:
                traffic = tj["bytes_per_launch"].get(dom)
                traffic_note = "rocprofv3 FETCH_SIZE + WRITE_SIZE per launch, measured at source digest %s" % tj["csrc_digest"]
        except Exception as exc:
            traffic_note = "unreadable: %r" % (exc,)
    roofline = {"bound": "mfma", "kernel": dom, "achieved": kern[dom]["tflops"], "peak": PEAK_TFLOPS[dt],
                "unit": "TFLOP/s", "frac": kern[dom]["frac_of_peak"], "traffic": traffic, "traffic_note": traffic_note,
                "flop_per_launch": flop, "avg_launch_us": kern[dom]["avg_us"],
                "timing": "median of %d launches timed in step order by HIP events" % len(per[dom])}

    out = {
        "metric": "per-rank 3-D linear fwd+bwd TFLOP/s (bf16)" if dt == "bf16" else
                  "per-rank 3-D linear fwd+bwd TFLOP/s (%s)" % dt,
        "value": round(value, 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp8_e4m3": "fp8", "f32": "f32"}[dt], "data": "synthetic",
        "config": {"workload": args.workload + ": " + desc, "rank_block": [Mb, Kb, Nb], "operands": args.dist,
                   "step": "fwd + bwd_dx + bwd_dw, 3 launches", "frac_of_bf16_peak": round(value / PEAK_TFLOPS["bf16"], 4),
                   "ms_per_step_repeats": [round(v, 4) for v in plain_ms],
                   "ms_per_step_with_events_between_kernels": round(median(step_ms), 4), "csrc_digest": csrc_digest()},
        "roofline": roofline,
        "kernels": kern,
    }

    if args.copy_calibration:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    # ---- the other configurations (short runs) ------------------------------------------------------
    if not args.no_extra:
        extra = {}
        for name in sorted(RANK_SHARE):
            if name == args.workload:
                continue
            try:
                extra[name] = bench_small_config(name, SEEDS[name], rank_share, timed, timed_graph, timed_once, torch, REP)
                torch.cuda.empty_cache()
            except Exception as exc:   # a failed side run must not lose the headline line
                extra[name] = {"error": repr(exc)}
        try:
            extra["config3"] = bench_virtual_cube(c3, synth, torch, np, timed, args.config3_linear)
        except Exception as exc:
            extra["config3"] = {"error": repr(exc)}
        if args.config3_linear is None:
            try:
                extra["config3"]["layer_chain"] = bench_layer_chain(c3, torch, stream, REP)
            except Exception as exc:
                extra["config3"]["layer_chain"] = {"error": repr(exc)}
        out["per_config"] = extra

    # ---- the oracle on the host cores, bounded sample -------------------------------------------------
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(host, dt, args.cpu_seconds)

    print(json.dumps(out))
    return 0


def bench_small_config(name, seed, rank_share, timed, timed_graph, timed_once, torch, REP):
    """A configuration whose launches may be shorter than 20 us: per product the graph-replayed time on
    one set of buffers (which then sits in the caches: `avg_us`), and a cold figure (`cold_us`): the same
    launches replayed from a graph that walks through enough separate buffer sets (> 512 MB in all, twice
    the Infinity Cache) that no launch finds its operands in a cache."""
    o, f, blk, _, d2, _h, set_bytes = rank_share(name, seed)
    r = {}
    small = f < 5e10
    for k, fn in o.items():
        ms = timed_graph(fn, 50) if small else timed(fn, 20)
        r[k] = {"avg_us": round(ms * 1e3, 2), "tflops": round(f / (ms * 1e-3) / 1e12, 1)}
    r["fwd_bwd_tflops"] = round(3 * f / sum(v["avg_us"] for v in r.values()) / 1e6, 1)
    r["frac_of_bf16_peak"] = round(r["fwd_bwd_tflops"] / PEAK_TFLOPS["bf16"], 4)
    r["frac_of_own_peak"] = round(r["fwd_bwd_tflops"] / PEAK_TFLOPS[d2], 4)
    r["dtype"] = d2
    if small:
        # dX and dW of one layer do not depend on each other: as two branches of the graph (two streams) their
        # launches overlap where neither fills the chip.  Reported beside the one-stream figures, not in them.
        s1 = torch.cuda.Stream()

        def pair():
            cur = torch.cuda.current_stream()
            s1.wait_stream(cur)
            with torch.cuda.stream(s1):
                o["bwd_dx"]()
            o["bwd_dw"]()
            cur.wait_stream(s1)
        us = timed_graph(pair, 50) * 1e3
        r["bwd_pair_two_streams"] = {"avg_us": round(us, 2),
                                     "fwd_bwd_tflops": round(3 * f / (r["fwd"]["avg_us"] + us) / 1e6, 1)}
    r["timing"] = "median of %d graph replays of 50 launches each" % REP if small else "median of %d loops of 20 launches" % REP
    del o
    if small:
        copies = int((512 << 20) // set_bytes) + 2
        sets, f, _, _, _, _, _ = rank_share(name, seed, copies=copies)
        cold = {}
        for k in ("fwd", "bwd_dx", "bwd_dw"):
            def walk(k=k):
                for ops in sets:
                    ops[k]()
            ms = timed_graph(walk, 1) / copies
            cold[k] = round(ms * 1e3, 2)
        r["cold_us"] = cold
        r["cold_fwd_bwd_tflops"] = round(3 * f / sum(cold.values()) / 1e6, 1)
        r["cold_buffer_sets"] = copies
        del sets
    return r


def bench_virtual_cube(c3, synth, torch, np, timed, only=None):
    """Config 3: the four linears of one Transformer layer on the 64-processor virtual cube (q = 4,
    8192 tokens, bf16): batched products over all ranks plus the on-HBM gathers and reduce-scatters."""
    q, M = 4, 8192
    n = q ** 3
    res = {}
    tot_flop, tot_ms = 0.0, 0.0
    cube_flop, cube_ms = 0.0, 0.0
    for name, K, N, ax in CONFIG3:
        if only is not None and name != only:
            continue
        in_axis = c3.AXIS_Y if ax == "y" else c3.AXIS_Z
        out_axis = c3.AXIS_Z if ax == "y" else c3.AXIS_Y
        d = c3.make_desc(q, M, K, N, in_dtype=c3.BF16, out_dtype=c3.F32, shard_dtype=c3.BF16, in_axis=in_axis)
        Mb, Kb, Nb, Ms, Ns = M // q, K // q, N // q, M // q ** 2, N // q ** 2
        i16, f32 = torch.int16, torch.float32
        g = torch.Generator(device="cuda").manual_seed(31)
        mk = lambda shape, s: (torch.randn(shape, device="cuda", generator=g) * s).to(torch.bfloat16).view(i16)
        xs, ws, gs = mk((n, Ms, Kb), 1.0), mk((n, Kb, Ns), 0.02), mk((n, Ms, Nb), 1.0)
        xb = torch.empty((n, Mb, Kb), dtype=i16, device="cuda")
        wb = torch.empty((n, Kb, Nb), dtype=i16, device="cuda")
        gb = torch.empty((n, Mb, Nb), dtype=i16, device="cuda")
        big = max(Mb * Nb, Mb * Kb, Kb * Nb)
        buf = torch.empty((n * big,), dtype=f32, device="cuda")   # partial products of all three passes
        P = buf[: n * Mb * Nb].view(n, Mb, Nb)
        ysh = torch.empty((n, Ms, Nb), dtype=i16, device="cuda")
        wsb = {}
        for op in (c3.OP_FWD, c3.OP_BWD_DX, c3.OP_BWD_DW):
            nb = c3.cube3d_workspace_bytes(d, op, True)
            wsb[op] = torch.empty(nb, dtype=torch.uint8, device="cuda") if nb else None
        r = {}
        flop = 2.0 * Mb * Kb * Nb * n
        steps = {
            "gather_x": (lambda: c3.virtual_cube_gather(d, c3.OPERAND_X, in_axis, xs, xb), (1 + q) * xs.numel() * 2),
            "gather_w": (lambda: c3.virtual_cube_gather(d, c3.OPERAND_W, c3.AXIS_X, ws, wb), (1 + q) * ws.numel() * 2),
            "gather_dy": (lambda: c3.virtual_cube_gather(d, c3.OPERAND_DY, out_axis, gs, gb), (1 + q) * gs.numel() * 2),
            "fwd": (lambda: c3.cube3d_linear_fwd(d, c3.ALL_RANKS, xb, wb, P, wsb[c3.OP_FWD]), None),
            "reduce_scatter_y": (lambda: c3.virtual_cube_reduce_scatter(d, c3.OPERAND_Y, out_axis, P, ysh),
                                 P.numel() * 4 + ysh.numel() * 2),
        }
        for k, (fn, nbytes) in steps.items():
            fn()
            ms = timed(fn, 10)
            if nbytes is None:
                r[k] = {"avg_us": round(ms * 1e3, 1), "tflops": round(flop / (ms * 1e-3) / 1e12, 1)}
                tot_flop += flop
                tot_ms += ms
            else:
                r[k] = {"avg_us": round(ms * 1e3, 1), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                        "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)}
        Qv = buf[: n * Mb * Kb].view(n, Mb, Kb)
        Rv = buf[: n * Kb * Nb].view(n, Kb, Nb)
        dxsh = torch.empty((n, Ms, Kb), dtype=i16, device="cuda")
        dwsh = torch.empty((n, Kb, Ns), dtype=i16, device="cuda")
        for k, fn, nbytes in (
                ("bwd_dx", lambda: c3.cube3d_linear_bwd_dx(d, c3.ALL_RANKS, gb, wb, Qv, wsb[c3.OP_BWD_DX]), None),
                ("reduce_scatter_dx", lambda: c3.virtual_cube_reduce_scatter(d, c3.OPERAND_DX, in_axis, Qv, dxsh),
                 Qv.numel() * 4 + dxsh.numel() * 2),
                ("bwd_dw", lambda: c3.cube3d_linear_bwd_dw(d, c3.ALL_RANKS, xb, gb, Rv, wsb[c3.OP_BWD_DW]), None),
                ("reduce_scatter_dw", lambda: c3.virtual_cube_reduce_scatter(d, c3.OPERAND_DW, c3.AXIS_X, Rv, dwsh),
                 Rv.numel() * 4 + dwsh.numel() * 2)):
            fn()
            ms = timed(fn, 10)
            if nbytes is None:
                r[k] = {"avg_us": round(ms * 1e3, 1), "tflops": round(flop / (ms * 1e-3) / 1e12, 1)}
                tot_flop += flop
                tot_ms += ms
            else:
                r[k] = {"avg_us": round(ms * 1e3, 1), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                        "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)}
        # bias (Algorithms 7-8): block gather, reduce-scatter with the add fused, gradient from the dY shards
        b_diag = torch.randn((n, Ns), device="cuda", generator=g)
        b_blk = torch.empty((n, Nb), dtype=f32, device="cuda")
        db = torch.empty((n, Ns), dtype=f32, device="cuda")
        db_ws = torch.empty(c3.cube3d_workspace_bytes(d, c3.OP_BIAS_BWD, True), dtype=torch.uint8, device="cuda")
        for k, fn, nbytes in (
                ("bias_gather", lambda: c3.virtual_cube_bias_gather(d, b_diag, b_blk), (q * q * Ns + n * Nb) * 4),
                ("reduce_scatter_y_bias", lambda: c3.virtual_cube_reduce_scatter_bias(d, out_axis, P, b_blk, ysh),
                 P.numel() * 4 + ysh.numel() * 2 + b_blk.numel() * 4),
                ("bias_bwd", lambda: c3.virtual_cube_bias_bwd(d, gs, db, db_ws), gs.numel() * 2 + q * q * Ns * 4)):
            fn()
            ms = timed(fn, 10)
            r[k] = {"avg_us": round(ms * 1e3, 1), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                    "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)}
        # the same three passes as ONE product each over the whole cube, shards read and written in
        # place (no gathered copies, no partial products): flop as above, bytes = operands + result once
        fused_ms = {}
        for k, fn in (("cube_fwd_bias", lambda: c3.virtual_cube_linear_fwd(d, xs, ws, b_diag, ysh)),
                      ("cube_bwd_dx", lambda: c3.virtual_cube_linear_bwd_dx(d, gs, ws, dxsh)),
                      ("cube_bwd_dw", lambda: c3.virtual_cube_linear_bwd_dw(d, xs, gs, dwsh))):
            fn()
            ms = timed(fn, 10)
            fused_ms[k] = ms
            r[k] = {"avg_us": round(ms * 1e3, 1), "tflops": round(flop / (ms * 1e-3) / 1e12, 1)}
        cube_flop += 3 * flop
        cube_ms += sum(fused_ms.values())
        # time of the same work through explicit collectives: gathers + batched product + reduce-scatter
        r["speedup_vs_collective_path"] = {
            "fwd": round((r["gather_x"]["avg_us"] + r["gather_w"]["avg_us"] + r["fwd"]["avg_us"] +
                          r["reduce_scatter_y_bias"]["avg_us"]) / r["cube_fwd_bias"]["avg_us"], 2),
            "bwd_dx": round((r["gather_dy"]["avg_us"] + r["gather_w"]["avg_us"] + r["bwd_dx"]["avg_us"] +
                             r["reduce_scatter_dx"]["avg_us"]) / r["cube_bwd_dx"]["avg_us"], 2),
            "bwd_dw": round((r["gather_x"]["avg_us"] + r["gather_dy"]["avg_us"] + r["bwd_dw"]["avg_us"] +
                             r["reduce_scatter_dw"]["avg_us"]) / r["cube_bwd_dw"]["avg_us"], 2)}
        res[name] = r
        del xs, ws, gs, xb, wb, gb, P, ysh, Qv, Rv, buf, dxsh, dwsh, b_diag, b_blk, db
        torch.cuda.empty_cache()
    res["products_tflops"] = round(tot_flop / (tot_ms * 1e-3) / 1e12, 1)
    res["frac_of_bf16_peak"] = round(res["products_tflops"] / PEAK_TFLOPS["bf16"], 4)
    res["cube_products_tflops"] = round(cube_flop / (cube_ms * 1e-3) / 1e12, 1)
    res["cube_frac_of_bf16_peak"] = round(res["cube_products_tflops"] / PEAK_TFLOPS["bf16"], 4)
    return res


def bench_layer_chain(c3, torch, stream, REP=5):
    """The four linears of config 3 as one chained layer step on the 64-processor virtual cube, forward and
    backward, in-place cube products with bias, the direction exchange between consecutive linears
    (y, z, y, z) and the activation between the two MLP linears: timed eagerly and as one captured graph."""
    q, M = 4, 8192
    n = q ** 3
    i16, f32 = torch.int16, torch.float32
    g = torch.Generator(device="cuda").manual_seed(33)
    mk = lambda shape, s: (torch.randn(shape, device="cuda", generator=g) * s).to(torch.bfloat16).view(i16)
    new = lambda shape, dt=i16: torch.empty(shape, dtype=dt, device="cuda")
    L = {}
    flop = 0.0
    for name, K, N, ax in CONFIG3:
        d = c3.make_desc(q, M, K, N, in_dtype=c3.BF16, out_dtype=c3.F32, shard_dtype=c3.BF16,
                         in_axis=c3.AXIS_Y if ax == "y" else c3.AXIS_Z)
        Kb, Nb, Ms, Ns = K // q, N // q, M // q ** 2, N // q ** 2
        L[name] = dict(d=d, x=mk((n, Ms, Kb), 1.0), w=mk((n, Kb, Ns), 0.02), b=torch.randn((n, Ns), device="cuda", generator=g),
                       y=new((n, Ms, Nb)), dy=mk((n, Ms, Nb), 1.0), dx=new((n, Ms, Kb)), dw=new((n, Kb, Ns)),
                       db=new((n, Ns), f32),
                       ws=new((c3.cube3d_workspace_bytes(d, c3.OP_BIAS_BWD, True),), torch.uint8))
        flop += 3 * 2.0 * M * K * N
    up, down = L["mlp_up"], L["mlp_down"]
    down["x"] = new(tuple(up["y"].shape))      # H = act(Z): the up-projection's output shards, as stored, are its input
    dz = new(tuple(up["y"].shape))

    def fwd(l):
        c3.virtual_cube_linear_fwd(l["d"], l["x"], l["w"], l["b"], l["y"])

    def bwd(l, dy):
        c3.virtual_cube_linear_bwd_dx(l["d"], dy, l["w"], l["dx"])
        c3.virtual_cube_linear_bwd_dw(l["d"], l["x"], dy, l["dw"])
        c3.virtual_cube_bias_bwd(l["d"], dy, l["db"], l["ws"])

    def step():
        fwd(L["qkv"])
        fwd(L["attn_out"])
        fwd(up)
        c3.cube3d_activation_fwd(c3.ACT_GELU, c3.BF16, c3.BF16, up["y"], down["x"])
        fwd(down)
        bwd(down, down["dy"])
        c3.cube3d_activation_bwd(c3.ACT_GELU, c3.BF16, c3.BF16, c3.BF16, up["y"], down["dx"], dz)
        bwd(up, dz)
        bwd(L["attn_out"], L["attn_out"]["dy"])
        bwd(L["qkv"], L["qkv"]["dy"])

    def timed(run, iters):
        vals = []
        for _ in range(REP):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            for _ in range(iters):
                run()
            e1.record(stream)
            torch.cuda.synchronize()
            vals.append(e0.elapsed_time(e1) / iters)
        return median(vals)

    step()
    step()
    eager_ms = timed(step, 10)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    graph.replay()
    graph_ms = timed(graph.replay, 10)
    act_n = up["y"].numel()
    act_ms = timed(lambda: c3.cube3d_activation_fwd(c3.ACT_GELU, c3.BF16, c3.BF16, up["y"], down["x"]), 10)
    actb_ms = timed(lambda: c3.cube3d_activation_bwd(c3.ACT_GELU, c3.BF16, c3.BF16, c3.BF16, up["y"], down["dx"], dz), 10)
    return {"what": "qkv, attn-out, MLP-up, GELU, MLP-down forward, then the backward of all four: in-place cube "
                    "products with bias, bf16, M = 8192 tokens, q = 4 (26 kernel launches)",
            "flop": flop, "eager_ms": round(eager_ms, 3), "graph_ms": round(graph_ms, 3),
            "tflops_graph": round(flop / (graph_ms * 1e-3) / 1e12, 1),
            "frac_of_bf16_peak": round(flop / (graph_ms * 1e-3) / 1e12 / PEAK_TFLOPS["bf16"], 4),
            "activation_fwd": {"avg_us": round(act_ms * 1e3, 1), "GBps": round(act_n * 4 / (act_ms * 1e-3) / 1e9, 1)},
            "activation_bwd": {"avg_us": round(actb_ms * 1e3, 1), "GBps": round(act_n * 6 / (actb_ms * 1e-3) / 1e9, 1)}}


def cpu_baseline(host, dt, seconds):
    """Time the CPU oracle, as it stands, on a slab of the same workload: the first `rows` rows of
    the forward and dX outputs and the first `rows_w` rows of dW, sized from a short calibration
    run so that the whole sample takes about `seconds` of wall time (at most the full step)."""
    import numpy as np

    from oracle import matmul as om
    from oracle import numfmt
    X = numfmt.decode(host["X"][0], dt, host["X"][1])
    W = numfmt.decode(host["W"][0], dt, host["W"][1])
    G = numfmt.decode(host["G"][0], dt, host["G"][1])
    threads = om.max_threads()
    try:
        threads = min(threads, len(os.sched_getaffinity(0)))
    except AttributeError:
        pass
    Mb, Kb = X.shape
    Nb = W.shape[1]
    t0 = time.time()
    om.forward(X[:64], W, threads)
    rate = 2.0 * 64 * Kb * Nb / max(time.time() - t0, 1e-6)          # flop/s, calibration only
    step_flop = 3 * 2.0 * Mb * Kb * Nb
    frac = min(1.0, rate * seconds / step_flop)
    rows = max(64, min(Mb, int(Mb * frac)))
    rows_w = max(8, min(Kb, int(Kb * frac)))
    t0 = time.time()
    om.forward(X[:rows], W, threads)
    om.backward_dx(G[:rows], W, threads)
    om.backward_dw(np.ascontiguousarray(X[:, :rows_w]), G, threads)
    dt_s = time.time() - t0
    flop = 2.0 * rows * Kb * Nb * 2 + 2.0 * Mb * rows_w * Nb
    return {"value": round(flop / dt_s / 1e12, 6), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "seconds": round(dt_s, 2),
            "sample": "fp64 triple-loop oracle on the same inputs: rows [0,%d) of the forward and dX outputs and "
                      "rows [0,%d) of dW (%.1f GFLOP of the step's %.1f)" % (rows, rows_w, flop / 1e9,
                                                                             step_flop / 1e9)}


if __name__ == "__main__":
    sys.exit(main())
