#!/usr/bin/env python3
"""Benchmark of the LASAD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A prefill "step" is one lasad_forward_chunked call over the whole token grid of the chosen
workload (the decay factors are computed inside the kernel from each token's position); the
default workload is the base-size layer prefill (batch 8, 12 heads, d 64, 16x16 grid, bf16).
A decode "step" is one lasad_decode_step call for the AR-decode workload (batch 256, 20 heads,
fp32 64x64 states), walked over the 16x16 grid in raster order.  Inputs are seeded synthetic
tensors resident in HBM before the timed region.  Every step works on a different buffer set
(more than 1 GB in rotation) so that nothing is served from a cache left warm by the previous
step.  The K timed steps are captured once into a HIP graph and replayed as one submission
(the eager per-call figure is reported next to it).

Prints ONE JSON line: whole-job prefill tokens/s as `value`, the roofline of the forward
kernel, the CPU oracle timed on the host cores (`cpu_baseline`), and the decode leg under
`decode` with its own roofline and CPU baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix-core peak

# HBM bytes per step (read + write, all kernels of the step) measured with two rocprofv3 --pmc
# runs (FETCH_SIZE, WRITE_SIZE), scaled by the same counters on a 256 MiB device copy; the
# summaries are profiles/*_traffic.txt.
MEASURED_TRAFFIC_BYTES = {
    "base_prefill_16x16": 12790811,      # algorithmic 12582912
    "large_prefill_24x24": 151152333,    # algorithmic 150994944
    "highres_64x64": 305351320,          # algorithmic 201326592; the segment plan re-reads K, V once
    "ar_decode_16x16": 170453679,        # algorithmic 170393600
    # vector-decay kernels (key tied to the gate): same algorithmic bytes as the scalar ones
    "gated:base_prefill_16x16": 12839020,    # algorithmic 12582912
    "gated:large_prefill_24x24": 158462226,  # algorithmic 150994944
    "gated:highres_64x64": 201564895,        # algorithmic 201326592 (single launch, no segment plan)
    "gated:ar_decode_16x16": 170444251,      # algorithmic 170393600
    # backward of the scalar-decay forward (3 passes in one launch; operands shared through the L2 of an XCD)
    "backward:base_prefill_16x16": 23862317,     # algorithmic 22020096
    "backward:large_prefill_24x24": 394549254,   # algorithmic 264241152
    "backward:highres_64x64": 658803305,         # algorithmic 352321536
    # backward of the vector-decay forward (dq, dk make a round trip through the fp32 workspace)
    "gated_backward:base_prefill_16x16": 54266073,     # algorithmic 22020096
    "gated_backward:large_prefill_24x24": 696467867,   # algorithmic 264241152
    "gated_backward:highres_64x64": 1304421401,        # algorithmic 352321536
    # backward of the fused layer (adds the recomputed forward with o in fp32 and the bf16 round trip of d_o)
    "layer_backward:base_prefill_16x16": 89688632,     # algorithmic 22020096
    "layer_backward:large_prefill_24x24": 1153303753,  # algorithmic 264241152
    "layer_backward:highres_64x64": 1972316628,        # algorithmic 352321536
}

PREFILL_WORKLOADS = {"base_prefill": "base_prefill_16x16", "large_prefill": "large_prefill_24x24",
                     "highres_prefill": "highres_64x64"}


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=200)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--workload", default="base_prefill", choices=sorted(PREFILL_WORKLOADS))
    p.add_argument("--decode-walks", type=int, default=4, help="timed raster walks of 256 decode steps (0 = skip)")
    p.add_argument("--decode-layers", type=int, default=8, help="state sets in rotation (layers of a model)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-backward", action="store_true", help="skip the backward-pass leg")
    p.add_argument("--no-gated", action="store_true",
                   help="skip the vector-decay (per-channel gate) forward and decode legs")
    p.add_argument("--no-graph", action="store_true", help="time eager launches only")
    p.add_argument("--layout", default="bnhd", choices=["bnhd", "bhnd"],
                   help="memory order of q, k, v, o: [B, N, Hh, d] (default) or [B, Hh, N, d]")
    p.add_argument("--buffer-sets", type=int, default=0,
                   help="prefill buffer sets in rotation (0 = enough for > 1 GB; 1 = warm caches)")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run three plain 256 MiB device copies (reference dispatches of known "
                        "traffic for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return p.parse_args()


def time_region(torch, fn):
    """Run fn() between two events on the current stream; returns milliseconds."""
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1)


def capture(torch, fn):
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):     # launches go to the capturing stream (the binding reads the current stream)
        fn()
    torch.cuda.synchronize()
    return g


def bench_prefill(args, torch, lasad, wl):
    import numpy as np
    w = wl.CONFIGS[PREFILL_WORKLOADS[args.workload]]
    q, k, v, gam = wl.prefill_inputs(w, layout=args.layout)
    tq, tk, tv = (lasad.to_device(x, w.dtype) for x in (q, k, v))
    tg = torch.from_numpy(gam).cuda()
    token_heads = w.B * w.N * w.Hh
    bytes_per_launch = token_heads * 4 * w.d * 2            # q, k, v read + o written, bf16
    sets = args.buffer_sets if args.buffer_sets > 0 else max(4, min(96, -(-(1 << 30) // bytes_per_launch)))
    bufs = [(tq, tk, tv, torch.empty_like(tq))]
    for _ in range(sets - 1):
        bufs.append((tq.clone(), tk.clone(), tv.clone(), torch.empty_like(tq)))
    ws_bytes = lasad.lasad_forward_workspace_bytes(w.B, w.Hh, w.N, w.d, lasad.BF16)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda") if ws_bytes else None

    def step(i):
        a, b, c, o = bufs[i % sets]
        lasad.lasad_forward_chunked(a, b, c, tg, w.grid_h, w.grid_w, out=o, workspace=ws)

    def run(nsteps, first=0):
        for i in range(nsteps):
            step(first + i)

    run(args.warmup)
    eager_ms = time_region(torch, lambda: run(args.steps, args.warmup))
    graph_ms = None
    if not args.no_graph:
        g = capture(torch, lambda: run(args.steps, args.warmup))
        g.replay()
        graph_ms = time_region(torch, g.replay)
    total_ms = graph_ms if graph_ms is not None else eager_ms
    ms_per_step = total_ms / args.steps
    dur_s = ms_per_step * 1e-3
    tokens_per_s = w.B * w.N / dur_s
    # For information only (never `value`): the same steps issued alternately on two streams, so that the launch
    # and drain of one step overlap the other step's work, as independent batches in flight would.
    two_ms = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        ws2 = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda") if ws_bytes else None

        def run_two(nsteps, first=0):
            main = torch.cuda.current_stream()
            side.wait_stream(main)
            for i in range(nsteps):
                a, b, c, o = bufs[(first + i) % sets]
                if i % 2 == 0:
                    lasad.lasad_forward_chunked(a, b, c, tg, w.grid_h, w.grid_w, out=o, workspace=ws)
                else:
                    with torch.cuda.stream(side):
                        lasad.lasad_forward_chunked(a, b, c, tg, w.grid_h, w.grid_w, out=o, workspace=ws2)
            main.wait_stream(side)

        g2 = capture(torch, lambda: run_two(args.steps, args.warmup))
        g2.replay()
        two_ms = time_region(torch, g2.replay) / args.steps

    C = 64
    useful_flops = token_heads * (2 * w.d * (C + 1) + 4 * w.d * w.d)   # causal-useful, chunk 64
    executed_flops = token_heads * (4 * C * w.d + 4 * w.d * w.d)
    achieved_gbs = bytes_per_launch / dur_s / 1e9
    res = {
        "workload": w, "ms_per_step": ms_per_step, "tokens_per_s": tokens_per_s,
        "eager_ms_per_step": eager_ms / args.steps, "graph_ms_per_step": None if graph_ms is None else graph_ms / args.steps,
        "buffer_sets": sets, "workspace_bytes": ws_bytes, "two_streams_ms_per_step": two_ms,
        "roofline": {"bound": "hbm", "kernel": "lasad_forward_chunked", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved_gbs / HBM_PEAK_GBS,
                     "algorithmic_bytes_per_launch": bytes_per_launch,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.name)},
        "roofline_mfma": {"bound": "mfma", "achieved": useful_flops / dur_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                          "unit": "TFLOP/s", "frac": useful_flops / dur_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                          "flops_counted": "causal-useful, chunk 64",
                          "executed_frac": executed_flops / dur_s / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "inputs": (q, k, v, gam),
    }
    return res


def cpu_baseline_prefill(res, budget_s=20.0):
    """The fp64 full-mask oracle on a bounded sample of the same workload."""
    import numpy as np
    from oracle import lasad_oracle as oracle
    w = res["workload"]
    q, k, v, gam = res["inputs"]
    cores = oracle.num_threads()
    # cost model: 4 N^2 d flops per sequence at roughly 1 GFLOP/s per core
    per_seq = 4.0 * w.N * w.N * w.d / 1e9
    n_seq = int(max(cores, min(w.B * w.Hh, budget_s * cores / max(per_seq, 1e-9))))
    n_seq = min(n_seq, w.B * w.Hh)
    pairs = [(i // w.Hh, i % w.Hh) for i in np.linspace(0, w.B * w.Hh - 1, n_seq).astype(int)]
    gq, gk, gv = (np.stack([x[b, :, h, :] for b, h in pairs], axis=1)[None] for x in (q, k, v))
    lam, _ = oracle.decay_factors(gam[[h for _, h in pairs]], w.grid_h, w.grid_w, 0, w.N)
    passes, t0 = 0, time.perf_counter()
    while True:                     # whole passes over the sample until about 5 s of wall time
        oracle.forward_fullmask(gq, gk, gv, lam)
        passes += 1
        dt = time.perf_counter() - t0
        if dt > 5.0 or passes >= 200:
            break
    return {"value": passes * n_seq * w.N / w.Hh / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{n_seq} of {w.B * w.Hh} (batch, head) sequences of the workload, full {w.N}x{w.N} mask, "
                      f"{passes} pass(es), {dt:.2f} s wall; tokens/s = passes*sequences*N/heads/time"}


def bench_decode(args, torch, lasad, wl):
    w = wl.AR_DECODE
    q, k, v, gam = wl.decode_inputs(w)
    tq, tk, tv = (lasad.to_device(x, w.dtype) for x in (q, k, v))
    tg = torch.from_numpy(gam).cuda()
    L = args.decode_layers
    states = [torch.zeros((w.B, w.Hh, w.d, w.d), dtype=torch.float32, device="cuda") for _ in range(L)]
    outs = [torch.empty((w.B, w.Hh, w.d), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    n_steps = args.decode_walks * w.steps

    def run(nsteps):
        for i in range(nsteps):
            t = i % w.steps
            lasad.lasad_decode_step(tq[t], tk[t], tv[t], tg, states[i % L], w.grid_h, w.grid_w, t, out=outs[i % L])

    run(w.steps)    # one untimed walk
    eager_ms = time_region(torch, lambda: run(n_steps))
    graph_ms = None
    if not args.no_graph:
        g = capture(torch, lambda: run(n_steps))
        g.replay()
        graph_ms = time_region(torch, g.replay)
    total_ms = graph_ms if graph_ms is not None else eager_ms
    dur_s = total_ms / n_steps * 1e-3
    n_states = w.B * w.Hh
    bytes_per_launch = n_states * (2 * w.d * w.d * 4 + 4 * w.d * 2)   # state read + write, q k v o bf16
    achieved = bytes_per_launch / dur_s / 1e9
    res = {
        "workload": w.name, "value": 1.0 / dur_s, "unit": "steps/s", "tokens_per_s": w.B / dur_s,
        "ms_per_step": dur_s * 1e3, "steps_timed": n_steps, "state_sets_in_rotation": L,
        "eager_ms_per_step": eager_ms / n_steps, "graph_ms_per_step": None if graph_ms is None else graph_ms / n_steps,
        "roofline": {"bound": "hbm", "kernel": "lasad_decode_step", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": bytes_per_launch,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.name)},
    }
    # The same walk with the first positions served from a key / value cache (fewer bytes than the state while
    # t < 2 d), the state built from the cache once, and the state form for the rest.  As above every launch
    # works on the next of L buffer sets; a launch's cost depends on its position only.
    switch = min(2 * w.d, w.steps)
    # (capacity switch + 8 rows: with a power-of-two distance between the sequences' caches the first rows of all
    # caches fall on the same few memory channels and the early steps run at a fraction of the bandwidth)
    cap = switch + 8
    kcs = [torch.zeros((w.B, w.Hh, cap, w.d), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    vcs = [torch.zeros_like(kcs[0]) for _ in range(L)]
    fwd_out = torch.empty((w.B, switch, w.Hh, w.d), dtype=torch.bfloat16, device="cuda")
    as_seq = lambda c: c.permute(0, 2, 1, 3)

    def run_hybrid(nsteps):
        for i in range(nsteps):
            t, l = i % w.steps, i % L
            if t < switch:
                lasad.lasad_decode_step_cached(tq[t], tk[t], tv[t], tg, kcs[l], vcs[l], w.grid_h, w.grid_w, t, out=outs[l])
            else:
                if t == switch:
                    lasad.lasad_forward_chunked(as_seq(kcs[l][:, :, :switch]), as_seq(kcs[l][:, :, :switch]),
                                                as_seq(vcs[l][:, :, :switch]), tg, w.grid_h, w.grid_w,
                                                state_out=states[l], out=fwd_out, use_workspace=False)
                lasad.lasad_decode_step(tq[t], tk[t], tv[t], tg, states[l], w.grid_h, w.grid_w, t, out=outs[l])

    run_hybrid(w.steps)
    hyb_ms = time_region(torch, lambda: run_hybrid(n_steps))
    if not args.no_graph:
        gh = capture(torch, lambda: run_hybrid(n_steps))
        gh.replay()
        hyb_ms = time_region(torch, gh.replay)
    res["cache_then_state"] = {
        "what": f"positions 0..{switch - 1} from a k/v cache (lasad_decode_step_cached), the state built from the cache by one "
                "lasad_forward_chunked call per walk, lasad_decode_step afterwards",
        "ms_per_step": hyb_ms / n_steps, "value": n_steps / (hyb_ms * 1e-3), "unit": "steps/s",
        "speedup_vs_state_form": total_ms / hyb_ms}
    del kcs, vcs, fwd_out
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import lasad_oracle as oracle
        rows, steps = 64, w.steps    # bounded sample: 64 of 256 batch rows, one full raster walk
        state = np.zeros((rows, w.Hh, w.d, w.d))
        qs, ks, vs = (np.ascontiguousarray(x[:, :rows], dtype=np.float64) for x in (q, k, v))
        t0 = time.perf_counter()
        for t in range(steps):
            lam_t, _ = oracle.decay_factors(gam, w.grid_h, w.grid_w, t, 1)
            oracle.decode_step(qs[t], ks[t], vs[t], lam_t[:, 0], state)
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": steps / dt * rows / w.B, "unit": "steps/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"{rows} of {w.B} batch rows, {steps} raster steps (inputs pre-widened to fp64), {dt:.2f} s wall; "
                                         "steps/s scaled by rows/batch to the full batch"}
    return res


def bench_backward(args, torch, lasad, wl):
    """Backward leg: one lasad_backward_chunked call (dq, dk, dv, dgamma from q, k, v, d_o) per step over the
    prefill workload's shape, timed like the forward."""
    import numpy as np
    w = wl.CONFIGS[PREFILL_WORKLOADS[args.workload]]
    q, k, v, gam = wl.prefill_inputs(w, layout=args.layout)
    rng = np.random.default_rng(w.seed + 101)
    g = wl.store_round(rng.standard_normal(q.shape, dtype=np.float32) / np.float32(np.sqrt(w.d)), w.dtype)
    if args.layout == "bhnd":
        g = np.ascontiguousarray(g.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    tq, tk, tv, td = (lasad.to_device(x, w.dtype) for x in (q, k, v, g))
    tg = torch.from_numpy(gam).cuda()
    token_heads = w.B * w.N * w.Hh
    bytes_bwd = token_heads * 7 * w.d * 2             # q, k, v, d_o read + dq, dk, dv written, bf16
    sets = max(4, min(64, -(-(1 << 30) // bytes_bwd)))
    bufs = []
    for i in range(sets):
        ins = (tq, tk, tv, td) if i == 0 else tuple(x.clone() for x in (tq, tk, tv, td))
        bufs.append(ins + (tuple(torch.empty_like(tq) for _ in range(3)),))
    dgam = torch.empty((w.Hh,), dtype=torch.float32, device="cuda")
    ws_bytes = lasad.lasad_backward_workspace_bytes(w.B, w.Hh, w.N, w.d, lasad.BF16)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
    steps = max(1, min(args.steps, 50))

    def run(nsteps, first=0):
        for i in range(nsteps):
            a, b, c, d_o, grads = bufs[(first + i) % sets]
            lasad.lasad_backward_chunked(a, b, c, d_o, tg, w.grid_h, w.grid_w, grads=grads, dgamma=dgam, workspace=ws)

    run(min(args.warmup, 5))
    eager_ms = time_region(torch, lambda: run(steps, 5))
    graph_ms = None
    if not args.no_graph:
        g_ = capture(torch, lambda: run(steps, 5))
        g_.replay()
        graph_ms = time_region(torch, g_.replay)
    dur_s = (graph_ms if graph_ms is not None else eager_ms) / steps * 1e-3
    res = {"workload": w.name, "value": w.B * w.N / dur_s, "unit": "tokens/s", "ms_per_step": dur_s * 1e3,
           "steps_timed": steps, "eager_ms_per_step": eager_ms / steps, "workspace_bytes": ws_bytes,
           "launches_per_step": "one launch of the forward kernel over the 3 passes (dq, dv, dk; decay-gradient sums in its "
                                "epilogue) + 1 reduction kernel; few long sequences: 3 segmented passes + 2 finishing kernels",
           "roofline": {"bound": "hbm", "kernel": "lasad_backward_chunked (all launches of one call)",
                        "achieved": bytes_bwd / dur_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": bytes_bwd / dur_s / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": bytes_bwd,
                        "traffic": MEASURED_TRAFFIC_BYTES.get("backward:" + w.name)}}
    if not args.no_cpu_baseline:
        from oracle import lasad_oracle as oracle
        n_seq = min(w.B * w.Hh, 2 * oracle.num_threads())
        pairs = [(i // w.Hh, i % w.Hh) for i in np.linspace(0, w.B * w.Hh - 1, n_seq).astype(int)]
        gq, gk, gv, gg = (np.stack([x[b, :, h, :] for b, h in pairs], axis=1)[None] for x in (q, k, v, g))
        lam, _ = oracle.decay_factors(gam[[h for _, h in pairs]], w.grid_h, w.grid_w, 0, w.N)
        passes, t0 = 0, time.perf_counter()
        while True:
            oracle.backward(gq, gk, gv, lam, gg)
            passes += 1
            dt = time.perf_counter() - t0
            if dt > 3.0 or passes >= 100:
                break
        res["cpu_baseline"] = {"value": passes * n_seq * w.N / w.Hh / dt, "unit": "tokens/s", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"{n_seq} of {w.B * w.Hh} (batch, head) sequences, fp64 reverse-mode recurrence, "
                                         f"{passes} pass(es), {dt:.2f} s wall"}
    return res


def bench_gated(args, torch, lasad, wl):
    """Vector-decay legs (Section 3.4 as written, key tied to the gate): the forward over the prefill
    workload's shape and the decode step over the AR-decode shape, timed like the scalar legs."""
    import numpy as np
    w = wl.CONFIGS[PREFILL_WORKLOADS[args.workload]]
    q, _, v, _ = wl.prefill_inputs(w, layout=args.layout)
    lam = wl.gate_inputs(q.shape, w.dtype, w.seed + 7)
    if args.layout == "bhnd":
        lam = np.ascontiguousarray(lam.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    tq, tl, tv = (lasad.to_device(x, w.dtype) for x in (q, lam, v))
    token_heads = w.B * w.N * w.Hh
    bytes_fwd = token_heads * 4 * w.d * 2               # q, lambda, v read + o written, bf16
    sets = max(4, min(96, -(-(1 << 30) // bytes_fwd)))
    bufs = [(tq, tl, tv, torch.empty_like(tq))]
    for _ in range(sets - 1):
        bufs.append((tq.clone(), tl.clone(), tv.clone(), torch.empty_like(tq)))
    steps = max(1, min(args.steps, 50))

    def run(nsteps, first=0):
        for i in range(nsteps):
            a, b, c, o = bufs[(first + i) % sets]
            lasad.lasad_forward_gated(a, b, c, w.grid_h, w.grid_w, out=o)

    run(min(args.warmup, 5))
    eager_ms = time_region(torch, lambda: run(steps, 5))
    graph_ms = None
    if not args.no_graph:
        g = capture(torch, lambda: run(steps, 5))
        g.replay()
        graph_ms = time_region(torch, g.replay)
    dur_s = (graph_ms if graph_ms is not None else eager_ms) / steps * 1e-3
    # backward of the same call (dq, dlam, dv from q, gate, v, d_o; key tied to the gate)
    bwd = None
    if not args.no_backward:
        td = lasad.to_device(wl.store_round(np.random.default_rng(w.seed + 101).standard_normal(q.shape, dtype=np.float32)
                                            / np.float32(np.sqrt(w.d)), w.dtype), w.dtype)
        if args.layout == "bhnd":
            td = td.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        gsets = min(sets, 8)
        grads = [tuple(torch.empty_like(tq) for _ in range(3)) for _ in range(gsets)]
        ws_b = torch.empty((lasad.lasad_backward_gated_workspace_bytes(w.B, w.Hh, w.N, w.d),), dtype=torch.uint8, device="cuda")
        bsteps = max(1, min(steps, 20))

        def run_bwd(nsteps, first=0):
            for i in range(nsteps):
                a, b, c, _ = bufs[(first + i) % sets]
                lasad.lasad_backward_gated(a, b, c, td, w.grid_h, w.grid_w, grads=grads[(first + i) % gsets], workspace=ws_b)

        run_bwd(3)
        b_ms = time_region(torch, lambda: run_bwd(bsteps, 3))
        if not args.no_graph:
            gb = capture(torch, lambda: run_bwd(bsteps, 3))
            gb.replay()
            b_ms = time_region(torch, gb.replay)
        b_s = b_ms / bsteps * 1e-3
        bytes_bwd = token_heads * 7 * w.d * 2          # q, gate, v, d_o read + dq, dlam, dv written, bf16
        bwd = {"workload": w.name + " (q, gate, v, d_o; k = 1 - gate)", "value": w.B * w.N / b_s, "unit": "tokens/s",
               "ms_per_step": b_s * 1e3, "steps_timed": bsteps,
               "launches_per_step": "one launch of the chunked matrix-core kernel over the 3 passes (dq, dv, dk) + 1 finishing kernel "
                                    "(suffix sums for dlam)",
               "roofline": {"bound": "hbm", "kernel": "lasad_backward_gated (both launches of one call)",
                            "achieved": bytes_bwd / b_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": bytes_bwd / b_s / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": bytes_bwd,
                            "traffic": MEASURED_TRAFFIC_BYTES.get("gated_backward:" + w.name)}}
        del grads, ws_b, td
    # the same launch with Algorithm 1's elementwise steps fused in (SiLU, sigmoid, RMS norm): the gate buffers
    # now hold the pre-sigmoid logits N(2, 1) of the same recipe, q is read as the pre-SiLU query
    tz = lasad.to_device(wl.store_round(np.random.default_rng(w.seed + 7).standard_normal(q.shape, dtype=np.float32)
                                        + np.float32(2.0), w.dtype), w.dtype)
    for _, b, _, _ in bufs:
        b.copy_(tz)
    del tz

    def run_layer(nsteps, first=0):
        for i in range(nsteps):
            a, b, c, o = bufs[(first + i) % sets]
            lasad.lasad_forward_layer(a, b, c, w.grid_h, w.grid_w, out=o)

    run_layer(min(args.warmup, 5))
    layer_ms = time_region(torch, lambda: run_layer(steps, 5))
    if not args.no_graph:
        gl = capture(torch, lambda: run_layer(steps, 5))
        gl.replay()
        layer_ms = time_region(torch, gl.replay)
    # backward of the fused layer: forward recomputation (o in fp32), norm backward, the three passes with the
    # activations on load, finishing kernel with the chain rule, weight-gradient sum
    layer_bwd = None
    if not args.no_backward:
        td = lasad.to_device(wl.store_round(np.random.default_rng(w.seed + 101).standard_normal(q.shape, dtype=np.float32)
                                            / np.float32(np.sqrt(w.d)), w.dtype), w.dtype)
        gsets = min(sets, 8)
        grads = [tuple(torch.empty_like(tq) for _ in range(3)) for _ in range(gsets)]
        dwt = torch.empty((w.Hh, w.d), dtype=torch.float32, device="cuda")
        ws_l = torch.empty((lasad.lasad_backward_layer_workspace_bytes(tq),), dtype=torch.uint8, device="cuda")
        lsteps = max(1, min(steps, 20))

        def run_lbwd(nsteps, first=0):
            for i in range(nsteps):
                a, b, c, _ = bufs[(first + i) % sets]
                lasad.lasad_backward_layer(a, b, c, td, w.grid_h, w.grid_w, grads=grads[(first + i) % gsets], dweight=dwt,
                                           workspace=ws_l)

        run_lbwd(3)
        lb_ms = time_region(torch, lambda: run_lbwd(lsteps, 3))
        if not args.no_graph:
            glb = capture(torch, lambda: run_lbwd(lsteps, 3))
            glb.replay()
            lb_ms = time_region(torch, glb.replay)
        lb_s = lb_ms / lsteps * 1e-3
        bytes_lb = token_heads * 7 * w.d * 2           # q_pre, z, v, d_out read + dq_pre, dz, dv written, bf16
        layer_bwd = {"workload": w.name + " (q_pre, z, v, d_out; SiLU, sigmoid gate, tied key, RMS norm)",
                     "value": w.B * w.N / lb_s, "unit": "tokens/s", "ms_per_step": lb_s * 1e3, "steps_timed": lsteps,
                     "launches_per_step": "forward recomputation + norm backward + 3-pass kernel + finishing kernel + weight-gradient sum",
                     "roofline": {"bound": "hbm", "kernel": "lasad_backward_layer (all launches of one call)",
                                  "achieved": bytes_lb / lb_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                  "frac": bytes_lb / lb_s / 1e9 / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": bytes_lb,
                                  "traffic": MEASURED_TRAFFIC_BYTES.get("layer_backward:" + w.name)}}
        del grads, ws_l, td, dwt
    res = {"forward": {
        "workload": w.name + " (q, gate, v; k = 1 - gate)",
        "fused_layer_ms_per_step": layer_ms / steps, "value": w.B * w.N / dur_s, "unit": "tokens/s",
        "ms_per_step": dur_s * 1e3, "steps_timed": steps, "eager_ms_per_step": eager_ms / steps,
        "roofline": {"bound": "hbm", "kernel": "lasad_forward_gated", "achieved": bytes_fwd / dur_s / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bytes_fwd / dur_s / 1e9 / HBM_PEAK_GBS,
                     "algorithmic_bytes_per_launch": bytes_fwd,
                     "traffic": MEASURED_TRAFFIC_BYTES.get("gated:" + w.name)}}}
    if bwd is not None:
        res["backward"] = bwd
    if layer_bwd is not None:
        res["layer_backward"] = layer_bwd
    if not args.no_cpu_baseline:
        from oracle import lasad_oracle as oracle
        n_seq = min(w.B * w.Hh, 4 * oracle.num_threads())
        pairs = [(i // w.Hh, i % w.Hh) for i in np.linspace(0, w.B * w.Hh - 1, n_seq).astype(int)]
        gq, gl, gv = (np.stack([x[b, :, h, :] for b, h in pairs], axis=1)[None] for x in (q, lam, v))
        passes, t0 = 0, time.perf_counter()
        while True:
            oracle.gated_recurrent(gq, gl, gv, w.grid_w)
            passes += 1
            dt = time.perf_counter() - t0
            if dt > 3.0 or passes >= 200:
                break
        res["forward"]["cpu_baseline"] = {
            "value": passes * n_seq * w.N / w.Hh / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n_seq} of {w.B * w.Hh} (batch, head) sequences, fp64 recurrence, {passes} pass(es), {dt:.2f} s wall"}
    del bufs

    if args.decode_walks > 0:
        wd = wl.AR_DECODE
        dq, _, dv, _ = wl.decode_inputs(wd)
        dl = wl.gate_inputs(dq.shape, wd.dtype, wd.seed + 7)
        tq, tl, tv = (lasad.to_device(x, wd.dtype) for x in (dq, dl, dv))
        L = args.decode_layers
        states = [torch.zeros((wd.B, wd.Hh, wd.d, wd.d), dtype=torch.float32, device="cuda") for _ in range(L)]
        outs = [torch.empty((wd.B, wd.Hh, wd.d), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
        n_steps = args.decode_walks * wd.steps

        def drun(nsteps):
            for i in range(nsteps):
                t = i % wd.steps
                lasad.lasad_decode_step_gated(tq[t], tl[t], tv[t], states[i % L], wd.grid_h, wd.grid_w, t, out=outs[i % L])

        drun(wd.steps)
        eager_ms = time_region(torch, lambda: drun(n_steps))
        graph_ms = None
        if not args.no_graph:
            g = capture(torch, lambda: drun(n_steps))
            g.replay()
            graph_ms = time_region(torch, g.replay)
        dur_s = (graph_ms if graph_ms is not None else eager_ms) / n_steps * 1e-3
        bytes_dec = wd.B * wd.Hh * (2 * wd.d * wd.d * 4 + 4 * wd.d * 2)
        res["decode"] = {
            "workload": wd.name + " (q, gate, v; k = 1 - gate)", "value": 1.0 / dur_s, "unit": "steps/s",
            "ms_per_step": dur_s * 1e3, "steps_timed": n_steps, "eager_ms_per_step": eager_ms / n_steps,
            "roofline": {"bound": "hbm", "kernel": "lasad_decode_step_gated", "achieved": bytes_dec / dur_s / 1e9,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bytes_dec / dur_s / 1e9 / HBM_PEAK_GBS,
                         "algorithmic_bytes_per_launch": bytes_dec,
                         "traffic": MEASURED_TRAFFIC_BYTES.get("gated:" + wd.name)}}
    return res


def measure_copy_peak(torch):
    """Streaming ceiling of this GPU as a plain device copy reaches it: 1 GiB read + 1 GiB written per copy."""
    n = 1 << 30
    src = torch.empty((n,), dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    reps = 10
    ms = time_region(torch, lambda: [dst.copy_(src) for _ in range(reps)])
    del src, dst
    return 2.0 * n * reps / (ms * 1e-3) / 1e9


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (single process, no collectives); "
              f"--gpus {args.gpus} is not supported, use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2507_01652_amd import binding as lasad, workloads as wl
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    lasad.load()

    if args.calibrate_copy:
        src = torch.empty((256 << 20,), dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # one elementwise copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    copy_gbs = measure_copy_peak(torch)
    pre = bench_prefill(args, torch, lasad, wl)
    w = pre["workload"]
    line = {
        "metric": "lasad_prefill_tokens_per_s", "value": pre["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": pre["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": w.B, "heads": w.Hh, "head_dim": w.d,
                   "grid": [w.grid_h, w.grid_w], "tokens_per_step": w.B * w.N, "chunk": 64,
                   "io": "bf16 q,k,v in, bf16 o out, fp32 accumulation", "layout": args.layout,
                   "timing": "HIP graph replay of the timed steps" if pre["graph_ms_per_step"] is not None else "eager launches",
                   "buffer_sets_in_rotation": pre["buffer_sets"]},
        "eager_ms_per_step": pre["eager_ms_per_step"],
        "two_streams_ms_per_step": pre["two_streams_ms_per_step"],     # information only: two independent steps in flight
        "roofline": pre["roofline"], "roofline_mfma": pre["roofline_mfma"],
        "hbm_copy_measured": {"value": copy_gbs, "unit": "GB/s",
                              "what": "1 GiB device-to-device copy (read + written bytes over time), the streaming rate a "
                                      "plain copy kernel reaches on this GPU; roofline.frac stays against the published 8 TB/s"},
    }
    line["roofline"]["frac_of_measured_copy"] = line["roofline"]["achieved"] / copy_gbs
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline_prefill(pre)
    if args.decode_walks > 0:
        line["decode"] = bench_decode(args, torch, lasad, wl)
        line["decode"]["roofline"]["frac_of_measured_copy"] = line["decode"]["roofline"]["achieved"] / copy_gbs
    if not args.no_backward:
        line["backward"] = bench_backward(args, torch, lasad, wl)
    if not args.no_gated:
        line["gated"] = bench_gated(args, torch, lasad, wl)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
