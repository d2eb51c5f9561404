#!/usr/bin/env python3
"""Benchmark of the LASAD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--legs a,b]

A prefill "step" is one lasad_forward_chunked call over the whole token grid of a workload (the
decay factors are computed inside the kernel from each token's position).  The headline workload
is the large-size layer prefill (batch 32, 16 heads, d 64, 24x24 grid, bf16: the 384-pixel
generation shape); the base-size (16x16) and the high-resolution (64x64) prefill are timed the
same way as nested legs, and the three together give the time per token-head against the
sequence length (`linear_in_n`).  A decode "step" is one lasad_decode_step call for the
AR-decode workload (batch 256, 20 heads, fp32 64x64 states), walked over the 16x16 grid in
raster order.

Inputs are seeded synthetic tensors resident in HBM before the timed region.  Cold caches,
whatever K is: every step works on the next of several buffer sets (more than 1 GB in rotation),
and before every timed region a 1 GiB copy sweeps the caches (the last-level cache holds 256 MB),
so that nothing a step reads was left there by an earlier step, the warm-up or the capture.  The
K timed steps are captured once into a HIP graph and replayed as one submission; the figure is
the median of several such replays, each after its own sweep (the eager per-call figure is
reported next to it).  Timing is by HIP events on the stream the kernels run on.

Prints ONE JSON line: whole-job prefill tokens/s of the headline workload as `value`, the
roofline of its forward kernel, the CPU oracle timed on the host cores (`cpu_baseline`), the
other prefill shapes under `prefill_legs`, `linear_in_n`, and the decode, backward and
vector-decay legs with their own rooflines and CPU baselines.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix-core peak

PREFILL_WORKLOADS = {"base_prefill": "base_prefill_16x16", "large_prefill": "large_prefill_24x24",
                     "highres_prefill": "highres_64x64"}

# rocprofv3 --pmc summaries (FETCH_SIZE + WRITE_SIZE per step, scaled on a copy of known size) of earlier runs
# of this file; `roofline.traffic` quotes them, it is not measured in the run that prints the line.
TRAFFIC_FILES = {
    "forward": "forward_mfma_{w}_traffic.txt",
    "decode": "decode_kernel_{w}_traffic.txt",
    "gated": "forward_gated_mfma_{w}_traffic.txt",
    "gated_decode": "decode_kernel_gated_{w}_traffic.txt",
    "backward": "backward_{w}_traffic.txt",
    "gated_backward": "backward_gated_{w}_traffic.txt",
    "layer_backward": "backward_layer_{w}_traffic.txt",
}


def measured_traffic(kind: str, workload: str):
    """HBM bytes per step from profiles/<kernel>_<workload>_traffic.txt, or None if there is no such summary."""
    path = os.path.join(ROOT, "profiles", TRAFFIC_FILES[kind].format(w=workload))
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"HBM traffic per step.*?=\s*(\d+)\s*bytes", text)
    return int(m.group(1)) if m else None


def parse(argv=None):
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=40)
    p.add_argument("--warmup", type=int, default=10)
    p.add_argument("--workload", default="large_prefill", choices=sorted(PREFILL_WORKLOADS),
                   help="headline prefill workload (also the shape of the backward and vector-decay legs)")
    p.add_argument("--legs", default="base_prefill,highres_prefill",
                   help="other prefill workloads timed as nested legs (comma separated, '' = none)")
    p.add_argument("--replays", type=int, default=5, help="timed graph replays per figure (the median is reported)")
    p.add_argument("--decode-walks", type=int, default=4, help="timed raster walks of 256 decode steps (0 = skip)")
    p.add_argument("--decode-layers", type=int, default=8, help="state sets in rotation (layers of a model)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-backward", action="store_true", help="skip the backward-pass legs")
    p.add_argument("--no-gated", action="store_true",
                   help="skip the vector-decay (per-channel gate) forward, backward and decode legs")
    p.add_argument("--no-small-gamma", action="store_true",
                   help="skip the leg that times the headline shape with every head's decay below the chunked form's range")
    p.add_argument("--no-graph", action="store_true", help="time eager launches only")
    p.add_argument("--layout", default="bnhd", choices=["bnhd", "bhnd"],
                   help="memory order of q, k, v, o: [B, N, Hh, d] (default) or [B, Hh, N, d]")
    p.add_argument("--buffer-sets", type=int, default=0,
                   help="prefill buffer sets in rotation (0 = enough for > 1 GB; 1 with --warm = warm caches)")
    p.add_argument("--warm", action="store_true", help="no cache sweep before the timed regions (for comparison)")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run three plain 256 MiB device copies (reference dispatches of known "
                        "traffic for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return p.parse_args(argv)


class Timer:
    """Event timing of step sequences on torch's current stream, with a cache sweep before every timed region."""

    def __init__(self, torch, args):
        self.torch, self.args = torch, args
        self.sweep_src = self.sweep_dst = None
        if not args.warm:
            n = 512 << 20          # 512 MiB read + 512 MiB written: four times the last-level cache
            self.sweep_src = torch.empty((n,), dtype=torch.uint8, device="cuda").fill_(1)
            self.sweep_dst = torch.empty_like(self.sweep_src)

    def sweep(self):
        if self.sweep_src is not None:
            self.sweep_dst.copy_(self.sweep_src)

    def region(self, fn):
        """Milliseconds of fn() between two events on the current stream, after a cache sweep."""
        torch = self.torch
        torch.cuda.synchronize()
        self.sweep()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def steps(self, run, steps, warmup):
        """run(n, first) issues steps first .. first+n-1.  Returns (ms per step, eager ms per step, replay list):
        `warmup` untimed steps, `steps` eager steps timed once, then the same steps as a HIP graph replayed
        args.replays times (median)."""
        torch = self.torch
        run(warmup, 0)
        eager = self.region(lambda: run(steps, warmup)) / steps
        if self.args.no_graph:
            return eager, eager, None
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):     # launches go to the capturing stream (the binding reads the current stream)
            run(steps, warmup)
        torch.cuda.synchronize()
        g.replay()                    # untimed: the first replay uploads the graph
        reps = [self.region(g.replay) / steps for _ in range(max(1, self.args.replays))]
        return statistics.median(reps), eager, reps


def n_sets(args, bytes_per_step, cap=96):
    return args.buffer_sets if args.buffer_sets > 0 else max(4, min(cap, -(-(1 << 30) // bytes_per_step)))


def hbm_roofline(kernel, bytes_per_launch, dur_s, traffic):
    achieved = bytes_per_launch / dur_s / 1e9
    return {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": bytes_per_launch,
            "traffic": traffic, "traffic_source": "profiles/ (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE of an earlier "
                                                  "run of this file; not measured in this run)"}


def bench_prefill(args, timer, torch, lasad, wl, name):
    w = wl.CONFIGS[PREFILL_WORKLOADS[name]]
    q, k, v, gam = wl.prefill_inputs(w, layout=args.layout)
    tq, tk, tv = (lasad.to_device(x, w.dtype) for x in (q, k, v))
    tg = torch.from_numpy(gam).cuda()
    token_heads = w.B * w.N * w.Hh
    bytes_per_launch = token_heads * 4 * w.d * 2            # q, k, v read + o written, bf16
    sets = n_sets(args, bytes_per_launch)
    bufs = [(tq, tk, tv, torch.empty_like(tq))]
    for _ in range(sets - 1):
        bufs.append((tq.clone(), tk.clone(), tv.clone(), torch.empty_like(tq)))
    ws_bytes = lasad.lasad_forward_workspace_bytes(w.B, w.Hh, w.N, w.d, lasad.BF16)
    ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda") if ws_bytes else None

    def run(nsteps, first=0):
        for i in range(nsteps):
            a, b, c, o = bufs[(first + i) % sets]
            lasad.lasad_forward_chunked(a, b, c, tg, w.grid_h, w.grid_w, out=o, workspace=ws)

    ms_per_step, eager_ms, reps = timer.steps(run, args.steps, args.warmup)
    dur_s = ms_per_step * 1e-3
    C = 64
    useful_flops = token_heads * (2 * w.d * (C + 1) + 4 * w.d * w.d)   # causal-useful, chunk 64
    executed_flops = token_heads * (4 * C * w.d + 4 * w.d * w.d)
    res = {
        "workload": w.name, "value": w.B * w.N / dur_s, "unit": "tokens/s", "ms_per_step": ms_per_step,
        "steps": args.steps, "eager_ms_per_step": eager_ms, "replays_ms_per_step": reps,
        "ns_per_token_head": dur_s * 1e9 / token_heads,
        "config": {"workload": w.name, "batch": w.B, "heads": w.Hh, "head_dim": w.d,
                   "grid": [w.grid_h, w.grid_w], "tokens_per_step": w.B * w.N, "chunk": 64,
                   "io": "bf16 q,k,v in, bf16 o out, fp32 accumulation", "layout": args.layout,
                   "timing": ("eager launches" if reps is None else
                              f"HIP graph replay of the timed steps, median of {len(reps)} replays") +
                             ("" if args.warm else ", caches swept before every timed region"),
                   "buffer_sets_in_rotation": sets, "workspace_bytes": ws_bytes},
        "roofline": hbm_roofline("lasad_forward_chunked", bytes_per_launch, dur_s, measured_traffic("forward", w.name)),
        "roofline_mfma": {"bound": "mfma", "achieved": useful_flops / dur_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                          "unit": "TFLOP/s", "frac": useful_flops / dur_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                          "flops_counted": "causal-useful, chunk 64",
                          "executed_frac": executed_flops / dur_s / 1e12 / MFMA_BF16_PEAK_TFLOPS},
    }
    del bufs, ws
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline_prefill(w, (q, k, v, gam))
    return res


def bench_small_gamma(args, timer, torch, lasad, wl, name, headline_ms):
    """What a head costs whose decay is outside the range of the chunked form (gamma <= 0.5: the separable in-chunk
    factors would overflow, so the workgroup of such a head walks its sequence with the fp32 recurrence inside the
    same launch).  No paper-shaped workload has such heads; the leg exists so that the cost is on record: every
    head of the headline shape gets gamma = 0.4 here."""
    w = wl.CONFIGS[PREFILL_WORKLOADS[name]]
    q, k, v, _ = wl.prefill_inputs(w, layout=args.layout)
    tq, tk, tv = (lasad.to_device(x, w.dtype) for x in (q, k, v))
    tg = torch.full((w.Hh,), 0.4, dtype=torch.float32, device="cuda")
    # (fp32 output: another instantiation of the kernel, so that a kernel trace of this run keeps the headline
    # kernel's row free of these launches; the walk costs the same)
    o = torch.empty_like(tq, dtype=torch.float32)

    def run(nsteps, first=0):
        for _ in range(nsteps):
            lasad.lasad_forward_chunked(tq, tk, tv, tg, w.grid_h, w.grid_w, out=o, use_workspace=False)

    for _ in range(2):
        run(1)
    ms = timer.region(lambda: run(4)) / 4
    return {"workload": w.name, "gamma": 0.4, "ms_per_step": ms, "slowdown_vs_headline": ms / headline_ms,
            "what": "every head on the fp32 token-serial recurrence (decay outside the chunked form's range); fp32 output, eager launches"}


def cpu_baseline_prefill(w, inputs, budget_s=20.0):
    """The fp64 full-mask oracle on a bounded sample of the same workload."""
    import numpy as np
    from oracle import lasad_oracle as oracle
    q, k, v, gam = inputs
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


def bench_decode(args, timer, torch, lasad, wl):
    w = wl.AR_DECODE
    q, k, v, gam = wl.decode_inputs(w)
    tq, tk, tv = (lasad.to_device(x, w.dtype) for x in (q, k, v))
    tg = torch.from_numpy(gam).cuda()
    L = args.decode_layers
    states = [torch.zeros((w.B, w.Hh, w.d, w.d), dtype=torch.float32, device="cuda") for _ in range(L)]
    outs = [torch.empty((w.B, w.Hh, w.d), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    n_steps = args.decode_walks * w.steps

    def run(nsteps, first=0):
        for i in range(first, first + nsteps):
            t = i % w.steps
            lasad.lasad_decode_step(tq[t], tk[t], tv[t], tg, states[i % L], w.grid_h, w.grid_w, t, out=outs[i % L])

    ms_per_step, eager_ms, reps = timer.steps(run, n_steps, w.steps)     # one untimed walk first
    dur_s = ms_per_step * 1e-3
    n_states = w.B * w.Hh
    bytes_per_launch = n_states * (2 * w.d * w.d * 4 + 4 * w.d * 2)   # state read + write, q k v o bf16
    res = {
        "workload": w.name, "value": 1.0 / dur_s, "unit": "steps/s", "tokens_per_s": w.B / dur_s,
        "ms_per_step": ms_per_step, "steps_timed": n_steps, "state_sets_in_rotation": L,
        "eager_ms_per_step": eager_ms, "replays_ms_per_step": reps,
        "roofline": hbm_roofline("lasad_decode_step", bytes_per_launch, dur_s, measured_traffic("decode", w.name)),
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

    def run_hybrid(nsteps, first=0):
        for i in range(first, first + nsteps):
            t, l = i % w.steps, i % L
            if t < switch:
                lasad.lasad_decode_step_cached(tq[t], tk[t], tv[t], tg, kcs[l], vcs[l], w.grid_h, w.grid_w, t, out=outs[l])
            else:
                if t == switch:
                    lasad.lasad_forward_chunked(as_seq(kcs[l][:, :, :switch]), as_seq(kcs[l][:, :, :switch]),
                                                as_seq(vcs[l][:, :, :switch]), tg, w.grid_h, w.grid_w,
                                                state_out=states[l], out=fwd_out, use_workspace=False)
                lasad.lasad_decode_step(tq[t], tk[t], tv[t], tg, states[l], w.grid_h, w.grid_w, t, out=outs[l])

    hyb_ms, _, _ = timer.steps(run_hybrid, n_steps, w.steps)
    res["cache_then_state"] = {
        "what": f"positions 0..{switch - 1} from a k/v cache (lasad_decode_step_cached), the state built from the cache by one "
                "lasad_forward_chunked call per walk, lasad_decode_step afterwards",
        "ms_per_step": hyb_ms, "value": 1.0 / (hyb_ms * 1e-3), "unit": "steps/s",
        "speedup_vs_state_form": ms_per_step / hyb_ms}
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


def bench_backward(args, timer, torch, lasad, wl):
    """Backward leg: one lasad_backward_chunked call (dq, dk, dv, dgamma from q, k, v, d_o) per step over the
    headline workload's shape, timed like the forward."""
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
    sets = n_sets(args, bytes_bwd, cap=64)
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

    ms_per_step, eager_ms, reps = timer.steps(run, steps, min(args.warmup, 5))
    dur_s = ms_per_step * 1e-3
    res = {"workload": w.name, "value": w.B * w.N / dur_s, "unit": "tokens/s", "ms_per_step": ms_per_step,
           "steps_timed": steps, "eager_ms_per_step": eager_ms, "workspace_bytes": ws_bytes,
           "launches_per_step": "one launch of the forward kernel over the 3 passes (dq, dv, dk; decay-gradient sums in its "
                                "epilogue) + 1 reduction kernel; few long sequences: 3 segmented passes + 2 finishing kernels",
           "roofline": hbm_roofline("lasad_backward_chunked (all launches of one call)", bytes_bwd, dur_s,
                                    measured_traffic("backward", w.name))}
    del bufs, ws
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


def bench_gated(args, timer, torch, lasad, wl):
    """Vector-decay legs (Section 3.4 as written, key tied to the gate): the forward over the headline
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
    sets = n_sets(args, bytes_fwd)
    bufs = [(tq, tl, tv, torch.empty_like(tq))]
    for _ in range(sets - 1):
        bufs.append((tq.clone(), tl.clone(), tv.clone(), torch.empty_like(tq)))
    steps = max(1, min(args.steps, 50))
    warm = min(args.warmup, 5)

    def run(nsteps, first=0):
        for i in range(nsteps):
            a, b, c, o = bufs[(first + i) % sets]
            lasad.lasad_forward_gated(a, b, c, w.grid_h, w.grid_w, out=o)

    fwd_ms, eager_ms, _ = timer.steps(run, steps, warm)
    dur_s = fwd_ms * 1e-3
    # backward of the same call (dq, dlam, dv from q, gate, v, d_o; key tied to the gate)
    bwd = None
    bytes_bwd = token_heads * 7 * w.d * 2          # four tensors read + three gradients written, bf16
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

        b_ms, _, _ = timer.steps(run_bwd, bsteps, 3)
        b_s = b_ms * 1e-3
        bwd = {"workload": w.name + " (q, gate, v, d_o; k = 1 - gate)", "value": w.B * w.N / b_s, "unit": "tokens/s",
               "ms_per_step": b_ms, "steps_timed": bsteps,
               "launches_per_step": "one launch of the chunked matrix-core kernel over the 3 passes (dq, dv, dk) + 1 finishing kernel "
                                    "(suffix sums for dlam)",
               "roofline": hbm_roofline("lasad_backward_gated (both launches of one call)", bytes_bwd, b_s,
                                        measured_traffic("gated_backward", w.name))}
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

    layer_ms, _, _ = timer.steps(run_layer, steps, warm)
    # backward of the fused layer: forward recomputation, norm backward, the three passes with the
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

        lb_ms, _, _ = timer.steps(run_lbwd, lsteps, 3)
        lb_s = lb_ms * 1e-3
        layer_bwd = {"workload": w.name + " (q_pre, z, v, d_out; SiLU, sigmoid gate, tied key, RMS norm)",
                     "value": w.B * w.N / lb_s, "unit": "tokens/s", "ms_per_step": lb_ms, "steps_timed": lsteps,
                     "launches_per_step": "forward recomputation + norm backward + 3-pass kernel + finishing kernel + weight-gradient sum",
                     "roofline": hbm_roofline("lasad_backward_layer (all launches of one call)", bytes_bwd, lb_s,
                                              measured_traffic("layer_backward", w.name))}
        del grads, ws_l, td, dwt
    res = {"forward": {
        "workload": w.name + " (q, gate, v; k = 1 - gate)",
        "fused_layer_ms_per_step": layer_ms, "value": w.B * w.N / dur_s, "unit": "tokens/s",
        "ms_per_step": fwd_ms, "steps_timed": steps, "eager_ms_per_step": eager_ms,
        "roofline": hbm_roofline("lasad_forward_gated", bytes_fwd, dur_s, measured_traffic("gated", w.name))}}
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

        def drun(nsteps, first=0):
            for i in range(first, first + nsteps):
                t = i % wd.steps
                lasad.lasad_decode_step_gated(tq[t], tl[t], tv[t], states[i % L], wd.grid_h, wd.grid_w, t, out=outs[i % L])

        d_ms, d_eager, _ = timer.steps(drun, n_steps, wd.steps)
        dur_s = d_ms * 1e-3
        bytes_dec = wd.B * wd.Hh * (2 * wd.d * wd.d * 4 + 4 * wd.d * 2)
        res["decode"] = {
            "workload": wd.name + " (q, gate, v; k = 1 - gate)", "value": 1.0 / dur_s, "unit": "steps/s",
            "ms_per_step": d_ms, "steps_timed": n_steps, "eager_ms_per_step": d_eager,
            "roofline": hbm_roofline("lasad_decode_step_gated", bytes_dec, dur_s, measured_traffic("gated_decode", wd.name))}
        # the first positions from gate / value caches (tied key: two rows per cached token, as for the scalar decay)
        switch = min(2 * wd.d, wd.steps)
        cap = switch + 8                   # (not a power-of-two distance between the sequences' caches: see bench_decode)
        lcs = [torch.zeros((wd.B, wd.Hh, cap, wd.d), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
        vcs = [torch.zeros_like(lcs[0]) for _ in range(L)]
        for c in lcs:       # a set sees every L-th step only: the rows its own steps do not write hold the walk's gates too
            c[:, :, :switch] = tl[:switch].permute(1, 2, 0, 3)     # (zero gates would send the state build to its range fallback)
        fwd_out = torch.empty((wd.B, switch, wd.Hh, wd.d), dtype=torch.bfloat16, device="cuda")
        as_seq = lambda c: c.permute(0, 2, 1, 3)

        def dhybrid(nsteps, first=0):
            for i in range(first, first + nsteps):
                t, l = i % wd.steps, i % L
                if t < switch:
                    lasad.lasad_decode_step_gated_cached(tq[t], tl[t], tv[t], lcs[l], vcs[l], wd.grid_h, wd.grid_w, t, out=outs[l])
                else:
                    if t == switch:
                        # (only state_out is wanted: the query operand is a stand-in with the caches' layout)
                        lasad.lasad_forward_gated(as_seq(lcs[l][:, :, :switch]), as_seq(lcs[l][:, :, :switch]),
                                                  as_seq(vcs[l][:, :, :switch]), wd.grid_h, wd.grid_w,
                                                  state_out=states[l], out=fwd_out)
                    lasad.lasad_decode_step_gated(tq[t], tl[t], tv[t], states[l], wd.grid_h, wd.grid_w, t, out=outs[l])

        h_ms, _, _ = timer.steps(dhybrid, n_steps, wd.steps)
        res["decode"]["cache_then_state"] = {
            "what": f"positions 0..{switch - 1} from gate / value caches (lasad_decode_step_gated_cached), the state built from "
                    "the caches by one lasad_forward_gated call per walk, lasad_decode_step_gated afterwards",
            "ms_per_step": h_ms, "value": 1.0 / (h_ms * 1e-3), "unit": "steps/s",
            "speedup_vs_state_form": d_ms / h_ms}
        del lcs, vcs, fwd_out
    return res


def measure_copy_peak(torch, timer):
    """Streaming ceiling of this GPU as a plain device copy reaches it: 1 GiB read + 1 GiB written per copy."""
    n = 1 << 30
    src = torch.empty((n,), dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    reps = 10
    ms = timer.region(lambda: [dst.copy_(src) for _ in range(reps)])
    del src, dst
    return 2.0 * n * reps / (ms * 1e-3) / 1e9


def measure_stream_3r1w(torch, timer, shape):
    """The traffic mix of the forward (three bf16 tensors read, one written) as one plain elementwise kernel
    (torch.addcmul) over tensors of the headline workload's size, cold caches, rotating buffer sets: the rate a
    streaming kernel without any of the method's structure reaches on this mix."""
    n_sets = 8
    bufs = [tuple(torch.ones(shape, dtype=torch.bfloat16, device="cuda") for _ in range(4)) for _ in range(n_sets)]
    steps = 16

    def run():
        for i in range(steps):
            a, b, c, o = bufs[i % n_sets]
            torch.addcmul(a, b, c, out=o)

    run()
    ms = min(timer.region(run) for _ in range(3)) / steps
    nbytes = 4 * bufs[0][0].numel() * 2
    del bufs
    return {"value": nbytes / (ms * 1e-3) / 1e9, "unit": "GB/s", "ms_per_step": ms,
            "what": "torch.addcmul(q, k, v, out=o) on bf16 tensors of the headline workload's size (3 read + 1 written, "
                    "the forward's algorithmic bytes), eager launches, cold caches"}


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

    timer = Timer(torch, args)
    copy_gbs = measure_copy_peak(torch, timer)
    pre = bench_prefill(args, timer, torch, lasad, wl, args.workload)
    line = {
        "metric": "lasad_prefill_tokens_per_s", "value": pre["value"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": pre["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": pre["config"],
        "eager_ms_per_step": pre["eager_ms_per_step"], "replays_ms_per_step": pre["replays_ms_per_step"],
        "roofline": pre["roofline"], "roofline_mfma": pre["roofline_mfma"],
        "hbm_copy_measured": {"value": copy_gbs, "unit": "GB/s",
                              "what": "1 GiB device-to-device copy (read + written bytes over time), the streaming rate a "
                                      "plain copy kernel reaches on this GPU; roofline.frac stays against the published 8 TB/s"},
    }
    line["roofline"]["frac_of_measured_copy"] = line["roofline"]["achieved"] / copy_gbs
    w0 = wl.CONFIGS[PREFILL_WORKLOADS[args.workload]]
    line["hbm_stream_3r1w_measured"] = measure_stream_3r1w(torch, timer, (w0.B, w0.N, w0.Hh, w0.d))
    line["roofline"]["frac_of_measured_stream_3r1w"] = line["roofline"]["achieved"] / line["hbm_stream_3r1w_measured"]["value"]
    if "cpu_baseline" in pre:
        line["cpu_baseline"] = pre["cpu_baseline"]
    legs = {pre["workload"]: pre}
    for name in [x for x in args.legs.split(",") if x and x != args.workload]:
        if name not in PREFILL_WORKLOADS:
            raise SystemExit(f"bench.py: unknown prefill leg {name!r}")
        leg = bench_prefill(args, timer, torch, lasad, wl, name)
        leg["roofline"]["frac_of_measured_copy"] = leg["roofline"]["achieved"] / copy_gbs
        legs[leg["workload"]] = leg
    line["prefill_legs"] = {k: v for k, v in legs.items() if k != pre["workload"]}
    # time per token-head against the sequence length: the method is linear in N (Section 1, Section 3.2), so the
    # figures of the shapes that fill the GPU should agree
    per = {k: {"n_tokens": v["config"]["grid"][0] * v["config"]["grid"][1], "ns_per_token_head": v["ns_per_token_head"],
               "frac_hbm": v["roofline"]["frac"]} for k, v in legs.items()}
    line["linear_in_n"] = {"per_workload": per, "unit": "ns per token-head (one head's token: 512 B moved)"}
    if "large_prefill_24x24" in per and "highres_64x64" in per:
        line["linear_in_n"]["highres_over_large"] = (per["highres_64x64"]["ns_per_token_head"] /
                                                     per["large_prefill_24x24"]["ns_per_token_head"])
    if not args.no_small_gamma:
        line["small_gamma_fallback"] = bench_small_gamma(args, timer, torch, lasad, wl, args.workload, pre["ms_per_step"])
    if args.decode_walks > 0:
        line["decode"] = bench_decode(args, timer, torch, lasad, wl)
        line["decode"]["roofline"]["frac_of_measured_copy"] = line["decode"]["roofline"]["achieved"] / copy_gbs
    if not args.no_backward:
        line["backward"] = bench_backward(args, timer, torch, lasad, wl)
    if not args.no_gated:
        line["gated"] = bench_gated(args, timer, torch, lasad, wl)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
