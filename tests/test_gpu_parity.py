"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element,
on the same seeded inputs.  Tolerances: max |gpu - oracle| / rms(oracle) <= 1e-5 for fp32 inputs,
2e-2 for bf16 inputs, on the bare difference of the fp32 result; the decay table is compared bit
for bit.  With bf16 inputs every call is made twice, with fp32 and with bf16 output: the fp32
result is held to the tolerance and the bf16 result must be that fp32 result rounded to nearest
even, bit for bit (helpers.both_outputs)."""
import zlib

import numpy as np
import pytest

from paper_2507_01652_amd import workloads as wl
from helpers import TOL, both_outputs, decode_both, gather_pairs, rel_err, sample_pairs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lasad():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2507_01652_amd import binding
    binding.load()          # fails loudly if liblasad.so is missing
    return binding


def _torch():
    import torch
    return torch


def _odt(name):
    torch = _torch()
    return {"bf16": torch.bfloat16, "f32": torch.float32}[name]


def _gpu_forward(lasad, w, q, k, v, g, *, start_pos=0, n=None, mode=0, q_scale=1.0, s0=None,
                 want_state=False, out_dtype=None, use_workspace=True):
    """The call with fp32 output (returned); unless fp32 output is asked for explicitly, bf16 inputs also
    run it with bf16 output, which must be the fp32 output rounded (same final state)."""
    torch = _torch()
    n = q.shape[1] if n is None else n
    tq, tk, tv = (lasad.to_device(x, w.dtype) for x in (q, k, v))
    tg = torch.from_numpy(g).cuda()
    ts0 = None if s0 is None else torch.from_numpy(np.ascontiguousarray(s0, dtype=np.float32)).cuda()
    ts1 = torch.empty((q.shape[0], q.shape[2], w.d, w.d), dtype=torch.float32, device="cuda") if want_state else None
    o = both_outputs(lasad.lasad_forward_chunked, w.dtype == "bf16" and out_dtype != torch.float32,
                     q=tq, k=tk, v=tv, gamma=tg, grid_h=w.grid_h, grid_w=w.grid_w, start_pos=start_pos,
                     boundary_mode=mode, q_scale=q_scale, state_in=ts0, state_out=ts1, use_workspace=use_workspace)
    torch.cuda.synchronize()
    o = o.cpu().numpy()
    return (o, ts1.cpu().numpy()) if want_state else o


# ------------------------------------------------------------------ decay table (bit-exact)

@pytest.mark.parametrize("H,W,start,n", [(2, 3, 0, 6), (16, 16, 0, 256), (24, 24, 0, 576), (64, 64, 0, 4096),
                                         (5, 7, 9, 20), (1, 13, 0, 13), (9, 1, 2, 5), (16, 16, 255, 1),
                                         (16, 16, 17, 0)])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_decay_factors_bit_exact(lasad, oracle, H, W, start, n, mode):
    torch = _torch()
    g = np.random.default_rng(H * 131 + W).uniform(0.0, 1.0, size=(5,)).astype(np.float32)
    g[0], g[1] = 0.0, 1.0
    lam, cum = lasad.lasad_decay_factors(torch.from_numpy(g).cuda(), H, W, start, n, mode)
    torch.cuda.synchronize()
    lam_ref, cum_ref = oracle.decay_factors(g, H, W, start, n, mode)
    assert lam.cpu().numpy().tobytes() == lam_ref.tobytes()
    assert cum.cpu().numpy().tobytes() == cum_ref.tobytes()


# ------------------------------------------------------------------ forward: the benchmark configurations

def test_forward_tiny_fp32(lasad, oracle):
    w = wl.TINY
    q, k, v, g = wl.prefill_inputs(w)
    lam, _ = oracle.decay_factors(g, w.grid_h, w.grid_w, 0, w.N)
    ref, s_ref = oracle.forward_fullmask(q, k, v, lam, want_state=True)
    got, s_got = _gpu_forward(lasad, w, q, k, v, g, want_state=True)
    assert rel_err(got, ref) <= TOL["f32"]
    assert rel_err(s_got, s_ref) <= TOL["f32"]


@pytest.mark.parametrize("segmented", [True, False], ids=["segments", "single_pass"])
@pytest.mark.parametrize("out", ["bf16", "f32"])
def test_forward_base_prefill_full(lasad, oracle, out, segmented):
    w = wl.BASE_PREFILL
    q, k, v, g = wl.prefill_inputs(w)
    lam, _ = oracle.decay_factors(g, w.grid_h, w.grid_w, 0, w.N)
    ref, s_ref = oracle.forward_fullmask(q, k, v, lam, want_state=True)
    got, s_got = _gpu_forward(lasad, w, q, k, v, g, want_state=True, out_dtype=_odt(out),
                              use_workspace=segmented)
    assert rel_err(got, ref) <= TOL["bf16"]
    assert rel_err(s_got, s_ref) <= TOL["bf16"]


@pytest.mark.parametrize("out", ["bf16", "f32"])
@pytest.mark.parametrize("w,count", [(wl.LARGE_PREFILL, 32), (wl.HIGHRES, 6)], ids=["large", "highres"])
def test_forward_full_size_sampled_sequences(lasad, oracle, w, count, out):
    """Full-size launch (the shape the benchmark times); the oracle recomputes sampled
    (batch, head) sequences in full and every element of those is compared."""
    q, k, v, g = wl.prefill_inputs(w)
    got, s_got = _gpu_forward(lasad, w, q, k, v, g, want_state=True, out_dtype=_odt(out))
    pairs = sample_pairs(w.B, w.Hh, count, seed=w.seed)
    lam, _ = oracle.decay_factors(g[[h for _, h in pairs]], w.grid_h, w.grid_w, 0, w.N)
    ref, s_ref = oracle.forward_fullmask(gather_pairs(q, pairs), gather_pairs(k, pairs),
                                         gather_pairs(v, pairs), lam, want_state=True)
    assert rel_err(gather_pairs(got, pairs), ref) <= TOL["bf16"]
    s_sel = np.stack([s_got[b, h] for b, h in pairs])[None]
    assert rel_err(s_sel, s_ref) <= TOL["bf16"]
    # property that holds at any size: the last token of each grid row is a free step, so for
    # gamma-independent sanity the output must be finite everywhere
    assert np.isfinite(got).all() and np.isfinite(s_got).all()


# ------------------------------------------------------------------ forward: shapes, layouts, modes, edge cases

CASES = [
    # name, B, Hh, d, H, W, dtype
    ("ragged_5x7_d64", 2, 3, 64, 5, 7, "bf16"),
    ("ragged_9x11_d64", 1, 2, 64, 9, 11, "bf16"),
    ("three_chunks_plus_tail", 2, 2, 64, 13, 17, "bf16"),
    ("single_token", 1, 2, 64, 1, 1, "bf16"),
    ("single_row", 1, 2, 64, 1, 70, "bf16"),
    ("single_col", 1, 2, 64, 70, 1, "bf16"),
    ("d32_bf16", 2, 2, 32, 6, 9, "bf16"),
    ("d128_bf16", 1, 2, 128, 6, 9, "bf16"),
    ("d64_f32", 2, 2, 64, 10, 10, "f32"),
    ("d128_f32", 1, 1, 128, 5, 5, "f32"),
    ("d64_f32_many_seqs", 6, 50, 64, 3, 13, "f32"),
    ("bf16_160_seqs", 10, 16, 64, 9, 16, "bf16"),      # between 128 and 256 sequences: one twelve-wave workgroup each    # > 256 sequences: one workgroup per head in the fp32 kernel
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("layout", ["bnhd", "bhnd"])
def test_forward_shapes(lasad, oracle, case, mode, layout):
    name, B, Hh, d, H, W, dtype = case
    w = wl.Workload(name, B, Hh, d, H, W, dtype, 0.5, 0.999, seed=zlib.crc32(name.encode()) % 10000 + mode)
    q, k, v, g = wl.prefill_inputs(w, layout=layout)
    lam, _ = oracle.decay_factors(g, H, W, 0, w.N, mode)
    ref, s_ref = oracle.forward_fullmask(q, k, v, lam, q_scale=0.5, want_state=True)
    got, s_got = _gpu_forward(lasad, w, q, k, v, g, mode=mode, q_scale=0.5, want_state=True)
    assert rel_err(got, ref) <= TOL[dtype]
    assert rel_err(s_got, s_ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("start,n", [(0, 100), (37, 130), (100, 1), (5, 64), (63, 65), (192, 0)])
def test_forward_carried_state_mid_row(lasad, oracle, dtype, start, n):
    """A call that starts mid-row from a carried state and stops mid-row."""
    w = wl.Workload("carry", 2, 3, 64, 12, 16, dtype, 0.7, 0.999, seed=77 + start)
    q, k, v, g = wl.prefill_inputs(w)
    q, k, v = q[:, start:start + n], k[:, start:start + n], v[:, start:start + n]
    s0 = wl.random_state(w, seed=5)
    lam, _ = oracle.decay_factors(g, w.grid_h, w.grid_w, start, n)
    ref, s_ref = oracle.forward_fullmask(q, k, v, lam, s0=s0.astype(np.float64), want_state=True)
    got, s_got = _gpu_forward(lasad, w, np.ascontiguousarray(q), np.ascontiguousarray(k),
                              np.ascontiguousarray(v), g, start_pos=start, n=n, s0=s0, want_state=True)
    if n > 0:
        assert rel_err(got, ref) <= TOL[dtype]
    assert rel_err(s_got, s_ref) <= TOL[dtype]


@pytest.mark.parametrize("name,B,Hh,H,W", [("seg_ragged", 1, 3, 33, 19), ("seg_two", 2, 2, 32, 16), ("seg_long", 1, 1, 40, 33), ("seg_many", 70, 1, 24, 24)])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_forward_segmented_vs_oracle(lasad, oracle, name, B, Hh, H, W, mode):
    """Few sequences of several chunks: the segment-parallel plan (state pass + full pass), with a
    carried-in state, a ragged last chunk, and one head whose small gamma takes the fp32 recurrence."""
    torch = _torch()
    w = wl.Workload(name, B, Hh, 64, H, W, "bf16", 0.6, 0.999, seed=zlib.crc32(name.encode()) % 1000 + mode)
    q, k, v, g = wl.prefill_inputs(w)
    if Hh >= 3:
        g[1] = 0.3
    assert lasad.lasad_forward_workspace_bytes(B, Hh, w.N, 64, lasad.BF16) > 0
    s0 = wl.random_state(w, seed=11)
    lam, _ = oracle.decay_factors(g, H, W, 0, w.N, mode)
    ref, s_ref = oracle.forward_fullmask(q, k, v, lam, s0=s0.astype(np.float64), want_state=True)
    for segmented in (True, False):
        got, s_got = _gpu_forward(lasad, w, q, k, v, g, mode=mode, s0=s0, want_state=True,
                                  out_dtype=torch.float32, use_workspace=segmented)
        assert rel_err(got, ref) <= TOL["bf16"], segmented
        assert rel_err(s_got, s_ref) <= TOL["bf16"], segmented


def test_forward_split_equals_single_call_on_gpu(lasad, oracle):
    """Two GPU calls joined by the carried state reproduce one GPU call (to rounding)."""
    torch = _torch()
    w = wl.scaled(wl.BASE_PREFILL, B=2, Hh=4)
    q, k, v, g = wl.prefill_inputs(w)
    full, s_full = _gpu_forward(lasad, w, q, k, v, g, want_state=True)
    p = 101
    o1, s1 = _gpu_forward(lasad, w, np.ascontiguousarray(q[:, :p]), np.ascontiguousarray(k[:, :p]),
                          np.ascontiguousarray(v[:, :p]), g, want_state=True)
    o2, s2 = _gpu_forward(lasad, w, np.ascontiguousarray(q[:, p:]), np.ascontiguousarray(k[:, p:]),
                          np.ascontiguousarray(v[:, p:]), g, start_pos=p, s0=s1, want_state=True)
    assert rel_err(np.concatenate([o1, o2], axis=1), full) <= 2 * TOL["bf16"]
    assert rel_err(s2, s_full) <= TOL["bf16"]


@pytest.mark.parametrize("gval", [0.0, 1.0, 0.05, 0.3])
def test_forward_extreme_gamma(lasad, oracle, gval):
    """gamma = 0 (only boundary steps carry anything), gamma = 1 (plain causal linear attention,
    Section 3.2) and small gammas whose powers underflow inside a chunk."""
    w = wl.Workload("extreme", 1, 2, 64, 9, 16, "bf16", 0.5, 0.9, seed=31)
    q, k, v, g = wl.prefill_inputs(w)
    g = np.array([gval, 0.9], dtype=np.float32)
    lam, _ = oracle.decay_factors(g, w.grid_h, w.grid_w, 0, w.N)
    ref, s_ref = oracle.forward_fullmask(q, k, v, lam, want_state=True)
    got, s_got = _gpu_forward(lasad, w, q, k, v, g, want_state=True)
    assert np.isfinite(got).all()
    assert rel_err(got, ref) <= TOL["bf16"]
    assert rel_err(s_got, s_ref) <= TOL["bf16"]


def test_forward_fp32_output_of_bf16_inputs(lasad, oracle):
    torch = _torch()
    w = wl.scaled(wl.BASE_PREFILL, B=1, Hh=2)
    q, k, v, g = wl.prefill_inputs(w)
    lam, _ = oracle.decay_factors(g, w.grid_h, w.grid_w, 0, w.N)
    ref = oracle.forward_fullmask(q, k, v, lam)
    got = _gpu_forward(lasad, w, q, k, v, g, out_dtype=torch.float32)
    assert rel_err(got, ref) <= TOL["bf16"]


def test_forward_causality_bitwise(lasad):
    """o_i is unchanged, bit for bit, when tokens after i change."""
    w = wl.scaled(wl.BASE_PREFILL, B=1, Hh=2)
    q, k, v, g = wl.prefill_inputs(w)
    base = _gpu_forward(lasad, w, q, k, v, g)
    j = 150
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[:, j:], k2[:, j:], v2[:, j:] = 0.5, -0.25, 2.0
    pert = _gpu_forward(lasad, w, q2, k2, v2, g)
    assert base[:, :j].tobytes() == pert[:, :j].tobytes()
    assert not np.array_equal(base[:, j:], pert[:, j:])


def test_forward_deterministic(lasad):
    w = wl.scaled(wl.LARGE_PREFILL, B=2)
    q, k, v, g = wl.prefill_inputs(w)
    a, sa = _gpu_forward(lasad, w, q, k, v, g, want_state=True)
    b, sb = _gpu_forward(lasad, w, q, k, v, g, want_state=True)
    assert a.tobytes() == b.tobytes() and sa.tobytes() == sb.tobytes()


# ------------------------------------------------------------------ decode

def _decode_walk(lasad, w, q, k, v, g, batch_rows=None, q_scale=1.0, out_dtype=None, mode=0):
    """Run w.steps decode steps on the GPU for the whole batch; return o[steps, rows, Hh, d], final state."""
    torch = _torch()
    steps = q.shape[0]
    tq, tk, tv = (lasad.to_device(x, w.dtype) for x in (q, k, v))
    tg = torch.from_numpy(g).cuda()
    state = torch.zeros((w.B, w.Hh, w.d, w.d), dtype=torch.float32, device="cuda")
    outs = []
    for t in range(steps):
        o = decode_both(lambda st, odt: lasad.lasad_decode_step(tq[t], tk[t], tv[t], tg, st, w.grid_h, w.grid_w, t,
                                                                boundary_mode=mode, q_scale=q_scale, out_dtype=odt),
                        state, w.dtype == "bf16" and out_dtype != torch.float32)
        outs.append(o if batch_rows is None else o[batch_rows])
    torch.cuda.synchronize()
    o = torch.stack(outs).cpu().numpy()
    s = state.cpu().numpy()
    return o, (s if batch_rows is None else s[batch_rows])


def _oracle_walk(oracle, w, q, k, v, g, q_scale=1.0, mode=0):
    steps, B = q.shape[0], q.shape[1]
    state = np.zeros((B, w.Hh, w.d, w.d))
    outs = []
    for t in range(steps):
        lam_t, _ = oracle.decay_factors(g, w.grid_h, w.grid_w, t, 1, mode)
        outs.append(oracle.decode_step(q[t], k[t], v[t], lam_t[:, 0], state, q_scale=q_scale))
    return np.stack(outs), state


@pytest.mark.parametrize("d,dtype,H,W,B,Hh", [(64, "bf16", 16, 16, 3, 5), (32, "bf16", 4, 6, 2, 3),
                                             (128, "bf16", 3, 5, 1, 2), (64, "f32", 8, 8, 2, 3),
                                             (32, "f32", 8, 8, 1, 1)])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_decode_walk_small(lasad, oracle, d, dtype, H, W, B, Hh, mode):
    w = wl.Workload("dec", B, Hh, d, H, W, dtype, 0.85, 0.999, seed=900 + d + mode, kind="decode", steps=H * W)
    q, k, v, g = wl.decode_inputs(w)
    got, s_got = _decode_walk(lasad, w, q, k, v, g, q_scale=0.7, mode=mode)
    ref, s_ref = _oracle_walk(oracle, w, q, k, v, g, q_scale=0.7, mode=mode)
    for t in range(w.steps):
        assert rel_err(got[t], ref[t]) <= TOL[dtype], f"step {t}"
    assert rel_err(s_got, s_ref) <= TOL[dtype]


@pytest.mark.parametrize("out", ["bf16", "f32"])
def test_decode_full_batch_sampled_rows(lasad, oracle, out):
    """The full AR-decode configuration (256 x 20 states, 256 raster steps) on the GPU; the
    oracle walks sampled batch rows and every output of those rows is compared."""
    w = wl.AR_DECODE
    q, k, v, g = wl.decode_inputs(w)
    rows = [0, 101, 255]
    got, s_got = _decode_walk(lasad, w, q, k, v, g, batch_rows=rows, out_dtype=_odt(out))
    ref, s_ref = _oracle_walk(oracle, w, q[:, rows], k[:, rows], v[:, rows], g)
    worst = max(rel_err(got[t], ref[t]) for t in range(w.steps))
    assert worst <= TOL["bf16"], worst
    assert rel_err(s_got, s_ref) <= TOL["bf16"]


def test_decode_equals_forward_on_gpu(lasad, oracle):
    """N decode steps and one chunked forward over the same tokens agree (both within tolerance
    of the oracle, and with each other)."""
    torch = _torch()
    w = wl.Workload("dec_vs_fwd", 2, 4, 64, 16, 16, "bf16", 0.85, 0.999, seed=55, kind="decode", steps=256)
    q, k, v, g = wl.decode_inputs(w)
    o_dec, s_dec = _decode_walk(lasad, w, q, k, v, g, out_dtype=torch.float32)
    qf, kf, vf = (np.ascontiguousarray(x.transpose(1, 0, 2, 3)) for x in (q, k, v))
    o_fwd, s_fwd = _gpu_forward(lasad, w, qf, kf, vf, g, want_state=True, out_dtype=torch.float32)
    assert rel_err(o_dec.transpose(1, 0, 2, 3), o_fwd) <= TOL["bf16"]
    assert rel_err(s_dec, s_fwd) <= TOL["bf16"]


VARIANT_SCRIPT = r"""
import sys, numpy as np, torch
sys.path.insert(0, sys.argv[1]); sys.path.insert(0, sys.argv[1] + '/tests')
from paper_2507_01652_amd import binding as lasad, workloads as wl
from oracle import lasad_oracle as oracle
from helpers import rel_err
worst = 0.0
for B, Hh, H, W in ((2, 3, 13, 17), (1, 2, 40, 33)):
    w = wl.Workload('variant', B, Hh, 64, H, W, 'bf16', 0.6, 0.999, seed=11 + B)
    q, k, v, g = wl.prefill_inputs(w)
    lam, _ = oracle.decay_factors(g, H, W, 0, w.N)
    s0 = wl.random_state(w, 3)
    ref, s_ref = oracle.forward_fullmask(q, k, v, lam, s0=s0.astype(np.float64), want_state=True)
    s1 = torch.empty((B, Hh, 64, 64), dtype=torch.float32, device='cuda')
    o = lasad.lasad_forward_chunked(*(lasad.to_device(x, 'bf16') for x in (q, k, v)), torch.from_numpy(g).cuda(), H, W,
                                    state_in=torch.from_numpy(s0).cuda(), state_out=s1, out_dtype=torch.float32)
    torch.cuda.synchronize()
    worst = max(worst, rel_err(o.cpu().numpy(), ref), rel_err(s1.cpu().numpy(), s_ref))
print('WORST', worst)
assert worst <= 2e-2
"""


@pytest.mark.parametrize("env", [{"LASAD_WS": "0"}, {"LASAD_WS": "8"}, {"LASAD_WS": "12", "LASAD_SPLIT": "1"},
                                 {"LASAD_WS": "12", "LASAD_SPLIT": "2"}],
                         ids=["four_wave", "eight_wave", "twelve_wave_whole", "twelve_wave_split"])
def test_forward_kernel_variants(env):
    """Every full-pass kernel variant (the launcher picks one by the number of workgroups; the choice is read
    from the environment once per process, hence the child process) against the oracle, with and without the
    segment plan (the second shape is long enough to be cut into segments)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", VARIANT_SCRIPT, root], env={**os.environ, **env},
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
