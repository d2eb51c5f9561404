"""GPU parity of the vector-decay path (Section 3.4 / Algorithm 1 as written: a decay vector per
token, key tied to the decay) against the fp64 oracle.  Same tolerances as the scalar path, on the
fp32 result; a bf16 result must be the fp32 result rounded, bit for bit (helpers.both_outputs)."""
import numpy as np
import pytest

from paper_2507_01652_amd import workloads as wl
from helpers import TOL, both_outputs, decode_both, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lasad():
    import torch
    assert torch.cuda.is_available()
    from paper_2507_01652_amd import binding
    binding.load()
    return binding


def _inputs(B, n, Hh, d, dtype, seed, tied):
    rng = np.random.default_rng(seed)
    sc = np.float32(1.0 / np.sqrt(d))
    q = wl.store_round(rng.standard_normal((B, n, Hh, d), dtype=np.float32) * sc, dtype)
    v = wl.store_round(rng.standard_normal((B, n, Hh, d), dtype=np.float32) * sc, dtype)
    k = None if tied else wl.store_round(rng.standard_normal((B, n, Hh, d), dtype=np.float32) * sc, dtype)
    lam = wl.gate_inputs((B, n, Hh, d), dtype, seed + 1)
    return q, lam, k, v


@pytest.mark.parametrize("d,dtype,H,W,B,Hh", [(64, "bf16", 16, 16, 2, 3), (64, "f32", 8, 8, 1, 2),
                                             (32, "bf16", 5, 7, 2, 2), (128, "bf16", 3, 5, 1, 2),
                                             (64, "bf16", 1, 37, 1, 1),
                                             # more than 256 sequences: one workgroup per head, ragged tail
                                             (64, "bf16", 5, 7, 9, 32), (64, "f32", 3, 11, 5, 53)])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("tied", [True, False], ids=["k=1-lam", "own_k"])
def test_forward_gated(lasad, oracle, d, dtype, H, W, B, Hh, mode, tied):
    import torch
    n = H * W
    q, lam, k, v = _inputs(B, n, Hh, d, dtype, 300 + d + mode, tied)
    s0 = (np.random.default_rng(5).standard_normal((B, Hh, d, d)) * 0.5).astype(np.float32)
    ref, s_ref = oracle.gated_recurrent(q, lam, v, W, k=k, mode=mode, q_scale=0.8,
                                        s0=s0.astype(np.float64), want_state=True)
    dev = lambda x: None if x is None else lasad.to_device(x, dtype)
    s1 = torch.empty((B, Hh, d, d), dtype=torch.float32, device="cuda")
    o = both_outputs(lasad.lasad_forward_gated, dtype == "bf16", q=dev(q), lam=dev(lam), v=dev(v), grid_h=H, grid_w=W,
                     k=dev(k), boundary_mode=mode, q_scale=0.8, state_in=torch.from_numpy(s0).cuda(), state_out=s1)
    torch.cuda.synchronize()
    assert rel_err(o.cpu().numpy(), ref) <= TOL[dtype]
    assert rel_err(s1.cpu().numpy(), s_ref) <= TOL[dtype]


def test_forward_gated_split_and_layout(lasad, oracle):
    """[B, Hh, N, d] memory order and a call that starts mid-row from a carried state."""
    import torch
    H, W, B, Hh, d = 6, 10, 2, 2, 64
    n = H * W
    q, lam, k, v = _inputs(B, n, Hh, d, "bf16", 77, True)
    ref, s_ref = oracle.gated_recurrent(q, lam, v, W, want_state=True)
    perm = lambda x: lasad.to_device(np.ascontiguousarray(x.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3), "bf16")
    p = 23
    s1 = torch.empty((B, Hh, d, d), dtype=torch.float32, device="cuda")
    s2 = torch.empty_like(s1)
    o1 = lasad.lasad_forward_gated(perm(q[:, :p]), perm(lam[:, :p]), perm(v[:, :p]), H, W, state_out=s1,
                                   out_dtype=torch.float32)
    o2 = lasad.lasad_forward_gated(perm(q[:, p:]), perm(lam[:, p:]), perm(v[:, p:]), H, W, start_pos=p,
                                   state_in=s1, state_out=s2, out_dtype=torch.float32)
    torch.cuda.synchronize()
    got = np.concatenate([o1.cpu().numpy(), o2.cpu().numpy()], axis=1)
    assert rel_err(got, ref) <= TOL["bf16"]
    assert rel_err(s2.cpu().numpy(), s_ref) <= TOL["bf16"]


@pytest.mark.parametrize("d,dtype,H,W,B,Hh", [(64, "bf16", 16, 16, 3, 5), (32, "f32", 4, 6, 2, 3), (128, "bf16", 3, 5, 1, 2)])
@pytest.mark.parametrize("tied", [True, False], ids=["k=1-lam", "own_k"])
def test_decode_gated_walk(lasad, oracle, d, dtype, H, W, B, Hh, tied):
    """Raster walk of decode steps against the oracle's sequential recurrence, every step's output."""
    import torch
    n = H * W
    q, lam, k, v = _inputs(B, n, Hh, d, dtype, 500 + d, tied)
    ref, s_ref = oracle.gated_recurrent(q, lam, v, W, k=k, q_scale=1.1, want_state=True)
    dev = lambda x: None if x is None else lasad.to_device(np.ascontiguousarray(x.transpose(1, 0, 2, 3)), dtype)
    tq, tl, tk, tv = dev(q), dev(lam), dev(k), dev(v)
    state = torch.zeros((B, Hh, d, d), dtype=torch.float32, device="cuda")
    outs = []
    for t in range(n):
        outs.append(decode_both(lambda st, odt: lasad.lasad_decode_step_gated(
            tq[t], tl[t], tv[t], st, H, W, t, k=None if tk is None else tk[t], q_scale=1.1, out_dtype=odt),
            state, dtype == "bf16"))
    torch.cuda.synchronize()
    got = torch.stack(outs).cpu().numpy().transpose(1, 0, 2, 3)
    for t in range(n):
        assert rel_err(got[:, t], ref[:, t]) <= TOL[dtype], f"step {t}"
    assert rel_err(state.cpu().numpy(), s_ref) <= TOL[dtype]


def test_decode_gated_full_batch_sampled_rows(lasad, oracle):
    """AR-decode shape (256 x 20 states) with the vector decay; oracle on sampled batch rows."""
    import torch
    w = wl.AR_DECODE
    steps = 64
    q, lam, k, v = _inputs(w.B, steps, w.Hh, w.d, "bf16", 900, True)
    rows = [0, 130, 255]
    ref, s_ref = oracle.gated_recurrent(q[rows], lam[rows], v[rows], w.grid_w, want_state=True)
    dev = lambda x: lasad.to_device(np.ascontiguousarray(x.transpose(1, 0, 2, 3)), "bf16")
    tq, tl, tv = dev(q), dev(lam), dev(v)
    state = torch.zeros((w.B, w.Hh, w.d, w.d), dtype=torch.float32, device="cuda")
    outs = []
    for t in range(steps):
        outs.append(lasad.lasad_decode_step_gated(tq[t], tl[t], tv[t], state, w.grid_h, w.grid_w, t,
                                                  out_dtype=torch.float32)[rows])
    torch.cuda.synchronize()
    got = torch.stack(outs).cpu().numpy().transpose(1, 0, 2, 3)
    assert rel_err(got, ref) <= TOL["bf16"]
    assert rel_err(state[rows].cpu().numpy(), s_ref) <= TOL["bf16"]


def _sampled_check(lasad, oracle, w, lam_fn, tied, n_pairs, out_dtype_name):
    """Full-size forward on the GPU, oracle on sampled (batch, head) sequences."""
    import torch
    from helpers import sample_pairs, gather_pairs
    q, k, v, _ = wl.prefill_inputs(w)
    lam = lam_fn((w.B, w.N, w.Hh, w.d))
    if tied:
        k = None
    dev = lambda x: None if x is None else lasad.to_device(x, w.dtype)
    out_dtype = {"bf16": torch.bfloat16, "f32": torch.float32}[out_dtype_name]
    s1 = torch.empty((w.B, w.Hh, w.d, w.d), dtype=torch.float32, device="cuda")
    o = both_outputs(lasad.lasad_forward_gated, out_dtype == torch.bfloat16, q=dev(q), lam=dev(lam), v=dev(v),
                     grid_h=w.grid_h, grid_w=w.grid_w, k=dev(k), state_out=s1)
    torch.cuda.synchronize()
    pairs = sample_pairs(w.B, w.Hh, n_pairs, seed=w.seed)
    ref, s_ref = oracle.gated_recurrent(gather_pairs(q, pairs), gather_pairs(lam, pairs), gather_pairs(v, pairs),
                                        w.grid_w, k=None if k is None else gather_pairs(k, pairs), want_state=True)
    got = gather_pairs(o.float().cpu().numpy(), pairs)
    s_got = np.stack([s1.cpu().numpy()[b, h] for b, h in pairs])[None]
    assert rel_err(got, ref) <= TOL["bf16"]
    assert rel_err(s_got, s_ref) <= TOL["bf16"]


@pytest.mark.parametrize("name,n_pairs", [("base_prefill_16x16", 24), ("large_prefill_24x24", 24), ("highres_64x64", 4)])
@pytest.mark.parametrize("tied", [True, False], ids=["k=1-lam", "own_k"])
def test_forward_gated_bench_shapes(lasad, oracle, name, n_pairs, tied):
    """The shapes bench.py times, in the launch configuration it uses: the fp32 output meets the bare
    tolerance on sampled sequences and the bf16 output is its rounding."""
    w = wl.CONFIGS[name]
    _sampled_check(lasad, oracle, w, lambda shape: wl.gate_inputs(shape, w.dtype, w.seed + 7), tied, n_pairs, "bf16")


GATE_EXTREMES = {
    # every chunk's total decay is far below what the chunked factorisation takes: token-serial redo
    "strong_decay": lambda rng, shape: rng.uniform(0.0, 0.3, size=shape),
    # exact zeros and ones mixed into ordinary gates
    "zeros_and_ones": lambda rng, shape: np.where(rng.random(shape) < 0.02, 0.0,
                                                  np.where(rng.random(shape) < 0.3, 1.0, rng.uniform(0.5, 1.0, size=shape))),
    # never decays: plain linear attention
    "all_ones": lambda rng, shape: np.ones(shape),
    # decay strong enough for some sequences only (head 0 weak, others strong)
    "mixed_heads": lambda rng, shape: np.concatenate([rng.uniform(0.9, 1.0, size=shape[:2] + (1,) + shape[3:]),
                                                      rng.uniform(0.2, 0.6, size=shape[:2] + (shape[2] - 1,) + shape[3:])], axis=2),
    # a chunk total of about 2^-50, just inside what the chunked factorisation takes
    "near_limit": lambda rng, shape: 0.57 * np.ones(shape),
    # one channel just outside it (about 2^-65 per chunk), all others mild
    "one_channel_below_limit": lambda rng, shape: np.where(np.arange(shape[3]) == 5, 0.48, 0.95) * np.ones(shape),
}


@pytest.mark.parametrize("kind", sorted(GATE_EXTREMES))
@pytest.mark.parametrize("tied", [True, False], ids=["k=1-lam", "own_k"])
def test_forward_gated_extreme_gates(lasad, oracle, kind, tied):
    import torch
    B, Hh, d, H, W = 2, 3, 64, 9, 17          # 153 tokens: two full chunks and a tail
    n = H * W
    q, _, k, v = _inputs(B, n, Hh, d, "bf16", 900, tied)
    rng = np.random.default_rng(zlib_seed(kind))
    lam = wl.store_round(GATE_EXTREMES[kind](rng, (B, n, Hh, d)).astype(np.float32), "bf16")
    ref, s_ref = oracle.gated_recurrent(q, lam, v, W, k=k, want_state=True)
    dev = lambda x: None if x is None else lasad.to_device(x, "bf16")
    s1 = torch.empty((B, Hh, d, d), dtype=torch.float32, device="cuda")
    o = lasad.lasad_forward_gated(dev(q), dev(lam), dev(v), H, W, k=dev(k), state_out=s1, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.isfinite(o.cpu().numpy()).all()
    assert rel_err(o.cpu().numpy(), ref) <= TOL["bf16"]
    assert rel_err(s1.cpu().numpy(), s_ref) <= TOL["bf16"]


def zlib_seed(name):
    import zlib
    return zlib.crc32(name.encode()) % 100000


def test_forward_gated_deterministic(lasad):
    import torch
    w = wl.scaled(wl.BASE_PREFILL, B=2)
    q, _, v, _ = wl.prefill_inputs(w)
    lam = wl.gate_inputs(q.shape, w.dtype, 3)
    tq, tl, tv = (lasad.to_device(x, w.dtype) for x in (q, lam, v))
    o1 = lasad.lasad_forward_gated(tq, tl, tv, w.grid_h, w.grid_w)
    o2 = lasad.lasad_forward_gated(tq, tl, tv, w.grid_h, w.grid_w)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)


GATED_VARIANT_SCRIPT = r"""
import sys, numpy as np, torch
sys.path.insert(0, sys.argv[1]); sys.path.insert(0, sys.argv[1] + '/tests')
from paper_2507_01652_amd import binding as lasad, workloads as wl
from oracle import lasad_oracle as oracle
from helpers import both_outputs, rel_err
worst = 0.0
for B, Hh, H, W in ((2, 3, 13, 17), (1, 2, 1, 50)):
    rng = np.random.default_rng(5 + B)
    shape = (B, H * W, Hh, 64)
    q = wl.store_round(rng.standard_normal(shape, dtype=np.float32), 'bf16')
    z = wl.store_round(rng.standard_normal(shape, dtype=np.float32) + np.float32(2.0), 'bf16')
    v = wl.store_round(rng.standard_normal(shape, dtype=np.float32) / np.float32(8.0), 'bf16')
    lam = wl.store_round(oracle.sigmoid(z).astype(np.float32), 'bf16')
    wgt = rng.uniform(0.5, 1.5, size=(Hh, 64)).astype(np.float32)
    dev = lambda x: lasad.to_device(x, 'bf16')
    # the vector-decay forward (key tied to the gate) and the fused layer with its norm
    ref, s_ref = oracle.gated_recurrent(q, lam, v, W, want_state=True)
    s1 = torch.empty((B, Hh, 64, 64), dtype=torch.float32, device='cuda')
    o = lasad.lasad_forward_gated(dev(q), dev(lam), dev(v), H, W, state_out=s1, out_dtype=torch.float32)
    torch.cuda.synchronize()
    worst = max(worst, rel_err(o.cpu().numpy(), ref), rel_err(s1.cpu().numpy(), s_ref))
    both_outputs(lasad.lasad_forward_gated, True, q=dev(q), lam=dev(lam), v=dev(v), grid_h=H, grid_w=W, state_out=s1)
    ref = oracle.gated_layer(q, z, v, W, norm_weight=wgt, eps=1e-5)
    o = both_outputs(lasad.lasad_forward_layer, True, q_pre=dev(q), z=dev(z), v=dev(v), grid_h=H, grid_w=W,
                     norm_weight=torch.from_numpy(wgt).cuda(), norm_eps=1e-5)
    torch.cuda.synchronize()
    worst = max(worst, rel_err(o.cpu().numpy(), ref))
print('WORST', worst)
assert worst <= 2e-2
"""


@pytest.mark.parametrize("env", [{"LASAD_GATED_WS": "0"}, {"LASAD_GATED_WS": "1"}], ids=["four_wave", "twelve_wave"])
def test_gated_kernel_variants(env):
    """Both vector-decay kernels, forced (the launcher's choice is read from the environment once per process,
    hence the child process), on the forward and on the fused layer, several chunks with a ragged tail and a
    single short chunk."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", GATED_VARIANT_SCRIPT, root], env={**os.environ, **env},
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
