"""GPU parity of the backward pass (gradients of the Section 3.4 recurrence with the per-head scalar decay,
zero initial state) against the fp64 oracle's reverse-mode routine.  Same metric and tolerances as the
forward: max |gpu - oracle| / rms(oracle) per gradient tensor (1e-5 for fp32 storage, 2e-2 for bf16 storage)
on the fp32 gradients; gradients stored as bf16 must be the fp32 gradients rounded, bit for bit, and dgamma the
same in both runs (helpers.both_outputs); the decay gradient is compared relative to the largest |dgamma| over
the heads."""
import zlib

import numpy as np
import pytest

from paper_2507_01652_amd import workloads as wl
from helpers import TOL, both_outputs, rel_err, sample_pairs, gather_pairs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lasad():
    import torch
    assert torch.cuda.is_available()
    from paper_2507_01652_amd import binding
    binding.load()
    return binding


def _d_o(w, layout="bnhd"):
    rng = np.random.default_rng(w.seed + 101)
    x = wl.store_round(rng.standard_normal((w.B, w.N, w.Hh, w.d), dtype=np.float32) / np.float32(np.sqrt(w.d)), w.dtype)
    if layout == "bhnd":
        x = np.ascontiguousarray(x.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    return x


def _gpu_backward(lasad, w, q, k, v, g, gam, start=0, mode=0, q_scale=1.0, grad_dtype=None):
    import torch
    tq, tk, tv, tg = (lasad.to_device(x, w.dtype) for x in (q, k, v, g))
    # fp32 gradients are returned; unless they are asked for explicitly, bf16 inputs run the bf16 gradients too
    dq, dk, dv, dgam = both_outputs(lasad.lasad_backward_chunked, w.dtype == "bf16" and grad_dtype != torch.float32,
                                    dtype_kw="grad_dtype", q=tq, k=tk, v=tv, d_o=tg, gamma=torch.from_numpy(gam).cuda(),
                                    grid_h=w.grid_h, grid_w=w.grid_w, start_pos=start, boundary_mode=mode, q_scale=q_scale)
    torch.cuda.synchronize()
    return dq, dk, dv, dgam.cpu().numpy()


def _check(lasad, oracle, w, start=0, mode=0, q_scale=1.0, grad_bf16=None, layout="bnhd", n=None):
    import torch
    q, k, v, gam = wl.prefill_inputs(w, layout=layout)
    g = _d_o(w, layout)
    n = w.N - start if n is None else n
    q, k, v, g = (x[:, start:start + n] for x in (q, k, v, g))
    if grad_bf16 is None:
        grad_bf16 = w.dtype == "bf16"
    dq, dk, dv, dgam = _gpu_backward(lasad, w, q, k, v, g, gam, start, mode, q_scale,
                                     torch.bfloat16 if grad_bf16 else torch.float32)
    lam, _ = oracle.decay_factors(gam, w.grid_h, w.grid_w, start, n, mode)
    rq, rk, rv, rlam = oracle.backward(q, k, v, lam, g, q_scale=q_scale)
    rgam = oracle.dgamma(rlam, w.grid_w, start, mode)
    tol = TOL[w.dtype]
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        err = rel_err(got.cpu().numpy(), ref)
        assert err <= tol, (name, err)
    _check_dgamma(dgam, rgam, w, q, k, rq, rk, gam, start, mode, oracle)


def _check_dgamma(dgam, rgam, w, q, k, rq, rk, gam, start, mode, oracle):
    """Relative to the largest |dgamma| over the heads, plus an fp32 rounding floor: the kernel sums
    E_t (q_t . dq_t - k_t . dk_t) / gamma in fp32, so its rounding scales with the sum of the absolute terms."""
    n = q.shape[1]
    _, cum = oracle.decay_factors(gam, w.grid_h, w.grid_w, start, n, mode)     # E(start) .. E(start + n)
    E = (cum[1:] - cum[0]).astype(np.float64)                                  # [n]
    terms = (np.abs(q * rq).sum(axis=3) + np.abs(k * rk).sum(axis=3)) * E[None, :, None]  # [B, n, Hh]
    floor = 1e-6 * terms.sum(axis=(0, 1)).max() / float(gam.min())
    rel = 2e-2 if w.dtype == "bf16" else 1e-4
    assert np.abs(dgam - rgam).max() <= rel * np.abs(rgam).max() + floor, (dgam, rgam)


CASES = [
    # name, B, Hh, d, H, W, dtype
    ("tiny_f32_d32", 1, 2, 32, 4, 5, "f32"),
    ("f32_d64", 2, 2, 64, 7, 9, "f32"),
    ("f32_d128", 1, 1, 128, 3, 5, "f32"),
    ("bf16_d64_one_chunk", 2, 3, 64, 5, 7, "bf16"),
    ("bf16_d64_chunks_and_tail", 2, 2, 64, 13, 17, "bf16"),
    ("bf16_d64_single_row", 1, 2, 64, 1, 70, "bf16"),
    ("bf16_d64_single_col", 1, 2, 64, 70, 1, "bf16"),
    ("bf16_d32", 2, 2, 32, 6, 9, "bf16"),
    ("bf16_single_token", 1, 2, 64, 1, 1, "bf16"),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_backward_shapes(lasad, oracle, case, mode):
    name, B, Hh, d, H, W, dtype = case
    w = wl.Workload(name, B, Hh, d, H, W, dtype, 0.6, 0.999, seed=zlib.crc32(name.encode()) % 10000 + mode)
    _check(lasad, oracle, w, mode=mode, q_scale=0.5)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("start,n", [(5, 100), (17, 64), (16, 3)])
def test_backward_partial_range(lasad, oracle, mode, start, n):
    """A call over positions start+1 .. start+n (mid-row start and end), zero incoming state."""
    w = wl.Workload("bwd_range", 2, 2, 64, 9, 17, "bf16", 0.7, 0.999, seed=4242 + start)
    _check(lasad, oracle, w, start=start, mode=mode, n=n, grad_bf16=False)


@pytest.mark.parametrize("layout", ["bnhd", "bhnd"])
@pytest.mark.parametrize("grad_bf16", [True, False])
def test_backward_layouts_and_grad_types(lasad, oracle, layout, grad_bf16):
    w = wl.Workload("bwd_layout", 2, 3, 64, 10, 12, "bf16", 0.8, 0.999, seed=77)
    _check(lasad, oracle, w, layout=layout, grad_bf16=grad_bf16)


def test_backward_small_gamma_heads(lasad, oracle):
    """Heads whose decay is too small for the matrix-core kernel's separable factors take its fp32 route."""
    import torch
    w = wl.Workload("bwd_small_gamma", 1, 3, 64, 6, 16, "bf16", 0.8, 0.99, seed=5)
    q, k, v, gam = wl.prefill_inputs(w)
    gam = np.array([0.3, 0.95, 0.05], dtype=np.float32)
    g = _d_o(w)
    dq, dk, dv, dgam = _gpu_backward(lasad, w, q, k, v, g, gam, grad_dtype=torch.float32)
    lam, _ = oracle.decay_factors(gam, w.grid_h, w.grid_w, 0, w.N, 0)
    rq, rk, rv, rlam = oracle.backward(q, k, v, lam, g)
    rgam = oracle.dgamma(rlam, w.grid_w, 0, 0)
    for got, ref in ((dq, rq), (dk, rk), (dv, rv)):
        assert rel_err(got.cpu().numpy(), ref) <= TOL["bf16"]
    _check_dgamma(dgam, rgam, w, q, k, rq, rk, gam, 0, 0, oracle)


@pytest.mark.parametrize("name", ["base_prefill_16x16", "large_prefill_24x24", "highres_64x64"])
def test_backward_bench_shapes_sampled(lasad, oracle, name):
    """The benchmark shapes in the benchmark's launch configuration; the oracle on sampled sequences (fp32
    gradients against the bare tolerance).  dgamma sums over the whole batch, so it is checked on the
    small shapes only."""
    import torch
    w = wl.CONFIGS[name]
    q, k, v, gam = wl.prefill_inputs(w)
    g = _d_o(w)
    dq, dk, dv, dgam = _gpu_backward(lasad, w, q, k, v, g, gam, grad_dtype=torch.float32)
    pairs = sample_pairs(w.B, w.Hh, 4 if w.N > 1000 else 16, seed=w.seed)
    lam, _ = oracle.decay_factors(gam[[h for _, h in pairs]], w.grid_h, w.grid_w, 0, w.N, 0)
    rq, rk, rv, _ = oracle.backward(gather_pairs(q, pairs), gather_pairs(k, pairs), gather_pairs(v, pairs), lam,
                                    gather_pairs(g, pairs))
    for nm, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        err = rel_err(gather_pairs(got.cpu().numpy(), pairs), ref)
        assert err <= TOL["bf16"], (nm, err)
    assert np.isfinite(dgam).all()


def test_backward_dgamma_full_batch(lasad, oracle):
    """dgamma over a whole (small) batch of the base shape."""
    w = wl.scaled(wl.BASE_PREFILL, B=3)
    _check(lasad, oracle, w, grad_bf16=True)


@pytest.mark.parametrize("B,Hh,H,W", [(4, 12, 16, 16), (8, 12, 16, 16), (11, 8, 9, 15), (1, 2, 40, 16)],
                         ids=["48seq_twelve_wave", "96seq_eight_wave", "88seq_tail", "2seq_segmented"])
def test_backward_launch_shapes(lasad, oracle, B, Hh, H, W):
    """Every launch shape of the three passes, all gradients against the oracle on the full batch: one merged
    launch of the twelve-wave kernel (whole and split sequences: the smaller cases above), of the eight-wave
    kernel (more than 85 sequences), and three separate segmented passes (few long sequences)."""
    w = wl.Workload("bwd_launch", B, Hh, 64, H, W, "bf16", 0.85, 0.999, seed=31 * B + Hh)
    _check(lasad, oracle, w, grad_bf16=True)
    _check(lasad, oracle, w, grad_bf16=False, mode=1, q_scale=0.25)


def test_backward_small_gamma_bf16_grads(lasad, oracle):
    """As test_backward_small_gamma_heads with bf16 gradients (the decay-gradient sums of the fp32 route then
    are taken from its fp32 values) and enough sequences for the eight-wave launch."""
    w = wl.Workload("bwd_small_gamma16", 30, 3, 64, 5, 16, "bf16", 0.8, 0.99, seed=6)
    q, k, v, gam = wl.prefill_inputs(w)
    gam = np.array([0.3, 0.95, 0.05], dtype=np.float32)
    g = _d_o(w)
    dq, dk, dv, dgam = _gpu_backward(lasad, w, q, k, v, g, gam)
    lam, _ = oracle.decay_factors(gam, w.grid_h, w.grid_w, 0, w.N, 0)
    rq, rk, rv, rlam = oracle.backward(q, k, v, lam, g)
    rgam = oracle.dgamma(rlam, w.grid_w, 0, 0)
    for nm, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        assert rel_err(got.cpu().numpy(), ref) <= TOL["bf16"], nm
    _check_dgamma(dgam, rgam, w, q, k, rq, rk, gam, 0, 0, oracle)


def test_backward_deterministic(lasad):
    import torch
    w = wl.scaled(wl.BASE_PREFILL, B=2)
    q, k, v, gam = wl.prefill_inputs(w)
    g = _d_o(w)
    r1 = _gpu_backward(lasad, w, q, k, v, g, gam)
    r2 = _gpu_backward(lasad, w, q, k, v, g, gam)
    for a, b in zip(r1[:3], r2[:3]):
        assert torch.equal(a, b)
    assert np.array_equal(r1[3], r2[3])


def test_backward_rejects_bad_arguments(lasad):
    import torch
    w = wl.scaled(wl.BASE_PREFILL, B=1, Hh=2)
    q, k, v, gam = wl.prefill_inputs(w)
    tq, tk, tv = (lasad.to_device(x, w.dtype) for x in (q, k, v))
    tg = torch.from_numpy(gam).cuda()
    with pytest.raises(lasad.LasadError) as e:
        lasad.lasad_backward_chunked(tq, tk, tv, tq.clone(), tg, w.grid_h, w.grid_w,
                                     workspace=torch.empty((1024,), dtype=torch.uint8, device="cuda"))
    assert e.value.status == 3       # workspace too small
    with pytest.raises(lasad.LasadError):
        lasad.lasad_backward_chunked(tq, tk, tv, tq.clone(), tg, w.grid_h, w.grid_w, grads=(tq, tk, tv))   # aliasing


def test_backward_empty_call(lasad):
    """No tokens: dgamma is zero, nothing else is touched."""
    import torch
    q = torch.zeros((2, 0, 3, 64), dtype=torch.bfloat16, device="cuda")
    gam = torch.full((3,), 0.9, dtype=torch.float32, device="cuda")
    dgam = torch.full((3,), 7.0, dtype=torch.float32, device="cuda")
    lasad.lasad_backward_chunked(q, q.clone(), q.clone(), q.clone(), gam, 4, 4, dgamma=dgam)
    torch.cuda.synchronize()
    assert not dgam.cpu().numpy().any()
