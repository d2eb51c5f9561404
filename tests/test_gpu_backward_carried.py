"""GPU parity of lasad_backward_chunked_carried (gradients of the Section 3.4 recurrence through a carried
state: incoming state given, loss also on the final state) against the oracle's reverse differentiation.
Tolerances as in the zero-state backward tests, on the fp32 gradients; bf16 gradients must be their rounding."""
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


def _inputs(w, start, n, layout="bnhd"):
    q, k, v, gam = wl.prefill_inputs(w, layout=layout)
    rng = np.random.default_rng(w.seed + 101)
    g = wl.store_round(rng.standard_normal((w.B, w.N, w.Hh, w.d), dtype=np.float32) / np.float32(np.sqrt(w.d)), w.dtype)
    if layout == "bhnd":
        g = np.ascontiguousarray(g.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    q, k, v, g = (x[:, start:start + n] for x in (q, k, v, g))
    s0 = wl.random_state(w, w.seed + 3)
    h = wl.random_state(w, w.seed + 4) * np.float32(0.25)
    return q, k, v, g, gam, s0, h


def _gpu(lasad, w, q, k, v, g, gam, s0, h, start, mode, q_scale, grad_bf16):
    import torch
    dev = lambda x: lasad.to_device(x, w.dtype)
    st = lambda x: None if x is None else torch.from_numpy(np.ascontiguousarray(x)).cuda()
    res = both_outputs(lasad.lasad_backward_chunked_carried, grad_bf16 and w.dtype == "bf16", dtype_kw="grad_dtype",
                       q=dev(q), k=dev(k), v=dev(v), d_o=dev(g), gamma=torch.from_numpy(gam).cuda(),
                       grid_h=w.grid_h, grid_w=w.grid_w, state_in=st(s0), d_state_out=st(h),
                       start_pos=start, boundary_mode=mode, q_scale=q_scale)
    torch.cuda.synchronize()
    return [r.cpu().numpy() for r in res]


def _check(lasad, oracle, w, start=0, n=None, mode=0, q_scale=1.0, grad_bf16=False, layout="bnhd",
           with_s0=True, with_h=True):
    n = w.N - start if n is None else n
    q, k, v, g, gam, s0, h = _inputs(w, start, n, layout)
    s0 = s0 if with_s0 else None
    h = h if with_h else None
    dq, dk, dv, dgam, ds0 = _gpu(lasad, w, q, k, v, g, gam, s0, h, start, mode, q_scale, grad_bf16)
    lam, cum = oracle.decay_factors(gam, w.grid_h, w.grid_w, start, n, mode)
    rq, rk, rv, rlam, rs0 = oracle.backward_carried(q, k, v, lam, g, s0=s0, d_state=h, q_scale=q_scale)
    rgam = oracle.dgamma(rlam, w.grid_w, start, mode)
    tol = TOL[w.dtype]
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv), ("d_state_in", ds0, rs0)):
        if got.size:
            err = rel_err(got, ref)
            assert err <= tol, (name, err)
    # dgamma: relative to its largest entry plus the fp32 rounding floor of the kernel's sum
    # (1 / gamma) [ sum_t E_t (q_t . dq_t - k_t . dk_t) + E_n <H, s_n> ], which scales with the sum of the absolute terms
    E = (cum[1:] - cum[0]).astype(np.float64)
    terms = (np.abs(q * rq).sum(axis=3) + np.abs(k * rk).sum(axis=3)) * E[None, :, None]
    floor = terms.sum(axis=(0, 1)).max()
    if h is not None and n > 0:
        _, sn = oracle.recurrent(q, k, v, lam, q_scale=1.0, s0=s0, want_state=True)
        floor += float(E[-1]) * np.abs(h * sn).sum(axis=(2, 3)).sum(axis=0).max()
    rel = 2e-2 if w.dtype == "bf16" else 1e-4
    assert np.abs(dgam - rgam).max() <= rel * np.abs(rgam).max() + 1e-6 * floor / float(gam.min()), (dgam, rgam)


CASES = [
    # name, B, Hh, d, H, W, dtype
    ("f32_d32", 1, 2, 32, 4, 5, "f32"),
    ("f32_d64", 2, 2, 64, 7, 9, "f32"),
    ("f32_d128", 1, 1, 128, 3, 5, "f32"),
    ("bf16_one_chunk", 2, 3, 64, 5, 7, "bf16"),
    ("bf16_chunks_and_tail", 2, 2, 64, 13, 17, "bf16"),
    ("bf16_single_row", 1, 2, 64, 1, 70, "bf16"),
    ("bf16_d32", 2, 2, 32, 6, 9, "bf16"),
    ("bf16_single_token", 1, 2, 64, 1, 1, "bf16"),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_backward_carried_shapes(lasad, oracle, case, mode):
    name, B, Hh, d, H, W, dtype = case
    w = wl.Workload(name, B, Hh, d, H, W, dtype, 0.6, 0.999, seed=zlib.crc32(name.encode()) % 10000 + mode)
    _check(lasad, oracle, w, mode=mode, q_scale=0.5, grad_bf16=True)


@pytest.mark.parametrize("with_s0,with_h", [(True, False), (False, True), (False, False)])
def test_backward_carried_optional_states(lasad, oracle, with_s0, with_h):
    """Either state may be absent (zeros); without both the call is lasad_backward_chunked plus dL/d(state_in)."""
    w = wl.Workload("carried_opt", 2, 3, 64, 9, 17, "bf16", 0.7, 0.999, seed=77)
    _check(lasad, oracle, w, with_s0=with_s0, with_h=with_h)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("start,n", [(5, 100), (17, 64), (16, 3), (33, 0)])
def test_backward_carried_partial_range(lasad, oracle, mode, start, n):
    """Mid-row start and end; n = 0: the state gradient passes through, dgamma is zero."""
    w = wl.Workload("carried_range", 2, 2, 64, 9, 17, "bf16", 0.7, 0.999, seed=4242 + start)
    _check(lasad, oracle, w, start=start, mode=mode, n=n)


@pytest.mark.parametrize("layout", ["bnhd", "bhnd"])
def test_backward_carried_layouts(lasad, oracle, layout):
    w = wl.Workload("carried_layout", 2, 3, 64, 10, 12, "bf16", 0.8, 0.999, seed=78)
    _check(lasad, oracle, w, layout=layout, grad_bf16=True)


def test_backward_carried_small_gamma_heads(lasad, oracle):
    """Heads whose decay is too small for the separable factors take the fp32 recurrence, which skips the first
    decay of the reversed passes itself (no division by the decay); gamma = 0 included."""
    import torch
    w = wl.Workload("carried_small_gamma", 1, 4, 64, 6, 16, "bf16", 0.8, 0.99, seed=5)
    q, k, v, g, gam, s0, h = _inputs(w, 0, w.N)
    gam = np.array([0.3, 0.95, 0.05, 0.0], dtype=np.float32)
    dq, dk, dv, dgam, ds0 = _gpu(lasad, w, q, k, v, g, gam, s0, h, 0, 0, 1.0, False)
    lam, _ = oracle.decay_factors(gam, w.grid_h, w.grid_w, 0, w.N, 0)
    rq, rk, rv, rlam, rs0 = oracle.backward_carried(q, k, v, lam, g, s0=s0, d_state=h)
    for nm, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv), ("d_state_in", ds0, rs0)):
        assert rel_err(got, ref) <= TOL["bf16"], nm
    rgam = oracle.dgamma(rlam, w.grid_w, 0, 0)
    assert np.abs(dgam[:3] - rgam[:3]).max() <= 2e-2 * np.abs(rgam[:3]).max()      # gamma = 0: dgamma is not defined by the formula


@pytest.mark.parametrize("B,Hh,H,W", [(4, 12, 16, 16), (8, 12, 16, 16), (11, 8, 9, 15), (1, 2, 40, 16)],
                         ids=["48seq_twelve_wave", "96seq_eight_wave", "88seq_tail", "2seq_segmented"])
def test_backward_carried_launch_shapes(lasad, oracle, B, Hh, H, W):
    """Every launch shape of the three passes (merged twelve-wave and eight-wave launches, separate segmented passes)."""
    w = wl.Workload("carried_launch", B, Hh, 64, H, W, "bf16", 0.85, 0.999, seed=31 * B + Hh)
    _check(lasad, oracle, w, grad_bf16=True)
    _check(lasad, oracle, w, mode=1, q_scale=0.25)


def test_two_chained_gpu_calls_equal_one_call(lasad, oracle):
    """A sequence cut in two on the GPU: the forward hands its state over, the second backward call's d_state_in is the
    first call's d_state_out.  All gradients of the pair against the single call over the whole sequence."""
    import torch
    w = wl.Workload("carried_chain", 2, 3, 64, 12, 16, "bf16", 0.8, 0.999, seed=91)
    q, k, v, g, gam, s0, h = _inputs(w, 0, w.N)
    dev = lambda x: lasad.to_device(np.ascontiguousarray(x), "bf16")
    tg = torch.from_numpy(gam).cuda()
    ts0, th = torch.from_numpy(s0).cuda(), torch.from_numpy(h).cuda()
    kw = dict(grad_dtype=torch.float32)
    whole = lasad.lasad_backward_chunked_carried(dev(q), dev(k), dev(v), dev(g), tg, w.grid_h, w.grid_w,
                                                 state_in=ts0, d_state_out=th, **kw)
    p = 101
    s_mid = torch.empty_like(ts0)
    lasad.lasad_forward_chunked(dev(q[:, :p]), dev(k[:, :p]), dev(v[:, :p]), tg, w.grid_h, w.grid_w, state_in=ts0, state_out=s_mid)
    second = lasad.lasad_backward_chunked_carried(dev(q[:, p:]), dev(k[:, p:]), dev(v[:, p:]), dev(g[:, p:]), tg, w.grid_h, w.grid_w,
                                                  state_in=s_mid, d_state_out=th, start_pos=p, **kw)
    first = lasad.lasad_backward_chunked_carried(dev(q[:, :p]), dev(k[:, :p]), dev(v[:, :p]), dev(g[:, :p]), tg, w.grid_h, w.grid_w,
                                                 state_in=ts0, d_state_out=second[4], **kw)
    torch.cuda.synchronize()
    for i, nm in enumerate(("dq", "dk", "dv")):
        both = torch.cat([first[i], second[i]], dim=1).cpu().numpy()
        assert rel_err(both, whole[i].cpu().numpy()) <= TOL["bf16"], nm
    assert rel_err(first[4].cpu().numpy(), whole[4].cpu().numpy()) <= TOL["bf16"]
    dg = (first[3] + second[3]).cpu().numpy()
    assert np.abs(dg - whole[3].cpu().numpy()).max() <= 2e-2 * np.abs(whole[3].cpu().numpy()).max()


@pytest.mark.parametrize("name", ["base_prefill_16x16", "large_prefill_24x24"])
def test_backward_carried_bench_shapes_sampled(lasad, oracle, name):
    """The benchmark shapes with carried states; the oracle on sampled sequences (fp32 gradients, bare tolerance)."""
    w = wl.CONFIGS[name]
    q, k, v, g, gam, s0, h = _inputs(w, 0, w.N)
    dq, dk, dv, dgam, ds0 = _gpu(lasad, w, q, k, v, g, gam, s0, h, 0, 0, 1.0, False)
    pairs = sample_pairs(w.B, w.Hh, 12, seed=w.seed)
    lam, _ = oracle.decay_factors(gam[[hh for _, hh in pairs]], w.grid_h, w.grid_w, 0, w.N, 0)
    sel = lambda x: np.stack([x[b, hh] for b, hh in pairs])[None]
    rq, rk, rv, _, rs0 = oracle.backward_carried(gather_pairs(q, pairs), gather_pairs(k, pairs), gather_pairs(v, pairs), lam,
                                                 gather_pairs(g, pairs), s0=sel(s0), d_state=sel(h))
    for nm, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        assert rel_err(gather_pairs(got, pairs), ref) <= TOL["bf16"], nm
    assert rel_err(sel(ds0), rs0) <= TOL["bf16"]
    assert np.isfinite(dgam).all()
