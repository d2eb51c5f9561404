"""GPU parity of lasad_backward_gated_carried (vector-decay gradients through a carried state) against the
oracle's reverse differentiation.  fp32 gradients against the bare tolerance; bf16 gradients are their rounding."""
import zlib

import numpy as np
import pytest

from paper_2507_01652_amd import workloads as wl
from helpers import TOL, both_outputs, gather_pairs, rel_err, sample_pairs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lasad():
    import torch
    assert torch.cuda.is_available()
    from paper_2507_01652_amd import binding
    binding.load()
    return binding


def _inputs(B, n, Hh, dtype, seed, own_key, layout="bnhd", d=64):
    rng = np.random.default_rng(seed)
    shape = (B, n, Hh, d)
    q, v, g = (wl.store_round(rng.standard_normal(shape, dtype=np.float32) / np.float32(np.sqrt(d)), dtype) for _ in range(3))
    lam = wl.gate_inputs(shape, dtype, seed + 1)
    k = wl.store_round(rng.uniform(0.0, 1.0, size=shape).astype(np.float32), dtype) if own_key else None
    out = [q, lam, v, g, k]
    if layout == "bhnd":
        out = [None if x is None else np.ascontiguousarray(x.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3) for x in out]
    s0 = (rng.standard_normal((B, Hh, d, d)) * 0.5).astype(np.float32)
    h = (rng.standard_normal((B, Hh, d, d)) * 0.125).astype(np.float32)
    return out + [s0, h]


def _check(lasad, oracle, B, Hh, H, W, dtype, seed, own_key, start=0, n=None, mode=0, q_scale=1.0, grad_bf16=False,
           layout="bnhd", with_s0=True, with_h=True, d=64):
    import torch
    n = H * W - start if n is None else n
    q, lam, v, g, k, s0, h = _inputs(B, n, Hh, dtype, seed, own_key, layout, d)
    s0 = s0 if with_s0 else None
    h = h if with_h else None
    dev = lambda x: None if x is None else lasad.to_device(x, dtype)
    st = lambda x: None if x is None else torch.from_numpy(x).cuda()
    got = both_outputs(lasad.lasad_backward_gated_carried, grad_bf16 and dtype == "bf16", dtype_kw="grad_dtype",
                       q=dev(q), lam=dev(lam), v=dev(v), d_o=dev(g), grid_h=H, grid_w=W, k=dev(k),
                       state_in=st(s0), d_state_out=st(h), start_pos=start, boundary_mode=mode, q_scale=q_scale)
    torch.cuda.synchronize()
    got = [x.cpu().numpy() for x in got]
    ref = oracle.gated_backward_carried(q, lam, v, g, W, k=k, s0=s0, d_state=h, start_pos=start, mode=mode, q_scale=q_scale)
    names = ("dq", "dlam", "dv", "dk", "d_state_in") if own_key else ("dq", "dlam", "dv", "d_state_in")
    for nm, a, r in zip(names, got, ref):
        if a.size == 0:
            continue
        # dlam is a suffix sum divided by lambda (see the zero-state tests): for fp32 the tolerance, which sits at the
        # rounding level of the walks, is divided by the smallest decay of the input
        tol = TOL[dtype] / float(lam.min()) if nm == "dlam" and dtype == "f32" else TOL[dtype]
        assert rel_err(a, r) <= tol, (nm, rel_err(a, r))


CASES = [
    ("f32_small", 1, 2, 4, 5, "f32"),
    ("f32_batches", 2, 2, 7, 9, "f32"),
    ("bf16_one_chunk", 2, 3, 3, 5, "bf16"),
    ("bf16_chunks_and_tail", 2, 2, 13, 17, "bf16"),
    ("bf16_single_row", 1, 2, 1, 70, "bf16"),
    ("bf16_single_token", 1, 2, 1, 1, "bf16"),
]


@pytest.mark.parametrize("d", [32, 128])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("own_key", [False, True], ids=["tied_key", "own_key"])
def test_backward_gated_carried_other_head_dims(lasad, oracle, d, dtype, own_key):
    for mode in (0, 1, 2):
        _check(lasad, oracle, 2, 2, 5, 7, dtype, 700 + d + mode, own_key, mode=mode, q_scale=0.5, d=d, grad_bf16=True)
    _check(lasad, oracle, 1, 2, 9, 17, dtype, 750 + d, own_key, start=22, n=101, d=d, layout="bhnd")
    _check(lasad, oracle, 1, 2, 6, 5, dtype, 760 + d, own_key, d=d, with_s0=False)
    _check(lasad, oracle, 1, 2, 6, 5, dtype, 770 + d, own_key, d=d, with_h=False)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("own_key", [False, True], ids=["tied_key", "own_key"])
def test_backward_gated_carried_shapes(lasad, oracle, case, mode, own_key):
    name, B, Hh, H, W, dtype = case
    _check(lasad, oracle, B, Hh, H, W, dtype, zlib.crc32(name.encode()) % 10000 + mode, own_key, mode=mode, q_scale=0.5,
           grad_bf16=True)


@pytest.mark.parametrize("with_s0,with_h", [(True, False), (False, True), (False, False)])
def test_backward_gated_carried_optional_states(lasad, oracle, with_s0, with_h):
    _check(lasad, oracle, 2, 3, 9, 17, "bf16", 77, False, with_s0=with_s0, with_h=with_h)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("start,n", [(5, 100), (17, 64), (16, 3), (33, 0)])
def test_backward_gated_carried_partial_range(lasad, oracle, mode, start, n):
    _check(lasad, oracle, 2, 2, 9, 17, "bf16", 4242 + start, False, start=start, n=n, mode=mode)


def test_backward_gated_carried_layout_and_many_sequences(lasad, oracle):
    _check(lasad, oracle, 2, 3, 10, 12, "bf16", 78, True, layout="bhnd", grad_bf16=True)
    _check(lasad, oracle, 60, 3, 5, 8, "bf16", 9, False)


@pytest.mark.parametrize("H,W,own_key", [(40, 16, False), (29, 17, True)])
def test_backward_gated_carried_long_sequences(lasad, oracle, H, W, own_key):
    """Few long sequences: the finishing kernel works on several segments per sequence; every segment's suffix sums
    start from the products that end in the final state."""
    _check(lasad, oracle, 1, 2, H, W, "bf16", 300 + H, own_key, grad_bf16=True)
    _check(lasad, oracle, 1, 2, H, W, "f32", 400 + H, own_key)


def test_backward_gated_carried_strong_decay_takes_the_walks(lasad, oracle):
    """Gates around 0.18: every chunk leaves the chunked passes' range, the token-serial walks carry the states
    (the column walks read and write them transposed)."""
    import torch
    B, Hh, H, W = 1, 2, 6, 11
    rng = np.random.default_rng(5)
    shape = (B, H * W, Hh, 64)
    q, v, g = (wl.store_round(rng.standard_normal(shape, dtype=np.float32) / np.float32(8.0), "bf16") for _ in range(3))
    lam = wl.store_round((1.0 / (1.0 + np.exp(-(rng.standard_normal(shape) - 1.5)))).astype(np.float32), "bf16")
    s0 = (rng.standard_normal((B, Hh, 64, 64)) * 0.5).astype(np.float32)
    h = (rng.standard_normal((B, Hh, 64, 64)) * 0.125).astype(np.float32)
    dev = lambda x: lasad.to_device(x, "bf16")
    got = lasad.lasad_backward_gated_carried(dev(q), dev(lam), dev(v), dev(g), H, W, state_in=torch.from_numpy(s0).cuda(),
                                             d_state_out=torch.from_numpy(h).cuda(), grad_dtype=torch.float32)
    torch.cuda.synchronize()
    ref = oracle.gated_backward_carried(q, lam, v, g, W, s0=s0, d_state=h)
    for nm, a, r in zip(("dq", "dlam", "dv", "d_state_in"), got, ref):
        assert rel_err(a.cpu().numpy(), r) <= TOL["bf16"], nm


def test_two_chained_gated_gpu_calls_equal_one_call(lasad, oracle):
    import torch
    B, Hh, H, W = 2, 3, 12, 16
    n = H * W
    q, lam, v, g, _, s0, h = _inputs(B, n, Hh, "bf16", 91, False)
    dev = lambda x: lasad.to_device(np.ascontiguousarray(x), "bf16")
    ts0, th = torch.from_numpy(s0).cuda(), torch.from_numpy(h).cuda()
    kw = dict(grad_dtype=torch.float32)
    whole = lasad.lasad_backward_gated_carried(dev(q), dev(lam), dev(v), dev(g), H, W, state_in=ts0, d_state_out=th, **kw)
    p = 101
    s_mid = torch.empty_like(ts0)
    lasad.lasad_forward_gated(dev(q[:, :p]), dev(lam[:, :p]), dev(v[:, :p]), H, W, state_in=ts0, state_out=s_mid)
    second = lasad.lasad_backward_gated_carried(dev(q[:, p:]), dev(lam[:, p:]), dev(v[:, p:]), dev(g[:, p:]), H, W,
                                                state_in=s_mid, d_state_out=th, start_pos=p, **kw)
    first = lasad.lasad_backward_gated_carried(dev(q[:, :p]), dev(lam[:, :p]), dev(v[:, :p]), dev(g[:, :p]), H, W,
                                               state_in=ts0, d_state_out=second[3], **kw)
    torch.cuda.synchronize()
    for i, nm in enumerate(("dq", "dlam", "dv")):
        both = torch.cat([first[i], second[i]], dim=1).cpu().numpy()
        assert rel_err(both, whole[i].cpu().numpy()) <= TOL["bf16"], nm
    assert rel_err(first[3].cpu().numpy(), whole[3].cpu().numpy()) <= TOL["bf16"]


@pytest.mark.parametrize("name,n_pairs", [("base_prefill_16x16", 8), ("large_prefill_24x24", 8)])
def test_backward_gated_carried_bench_shapes_sampled(lasad, oracle, name, n_pairs):
    import torch
    w = wl.CONFIGS[name]
    q, lam, v, g, _, s0, h = _inputs(w.B, w.N, w.Hh, "bf16", w.seed + 11, False)
    dev = lambda x: lasad.to_device(x, "bf16")
    got = lasad.lasad_backward_gated_carried(dev(q), dev(lam), dev(v), dev(g), w.grid_h, w.grid_w,
                                             state_in=torch.from_numpy(s0).cuda(), d_state_out=torch.from_numpy(h).cuda(),
                                             grad_dtype=torch.float32)
    torch.cuda.synchronize()
    pairs = sample_pairs(w.B, w.Hh, n_pairs, seed=w.seed)
    sel = lambda x: np.stack([x[b, hh] for b, hh in pairs])[None]
    ref = oracle.gated_backward_carried(*(gather_pairs(x, pairs) for x in (q, lam, v, g)), w.grid_w, s0=sel(s0), d_state=sel(h))
    for nm, a, r in zip(("dq", "dlam", "dv"), got, ref):
        assert rel_err(gather_pairs(a.cpu().numpy(), pairs), r) <= TOL["bf16"], nm
    assert rel_err(sel(got[3].cpu().numpy()), ref[3]) <= TOL["bf16"]
