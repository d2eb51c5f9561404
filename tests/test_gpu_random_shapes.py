"""Seeded sweep over irregular shapes (batch, heads, grid, start position, length, boundary rule, q_scale) for
every bf16 head-dim-64 entry point against the oracle: small enough for the oracle, ragged enough to hit chunk
tails, mid-row starts, single-chunk and multi-chunk sequences and every launch shape that depends on the number
of sequences."""
import numpy as np
import pytest

from paper_2507_01652_amd import workloads as wl
from helpers import TOL, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lasad():
    import torch
    assert torch.cuda.is_available()
    from paper_2507_01652_amd import binding
    binding.load()
    return binding


def _configs(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        H, W = int(rng.integers(1, 14)), int(rng.integers(1, 40))
        total = H * W
        start = int(rng.integers(0, total))
        n = int(rng.integers(1, total - start + 1))
        B = int(rng.choice([1, 2, 3, 7, 50, 130, 260]))      # (with 1-3 heads: both sides of the 128 / 256 / 512 sequence thresholds)
        Hh = int(rng.integers(1, 4))
        if B * Hh * n > 60000:           # keep the oracle fast
            B = 2
        out.append(dict(B=B, Hh=Hh, H=H, W=W, start=start, n=n, mode=int(rng.integers(0, 3)),
                        q_scale=float(rng.choice([1.0, 0.125, 0.7])), seed=1000 * seed + i))
    return out


def _id(c):
    return f"B{c['B']}h{c['Hh']}_{c['H']}x{c['W']}_s{c['start']}n{c['n']}m{c['mode']}"


SCALAR = _configs(40, 1)
GATED = _configs(40, 2)


@pytest.mark.parametrize("c", SCALAR, ids=[_id(c) for c in SCALAR])
def test_scalar_forward_and_backward(lasad, oracle, c):
    import torch
    rng = np.random.default_rng(c["seed"])
    shape = (c["B"], c["n"], c["Hh"], 64)
    q, k, v, g = (wl.store_round(rng.standard_normal(shape, dtype=np.float32) / np.float32(8.0), "bf16") for _ in range(4))
    gam = rng.uniform(0.55, 0.999, size=(c["Hh"],)).astype(np.float32)
    s0 = (rng.standard_normal((c["B"], c["Hh"], 64, 64)) * 0.2).astype(np.float32)
    dev = lambda x: lasad.to_device(x, "bf16")
    tg = torch.from_numpy(gam).cuda()
    s1 = torch.empty((c["B"], c["Hh"], 64, 64), dtype=torch.float32, device="cuda")
    o = lasad.lasad_forward_chunked(dev(q), dev(k), dev(v), tg, c["H"], c["W"], start_pos=c["start"], boundary_mode=c["mode"],
                                    q_scale=c["q_scale"], state_in=torch.from_numpy(s0).cuda(), state_out=s1,
                                    out_dtype=torch.float32)
    dq, dk, dv, dgam = lasad.lasad_backward_chunked(dev(q), dev(k), dev(v), dev(g), tg, c["H"], c["W"], start_pos=c["start"],
                                                    boundary_mode=c["mode"], q_scale=c["q_scale"], grad_dtype=torch.float32)
    torch.cuda.synchronize()
    lam, _ = oracle.decay_factors(gam, c["H"], c["W"], c["start"], c["n"], c["mode"])
    ref, s_ref = oracle.recurrent(q, k, v, lam, q_scale=c["q_scale"], s0=s0.astype(np.float64), want_state=True)
    assert rel_err(o.cpu().numpy(), ref) <= TOL["bf16"]
    assert rel_err(s1.cpu().numpy(), s_ref) <= TOL["bf16"]
    rq, rk, rv, rlam = oracle.backward(q, k, v, lam, g, q_scale=c["q_scale"])
    for nm, got, want in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        assert rel_err(got.cpu().numpy(), want) <= TOL["bf16"], nm
    rgam = oracle.dgamma(rlam, c["W"], c["start"], c["mode"])
    # relative to the largest |dgamma| plus an fp32 rounding floor: the kernel sums E_t (q.dq - k.dk) / gamma in fp32
    _, cum = oracle.decay_factors(gam, c["H"], c["W"], c["start"], c["n"], c["mode"])
    E = (cum[1:] - cum[0]).astype(np.float64)
    terms = (np.abs(q * rq).sum(axis=3) + np.abs(k * rk).sum(axis=3)) * E[None, :, None]
    floor = 1e-6 * terms.sum(axis=(0, 1)).max() / float(gam.min()) + 1e-30
    assert np.abs(dgam.cpu().numpy() - rgam).max() <= 2e-2 * np.abs(rgam).max() + floor


@pytest.mark.parametrize("c", GATED, ids=[_id(c) for c in GATED])
def test_gated_forward_layer_and_backward(lasad, oracle, c):
    import torch
    rng = np.random.default_rng(c["seed"])
    shape = (c["B"], c["n"], c["Hh"], 64)
    q, v, g = (wl.store_round(rng.standard_normal(shape, dtype=np.float32) / np.float32(8.0), "bf16") for _ in range(3))
    z = wl.store_round(rng.standard_normal(shape, dtype=np.float32) + np.float32(2.0), "bf16")
    lam = wl.gate_inputs(shape, "bf16", c["seed"] + 1)
    dev = lambda x: lasad.to_device(x, "bf16")
    kw = dict(start_pos=c["start"], boundary_mode=c["mode"], q_scale=c["q_scale"])
    o = lasad.lasad_forward_gated(dev(q), dev(lam), dev(v), c["H"], c["W"], out_dtype=torch.float32, **kw)
    ol = lasad.lasad_forward_layer(dev(q), dev(z), dev(v), c["H"], c["W"], norm_eps=1e-5, out_dtype=torch.float32, **kw)
    dq, dlam, dv = lasad.lasad_backward_gated(dev(q), dev(lam), dev(v), dev(g), c["H"], c["W"], grad_dtype=torch.float32, **kw)
    torch.cuda.synchronize()
    okw = dict(start_pos=c["start"], mode=c["mode"], q_scale=c["q_scale"])
    assert rel_err(o.cpu().numpy(), oracle.gated_recurrent(q, lam, v, c["W"], **okw)) <= TOL["bf16"]
    assert rel_err(ol.cpu().numpy(), oracle.gated_layer(q, z, v, c["W"], eps=1e-5, **okw)) <= TOL["bf16"]
    rq, rlam, rv = oracle.gated_backward(q, lam, v, g, c["W"], **okw)
    for nm, got, want in (("dq", dq, rq), ("dlam", dlam, rlam), ("dv", dv, rv)):
        assert rel_err(got.cpu().numpy(), want) <= TOL["bf16"], nm
    # backward of the layer: its two parts as calls of their own, and the whole call
    d_o, dw = lasad.lasad_backward_layer_norm(dev(q), dev(z), dev(v), dev(g), c["H"], c["W"], norm_eps=1e-5,
                                              d_o_dtype=torch.float32, **kw)
    r_d_o, r_dw = oracle.layer_norm_backward(q, z, v, g, c["W"], eps=1e-5, **okw)
    d_o_in = wl.store_round(r_d_o.astype(np.float32), "bf16")
    lq, lz, lv, _ = lasad.lasad_backward_layer(dev(q), dev(z), dev(v), dev(d_o_in), c["H"], c["W"], norm_eps=-1.0,
                                               grad_dtype=torch.float32, **kw)
    whole = lasad.lasad_backward_layer(dev(q), dev(z), dev(v), dev(g), c["H"], c["W"], norm_eps=1e-5,
                                       grad_dtype=torch.float32, **kw)
    torch.cuda.synchronize()
    assert rel_err(d_o.cpu().numpy(), r_d_o) <= TOL["bf16"]
    assert rel_err(dw.cpu().numpy(), r_dw) <= TOL["bf16"]
    for nm, got, want in zip(("dq_pre", "dz", "dv"), (lq, lz, lv), oracle.layer_core_backward(q, z, v, d_o_in, c["W"], **okw)):
        assert rel_err(got.cpu().numpy(), want) <= TOL["bf16"], nm
    for nm, got, want in zip(("dq_pre", "dz", "dv"), whole, oracle.gated_layer_backward(q, z, v, g, c["W"], eps=1e-5, **okw)):
        assert rel_err(got.cpu().numpy(), want) <= TOL["bf16"], nm
    assert torch.equal(whole[3], dw)
