"""Vector-decay entry points over the range of chunk decays the factorised (chunked) form covers: independent
sigmoid gates of logits N(m, 1) for m from 2 (the benchmark's recipe, worst channel of a 64-token chunk near 2^-25)
down to 0 (median gate one half, worst channel near 2^-97, at the edge of the 2^-100 limit) and -0.5 (beyond it:
the token-serial walk).  Forward, backward, fused layer and its backward against the oracle at the bare tolerance;
the test also checks that the inputs' chunk decays are where this text says, so that each case runs the intended
path."""
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


# logit mean, bounds on log2 of the smallest chunk decay over all (sequence, chunk, channel)
CASES = [(2.0, -40, -15), (1.0, -60, -40), (0.5, -85, -62), (0.25, -95, -70), (0.0, -100, -85), (-0.5, -160, -105)]


@pytest.mark.parametrize("mu,lo,hi", CASES, ids=[f"logit_mean_{c[0]}" for c in CASES])
def test_gate_distributions(lasad, oracle, mu, lo, hi):
    import torch
    B, Hh, H, W, d = 4, 4, 16, 16, 64
    n = H * W
    shape = (B, n, Hh, d)
    rng = np.random.default_rng(int(mu * 100) + 1000)
    q, v, g = (wl.store_round(rng.standard_normal(shape, dtype=np.float32) / np.float32(8), "bf16") for _ in range(3))
    z = wl.store_round(rng.standard_normal(shape).astype(np.float32) + np.float32(mu), "bf16")
    lam = wl.store_round(oracle.sigmoid(z).astype(np.float32), "bf16")
    worst = np.log2(lam.astype(np.float64)).reshape(B, n // 64, 64, Hh, d).sum(axis=2).min()
    assert lo <= worst <= hi, worst
    dev = lambda x: lasad.to_device(x, "bf16")
    s1 = torch.empty((B, Hh, d, d), dtype=torch.float32, device="cuda")
    o = lasad.lasad_forward_gated(dev(q), dev(lam), dev(v), H, W, state_out=s1, out_dtype=torch.float32)
    dq, dl, dv = lasad.lasad_backward_gated(dev(q), dev(lam), dev(v), dev(g), H, W, grad_dtype=torch.float32)[:3]
    qp = wl.store_round(rng.standard_normal(shape, dtype=np.float32), "bf16")
    ol = lasad.lasad_forward_layer(dev(qp), dev(z), dev(v), H, W, norm_eps=1e-5, out_dtype=torch.float32)
    gl = lasad.lasad_backward_layer(dev(qp), dev(z), dev(v), dev(g), H, W, norm_eps=1e-5, grad_dtype=torch.float32)
    torch.cuda.synchronize()
    ro, rs = oracle.gated_recurrent(q, lam, v, W, want_state=True)
    rq, rl, rv = oracle.gated_backward(q, lam, v, g, W)[:3]
    rol = oracle.gated_layer(qp, z, v, W, eps=1e-5)
    rgl = oracle.gated_layer_backward(qp, z, v, g, W, eps=1e-5)
    got = dict(o=(o, ro), state=(s1, rs), dq=(dq, rq), dlam=(dl, rl), dv=(dv, rv), layer_o=(ol, rol),
               layer_dq=(gl[0], rgl[0]), layer_dz=(gl[1], rgl[1]), layer_dv=(gl[2], rgl[2]))
    for nm, (a, r) in got.items():
        err = rel_err(a.cpu().numpy(), r)
        assert err <= TOL["bf16"], (nm, err)
