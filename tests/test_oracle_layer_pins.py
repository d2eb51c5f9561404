"""Pins of the elementwise steps of Algorithm 1 that surround the recurrence (oracle.silu, oracle.sigmoid,
oracle.rms_norm, oracle.gated_layer): known values and identities of the two activations, the defining
properties of a root-mean-square normalisation, and a hand-worked two-token layer."""
import math

import numpy as np
import pytest


def test_sigmoid_values_and_identities(oracle):
    assert oracle.sigmoid(0.0) == 0.5
    assert abs(oracle.sigmoid(math.log(3.0)) - 0.75) < 1e-15          # 1 / (1 + 1/3)
    assert abs(oracle.sigmoid(-math.log(3.0)) - 0.25) < 1e-15
    x = np.linspace(-40, 40, 161)
    s = oracle.sigmoid(x)
    assert np.allclose(s + oracle.sigmoid(-x), 1.0, atol=1e-15)          # sigma(-x) = 1 - sigma(x)
    assert np.all(np.diff(s) >= 0) and s[0] < 1e-17 and s[-1] == 1.0
    assert np.isfinite(oracle.sigmoid(np.array([-800.0, 800.0]))).all()  # no overflow
    # derivative sigma' = sigma (1 - sigma), by a central difference
    h = 1e-5
    d = (oracle.sigmoid(x + h) - oracle.sigmoid(x - h)) / (2 * h)
    assert np.allclose(d, s * (1 - s), atol=1e-9)


def test_silu_values(oracle):
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(math.log(3.0)) - 0.75 * math.log(3.0)) < 1e-15
    assert abs(oracle.silu(-math.log(3.0)) + 0.25 * math.log(3.0)) < 1e-15
    assert abs(oracle.silu(50.0) - 50.0) < 1e-12 and abs(oracle.silu(-50.0)) < 1e-12
    x = np.linspace(-6, 6, 49)
    assert np.allclose(oracle.silu(x) - oracle.silu(-x), x, atol=1e-14)   # SiLU(x) - SiLU(-x) = x


def test_rms_norm_properties(oracle):
    rng = np.random.default_rng(1)
    o = rng.standard_normal((2, 5, 3, 8))
    y = oracle.rms_norm(o, eps=0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, atol=1e-14)           # unit RMS per token and head
    assert np.allclose(oracle.rms_norm(7.5 * o, eps=0.0), y, atol=1e-13)             # scale invariant
    assert np.allclose(oracle.rms_norm(np.array([3.0, -4.0, 0.0, 0.0]), eps=0.0), [1.2, -1.6, 0.0, 0.0])  # rms = 2.5
    w = rng.standard_normal((3, 8))
    assert np.allclose(oracle.rms_norm(o, w, eps=0.0), y * w[None, None], atol=1e-14)
    assert np.allclose(oracle.rms_norm(np.array([2.0, 2.0]), eps=5.0), [2.0 / 3.0] * 2)   # sqrt(4 + 5) = 3
    assert not oracle.rms_norm(np.zeros(4), eps=1e-6).any()


def test_layer_hand_worked(oracle):
    """Two tokens on a 1 x 2 grid (the second is a row end), d = 2, inputs chosen so that the activations are
    exact: z = +-ln 3 gives lambda = 0.75 / 0.25, q_pre = ln 3 gives q = 0.75 ln 3.
      token 1: lambda = (0.75, 0.25), k = (0.25, 0.75), v = (4, 8):  s = [[1, 2], [3, 6]]
               q = (a, 0) with a = 0.75 ln 3:  o = a (1, 2) -> rms norm (eps 0): (1, 2) / sqrt(2.5)
      token 2 (boundary, decay 1): lambda = (0.25, 0.25) -> k = (0.75, 0.75), v = (4, 0): s = [[4, 2], [6, 6]]
               q = (0, a):  o = a (6, 6) -> (1, 1)."""
    L = math.log(3.0)
    q_pre = np.array([[L, 0.0], [0.0, L]]).reshape(1, 2, 1, 2)
    z = np.array([[L, -L], [-L, -L]]).reshape(1, 2, 1, 2)
    v = np.array([[4.0, 8.0], [4.0, 0.0]]).reshape(1, 2, 1, 2)
    o, s = oracle.gated_layer(q_pre, z, v, grid_w=2, eps=0.0, want_state=True)
    assert np.allclose(s[0, 0], [[4.0, 2.0], [6.0, 6.0]], atol=1e-14)
    assert np.allclose(o[0, 0, 0], np.array([1.0, 2.0]) / math.sqrt(2.5), atol=1e-14)
    assert np.allclose(o[0, 1, 0], [1.0, 1.0], atol=1e-14)
    # the same layer assembled by hand from the pinned pieces
    ref = oracle.rms_norm(oracle.gated_recurrent(oracle.silu(q_pre), oracle.sigmoid(z), v, 2), eps=0.0)
    assert np.array_equal(o, ref)


# ---- gradients of the layer ---------------------------------------------------------------------

def _num_grad(f, x, h):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = f()
        x[i] = old - h
        fm = f()
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


@pytest.mark.parametrize("weighted", [False, True])
@pytest.mark.parametrize("mode", [0, 2])
def test_layer_backward_against_finite_differences_of_the_layer(oracle, weighted, mode):
    """gated_layer_backward against central differences of gated_layer (pinned above) in every input entry."""
    rng = np.random.default_rng(7 + mode)
    B, Hh, H, W, d = 1, 2, 2, 3, 3
    n = H * W
    q, z, v, g = (rng.standard_normal((B, n, Hh, d)) for _ in range(4))
    w = rng.uniform(0.5, 1.5, size=(Hh, d)) if weighted else None
    kw = dict(norm_weight=w, eps=1e-3, mode=mode, q_scale=0.8)
    dq, dz, dv, dw = oracle.gated_layer_backward(q, z, v, g, W, **kw)
    loss = lambda: float((oracle.gated_layer(q, z, v, W, **kw) * g).sum())
    assert np.allclose(dq, _num_grad(loss, q, 1e-5), rtol=1e-6, atol=1e-8)
    assert np.allclose(dz, _num_grad(loss, z, 1e-5), rtol=1e-6, atol=1e-8)
    assert np.allclose(dv, _num_grad(loss, v, 1e-5), rtol=1e-6, atol=1e-8)
    if not weighted:                       # without a weight: the gradient at a weight of ones
        w = kw["norm_weight"] = np.ones((Hh, d))
    assert np.allclose(dw, _num_grad(loss, w, 1e-5), rtol=1e-6, atol=1e-8)


def test_layer_backward_is_blind_to_the_scale_of_v(oracle):
    """With eps = 0 the normalisation removes any common factor of the recurrence output, and that output is
    linear in v: scaling v leaves the layer output unchanged, so the gradient is orthogonal to v, <dv, v> = 0."""
    rng = np.random.default_rng(3)
    q, z, v, g = (rng.standard_normal((1, 6, 1, 4)) for _ in range(4))
    _, _, dv, _ = oracle.gated_layer_backward(q, z, v, g, 3, eps=0.0)
    assert abs(float((dv * v).sum())) <= 1e-10 * float(np.abs(dv * v).sum())


def test_layer_backward_is_the_chain_of_its_two_parts(oracle):
    """gated_layer_backward = layer_core_backward after layer_norm_backward; the tensor gradients are linear in
    the gradient that passes between the two parts, the weight gradient does not depend on it."""
    rng = np.random.default_rng(11)
    q, z, v, g = (rng.standard_normal((1, 6, 2, 4)) for _ in range(4))
    w = rng.uniform(0.5, 1.5, size=(2, 4))
    base = oracle.gated_layer_backward(q, z, v, g, 3, norm_weight=w)
    d_o, dw = oracle.layer_norm_backward(q, z, v, g, 3, norm_weight=w)
    once = oracle.layer_core_backward(q, z, v, d_o, 3)
    twice = oracle.layer_core_backward(q, z, v, 2 * d_o, 3)
    for i in range(3):
        assert np.array_equal(base[i], once[i])
        assert np.allclose(twice[i], 2 * base[i], rtol=1e-12, atol=0)
    assert np.array_equal(base[3], dw)


@pytest.mark.parametrize("mode", [0, 1])
def test_layer_backward_against_torch_autograd_of_a_mask_form(oracle, mode):
    """Automatic differentiation (torch, fp64) of an independent implementation of the whole layer: activations,
    tied key, the recurrence unrolled as a per-channel mask o_i = sum_{j<=i} sum_c q_i[c] k_j[c] D[i][j][c] v_j with
    D from cumulative log-decays (0 at boundary positions), then the root-mean-square normalisation."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(21 + mode)
    B, Hh, H, W, d = 2, 2, 3, 4, 5
    n = H * W
    q, z, v, g = (rng.standard_normal((B, n, Hh, d)) for _ in range(4))
    w = rng.uniform(0.5, 1.5, size=(Hh, d))
    eps, qs = 1e-4, 0.7
    tq, tz, tv, tw = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, z, v, w))
    lam = torch.sigmoid(tz)
    key = 1.0 - lam
    pos = np.arange(1, n + 1)
    boundary = (pos % W == 0) if mode == 0 else ((pos - 1) % W == 0)
    keep = torch.tensor(~boundary, dtype=torch.float64)[None, :, None, None]
    cl = torch.cumsum(torch.log(lam) * keep, dim=1)                          # [B, n, Hh, d]
    D = torch.exp(cl[:, :, None] - cl[:, None, :])                           # [B, i, j, Hh, d]
    causal = torch.tril(torch.ones(n, n, dtype=torch.float64))[None, :, :, None]
    scores = torch.einsum("bihc,bjhc,bijhc->bijh", torch.nn.functional.silu(tq), key, D) * causal * qs
    o = torch.einsum("bijh,bjhe->bihe", scores, tv)
    y = o * torch.rsqrt((o * o).mean(dim=-1, keepdim=True) + eps) * tw
    assert np.allclose(y.detach().numpy(), oracle.gated_layer(q, z, v, W, norm_weight=w, eps=eps, mode=mode, q_scale=qs),
                       rtol=1e-10, atol=1e-12)
    (y * torch.tensor(g)).sum().backward()
    dq, dz, dv, dw = oracle.gated_layer_backward(q, z, v, g, W, norm_weight=w, eps=eps, mode=mode, q_scale=qs)
    for got, want in ((dq, tq.grad), (dz, tz.grad), (dv, tv.grad), (dw, tw.grad)):
        assert np.allclose(got, want.numpy(), rtol=1e-9, atol=1e-11)
