"""Pins of the oracle's gradient routine (oracle/lasad_oracle.c: lasad_oracle_backward, lasad_oracle_dgamma)
against things other than itself: a hand-differentiated two-token example, central finite differences of the
oracle's FORWARD full-mask form (a different function), automatic differentiation of a plain torch (fp64)
implementation of the full-mask form, the lambda = 1 reduction to causal linear attention (Section 3.2) whose
gradients are library matmuls, and structural properties (linearity in d_o, which d_o each gradient may see)."""
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_hand_worked_two_tokens(oracle):
    g = json.load(open(os.path.join(GOLDEN, "sad_backward_2tok.json")))
    as4 = lambda x: np.array(x, dtype=np.float64).reshape(1, 2, 1, 1)
    dq, dk, dv, dlam = oracle.backward(as4(g["q"]), as4(g["k"]), as4(g["v"]), np.array([g["lam"]]), as4(g["d_o"]))
    assert np.allclose(dq.ravel(), g["dq"], rtol=0, atol=1e-12)
    assert np.allclose(dk.ravel(), g["dk"], rtol=0, atol=1e-12)
    assert np.allclose(dv.ravel(), g["dv"], rtol=0, atol=1e-12)
    assert np.allclose(dlam.ravel(), g["dlam"], rtol=0, atol=1e-12)


def _loss(oracle, q, k, v, lam, d_o, q_scale):
    return float((oracle.forward_fullmask(q, k, v, lam, q_scale=q_scale) * d_o).sum())


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_finite_differences_of_the_forward_form(oracle, mode):
    """L = <forward(q, k, v, lam), d_o> is linear in q, in k and in v separately, so a central difference with
    any step is exact up to rounding; in lam it is a polynomial, and a small step is used."""
    B, Hh, H, W, d = 2, 2, 3, 4, 3
    n = H * W
    q, k, v, d_o = (_rand((B, n, Hh, d), s) for s in (1, 2, 3, 4))
    gam = np.array([0.8, 0.6], dtype=np.float32)
    lam, _ = oracle.decay_factors(gam, H, W, 0, n, mode)
    lam = lam.astype(np.float64)
    dq, dk, dv, dlam = oracle.backward(q, k, v, lam, d_o, q_scale=0.7)
    rng = np.random.default_rng(9)
    for name, x, gx in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[idx] += 0.5
            xm[idx] -= 0.5
            args = {"q": q, "k": k, "v": v}
            fd = _loss(oracle, **{**args, name: xp}, lam=lam, d_o=d_o, q_scale=0.7) - \
                 _loss(oracle, **{**args, name: xm}, lam=lam, d_o=d_o, q_scale=0.7)
            assert abs(fd - gx[idx]) <= 1e-9 * max(1.0, abs(gx[idx])), (name, idx)
    # lam is shared by the batch: d L / d lam[h, t] = sum_b dlam[b, h, t]
    for h in range(Hh):
        for t in range(n):
            lp, lm = lam.copy(), lam.copy()
            lp[h, t] += 1e-4
            lm[h, t] -= 1e-4
            fd = (_loss(oracle, q, k, v, lp, d_o, 0.7) - _loss(oracle, q, k, v, lm, d_o, 0.7)) / 2e-4
            assert abs(fd - dlam[:, h, t].sum()) <= 1e-6 * max(1.0, abs(fd)), (h, t)
    # and gamma: every non-boundary position of head h carries gamma_h
    dg = oracle.dgamma(dlam, W, 0, mode)
    for h in range(Hh):
        eps = 2.0 ** -12
        gp, gm = gam.copy(), gam.copy()
        gp[h] += eps
        gm[h] -= eps
        lp, _ = oracle.decay_factors(gp, H, W, 0, n, mode)
        lm, _ = oracle.decay_factors(gm, H, W, 0, n, mode)
        step = float(gp[h]) - float(gm[h])
        fd = (_loss(oracle, q, k, v, lp.astype(np.float64), d_o, 0.7) -
              _loss(oracle, q, k, v, lm.astype(np.float64), d_o, 0.7)) / step
        assert abs(fd - dg[h]) <= 1e-5 * max(1.0, abs(fd)), h


def test_against_torch_autograd_fullmask(oracle):
    torch = pytest.importorskip("torch")
    B, Hh, H, W, d = 1, 3, 4, 5, 4
    n = H * W
    q, k, v, d_o = (_rand((B, n, Hh, d), s) for s in (11, 12, 13, 14))
    gam = np.array([0.9, 0.5, 0.97], dtype=np.float32)
    lam, _ = oracle.decay_factors(gam, H, W, 0, n, 0)
    lam = lam.astype(np.float64)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    tl = torch.tensor(lam, dtype=torch.float64, requires_grad=True)
    # M[h, i, j] = prod_{s=j+1..i} lam[h, s] for j <= i, from cumulative logs
    cl = torch.cumsum(torch.log(tl), dim=1)
    M = torch.tril(torch.exp(cl[:, :, None] - cl[:, None, :]))
    scores = torch.einsum("bihd,bjhd->bhij", tq, tk) * M[None]
    o = torch.einsum("bhij,bjhd->bihd", scores, tv)
    (o * torch.tensor(d_o)).sum().backward()
    dq, dk, dv, dlam = oracle.backward(q, k, v, lam, d_o)
    for got, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad), (dlam.sum(axis=0), tl.grad)):
        ref = ref.numpy()
        assert np.abs(got - ref).max() <= 1e-10 * max(1.0, np.abs(ref).max())


def test_no_decay_reduces_to_causal_linear_attention(oracle):
    """lambda = 1 (Section 3.2): O = tril(Q K^T) V, so dQ = tril(dO V^T) K, dK = tril(dO V^T)^T Q,
    dV = tril(Q K^T)^T dO."""
    n, d = 9, 5
    q, k, v, d_o = (_rand((1, n, 1, d), s) for s in (21, 22, 23, 24))
    dq, dk, dv, _ = oracle.backward(q, k, v, np.ones((1, n)), d_o)
    Q, K, V, G = (x[0, :, 0, :] for x in (q, k, v, d_o))
    W = np.tril(G @ V.T)
    assert np.allclose(dq[0, :, 0], W @ K, atol=1e-12)
    assert np.allclose(dk[0, :, 0], W.T @ Q, atol=1e-12)
    assert np.allclose(dv[0, :, 0], np.tril(Q @ K.T).T @ G, atol=1e-12)


def test_structure(oracle):
    """Linear in d_o; dq_t sees only d_o_t; dk_t, dv_t see only d_o at tokens >= t; dlam of the first token
    is zero from a zero state."""
    B, n, Hh, d = 1, 7, 2, 3
    q, k, v, g1, g2 = (_rand((B, n, Hh, d), s) for s in (31, 32, 33, 34, 35))
    lam = np.random.default_rng(36).uniform(0.3, 1.0, size=(Hh, n))
    r1, r2 = oracle.backward(q, k, v, lam, g1), oracle.backward(q, k, v, lam, g2)
    r12 = oracle.backward(q, k, v, lam, 2.0 * g1 - 3.0 * g2)
    for a, b, c in zip(r1, r2, r12):
        assert np.allclose(c, 2.0 * a - 3.0 * b, atol=1e-12)
    t = 4
    g3 = g1.copy()
    g3[:, :t] = 0.0                      # keep only d_o at tokens >= t
    r3 = oracle.backward(q, k, v, lam, g3)
    assert np.array_equal(r3[0][:, t:], r1[0][:, t:]) and not r3[0][:, :t].any()     # dq
    assert np.allclose(r3[1][:, t:], r1[1][:, t:], atol=1e-13)                        # dk at t.. unchanged
    assert np.allclose(r3[2][:, t:], r1[2][:, t:], atol=1e-13)
    assert not r1[3][:, :, 0].any()


def test_dgamma_counts_only_decaying_positions(oracle):
    dlam = np.arange(2 * 1 * 6, dtype=np.float64).reshape(2, 1, 6)
    # grid width 3, positions 1..6: boundaries at 3, 6 (last column) or 1, 4 (first column)
    assert oracle.dgamma(dlam, 3, 0, 0)[0] == (0 + 1 + 3 + 4) + (6 + 7 + 9 + 10)
    assert oracle.dgamma(dlam, 3, 0, 1)[0] == (1 + 2 + 4 + 5) + (7 + 8 + 10 + 11)
    assert oracle.dgamma(dlam, 3, 0, 2)[0] == dlam.sum()
    assert oracle.dgamma(dlam, 3, 2, 0)[0] == (1 + 2 + 4 + 5) + (7 + 8 + 10 + 11)     # positions 3..8: boundaries 3, 6
