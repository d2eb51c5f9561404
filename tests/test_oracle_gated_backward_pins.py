"""Pins of the oracle's vector-decay gradient routine (oracle/lasad_oracle.c: lasad_oracle_gated_backward)
against things other than itself: a hand-differentiated two-token example with and without a row boundary,
central finite differences of the oracle's vector-decay FORWARD (a different function, itself pinned against
brute force), the reduction to the one-decay-per-token gradients when every channel carries the same decay,
and structural properties (what a boundary position and the tied key contribute)."""
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


@pytest.mark.parametrize("case", ["no_boundary", "token_2_is_a_boundary"])
def test_hand_worked_two_tokens(oracle, case):
    g = json.load(open(os.path.join(GOLDEN, "gated_backward_2tok.json")))
    c = g[case]
    as4 = lambda x: np.array(x, dtype=np.float64).reshape(1, 2, 1, 1)
    o = oracle.gated_recurrent(as4(g["q"]), as4(g["lam"]), as4(g["v"]), c["grid_w"])
    assert np.allclose(o.ravel(), c["o"], rtol=0, atol=1e-12)
    dq, dlam, dv = oracle.gated_backward(as4(g["q"]), as4(g["lam"]), as4(g["v"]), as4(g["d_o"]), c["grid_w"])
    assert np.allclose(dq.ravel(), c["dq"], rtol=0, atol=1e-12)
    assert np.allclose(dv.ravel(), c["dv"], rtol=0, atol=1e-12)
    assert np.allclose(dlam.ravel(), c["dlam"], rtol=0, atol=1e-12)


def _numeric_grad(f, x, h):
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


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("own_key", [False, True])
def test_finite_differences_of_the_forward(oracle, mode, own_key):
    """L = <gated_recurrent(q, lam, v[, k]), d_o> is linear in q, v and k separately (central differences exact
    up to rounding) and a polynomial in lam (small step)."""
    B, Hh, H, W, d, start = 1, 2, 3, 3, 3, 2
    n = H * W - start
    q, v, d_o = (_rand((B, n, Hh, d), s) for s in (1, 2, 3))
    lam = np.random.default_rng(4).uniform(0.2, 0.95, size=(B, n, Hh, d))
    k = _rand((B, n, Hh, d), 5) if own_key else None
    res = oracle.gated_backward(q, lam, v, d_o, W, k=k, start_pos=start, mode=mode, q_scale=0.7)
    loss = lambda: float((oracle.gated_recurrent(q, lam, v, W, k=k, start_pos=start, mode=mode, q_scale=0.7) * d_o).sum())
    assert np.allclose(res[0], _numeric_grad(loss, q, 0.5), rtol=1e-9, atol=1e-9)
    assert np.allclose(res[2], _numeric_grad(loss, v, 0.5), rtol=1e-9, atol=1e-9)
    assert np.allclose(res[1], _numeric_grad(loss, lam, 1e-4), rtol=1e-6, atol=1e-7)
    if own_key:
        assert np.allclose(res[3], _numeric_grad(loss, k, 0.5), rtol=1e-9, atol=1e-9)


@pytest.mark.parametrize("mode", [0, 1])
def test_same_decay_in_every_channel_reduces_to_the_scalar_gradients(oracle, mode):
    """With an own key and lambda_t[c] = the per-head table value for every channel c, dq, dk, dv are those of the
    one-decay-per-token routine, and the channel sum of dlam is its dlam at non-boundary positions (0 at boundaries,
    where the applied decay is the constant 1 in both routines' callers)."""
    B, Hh, H, W, d = 2, 2, 4, 3, 4
    n = H * W
    q, k, v, d_o = (_rand((B, n, Hh, d), s) for s in (11, 12, 13, 14))
    gam = np.array([0.9, 0.55], dtype=np.float32)
    lam_tab, _ = oracle.decay_factors(gam, H, W, 0, n, mode)               # [Hh, n], 1 at boundaries
    base = np.broadcast_to(gam.astype(np.float64)[None, None, :, None], (B, n, Hh, d)).copy()
    dq, dlam, dv, dk = oracle.gated_backward(q, base, v, d_o, W, k=k, mode=mode)
    rq, rk, rv, rlam = oracle.backward(q, k, v, lam_tab, d_o)
    assert np.allclose(dq, rq, rtol=1e-12, atol=1e-12)
    assert np.allclose(dk, rk, rtol=1e-12, atol=1e-12)
    assert np.allclose(dv, rv, rtol=1e-12, atol=1e-12)
    boundary = (lam_tab == 1.0)                                            # [Hh, n]
    want = np.where(boundary.T[None], 0.0, rlam.transpose(0, 2, 1))       # rlam: [B, Hh, n] -> [B, n, Hh]
    assert np.allclose(dlam.sum(axis=3), want, rtol=1e-10, atol=1e-10)


def test_tied_key_is_the_own_key_result_minus_dk(oracle):
    """k = 1 - lambda adds -dk to the decay gradient and changes nothing else (chain rule)."""
    B, Hh, H, W, d = 1, 2, 3, 4, 3
    n = H * W
    q, v, d_o = (_rand((B, n, Hh, d), s) for s in (21, 22, 23))
    lam = np.random.default_rng(24).uniform(0.1, 0.99, size=(B, n, Hh, d))
    dq, dlam, dv = oracle.gated_backward(q, lam, v, d_o, W)
    oq, olam, ov, ok = oracle.gated_backward(q, lam, v, d_o, W, k=1.0 - lam)
    assert np.allclose(dq, oq) and np.allclose(dv, ov)
    assert np.allclose(dlam, olam - ok, rtol=1e-12, atol=1e-12)
    pos = np.arange(1, n + 1)
    assert np.all(olam[:, pos % W == 0] == 0.0)           # boundary positions: no gradient through the decay
    assert np.all(olam[:, 0] == 0.0)                      # first token: its decay multiplies the zero state


@pytest.mark.parametrize("own_key", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_against_torch_autograd_of_a_mask_form(oracle, mode, own_key):
    """Automatic differentiation (torch, fp64) of an independent implementation: the recurrence unrolled as a
    per-channel mask, o_i = q_scale sum_{j<=i} (sum_c q_i[c] k_j[c] D[i][j][c]) v_j, with D from cumulative
    log-decays that skip the boundary positions; the key either given or 1 - lambda."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(100 + 2 * mode + own_key)
    B, Hh, H, W, d, start = 1, 2, 3, 4, 3, 2
    n = H * W - start
    q, v, g = (rng.standard_normal((B, n, Hh, d)) for _ in range(3))
    lam = rng.uniform(0.3, 0.99, size=(B, n, Hh, d))
    k = rng.uniform(0.0, 1.0, size=(B, n, Hh, d)) if own_key else None
    tq, tl, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, lam, v))
    tk = torch.tensor(k, dtype=torch.float64, requires_grad=True) if own_key else None
    key = tk if own_key else 1.0 - tl
    pos = start + np.arange(1, n + 1)
    boundary = (pos % W == 0) if mode == 0 else ((pos - 1) % W == 0) if mode == 1 else np.zeros(n, dtype=bool)
    keep = torch.tensor(~boundary, dtype=torch.float64)[None, :, None, None]
    cl = torch.cumsum(torch.log(tl) * keep, dim=1)
    D = torch.exp(cl[:, :, None] - cl[:, None, :])
    causal = torch.tril(torch.ones(n, n, dtype=torch.float64))[None, :, :, None]
    scores = torch.einsum("bihc,bjhc,bijhc->bijh", tq, key, D) * causal * 0.6
    o = torch.einsum("bijh,bjhe->bihe", scores, tv)
    (o * torch.tensor(g)).sum().backward()
    res = oracle.gated_backward(q, lam, v, g, W, k=k, start_pos=start, mode=mode, q_scale=0.6)
    want = [tq.grad, tl.grad, tv.grad] + ([tk.grad] if own_key else [])
    # the first token's decay multiplies the zero state: the oracle returns 0 there by definition, and so does autograd
    for got, w in zip(res, want):
        assert np.allclose(got, w.numpy(), rtol=1e-9, atol=1e-11)
