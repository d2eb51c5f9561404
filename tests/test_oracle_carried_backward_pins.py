"""Pins of the oracle's gradients THROUGH A CARRIED STATE (the Section 3.4 recurrence differentiated with
s_0 given and a loss that also depends on the final state): a hand-differentiated example, central finite
differences of the oracle's forward functions (which are pinned on their own), automatic differentiation of an
independent mask form, the reduction to the zero-state routines, and the chain of two calls over a split
sequence against one call over the whole."""
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _loss_scalar(oracle, q, k, v, lam, s0, g, h, q_scale):
    o, sn = oracle.recurrent(q, k, v, lam, q_scale=q_scale, s0=s0, want_state=True)
    return float((o * g).sum() + (sn * h).sum())


def _num_grad(f, x, eps):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps
        fp = f()
        x[i] = old - eps
        fm = f()
        x[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


def test_hand_worked_two_tokens_with_carried_state(oracle):
    j = json.load(open(os.path.join(HERE, "golden", "sad_backward_carried_2tok.json")))
    col = lambda x: np.array(x, dtype=np.float64).reshape(1, 2, 1, 1)
    dq, dk, dv, dlam, d_s0 = oracle.backward_carried(col(j["q"]), col(j["k"]), col(j["v"]), np.array([j["lam"]]), col(j["d_o"]),
                                                     s0=np.full((1, 1, 1, 1), j["s0"]), d_state=np.full((1, 1, 1, 1), j["d_state"]))
    assert dq.ravel().tolist() == j["dq"] and dk.ravel().tolist() == j["dk"] and dv.ravel().tolist() == j["dv"]
    assert dlam.ravel().tolist() == j["dlam"] and d_s0.ravel().tolist() == [j["d_s0"]]


@pytest.mark.parametrize("seed,n,d", [(1, 5, 3), (2, 1, 2), (3, 7, 4)])
def test_scalar_carried_against_finite_differences_of_the_forward(oracle, seed, n, d):
    rng = np.random.default_rng(seed)
    B, Hh = 2, 2
    q, k, v, g = (rng.standard_normal((B, n, Hh, d)) for _ in range(4))
    lam = rng.uniform(0.3, 1.0, size=(Hh, n))
    s0, h = rng.standard_normal((B, Hh, d, d)), rng.standard_normal((B, Hh, d, d))
    dq, dk, dv, dlam, d_s0 = oracle.backward_carried(q, k, v, lam, g, s0=s0, d_state=h, q_scale=0.7)
    f = lambda: _loss_scalar(oracle, q, k, v, lam, s0, g, h, 0.7)
    for got, x in ((dq, q), (dk, k), (dv, v), (d_s0, s0)):          # the loss is linear in each: central differences are exact
        assert np.allclose(got, _num_grad(f, x, 1e-3), rtol=1e-7, atol=1e-8)
    # every lambda_t of head hh is shared by the batch rows: the finite difference sees the sum over b
    assert np.allclose(dlam.sum(axis=0), _num_grad(f, lam, 1e-5), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("own_key", [False, True])
@pytest.mark.parametrize("mode,start", [(0, 0), (0, 4), (1, 2), (2, 0)])
def test_gated_carried_against_finite_differences_of_the_forward(oracle, own_key, mode, start):
    rng = np.random.default_rng(10 + mode + start)
    B, Hh, n, d, W = 1, 2, 6, 3, 3
    q, v, g = (rng.standard_normal((B, n, Hh, d)) for _ in range(3))
    lam = rng.uniform(0.3, 0.95, size=(B, n, Hh, d))
    k = rng.standard_normal((B, n, Hh, d)) if own_key else None
    s0, h = rng.standard_normal((B, Hh, d, d)), rng.standard_normal((B, Hh, d, d))
    res = oracle.gated_backward_carried(q, lam, v, g, W, k=k, s0=s0, d_state=h, start_pos=start, mode=mode, q_scale=1.3)

    def f():
        o, sn = oracle.gated_recurrent(q, lam, v, W, k=k, start_pos=start, mode=mode, q_scale=1.3, s0=s0, want_state=True)
        return float((o * g).sum() + (sn * h).sum())

    pairs = [(res[0], q), (res[1], lam), (res[2], v), (res[-1], s0)] + ([(res[3], k)] if own_key else [])
    for got, x in pairs:
        assert np.allclose(got, _num_grad(f, x, 1e-5), rtol=2e-6, atol=1e-7)


def test_zero_states_reduce_to_the_zero_state_routines(oracle):
    rng = np.random.default_rng(5)
    B, n, Hh, d, W = 2, 7, 2, 4, 3
    q, k, v, g = (rng.standard_normal((B, n, Hh, d)) for _ in range(4))
    lam, _ = oracle.decay_factors(np.array([0.8, 0.6], dtype=np.float32), 3, W, 1, n)
    zero = np.zeros((B, Hh, d, d))
    for a, b in zip(oracle.backward(q, k, v, lam, g), oracle.backward_carried(q, k, v, lam, g, s0=zero, d_state=zero)):
        assert np.array_equal(a, b)
    gate = rng.uniform(0.3, 0.95, size=q.shape)
    for a, b in zip(oracle.gated_backward(q, gate, v, g, W), oracle.gated_backward_carried(q, gate, v, g, W, s0=zero, d_state=zero)):
        assert np.array_equal(a, b)


def test_scalar_and_vector_routines_agree_when_every_channel_carries_the_same_decay(oracle):
    rng = np.random.default_rng(6)
    B, n, Hh, d, W = 1, 6, 2, 3, 3
    q, k, v, g = (rng.standard_normal((B, n, Hh, d)) for _ in range(4))
    gam = np.array([0.8, 0.6], dtype=np.float32)
    lam, _ = oracle.decay_factors(gam, 2, W, 0, n)
    s0, h = rng.standard_normal((B, Hh, d, d)), rng.standard_normal((B, Hh, d, d))
    dq, dk, dv, dlam, d_s0 = oracle.backward_carried(q, k, v, lam, g, s0=s0, d_state=h)
    gate = np.broadcast_to(gam.astype(np.float64)[None, None, :, None], q.shape).copy()
    gq, gl, gv, gk, g_s0 = oracle.gated_backward_carried(q, gate, v, g, W, k=k, s0=s0, d_state=h)
    for a, b in ((dq, gq), (dk, gk), (dv, gv), (d_s0, g_s0)):
        assert np.allclose(a, b, rtol=1e-12, atol=1e-12)
    # the scalar decay's gradient per token is the sum of the channel gradients (0 at boundary positions on both sides
    # after the boundary mask that dgamma applies)
    per_tok = gl.sum(axis=3).transpose(0, 2, 1)                    # [B, Hh, n]
    assert np.allclose(oracle.dgamma(dlam, W), oracle.dgamma(per_tok, W), rtol=1e-12)


@pytest.mark.parametrize("split", [1, 4, 6])
def test_two_chained_calls_equal_one_call(oracle, split):
    """A sequence cut in two: the second call starts from the first call's final state and hands its d_s0 back as the
    first call's dL/ds_n.  Gradients of both calls together = gradients of the single call over the whole sequence."""
    rng = np.random.default_rng(7)
    B, n, Hh, d, W = 2, 7, 2, 3, 3
    q, k, v, g = (rng.standard_normal((B, n, Hh, d)) for _ in range(4))
    gam = np.array([0.9, 0.5], dtype=np.float32)
    lam, _ = oracle.decay_factors(gam, 3, W, 0, n)
    s0, h = rng.standard_normal((B, Hh, d, d)), rng.standard_normal((B, Hh, d, d))
    whole = oracle.backward_carried(q, k, v, lam, g, s0=s0, d_state=h)
    a, b = slice(0, split), slice(split, n)
    _, s_mid = oracle.recurrent(q[:, a], k[:, a], v[:, a], lam[:, a], s0=s0, want_state=True)
    second = oracle.backward_carried(q[:, b], k[:, b], v[:, b], lam[:, b], g[:, b], s0=s_mid, d_state=h)
    first = oracle.backward_carried(q[:, a], k[:, a], v[:, a], lam[:, a], g[:, a], s0=s0, d_state=second[4])
    for i in range(3):
        assert np.allclose(np.concatenate([first[i], second[i]], axis=1), whole[i], rtol=1e-12, atol=1e-13)
    assert np.allclose(np.concatenate([first[3], second[3]], axis=2), whole[3], rtol=1e-12, atol=1e-13)
    assert np.allclose(first[4], whole[4], rtol=1e-12, atol=1e-13)
    # the vector-decay routine chains the same way
    gate = rng.uniform(0.3, 0.95, size=q.shape)
    gw = oracle.gated_backward_carried(q, gate, v, g, W, s0=s0, d_state=h)
    _, g_mid = oracle.gated_recurrent(q[:, a], gate[:, a], v[:, a], W, s0=s0, want_state=True)
    g2 = oracle.gated_backward_carried(q[:, b], gate[:, b], v[:, b], g[:, b], W, s0=g_mid, d_state=h, start_pos=split)
    g1 = oracle.gated_backward_carried(q[:, a], gate[:, a], v[:, a], g[:, a], W, s0=s0, d_state=g2[3])
    for i in range(3):
        assert np.allclose(np.concatenate([g1[i], g2[i]], axis=1), gw[i], rtol=1e-12, atol=1e-13)
    assert np.allclose(g1[3], gw[3], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("mode", [0, 1])
def test_scalar_carried_against_torch_autograd_of_a_mask_form(oracle, mode):
    """Automatic differentiation (torch, fp64) of an independent closed form: with c_i the cumulative log-decay,
    o_i = q_scale [ sum_{j<=i} exp(c_i - c_j) (q_i . k_j) v_j + exp(c_i) s_0^T q_i ],
    s_n = exp(c_n) s_0 + sum_j exp(c_n - c_j) k_j v_j^T."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(30 + mode)
    B, n, Hh, d, H, W = 2, 8, 2, 3, 3, 3
    q, k, v, g = (rng.standard_normal((B, n, Hh, d)) for _ in range(4))
    gam = np.array([0.85, 0.55], dtype=np.float32)
    lam, _ = oracle.decay_factors(gam, H, W, 1, n, mode)
    s0, h = rng.standard_normal((B, Hh, d, d)), rng.standard_normal((B, Hh, d, d))
    got = oracle.backward_carried(q, k, v, lam, g, s0=s0, d_state=h, q_scale=0.9)
    tq, tk, tv, ts0 = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v, s0))
    tl = torch.tensor(lam, dtype=torch.float64, requires_grad=True)          # [Hh, n]
    c = torch.cumsum(torch.log(tl), dim=1)                                    # [Hh, n]
    mask = torch.tril(torch.ones(n, n, dtype=torch.float64))
    M = torch.exp(c[:, :, None] - c[:, None, :]) * mask                       # [Hh, i, j]
    A = torch.einsum("bihd,bjhd->bhij", tq, tk)
    o = torch.einsum("bhij,bjhe->bihe", A * M[None], tv) + torch.einsum("hi,bihd,bhde->bihe", torch.exp(c), tq, ts0)
    sn = torch.exp(c[:, -1])[None, :, None, None] * ts0 + torch.einsum("hj,bjhd,bjhe->bhde", torch.exp(c[:, -1:] - c), tk, tv)
    loss = 0.9 * (o * torch.tensor(g)).sum() + (sn * torch.tensor(h)).sum()
    loss.backward()
    for a, b in ((got[0], tq.grad), (got[1], tk.grad), (got[2], tv.grad), (got[4], ts0.grad)):
        assert np.allclose(a, b.numpy(), rtol=1e-10, atol=1e-11)
    assert np.allclose(got[3].sum(axis=0), tl.grad.numpy(), rtol=1e-10, atol=1e-11)
