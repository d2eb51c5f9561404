"""Pins of the vector-decay (data-dependent, key tied to the decay) oracle: the recurrence of
Section 3.4 / Algorithm 1 as the paper writes it.  CPU only."""
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


@pytest.mark.parametrize("form", ["recurrent", "bruteforce"])
def test_gated_hand_example(oracle, form):
    g = json.load(open(os.path.join(GOLDEN, "sad_gated_2x2.json")))
    q, lam, v = (np.array(g[x], dtype=np.float64) for x in ("q", "lambda", "v"))
    if form == "bruteforce":
        o = oracle.gated_bruteforce(q, lam, v, g["grid_w"])
    else:
        o, s = oracle.gated_recurrent(q[None, :, None], lam[None, :, None], v[None, :, None], g["grid_w"],
                                      want_state=True)
        assert s[0, 0].tolist() == g["final_state"]
        o = o[0, :, 0]
    assert o.tolist() == g["o"]


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("tied", [True, False])
def test_gated_forms_agree(oracle, mode, tied):
    H, W, d, B, Hh = 3, 4, 5, 2, 2
    n = H * W
    rng = np.random.default_rng(40 + mode)
    q, v = _rand((B, n, Hh, d), 1), _rand((B, n, Hh, d), 2)
    lam = rng.uniform(0.2, 1.0, size=(B, n, Hh, d))
    k = None if tied else _rand((B, n, Hh, d), 3)
    o = oracle.gated_recurrent(q, lam, v, W, k=k, mode=mode, q_scale=0.7)
    for b in range(B):
        for h in range(Hh):
            ob = oracle.gated_bruteforce(q[b, :, h], lam[b, :, h], v[b, :, h], W,
                                         k=None if tied else k[b, :, h], mode=mode, q_scale=0.7)
            np.testing.assert_allclose(o[b, :, h], ob, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_gated_reduces_to_scalar_decay(oracle, mode):
    """A decay vector equal to gamma_h on every channel, with an independent key, is the scalar
    per-head decay path (its full-mask oracle)."""
    H, W, d, B, Hh = 4, 5, 6, 1, 2
    n = H * W
    q, k, v = _rand((B, n, Hh, d), 4), _rand((B, n, Hh, d), 5), _rand((B, n, Hh, d), 6)
    gam = np.array([0.8, 0.95], dtype=np.float32)
    lam_vec = np.broadcast_to(gam.astype(np.float64)[None, None, :, None], (B, n, Hh, d)).copy()
    got, s_got = oracle.gated_recurrent(q, lam_vec, v, W, k=k, mode=mode, want_state=True)
    lam_tab, _ = oracle.decay_factors(gam, H, W, 0, n, mode)
    ref, s_ref = oracle.forward_fullmask(q, k, v, lam_tab, want_state=True)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(s_got, s_ref, rtol=1e-12, atol=1e-13)


def test_gated_lambda_one_is_plain_linear_attention(oracle):
    """lambda = 1 on every channel with an independent key: Section 3.2, O = tril(Q K^T) V."""
    n, d = 11, 4
    q, k, v = _rand((1, n, 1, d), 7), _rand((1, n, 1, d), 8), _rand((1, n, 1, d), 9)
    o, s = oracle.gated_recurrent(q, np.ones((1, n, 1, d)), v, 3, k=k, want_state=True)
    Q, K, V = q[0, :, 0], k[0, :, 0], v[0, :, 0]
    np.testing.assert_allclose(o[0, :, 0], np.tril(Q @ K.T) @ V, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(s[0, 0], K.T @ V, rtol=1e-12, atol=1e-12)


def test_gated_tied_key_uses_base_decay_at_boundary(oracle):
    """At a boundary the decay is 1 but the key stays 1 - lambda (base), not 1 - 1 = 0."""
    d = 2
    lam = np.full((1, 2, 1, d), 0.25)
    q = np.ones((1, 2, 1, d)); v = np.ones((1, 2, 1, d))
    o = oracle.gated_recurrent(q, lam, v, 2)       # w = 2: t = 2 is a boundary
    # s_1 = 0.75 * 1 per row; s_2 = 1 * s_1 + 0.75 -> rows 1.5; o = sum over 2 rows
    assert o[0, :, 0, 0].tolist() == [1.5, 3.0]


@pytest.mark.parametrize("split", [1, 5, 8])
def test_gated_split_with_carried_state(oracle, split):
    H, W, d = 3, 4, 3
    n = H * W
    rng = np.random.default_rng(50)
    q, v = _rand((2, n, 2, d), 10), _rand((2, n, 2, d), 11)
    lam = rng.uniform(0.1, 1.0, size=(2, n, 2, d))
    o_all, s_all = oracle.gated_recurrent(q, lam, v, W, want_state=True)
    o1, s1 = oracle.gated_recurrent(q[:, :split], lam[:, :split], v[:, :split], W, want_state=True)
    o2, s2 = oracle.gated_recurrent(q[:, split:], lam[:, split:], v[:, split:], W, start_pos=split, s0=s1,
                                    want_state=True)
    np.testing.assert_allclose(np.concatenate([o1, o2], axis=1), o_all, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(s2, s_all, rtol=1e-12, atol=1e-13)
