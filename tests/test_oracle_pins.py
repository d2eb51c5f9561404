"""Pins of the CPU oracle against what the paper's equations and plain mathematics fix.

Nothing here touches the GPU or the HIP library.  Each test is chosen so that a
plausible mistake in the oracle (a dropped term, a wrong boundary index, a
transposed operand or state, o_t read from s_{t-1}) fails at least one of them.
"""
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
MODES = {"last_col": 0, "first_col": 1, "none": 2}


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- decay table

@pytest.mark.parametrize("rule", ["last_col", "first_col", "none"])
def test_decay_table_hand_example(oracle, rule):
    g = json.load(open(os.path.join(GOLDEN, "sad_scalar_2x3.json")))
    lam, cum = oracle.decay_factors([g["gamma"]], g["grid_h"], g["grid_w"], 0, 6, MODES[rule])
    assert lam.dtype == np.float32 and cum.dtype == np.int32
    assert lam[0].tolist() == g[rule]["lambda"]
    assert cum.tolist() == g[rule]["cum_exp"]


def test_decay_table_copies_gamma_bits_and_offsets(oracle):
    gam = np.array([0.85, 0.999, 0.123456789], dtype=np.float32)
    H, W = 5, 7
    lam_full, cum_full = oracle.decay_factors(gam, H, W, 0, H * W)
    # closed form of the paper's rule in 0-indexed (row, col): lambda = 1 exactly at col == W-1
    for h in range(3):
        for i in range(H * W):
            want = np.float32(1.0) if (i % W) == W - 1 else gam[h]
            assert lam_full[h, i].tobytes() == want.tobytes()
    t = np.arange(H * W + 1)
    assert np.array_equal(cum_full, t - t // W)          # E(t) = t - floor(t / W)
    # a window that starts mid-row reproduces the matching slice
    lam_win, cum_win = oracle.decay_factors(gam, H, W, 10, 13)
    assert np.array_equal(lam_win, lam_full[:, 10:23])
    assert np.array_equal(cum_win, cum_full[10:24])
    # first-column rule: lambda = 1 at col == 0; E(t) = t - ceil(t / W)
    lam_f, cum_f = oracle.decay_factors(gam, H, W, 0, H * W, 1)
    assert np.array_equal(lam_f[0] == 1.0, (np.arange(H * W) % W) == 0)
    assert np.array_equal(cum_f, t - (t + W - 1) // W)
    with pytest.raises(ValueError):
        oracle.decay_factors(gam, H, W, 30, 6)            # runs past the grid


def test_mask_exponents_row_col_form(oracle):
    """prod lambda over (j, i] equals gamma^(raster steps minus one free step per row end crossed)."""
    g = json.load(open(os.path.join(GOLDEN, "sad_scalar_2x3.json")))
    _, cum = oracle.decay_factors([0.5], 2, 3, 0, 6)
    for i in range(1, 7):
        assert [int(cum[i] - cum[j]) for j in range(1, i + 1)] == g["last_col"]["mask_exponents"][i - 1]
    for H, W in [(4, 1), (4, 2), (3, 5), (2, 16), (3, 24)]:
        _, cum = oracle.decay_factors([0.5], H, W, 0, H * W)
        for i in range(1, H * W + 1):
            ri, ci = divmod(i - 1, W)
            for j in range(1, i + 1):
                rj, cj = divmod(j - 1, W)
                want = (ri - rj) * (W - 1) + (ci - cj) - (ci == W - 1) + (cj == W - 1)
                assert cum[i] - cum[j] == want


# ---------------------------------------------------------------- hand-worked recurrences

@pytest.mark.parametrize("rule", ["last_col", "first_col", "none"])
@pytest.mark.parametrize("form", ["forward_fullmask", "recurrent", "bruteforce"])
def test_scalar_worked_example(oracle, rule, form):
    g = json.load(open(os.path.join(GOLDEN, "sad_scalar_2x3.json")))
    lam, _ = oracle.decay_factors([g["gamma"]], 2, 3, 0, 6, MODES[rule])
    ones = np.ones((1, 6, 1, 1))
    if form == "bruteforce":
        o = oracle.bruteforce(ones[0, :, 0], ones[0, :, 0], ones[0, :, 0], lam[0])
    else:
        o = getattr(oracle, form)(ones, ones, ones, lam)
    assert o.ravel().tolist() == g[rule]["o"]


@pytest.mark.parametrize("form", ["forward_fullmask", "recurrent", "bruteforce"])
def test_vector_worked_example(oracle, form):
    g = json.load(open(os.path.join(GOLDEN, "sad_vector_2x2.json")))
    q, k, v = (np.array(g[x], dtype=np.float64) for x in "qkv")
    lam, _ = oracle.decay_factors([g["gamma"]], 2, 2, 0, 4)
    if form == "bruteforce":
        o = oracle.bruteforce(q, k, v, lam[0])
    else:
        o, s = getattr(oracle, form)(q[None, :, None, :], k[None, :, None, :], v[None, :, None, :],
                                     lam, want_state=True)
        assert s[0, 0].tolist() == g["final_state"]      # rows = key channel, cols = value channel
        o = o[0, :, 0, :]
    assert o.tolist() == g["o"]


# ---------------------------------------------------------------- closed forms and library reductions

def test_geometric_series_closed_form(oracle):
    """No boundary, q = k = v = 1, d = 1: o_t = sum_{m<t} gamma^m = (1 - gamma^t) / (1 - gamma)."""
    gam, n = 0.9, 40
    lam, _ = oracle.decay_factors([gam], 1, n, 0, n, 2)
    ones = np.ones((1, n, 1, 1))
    want = (1 - np.float64(np.float32(gam)) ** np.arange(1, n + 1)) / (1 - np.float64(np.float32(gam)))
    for form in ("forward_fullmask", "recurrent"):
        got = getattr(oracle, form)(ones, ones, ones, lam).ravel()
        np.testing.assert_allclose(got, want, rtol=1e-13)


def test_rows_closed_form(oracle):
    """Paper's rule, q = k = v = 1, d = 1, t = r W + c + 1: within a row the state follows
    s = gamma s + 1 for c < W-1 and s = s + 1 at c = W-1."""
    gam, H, W = 0.75, 3, 4
    lam, _ = oracle.decay_factors([gam], H, W, 0, H * W)
    ones = np.ones((1, H * W, 1, 1))
    s, want = 0.0, []
    for r in range(H):
        for c in range(W):
            s = (gam * s if c < W - 1 else s) + 1.0
            want.append(s)
    got = oracle.forward_fullmask(ones, ones, ones, lam).ravel()
    np.testing.assert_allclose(got, want, rtol=1e-14)


@pytest.mark.parametrize("case", ["gamma_one", "width_one"])
def test_reduces_to_plain_causal_linear_attention(oracle, case):
    """gamma = 1 (or W = 1: every position is a boundary) gives Section 3.2's recurrence,
    i.e. O = tril(Q K^T) V and final state K^T V -- library matmuls."""
    B, n, Hh, d = 2, 12, 3, 5
    q, k, v = _rand((B, n, Hh, d), 1), _rand((B, n, Hh, d), 2), _rand((B, n, Hh, d), 3)
    if case == "gamma_one":
        lam, _ = oracle.decay_factors([1.0] * Hh, 3, 4, 0, n)
    else:
        lam, _ = oracle.decay_factors([0.3, 0.6, 0.9], n, 1, 0, n)
    assert np.all(lam == 1.0)
    for form in ("forward_fullmask", "recurrent"):
        o, s = getattr(oracle, form)(q, k, v, lam, want_state=True)
        for b in range(B):
            for h in range(Hh):
                Q, K, V = q[b, :, h], k[b, :, h], v[b, :, h]
                np.testing.assert_allclose(o[b, :, h], np.tril(Q @ K.T) @ V, rtol=1e-12, atol=1e-12)
                np.testing.assert_allclose(s[b, h], K.T @ V, rtol=1e-12, atol=1e-12)


def test_constant_decay_is_toeplitz_mask(oracle):
    """No boundary: M[i, j] = gamma^(i-j) (Section 3.3 constant decay), a Toeplitz matrix."""
    from scipy.linalg import toeplitz
    n, d = 17, 4
    gam = np.array([0.8, 0.95], dtype=np.float32)
    q, k, v = _rand((1, n, 2, d), 4), _rand((1, n, 2, d), 5), _rand((1, n, 2, d), 6)
    lam, _ = oracle.decay_factors(gam, 1, n, 0, n, 2)
    o = oracle.forward_fullmask(q, k, v, lam)
    for h in range(2):
        T = np.tril(toeplitz(np.float64(gam[h]) ** np.arange(n)))
        np.testing.assert_allclose(o[0, :, h], ((q[0, :, h] @ k[0, :, h].T) * T) @ v[0, :, h],
                                   rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- cross-form agreement and invariants

@pytest.mark.parametrize("H,W", [(1, 9), (3, 3), (5, 7), (8, 8), (4, 1)])
@pytest.mark.parametrize("rule", [0, 1, 2])
def test_three_forms_agree(oracle, H, W, rule):
    n, d, Hh, B = H * W, 6, 2, 2
    q, k, v = _rand((B, n, Hh, d), 7), _rand((B, n, Hh, d), 8), _rand((B, n, Hh, d), 9)
    lam, _ = oracle.decay_factors([0.6, 0.93], H, W, 0, n, rule)
    o_full, s_full = oracle.forward_fullmask(q, k, v, lam, q_scale=0.7, want_state=True)
    o_rec, s_rec = oracle.recurrent(q, k, v, lam, q_scale=0.7, want_state=True)
    np.testing.assert_allclose(o_full, o_rec, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(s_full, s_rec, rtol=1e-12, atol=1e-13)
    for b in range(B):
        for h in range(Hh):
            o_bf = oracle.bruteforce(q[b, :, h], k[b, :, h], v[b, :, h], lam[h], q_scale=0.7)
            np.testing.assert_allclose(o_full[b, :, h], o_bf, rtol=1e-12, atol=1e-13)


def test_gamma_zero(oracle):
    """gamma = 0: only tokens reachable through boundary steps survive (0^0 = 1 on the diagonal)."""
    H, W, d = 2, 3, 3
    q, k, v = _rand((1, 6, 1, d), 10), _rand((1, 6, 1, d), 11), _rand((1, 6, 1, d), 12)
    lam, _ = oracle.decay_factors([0.0], H, W, 0, 6)
    o = oracle.forward_fullmask(q, k, v, lam)[0, :, 0]
    Q, K, V = q[0, :, 0], k[0, :, 0], v[0, :, 0]
    # lambda = [0, 0, 1, 0, 0, 1]: token 3 (1-indexed) also sees token 2; token 6 also sees token 5
    np.testing.assert_allclose(o[0], (Q[0] @ K[0]) * V[0], rtol=1e-13)
    np.testing.assert_allclose(o[2], (Q[2] @ K[2]) * V[2] + (Q[2] @ K[1]) * V[1], rtol=1e-13)
    np.testing.assert_allclose(o[3], (Q[3] @ K[3]) * V[3], rtol=1e-13)
    np.testing.assert_allclose(o[5], (Q[5] @ K[5]) * V[5] + (Q[5] @ K[4]) * V[4], rtol=1e-13)
    np.testing.assert_allclose(oracle.recurrent(q, k, v, lam)[0, :, 0], o, rtol=1e-13, atol=1e-15)


def test_causality(oracle):
    """o_i depends only on tokens at or before i in raster order."""
    H, W, d = 4, 5, 4
    n = H * W
    q, k, v = _rand((1, n, 1, d), 13), _rand((1, n, 1, d), 14), _rand((1, n, 1, d), 15)
    lam, _ = oracle.decay_factors([0.9], H, W, 0, n)
    base = oracle.forward_fullmask(q, k, v, lam)
    j = 11
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[0, j:], k2[0, j:], v2[0, j:] = 3.0, -2.0, 5.0
    pert = oracle.forward_fullmask(q2, k2, v2, lam)
    assert np.array_equal(base[0, :j], pert[0, :j])
    assert not np.allclose(base[0, j:], pert[0, j:])


def test_linearity_in_v_and_q(oracle):
    H, W, d = 3, 4, 5
    n = H * W
    q, k, v = _rand((1, n, 2, d), 16), _rand((1, n, 2, d), 17), _rand((1, n, 2, d), 18)
    v2, q2 = _rand((1, n, 2, d), 19), _rand((1, n, 2, d), 20)
    lam, _ = oracle.decay_factors([0.7, 0.95], H, W, 0, n)
    f = lambda a, c: oracle.forward_fullmask(a, k, c, lam)
    np.testing.assert_allclose(f(q, 2 * v - 3 * v2), 2 * f(q, v) - 3 * f(q, v2), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(f(q + q2, v), f(q, v) + f(q2, v), rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("split", [1, 7, 10, 19])
def test_split_with_carried_state_equals_single_call(oracle, split):
    """Running tokens 1..p, then p+1..n from the carried state, equals one call (also mid-row)."""
    H, W, d = 4, 5, 4
    n = H * W
    q, k, v = _rand((2, n, 2, d), 21), _rand((2, n, 2, d), 22), _rand((2, n, 2, d), 23)
    gam = [0.8, 0.97]
    lam, _ = oracle.decay_factors(gam, H, W, 0, n)
    o_all, s_all = oracle.forward_fullmask(q, k, v, lam, want_state=True)
    lam1, _ = oracle.decay_factors(gam, H, W, 0, split)
    lam2, _ = oracle.decay_factors(gam, H, W, split, n - split)
    for form in ("forward_fullmask", "recurrent"):
        f = getattr(oracle, form)
        o1, s1 = f(q[:, :split], k[:, :split], v[:, :split], lam1, want_state=True)
        o2, s2 = f(q[:, split:], k[:, split:], v[:, split:], lam2, s0=s1, want_state=True)
        np.testing.assert_allclose(np.concatenate([o1, o2], axis=1), o_all, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(s2, s_all, rtol=1e-12, atol=1e-13)


def test_decode_steps_equal_forward(oracle):
    """Stepping the one-token update over the grid reproduces the parallel form and its final state."""
    H, W, d, B, Hh = 3, 4, 5, 2, 2
    n = H * W
    q, k, v = _rand((B, n, Hh, d), 24), _rand((B, n, Hh, d), 25), _rand((B, n, Hh, d), 26)
    gam = [0.85, 0.99]
    lam, _ = oracle.decay_factors(gam, H, W, 0, n)
    o_all, s_all = oracle.forward_fullmask(q, k, v, lam, q_scale=1.3, want_state=True)
    state = np.zeros((B, Hh, d, d))
    for t in range(n):
        lam_t, _ = oracle.decay_factors(gam, H, W, t, 1)
        o_t = oracle.decode_step(q[:, t], k[:, t], v[:, t], lam_t[:, 0], state, q_scale=1.3)
        np.testing.assert_allclose(o_t, o_all[:, t], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(state, s_all, rtol=1e-12, atol=1e-13)


def test_empty_sequence(oracle):
    d = 3
    z = np.zeros((1, 0, 1, d))
    s0 = _rand((1, 1, d, d), 27)
    lam = np.zeros((1, 0))
    for form in ("forward_fullmask", "recurrent"):
        o, s = getattr(oracle, form)(z, z, z, lam, s0=s0, want_state=True)
        assert o.shape == (1, 0, 1, d)
        assert np.array_equal(s, s0)
