"""Tensors of more than 2^31 elements (the sizes 288 GB of device memory invite): the addressing of the forward,
backward (scalar and vector decay, fused layer), decode and cached-decode kernels must be 64-bit.  Inputs are drawn on the GPU
from seeded generators (the host never holds a whole tensor); the oracle recomputes sampled (batch, head)
sequences in full: the first, the last, the two on either side of element offset 2^31, and some in between.  Same
tolerances as everywhere; the bf16 output of a sampled sequence must be the rounding of its fp32 output."""
import numpy as np
import pytest

from helpers import TOL, assert_rne_bf16, rel_err

pytestmark = pytest.mark.gpu

D = 64


@pytest.fixture(scope="module")
def lasad():
    import torch
    assert torch.cuda.is_available()
    from paper_2507_01652_amd import binding
    binding.load()
    return binding


def _normal(shape, seed, scale=1.0, mean=0.0, dtype=None):
    """N(mean, 1) * scale in the given dtype, filled slab by slab along the first axis."""
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    x = torch.empty(shape, dtype=dtype or torch.bfloat16, device="cuda")
    step = max(1, (1 << 28) // max(1, x[0].numel()))
    for b0 in range(0, shape[0], step):
        x[b0:b0 + step].normal_(mean, 1.0, generator=gen)
    if scale != 1.0:
        x.mul_(scale)
    return x


def _pairs(B, Hh, per_pair_elements):
    """First, last, both sides of element offset 2^31, two more."""
    cut = (1 << 31) // per_pair_elements          # first (b, h) index whose elements start at or beyond 2^31
    assert 0 < cut < B * Hh, "the tensor must cross 2^31 elements"
    idx = sorted({0, cut - 1, cut, B * Hh - 1, (cut // 2) | 1, (cut + B * Hh) // 2})
    return [(i // Hh, i % Hh) for i in idx]


def _seqs(x, pairs):
    """[B, n, Hh, d] device tensor -> [1, n, P, d] float32 numpy of the sampled sequences."""
    import torch
    return torch.stack([x[b, :, h, :] for b, h in pairs], dim=1)[None].float().cpu().numpy()


def _rows(x, pairs):
    """[B, Hh, ...] device tensor -> [P, 1, ...] float32 numpy of the sampled rows (each its own batch entry)."""
    import torch
    return torch.stack([x[b, h] for b, h in pairs])[:, None].float().cpu().numpy()


B_SEQ, HH, GRID_H, GRID_W = 4300, 64, 8, 16          # 4300 x 128 x 64 x 64 = 2.25e9 elements
N = GRID_H * GRID_W


@pytest.fixture(scope="module")
def seq_inputs():
    import torch
    shape = (B_SEQ, N, HH, D)
    assert B_SEQ * N * HH * D > 1 << 31
    q, k, v, g = (_normal(shape, 100 + i, 0.125) for i in range(4))
    lam = _normal(shape, 104, mean=2.0).sigmoid_()
    gam = np.random.default_rng(5).uniform(0.85, 0.999, size=(HH,)).astype(np.float32)
    yield q, k, v, g, lam, gam
    del q, k, v, g, lam
    torch.cuda.empty_cache()


def test_forward_chunked_beyond_2g_elements(lasad, oracle, seq_inputs):
    import torch
    q, k, v, _, _, gam = seq_inputs
    cut_b = (1 << 31) // (N * HH * D)          # in [B, n, Hh, d] the first batch entry at or beyond element 2^31
    pairs = [(0, 0), (2000, 5), (cut_b - 1, HH - 1), (cut_b, 0), (cut_b, 17), (B_SEQ - 1, HH - 1)]
    tg = torch.from_numpy(gam).cuda()
    s1 = torch.empty((B_SEQ, HH, D, D), dtype=torch.float32, device="cuda")
    o32 = lasad.lasad_forward_chunked(q, k, v, tg, GRID_H, GRID_W, q_scale=0.5, state_out=s1, out_dtype=torch.float32)
    o16 = lasad.lasad_forward_chunked(q, k, v, tg, GRID_H, GRID_W, q_scale=0.5)
    torch.cuda.synchronize()
    lam, _ = oracle.decay_factors(gam[[h for _, h in pairs]], GRID_H, GRID_W, 0, N)
    ref, s_ref = oracle.recurrent(_seqs(q, pairs), _seqs(k, pairs), _seqs(v, pairs), lam, q_scale=0.5, want_state=True)
    assert rel_err(_seqs(o32, pairs), ref) <= TOL["bf16"]
    assert rel_err(np.stack([s1[b, h].cpu().numpy() for b, h in pairs])[None], s_ref) <= TOL["bf16"]
    for b, h in pairs:
        assert_rne_bf16(o16[b, :, h], o32[b, :, h], f"forward sequence ({b}, {h})")
    assert bool(torch.isfinite(o32[-1]).all())


def test_backward_chunked_beyond_2g_elements(lasad, oracle, seq_inputs):
    import torch
    q, k, v, g, _, gam = seq_inputs
    cut_b = (1 << 31) // (N * HH * D)
    pairs = [(0, 0), (cut_b - 1, HH - 1), (cut_b, 0), (cut_b, 17), (B_SEQ - 1, HH - 1)]
    tg = torch.from_numpy(gam).cuda()
    dq, dk, dv, dgam = lasad.lasad_backward_chunked(q, k, v, g, tg, GRID_H, GRID_W, q_scale=0.5, grad_dtype=torch.float32)
    torch.cuda.synchronize()
    lam, _ = oracle.decay_factors(gam[[h for _, h in pairs]], GRID_H, GRID_W, 0, N)
    rq, rk, rv, _ = oracle.backward(_seqs(q, pairs), _seqs(k, pairs), _seqs(v, pairs), lam, _seqs(g, pairs), q_scale=0.5)
    for nm, got, want in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        assert rel_err(_seqs(got, pairs), want) <= TOL["bf16"], nm
    assert bool(torch.isfinite(dgam).all())


def test_forward_and_backward_gated_beyond_2g_elements(lasad, oracle, seq_inputs):
    import torch
    q, _, v, g, lam, _ = seq_inputs
    cut_b = (1 << 31) // (N * HH * D)
    pairs = [(0, 0), (cut_b - 1, HH - 1), (cut_b, 0), (cut_b, 33), (B_SEQ - 1, HH - 1)]
    s1 = torch.empty((B_SEQ, HH, D, D), dtype=torch.float32, device="cuda")
    o = lasad.lasad_forward_gated(q, lam, v, GRID_H, GRID_W, q_scale=0.5, state_out=s1, out_dtype=torch.float32)
    torch.cuda.synchronize()
    ref, s_ref = oracle.gated_recurrent(_seqs(q, pairs), _seqs(lam, pairs), _seqs(v, pairs), GRID_W, q_scale=0.5, want_state=True)
    assert rel_err(_seqs(o, pairs), ref) <= TOL["bf16"]
    assert rel_err(np.stack([s1[b, h].cpu().numpy() for b, h in pairs])[None], s_ref) <= TOL["bf16"]
    del o, s1
    dq, dlam, dv = lasad.lasad_backward_gated(q, lam, v, g, GRID_H, GRID_W, q_scale=0.5, grad_dtype=torch.float32)[:3]
    torch.cuda.synchronize()
    want = oracle.gated_backward(_seqs(q, pairs), _seqs(lam, pairs), _seqs(v, pairs), _seqs(g, pairs), GRID_W, q_scale=0.5)
    for nm, got, r in zip(("dq", "dlam", "dv"), (dq, dlam, dv), want):
        assert rel_err(_seqs(got, pairs), r) <= TOL["bf16"], nm


def test_layer_forward_and_backward_beyond_2g_elements(lasad, oracle, seq_inputs):
    """Algorithm 1's fused layer (activations, tied key, recurrence, norm) and its backward at the same size."""
    import torch
    q, _, v, g, _, _ = seq_inputs
    z = _normal((B_SEQ, N, HH, D), 105, mean=2.0)
    cut_b = (1 << 31) // (N * HH * D)
    pairs = [(0, 0), (cut_b - 1, HH - 1), (cut_b, 0), (cut_b, 41), (B_SEQ - 1, HH - 1)]
    w = np.random.default_rng(8).uniform(0.5, 1.5, size=(HH, D)).astype(np.float32)
    wt, wp = torch.from_numpy(w).cuda(), w[[h for _, h in pairs]]
    o = lasad.lasad_forward_layer(q, z, v, GRID_H, GRID_W, norm_weight=wt, norm_eps=1e-5, q_scale=0.5, out_dtype=torch.float32)
    torch.cuda.synchronize()
    sq, sz, sv, sg = (_seqs(x, pairs) for x in (q, z, v, g))
    ref = oracle.gated_layer(sq, sz, sv, GRID_W, norm_weight=wp, eps=1e-5, q_scale=0.5)
    assert rel_err(_seqs(o, pairs), ref) <= TOL["bf16"]
    del o
    dq, dz, dv, dw = lasad.lasad_backward_layer(q, z, v, g, GRID_H, GRID_W, norm_weight=wt, norm_eps=1e-5, q_scale=0.5,
                                                grad_dtype=torch.float32)
    torch.cuda.synchronize()
    want = oracle.gated_layer_backward(sq, sz, sv, sg, GRID_W, norm_weight=wp, eps=1e-5, q_scale=0.5)
    for nm, got, r in zip(("dq_pre", "dz", "dv"), (dq, dz, dv), want):
        assert rel_err(_seqs(got, pairs), r) <= TOL["bf16"], (nm, rel_err(_seqs(got, pairs), r))
    assert bool(torch.isfinite(dw).all())


def test_decode_states_beyond_2g_elements(lasad, oracle):
    """State tensor of 8200 x 64 states (2.15e9 fp32 elements): scalar- and vector-decay steps."""
    import torch
    B, Hh, H, W, pos = 8200, 64, 16, 16, 37
    assert B * Hh * D * D > 1 << 31
    pairs = _pairs(B, Hh, D * D)
    q, k, v = (_normal((B, Hh, D), 200 + i, 0.125) for i in range(3))
    lam = _normal((B, Hh, D), 204, mean=2.0).sigmoid_()
    s0 = _normal((B, Hh, D, D), 205, 0.3, dtype=torch.float32)
    gam = np.random.default_rng(6).uniform(0.85, 0.999, size=(Hh,)).astype(np.float32)
    s0_rows = _rows(s0, pairs)                                           # [P, 1, d, d]
    sq, sk, sv, sl = (_rows(x, pairs)[:, :, None] for x in (q, k, v, lam))   # [P, 1 (token), 1 (head), d]
    st = s0.clone()
    o = lasad.lasad_decode_step(q, k, v, torch.from_numpy(gam).cuda(), st, H, W, pos, q_scale=0.5, out_dtype=torch.float32)
    torch.cuda.synchronize()
    for i, (b, h) in enumerate(pairs):
        lam1, _ = oracle.decay_factors(gam[[h]], H, W, pos, 1)
        ro, rs = oracle.recurrent(sq[i:i + 1], sk[i:i + 1], sv[i:i + 1], lam1, q_scale=0.5,
                                  s0=s0_rows[i:i + 1], want_state=True)
        assert rel_err(o[b, h].cpu().numpy(), ro[0, 0, 0]) <= TOL["bf16"], (b, h)
        assert rel_err(st[b, h].cpu().numpy(), rs[0, 0]) <= TOL["bf16"], (b, h)
    st.copy_(s0)
    o = lasad.lasad_decode_step_gated(q, lam, v, st, H, W, pos, q_scale=0.5, out_dtype=torch.float32)
    torch.cuda.synchronize()
    for i, (b, h) in enumerate(pairs):
        ro, rs = oracle.gated_recurrent(sq[i:i + 1], sl[i:i + 1], sv[i:i + 1], W, start_pos=pos, q_scale=0.5,
                                        s0=s0_rows[i:i + 1], want_state=True)
        assert rel_err(o[b, h].cpu().numpy(), ro[0, 0, 0]) <= TOL["bf16"], (b, h)
        assert rel_err(st[b, h].cpu().numpy(), rs[0, 0]) <= TOL["bf16"], (b, h)


def test_cached_decode_caches_beyond_2g_elements(lasad, oracle):
    """Key / value (/ gate) caches of 600 x 64 x 1024 x 64 = 2.5e9 elements, one step at position 1000."""
    import torch
    B, Hh, T, H, W, pos = 600, 64, 1024, 32, 32, 1000
    assert B * Hh * T * D > 1 << 31
    pairs = _pairs(B, Hh, T * D)
    q, k, v = (_normal((B, Hh, D), 300 + i, 0.125) for i in range(3))
    lam = _normal((B, Hh, D), 304, mean=2.0).sigmoid_()
    kc, vc = (_normal((B, Hh, T, D), 305 + i, 0.125) for i in range(2))
    gam = np.random.default_rng(7).uniform(0.85, 0.999, size=(Hh,)).astype(np.float32)

    def seq_of(cache, now):                   # [1, pos + 1, P, d]: the cached rows, then this step's row
        rows = [torch.cat([cache[b, h, :pos], now[b, h][None]]) for b, h in pairs]
        return torch.stack(rows, dim=1)[None].float().cpu().numpy()

    sq = np.zeros((1, pos + 1, len(pairs), D), dtype=np.float32)
    sq[0, pos] = np.stack([q[b, h].float().cpu().numpy() for b, h in pairs])
    sk, sv = seq_of(kc, k), seq_of(vc, v)
    o = lasad.lasad_decode_step_cached(q, k, v, torch.from_numpy(gam).cuda(), kc, vc, H, W, pos, q_scale=0.5,
                                       out_dtype=torch.float32)
    torch.cuda.synchronize()
    lam_t, _ = oracle.decay_factors(gam[[h for _, h in pairs]], H, W, 0, pos + 1)
    ref = oracle.recurrent(sq, sk, sv, lam_t, q_scale=0.5)[0, pos]
    got = np.stack([o[b, h].cpu().numpy() for b, h in pairs])
    assert rel_err(got, ref) <= TOL["bf16"]
    for b, h in pairs:
        assert torch.equal(kc[b, h, pos], k[b, h]) and torch.equal(vc[b, h, pos], v[b, h])
    # vector decay: the key cache now serves as the gate cache (values squashed into (0, 1))
    lc = kc.mul_(8.0).add_(2.0).sigmoid_()
    sl = seq_of(lc, lam)
    o = lasad.lasad_decode_step_gated_cached(q, lam, v, lc, vc, H, W, pos, q_scale=0.5, out_dtype=torch.float32)
    torch.cuda.synchronize()
    ref = oracle.gated_recurrent(sq, sl, sv, W, q_scale=0.5)[0, pos]
    got = np.stack([o[b, h].cpu().numpy() for b, h in pairs])
    assert rel_err(got, ref) <= TOL["bf16"]
    for b, h in pairs:
        assert torch.equal(lc[b, h, pos], lam[b, h])


def test_carried_backward_states_beyond_2g_elements(lasad, oracle):
    """Gradients through carried states with 8200 x 64 sequences of 8 tokens: the incoming state, the gradient of
    the final state and the gradient of the incoming state are 2.15e9 fp32 elements each."""
    import torch
    B, Hh, H, W = 8200, 64, 2, 4
    n = H * W
    assert B * Hh * D * D > 1 << 31
    pairs = _pairs(B, Hh, D * D)
    q, k, v, g = (_normal((B, n, Hh, D), 400 + i, 0.125) for i in range(4))
    lam = _normal((B, n, Hh, D), 404, mean=2.0).sigmoid_()
    s0 = _normal((B, Hh, D, D), 405, 0.3, dtype=torch.float32)
    h = _normal((B, Hh, D, D), 406, 0.1, dtype=torch.float32)
    gam = np.random.default_rng(9).uniform(0.85, 0.999, size=(Hh,)).astype(np.float32)
    sq, sk, sv, sg, sl = (_seqs(x, pairs) for x in (q, k, v, g, lam))
    sel = lambda x: np.stack([x[b, hh].cpu().numpy() for b, hh in pairs])[None]
    s0p, hp = sel(s0), sel(h)
    dq, dk, dv, dgam, ds0 = lasad.lasad_backward_chunked_carried(q, k, v, g, torch.from_numpy(gam).cuda(), H, W, state_in=s0,
                                                                 d_state_out=h, q_scale=0.5, grad_dtype=torch.float32)
    torch.cuda.synchronize()
    lam_t, _ = oracle.decay_factors(gam[[hh for _, hh in pairs]], H, W, 0, n)
    rq, rk, rv, _, rs0 = oracle.backward_carried(sq, sk, sv, lam_t, sg, s0=s0p, d_state=hp, q_scale=0.5)
    for nm, got, want in (("dq", _seqs(dq, pairs), rq), ("dk", _seqs(dk, pairs), rk), ("dv", _seqs(dv, pairs), rv),
                          ("d_state_in", sel(ds0), rs0)):
        assert rel_err(got, want) <= TOL["bf16"], nm
    assert bool(torch.isfinite(dgam).all())
    del dq, dk, dv, ds0
    dq, dlam, dv, ds0 = lasad.lasad_backward_gated_carried(q, lam, v, g, H, W, state_in=s0, d_state_out=h, q_scale=0.5,
                                                           grad_dtype=torch.float32)
    torch.cuda.synchronize()
    want = oracle.gated_backward_carried(sq, sl, sv, sg, W, s0=s0p, d_state=hp, q_scale=0.5)
    for nm, got, r in zip(("dq", "dlam", "dv", "d_state_in"), (_seqs(dq, pairs), _seqs(dlam, pairs), _seqs(dv, pairs), sel(ds0)), want):
        assert rel_err(got, r) <= TOL["bf16"], nm


@pytest.mark.parametrize("mode", [0, 2])
def test_forward_quarter_million_tokens_per_sequence(lasad, oracle, mode):
    """A 512 x 512 grid entered mid-row (262 000 tokens per sequence, 4096 chunks, the segment plan's long
    segments), decays close to one: scalar and vector decay against the oracle's recurrence, outputs and final
    states.  The call is also cut in two at an odd token and must give the same final state as the single call."""
    import torch
    H = W = 512
    start = 3 * W + 77
    n = H * W - start
    B, Hh = 1, 2
    q, k, v = (_normal((B, n, Hh, D), 500 + i, 0.125) for i in range(3))
    lam = _normal((B, n, Hh, D), 504, mean=3.0).sigmoid_()
    gam = np.array([0.9993, 0.99995], dtype=np.float32)
    tg = torch.from_numpy(gam).cuda()
    s1 = torch.empty((B, Hh, D, D), dtype=torch.float32, device="cuda")
    o = lasad.lasad_forward_chunked(q, k, v, tg, H, W, start_pos=start, boundary_mode=mode, state_out=s1, out_dtype=torch.float32)
    torch.cuda.synchronize()
    host = lambda x: x.float().cpu().numpy()
    lam_t, _ = oracle.decay_factors(gam, H, W, start, n, mode)
    ref, s_ref = oracle.recurrent(host(q), host(k), host(v), lam_t, want_state=True)
    assert rel_err(host(o), ref) <= TOL["bf16"]
    assert rel_err(host(s1), s_ref) <= TOL["bf16"]
    cut = 100001
    sa, sb = torch.empty_like(s1), torch.empty_like(s1)
    lasad.lasad_forward_chunked(q[:, :cut], k[:, :cut], v[:, :cut], tg, H, W, start_pos=start, boundary_mode=mode, state_out=sa)
    lasad.lasad_forward_chunked(q[:, cut:], k[:, cut:], v[:, cut:], tg, H, W, start_pos=start + cut, boundary_mode=mode,
                                state_in=sa, state_out=sb)
    torch.cuda.synchronize()
    assert rel_err(host(sb), s_ref) <= TOL["bf16"]
    og = lasad.lasad_forward_gated(q, lam, v, H, W, start_pos=start, boundary_mode=mode, state_out=s1, out_dtype=torch.float32)
    torch.cuda.synchronize()
    ref, s_ref = oracle.gated_recurrent(host(q), host(lam), host(v), W, start_pos=start, mode=mode, want_state=True)
    assert rel_err(host(og), ref) <= TOL["bf16"]
    assert rel_err(host(s1), s_ref) <= TOL["bf16"]
