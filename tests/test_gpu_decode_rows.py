"""Decode step with one raster position per batch row (continuous batching) against the oracle: every row is
checked with the oracle's one-token step at ITS position; rows marked inactive must keep their states
bit for bit and produce zero output."""
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


@pytest.mark.parametrize("d,dtype", [(64, "bf16"), (64, "f32"), (32, "bf16"), (128, "bf16")])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("gated", [False, True], ids=["scalar", "vector"])
def test_decode_rows(lasad, oracle, d, dtype, mode, gated):
    import torch
    B, Hh, H, W = 9, 3, 5, 7
    rng = np.random.default_rng(1000 + d + mode)
    sc = np.float32(1.0 / np.sqrt(d))
    q, k, v = (wl.store_round(rng.standard_normal((B, Hh, d), dtype=np.float32) * sc, dtype) for _ in range(3))
    lam = wl.gate_inputs((B, Hh, d), dtype, 5) if gated else None
    gam = rng.uniform(0.5, 0.99, size=(Hh,)).astype(np.float32)
    s0 = (rng.standard_normal((B, Hh, d, d)) * 0.3).astype(np.float32)
    pos = np.array([0, 6, 7, 34, -1, 13, 20, 35, 27], dtype=np.int32)     # 35 = H*W is outside the grid
    state = torch.from_numpy(s0.copy()).cuda()
    dev = lambda x: None if x is None else lasad.to_device(x, dtype)
    o = lasad.lasad_decode_step_rows(dev(q), dev(v), state, torch.from_numpy(pos).cuda(), H, W,
                                     k=dev(k), lam=dev(lam), gamma=None if gated else torch.from_numpy(gam).cuda(),
                                     boundary_mode=mode, q_scale=0.9, out_dtype=torch.float32)
    torch.cuda.synchronize()
    got_o, got_s = o.cpu().numpy(), state.cpu().numpy()
    for b in range(B):
        if pos[b] < 0 or pos[b] >= H * W:
            assert not got_o[b].any()
            assert np.array_equal(got_s[b], s0[b])
            continue
        ref_s = s0[b:b + 1].astype(np.float64)
        if gated:
            ref_o, ref_s1 = oracle.gated_recurrent(q[b:b + 1, None], lam[b:b + 1, None], v[b:b + 1, None], W, k=k[b:b + 1, None],
                                                   start_pos=int(pos[b]), mode=mode, q_scale=0.9, s0=ref_s, want_state=True)
            ref_o = ref_o[:, 0]
        else:
            lam_t, _ = oracle.decay_factors(gam, H, W, int(pos[b]), 1, mode)
            ref_o = oracle.decode_step(q[b:b + 1], k[b:b + 1], v[b:b + 1], lam_t[:, 0], ref_s, q_scale=0.9)
            ref_s1 = ref_s
        assert rel_err(got_o[b:b + 1], ref_o) <= TOL[dtype], b
        assert rel_err(got_s[b:b + 1], ref_s1) <= TOL[dtype], b


def test_decode_rows_equals_uniform_step(lasad):
    """All rows at one position: bit-identical to lasad_decode_step."""
    import torch
    w = wl.scaled(wl.AR_DECODE, B=16)
    q, k, v, gam = wl.decode_inputs(w, steps=1)
    tq, tk, tv = (lasad.to_device(x[0], w.dtype) for x in (q, k, v))
    tg = torch.from_numpy(gam).cuda()
    s_a = torch.randn((w.B, w.Hh, w.d, w.d), device="cuda")
    s_b = s_a.clone()
    o_a = lasad.lasad_decode_step(tq, tk, tv, tg, s_a, w.grid_h, w.grid_w, 47)
    o_b = lasad.lasad_decode_step_rows(tq, tv, s_b, torch.full((w.B,), 47, dtype=torch.int32, device="cuda"),
                                       w.grid_h, w.grid_w, k=tk, gamma=tg)
    torch.cuda.synchronize()
    assert torch.equal(o_a, o_b) and torch.equal(s_a, s_b)
