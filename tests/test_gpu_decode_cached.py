"""Decode steps from a key / value cache (lasad_decode_step_cached) against the oracle: the outputs of a raster
walk from a zero state must be those of the oracle's recurrence, the caches must hold the walk's k and v bit for
bit, and the state built from the cache must let the state-form step continue the walk."""
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


def _walk_inputs(steps, B, Hh, d, dtype, seed):
    rng = np.random.default_rng(seed)
    sc = np.float32(1.0 / np.sqrt(d))
    q, k, v = (wl.store_round(rng.standard_normal((steps, B, Hh, d), dtype=np.float32) * sc, dtype) for _ in range(3))
    gam = rng.uniform(0.6, 0.99, size=(Hh,)).astype(np.float32)
    return q, k, v, gam


@pytest.mark.parametrize("d,dtype", [(64, "bf16"), (64, "f32"), (32, "bf16"), (128, "bf16")])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_cached_walk_matches_the_recurrence(lasad, oracle, d, dtype, mode):
    import torch
    B, Hh, H, W = 3, 2, 5, 7
    steps = H * W
    q, k, v, gam = _walk_inputs(steps, B, Hh, d, dtype, 100 + d + mode)
    tq, tk, tv = (lasad.to_device(x, dtype) for x in (q, k, v))
    tg = torch.from_numpy(gam).cuda()
    kc = torch.zeros((B, Hh, steps + 3, d), dtype=tq.dtype, device="cuda")
    vc = torch.zeros_like(kc)
    outs = [lasad.lasad_decode_step_cached(tq[t], tk[t], tv[t], tg, kc, vc, H, W, t, boundary_mode=mode, q_scale=0.8,
                                           out_dtype=torch.float32) for t in range(steps)]
    torch.cuda.synchronize()
    lam, _ = oracle.decay_factors(gam, H, W, 0, steps, mode)
    tr = lambda x: np.ascontiguousarray(x.transpose(1, 0, 2, 3))            # [steps, B, Hh, d] -> [B, n, Hh, d]
    ref = oracle.recurrent(tr(q), tr(k), tr(v), lam, q_scale=0.8)
    got = np.stack([o.cpu().numpy() for o in outs], axis=1)
    assert rel_err(got, ref) <= TOL[dtype]
    assert torch.equal(kc[:, :, :steps], tk.permute(1, 2, 0, 3)) and torch.equal(vc[:, :, :steps], tv.permute(1, 2, 0, 3))
    assert not kc[:, :, steps:].any() and not vc[:, :, steps:].any()


def test_cached_walk_longer_than_one_tile(lasad, oracle):
    """More than 256 cached tokens: the kernel's token tiles."""
    import torch
    B, Hh, H, W, d = 1, 2, 20, 16, 64
    steps = H * W
    q, k, v, gam = _walk_inputs(steps, B, Hh, d, "bf16", 7)
    tq, tk, tv = (lasad.to_device(x, "bf16") for x in (q, k, v))
    tg = torch.from_numpy(gam).cuda()
    kc = torch.zeros((B, Hh, steps, d), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    outs = [lasad.lasad_decode_step_cached(tq[t], tk[t], tv[t], tg, kc, vc, H, W, t, out_dtype=torch.float32)
            for t in range(steps)]
    torch.cuda.synchronize()
    lam, _ = oracle.decay_factors(gam, H, W, 0, steps)
    tr = lambda x: np.ascontiguousarray(x.transpose(1, 0, 2, 3))
    ref = oracle.recurrent(tr(q), tr(k), tr(v), lam)
    got = np.stack([o.cpu().numpy() for o in outs], axis=1)
    assert rel_err(got, ref) <= TOL["bf16"]


def test_switch_from_the_cache_to_the_state(lasad, oracle):
    """The AR-decode shape's recipe: cache form for the first 128 positions, the state built from the cache by one
    forward call, state form afterwards; every output against the oracle's recurrence."""
    import torch
    B, Hh, H, W, d, switch = 4, 3, 16, 16, 64, 128
    steps = H * W
    q, k, v, gam = _walk_inputs(steps, B, Hh, d, "bf16", 11)
    tq, tk, tv = (lasad.to_device(x, "bf16") for x in (q, k, v))
    tg = torch.from_numpy(gam).cuda()
    kc = torch.zeros((B, Hh, switch, d), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    outs = [lasad.lasad_decode_step_cached(tq[t], tk[t], tv[t], tg, kc, vc, H, W, t, out_dtype=torch.float32)
            for t in range(switch)]
    state = torch.empty((B, Hh, d, d), dtype=torch.float32, device="cuda")
    as_seq = lambda c: c.permute(0, 2, 1, 3)                                # [B, Hh, T, d] viewed as [B, T, Hh, d]
    lasad.lasad_forward_chunked(as_seq(kc), as_seq(kc), as_seq(vc), tg, H, W, start_pos=0, state_out=state)
    outs += [lasad.lasad_decode_step(tq[t], tk[t], tv[t], tg, state, H, W, t, out_dtype=torch.float32)
             for t in range(switch, steps)]
    torch.cuda.synchronize()
    lam, _ = oracle.decay_factors(gam, H, W, 0, steps)
    tr = lambda x: np.ascontiguousarray(x.transpose(1, 0, 2, 3))
    ref = oracle.recurrent(tr(q), tr(k), tr(v), lam)
    got = np.stack([o.cpu().numpy() for o in outs], axis=1)
    assert rel_err(got, ref) <= TOL["bf16"]


def test_cached_rejects_bad_arguments(lasad):
    import torch
    q = torch.zeros((1, 2, 64), dtype=torch.bfloat16, device="cuda")
    g = torch.full((2,), 0.9, dtype=torch.float32, device="cuda")
    kc = torch.zeros((1, 2, 4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(Exception):
        lasad.lasad_decode_step_cached(q, q.clone(), q.clone(), g, kc, kc.clone(), 4, 4, 4)      # pos = capacity
    with pytest.raises(Exception):
        lasad.lasad_decode_step_cached(q, q.clone(), q.clone(), g, kc, kc, 4, 4, 0)              # caches alias
