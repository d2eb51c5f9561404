"""GPU parity of the fused layer (Algorithm 1 between its Linear maps: SiLU on q, sigmoid gate, tied key,
spatially aware recurrence, root-mean-square Norm) against the oracle's gated_layer, forward and decode."""
import numpy as np
import pytest

from paper_2507_01652_amd import workloads as wl
from helpers import TOL, both_outputs, decode_both, rel_err, sample_pairs, gather_pairs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lasad():
    import torch
    assert torch.cuda.is_available()
    from paper_2507_01652_amd import binding
    binding.load()
    return binding


def _pre_inputs(B, n, Hh, d, dtype, seed):
    """Pre-activation query ~ N(0, 1), gate logits ~ N(2, 1) (sigmoid of which is the gate recipe of the
    vector-decay tests), values ~ N(0, 1)/sqrt(d); all rounded to the storage type."""
    rng = np.random.default_rng(seed)
    q = wl.store_round(rng.standard_normal((B, n, Hh, d), dtype=np.float32), dtype)
    z = wl.store_round(rng.standard_normal((B, n, Hh, d), dtype=np.float32) + np.float32(2.0), dtype)
    v = wl.store_round(rng.standard_normal((B, n, Hh, d), dtype=np.float32) / np.float32(np.sqrt(d)), dtype)
    return q, z, v


@pytest.mark.parametrize("dtype,H,W,B,Hh", [("bf16", 16, 16, 2, 3), ("bf16", 9, 17, 1, 2), ("f32", 7, 9, 2, 2),
                                             ("bf16", 3, 5, 70, 4), ("bf16", 9, 17, 65, 4), ("bf16", 1, 1, 1, 1)])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("norm", ["weighted", "plain", "off"])
def test_forward_layer(lasad, oracle, dtype, H, W, B, Hh, mode, norm):
    import torch
    d, n = 64, H * W
    q, z, v = _pre_inputs(B, n, Hh, d, dtype, 40 + H + mode)
    w = None if norm != "weighted" else np.random.default_rng(3).uniform(0.5, 1.5, size=(Hh, d)).astype(np.float32)
    eps = -1.0 if norm == "off" else 1e-5
    if norm == "off":
        ref, s_ref = oracle.gated_recurrent(oracle.silu(q), oracle.sigmoid(z), v, W, mode=mode, want_state=True)
    else:
        ref, s_ref = oracle.gated_layer(q, z, v, W, norm_weight=w, eps=eps, mode=mode, want_state=True)
    dev = lambda x: lasad.to_device(x, dtype)
    s1 = torch.empty((B, Hh, d, d), dtype=torch.float32, device="cuda")
    # fp32 output against the bare tolerance; with bf16 inputs the bf16 output must be its rounding
    o = both_outputs(lasad.lasad_forward_layer, dtype == "bf16", q_pre=dev(q), z=dev(z), v=dev(v), grid_h=H, grid_w=W,
                     norm_weight=None if w is None else torch.from_numpy(w).cuda(), norm_eps=eps, boundary_mode=mode,
                     state_out=s1)
    torch.cuda.synchronize()
    assert rel_err(o.cpu().numpy(), ref) <= TOL[dtype]
    assert rel_err(s1.cpu().numpy(), s_ref) <= TOL[dtype]


def test_forward_layer_strong_gates_take_the_serial_route(lasad, oracle):
    """Gate logits around -1.5 (lambda ~ 0.18): every chunk leaves the chunked kernel's range."""
    import torch
    B, Hh, d, H, W = 2, 2, 64, 9, 17
    q, z, v = _pre_inputs(B, H * W, Hh, d, "bf16", 99)
    z = wl.store_round(z - np.float32(3.5), "bf16")
    ref = oracle.gated_layer(q, z, v, W, eps=1e-6)
    dev = lambda x: lasad.to_device(x, "bf16")
    o = lasad.lasad_forward_layer(dev(q), dev(z), dev(v), H, W, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert rel_err(o.cpu().numpy(), ref) <= TOL["bf16"]


@pytest.mark.parametrize("name,n_pairs", [("base_prefill_16x16", 16), ("large_prefill_24x24", 16), ("highres_64x64", 4)])
def test_forward_layer_bench_shape_sampled(lasad, oracle, name, n_pairs):
    """The shapes bench.py times, full size; the oracle on sampled sequences; bf16 output = rounded fp32 output."""
    import torch
    w = wl.CONFIGS[name]
    q, z, v = _pre_inputs(w.B, w.N, w.Hh, w.d, "bf16", 7)
    dev = lambda x: lasad.to_device(x, "bf16")
    o = both_outputs(lasad.lasad_forward_layer, True, q_pre=dev(q), z=dev(z), v=dev(v), grid_h=w.grid_h, grid_w=w.grid_w)
    torch.cuda.synchronize()
    pairs = sample_pairs(w.B, w.Hh, n_pairs, seed=1)
    ref = oracle.gated_layer(gather_pairs(q, pairs), gather_pairs(z, pairs), gather_pairs(v, pairs), w.grid_w)
    assert rel_err(gather_pairs(o.cpu().numpy(), pairs), ref) <= TOL["bf16"]


@pytest.mark.parametrize("d,dtype", [(64, "bf16"), (32, "f32"), (128, "bf16")])
def test_decode_layer_walk(lasad, oracle, d, dtype):
    import torch
    B, Hh, H, W = 3, 2, 4, 6
    n = H * W
    q, z, v = _pre_inputs(B, n, Hh, d, dtype, 200 + d)
    w = np.random.default_rng(4).uniform(0.5, 1.5, size=(Hh, d)).astype(np.float32)
    ref, s_ref = oracle.gated_layer(q, z, v, W, norm_weight=w, eps=1e-5, q_scale=1.3, want_state=True)
    dev = lambda x: lasad.to_device(np.ascontiguousarray(x.transpose(1, 0, 2, 3)), dtype)
    tq, tz, tv = dev(q), dev(z), dev(v)
    tw = torch.from_numpy(w).cuda()
    state = torch.zeros((B, Hh, d, d), dtype=torch.float32, device="cuda")
    worst = 0.0
    for t in range(n):
        o = decode_both(lambda st, odt: lasad.lasad_decode_step_layer(tq[t], tz[t], tv[t], st, H, W, t, norm_weight=tw,
                                                                      norm_eps=1e-5, q_scale=1.3, out_dtype=odt),
                        state, dtype == "bf16")
        worst = max(worst, rel_err(o.cpu().numpy()[:, None], ref[:, t:t + 1]))
    assert worst <= TOL[dtype]
    assert rel_err(state.cpu().numpy(), s_ref) <= TOL[dtype]
