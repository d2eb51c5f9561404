"""Calls on a stream that is not torch's current one: the kernels run on the stream handed in, and the workspace
that the binding takes from torch's caching allocator is tied to that stream (a block freed on return may otherwise
be handed to later work on the current stream while the kernels still use it)."""
import numpy as np
import pytest

from paper_2507_01652_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lasad():
    import torch
    assert torch.cuda.is_available()
    from paper_2507_01652_amd import binding
    binding.load()
    return binding


def _inputs(B, n, Hh, seed):
    rng = np.random.default_rng(seed)
    return [wl.store_round(rng.standard_normal((B, n, Hh, 64), dtype=np.float32) / np.float32(8.0), "bf16") for _ in range(4)]


def test_forward_and_backward_on_a_side_stream(lasad):
    import torch
    B, Hh, H, W = 1, 4, 48, 32                    # few long sequences: the segment plan, i.e. a workspace in the forward
    n = H * W
    q, k, v, g = (lasad.to_device(x, "bf16") for x in _inputs(B, n, Hh, 5))
    gam = torch.full((Hh,), 0.97, device="cuda")
    assert lasad.lasad_forward_workspace_bytes(B, Hh, n, 64, lasad.BF16) > 0
    ref_o = lasad.lasad_forward_chunked(q, k, v, gam, H, W)
    ref_g = lasad.lasad_backward_chunked(q, k, v, g, gam, H, W)
    lam = torch.sigmoid(q.float() * 8 + 2).to(torch.bfloat16)
    ref_v = lasad.lasad_backward_gated(q, lam, v, g, H, W)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()                    # default priority
    side.wait_stream(torch.cuda.current_stream())
    o = lasad.lasad_forward_chunked(q, k, v, gam, H, W, stream=side)
    gs = lasad.lasad_backward_chunked(q, k, v, g, gam, H, W, stream=side)
    gv = lasad.lasad_backward_gated(q, lam, v, g, H, W, stream=side)
    # allocator traffic on the current stream while the side stream works: blocks of the workspaces' sizes
    sizes = [lasad.lasad_forward_workspace_bytes(B, Hh, n, 64, lasad.BF16), lasad.lasad_backward_workspace_bytes(B, Hh, n, 64, lasad.BF16),
             lasad.lasad_backward_gated_workspace_bytes(B, Hh, n, 64)]
    for _ in range(8):
        for sz in sizes:
            torch.empty((sz,), dtype=torch.uint8, device="cuda").fill_(0x7f)
    side.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(o, ref_o)
    for a, b in zip(gs, ref_g):
        assert torch.equal(a, b)
    for a, b in zip(gv, ref_v):
        assert torch.equal(a, b)


def test_decode_steps_on_a_side_stream(lasad):
    import torch
    B, Hh, H, W = 8, 4, 6, 9
    rng = np.random.default_rng(9)
    q, k, v = (lasad.to_device(wl.store_round(rng.standard_normal((H * W, B, Hh, 64), dtype=np.float32) / np.float32(8.0), "bf16"), "bf16")
               for _ in range(3))
    gam = torch.full((Hh,), 0.93, device="cuda")
    s_ref = torch.zeros((B, Hh, 64, 64), device="cuda")
    ref = [lasad.lasad_decode_step(q[t], k[t], v[t], gam, s_ref, H, W, t) for t in range(H * W)]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    s_side = torch.zeros((B, Hh, 64, 64), device="cuda")
    side.wait_stream(torch.cuda.current_stream())
    got = [lasad.lasad_decode_step(q[t], k[t], v[t], gam, s_side, H, W, t, stream=side) for t in range(H * W)]
    side.synchronize()
    assert torch.equal(s_side, s_ref)
    for a, b in zip(got, ref):
        assert torch.equal(a, b)
