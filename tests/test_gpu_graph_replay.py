"""Every entry point under HIP graph capture: a graph holding one call of each is replayed several times, with eager
work and synchronisations between the replays and the inputs changed in place before each replay; every replay must
reproduce the eager results for the same inputs bit for bit (the kernels are deterministic)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lasad():
    import torch
    assert torch.cuda.is_available()
    from paper_2507_01652_amd import binding
    binding.load()
    return binding


def test_graph_replays_match_eager(lasad):
    import torch
    B, H, W, Hh, d = 3, 10, 13, 4, 64
    n = H * W
    gen = torch.Generator(device="cuda").manual_seed(5)
    rnd = lambda *shape: (torch.randn(*shape, device="cuda", generator=gen) / 8).to(torch.bfloat16)
    q, k, v, g = rnd(B, n, Hh, d), rnd(B, n, Hh, d), rnd(B, n, Hh, d), rnd(B, n, Hh, d)
    lam = torch.sigmoid(torch.randn(B, n, Hh, d, device="cuda", generator=gen) + 2).to(torch.bfloat16)
    gam = torch.linspace(0.9, 0.99, Hh, device="cuda")
    state = torch.zeros(B, Hh, d, d, device="cuda")
    qs, ks, vs = (rnd(B, Hh, d) for _ in range(3))
    kc = torch.zeros(B, Hh, 8, d, device="cuda", dtype=torch.bfloat16)
    vc = torch.zeros_like(kc)

    # static output buffers and workspaces: nothing is allocated inside the captured region
    o = torch.empty_like(q)
    og = torch.empty_like(q)
    ol = torch.empty_like(q)
    grads = tuple(torch.empty_like(q) for _ in range(3))
    dgam = torch.empty(Hh, device="cuda")
    ggrads = tuple(torch.empty_like(q) for _ in range(3))
    od = torch.empty_like(qs)
    oc = torch.empty_like(qs)
    ws_f = torch.empty(max(1, lasad.lasad_forward_workspace_bytes(B, Hh, n, d, lasad.BF16)), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(lasad.lasad_backward_workspace_bytes(B, Hh, n, d, lasad.BF16), dtype=torch.uint8, device="cuda")
    ws_g = torch.empty(lasad.lasad_backward_gated_workspace_bytes(B, Hh, n, d), dtype=torch.uint8, device="cuda")
    lgrads = tuple(torch.empty_like(q) for _ in range(3))
    dwt = torch.empty(Hh, d, device="cuda")
    ws_l = torch.empty(lasad.lasad_backward_layer_workspace_bytes(q), dtype=torch.uint8, device="cuda")
    # the entry points with carried states, the allocation-free forward, the vector-decay cache step
    s_in = torch.randn(B, Hh, d, d, device="cuda", generator=gen) * 0.3
    h_out = torch.randn(B, Hh, d, d, device="cuda", generator=gen) * 0.1
    cgrads = tuple(torch.empty_like(q) for _ in range(3))
    cdgam, cds = torch.empty(Hh, device="cuda"), torch.empty(B, Hh, d, d, device="cuda")
    ws_c = torch.empty(lasad.lasad_backward_carried_workspace_bytes(B, Hh, n, d, lasad.BF16), dtype=torch.uint8, device="cuda")
    cggrads = tuple(torch.empty_like(q) for _ in range(3))
    cgds = torch.empty(B, Hh, d, d, device="cuda")
    ws_cg = torch.empty(lasad.lasad_backward_gated_carried_workspace_bytes(B, Hh, n, d), dtype=torch.uint8, device="cuda")
    o_static = torch.empty_like(q)
    lams = torch.sigmoid(torch.randn(B, Hh, d, device="cuda", generator=gen) + 2).to(torch.bfloat16)
    lc = torch.sigmoid(torch.randn(B, Hh, 8, d, device="cuda", generator=gen) + 2).to(torch.bfloat16)
    vc2 = rnd(B, Hh, 8, d)
    ogc = torch.empty_like(qs)

    def run():
        lasad.lasad_forward_chunked(q, k, v, gam, H, W, out=o, workspace=ws_f)
        lasad.lasad_backward_chunked(q, k, v, g, gam, H, W, grads=grads, dgamma=dgam, workspace=ws_b)
        lasad.lasad_forward_gated(q, lam, v, H, W, out=og)
        lasad.lasad_forward_layer(q, lam, v, H, W, out=ol)
        lasad.lasad_backward_gated(q, lam, v, g, H, W, grads=ggrads, workspace=ws_g)
        lasad.lasad_backward_layer(q, lam, v, g, H, W, grads=lgrads, dweight=dwt, workspace=ws_l)
        state.zero_()
        lasad.lasad_decode_step(qs, ks, vs, gam, state, H, W, 3, out=od)
        lasad.lasad_decode_step_cached(qs, ks, vs, gam, kc, vc, H, W, 3, out=oc)
        lasad.lasad_backward_chunked_carried(q, k, v, g, gam, H, W, state_in=s_in, d_state_out=h_out, grads=cgrads, dgamma=cdgam,
                                             d_state_in=cds, workspace=ws_c)
        lasad.lasad_backward_gated_carried(q, lam, v, g, H, W, state_in=s_in, d_state_out=h_out, grads=cggrads, d_state_in=cgds,
                                           workspace=ws_cg)
        lasad.lasad_forward_chunked_static(q, k, v, gam, H, W, o_static)
        lasad.lasad_decode_step_gated_cached(qs, lams, vs, lc, vc2, H, W, 3, out=ogc)

    outputs = lambda: [t.clone() for t in (o, og, ol, *grads, dgam, *ggrads, *lgrads, dwt, od, oc, state, kc, vc,
                                           *cgrads, cdgam, cds, *cggrads, cgds, o_static, ogc, lc, vc2)]
    run()                                   # warm-up (loads the code objects)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (q, k, v, g, qs, ks, vs):  # new inputs, in place
            t.copy_(rnd(*t.shape))
        run()                               # eager reference for these inputs
        torch.cuda.synchronize()
        want = outputs()
        for t in (o, og, ol, *grads, dgam, *ggrads, od, oc, *cgrads, cdgam, cds, *cggrads, cgds, o_static, ogc):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = outputs()
        for i, (a, b) in enumerate(zip(got, want)):
            assert torch.equal(a, b), (rep, i)
