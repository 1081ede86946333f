"""The operators under HIP graph capture: the library allocates nothing and launches only on the stream it is
given, so a captured step (forward, input gradient, filter gradient through the entry point that needs no
workspace) must replay to the same bits as the eager calls -- also after the inputs have changed in place."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cks():
    import torch
    from paper_2306_15951_amd import binding

    assert torch.cuda.is_available(), "this test needs the MI355X"
    binding.lib()
    return binding


GRAPH_LAYERS = [
    ("graph_s2", 96, 64, 11, 9, 96, 3, 3, 2, 1),          # general kernels, filter read in place
    ("graph_stem", 6, 3, 40, 37, 64, 7, 7, 2, 3),         # stem kernels (input gradient: one launch on the 4x4x1 matrix instruction)
    ("graph_stem_pad2", 6, 3, 40, 37, 64, 7, 7, 2, 2),    # stem kernels, another padding: two launches for the input gradient
]


@pytest.mark.parametrize("geo", GRAPH_LAYERS, ids=[g[0] for g in GRAPH_LAYERS])
def test_captured_step_replays_to_the_eager_result(cks, oracle, geo):
    import torch
    from paper_2306_15951_amd import synth

    L = synth.Layer(*geo)
    print("geometry", geo, flush=True)
    g = (L.N, L.IC, L.IH, L.IW, L.OC, L.FH, L.FW, L.stride, L.padding)
    st, pd = (L.stride,) * 2, (L.padding,) * 2
    X0, W0, dY0 = synth.make_inputs(L, "int", 90)
    X, W, dY = (torch.from_numpy(a).cuda() for a in (X0, W0, dY0))
    Y, dX, dW = torch.empty_like(dY), torch.empty_like(X), torch.empty_like(W)
    ws = torch.empty(max(cks.cks_deconv2d_workspace(*g) // 4, 1), device="cuda")

    def step():
        cks.cks_conv2d_fwd(X, W, Y, L.stride, L.padding)
        cks.cks_deconv2d(dY, W, dX, L.stride, L.padding, ws)
        cks.cks_dilated_conv2d_wgrad_noalloc_hw(X, dY, dW, st, pd)

    step()                                   # once eagerly: one-time set-up (kernel attributes, scratch address)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        Xh, Wh, dYh = synth.make_inputs(L, "int", 91 + rep)
        X.copy_(torch.from_numpy(Xh)); W.copy_(torch.from_numpy(Wh)); dY.copy_(torch.from_numpy(dYh))
        for out in (Y, dX, dW):
            out.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.cpu().numpy().copy() for t in (Y, dX, dW)]
        for out in (Y, dX, dW):
            out.fill_(float("nan"))
        step()                               # the program's own eager work between the replays
        torch.cuda.synchronize()
        for a, b, nm in zip(got, (Y, dX, dW), ("Y", "dX", "dW")):
            assert np.array_equal(a.view(np.uint32), b.cpu().numpy().view(np.uint32)), "%s replay %d: %s differs from eager" % (L.name, rep, nm)
        assert np.array_equal(got[0].astype(np.float64), oracle.conv_fwd(Xh, Wh, L.stride, L.padding))
        assert np.array_equal(got[1].astype(np.float64), oracle.deconv(dYh, Wh, L.IH, L.IW, L.stride, L.padding))
        assert np.array_equal(got[2].astype(np.float64), oracle.wgrad(Xh, dYh, L.FH, L.FW, L.stride, L.padding))
