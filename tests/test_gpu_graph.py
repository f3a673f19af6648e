"""The three entry points only enqueue kernels (no allocation, no memset, no host synchronisation),
so a caller may record them into a HIP graph.  The graph is replayed several times with new input
values in the same buffers and with eager work in between; every replay must equal the eager
result bit for bit."""
import numpy as np
import pytest

from paper_1501_06633_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_forward_and_both_gradients_replay_from_a_graph():
    import torch
    from paper_1501_06633_amd import binding as B

    L = W.custom("graph", 32, 20, 18, 24, 96, 3, 2, 1, 0.5)
    st, Wo, Ho = B.mdnn_out_dims(L.Wi, L.Hi, L.Sk, L.stride, L.pad)
    dims = (L.Nb, L.Wi, L.Hi, L.Nc, L.No, L.Sk, L.stride, L.pad)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)

    def fresh(shape):
        return torch.randint(-4, 5, shape, device="cuda", generator=gen).float()

    x, w, g = fresh((L.Nc, L.Hi, L.Wi, L.Nb)), fresh((L.Nc, L.Sk, L.Sk, L.No)), fresh((L.No, Ho, Wo, L.Nb))
    y = torch.empty((L.No, Ho, Wo, L.Nb), device="cuda")
    dx = torch.empty_like(x)
    dw = torch.empty_like(w)
    ws_d = torch.empty(B.mdnn_conv_bprop_data_workspace(*dims)[1], dtype=torch.uint8, device="cuda")
    ws_f = torch.empty(B.mdnn_conv_bprop_filter_workspace(*dims)[1], dtype=torch.uint8, device="cuda")

    def enqueue():
        B.mdnn_conv_fprop(x, w, L.stride, L.pad, L.alpha, out=y)
        B.mdnn_conv_bprop_data(g, w, (L.Hi, L.Wi), L.stride, L.pad, L.alpha, din=dx, workspace=ws_d)
        B.mdnn_conv_bprop_filter(x, g, L.Sk, L.stride, L.pad, L.alpha, dfilt=dw, workspace=ws_f)

    enqueue()                                   # warm-up outside the capture (function attributes are set here)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep in range(4):
        for t in (x, w, g):
            t.copy_(fresh(tuple(t.shape)))
        for t in (y, dx, dw):
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (y, dx, dw)]
        for t in (y, dx, dw):
            t.fill_(float("nan"))
        enqueue()                               # eager, same buffers
        torch.cuda.synchronize()
        for name, a, b in zip(("fprop", "bprop_data", "bprop_filter"), got, (y, dx, dw)):
            assert torch.isfinite(a).all(), (rep, name)
            assert torch.equal(a, b), (rep, name)
        assert float(got[0].abs().max()) > 0
