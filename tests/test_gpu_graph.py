"""The entry points only enqueue kernels on the caller's stream (no allocation, no memset, no host
synchronisation), so a chain of them can be captured into a HIP graph.  The graph is replayed several
times with eager work and synchronisations in between and new input each time; every replay must give
the bytes of the eager chain on that input."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_1910_06188_amd import synth  # noqa: E402


@pytest.fixture(scope="module")
def q8():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1910_06188_amd import q8 as mod
    return mod


def test_dynamic_ffn_chain_under_graph_capture(q8):
    M, H, F = 520, 256, 1024
    d = synth.ffn_block(11, M, H, F)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def quant_w(W):
        wd, a, s = dev(W), torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
        q8.q8_absmax(wd, a, s)
        wq = torch.empty(W.shape, dtype=torch.int8, device="cuda")
        q8.q8_quantize(wd, s, wq)
        return wq, s
    w1, s1 = quant_w(d["W1"])
    w2, s2 = quant_w(d["W2"])
    b1, b2 = dev(d["b1"]), dev(d["b2"])
    x = dev(d["x"])
    xq = torch.empty(M * F, dtype=torch.int8, device="cuda")
    scal = torch.zeros(q8.SCAL_WORK, device="cuda")
    gs = torch.zeros(2, device="cuda")
    g = torch.empty((M, F), device="cuda")
    y = torch.empty((M, H), device="cuda")

    def chain():
        q8.q8_linear_f32(x, w1, b1, s1, xq[: M * H], scal, g, out_amax=gs[0:1], flags=q8.EPI_GELU | q8.EPI_ABSMAX)
        q8.q8_quantize_amax(g, gs[0:1], gs[1:2], xq[: M * F].view(M, F))
        q8.q8_linear(xq[: M * F].view(M, F), w2, b2, gs[1:2], s2, y)

    chain()                                    # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            chain()
    torch.cuda.synchronize()
    rng = synth.rng(12)
    for rep in range(4):
        x.copy_(dev(synth.activations(rng, M, H) * np.float32(0.5 + rep)))
        y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        y_graph, g_graph, s_graph = y.clone(), g.clone(), gs.clone()
        y.zero_()
        g.zero_()
        chain()                                # eager, on the same input
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y) and torch.equal(g_graph, g) and torch.equal(s_graph, gs), rep
        assert float(y.abs().max()) > 0
