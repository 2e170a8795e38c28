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


def test_dynamic_quantizer_of_a_large_tensor_under_graph_capture(q8):
    """A tensor in the size range of the one-pass quantizer: under capture the library takes the two-pass kernels (the
    one-pass kernel's barrier ticket comes from the host and would be the same on every replay), so replays on new
    data give the eager result -- which runs the one-pass kernel."""
    n = 3_145_728
    x = torch.randn(n, device="cuda")
    q, scal = torch.empty(n, dtype=torch.int8, device="cuda"), torch.zeros(q8.SCAL_WORK, device="cuda")
    q8.q8_quantize_dynamic(x, q, scal)
    torch.cuda.synchronize()
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            q8.q8_quantize_dynamic(x, q, scal)
    torch.cuda.synchronize()
    for rep in range(4):
        x.copy_(torch.randn(n, device="cuda") * (0.5 + rep))
        q.zero_()
        graph.replay()
        torch.cuda.synchronize()
        q_graph, s_graph = q.clone(), scal[:2].clone()
        q.zero_()
        q8.q8_quantize_dynamic(x, q, scal)
        torch.cuda.synchronize()
        assert torch.equal(q_graph, q) and torch.equal(s_graph, scal[:2]), rep
        assert int(q.abs().max()) == 127


def test_attention_block_under_graph_capture(q8):
    """LayerNorm (abs-max slots) -> quantize -> fused QKV FC -> FP32 attention (abs-max slots) -> quantize ->
    attention-output FC -> residual + LayerNorm: the first half of an encoder layer, captured and replayed."""
    B, S, heads, d = 3, 100, 2, 64
    M, H = B * S, heads * d
    g = synth.rng(21)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def quant_w(W):
        wd, a, s = dev(W), torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
        q8.q8_absmax(wd, a, s)
        wq = torch.empty(W.shape, dtype=torch.int8, device="cuda")
        q8.q8_quantize(wd, s, wq)
        return wq, s
    parts = [quant_w(synth.weights(g, H, H) * np.float32(4.0)) for _ in range(3)]
    w_qkv = torch.cat([p[0] for p in parts], 0).contiguous()
    s_qkv = torch.cat([p[1] for p in parts]).contiguous()
    b_qkv = dev(synth.weights(g, 1, 3 * H)[0])
    w_o, s_o = quant_w(synth.weights(g, H, H))
    b_o = dev(synth.weights(g, 1, H)[0])
    gamma, beta = torch.ones(H, device="cuda"), torch.zeros(H, device="cuda")
    mask = np.zeros((B, S), np.float32)
    mask[1, 70:] = -10000.0
    mask_d = dev(mask)
    x = dev(synth.activations(g, M, H))
    x_ln, qkv, ctx, attn, y = (torch.empty((M, n), device="cuda") for n in (H, 3 * H, H, H, H))
    xq = torch.empty((M, H), dtype=torch.int8, device="cuda")
    slots_a, slots_b, slots_c = (torch.zeros(q8.AMAX_SLOTS, device="cuda") for _ in range(3))
    sx = torch.zeros(1, device="cuda")

    def chain():
        q8.q8_layernorm_absmax(x, gamma, beta, x_ln, amax_slots=slots_a)
        q8.q8_quantize_amax(x_ln, slots_a, sx, xq)
        q8.q8_linear(xq, w_qkv, b_qkv, sx, s_qkv, qkv, n_groups=3)
        q8.q8_attention(qkv, B, S, heads, d, ctx=ctx, mask=mask_d, amax_slots=slots_b)
        q8.q8_quantize_amax(ctx, slots_b, sx, xq)
        q8.q8_linear(xq, w_o, b_o, sx, s_o, attn)
        q8.q8_layernorm_absmax(x_ln, gamma, beta, y, residual=attn, amax_slots=slots_c)

    chain()                                    # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            chain()
    torch.cuda.synchronize()
    for rep in range(4):
        x.copy_(dev(synth.activations(g, M, H) * np.float32(0.5 + rep)))
        y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (y, ctx, qkv, slots_b, slots_c)]
        y.zero_()
        ctx.zero_()
        chain()                                # eager, on the same input
        torch.cuda.synchronize()
        for a, b in zip(got, (y, ctx, qkv, slots_b, slots_c)):
            assert torch.equal(a, b), rep
        assert float(y.abs().max()) > 0
