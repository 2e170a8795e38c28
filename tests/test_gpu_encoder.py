"""Whole encoder layers on the GPU, every operation in the library, checked stage by stage against the CPU oracle.

A layer is: quantize (scale from the abs-max slots of the producer) -> fused Q|K|V FC -> FP32 softmax attention ->
quantize -> attention-output FC -> residual + LayerNorm -> quantize -> FFN1 FC + GELU -> quantize -> FFN2 FC ->
residual + LayerNorm, each quantize + FC pair being one q8_linear_f32_slots call (Section 3: FC layers quantized,
Softmax / LayerNorm / GELU in FP32; Section 4.1: dynamic scales).
Each stage is compared with the oracle applied to the input the GPU itself gave that stage, at that stage's own
bar (int8 codes and scales bit-exact, FC outputs 1e-6 relative, LayerNorm 1e-6 relative, attention 2e-6 of
max|V|, GELU outputs abs 1e-6 + rel 1e-5): an end-to-end comparison would measure how rounding-boundary flips of
single codes propagate, not whether any kernel is right.  Shapes: the BERT-Base encoder layer at batch 32 x seq 128,
and the 12-layer BERT-Base forward at batch 64 x seq 128 with its int8 embedding tables.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import q8_oracle as O  # noqa: E402
from paper_1910_06188_amd import synth  # noqa: E402

THREADS = 16


@pytest.fixture(scope="module")
def q8():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1910_06188_amd import q8 as mod
    return mod


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def rel_close(got, ref, rtol, atol=0.0, what=""):
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    tol = atol + rtol * np.abs(ref.astype(np.float64))
    assert not (err > tol).any(), f"{what}: worst err/tol {np.max(err / np.maximum(tol, 1e-300)):.2f}"


class Layer:
    """Quantized weights of one encoder layer on the GPU (quantized there) and, bit-identical, on the host."""

    def __init__(self, q8, d):
        self.H, self.F, self.heads = d["hidden"], d["ffn"], d["heads"]

        def quant(W):
            wd, a, s = dev(W), torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda")
            q8.q8_absmax(wd, a, s)
            wq = torch.empty(W.shape, dtype=torch.int8, device="cuda")
            q8.q8_quantize(wd, s, wq)
            wq_ref, s_ref = O.quantize_tensor(W)
            assert np.array_equal(host(wq), wq_ref) and host(s)[0] == s_ref
            return wq, s, wq_ref, np.float32(s_ref)
        parts = [quant(d["W" + n]) for n in ("q", "k", "v")]
        self.w_qkv = torch.cat([p[0] for p in parts], 0).contiguous()
        self.s_qkv = torch.cat([p[1] for p in parts]).contiguous()
        self.w_qkv_h = np.concatenate([p[2] for p in parts], 0)
        self.s_qkv_h = np.array([p[3] for p in parts], np.float32)
        self.b_qkv_h = np.concatenate([d["bq"], d["bk"], d["bv"]])
        self.b_qkv = dev(self.b_qkv_h)
        self.w_o, self.s_o, self.w_o_h, self.s_o_h = quant(d["Wo"])
        self.w_1, self.s_1, self.w_1_h, self.s_1_h = quant(d["W1"])
        self.w_2, self.s_2, self.w_2_h, self.s_2_h = quant(d["W2"])
        self.b_o_h, self.b_1_h, self.b_2_h = d["bo"], d["b1"], d["b2"]
        self.b_o, self.b_1, self.b_2 = dev(d["bo"]), dev(d["b1"]), dev(d["b2"])
        g = synth.rng(1000 + self.H)
        self.gamma_h = [(1 + 0.1 * g.standard_normal(self.H)).astype(np.float32) for _ in range(2)]
        self.beta_h = [(0.1 * g.standard_normal(self.H)).astype(np.float32) for _ in range(2)]
        self.gamma, self.beta = [dev(a) for a in self.gamma_h], [dev(a) for a in self.beta_h]


class Work:
    """Work buffers of one layer pass, reused from layer to layer."""

    def __init__(self, q8, M, H, F):
        f = lambda *s: torch.empty(s, device="cuda")
        self.qkv, self.ctx, self.attn, self.h1, self.g, self.out = f(M, 3 * H), f(M, H), f(M, H), f(M, H), f(M, F), f(M, H)
        self.xq_x, self.xq_c, self.xq_h = (torch.empty((M, H), dtype=torch.int8, device="cuda") for _ in range(3))
        self.xq_g = torch.empty((M, F), dtype=torch.int8, device="cuda")
        self.slots_c, self.slots_h = (torch.zeros(q8.AMAX_SLOTS, device="cuda") for _ in range(2))
        self.sc = torch.zeros(8, device="cuda")       # (max|x|, S_x) of the layer's four FC inputs
        self.g_amax = torch.full((1,), 1e9, device="cuda")   # stale on purpose: the FFN1 call resets it


def gpu_layer(q8, L, w, x_in, slots_x, x_next, slots_next, B, S, mask=None):
    """Every FC is one q8_linear_f32_slots call: quantize with the scale from its producer's slots, then the GEMM."""
    H, F = L.H, L.F
    sc = w.sc
    q8.q8_linear_f32_slots(x_in, slots_x, L.w_qkv, L.b_qkv, L.s_qkv, w.xq_x, sc[0:2], w.qkv, n_groups=3)
    q8.q8_attention(w.qkv, B, S, L.heads, H // L.heads, ctx=w.ctx, mask=mask, amax_slots=w.slots_c)
    q8.q8_linear_f32_slots(w.ctx, w.slots_c, L.w_o, L.b_o, L.s_o, w.xq_c, sc[2:4], w.attn)
    q8.q8_layernorm_absmax(x_in, L.gamma[0], L.beta[0], w.h1, residual=w.attn, amax_slots=w.slots_h)
    q8.q8_linear_f32_slots(w.h1, w.slots_h, L.w_1, L.b_1, L.s_1, w.xq_h, sc[4:6], w.g, out_amax=w.g_amax,
                           flags=q8.EPI_GELU | q8.EPI_ABSMAX)
    q8.q8_linear_f32_slots(w.g, w.g_amax, L.w_2, L.b_2, L.s_2, w.xq_g, sc[6:8], w.out)
    q8.q8_layernorm_absmax(w.h1, L.gamma[1], L.beta[1], x_next, residual=w.out, amax_slots=slots_next)


def check_layer(L, w, x_in, x_next, B, S, mask=None):
    """Every stage against the oracle on the GPU's own input of that stage."""
    H = L.H
    x, qkv, ctx, attn, h1, g, out, xn = (host(t) for t in (x_in, w.qkv, w.ctx, w.attn, w.h1, w.g, w.out, x_next))
    sc = host(w.sc)
    # the four quantizers: scale = 127 / max|input| (Eq. 3), codes by Eq. 1
    for i, (src, codes) in enumerate(((x, w.xq_x), (ctx, w.xq_c), (h1, w.xq_h), (g, w.xq_g))):
        assert sc[2 * i] == O.absmax(src) and sc[2 * i + 1] == O.scale(O.absmax(src)), f"scale {i}"
        np.testing.assert_array_equal(host(codes), O.quantize(src, sc[2 * i + 1]), err_msg=f"codes {i}")
    r = O.linear(x, L.w_qkv_h, L.s_qkv_h, L.b_qkv_h, threads=THREADS)
    rel_close(qkv, r["y"], 1e-6, what="fused QKV")
    a = O.attention(qkv, B, S, L.heads, H // L.heads, mask=mask, threads=THREADS)
    assert np.abs(ctx.astype(np.float64) - a).max() <= 2e-6 * np.abs(qkv[:, 2 * H:]).max(), "attention"
    r = O.linear(ctx, L.w_o_h, L.s_o_h, L.b_o_h, threads=THREADS)
    rel_close(attn, r["y"], 1e-6, what="attention output")
    rel_close(h1, O.layernorm(x, L.gamma_h[0], L.beta_h[0], residual=attn), 1e-6, 2e-7, what="LayerNorm 1")
    r = O.linear(h1, L.w_1_h, L.s_1_h, L.b_1_h, act_gelu=True, threads=THREADS)
    rel_close(g, r["y"], 1e-5, 1e-6, what="FFN1 + GELU")
    assert host(w.g_amax)[0] == np.abs(g).max()
    r = O.linear(g, L.w_2_h, L.s_2_h, L.b_2_h, threads=THREADS)
    rel_close(out, r["y"], 1e-6, what="FFN2")
    rel_close(xn, O.layernorm(h1, L.gamma_h[1], L.beta_h[1], residual=out), 1e-6, 2e-7, what="LayerNorm 2")


def test_bert_base_encoder_layer_stagewise(q8):
    """BERT-Base encoder layer, batch 32 x seq 128, hidden 768, 12 heads, FFN 3072, with a padding mask."""
    d = synth.bert_base_layer(seed=2, batch=32, seq=128)
    B, S, H, F = d["batch"], d["seq"], d["hidden"], d["ffn"]
    M = B * S
    L = Layer(q8, d)
    w = Work(q8, M, H, F)
    g = synth.rng(31)
    mask = np.zeros((B, S), np.float32)
    for b in range(B):
        mask[b, int(g.integers(S // 2, S + 1)):] = -10000.0
    mask_d = dev(mask)
    # the layer input as a previous layer leaves it: a LayerNorm output with its abs-max slots
    x_in, slots_x = torch.empty((M, H), device="cuda"), torch.zeros(q8.AMAX_SLOTS, device="cuda")
    q8.q8_layernorm_absmax(dev(d["x"]), L.gamma[1], L.beta[1], x_in, amax_slots=slots_x)
    x_next, slots_next = torch.empty((M, H), device="cuda"), torch.zeros(q8.AMAX_SLOTS, device="cuda")
    gpu_layer(q8, L, w, x_in, slots_x, x_next, slots_next, B, S, mask=mask_d)
    torch.cuda.synchronize()
    check_layer(L, w, x_in, x_next, B, S, mask=mask)
    assert host(slots_next).max() == np.abs(host(x_next)).max()


def test_bert_large_encoder_layer_stagewise(q8):
    """The benchmark's shape: BERT-Large encoder layer, batch 32 x seq 384 = 12288 tokens, hidden 1024, 16 heads,
    FFN 4096, in the very chain bench.py times as its whole-layer step (each FC one q8_linear_f32_slots call fed by
    the abs-max slots of the FP32 kernel in front of it).  Every stage in full against the oracle: the four
    quantizers, the fused QKV, attention-output (12288 x 1024 x 1024), FFN1 + GELU and FFN2 GEMMs, the attention,
    and both residual + LayerNorm passes at 12288 x 1024."""
    d = synth.bert_large_layer(seed=3, batch=32, seq=384)
    B, S, H, F = d["batch"], d["seq"], d["hidden"], d["ffn"]
    M = B * S
    L = Layer(q8, d)
    w = Work(q8, M, H, F)
    x_in, slots_x = torch.empty((M, H), device="cuda"), torch.zeros(q8.AMAX_SLOTS, device="cuda")
    q8.q8_layernorm_absmax(dev(d["x"]), L.gamma[1], L.beta[1], x_in, amax_slots=slots_x)
    x_next, slots_next = torch.empty((M, H), device="cuda"), torch.zeros(q8.AMAX_SLOTS, device="cuda")
    gpu_layer(q8, L, w, x_in, slots_x, x_next, slots_next, B, S)
    torch.cuda.synchronize()
    check_layer(L, w, x_in, x_next, B, S)
    assert host(slots_next).max() == np.abs(host(x_next)).max()


def static_layer_stagewise(q8, d, B, S):
    """The stored-scale layer (Eq. 4) in the chain bench.py times as its stored-scale encoder layer: no quantize pass
    anywhere -- the attention kernel and both LayerNorms write the int8 codes the next FC reads, FFN1 writes int8
    through its GELU + requantize epilogue.  Every stage against the oracle on the GPU's own input of that stage; the
    stored scales are 127 / (0.9 max|.|) of a dynamic pass over the same data, so the clamp is exercised too."""
    H, F = d["hidden"], d["ffn"]
    M, heads = B * S, d["heads"]
    L = Layer(q8, d)
    w = Work(q8, M, H, F)
    x_in, slots_x = torch.empty((M, H), device="cuda"), torch.zeros(q8.AMAX_SLOTS, device="cuda")
    q8.q8_layernorm_absmax(dev(d["x"]), L.gamma[1], L.beta[1], x_in, amax_slots=slots_x)
    x_next, slots_next = torch.empty((M, H), device="cuda"), torch.zeros(q8.AMAX_SLOTS, device="cuda")
    gpu_layer(q8, L, w, x_in, slots_x, x_next, slots_next, B, S)            # calibration pass (dynamic scales)
    torch.cuda.synchronize()
    sh = (np.float32(127.0) / (np.float32(0.9) * host(w.sc)[0::2])).astype(np.float32)   # x, ctx, h1, gelu(ffn1)
    s = dev(sh)
    i8 = lambda *shape: torch.full(shape, 99, dtype=torch.int8, device="cuda")
    xq_x, xq_c, xq_c2, xq_h, gq, xq_n = i8(M, H), i8(M, H), i8(M, H), i8(M, H), i8(M, F), i8(M, H)
    g32 = torch.empty((M, F), device="cuda")
    q8.q8_quantize(x_in, s[0:1], xq_x)
    q8.q8_linear(xq_x, L.w_qkv, L.b_qkv, s[0:1], L.s_qkv, w.qkv, n_groups=3)
    q8.q8_attention(w.qkv, B, S, heads, H // heads, ctx=w.ctx, q_scale=s[1:2], q_out=xq_c)
    q8.q8_attention(w.qkv, B, S, heads, H // heads, q_scale=s[1:2], q_out=xq_c2)          # codes only, as the bench runs it
    q8.q8_linear(xq_c2, L.w_o, L.b_o, s[1:2], L.s_o, w.attn)
    q8.q8_layernorm_absmax(x_in, L.gamma[0], L.beta[0], w.h1, residual=w.attn, q_scale=s[2:3], q_out=xq_h)
    q8.q8_linear(xq_h, L.w_1, L.b_1, s[2:3], L.s_1, gq, next_scale=s[3:4], flags=q8.EPI_GELU | q8.EPI_REQUANT)
    q8.q8_linear(xq_h, L.w_1, L.b_1, s[2:3], L.s_1, g32, flags=q8.EPI_GELU)                # the fp32 values those codes stand for
    q8.q8_linear(gq, L.w_2, L.b_2, s[3:4], L.s_2, w.out)
    q8.q8_layernorm_absmax(w.h1, L.gamma[1], L.beta[1], x_next, residual=w.out, q_scale=s[0:1], q_out=xq_n)
    torch.cuda.synchronize()
    x, qkv, ctx, attn, h1, out, xn = (host(t) for t in (x_in, w.qkv, w.ctx, w.attn, w.h1, w.out, x_next))
    np.testing.assert_array_equal(host(xq_x), O.quantize(x, sh[0]))
    rel_close(qkv, O.linear(x, L.w_qkv_h, L.s_qkv_h, L.b_qkv_h, sx=sh[0], threads=THREADS)["y"], 1e-6, what="fused QKV")
    a = O.attention(qkv, B, S, heads, H // heads, threads=THREADS)
    assert np.abs(ctx.astype(np.float64) - a).max() <= 2e-6 * np.abs(qkv[:, 2 * H:]).max(), "attention"
    np.testing.assert_array_equal(host(xq_c), O.quantize(ctx, sh[1]))
    np.testing.assert_array_equal(host(xq_c2), host(xq_c))
    assert np.abs(host(xq_c)).max() == 127                                   # the stored scale saturates the tail
    rel_close(attn, O.linear(ctx, L.w_o_h, L.s_o_h, L.b_o_h, sx=sh[1], threads=THREADS)["y"], 1e-6, what="attention output")
    rel_close(h1, O.layernorm(x, L.gamma_h[0], L.beta_h[0], residual=attn), 1e-6, 2e-7, what="LayerNorm 1")
    np.testing.assert_array_equal(host(xq_h), O.quantize(h1, sh[2]))
    r1 = O.linear(h1, L.w_1_h, L.s_1_h, L.b_1_h, sx=sh[2], act_gelu=True, threads=THREADS)
    gh = host(g32)
    rel_close(gh, r1["y"], 1e-5, 1e-6, what="FFN1 + GELU")
    gqh = host(gq)
    np.testing.assert_array_equal(gqh, O.quantize(gh, sh[3]))               # codes of the GPU's own fp32 values
    dq = gqh.astype(np.int32) - O.quantize(r1["y"], sh[3]).astype(np.int32)  # against the oracle's: equal up to ties
    assert np.abs(dq).max() <= 1
    p = r1["y"].astype(np.float64) * float(sh[3])
    slack = float(sh[3]) * (1e-6 + 1e-5 * np.abs(r1["y"].astype(np.float64))) + 1e-6 * np.maximum(1.0, np.abs(p))
    assert np.all(np.abs(np.abs(p - np.trunc(p)) - 0.5)[dq != 0] <= slack[dq != 0])
    bq2 = O.quantize_bias(L.b_2_h, H, sh[3], np.array([L.s_2_h], np.float32))
    acc2 = O.gemm_i8(gqh, L.w_2_h, bq2, threads=THREADS)
    rel_close(out, O.dequant(acc2, sh[3], np.array([L.s_2_h], np.float32)), 1e-6, what="FFN2")
    rel_close(xn, O.layernorm(h1, L.gamma_h[1], L.beta_h[1], residual=out), 1e-6, 2e-7, what="LayerNorm 2")
    np.testing.assert_array_equal(host(xq_n), O.quantize(xn, sh[0]))
    # The same two sub-layers with the residual addition moved into the FC epilogue: the FC writes x + FC(ctx)
    # (one binary32 addition, as in the oracle's LayerNorm), the LayerNorm behind it reads that one tensor.
    sum1, sum2, h1_f, xn_f = (torch.empty((M, H), device="cuda") for _ in range(4))
    xq_hf, xq_nf = i8(M, H), i8(M, H)
    q8.q8_linear_residual(xq_c2, L.w_o, L.b_o, s[1:2], L.s_o, x_in, sum1)
    q8.q8_layernorm_absmax(sum1, L.gamma[0], L.beta[0], h1_f, q_scale=s[2:3], q_out=xq_hf)
    q8.q8_linear_residual(gq, L.w_2, L.b_2, s[3:4], L.s_2, w.h1, sum2)
    q8.q8_layernorm_absmax(sum2, L.gamma[1], L.beta[1], xn_f, q_scale=s[0:1], q_out=xq_nf)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(sum1), attn + x)
    np.testing.assert_array_equal(host(sum2), out + h1)
    rel_close(host(h1_f), O.layernorm(x, L.gamma_h[0], L.beta_h[0], residual=attn), 1e-6, 2e-7, what="LayerNorm 1 of the fused sum")
    np.testing.assert_array_equal(host(xq_hf), O.quantize(host(h1_f), sh[2]))
    rel_close(host(xn_f), O.layernorm(h1, L.gamma_h[1], L.beta_h[1], residual=out), 1e-6, 2e-7, what="LayerNorm 2 of the fused sum")
    np.testing.assert_array_equal(host(xq_nf), O.quantize(host(xn_f), sh[0]))


def test_bert_base_encoder_layer_stored_scales_stagewise(q8):
    static_layer_stagewise(q8, synth.bert_base_layer(seed=2, batch=32, seq=128), 32, 128)


def test_bert_large_encoder_layer_stored_scales_stagewise(q8):
    """The benchmark's stored-scale encoder layer at its own shape: 12288 tokens, hidden 1024, FFN 4096."""
    static_layer_stagewise(q8, synth.bert_large_layer(seed=3, batch=32, seq=384), 32, 384)


def test_bert_base_12_layer_forward(q8):
    """The full BERT-Base forward at batch 64 x seq 128: int8 embedding tables (30522 / 512 / 2 x 768) + LayerNorm,
    then 12 encoder layers, each with its own weights.  Layers 0, 5 and 11 are checked stage by stage against the
    oracle (on the activations the GPU chain really produced there); every layer's output must be finite and agree
    with the abs-max slots it hands on."""
    B, S, n_layers = 64, 128, 12
    M = B * S
    tabs = synth.embedding_tables(seed=5, hidden=768)
    ids = synth.token_ids(seed=6, batch=B, seq=S)
    tq = {k: O.quantize_tensor(tabs[k]) for k in ("word", "position", "token_type")}
    scales = np.array([tq[k][1] for k in ("word", "position", "token_type")], np.float32)
    wid, pid, tid = (ids[k].reshape(-1) for k in ("word", "position", "token_type"))
    g = synth.rng(41)
    gam, bet = (1 + 0.1 * g.standard_normal(768)).astype(np.float32), (0.1 * g.standard_normal(768)).astype(np.float32)
    x = [torch.empty((M, 768), device="cuda") for _ in range(2)]
    slots = [torch.zeros(q8.AMAX_SLOTS, device="cuda") for _ in range(2)]
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    q8.q8_embedding_sum3_layernorm(dev(tq["word"][0]), dev(tq["position"][0]), dev(tq["token_type"][0]), dev(scales),
                                   dev(wid), dev(pid), dev(tid), dev(gam), dev(bet), x[0], amax_slots=slots[0], err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    emb = O.embedding_sum3(tq["word"][0], scales[0], tq["position"][0], scales[1], tq["token_type"][0], scales[2], wid, pid, tid)
    rel_close(host(x[0]), O.layernorm(emb, gam, bet), 1e-6, 2e-7, what="embedding + LayerNorm")
    w = Work(q8, M, 768, 3072)
    for layer in range(n_layers):
        d = synth.bert_base_layer(seed=100 + layer, batch=1, seq=1)          # weights only
        L = Layer(q8, d)
        cur, nxt = x[layer & 1], x[(layer + 1) & 1]
        gpu_layer(q8, L, w, cur, slots[layer & 1], nxt, slots[(layer + 1) & 1], B, S)
        torch.cuda.synchronize()
        out = host(nxt)
        assert np.isfinite(out).all() and host(slots[(layer + 1) & 1]).max() == np.abs(out).max(), layer
        if layer in (0, 5, 11):
            check_layer(L, w, cur, nxt, B, S)
