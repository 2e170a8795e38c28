#!/usr/bin/env python3
"""Benchmark of the quantized fully-connected hot path on one MI355X.

One step = one pass of the whole hot path over one batch of the BERT-Large encoder-layer
workload (batch 32 x seq 384 = 12288 tokens, hidden 1024, FFN 4096):

    int8 embedding gather (word + position + type, fp32 out)                 -- secondary path
    for each FC of the layer (fused Q|K|V, attention-out, FFN1, FFN2):
        abs-max of the fp32 input -> S_x = 127/max -> quantize -> int8 MFMA GEMM with fused
        Int32 bias + dequantize (FFN1 also fuses GELU and the abs-max of its output, which
        feeds FFN2's scale)

All inputs are seeded synthetic tensors already resident in HBM when the timed region starts.
The fp32 glue between the FCs (attention, LayerNorm) is not part of the hot path: it is run
once, untimed, with PyTorch ops to give every FC an input of realistic distribution.

Prints ONE JSON line.  value = int8 tera-ops/s of the six FC GEMMs (2*M*N*K each) over the
whole step time (quantize passes and embedding included).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "int8 TOPS + % MFMA peak on BERT FC GEMMs; tokens/s per quantized BERT layer"
INT8_PEAK_TOPS = 5033.0      # MI355X published dense int8 matrix peak
FP32_PEAK_TFLOPS = 157.3    # MI355X published fp32 matrix peak
HBM_PEAK_GBS = 8000.0
PREWARM_STEPS = 200         # untimed steps in front of --warmup: the clock takes a few dozen launches to settle after idle
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_bert_large_layer_pmc_traffic.txt")


def profiled_traffic(key):
    """HBM-side bytes per launch of a kernel as the committed rocprofv3 --pmc summary recorded them (FETCH_SIZE and
    WRITE_SIZE runs, scaled on a copy of known size).  Counters cannot be read from inside this process, so the figure
    is the profile's, named as such in the JSON; None if the summary is missing or has no such line."""
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("traffic_bytes_per_launch " + key + " "):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--seq", type=int, default=384)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=12288)
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="after the timed region, copy a 256 MiB tensor three times (a kernel of known HBM traffic "
                         "against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled)")
    return ap.parse_args()


class Layer:
    """Device-resident quantized weights of one encoder layer plus work buffers."""

    def __init__(self, q8, torch, d, vocab_tables, ids):
        self.q8, self.torch = q8, torch
        dev = "cuda"
        self.batch, self.seq = d["batch"], d["seq"]
        self.M = d["batch"] * d["seq"]
        self.H, self.F, self.heads = d["hidden"], d["ffn"], d["heads"]
        M, H, F = self.M, self.H, self.F

        def up(a):
            return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

        def quant_weight(W):
            wd = up(W)
            a = torch.zeros(1, device=dev)
            s = torch.zeros(1, device=dev)
            q8.q8_absmax(wd, a, s)
            wq = torch.empty(W.shape, dtype=torch.int8, device=dev)
            q8.q8_quantize(wd, s, wq)
            return wq, s

        parts = [quant_weight(d["W" + n]) for n in ("q", "k", "v")]
        self.w_qkv = torch.cat([p[0] for p in parts], 0).contiguous()
        self.s_qkv = torch.cat([p[1] for p in parts]).contiguous()
        self.b_qkv = up(np.concatenate([d["bq"], d["bk"], d["bv"]]))
        self.w_o, self.s_o = quant_weight(d["Wo"])
        self.b_o = up(d["bo"])
        self.w_1, self.s_1 = quant_weight(d["W1"])
        self.b_1 = up(d["b1"])
        self.w_2, self.s_2 = quant_weight(d["W2"])
        self.b_2 = up(d["b2"])
        # embedding tables (int8) and ids
        tabs = [quant_weight(vocab_tables[k]) for k in ("word", "position", "token_type")]
        self.tables = [t[0] for t in tabs]
        self.table_scales = torch.cat([t[1] for t in tabs]).contiguous()
        self.ids = [up(ids[k]) for k in ("word", "position", "token_type")]
        self.emb = torch.empty((M, H), device=dev)
        self.err = torch.zeros(1, dtype=torch.int32, device=dev)
        # activations and work buffers
        self.x = up(d["x"])
        self.ctx = torch.empty((M, H), device=dev)
        self.h1 = torch.empty((M, H), device=dev)
        self.qkv = torch.empty((M, 3 * H), device=dev)
        self.attn_out = torch.empty((M, H), device=dev)
        self.g = torch.empty((M, F), device=dev)
        self.out = torch.empty((M, H), device=dev)
        self.xq = torch.empty(M * F, dtype=torch.int8, device=dev)
        self.scal = torch.zeros(q8.SCAL_WORK, device=dev)   # abs-max, S_x and partial maxima of the current FC
        self.gscal = torch.zeros(2, device=dev)             # abs-max of FFN1's output (fused epilogue) and its scale
        self.gemm_ops = 2.0 * M * (3 * H * H + H * H + 2 * H * F)
        self.events = None

    def _fc_dyn(self, x, K, wq, sw, b, y, n_groups=1, flags=0, out_amax=None):
        """Dynamic-quantization FC: the quantizer of Section 4.1 (one pass at these sizes: x stays in registers between the
        abs-max and the rounding), then the GEMM -- 2 launches."""
        M = self.M
        self.q8.q8_linear_f32(x, wq, b, sw, self.xq[: M * K], self.scal, y, n_groups=n_groups, out_amax=out_amax,
                              flags=flags)

    def step(self, ev=None):
        """The timed hot path.  ev: optional dict of (start, end) event pairs keyed "qkv", "attn_out", "ffn1", "ffn2",
        recorded around that FC's GEMM launch alone (each dynamic FC is the quantizer of Section 4.1 followed by the GEMM:
        the same launches q8_linear_f32 makes)."""
        q8 = self.q8
        M, H, F = self.M, self.H, self.F

        def gemm(name, *a, **kw):
            if ev is not None and name in ev:
                ev[name][0].record()
            q8.q8_linear(*a, **kw)
            if ev is not None and name in ev:
                ev[name][1].record()
        q8.q8_embedding_sum3(self.tables[0], self.tables[1], self.tables[2], self.table_scales, self.ids[0],
                             self.ids[1], self.ids[2], self.emb, err_flag=self.err)
        xq, sx = self.xq[: M * H].view(M, H), self.scal[1:2]
        q8.q8_quantize_dynamic(self.x, xq, self.scal)
        gemm("qkv", xq, self.w_qkv, self.b_qkv, sx, self.s_qkv, self.qkv, n_groups=3)
        q8.q8_quantize_dynamic(self.ctx, xq, self.scal)
        gemm("attn_out", xq, self.w_o, self.b_o, sx, self.s_o, self.attn_out)
        # FFN1: GELU and the abs-max of the GELU output come out of the GEMM epilogue (the quantizer clears the slot)
        g_amax, g_scale = self.gscal[0:1], self.gscal[1:2]
        q8.q8_quantize_dynamic(self.h1, xq, self.scal, zero_slot=g_amax)
        gemm("ffn1", xq, self.w_1, self.b_1, sx, self.s_1, self.g, out_amax=g_amax, flags=q8.EPI_GELU | q8.EPI_ABSMAX)
        # FFN2: S_x from the fused abs-max inside the quantize pass, then the GEMM
        xq = self.xq[: M * F].view(M, F)
        q8.q8_quantize_amax(self.g, g_amax, g_scale, xq)
        gemm("ffn2", xq, self.w_2, self.b_2, g_scale, self.s_2, self.out)

    def calibrate_static(self):
        """Stored activation scales for the static mode (Eq. 4 keeps such a scale from training; here the scale a
        dynamic pass over the same data gives)."""
        torch, q8 = self.torch, self.q8
        self.s_static = torch.zeros(4, device="cuda")      # x, ctx, h1, gelu(ffn1)
        tmp = torch.zeros(1, device="cuda")
        for i, t in enumerate((self.x, self.ctx, self.h1)):
            q8.q8_absmax(t, tmp, self.s_static[i:i + 1])
        self.step()                                         # leaves max|gelu(ffn1)| in gscal[0]
        q8.q8_scale_from_amax(self.gscal[0:1], self.s_static[3:4])
        self.gq = torch.empty((self.M, self.F), dtype=torch.int8, device="cuda")
        torch.cuda.synchronize()

    def step_static(self):
        """Same layer with stored activation scales: no abs-max passes, FFN1 writes int8 (GELU + requantize in the
        epilogue) and FFN2 reads it directly."""
        q8 = self.q8
        M, H, F = self.M, self.H, self.F
        s = self.s_static
        xq = self.xq[: M * H].view(M, H)
        q8.q8_embedding_sum3(self.tables[0], self.tables[1], self.tables[2], self.table_scales, self.ids[0],
                             self.ids[1], self.ids[2], self.emb, err_flag=self.err)
        q8.q8_quantize(self.x, s[0:1], xq)
        q8.q8_linear(xq, self.w_qkv, self.b_qkv, s[0:1], self.s_qkv, self.qkv, n_groups=3)
        q8.q8_quantize(self.ctx, s[1:2], xq)
        q8.q8_linear(xq, self.w_o, self.b_o, s[1:2], self.s_o, self.attn_out)
        q8.q8_quantize(self.h1, s[2:3], xq)
        q8.q8_linear(xq, self.w_1, self.b_1, s[2:3], self.s_1, self.gq, next_scale=s[3:4],
                     flags=q8.EPI_GELU | q8.EPI_REQUANT)
        q8.q8_linear(self.gq, self.w_2, self.b_2, s[3:4], self.s_2, self.out)

    def step_fused(self):
        """Dynamic quantization with the FP32 glue around the FCs fused (not part of the headline step): the
        embedding block and both LayerNorms of the layer run in the library and hand the abs-max of their
        output to the quantizer of the FC that follows, so QKV and FFN1 need no abs-max pass."""
        q8 = self.q8
        M, H, F = self.M, self.H, self.F
        if not hasattr(self, "ln_g"):
            torch = self.torch
            self.ln_g, self.ln_b = torch.ones(H, device="cuda"), torch.zeros(H, device="cuda")
            self.slots_x = torch.zeros(q8.AMAX_SLOTS, device="cuda")
            self.slots_h = torch.zeros(q8.AMAX_SLOTS, device="cuda")
            self.slots_e = torch.zeros(q8.AMAX_SLOTS, device="cuda")
            self.x_next = torch.empty((M, H), device="cuda")
            self.h1f = torch.empty((M, H), device="cuda")
            # abs-max slots of the layer input, as the previous layer's last LayerNorm would have left them
            q8.q8_layernorm_absmax(self.x, self.ln_g, self.ln_b, self.x_next, amax_slots=self.slots_x)
            self.x_in = self.x_next.clone()
        sc = self.scal[0:2]
        q8.q8_embedding_sum3_layernorm(self.tables[0], self.tables[1], self.tables[2], self.table_scales, self.ids[0],
                                       self.ids[1], self.ids[2], self.ln_g, self.ln_b, self.emb, amax_slots=self.slots_e,
                                       err_flag=self.err)
        xq = self.xq[: M * H]
        # QKV: slots from the LayerNorm
        q8.q8_linear_f32_slots(self.x_in, self.slots_x, self.w_qkv, self.b_qkv, self.s_qkv, xq, sc, self.qkv, n_groups=3)
        self._fc_dyn(self.ctx, H, self.w_o, self.s_o, self.b_o, self.attn_out)      # attention output: no LayerNorm in front
        q8.q8_layernorm_absmax(self.x_in, self.ln_g, self.ln_b, self.h1f, residual=self.attn_out, amax_slots=self.slots_h)
        g_amax = self.gscal[0:1]
        q8.q8_linear_f32_slots(self.h1f, self.slots_h, self.w_1, self.b_1, self.s_1, xq, sc, self.g, out_amax=g_amax,
                               flags=q8.EPI_GELU | q8.EPI_ABSMAX)                    # FFN1: slots from the LayerNorm
        q8.q8_linear_f32_slots(self.g, g_amax, self.w_2, self.b_2, self.s_2, self.xq[: M * F], sc, self.out)
        q8.q8_layernorm_absmax(self.h1f, self.ln_g, self.ln_b, self.x_next, residual=self.out, amax_slots=self.slots_x)

    def step_fused_static(self):
        """Stored activation scales with the FP32 glue fused: each LayerNorm (and the embedding block) also writes
        the int8 codes of its output, so QKV and FFN1 have no quantize pass at all.  Call step_fused() once first."""
        q8 = self.q8
        M, H, F = self.M, self.H, self.F
        s = self.s_static
        if not hasattr(self, "xq_x"):
            torch = self.torch
            self.xq_x = torch.empty((M, H), dtype=torch.int8, device="cuda")     # codes of the layer input (previous LayerNorm)
            self.xq_h = torch.empty((M, H), dtype=torch.int8, device="cuda")
            self.xq_e = torch.empty((M, H), dtype=torch.int8, device="cuda")
            q8.q8_quantize(self.x_in, s[0:1], self.xq_x)
        q8.q8_embedding_sum3_layernorm(self.tables[0], self.tables[1], self.tables[2], self.table_scales, self.ids[0],
                                       self.ids[1], self.ids[2], self.ln_g, self.ln_b, self.emb, q_scale=s[0:1],
                                       q_out=self.xq_e, err_flag=self.err)
        q8.q8_linear(self.xq_x, self.w_qkv, self.b_qkv, s[0:1], self.s_qkv, self.qkv, n_groups=3)
        xq = self.xq[: M * H].view(M, H)
        q8.q8_quantize(self.ctx, s[1:2], xq)
        q8.q8_linear(xq, self.w_o, self.b_o, s[1:2], self.s_o, self.attn_out)
        q8.q8_layernorm_absmax(self.x_in, self.ln_g, self.ln_b, self.h1f, residual=self.attn_out, q_scale=s[2:3], q_out=self.xq_h)
        q8.q8_linear(self.xq_h, self.w_1, self.b_1, s[2:3], self.s_1, self.gq, next_scale=s[3:4],
                     flags=q8.EPI_GELU | q8.EPI_REQUANT)
        q8.q8_linear(self.gq, self.w_2, self.b_2, s[3:4], self.s_2, self.out)
        q8.q8_layernorm_absmax(self.h1f, self.ln_g, self.ln_b, self.x_next, residual=self.out, q_scale=s[0:1], q_out=self.xq_x)

    def step_layer(self, ev=None):
        """One whole encoder layer on dynamic scales, every operation in the library: QKV FC, FP32 softmax attention,
        attention-output FC, residual + LayerNorm, FFN1 (GELU), FFN2, residual + LayerNorm.  Each FP32 operation hands
        the abs-max of its output to the quantizer of the FC behind it.  Call step_fused() once first (buffers).
        ev: optional (start, end) event pair recorded around the attention kernel."""
        q8 = self.q8
        M, H, F = self.M, self.H, self.F
        if not hasattr(self, "slots_c"):
            self.slots_c = self.torch.zeros(q8.AMAX_SLOTS, device="cuda")
            self.slots_o = self.torch.zeros(q8.AMAX_SLOTS, device="cuda")
            self.ctx_l = self.torch.empty((M, H), device="cuda")
        sc = self.scal[0:2]                                          # max|x| and S_x of the current FC
        xq = self.xq[: M * H]
        q8.q8_linear_f32_slots(self.x_in, self.slots_x, self.w_qkv, self.b_qkv, self.s_qkv, xq, sc, self.qkv, n_groups=3)
        if ev is not None:
            ev[0].record()
        q8.q8_attention(self.qkv, self.batch, self.seq, self.heads, H // self.heads, ctx=self.ctx_l, amax_slots=self.slots_c)
        if ev is not None:
            ev[1].record()
        q8.q8_linear_f32_slots(self.ctx_l, self.slots_c, self.w_o, self.b_o, self.s_o, xq, sc, self.attn_out)
        q8.q8_layernorm_absmax(self.x_in, self.ln_g, self.ln_b, self.h1f, residual=self.attn_out, amax_slots=self.slots_h)
        g_amax = self.gscal[0:1]                                      # reset by the call whose epilogue fills it
        q8.q8_linear_f32_slots(self.h1f, self.slots_h, self.w_1, self.b_1, self.s_1, xq, sc, self.g, out_amax=g_amax,
                               flags=q8.EPI_GELU | q8.EPI_ABSMAX)
        q8.q8_linear_f32_slots(self.g, g_amax, self.w_2, self.b_2, self.s_2, self.xq[: M * F], sc, self.out)
        q8.q8_layernorm_absmax(self.h1f, self.ln_g, self.ln_b, self.x_next, residual=self.out, amax_slots=self.slots_o)

    def step_layer_static(self):
        """The whole encoder layer on stored scales (Eq. 4): seven kernels, no quantize pass anywhere -- both LayerNorms
        and the attention kernel write the int8 codes the next FC reads, FFN1 writes int8 through its epilogue.
        Call step_fused_static() and step_layer() once first (buffers)."""
        q8 = self.q8
        H = self.H
        s = self.s_static
        if not hasattr(self, "xq_c"):
            self.xq_c = self.torch.empty((self.M, H), dtype=self.torch.int8, device="cuda")
            self.xq_n = self.torch.empty((self.M, H), dtype=self.torch.int8, device="cuda")
        q8.q8_linear(self.xq_x, self.w_qkv, self.b_qkv, s[0:1], self.s_qkv, self.qkv, n_groups=3)
        q8.q8_attention(self.qkv, self.batch, self.seq, self.heads, H // self.heads, q_scale=s[1:2], q_out=self.xq_c)
        q8.q8_linear(self.xq_c, self.w_o, self.b_o, s[1:2], self.s_o, self.attn_out)
        q8.q8_layernorm_absmax(self.x_in, self.ln_g, self.ln_b, self.h1f, residual=self.attn_out, q_scale=s[2:3], q_out=self.xq_h)
        q8.q8_linear(self.xq_h, self.w_1, self.b_1, s[2:3], self.s_1, self.gq, next_scale=s[3:4],
                     flags=q8.EPI_GELU | q8.EPI_REQUANT)
        q8.q8_linear(self.gq, self.w_2, self.b_2, s[3:4], self.s_2, self.out)
        q8.q8_layernorm_absmax(self.h1f, self.ln_g, self.ln_b, self.x_next, residual=self.out, q_scale=s[0:1], q_out=self.xq_n)

    def step_layer_static_residual_in_fc(self):
        """step_layer_static with the two residual additions moved from the LayerNorm kernels into the epilogues of the
        attention-output FC and FFN2 (q8_linear_residual): same traffic, the FC reads the second operand instead."""
        q8 = self.q8
        H = self.H
        s = self.s_static
        q8.q8_linear(self.xq_x, self.w_qkv, self.b_qkv, s[0:1], self.s_qkv, self.qkv, n_groups=3)
        q8.q8_attention(self.qkv, self.batch, self.seq, self.heads, H // self.heads, q_scale=s[1:2], q_out=self.xq_c)
        q8.q8_linear_residual(self.xq_c, self.w_o, self.b_o, s[1:2], self.s_o, self.x_in, self.attn_out)
        q8.q8_layernorm_absmax(self.attn_out, self.ln_g, self.ln_b, self.h1f, q_scale=s[2:3], q_out=self.xq_h)
        q8.q8_linear(self.xq_h, self.w_1, self.b_1, s[2:3], self.s_1, self.gq, next_scale=s[3:4],
                     flags=q8.EPI_GELU | q8.EPI_REQUANT)
        q8.q8_linear_residual(self.gq, self.w_2, self.b_2, s[3:4], self.s_2, self.h1f, self.out)
        q8.q8_layernorm_absmax(self.out, self.ln_g, self.ln_b, self.x_next, q_scale=s[0:1], q_out=self.xq_n)

    def glue_once(self):
        """Untimed fp32 glue (attention, residual, LayerNorm) so every FC sees realistic inputs."""
        torch = self.torch
        F_ = torch.nn.functional
        M, H = self.M, self.H
        self._fc_dyn(self.x, H, self.w_qkv, self.s_qkv, self.b_qkv, self.qkv, n_groups=3)
        B, S = self.batch, self.seq
        hd = H // self.heads
        q, k, v = (t.reshape(B, S, self.heads, hd).transpose(1, 2) for t in self.qkv.split(H, dim=1))
        ctx = F_.scaled_dot_product_attention(q, k, v)
        self.ctx.copy_(ctx.transpose(1, 2).reshape(M, H))
        self._fc_dyn(self.ctx, H, self.w_o, self.s_o, self.b_o, self.attn_out)
        self.h1.copy_(F_.layer_norm(self.x + self.attn_out, (H,), eps=1e-12))
        torch.cuda.synchronize()


def cpu_baseline(d, sample_tokens):
    """The CPU oracle, as it stands, on the first `sample_tokens` tokens of the same workload."""
    from oracle import q8_oracle as O
    threads = min(os.cpu_count() or 1, 16)
    M = sample_tokens
    x = d["x"][:M]
    g = np.random.default_rng(99)
    ctx = g.standard_normal((M, d["hidden"]), dtype=np.float32)
    h1 = g.standard_normal((M, d["hidden"]), dtype=np.float32)
    ws = {n: O.quantize_tensor(d["W" + n]) for n in ("q", "k", "v", "o", "1", "2")}   # offline, untimed
    t0 = time.perf_counter()
    for n in ("q", "k", "v"):
        O.linear(x, ws[n][0], ws[n][1], d["b" + n], threads=threads)
    O.linear(ctx, ws["o"][0], ws["o"][1], d["bo"], threads=threads)
    f1 = O.linear(h1, ws["1"][0], ws["1"][1], d["b1"], act_gelu=True, threads=threads)
    O.linear(f1["y"], ws["2"][0], ws["2"][1], d["b2"], threads=threads)
    dt = time.perf_counter() - t0
    H, F = d["hidden"], d["ffn"]
    ops = 2.0 * M * (4 * H * H + 2 * H * F)
    return dict(value=ops / dt / 1e12, unit="int8 TOPS", cores=threads, kind="oracle",
                sample=f"all six FC layers (abs-max, quantize, int8 GEMM, dequantize, GELU) of the same layer on the "
                       f"first {M} of {d['batch'] * d['seq']} tokens; {dt:.2f} s wall",
                tokens_per_s=M / dt)


def gemm_bound(M, N, K, out_bytes):
    """Roofline of one FC GEMM from its algorithmic work: int8 ops 2 M N K against the published matrix peak, bytes
    M K + N K + out_bytes M N + 4 N (codes, weights, output, bias) against the published HBM rate."""
    ops = 2.0 * M * N * K
    nbytes = float(M * K + N * K + out_bytes * M * N + 4 * N)
    t_mfma, t_hbm = ops / (INT8_PEAK_TOPS * 1e12), nbytes / (HBM_PEAK_GBS * 1e9)
    return dict(ops=ops, bytes=nbytes, bound="mfma" if t_mfma >= t_hbm else "hbm", bound_us=max(t_mfma, t_hbm) * 1e6)


def timed(torch, fn, n, warm):
    """Mean wall time of fn() in seconds over n calls after warm untimed ones, bracketed by synchronisations."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / n


def event_us(torch, fn, reps, warm=3):
    """Mean duration of fn(i) in microseconds between two events on the launch stream."""
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(reps):
        fn(i)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / reps


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from paper_1910_06188_amd import q8, synth

    d = synth.bert_large_layer(seed=3, batch=args.batch, seq=args.seq)
    tables = synth.embedding_tables(seed=5, hidden=d["hidden"])
    ids = synth.token_ids(seed=6, batch=args.batch, seq=args.seq)
    layer = Layer(q8, torch, d, tables, ids)
    layer.glue_once()
    M, H, F = layer.M, layer.H, layer.F

    # What a HIP event pair adds to the kernel it brackets (the launch behind the first event waits for that event's
    # marker, and the second event's marker waits for the kernel): pairs around one and around two launches of a
    # one-thread kernel give t1 = o + k and t2 = o + 2k, so the overhead is o = 2 t1 - t2.  It is subtracted from every
    # event-bracketed kernel time below; both the raw and the net figure are reported.
    def event_overhead_us():
        tiny_a, tiny_s = torch.ones(1, device="cuda"), torch.zeros(1, device="cuda")
        res = []
        for n in (1, 2):
            pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
            for a_, b_ in pairs:
                layer.step()                         # the same surroundings as in the timed steps: a busy queue in front
                a_.record()
                for _ in range(n):
                    q8.q8_scale_from_amax(tiny_a, tiny_s)
                b_.record()
            torch.cuda.synchronize()
            res.append(float(np.median([a_.elapsed_time(b_) for a_, b_ in pairs])) * 1e3)
        return max(0.0, 2.0 * res[0] - res[1])

    # ---- the timed region: K steps of the dynamic-quantization hot path -------------------------------------------------
    for _ in range(PREWARM_STEPS + args.warmup):
        layer.step()
    torch.cuda.synchronize()
    evs = [{"ffn1": (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))} for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        layer.step(evs[i])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert int(layer.err.item()) == 0
    if args.pmc_calibration:
        src = torch.ones(64 * 1024 * 1024, device="cuda")       # 256 MiB of fp32
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    ms_per_step = dt / args.steps * 1e3
    tops = layer.gemm_ops / (dt / args.steps) / 1e12
    tokens_per_s = M / (dt / args.steps)
    # the step's longest kernel: the FFN1 GEMM with GELU + abs-max epilogue (12288 x 4096 x 1024, 201 MB of fp32 out),
    # bound by its HBM write; timed with events on the launch stream around that launch in every timed step
    shapes = {"qkv": ("fused QKV", 3 * H, H, 4), "attn_out": ("attention-output", H, H, 4),
              "ffn1": ("FFN1 + GELU + abs-max", F, H, 4), "ffn2": ("FFN2", H, F, 4)}
    ev_over = event_overhead_us()
    ffn1_raw_us = float(np.mean([e["ffn1"][0].elapsed_time(e["ffn1"][1]) for e in evs])) * 1e3
    ffn1_us = ffn1_raw_us - ev_over
    rb = gemm_bound(M, F, H, 4)
    ffn1_gbs = rb["bytes"] / (ffn1_us * 1e-6) / 1e9
    default_shape = (args.batch, args.seq) == (32, 384)
    out = {
        "metric": METRIC, "value": round(tops, 2), "unit": "int8 TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "i8", "data": "synthetic",
        "config": {"workload": "BERT-Large encoder layer, batch %d x seq %d (BASELINE configs[3]): six quantized FC "
                               "layers (fused QKV, attn-out, FFN1+GELU, FFN2) with dynamic per-tensor scales, plus "
                               "the int8 3-table embedding gather" % (args.batch, args.seq),
                   "tokens": M, "hidden": H, "ffn": F, "fp32_glue_timed": False, "prewarm_steps": PREWARM_STEPS},
        "tokens_per_s": round(tokens_per_s, 1),
        "pct_int8_mfma_peak_whole_step": round(100.0 * tops / INT8_PEAK_TOPS, 2),
        "roofline": {"bound": "hbm", "kernel": "gemm_mfma_kernel, FFN1 %dx%dx%d + GELU + abs-max, fp32 out (the step's longest kernel)" % (M, F, H),
                     "achieved": round(ffn1_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(ffn1_gbs / HBM_PEAK_GBS, 4), "avg_launch_us": round(ffn1_us, 2),
                     "avg_event_pair_us": round(ffn1_raw_us, 2), "event_pair_overhead_us": round(ev_over, 2),
                     "algorithmic_bytes": rb["bytes"], "int8_tops": round(rb["ops"] / ffn1_us / 1e6, 1),
                     "pct_int8_mfma_peak": round(100.0 * rb["ops"] / ffn1_us / 1e6 / INT8_PEAK_TOPS, 2),
                     "traffic": profiled_traffic("FFN1_GELU_ABSMAX") if default_shape else None,
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary under profiles/ (not measured in this run)"},
    }
    # ---- every FC GEMM of the step against its own roofline: a second pass of steps with events around all four ---------
    n_pg = max(10, min(args.steps, 200))
    pevs = [{k: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for k in shapes} for _ in range(n_pg)]
    for i in range(n_pg):
        layer.step(pevs[i])
    torch.cuda.synchronize()
    per_gemm = {}
    for k, (label, N_, K_, ob) in shapes.items():
        us = float(np.mean([e[k][0].elapsed_time(e[k][1]) for e in pevs])) * 1e3 - ev_over
        b = gemm_bound(M, N_, K_, ob)
        per_gemm[label + " %dx%dx%d" % (M, N_, K_)] = {
            "us": round(us, 2), "bound": b["bound"], "bound_us": round(b["bound_us"], 2), "frac_of_roofline": round(b["bound_us"] / us, 4),
            "int8_tops": round(b["ops"] / us / 1e6, 1), "pct_int8_mfma_peak": round(100.0 * b["ops"] / us / 1e6 / INT8_PEAK_TOPS, 2),
            "algorithmic_GBps": round(b["bytes"] / us / 1e3, 1)}
    out["per_gemm"] = per_gemm
    # ---- what the chip itself sustains, measured in this run: the matrix pipes on register-resident operands (no memory
    # traffic; Gaussian codes as the layer's, and all-zero ones) and the HBM on streaming passes larger than every cache --------
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    gauss = torch.clamp(torch.round(torch.randn(65536, device="cuda") * 25.0), -127, 127).to(torch.int8)
    zeros = torch.zeros(65536, dtype=torch.int8, device="cuda")
    ceil = {}
    for name, ops_t in (("gaussian_codes", gauss), ("zero_codes", zeros)):
        n_ops = [0.0]

        def run(i, ops_t=ops_t):
            n_ops[0] = q8.debug_mfma_rate(ops_t, 8000, 256, sink)
        us = event_us(torch, run, 10)
        ceil["mfma_i8_register_resident_" + name] = {"int8_tops": round(n_ops[0] / us / 1e6, 1),
                                                     "frac_of_published_peak": round(n_ops[0] / us / 1e6 / INT8_PEAK_TOPS, 4)}
    big = [torch.empty(M * F, device="cuda") for _ in range(5)]          # 5 x 201 MB: beyond the 256 MB Infinity Cache
    for t in big:
        t.normal_()
    nb = big[0].numel() * 4
    us = event_us(torch, lambda i: q8.debug_stream_copy(big[i % 5], big[(i + 1) % 5]), 20)
    ceil["hbm_stream_copy_201MB"] = {"us": round(us, 1), "GBps_read_plus_write": round(2.0 * nb / us / 1e3, 1), "frac_of_8TBps": round(2.0 * nb / us / 1e3 / HBM_PEAK_GBS, 3)}
    us = event_us(torch, lambda i: q8.debug_stream_copy(None, big[i % 5]), 20)
    ceil["hbm_stream_fill_201MB"] = {"us": round(us, 1), "GBps_write": round(nb / us / 1e3, 1), "frac_of_8TBps": round(nb / us / 1e3 / HBM_PEAK_GBS, 3)}
    # one stage of a GEMM main loop (256 x 128 tile, 8 waves, 16 MFMAs per wave) piece by piece, zero operands: what the
    # loop's structure costs when the 48 KiB of operand loads and the 16 KiB of fp32 stores of a K = 1024 tile share the
    # compute unit's vector-memory path with it (64 KiB per stage = 64 B/clk at the matrix pipes' full rate)
    opw, stw = torch.zeros(4 << 20, dtype=torch.int8, device="cuda"), torch.empty(8 << 20, device="cuda")
    probe = {}
    for what, label in ((0, "mfma_only"), (7, "plus_lds_reads_barrier_operand_loads"), (15, "plus_fp32_stores"),
                        (64, "mfma_plus_gelu_arithmetic"), (71, "loads_and_gelu_arithmetic"), (79, "loads_gelu_and_stores")):
        us = event_us(torch, lambda i, what=what: q8.debug_loop_probe(what, opw, stw, 2400, sink), 5, warm=2)
        probe[label] = round(us * 1e3 / 2400, 1)
    ceil["gemm_stage_probe_ns_per_stage"] = probe
    del opw, stw
    out["measured_ceilings"] = ceil
    # The FFN2 launch on constant operands (every code 1): identical instruction stream and traffic, far fewer bits toggling
    # in the multipliers.  The gap to its per_gemm figure is the chip's power management, not the kernel's structure.
    xq1 = torch.ones((M, F), dtype=torch.int8, device="cuda")
    w1c = torch.ones((H, F), dtype=torch.int8, device="cuda")
    cs = torch.ones(2, device="cuda")
    const_us = event_us(torch, lambda i: q8.q8_linear(xq1, w1c, layer.b_2, cs[0:1], cs[1:2], layer.out), 50, warm=10)
    ffn2_ops = 2.0 * M * H * F
    out["ffn2_constant_operands"] = {"us": round(const_us, 2), "int8_tops": round(ffn2_ops / const_us / 1e6, 1),
                                     "pct_int8_mfma_peak": round(100.0 * ffn2_ops / const_us / 1e6 / INT8_PEAK_TOPS, 2)}
    del xq1, w1c
    # ---- the paper's own inference mode (stored activation scales, Eq. 4), reported beside the headline ---------------------
    layer.calibrate_static()
    n_static = max(50, args.steps // 4)   # at least 50: the synchronisation at both ends weighs on shorter runs
    n_warm = max(20, args.warmup // 4)
    dts = timed(torch, layer.step_static, n_static, n_warm)
    out["static_scale_mode"] = {"ms_per_step": round(dts * 1e3, 4), "int8_tops": round(layer.gemm_ops / dts / 1e12, 2),
                                "tokens_per_s": round(M / dts, 1), "steps": n_static,
                                "note": "stored activation scales: no abs-max passes; FFN1 emits int8 (GELU + "
                                        "requantize epilogue) straight into FFN2"}
    dtf = timed(torch, layer.step_fused, n_static, n_warm)
    out["fused_layernorm_mode"] = {"ms_per_step": round(dtf * 1e3, 4), "tokens_per_s": round(M / dtf, 1), "steps": n_static,
                                   "note": "dynamic scales; adds embedding+LayerNorm and the layer's two residual+LayerNorm "
                                           "passes to the step and drops the abs-max passes of QKV and FFN1 (their abs-max "
                                           "comes out of the LayerNorm kernels)"}
    dtfs = timed(torch, layer.step_fused_static, n_static, n_warm)
    out["fused_layernorm_static_mode"] = {"ms_per_step": round(dtfs * 1e3, 4), "tokens_per_s": round(M / dtfs, 1), "steps": n_static,
                                          "note": "stored scales; the embedding block and both residual+LayerNorm passes also "
                                                  "write the int8 codes of their output, so QKV and FFN1 have no quantize pass"}
    # the whole encoder layer, FP32 softmax attention included (fp32 matrix pipes: 4 S^2 d flops per head), every
    # operation in the library -- the layer-level tokens/s; the attention kernel is timed with events inside the step
    for _ in range(n_warm):
        layer.step_layer()
    torch.cuda.synchronize()
    aev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_static)]
    t0 = time.perf_counter()
    for i in range(n_static):
        layer.step_layer(aev[i])
    torch.cuda.synchronize()
    dtl = (time.perf_counter() - t0) / n_static
    attn_ms = sum(a.elapsed_time(b) for a, b in aev) / n_static
    attn_flops = 4.0 * layer.batch * layer.heads * layer.seq * layer.seq * (H // layer.heads)
    out["encoder_layer_mode"] = {"ms_per_step": round(dtl * 1e3, 4), "tokens_per_s": round(M / dtl, 1), "steps": n_static,
                                 "attention": {"avg_launch_us": round(attn_ms * 1e3, 2), "dtype": "f32",
                                               "achieved_tflops": round(attn_flops / (attn_ms * 1e-3) / 1e12, 1),
                                               "frac_of_fp32_mfma_peak": round(attn_flops / (attn_ms * 1e-3) / 1e12 / FP32_PEAK_TFLOPS, 4)},
                                 "note": "dynamic scales; QKV FC, FP32 softmax attention, attention-output FC, residual + "
                                         "LayerNorm, FFN1 + GELU, FFN2, residual + LayerNorm; no embedding block"}
    dtls = timed(torch, layer.step_layer_static, n_static, n_warm)
    out["encoder_layer_static_mode"] = {"ms_per_step": round(dtls * 1e3, 4), "tokens_per_s": round(M / dtls, 1), "steps": n_static,
                                        "note": "stored scales; seven kernels: the attention kernel and both LayerNorms write the "
                                                "int8 codes the next FC reads, FFN1 writes int8 through its epilogue"}
    dtlr = timed(torch, layer.step_layer_static_residual_in_fc, n_static, n_warm)
    out["encoder_layer_static_mode"]["residual_added_in_fc_epilogue_ms_per_step"] = round(dtlr * 1e3, 4)

    # ---- the two FFN GEMMs on their own, launched back to back: once on one set of buffers (operands and output stay in
    # the caches) and once rotating through sets that together exceed the 256 MB Infinity Cache
    def gemm_alone(N, K, flags, int8_out):
        per_set = M * K + N * K + (1 if int8_out else 4) * M * N
        R = int(1.0e9 // per_set) + 2
        sets = [(torch.randint(-127, 128, (M, K), dtype=torch.int8, device="cuda"),
                 torch.randint(-127, 128, (N, K), dtype=torch.int8, device="cuda"),
                 torch.empty((M, N), dtype=torch.int8 if int8_out else torch.float32, device="cuda")) for _ in range(R)]
        bb = torch.zeros(N, device="cuda")
        scl = torch.tensor([24.0, 1200.0, 20.0, 0.0], device="cuda")
        res = {}
        for mode in ("cache_warm", "rotating"):
            def launch(i):
                xq_, wq_, y_ = sets[i % R] if mode == "rotating" else sets[0]
                q8.q8_linear(xq_, wq_, bb, scl[0:1], scl[1:2], y_, out_amax=scl[3:4] if flags & 2 else None,
                             next_scale=scl[2:3] if flags & 4 else None, flags=flags)
            us = event_us(torch, launch, 4 * R, warm=R + 2)
            res[mode] = {"us": round(us, 1), "int8_tops": round(2.0 * M * N * K / us / 1e6, 1)}
        return res
    out["gemm_alone"] = {
        "FFN2 12288x1024x4096 fp32 out": gemm_alone(H, F, 0, False),
        "FFN1 12288x4096x1024 fp32 out": gemm_alone(F, H, 0, False),
        "FFN1 12288x4096x1024 GELU + requantize, int8 out": gemm_alone(F, H, 5, True),
    }
    # ---- the memory-bound kernels on their own, each launch on a different 201 MB (or 50 MB) tensor of a set larger than
    # the 256 MB Infinity Cache, so the rates are the HBM's: achieved algorithmic bytes/s against the published 8 TB/s
    def hbm_rate(fn, nbytes, reps=20):
        us = event_us(torch, fn, reps)
        return {"us_per_call": round(us, 1), "GBps": round(nbytes / us / 1e3, 1), "frac_of_8TBps": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 3)}
    nbig = M * F
    xq_big = layer.xq[:nbig]
    mid = [torch.randn((M, H), device="cuda") for _ in range(12)]         # 12 x 50 MB
    mid_out = [torch.empty((M, H), device="cuda") for _ in range(6)]
    out["hbm_kernels"] = {
        "q8_absmax fp32[12288,4096] (4 B/elt; 3 launches)": hbm_rate(lambda i: q8.q8_absmax(big[i % 5], layer.gscal[0:1], layer.gscal[1:2]), 4.0 * nbig),
        "q8_quantize fp32[12288,4096] (5 B/elt)": hbm_rate(lambda i: q8.q8_quantize(big[i % 5], layer.gscal[1:2], xq_big), 5.0 * nbig),
        "q8_quantize_dynamic fp32[12288,1024], one pass with x held in registers (5 B/elt; 1 launch)": hbm_rate(
            lambda i: q8.q8_quantize_dynamic(mid[i % 12], layer.xq[: M * H], layer.scal), 5.0 * M * H),
        "q8_embedding_sum3 12288 tokens x 1024 (3 int8 rows in, fp32 row out)": hbm_rate(
            lambda i: q8.q8_embedding_sum3(layer.tables[0], layer.tables[1], layer.tables[2], layer.table_scales, layer.ids[0],
                                           layer.ids[1], layer.ids[2], mid_out[i % 6], err_flag=layer.err), M * (3.0 * H + 12 + 4.0 * H)),
        "q8_layernorm_absmax fp32[12288,1024] + residual (12 B/elt)": hbm_rate(
            lambda i: q8.q8_layernorm_absmax(mid[i % 12], layer.ln_g, layer.ln_b, mid_out[i % 6], residual=mid[(i + 5) % 12], amax_slots=layer.slots_h),
            12.0 * M * H),
        "note": "every launch reads a tensor no earlier launch of the loop left in the 256 MB Infinity Cache",
    }
    q8.set_quantize_one_pass(False)
    out["hbm_kernels"]["q8_quantize_dynamic fp32[12288,1024], two passes (9 B/elt; 2 launches; what larger tensors and captured graphs take)"] = hbm_rate(
        lambda i: q8.q8_quantize_dynamic(mid[i % 12], layer.xq[: M * H], layer.scal), 9.0 * M * H)
    q8.set_quantize_one_pass(True)
    del mid, mid_out
    # training-side quantizer (Section 2.2 / Eq. 4): abs-max, moving-average step and fake quantization
    # of the FFN2-input-sized activation; bound by HBM (4 B read for the abs-max, 4 B + 4 B for the rest)
    ema_state = torch.zeros(2, device="cuda")
    us = event_us(torch, lambda i: q8.q8_fake_quantize_ema(big[i % 4], 0.9, ema_state, layer.scal, big[4]), 12)
    out["training_side"] = {"op": "q8_fake_quantize_ema on fp32[%d, %d]" % (M, F), "us_per_call": round(us, 1),
                            "algorithmic_GBps": round(12.0 * nbig / us / 1e3, 1), "bound": "hbm",
                            "frac_of_8TBps": round(12.0 * nbig / us / 1e3 / HBM_PEAK_GBS, 3)}
    del big
    # ---- the other BASELINE configurations, driver-visible: C1 one FC at 16 tokens, C3 one BERT-Base encoder layer at
    # 32 x 128 tokens, C5 the 12-layer BERT-Base forward at 64 x 128 tokens with its int8 embedding block (dynamic scales,
    # every operation in the library; the 12 layers reuse one set of weights, which does not change the work)
    c1 = synth.single_fc(0)
    x1 = torch.from_numpy(c1["x"]).cuda()
    w1q = torch.empty((768, 768), dtype=torch.int8, device="cuda")
    s1 = torch.zeros(2, device="cuda")
    q8.q8_absmax(torch.from_numpy(c1["W"]).cuda(), s1[0:1], s1[1:2])
    q8.q8_quantize(torch.from_numpy(c1["W"]).cuda(), s1[1:2], w1q)
    b1 = torch.from_numpy(c1["b"]).cuda()
    y1, xq1_ = torch.empty((16, 768), device="cuda"), torch.empty(16 * 768, dtype=torch.int8, device="cuda")
    us = event_us(torch, lambda i: q8.q8_linear_f32(x1, w1q, b1, s1[1:2], xq1_, layer.scal, y1), 200, warm=20)
    out["c1_single_fc_16x768x768"] = {"us_per_dynamic_fc_call": round(us, 2), "launches": 1,
                                      "note": "quantizer and GEMM in one kernel; calls issued back to back from Python, whose own launch rate "
                                              "(a one-thread kernel: 6-7 us per call) is most of the figure"}
    base = {}
    for key, batch in (("c3_bert_base_encoder_layer_32x128", 32), ("c5_bert_base_12_layer_forward_64x128", 64)):
        db = synth.bert_base_layer(seed=2, batch=batch, seq=128)
        lb = Layer(q8, torch, db, synth.embedding_tables(seed=5, hidden=768), synth.token_ids(seed=6, batch=batch, seq=128))
        lb.glue_once()
        lb.step_fused()
        lb.step_layer()
        torch.cuda.synchronize()
        if batch == 32:
            t = timed(torch, lb.step_layer, 100, 30)
            base[key] = {"us_per_layer": round(t * 1e6, 1), "tokens_per_s": round(lb.M / t, 1)}
        else:
            def forward(lb=lb):
                q8.q8_embedding_sum3_layernorm(lb.tables[0], lb.tables[1], lb.tables[2], lb.table_scales, lb.ids[0], lb.ids[1],
                                               lb.ids[2], lb.ln_g, lb.ln_b, lb.x_in, amax_slots=lb.slots_x, err_flag=lb.err)
                for _ in range(12):
                    lb.step_layer()
            t = timed(torch, forward, 30, 10)
            base[key] = {"ms_per_forward": round(t * 1e3, 3), "tokens_per_s": round(lb.M / t, 1), "sequences_per_s": round(batch / t, 1)}
        del lb
    out.update(base)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(d, args.cpu_sample_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
