"""Seeded synthetic inputs shaped like BERT-Base/Large fine-tuning workloads.

This module only draws random numbers and names shapes.  It holds none of the
quantization arithmetic, so both the CPU oracle's tests and the HIP path's tests
can take their inputs from it without sharing any part of the method.

Distributions: activations ~ N(0, 1); weights, biases and embedding tables
~ N(0, 0.02^2) (BERT's initialiser std); token ids uniform in [0, vocab).
All arrays are float32 / int32 NumPy arrays made on the host, so that the oracle
and the GPU see identical bytes.
"""
from __future__ import annotations

import numpy as np

W_STD = 0.02
VOCAB = 30522
MAX_POS = 512
N_TYPES = 2

# (name, tokens M, hidden, ffn, heads) for the encoder-shaped workloads.
BERT_BASE = dict(hidden=768, ffn=3072, heads=12)
BERT_LARGE = dict(hidden=1024, ffn=4096, heads=16)


def rng(seed: int) -> np.random.Generator:
    return np.random.default_rng(seed)


def activations(g: np.random.Generator, m: int, k: int) -> np.ndarray:
    return g.standard_normal((m, k), dtype=np.float32)


def weights(g: np.random.Generator, n: int, k: int) -> np.ndarray:
    return (g.standard_normal((n, k), dtype=np.float32) * np.float32(W_STD)).astype(np.float32)


def bias(g: np.random.Generator, n: int) -> np.ndarray:
    return (g.standard_normal((n,), dtype=np.float32) * np.float32(W_STD)).astype(np.float32)


def fc_layer(seed: int, m: int, k: int, n: int) -> dict:
    """One fully-connected layer y = x W^T + b: x[m,k], W[n,k], b[n]."""
    g = rng(seed)
    return dict(x=activations(g, m, k), W=weights(g, n, k), b=bias(g, n))


def single_fc(seed: int = 0) -> dict:
    """Smallest workload: 16 tokens x 768 -> 768."""
    return fc_layer(seed, 16, 768, 768)


def ffn_block(seed: int, m: int, hidden: int, ffn: int) -> dict:
    g = rng(seed)
    return dict(
        x=activations(g, m, hidden),
        W1=weights(g, ffn, hidden), b1=bias(g, ffn),
        W2=weights(g, hidden, ffn), b2=bias(g, hidden),
    )


def encoder_layer(seed: int, batch: int, seq: int, hidden: int, ffn: int, heads: int) -> dict:
    """Weights and input of one BERT encoder layer (LayerNorm gamma=1, beta=0)."""
    g = rng(seed)
    m = batch * seq
    d = dict(batch=batch, seq=seq, hidden=hidden, ffn=ffn, heads=heads)
    d["x"] = activations(g, m, hidden)
    for name in ("q", "k", "v", "o"):
        d["W" + name] = weights(g, hidden, hidden)
        d["b" + name] = bias(g, hidden)
    d["W1"] = weights(g, ffn, hidden)
    d["b1"] = bias(g, ffn)
    d["W2"] = weights(g, hidden, ffn)
    d["b2"] = bias(g, hidden)
    return d


def bert_base_layer(seed: int = 2, batch: int = 32, seq: int = 128) -> dict:
    return encoder_layer(seed, batch, seq, **BERT_BASE)


def bert_large_layer(seed: int = 3, batch: int = 32, seq: int = 384) -> dict:
    return encoder_layer(seed, batch, seq, **BERT_LARGE)


def embedding_tables(seed: int, hidden: int, vocab: int = VOCAB) -> dict:
    g = rng(seed)
    return dict(
        word=weights(g, vocab, hidden),
        position=weights(g, MAX_POS, hidden),
        token_type=weights(g, N_TYPES, hidden),
    )


def token_ids(seed: int, batch: int, seq: int, vocab: int = VOCAB) -> dict:
    """ids uniform in [0, vocab); positions 0..seq-1; type 0 for the first half, 1 after."""
    g = rng(seed)
    ids = g.integers(0, vocab, size=(batch, seq), dtype=np.int32)
    pos = np.broadcast_to(np.arange(seq, dtype=np.int32), (batch, seq)).copy()
    typ = np.broadcast_to((np.arange(seq) >= seq // 2).astype(np.int32), (batch, seq)).copy()
    return dict(word=ids.reshape(-1), position=pos.reshape(-1), token_type=typ.reshape(-1))


def random_int8(g: np.random.Generator, shape, lo: int = -127, hi: int = 127) -> np.ndarray:
    return g.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int8)
