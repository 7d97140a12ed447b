"""Seeded synthetic inputs shaped like the paper's workloads.

Holds NO arithmetic of the method: only the named model shapes, random draws
and the bf16 rounding of inputs.  Both the GPU library's tests and the fp64
oracle's tests receive the arrays made here, so the two sides start from
identical numbers.  The paper trains GPT-2 and BERT variants on WikiText and
GLUE (Section 5.1); those datasets are not used: dense compute cost does not
depend on token statistics, so uniform random ids stand in for them.
"""
from __future__ import annotations

from collections import OrderedDict

import numpy as np

# name -> model/workload shape.  M microbatches of b sequences.
CONFIGS = {
    # tiny GPT decoder, fp32, every pack one layer
    "tiny": dict(n_blocks=4, d_model=128, n_heads=4, d_ffn=512, seq_len=64, vocab=512,
                 causal=1, precision="fp32", M=4, b=2, budget=None),
    # GPT-2-medium-shaped decoder (the benchmark workload)
    "gpt2m": dict(n_blocks=24, d_model=1024, n_heads=16, d_ffn=4096, seq_len=1024, vocab=50257,
                  causal=1, precision="bf16", M=8, b=4, budget=4 * 10**9),
    # GPT-2-XL-shaped decoder
    "gpt2xl": dict(n_blocks=48, d_model=1600, n_heads=25, d_ffn=6400, seq_len=1024, vocab=50257,
                   causal=1, precision="bf16", M=16, b=2, budget=16 * 10**9),
    # BERT-large-shaped encoder, 15% of positions are targets
    "bertl": dict(n_blocks=24, d_model=1024, n_heads=16, d_ffn=4096, seq_len=512, vocab=30522,
                  causal=0, precision="bf16", M=32, b=8, budget=2 * 10**9),
    # 6.7B-parameter decoder
    "gpt6b7": dict(n_blocks=32, d_model=4096, n_heads=32, d_ffn=16384, seq_len=2048, vocab=50257,
                   causal=1, precision="bf16", M=16, b=1, budget=32 * 10**9),
}

LN_EPS = 1e-5


def shape_table(cfg) -> "OrderedDict[str, tuple]":
    """Parameter names and shapes in storage order (embedding, blocks, head)."""
    d, f, s, V = cfg["d_model"], cfg["d_ffn"], cfg["seq_len"], cfg["vocab"]
    t: "OrderedDict[str, tuple]" = OrderedDict()
    t["wte"] = (V, d)
    t["wpe"] = (s, d)
    for l in range(1, cfg["n_blocks"] + 1):
        p = f"h{l}."
        t[p + "ln1_g"] = (d,)
        t[p + "ln1_b"] = (d,)
        t[p + "wqkv"] = (3 * d, d)
        t[p + "bqkv"] = (3 * d,)
        t[p + "wo"] = (d, d)
        t[p + "bo"] = (d,)
        t[p + "ln2_g"] = (d,)
        t[p + "ln2_b"] = (d,)
        t[p + "w1"] = (f, d)
        t[p + "b1"] = (f,)
        t[p + "w2"] = (d, f)
        t[p + "b2"] = (d,)
    t["lnf_g"] = (d,)
    t["lnf_b"] = (d,)
    t["wh"] = (V, d)
    return t


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even to bfloat16, returned widened to float32."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def gen_params(cfg, seed: int = 0, bench_init: bool = True) -> "OrderedDict[str, np.ndarray]":
    """fp32 parameters.  bench_init: matrices and embeddings N(0, 0.02^2),
    biases 0, LayerNorm gamma 1 / beta 0 (the benchmark recipe).  Otherwise
    biases N(0, 0.02^2), gamma 1 + N(0, 0.1^2), beta N(0, 0.1^2) so that every
    gradient path is exercised."""
    rng = np.random.default_rng(seed)
    out: "OrderedDict[str, np.ndarray]" = OrderedDict()
    for name, shape in shape_table(cfg).items():
        base = name.split(".")[-1]
        if len(shape) == 2:
            a = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.02)
        elif base.endswith("_g"):
            a = np.ones(shape, np.float32)
            if not bench_init:
                a = a + rng.standard_normal(shape, dtype=np.float32) * np.float32(0.1)
        elif base.endswith("_b") and base.startswith("ln"):
            a = np.zeros(shape, np.float32)
            if not bench_init:
                a = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.1)
        else:  # linear biases
            a = np.zeros(shape, np.float32)
            if not bench_init:
                a = rng.standard_normal(shape, dtype=np.float32) * np.float32(0.02)
        out[name] = a
    return out


def gen_adam_state(cfg, seed: int, zero: bool = True, scale: float = 1e-2):
    """(m, v) per tensor: zeros (step 1) or a mid-training state with first
    moments N(0, scale^2) and second moments of matching size."""
    rng = np.random.default_rng(seed + 7919)
    m: "OrderedDict[str, np.ndarray]" = OrderedDict()
    v: "OrderedDict[str, np.ndarray]" = OrderedDict()
    for name, shape in shape_table(cfg).items():
        if zero:
            m[name] = np.zeros(shape, np.float32)
            v[name] = np.zeros(shape, np.float32)
        else:
            m[name] = rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)
            v[name] = (rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)) ** 2 \
                + np.float32(scale * scale * 1e-2)
    return m, v


def gen_tokens(cfg, seed: int = 0, M: int | None = None, b: int | None = None) -> np.ndarray:
    """ids[M, b, s] uniform in [0, vocab)."""
    M = cfg["M"] if M is None else M
    b = cfg["b"] if b is None else b
    rng = np.random.default_rng(seed + 104729)
    return rng.integers(0, cfg["vocab"], size=(M, b, cfg["seq_len"]), dtype=np.int32)


def decoder_targets(ids: np.ndarray) -> np.ndarray:
    """Next-token targets: y[., j] = id[., j+1]; the last position has none (-1)."""
    tgt = np.full_like(ids, -1)
    tgt[..., :-1] = ids[..., 1:]
    return tgt


def mlm_targets(ids: np.ndarray, frac: float = 0.15, seed: int = 0) -> np.ndarray:
    """round(frac*s) positions per sequence (seeded permutation) are targets,
    the target being the token at that position; others -1."""
    rng = np.random.default_rng(seed + 1299709)
    M, b, s = ids.shape
    k = int(round(frac * s))
    tgt = np.full_like(ids, -1)
    for i in range(M):
        for j in range(b):
            pos = rng.permutation(s)[:k]
            tgt[i, j, pos] = ids[i, j, pos]
    return tgt


def gen_targets(cfg, ids: np.ndarray, seed: int = 0) -> np.ndarray:
    return decoder_targets(ids) if cfg["causal"] else mlm_targets(ids, 0.15, seed)
