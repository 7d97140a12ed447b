"""Glue between the seeded inputs and the two sides under test (no arithmetic
of the method lives here)."""
from __future__ import annotations

import numpy as np

from oracle import model as om
from paper_2202_01306_amd import synth


def tiny_cfg(**kw):
    cfg = dict(n_blocks=2, d_model=16, n_heads=2, d_ffn=32, seq_len=8, vocab=32,
               causal=1, precision="fp32", M=2, b=2, budget=None)
    cfg.update(kw)
    return cfg


def oracle_spec(cfg) -> om.Spec:
    return om.Spec(cfg["n_blocks"], cfg["d_model"], cfg["n_heads"], cfg["d_ffn"],
                   cfg["seq_len"], cfg["vocab"], bool(cfg["causal"]), synth.LN_EPS)


def f64(d):
    return {k: np.asarray(v, dtype=np.float64) for k, v in d.items()}


def max_rel_err(x, ref) -> float:
    """max|x - ref| / max(max|ref|, 1e-30): the parity metric (element-wise
    relative error is meaningless at gradient zeros)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(x - ref).max() / max(np.abs(ref).max(), 1e-30))
