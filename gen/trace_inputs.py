"""Seeded float32 logit matrices for the trace-emission (top-K) tests and benchmark.

Input generation only: nothing here selects, sorts or rounds.  The shapes follow the paper's
vocabularies (128256 / 151936 entries per token row, K = 1024 kept; appendix A.2); the value
distributions cover what an LM head produces (roughly normal logits) and the degenerate rows a
selection must survive (repeated values, constant rows, masked vocabularies, signed zeros).
"""
from __future__ import annotations

import numpy as np

KINDS = ("normal", "ties", "equal", "masked", "zeros", "skewed")


def trace_logits(seed: int, rows: int, vocab: int, kind: str = "normal") -> np.ndarray:
    rng = np.random.default_rng([seed, rows, vocab, KINDS.index(kind)])
    if kind == "normal":       # LM-head-like: N(0, 1.3^2) plus a per-row offset
        x = rng.standard_normal((rows, vocab), dtype=np.float32) * np.float32(1.3)
        x += rng.standard_normal((rows, 1), dtype=np.float32)
    elif kind == "ties":       # values on a coarse grid: thousands of exact ties around any threshold
        x = np.round(rng.standard_normal((rows, vocab), dtype=np.float32) * 4) / np.float32(8)
    elif kind == "equal":      # constant rows (one of them -inf throughout)
        x = np.repeat(rng.standard_normal((rows, 1), dtype=np.float32), vocab, axis=1)
        if rows > 1:
            x[1, :] = -np.inf
    elif kind == "masked":     # all but a few hundred entries masked to -inf
        x = np.full((rows, vocab), -np.inf, dtype=np.float32)
        keep = max(1, min(vocab, 500))
        for m in range(rows):
            idx = rng.choice(vocab, size=keep, replace=False)
            x[m, idx] = rng.standard_normal(keep, dtype=np.float32)
    elif kind == "zeros":      # mostly +0.0 / -0.0 with a sprinkling of other values
        x = np.where(rng.random((rows, vocab)) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32)
        spr = rng.random((rows, vocab)) < 0.002
        x[spr] = rng.standard_normal(int(spr.sum()), dtype=np.float32)
    elif kind == "skewed":     # heavy right tail over a huge dynamic range, negative bulk
        x = -np.exp(rng.uniform(-40, 40, (rows, vocab))).astype(np.float32)
        top = rng.random((rows, vocab)) < 0.004
        x[top] = np.exp(rng.uniform(-40, 40, int(top.sum()))).astype(np.float32)
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(x, dtype=np.float32)
