"""Seeded inputs of the drafter-loss kernel: a batch of trace rows as the training side receives them.

Input generation only.  Shapes follow the paper (appendix A.2: K = 1024 target logits kept per token,
2 bytes each; a draft vocabulary of about 32K entries; appendix A.1: one trajectory code per token).  The
kept target logits of a row are drawn directly as an ordered list of values on distinct random ids - no
selection happens here - and the drafter's logits agree with them up to noise on those ids and sit lower
elsewhere, as a partly trained drafter's would.
"""
from __future__ import annotations

import numpy as np


def loss_inputs(seed: int, rows: int, draft_vocab: int, top_k: int = 1024, noise: float = 1.0,
                frac_accept: float = 0.45, frac_discard: float = 0.35, pad_rows: int = 0):
    """Returns (draft_logits f32 [rows, Vd], topk_ids i32 [rows, K], topk_logits bf16 bits u16 [rows, K],
    traj i8 [rows]).  If top_k > draft_vocab the tail of every row is padding (id -1, -inf).  The first
    `pad_rows` rows get a random number of trailing padding entries and a few -inf values besides."""
    rng = np.random.default_rng([seed, rows, draft_vocab, top_k])
    K, Vd = int(top_k), int(draft_vocab)
    keep = min(K, Vd)
    ids = np.full((rows, K), -1, np.int32)
    bits = np.full((rows, K), 0xFF80, np.uint16)  # -inf
    z = (rng.standard_normal((rows, Vd), dtype=np.float32) - np.float32(3.0)).astype(np.float32)
    for m in range(rows):
        n = keep
        if m < pad_rows:
            n = int(rng.integers(1, keep + 1))
        sel = rng.choice(Vd, size=n, replace=False).astype(np.int32)
        vals = np.sort((rng.standard_normal(n, dtype=np.float32) * np.float32(2.0) + np.float32(rng.normal())))[::-1]
        # bf16 storage: keep the high half of the float32 pattern (rounds toward zero - monotone, so the
        # list stays ordered)
        b = (np.ascontiguousarray(vals).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
        if m < pad_rows and n > 3:
            b[n - 2:] = 0xFF80  # kept entries whose value is -inf (a masked vocabulary)
        ids[m, :n] = sel
        bits[m, :n] = b
        shown = (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
        fin = np.isfinite(shown)
        z[m, sel[fin]] = shown[fin] + rng.standard_normal(int(fin.sum()), dtype=np.float32) * np.float32(noise)
    u = rng.random(rows)
    traj = np.where(u < frac_accept, 1, np.where(u < frac_accept + frac_discard, 2, 0)).astype(np.int8)
    return np.ascontiguousarray(z), ids, bits, traj
