"""Oracle of the drafter's training loss on one batch of trace rows (paper section 3.3, eq. 3).

TEST INFRASTRUCTURE ONLY (imported through the oracle package by tests).  Plain NumPy, float64, one row at
a time, the definition written out.

    L = mean over accepted rows of KL(p_target || p_draft)
        + lambda_discard * mean over discarded rows of KL(p_target || p_draft)

Readings (the paper gives the formula and the words "top-k filtering", no more):
  * a row is one token position of a verify step; its class is the trajectory code of the trace record
    (appendix A.1): 1 = on the accepted path, 2 = tested and rejected ("discarded"), 0 = not used.  The
    expectations are means over the rows of the class in this batch; an empty class contributes 0.
  * p_target of a row is the softmax over the target logits that were kept for it - the K largest,
    appendix A.2 - and zero on every other token; entries with id -1 (padding) or value -inf carry no mass.
  * p_draft is the softmax of the drafter's logits over its whole vocabulary.
  * "top-k filtering of the discarded tokens": on discarded rows only the discard_top_k largest kept target
    logits are used (renormalised), so that the term concentrates on the tokens the target rates highly.
  * the gradient with respect to the drafter's logits of row m is w_m (p_draft - p_target) with
    w_m = 1 / N_accept, lambda_discard / N_discard or 0 by class - the derivative of the formula above.
The kept logits arrive ordered by value, largest first (that is how trace emission writes them).
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def draft_loss(draft_logits, topk_ids, topk_logits_bits, traj, lambda_discard: float, discard_top_k=None,
               want_grad: bool = True):
    """Returns dict(row_kl [M], loss, mean_accept, mean_discard, n_accept, n_discard, grad [M, Vd] or None)."""
    z = np.asarray(draft_logits, dtype=np.float64)
    M, Vd = z.shape
    ids = np.asarray(topk_ids, dtype=np.int64)
    K = ids.shape[1]
    lt = bf16_bits_to_f64(topk_logits_bits)
    traj = np.asarray(traj, dtype=np.int64)
    assert ids.shape == (M, K) and lt.shape == (M, K) and traj.shape == (M,)
    n_acc = int((traj == 1).sum())
    n_disc = int((traj == 2).sum())
    row_kl = np.zeros(M, np.float64)
    grad = np.zeros((M, Vd), np.float64) if want_grad else None
    for m in range(M):
        k = K
        if traj[m] == 2 and discard_top_k is not None:
            k = min(K, int(discard_top_k))
        assert all(lt[m, j] >= lt[m, j + 1] for j in range(K - 1)), "kept logits must be ordered, largest first"
        kept = [j for j in range(k) if ids[m, j] >= 0 and lt[m, j] > -np.inf]
        # the drafter's log-probabilities over its whole vocabulary
        zmax = z[m].max()
        lse_d = zmax + np.log(np.exp(z[m] - zmax).sum())
        logpd = z[m] - lse_d
        kl = 0.0
        pt = np.zeros(len(kept))
        if kept:
            zt = lt[m, kept]
            lse_t = zt.max() + np.log(np.exp(zt - zt.max()).sum())
            logpt = zt - lse_t
            pt = np.exp(logpt)
            for j, a, b in zip(kept, pt, logpt):
                kl += a * (b - logpd[ids[m, j]])
        row_kl[m] = kl
        if want_grad:
            w = 1.0 / n_acc if traj[m] == 1 else (lambda_discard / n_disc if traj[m] == 2 else 0.0)
            if kept:
                g = w * np.exp(logpd)
                for j, a in zip(kept, pt):
                    g[ids[m, j]] -= w * a
                grad[m] = g
            # a row with no kept target logit has no target distribution: it contributes nothing
    mean_acc = float(row_kl[traj == 1].mean()) if n_acc else 0.0
    mean_disc = float(row_kl[traj == 2].mean()) if n_disc else 0.0
    return dict(row_kl=row_kl, loss=mean_acc + lambda_discard * mean_disc, mean_accept=mean_acc,
                mean_discard=mean_disc, n_accept=n_acc, n_discard=n_disc, grad=grad)
