"""Oracle of the backward pass of the tree / chunk attention (paper section 3.1, "Efficient Tree Attention":
all accepted and rejected branches of the speculative tree go through one batched forward and backward pass
under a mask that follows the tree).

TEST INFRASTRUCTURE ONLY.  Plain NumPy, float64, one (request, query head, node) row at a time - the chain
rule of out = softmax(scale * q K^T + mask) V written out:

    p_j   = softmax_j(scale * <q, k_j>)  over the visible positions j (prefix, the node itself, its ancestors)
    delta = <dout, out>
    dP_j  = <dout, v_j>
    dS_j  = p_j * (dP_j - delta)
    dq    = scale * sum_j dS_j k_j ;   dk_j += scale * dS_j q ;   dv_j += p_j dout

dk / dv of a KV position collect the contributions of every query row that sees it (all nodes, all query heads
of the KV head's group).  They are returned in the paged layout of the pools; positions no request uses stay 0.
Reading: the gradient flows to q and to every visible K / V position, the cached prefix included (the
drafter's own cache is a function of its weights); nothing else of the training step is part of this.
"""
from __future__ import annotations

import numpy as np


def attn_backward(q, k_pages, v_pages, block_table, seq_lens, parents, dout, sm_scale=0.0):
    """q, dout [B,Nq,Hq,D]; pools [P,Hkv,page,D] (float arrays holding the stored values); returns
    (out, dq, dk_pages, dv_pages), all float64.  Per (request, KV head) the request's K / V rows are gathered once
    and the gradients of its positions are scattered back once; in between, one query row at a time."""
    q = np.asarray(q, np.float64)
    dout = np.asarray(dout, np.float64)
    kp = np.asarray(k_pages, np.float64)
    vp = np.asarray(v_pages, np.float64)
    B, Nq, Hq, D = q.shape
    P, Hkv, page, _ = kp.shape
    G = Hq // Hkv
    scale = sm_scale if sm_scale > 0 else 1.0 / np.sqrt(D)
    out = np.zeros_like(q)
    dq = np.zeros_like(q)
    dk = np.zeros_like(kp)
    dv = np.zeros_like(vp)
    for b in range(B):
        L = int(seq_lens[b])
        prefix = L - Nq
        pos = np.arange(L)
        pg = np.asarray(block_table[b], np.int64)[pos // page]
        off = pos % page
        seen = np.zeros((Nq, L), bool)
        seen[:, :prefix] = True
        for n in range(Nq):
            a = n
            while a >= 0:
                seen[n, prefix + a] = True
                a = int(parents[b, a]) if parents is not None else a - 1
        for hk in range(Hkv):
            K = kp[pg, hk, off]                       # [L, D]: position j of this request
            V = vp[pg, hk, off]
            dK = np.zeros_like(K)
            dV = np.zeros_like(V)
            for n in range(Nq):
                vis = seen[n]
                for hq in range(hk * G, (hk + 1) * G):
                    s = scale * (K @ q[b, n, hq])
                    p = np.exp(np.where(vis, s - s[vis].max(), -np.inf))
                    p /= p.sum()
                    o = p @ V
                    out[b, n, hq] = o
                    g = dout[b, n, hq]
                    delta = float(g @ o)
                    dS = p * (V @ g - delta)
                    dq[b, n, hq] = scale * (dS @ K)
                    dK += scale * np.outer(dS, q[b, n, hq])
                    dV += np.outer(p, g)
            # a request's positions are distinct (page, offset) pairs: plain indexed accumulation
            dk[pg, hk, off] += dK
            dv[pg, hk, off] += dV
    return out, dq, dk, dv


def attn_lse(q, k_pages, block_table, seq_lens, parents, sm_scale=0.0):
    """Natural logarithm of every row's softmax denominator, lse[b, n, hq] = log sum_j exp(scale * <q, k_j>) over the
    positions j the row sees - the quantity a training step keeps from the forward pass.  float64 [B, Nq, Hq]."""
    q = np.asarray(q, np.float64)
    kp = np.asarray(k_pages, np.float64)
    B, Nq, Hq, D = q.shape
    P, Hkv, page, _ = kp.shape
    G = Hq // Hkv
    scale = sm_scale if sm_scale > 0 else 1.0 / np.sqrt(D)
    lse = np.zeros((B, Nq, Hq))
    for b in range(B):
        L = int(seq_lens[b])
        prefix = L - Nq
        for n in range(Nq):
            js = list(range(prefix))
            chain = []
            a = n
            while a >= 0:
                chain.append(prefix + a)
                a = int(parents[b, a]) if parents is not None else a - 1
            js += sorted(chain)
            for hq in range(Hq):
                s = np.array([scale * float(kp[int(block_table[b, j // page]), hq // G, j % page] @ q[b, n, hq]) for j in js])
                top = s.max()
                lse[b, n, hq] = top + np.log(np.exp(s - top).sum())
    return lse
