"""Pins of the attention-backward oracle (paper section 3.1: the speculative tree goes through one batched forward
and backward pass under a tree mask): the library's reverse-mode differentiation of a dense masked attention, and
central differences of the forward oracle."""
import numpy as np
import torch

import gen
import oracle


def _dense_case(w):
    """Dense K/V per request and the visibility mask, built here from the workload's definition."""
    B, Nq, Hq, D = w.q.shape
    Hkv, page = w.num_kv_heads, w.page_size
    kf, vf = gen.as_f32(w.k_pages, w.dtype).astype(np.float64), gen.as_f32(w.v_pages, w.dtype).astype(np.float64)
    out = []
    for b in range(B):
        L = int(w.seq_lens[b])
        pages = w.block_table[b, :(L + page - 1) // page]
        K = kf[pages].transpose(1, 0, 2, 3).reshape(Hkv, -1, D)[:, :L]
        V = vf[pages].transpose(1, 0, 2, 3).reshape(Hkv, -1, D)[:, :L]
        mask = np.zeros((Nq, L), bool)
        mask[:, :L - Nq] = True
        for n in range(Nq):
            a = n
            while a >= 0:
                mask[n, L - Nq + a] = True
                a = int(w.parents[b, a]) if w.parents is not None else a - 1
        out.append((K, V, mask))
    return out


def _autograd(w, dout):
    B, Nq, Hq, D = w.q.shape
    G = Hq // w.num_kv_heads
    qf = gen.as_f32(w.q, w.dtype).astype(np.float64)
    res = []
    for b, (K, V, mask) in enumerate(_dense_case(w)):
        q = torch.tensor(qf[b].transpose(1, 0, 2), requires_grad=True)            # [Hq, Nq, D]
        Kt = torch.tensor(K, requires_grad=True)
        Vt = torch.tensor(V, requires_grad=True)
        o = torch.nn.functional.scaled_dot_product_attention(
            q, Kt.repeat_interleave(G, 0), Vt.repeat_interleave(G, 0), attn_mask=torch.tensor(mask))
        o.backward(torch.tensor(dout[b].transpose(1, 0, 2)))
        res.append((o.detach().numpy().transpose(1, 0, 2), q.grad.numpy().transpose(1, 0, 2), Kt.grad.numpy(),
                    Vt.grad.numpy()))
    return res


def _check(w, seed):
    rng = np.random.default_rng(seed)
    dout = rng.standard_normal(w.q.shape)
    kf, vf = gen.as_f32(w.k_pages, w.dtype), gen.as_f32(w.v_pages, w.dtype)
    out, dq, dk, dv = oracle.attn_backward(gen.as_f32(w.q, w.dtype), kf, vf, w.block_table, w.seq_lens, w.parents, dout)
    fwd = oracle.attn_workload(w)
    assert np.allclose(out, fwd, rtol=1e-12, atol=1e-14)                          # same forward as the attention oracle
    page = w.page_size
    used = np.zeros(dk.shape[:3], bool)
    for b, (o_ref, dq_ref, dK_ref, dV_ref) in enumerate(_autograd(w, dout)):
        assert np.allclose(out[b], o_ref, rtol=1e-10, atol=1e-12)
        assert np.allclose(dq[b], dq_ref, rtol=1e-9, atol=1e-11)
        L = int(w.seq_lens[b])
        for j in range(L):
            pg, off = int(w.block_table[b, j // page]), j % page
            used[pg, :, off] = True
            assert np.allclose(dk[pg, :, off], dK_ref[:, j], rtol=1e-9, atol=1e-11), (b, j)
            assert np.allclose(dv[pg, :, off], dV_ref[:, j], rtol=1e-9, atol=1e-11), (b, j)
    assert not dk[~used].any() and not dv[~used].any()                             # unused positions stay zero


def test_chain_against_reverse_mode_differentiation():
    _check(gen.llama_chain(5, batch=2, len_lo=9, len_hi=40, vocab=32, hidden_size=16, num_q_heads=4, num_kv_heads=2,
                           head_dim=16, page_size=8), 1)
    _check(gen.llama_chain(6, batch=1, num_q=1, len_lo=12, len_hi=12, vocab=32, hidden_size=16, num_q_heads=2,
                           num_kv_heads=2, head_dim=8, page_size=4), 2)


def test_tree_against_reverse_mode_differentiation():
    _check(gen.llama_tree(7, batch=2, num_q=9, context=30, vocab=32, hidden_size=16, num_q_heads=6, num_kv_heads=2,
                          head_dim=16, page_size=8), 3)


def test_central_differences_of_the_forward_oracle():
    w = gen.llama_tree(8, batch=1, num_q=5, context=14, vocab=32, hidden_size=16, num_q_heads=2, num_kv_heads=1,
                       head_dim=8, page_size=4, dtype=gen.F32)
    rng = np.random.default_rng(4)
    dout = rng.standard_normal(w.q.shape)
    out, dq, dk, dv = oracle.attn_backward(w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, w.parents, dout)

    def loss(q=None, k=None, v=None):
        o = oracle.attn(q=(w.q if q is None else q).astype(np.float32), k_pages=(w.k_pages if k is None else k).astype(np.float32),
                        v_pages=(w.v_pages if v is None else v).astype(np.float32), block_table=w.block_table,
                        seq_lens=w.seq_lens, parents=w.parents, dtype="f32")
        return float((o * dout).sum())
    h = 1e-3   # the forward oracle takes float32 inputs: a step well above their spacing
    for idx in [(0, 2, 1, 3), (0, 4, 0, 7), (0, 0, 1, 0)]:
        qp, qm = w.q.copy(), w.q.copy()
        qp[idx] += h
        qm[idx] -= h
        fd = (loss(q=qp) - loss(q=qm)) / (float(qp[idx]) - float(qm[idx]))
        assert abs(fd - dq[idx]) < 1e-4 * max(1.0, abs(dq[idx]))
    pg = int(w.block_table[0, 1])
    for arr, grad, name in ((w.k_pages, dk, "k"), (w.v_pages, dv, "v")):
        idx = (pg, 0, 2, 5)
        ap, am = arr.copy(), arr.copy()
        ap[idx] += h
        am[idx] -= h
        fd = (loss(**{name: ap}) - loss(**{name: am})) / (float(ap[idx]) - float(am[idx]))
        assert abs(fd - grad[idx]) < 1e-4 * max(1.0, abs(grad[idx])), name


def test_lse_against_library_logsumexp_and_the_attention_oracle():
    """The logsumexp oracle against torch.logsumexp on dense masked scores, and tied to the (separately pinned)
    attention oracle: softmax weights rebuilt from it reproduce that oracle's output."""
    for w in (gen.llama_tree(9, batch=2, num_q=7, context=25, vocab=32, hidden_size=16, num_q_heads=4, num_kv_heads=2,
                             head_dim=16, page_size=8, dtype=gen.F32),
              gen.llama_chain(10, batch=2, len_lo=9, len_hi=33, vocab=32, hidden_size=16, num_q_heads=6, num_kv_heads=2,
                              head_dim=8, page_size=4, dtype=gen.F32)):
        B, Nq, Hq, D = w.q.shape
        G = Hq // w.num_kv_heads
        lse = oracle.attn_lse(w.q, w.k_pages, w.block_table, w.seq_lens, w.parents)
        fwd = oracle.attn_workload(w)
        scale = 1.0 / np.sqrt(D)
        for b, (K, V, mask) in enumerate(_dense_case(w)):
            s = torch.einsum("nhd,hjd->hnj", torch.tensor(w.q[b].astype(np.float64)),
                             torch.tensor(K).repeat_interleave(G, 0)) * scale
            s = s.masked_fill(~torch.tensor(mask)[None], float("-inf"))
            ref = torch.logsumexp(s, dim=-1).numpy().T                               # [Nq, Hq]
            assert np.allclose(lse[b], ref, rtol=1e-12, atol=1e-12)
            p = np.exp(s.numpy() - lse[b].T[:, :, None])                              # [Hq, Nq, L]
            o = np.einsum("hnj,hjd->nhd", p, np.repeat(V, G, axis=0))
            assert np.allclose(o, fwd[b], rtol=1e-9, atol=1e-11)
