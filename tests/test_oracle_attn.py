"""Pins for the oracle's chunk attention and LM-head projection (CPU only).

Each check compares the oracle with something that is not the oracle: a library routine
(torch scaled_dot_product_attention, NumPy float64 matmul), a closed form, or an invariance
the definition implies.
"""
import numpy as np
import pytest
import torch

import gen
import oracle


def _dense_kv(w, b):
    L = int(w.seq_lens[b])
    pos = np.arange(L)
    pages = w.block_table[b, pos // w.page_size]
    k = gen.as_f32(w.k_pages, w.dtype)[pages, :, pos % w.page_size, :]  # [L, Hkv, D]
    v = gen.as_f32(w.v_pages, w.dtype)[pages, :, pos % w.page_size, :]
    return k.astype(np.float64), v.astype(np.float64)


def _mask(w, b):
    L = int(w.seq_lens[b])
    Nq = w.num_q
    m = np.zeros((Nq, L), dtype=bool)
    m[:, : L - Nq] = True
    for n in range(Nq):
        a = n
        while a >= 0:
            m[n, L - Nq + a] = True
            a = int(w.parents[b, a]) if w.parents is not None else a - 1
    return m


def _library_attention(w):
    out = np.zeros((w.batch, w.num_q, w.num_q_heads, w.head_dim))
    G = w.num_q_heads // w.num_kv_heads
    for b in range(w.batch):
        k, v = _dense_kv(w, b)
        kt = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(G, dim=0)  # [Hq, L, D]
        vt = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(G, dim=0)
        qt = torch.from_numpy(gen.as_f32(w.q, w.dtype)[b].astype(np.float64)).permute(1, 0, 2)  # [Hq,Nq,D]
        mask = torch.from_numpy(_mask(w, b))
        o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask)
        out[b] = o.permute(1, 0, 2).numpy()
    return out


def _oracle_attn(w, **kw):
    args = dict(q=w.q, k_pages=w.k_pages, v_pages=w.v_pages, block_table=w.block_table,
                seq_lens=w.seq_lens, parents=w.parents, dtype=w.dtype)
    args.update(kw)
    return oracle.attn(**args)


@pytest.mark.parametrize("dtype", [gen.F32, gen.BF16])
def test_chain_matches_library_sdpa(dtype):
    w = gen.llama_chain(3, batch=3, num_q=4, num_q_heads=6, num_kv_heads=2, head_dim=16,
                        page_size=4, hidden_size=8, vocab=32, len_lo=5, len_hi=41, dtype=dtype)
    np.testing.assert_allclose(_oracle_attn(w), _library_attention(w), rtol=1e-11, atol=1e-13)


def test_tree_matches_library_sdpa():
    w = gen.llama_tree(5, batch=2, num_q=9, num_q_heads=4, num_kv_heads=4, head_dim=8,
                       page_size=8, hidden_size=8, vocab=32, context=37, dtype=gen.F32)
    assert (w.parents[:, 1:] < np.arange(1, 9)).all()
    np.testing.assert_allclose(_oracle_attn(w), _library_attention(w), rtol=1e-11, atol=1e-13)


def test_tiny_config_matches_library_sdpa():
    w = gen.tiny_chain(1)
    np.testing.assert_allclose(_oracle_attn(w), _library_attention(w), rtol=1e-10, atol=1e-13)


def test_equal_keys_give_mean_of_visible_values():
    """All keys equal => uniform weights => row i is the mean of the first L-Nq+i+1 value rows."""
    w = gen.tiny_chain(2, batch=2, seq_lens=np.array([40, 17], np.int32), page_size=64)
    w.k_pages[:] = w.k_pages[0, 0, 0]
    out = _oracle_attn(w)
    G = w.num_q_heads // w.num_kv_heads
    for b in range(w.batch):
        _, v = _dense_kv(w, b)
        L = int(w.seq_lens[b])
        for n in range(w.num_q):
            vis = L - w.num_q + n + 1
            want = v[:vis].mean(axis=0)  # [Hkv, D]
            for hq in range(w.num_q_heads):
                np.testing.assert_allclose(out[b, n, hq], want[hq // G], rtol=1e-12, atol=1e-14)


def test_dominant_key_selects_its_value():
    """One key with an overwhelming score => output equals that position's value row."""
    w = gen.tiny_chain(4, batch=1, seq_lens=np.array([33], np.int32), page_size=64,
                       num_q_heads=2, num_kv_heads=1)
    w.k_pages[:] = 0.0
    j = 11
    w.k_pages[0, 0, j] = 100.0 * np.sign(w.q[0, 0, 0])
    w.q[0] = np.abs(w.q[0, 0, 0]) * np.sign(w.q[0, 0, 0])
    out = _oracle_attn(w)
    np.testing.assert_allclose(out[0, :, :, :], np.broadcast_to(w.v_pages[0, 0, j], out[0].shape),
                               rtol=1e-9, atol=1e-9)


def test_block_table_permutation_invariance():
    w = gen.llama_chain(7, batch=2, num_q=3, num_q_heads=4, num_kv_heads=2, head_dim=8, page_size=4,
                        hidden_size=8, vocab=32, len_lo=20, len_hi=30, dtype=gen.F32)
    ref = _oracle_attn(w)
    perm = np.random.default_rng(0).permutation(w.num_pages)
    inv = np.argsort(perm)
    k2 = w.k_pages[perm]  # new slot s holds old page perm[s]
    v2 = w.v_pages[perm]
    bt2 = np.where(w.block_table >= 0, inv[np.maximum(w.block_table, 0)], -1).astype(np.int32)
    got = _oracle_attn(w, k_pages=k2, v_pages=v2, block_table=bt2)
    assert np.array_equal(got, ref)


def test_paged_equals_contiguous():
    """The same tokens in one big page per request or in 4-token pages give identical results."""
    w = gen.llama_chain(8, batch=2, num_q=3, num_q_heads=4, num_kv_heads=2, head_dim=8, page_size=4,
                        hidden_size=8, vocab=32, len_lo=9, len_hi=23, dtype=gen.F32)
    ref = _oracle_attn(w)
    big = 32
    kc = np.zeros((w.batch, w.num_kv_heads, big, w.head_dim), np.float32)
    vc = np.zeros_like(kc)
    for b in range(w.batch):
        k, v = _dense_kv(w, b)
        kc[b, :, : k.shape[0]] = k.transpose(1, 0, 2)
        vc[b, :, : v.shape[0]] = v.transpose(1, 0, 2)
    bt = np.arange(w.batch, dtype=np.int32).reshape(-1, 1)
    got = _oracle_attn(w, k_pages=kc, v_pages=vc, block_table=bt)
    assert np.array_equal(got, ref)


def test_chain_equals_tree_with_chain_parents():
    w = gen.llama_chain(9, batch=2, num_q=5, num_q_heads=4, num_kv_heads=2, head_dim=8, page_size=4,
                        hidden_size=8, vocab=32, len_lo=9, len_hi=23, dtype=gen.F32)
    assert np.array_equal(_oracle_attn(w), _oracle_attn(w, parents=gen.chain_parents(2, 5)))


def test_tree_node_ignores_non_ancestors():
    w = gen.llama_tree(11, batch=1, num_q=8, num_q_heads=2, num_kv_heads=1, head_dim=8, page_size=4,
                       hidden_size=8, vocab=32, context=21, dtype=gen.F32)
    ref = _oracle_attn(w)
    L, Nq = 21, 8
    for victim in range(1, Nq):
        k2, v2 = w.k_pages.copy(), w.v_pages.copy()
        pos = L - Nq + victim
        page = w.block_table[0, pos // 4]
        k2[page, :, pos % 4] += 3.0
        v2[page, :, pos % 4] -= 5.0
        got = _oracle_attn(w, k_pages=k2, v_pages=v2)
        for n in range(Nq):
            anc = set()
            a = n
            while a >= 0:
                anc.add(a)
                a = int(w.parents[0, a])
            same = np.array_equal(got[0, n], ref[0, n])
            assert same == (victim not in anc), (victim, n)


def test_gqa_head_mapping():
    """Query head hq must read KV head hq // G: zeroing V of one KV head zeroes exactly its group."""
    w = gen.tiny_chain(5, batch=1, seq_lens=np.array([20], np.int32), page_size=32)
    w.v_pages[:, 1] = 0.0
    out = _oracle_attn(w)
    G = w.num_q_heads // w.num_kv_heads
    assert np.all(out[:, :, G:] == 0.0) and np.all(np.abs(out[:, :, :G]).sum(-1) > 0)


def test_scale_argument():
    w = gen.tiny_chain(6, batch=1, seq_lens=np.array([20], np.int32), page_size=32)
    a = _oracle_attn(w, sm_scale=0.0)
    b = _oracle_attn(w, sm_scale=1.0 / np.sqrt(w.head_dim))
    np.testing.assert_allclose(a, b, rtol=1e-13)
    k_half = (w.k_pages * np.float32(0.5)).astype(np.float32)
    c = _oracle_attn(w, k_pages=k_half, sm_scale=2.0 / np.sqrt(w.head_dim))
    np.testing.assert_allclose(a, c, rtol=1e-12)


def test_bad_page_is_reported():
    w = gen.tiny_chain(6, batch=1, seq_lens=np.array([20], np.int32), page_size=32)
    bt = w.block_table.copy()
    bt[0, 0] = -1
    with pytest.raises(ValueError):
        _oracle_attn(w, block_table=bt)


# ---------------------------------------------------------------- LM head
@pytest.mark.parametrize("dtype", [gen.F32, gen.BF16])
def test_logits_match_float64_matmul(dtype):
    rng = np.random.default_rng(0)
    h = rng.standard_normal((7, 3, 37), dtype=np.float32)
    wt = rng.standard_normal((53, 37), dtype=np.float32) * np.float32(0.02)
    if dtype == gen.BF16:
        h, wt = gen.f32_to_bf16_bits(h), gen.f32_to_bf16_bits(wt)
    got = oracle.logits(hidden=h, lm_head=wt, dtype=dtype)
    want = gen.as_f32(h, dtype).astype(np.float64) @ gen.as_f32(wt, dtype).astype(np.float64).T
    assert got.shape == (7, 3, 53)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-15)


def test_logits_unit_rows_pick_hidden_entries():
    """W row v = e_{perm[v]} => logits[m, v] = hidden[m, perm[v]] exactly (catches a transposed W)."""
    rng = np.random.default_rng(1)
    H, V = 12, 29
    h = rng.standard_normal((5, H), dtype=np.float32)
    perm = rng.integers(0, H, size=V)
    wt = np.zeros((V, H), np.float32)
    wt[np.arange(V), perm] = 1.0
    got = oracle.logits(hidden=h, lm_head=wt, dtype=gen.F32)
    assert np.array_equal(got, h[:, perm].astype(np.float64))
