"""The seeded generators: determinism, layout, and the acceptance statistics their recipes imply
(checked through the oracle, as sanity pins on both)."""
import numpy as np
from scipy.stats import norm

import gen
import oracle


def test_bf16_round_trip_matches_torch():
    import torch
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 3
    x[:4] = [1.0, 1.00390625, 1.01171875, -0.0]  # includes exact ties (round to even)
    bits = gen.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), want.view(torch.int16).numpy())
    assert np.array_equal(gen.bf16_bits_to_f32(bits), want.float().numpy())


def test_deterministic_and_seed_sensitive():
    a = gen.llama_chain(1, batch=3, vocab=512, hidden_size=64, len_lo=20, len_hi=60)
    b = gen.llama_chain(1, batch=3, vocab=512, hidden_size=64, len_lo=20, len_hi=60)
    c = gen.llama_chain(2, batch=3, vocab=512, hidden_size=64, len_lo=20, len_hi=60)
    for f in ("q", "k_pages", "v_pages", "block_table", "seq_lens", "hidden", "lm_head", "draft_tokens",
              "draft_probs", "uniforms"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f
    assert not np.array_equal(a.hidden, c.hidden)


def test_layout_and_block_table():
    w = gen.llama_chain(1, batch=5, vocab=512, hidden_size=64, len_lo=20, len_hi=200)
    assert w.q.shape == (5, 5, 32, 128) and w.q.dtype == np.uint16
    assert w.k_pages.shape == (w.num_pages, 8, 16, 128)
    used = w.block_table[w.block_table >= 0]
    assert len(np.unique(used)) == len(used) and used.max() < w.num_pages
    per = (w.seq_lens + 15) // 16
    assert ((w.block_table >= 0).sum(1) == per).all()
    assert np.allclose(w.draft_probs.sum(-1), 1.0, atol=1e-5)
    assert w.uniforms.min() >= 0 and w.uniforms.max() < 1
    assert np.array_equal(w.uniforms, np.round(w.uniforms * 2 ** 24) / 2 ** 24)


def test_tiny_config_shapes():
    w = gen.tiny_chain(1)
    assert (w.batch, w.num_q, w.vocab, w.hidden_size, w.page_size) == (4, 5, 1024, 256, 256)
    assert w.k_pages.shape == (4, 2, 256, 64) and w.k_pages.dtype == np.float32
    assert np.array_equal(w.block_table[:, 0], np.arange(4))


def test_tree_constraints():
    w = gen.llama_tree(1, batch=6, vocab=256, hidden_size=32, context=64)
    for b in range(w.batch):
        par = w.parents[b]
        assert par[0] == -1 and (par[1:] < np.arange(1, 32)).all() and (par[1:] >= 0).all()
        depth = np.zeros(32, int)
        for n in range(1, 32):
            depth[n] = depth[par[n]] + 1
        assert depth.max() <= 6 and np.bincount(par[1:]).max() <= 4


def test_sparse_pool_block_table_maps_to_compact_slots():
    w = gen.stress_chain(1, batch=6, vocab=256, hidden_size=32, len_lo=16, len_hi=200, pool_pages=5000)
    assert w.k_pages.shape[0] == len(w.page_ids) < 5000 and w.num_pages == 5000
    hb = w.host_block_table()
    ok = w.block_table >= 0
    assert np.array_equal(w.page_ids[hb[ok]], w.block_table[ok])
    assert (hb[~ok] == -1).all()


def test_noisy_target_recipe_gives_the_predicted_acceptance_rate():
    """q ~ p * exp(N(0, s^2)) over a large vocabulary => alpha -> 2 * Phi(-s/2) (0.617 at s = 1);
    chain of k = 4 then keeps sum_{i=1..4} alpha^i = 1.38 drafts on average (eq. 1 minus one)."""
    w = gen.llama_chain(1, batch=384, num_q_heads=2, num_kv_heads=1, head_dim=8, vocab=8192,
                        hidden_size=64, len_lo=8, len_hi=16)
    r = oracle.accept(hidden=w.hidden, lm_head=w.lm_head, draft_tokens=w.draft_tokens,
                      draft_probs=w.draft_probs, uniforms=w.uniforms, dtype=w.dtype, temperature=1.0)
    alpha = 2 * norm.cdf(-0.5)
    want = sum(alpha ** i for i in range(1, 5))
    assert abs(r.accept_len.mean() - want) < 4 * r.accept_len.std() / np.sqrt(w.batch) + 0.05


def test_greedy_mix_recipe_gives_geometric_acceptance():
    """Draft = arg-max w.p. 0.7 => E[accept_len] = sum_{i=1..6} 0.7^i = 2.059 (eq. 1, alpha .7, gamma 6)."""
    w = gen.qwen_greedy_chain(1, batch=512, num_q_heads=2, num_kv_heads=1, head_dim=8, vocab=4096,
                              hidden_size=64, len_lo=8, len_hi=16)
    assert w.draft_probs is None and w.uniforms is None and w.temperature == 0.0
    r = oracle.accept(hidden=w.hidden, lm_head=w.lm_head, draft_tokens=w.draft_tokens, dtype=w.dtype,
                      temperature=0.0)
    want = sum(0.7 ** i for i in range(1, 7))
    assert abs(r.accept_len.mean() - want) < 4 * r.accept_len.std() / np.sqrt(w.batch)
