"""Pins of the 8-bit floating-point LM-head oracle (oracle_logits_fp8): the E4M3 decoding against
hand-computed values and a library conversion, the projection against a library float64 product of
library-decoded operands, and a unit-row weight that catches a transposed operand.  Paper: the
frontier targets are served in FP8 (sections 1, 4.3); the format and scaling are this build's reading."""
import numpy as np
import torch

import gen
import oracle


def test_e4m3_decoding_hand_values_and_library():
    hand = {0x00: 0.0, 0x38: 1.0, 0x40: 2.0, 0x3C: 1.5, 0x7E: 448.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9,
            0x08: 2.0 ** -6, 0xC0: -2.0, 0xB8: -1.0, 0x77: 240.0}
    codes = np.array(sorted(hand), np.uint8)
    got = oracle.decode_e4m3(codes)
    assert got.tolist() == [hand[int(c)] for c in codes]
    allc = np.arange(256, dtype=np.uint8)
    mine = oracle.decode_e4m3(allc)
    lib = torch.from_numpy(allc).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    nan = np.isnan(lib)
    assert nan.sum() == 2 and np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan], lib[~nan])
    assert np.signbit(mine[0x80]) and mine[0x80] == 0.0


def test_fp8_logits_equal_library_product_of_library_decoded_operands():
    rng = np.random.default_rng(4)
    hid, hs = gen.quantize_e4m3_rows(rng.standard_normal((3, 5, 40)).astype(np.float32))
    W, ws = gen.quantize_e4m3_rows((rng.standard_normal((23, 40)) * 0.02).astype(np.float32))
    got = oracle.logits_fp8(hidden=hid, hidden_scale=hs, lm_head=W, lm_head_scale=ws)
    hd = torch.from_numpy(hid).view(torch.float8_e4m3fn).double().numpy() * hs.astype(np.float64)[..., None]
    wd = torch.from_numpy(W).view(torch.float8_e4m3fn).double().numpy() * ws.astype(np.float64)[:, None]
    ref = hd @ wd.T
    assert got.shape == (3, 5, 23)
    assert np.allclose(got, ref, rtol=1e-13, atol=1e-15)
    # the quantised operands stay close to what they were drawn from
    assert np.abs(gen.e4m3_rows_to_f32(hid, hs)).max() <= np.abs(hd).max() + 1e-6


def test_fp8_unit_rows_select_single_products():
    H, V = 16, 16
    hid = np.arange(2 * H, dtype=np.uint8).reshape(2, H) + 0x30      # codes 0x30.. : distinct positive values
    W = np.zeros((V, H), np.uint8)
    W[np.arange(V), (np.arange(V) * 5) % H] = 0x38                   # 1.0 at column 5v mod 16
    hs = np.array([0.5, 2.0], np.float32)
    ws = np.linspace(1.0, 2.5, V).astype(np.float32)
    got = oracle.logits_fp8(hidden=hid, hidden_scale=hs, lm_head=W, lm_head_scale=ws)
    dec = oracle.decode_e4m3(hid)
    for m in range(2):
        for v in range(V):
            assert got[m, v] == float(hs[m]) * dec[m, (v * 5) % H] * float(ws[v])


def test_fp8_workload_runs_through_the_acceptance_oracle():
    w = gen.llama_chain(41, batch=4, len_lo=20, len_hi=40, vocab=600, hidden_size=128, head_fp8=True, draft_noise=0.5)
    assert w.hidden.dtype == np.uint8 and w.lm_head.dtype == np.uint8 and w.head_dtype == "fp8"
    a = oracle.accept_workload(w, want_logits=True)
    # per-row scaling keeps the dequantised logits at the magnitude of the float32 recipe (N(0,1) x N(0, 0.02))
    assert 0.05 < a.logits.std() < 0.5
    assert a.accept_len.max() >= 1


# ---- 8-bit KV cache (E4M3 codes, one float32 scale per KV head for K and for V) ---------------------------
def _fp8kv_case(seed=7, **kw):
    p = dict(batch=3, len_lo=9, len_hi=70, vocab=64, hidden_size=32, num_q_heads=6, num_kv_heads=3, head_dim=16,
             page_size=8, kv_fp8=True)
    p.update(kw)
    return gen.llama_chain(seed, **p)


def test_fp8_kv_attention_equals_attention_on_library_decoded_pools():
    """Decode the pools with the library's float8 type, apply the head's scale, run the float32 oracle path."""
    for w in (_fp8kv_case(), gen.llama_tree(8, batch=2, num_q=9, context=40, vocab=64, hidden_size=32, num_q_heads=4,
                                           num_kv_heads=2, head_dim=16, kv_fp8=True)):
        assert w.k_pages.dtype == np.uint8 and w.kv_dtype == "fp8" and w.k_scale.shape == (w.num_kv_heads,)
        assert len(set(w.k_scale.tolist())) > 1, "the heads' scales must differ for this pin to see a wrong head index"
        got = oracle.attn_workload(w)
        kd = torch.from_numpy(w.k_pages).view(torch.float8_e4m3fn).float().numpy() * w.k_scale[None, :, None, None]
        vd = torch.from_numpy(w.v_pages).view(torch.float8_e4m3fn).float().numpy() * w.v_scale[None, :, None, None]
        # the float32 products scale * decode are exact in float64 as well only up to one rounding: compare loosely,
        # then exactly against a float64 product formed here
        ref32 = oracle.attn(q=gen.as_f32(w.q, w.dtype), k_pages=kd, v_pages=vd, block_table=w.block_table,
                            seq_lens=w.seq_lens, parents=w.parents, dtype="f32")
        assert np.allclose(got, ref32, rtol=1e-5, atol=1e-6)


def test_fp8_kv_equal_keys_give_the_mean_of_the_decoded_values():
    w = _fp8kv_case(11, batch=2)
    k = np.full_like(w.k_pages, 0x3A)           # every key identical: softmax is uniform over what is visible
    o = oracle.attn(q=w.q, k_pages=k, v_pages=w.v_pages, block_table=w.block_table, seq_lens=w.seq_lens, dtype=w.dtype,
                    k_scale=w.k_scale, v_scale=w.v_scale)
    dec = oracle.decode_e4m3(w.v_pages)
    G = w.num_q_heads // w.num_kv_heads
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        for n in range(w.num_q):
            vis = L - w.num_q + n + 1           # chain: the prefix and the chunk slots up to its own
            for hq in range(w.num_q_heads):
                hk = hq // G
                rows = [dec[w.block_table[b, j // w.page_size], hk, j % w.page_size] for j in range(vis)]
                want = float(w.v_scale[hk]) * np.mean(rows, axis=0)
                assert np.allclose(o[b, n, hq], want, rtol=1e-12, atol=1e-14)


def test_fp8_kv_scales_act_where_the_definition_says():
    w = _fp8kv_case(13)
    base = oracle.attn_workload(w)
    args = dict(q=w.q, k_pages=w.k_pages, v_pages=w.v_pages, block_table=w.block_table, seq_lens=w.seq_lens,
                dtype=w.dtype)
    s0 = 1.0 / np.sqrt(w.head_dim)
    # K scale and softmax scale enter as a product; V scale is linear in the output - per head
    twice = oracle.attn(**args, k_scale=w.k_scale * 2, v_scale=w.v_scale, sm_scale=s0 / 2)
    assert np.allclose(twice, base, rtol=1e-12, atol=1e-14)
    vs = w.v_scale.copy()
    vs[1] *= 4
    scaled = oracle.attn(**args, k_scale=w.k_scale, v_scale=vs)
    G = w.num_q_heads // w.num_kv_heads
    for hq in range(w.num_q_heads):
        f = 4.0 if hq // G == 1 else 1.0
        assert np.allclose(scaled[:, :, hq], f * base[:, :, hq], rtol=1e-12, atol=1e-14)


def test_fp8_kv_quantisation_error_is_within_the_format_bound():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((7, 3, 8, 16)).astype(np.float32)
    codes, scale = gen.quantize_e4m3_heads(x)
    back = oracle.decode_e4m3(codes) * scale.astype(np.float64)[None, :, None, None]
    # round to nearest with 3 mantissa bits: relative error <= 2^-4 for normal codes, absolute 2^-10 * scale below
    err = np.abs(back - x)
    bound = np.maximum(np.abs(x) * 2.0 ** -4, scale.astype(np.float64)[None, :, None, None] * 2.0 ** -10)
    assert (err <= bound * (1 + 1e-6)).all()
    assert int((codes & 0x7F).max()) == 0x7E  # the largest magnitude of a head maps to 448, the top code
