"""Pins of the trace-emission oracle (oracle/trace_oracle.c) against things other than itself:
brute-force selection, closed forms, hand-computed bfloat16 bit patterns, a library float32 ->
bfloat16 conversion, hand-worked trajectories, and consistency with the acceptance oracle.
Paper: section 3.1 (accepted and rejected outcomes are streamed), appendix A.1 eq. 4 (record
(h, l, x_in, y_out, R)), appendix A.2 (top-K logit filtering, K = 1024, 2 KB per token)."""
import struct

import numpy as np
import pytest
import torch

import gen
import oracle


def _brute_topk(row, k):
    """K rounds of 'largest remaining value, lowest id among equals' - no sorting involved."""
    taken = [False] * len(row)
    out = []
    for _ in range(min(k, len(row))):
        best = -1
        for i, x in enumerate(row):
            if taken[i]:
                continue
            if best < 0 or x > row[best]:
                best = i
        taken[best] = True
        out.append(best)
    return out + [-1] * (k - len(out))


@pytest.mark.parametrize("seed", range(6))
def test_topk_matches_brute_force_with_ties(seed):
    rng = np.random.default_rng(seed)
    V = int(rng.integers(1, 60))
    k = int(rng.integers(1, 70))
    # few distinct values => many ties; include signed zeros and -inf
    pool = np.array([-np.inf, -2.5, -0.0, 0.0, 0.5, 0.5000001, 3.0, 1e30], np.float32)
    x = pool[rng.integers(0, len(pool), size=(5, V))]
    ids, vals = oracle.trace_topk(x, k)
    for m in range(x.shape[0]):
        want = _brute_topk([float(t) for t in x[m]], k)
        assert ids[m].tolist() == want


def test_topk_over_a_sub_vocabulary_matches_brute_force_on_the_gathered_row():
    rng = np.random.default_rng(3)
    x = rng.integers(-5, 6, size=(4, 50)).astype(np.float32)   # many ties
    d2t = rng.permutation(50)[:17].astype(np.int32)
    ids, vals = oracle.trace_topk(x, 9, d2t)
    for m in range(4):
        assert ids[m].tolist() == _brute_topk([float(t) for t in x[m, d2t]], 9)
        assert np.array_equal(gen.bf16_bits_to_f32(vals[m]), x[m, d2t[ids[m]]])


def test_topk_of_a_permutation_is_the_permutation_prefix():
    rng = np.random.default_rng(11)
    V, k = 5000, 1024
    perm = rng.permutation(V)
    row = np.empty(V, np.float32)
    row[perm] = np.arange(V, 0, -1, dtype=np.float32) * 0.25  # perm[0] holds the largest value, ...
    ids, vals = oracle.trace_topk(row[None, :], k)
    assert ids[0].tolist() == perm[:k].tolist()
    # stored values are within half a bfloat16 ulp (relative 2^-8 bound) of the selected float32 values
    back = gen.bf16_bits_to_f32(vals[0])
    assert np.all(np.abs(back - row[perm[:k]]) <= np.abs(row[perm[:k]]) * 2.0 ** -8)


def test_all_equal_row_keeps_lowest_ids_and_short_rows_are_padded():
    ids, vals = oracle.trace_topk(np.full((2, 300), 1.5, np.float32), 7)
    assert ids.tolist() == [list(range(7))] * 2
    ids, vals = oracle.trace_topk(np.array([[2.0, -1.0, 7.0]], np.float32), 5)
    assert ids[0].tolist() == [2, 0, 1, -1, -1]
    assert vals[0].tolist() == [0x40E0, 0x4000, 0xBF80, 0xFF80, 0xFF80]


def test_signed_zeros_tie_and_minus_inf_ranks_last():
    x = np.array([[-np.inf, -0.0, 0.0, -1.0, -np.inf, 0.0]], np.float32)
    ids, vals = oracle.trace_topk(x, 6)
    assert ids[0].tolist() == [1, 2, 5, 3, 0, 4]
    assert vals[0, 4] == 0xFF80 and vals[0, 5] == 0xFF80


def test_nan_is_rejected():
    with pytest.raises(ValueError):
        oracle.trace_topk(np.array([[0.0, np.nan]], np.float32), 1)


def _f32(bits):
    return struct.unpack("<f", struct.pack("<I", bits))[0]


def test_bf16_rounding_hand_computed_patterns():
    cases = [
        (0x3F800000, 0x3F80),  # 1.0
        (0x3F808000, 0x3F80),  # halfway, keep even
        (0x3F818000, 0x3F82),  # halfway, round up to even
        (0x3F808001, 0x3F81),  # just above halfway
        (0x3F807FFF, 0x3F80),  # just below halfway
        (0xBF818000, 0xBF82),  # sign does not matter
        (0x7F7FFFFF, 0x7F80),  # largest float32 rounds to +inf
        (0x7F7F7FFF, 0x7F7F),  # largest bfloat16 stays
        (0x00000001, 0x0000),  # smallest subnormal rounds to zero
        (0x00018000, 0x0002),  # subnormal halfway, to even
        (0x7F800000, 0x7F80),  # +inf
        (0xFF800000, 0xFF80),  # -inf
        (0x80000000, 0x8000),  # -0.0 keeps its sign bit in the stored value
    ]
    row = np.array([_f32(b) for b, _ in cases], np.float32)
    for i, (_, want) in enumerate(cases):
        ids, vals = oracle.trace_topk(row[i:i + 1][None, :], 1)
        assert vals[0, 0] == want, (hex(cases[i][0]), hex(int(vals[0, 0])), hex(want))


def test_bf16_rounding_equals_library_conversion():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(4096) * np.exp(rng.uniform(-30, 30, 4096))).astype(np.float32)
    ids, vals = oracle.trace_topk(x[None, :], x.size)
    lib = torch.from_numpy(x[ids[0]]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(vals[0], lib)


def test_records_hand_worked_chain():
    tok = np.array([[0, 5, 6, 7, 8]] * 3, np.int32)
    mask = np.array([[1, 1, 1, 0, 0], [1, 1, 1, 1, 1], [1, 0, 0, 0, 0]], np.uint8)
    nxt = np.array([42, 43, 44], np.int32)
    y, r = oracle.trace_records(draft_tokens=tok, parents=None, next_token=nxt, accept_mask=mask)
    assert y.tolist() == [[5, 6, 42, -1, -1], [5, 6, 7, 8, 43], [44, -1, -1, -1, -1]]
    assert r.tolist() == [[1, 1, 1, 2, 0], [1, 1, 1, 1, 1], [1, 2, 0, 0, 0]]


def test_records_hand_worked_tree():
    #        0
    #      /   \
    #     1     2        children of 0 tried in order 1, 2; 1 rejected, 2 kept
    #    / \     \
    #   3   4     5      5 tried and rejected; 3, 4 never tested
    parents = np.array([[-1, 0, 0, 1, 1, 2]], np.int32)
    tok = np.array([[0, 11, 12, 13, 14, 15]], np.int32)
    mask = np.array([[1, 0, 1, 0, 0, 0]], np.uint8)
    y, r = oracle.trace_records(draft_tokens=tok, parents=parents, next_token=np.array([99], np.int32),
                                accept_mask=mask)
    assert y.tolist() == [[12, -1, 99, -1, -1, -1]]
    assert r.tolist() == [[1, 2, 1, 0, 0, 2]]
    # first child kept: its later sibling is never tested
    mask = np.array([[1, 1, 0, 0, 1, 0]], np.uint8)
    y, r = oracle.trace_records(draft_tokens=tok, parents=parents, next_token=np.array([98], np.int32),
                                accept_mask=mask)
    assert y.tolist() == [[11, 14, -1, -1, 98, -1]]
    assert r.tolist() == [[1, 1, 0, 2, 1, 0]]


@pytest.mark.parametrize("tree", [False, True])
def test_records_are_consistent_with_the_acceptance_oracle(tree):
    w = gen.tiny_chain(3) if not tree else gen.llama_tree(
        2, batch=6, num_q=12, vocab=400, hidden_size=32, context=40, num_q_heads=2, num_kv_heads=1, head_dim=16)
    a = oracle.accept(hidden=w.hidden, lm_head=w.lm_head, draft_tokens=w.draft_tokens, draft_probs=w.draft_probs,
                      uniforms=w.uniforms, parents=w.parents, dtype=w.dtype, temperature=w.temperature)
    y, r = oracle.trace_records(draft_tokens=w.draft_tokens, parents=w.parents, next_token=a.next_token,
                                accept_mask=a.accept_mask)
    B, Nq = w.draft_tokens.shape
    for b in range(B):
        on = np.flatnonzero(r[b] == 1)
        assert np.array_equal(on, np.flatnonzero(a.accept_mask[b]))
        assert len(on) == a.accept_len[b] + 1
        assert (y[b] >= 0).sum() == len(on) and np.all(y[b][r[b] != 1] == -1)
        # emitted tokens in path order: the accepted drafts, then the corrected / bonus token
        emitted = [int(y[b, n]) for n in on]
        assert emitted[:-1] == [int(w.draft_tokens[b, n]) for n in on[1:]]
        assert emitted[-1] == int(a.next_token[b])
        for c in np.flatnonzero(r[b] == 2):
            par = c - 1 if w.parents is None else int(w.parents[b, c])
            assert r[b, par] == 1
        if not tree:
            assert (r[b] == 2).sum() == (1 if a.accept_len[b] < Nq - 1 else 0)
