"""Trace emission on the GPU against the oracle, through the C ABI: top-K target logits per token
row (bit-exact: the answer is unique), y_out and the rejection trajectory (integer logic), and the
whole chain verify -> emit.  Paper: section 3.1, appendix A.1 eq. 4, appendix A.2."""
import numpy as np
import pytest
import torch

import gen
import oracle

pytestmark = pytest.mark.gpu


def _emit_topk(av, logits, k, d2t=None):
    rows, V = logits.shape
    dmap = None if d2t is None else torch.from_numpy(d2t).cuda()
    d = av.aurora_trace_desc(batch=rows, num_q=1, vocab=V, top_k=k, draft_vocab=0 if d2t is None else len(d2t),
                             draft_to_target=None if d2t is None else dmap.data_ptr())
    dl = torch.from_numpy(logits).cuda()
    ids = torch.full((rows, k), -9, dtype=torch.int32, device="cuda")
    vals = torch.full((rows, k), 0x1234, dtype=torch.int16, device="cuda")
    av.aurora_trace_emit(d, dl, None, None, None, None, ids, vals, None, None)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), vals.cpu().numpy().view(np.uint16)


def _check_topk(av, logits, k, d2t=None):
    print(f"[case] top-k rows={logits.shape[0]} V={logits.shape[1]} K={k} "
          f"draft_vocab={None if d2t is None else len(d2t)}", flush=True)
    ids, vals = _emit_topk(av, logits, k, d2t)
    rid, rvals = oracle.trace_topk(logits, k, d2t)
    assert np.array_equal(ids, rid), f"first mismatch at {np.argwhere(ids != rid)[:3].tolist()}"
    assert np.array_equal(vals, rvals)


@pytest.mark.parametrize("kind", gen.TRACE_KINDS)
def test_topk_value_distributions(gpu_lib, kind):
    """Roughly normal logits take the one-pass route; repeated values, constant rows, masked
    vocabularies and signed zeros overflow or starve the candidate list and take the exact route."""
    _check_topk(gpu_lib, gen.trace_logits(21, 6, 50001, kind), 1000)   # odd V: rows not 16-byte aligned


@pytest.mark.parametrize("vocab,k", [(1, 1), (1, 8), (700, 1024), (3000, 1024), (4096, 1024), (4097, 1024),
                                     (4100, 1), (9999, 17), (128256, 1)])
def test_topk_sizes(gpu_lib, vocab, k):
    """Rows shorter than K (padded), rows that fit the candidate list whole, the first size that does
    not, K = 1."""
    for kind in ("normal", "ties"):
        _check_topk(gpu_lib, gen.trace_logits(22, 3, vocab, kind), k)


def test_topk_full_size_llama_vocab(gpu_lib):
    """The benchmark's shape: 160 token rows of the 128256-entry vocabulary, K = 1024."""
    _check_topk(gpu_lib, gen.trace_logits(1, 160, 128256, "normal"), 1024)


@pytest.mark.parametrize("vocab,draft_vocab,k", [(128256, 32000, 1024), (50001, 4097, 1000), (20000, 3000, 1024),
                                                 (9999, 500, 1024), (151936, 32003, 1024)])
def test_topk_over_the_draft_vocabulary(gpu_lib, vocab, draft_vocab, k):
    """Selection restricted to the draft model's vocabulary (a sorted random subset of target ids, or an
    unsorted one): ids are positions in the subset."""
    rng = np.random.default_rng([vocab, draft_vocab])
    d2t = np.sort(rng.choice(vocab, size=draft_vocab, replace=False)).astype(np.int32)
    for kind in ("normal", "ties", "masked"):
        _check_topk(gpu_lib, gen.trace_logits(25, 4, vocab, kind), k, d2t)
    _check_topk(gpu_lib, gen.trace_logits(26, 3, vocab, "normal"), k, rng.permutation(d2t).astype(np.int32))


def _group_max(logits, group=32, pad_groups=0):
    """Maxima of consecutive groups of `group` entries per row (numpy; -inf pads the last group and `pad_groups`
    further ones, as the LM head pads its rows to whole tiles)."""
    rows, V = logits.shape
    n = (V + group - 1) // group
    x = np.full((rows, (n + pad_groups) * group), -np.inf, np.float32)
    x[:, :V] = logits
    return np.ascontiguousarray(x.reshape(rows, n + pad_groups, group).max(-1))


def _emit_topk_with_groups(av, logits, k, gmax):
    rows, V = logits.shape
    dg = torch.from_numpy(gmax).cuda()
    d = av.aurora_trace_desc(batch=rows, num_q=1, vocab=V, top_k=k, n_groups=gmax.shape[1], group_max=dg.data_ptr())
    dl = torch.from_numpy(logits).cuda()
    ids = torch.full((rows, k), -9, dtype=torch.int32, device="cuda")
    vals = torch.full((rows, k), 0x1234, dtype=torch.int16, device="cuda")
    av.aurora_trace_emit(d, dl, None, None, None, None, ids, vals, None, None)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), vals.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("kind", gen.TRACE_KINDS)
@pytest.mark.parametrize("vocab,k,pad", [(128256, 1024, 0), (50001, 1000, 5), (151936, 1024, 0), (40000, 300, 2),
                                         (32768, 1024, 0), (32737, 1024, 0), (262144, 1024, 0), (262145, 1024, 0),
                                         (20000, 1024, 0)])
def test_topk_with_group_maxima(gpu_lib, kind, vocab, k, pad):
    """The route that takes its cut-off from the maxima of groups of 32 consecutive ids (made here with numpy from the
    same seeded rows) and gathers only the groups that reach it.  All value kinds (ties and constant rows overflow
    the list and fall back to the whole-row route), rows that are not 16-byte aligned and end inside a group, exactly
    K groups (32768 / 32 and the ragged 32737), the largest vocabulary the route takes (8192 groups) and the first
    it does not, fewer groups than K (ignored), rows of maxima padded with -inf as the LM head pads them."""
    x = gen.trace_logits(31, 5, vocab, kind)
    print(f"[case] top-k with group maxima rows=5 V={vocab} K={k} pad={pad} kind={kind}", flush=True)
    ids, vals = _emit_topk_with_groups(gpu_lib, x, k, _group_max(x, 32, pad))
    rid, rvals = oracle.trace_topk(x, k)
    assert np.array_equal(ids, rid), f"first mismatch at {np.argwhere(ids != rid)[:3].tolist()}"
    assert np.array_equal(vals, rvals)


def test_topk_with_group_maxima_full_size(gpu_lib):
    """The benchmark's shape (160 rows x 128256, K = 1024), and 600 rows (two workgroups per compute unit)."""
    x = gen.trace_logits(2, 600, 50016, "normal")
    ids, vals = _emit_topk_with_groups(gpu_lib, x, 1024, _group_max(x))
    rid, rvals = oracle.trace_topk(x, 1024)
    assert np.array_equal(ids, rid) and np.array_equal(vals, rvals)
    x = gen.trace_logits(1, 160, 128256, "normal")
    ids, vals = _emit_topk_with_groups(gpu_lib, x, 1024, _group_max(x))
    rid, rvals = oracle.trace_topk(x, 1024)
    assert np.array_equal(ids, rid) and np.array_equal(vals, rvals)


@pytest.mark.parametrize("fill", [np.inf, -np.inf, 0.0, 1e30])
def test_topk_survives_group_maxima_that_are_uniformly_wrong(gpu_lib, fill):
    """The same wrong value in every group (a buffer that was never filled): too high a cut-off leaves the list
    short, too low a one overflows it, and both take the whole-row route - the result is still exact."""
    x = gen.trace_logits(32, 4, 50001, "normal")
    g = np.full((4, (50001 + 31) // 32), fill, np.float32)
    ids, vals = _emit_topk_with_groups(gpu_lib, x, 1024, g)
    rid, rvals = oracle.trace_topk(x, 1024)
    assert np.array_equal(ids, rid) and np.array_equal(vals, rvals)


def test_topk_qwen_vocab_with_ties(gpu_lib):
    _check_topk(gpu_lib, gen.trace_logits(2, 8, 151936, "ties"), 1024)


@pytest.mark.parametrize("tree", [False, True])
def test_records_from_acceptance_outputs(gpu_lib, tree):
    w = gen.llama_chain(23, batch=40, num_q=7, len_lo=20, len_hi=40, vocab=300, hidden_size=64, num_q_heads=2,
                        num_kv_heads=1, head_dim=64) if not tree else gen.llama_tree(
        23, batch=40, num_q=24, vocab=300, hidden_size=64, context=48, num_q_heads=2, num_kv_heads=1, head_dim=64)
    a = oracle.accept(hidden=w.hidden, lm_head=w.lm_head, draft_tokens=w.draft_tokens, draft_probs=w.draft_probs,
                      uniforms=w.uniforms, parents=w.parents, dtype=w.dtype, temperature=w.temperature)
    ry, rr = oracle.trace_records(draft_tokens=w.draft_tokens, parents=w.parents, next_token=a.next_token,
                                  accept_mask=a.accept_mask)
    av = gpu_lib
    B, Nq = w.draft_tokens.shape
    d = av.aurora_trace_desc(batch=B, num_q=Nq, vocab=w.vocab, top_k=1)
    dev = lambda x: None if x is None else torch.from_numpy(np.ascontiguousarray(x)).cuda()
    y = torch.full((B, Nq), -9, dtype=torch.int32, device="cuda")
    r = torch.full((B, Nq), -9, dtype=torch.int8, device="cuda")
    av.aurora_trace_emit(d, None, dev(w.draft_tokens), dev(w.parents), dev(a.next_token), dev(a.accept_mask), None,
                         None, y, r)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), ry)
    assert np.array_equal(r.cpu().numpy(), rr)
    assert (rr == 2).any() and (rr == 0).any()


def test_verify_then_emit(gpu_lib):
    """The whole chain: verify on the GPU, then emit from the logits it left in the workspace and its own
    acceptance outputs.  The GPU's fp32 logits differ from the oracle's in the last bits (tolerance 1e-3,
    as for the logits themselves), so ids may differ where values are closer than that: the kept values
    must agree rank by rank within that tolerance plus bfloat16 rounding, and every id the two sides
    disagree on must sit within the tolerance of the K-th value."""
    from paper_2602_06932_amd.device import DeviceVerify
    av = gpu_lib
    w = gen.llama_chain(24, batch=6, len_lo=30, len_hi=90, vocab=20011, hidden_size=256)
    dv = DeviceVerify(w)
    dv.verify()
    B, Nq, V, K = w.batch, w.num_q, w.vocab, 1024
    d = av.aurora_trace_desc(batch=B, num_q=Nq, vocab=V, top_k=K)
    lp = av.aurora_verify_logits_ptr(dv.attn_desc, dv.accept_desc, dv.workspace)
    ids = torch.empty((B * Nq, K), dtype=torch.int32, device="cuda")
    vals = torch.empty((B * Nq, K), dtype=torch.int16, device="cuda")
    y = torch.empty((B, Nq), dtype=torch.int32, device="cuda")
    r = torch.empty((B, Nq), dtype=torch.int8, device="cuda")
    av.aurora_trace_emit(d, lp, dv.draft_tokens, dv.parents, dv.next_token, dv.accept_mask, ids, vals, y, r)
    torch.cuda.synchronize()
    res = dv.results_host()
    # records: integer logic on the GPU's own acceptance outputs
    ry, rr = oracle.trace_records(draft_tokens=w.draft_tokens, parents=w.parents, next_token=res["next_token"],
                                  accept_mask=res["accept_mask"])
    assert np.array_equal(y.cpu().numpy(), ry) and np.array_equal(r.cpu().numpy(), rr)
    # top-K against the oracle's own logits
    ref = oracle.logits(hidden=w.hidden, lm_head=w.lm_head, dtype=w.dtype).reshape(B * Nq, V)
    rid, rvals = oracle.trace_topk(ref.astype(np.float32), K)
    gid = ids.cpu().numpy()
    gv = gen.bf16_bits_to_f32(vals.cpu().numpy().view(np.uint16))
    rv = gen.bf16_bits_to_f32(rvals)
    tol = 1e-3
    assert np.all(np.abs(gv - rv) <= tol + np.abs(rv) * 2.0 ** -7)
    for m in range(B * Nq):
        kth = ref[m, rid[m, -1]]
        diff = np.setxor1d(gid[m], rid[m])
        assert np.all(np.abs(ref[m, diff] - kth) <= 2 * tol), (m, diff[:5])
    assert len(np.setxor1d(gid, rid)) < 0.01 * gid.size


@pytest.mark.parametrize("case", ["chain", "tree", "fp8", "many_rows"])
def test_group_maxima_from_the_lm_head_give_the_same_records(gpu_lib, case):
    """verify -> emit with the group maxima the LM head left in the workspace against verify -> emit without them
    (the sampling route): identical ids and values, and the maxima themselves equal the largest fp32 logit of every
    32 consecutive ids (chain: the W-streaming kernel; tree / many rows: the tiled kernel; 8-bit head)."""
    from paper_2602_06932_amd.device import DeviceVerify
    av = gpu_lib
    if case == "chain":
        w = gen.llama_chain(27, batch=6, len_lo=30, len_hi=90, vocab=50011, hidden_size=256)
    elif case == "tree":
        w = gen.llama_tree(27, batch=14, num_q=32, vocab=40003, hidden_size=128, context=48, num_q_heads=4, num_kv_heads=2)
    elif case == "fp8":
        w = gen.llama_chain(27, batch=6, len_lo=30, len_hi=90, vocab=50011, hidden_size=256, head_fp8=True)
    else:
        w = gen.llama_chain(27, batch=90, len_lo=20, len_hi=40, vocab=40003, hidden_size=128, num_q_heads=4, num_kv_heads=2)
    dv = DeviceVerify(w)
    dv.verify()
    torch.cuda.synchronize()
    gptr, ng = av.aurora_verify_group_max_ptr(dv.attn_desc, dv.accept_desc, dv.workspace)
    assert gptr and ng == (w.vocab + 255) // 256 * 8
    rows = w.batch * w.num_q
    lg = dv.logits_host().reshape(rows, w.vocab)
    off = gptr - dv.workspace.data_ptr()
    gm = dv.workspace[off:off + 4 * rows * ng].view(torch.float32).view(rows, ng).cpu().numpy()
    want = _group_max(lg)
    assert np.array_equal(gm[:, :want.shape[1]], want) and np.all(gm[:, want.shape[1]:] == -np.inf)
    dv.trace(group_max=True)
    torch.cuda.synchronize()
    a = (dv.topk_ids.cpu().numpy().copy(), dv.topk_logits.cpu().numpy().copy())
    dv.topk_ids.fill_(-5)
    dv.trace(group_max=False)
    torch.cuda.synchronize()
    b = (dv.topk_ids.cpu().numpy(), dv.topk_logits.cpu().numpy())
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_verify_emit_pack_loss_replay_from_one_captured_graph(gpu_lib):
    """The serving-side sequence verify -> emit -> pack and the training-side loss on the emitted rows, captured as
    ONE graph (none of the calls allocates or records a memset) and replayed with eager work in between: every
    replay gives the eager sequence's bits."""
    from paper_2602_06932_amd.device import DeviceVerify
    av = gpu_lib
    w = gen.llama_chain(26, batch=6, len_lo=30, len_hi=90, vocab=20011, hidden_size=256)
    dv = DeviceVerify(w)
    B, Nq, V, K = w.batch, w.num_q, w.vocab, 256
    M = B * Nq
    td = av.aurora_trace_desc(batch=B, num_q=Nq, vocab=V, top_k=K)
    pd = av.aurora_pack_desc(rows=M, top_k=K, h_row_bytes=0)
    ld = av.aurora_loss_desc(rows=M, draft_vocab=V, top_k=K, discard_top_k=16, lambda_discard=0.5)
    lp = av.aurora_verify_logits_ptr(dv.attn_desc, dv.accept_desc, dv.workspace)
    dev = lambda shape, dt: torch.zeros(shape, dtype=dt, device="cuda")
    ids, vals, y, r = dev((M, K), torch.int32), dev((M, K), torch.int16), dev((B, Nq), torch.int32), dev((B, Nq), torch.int8)
    n_out, row_index = dev((1,), torch.int32), dev((M,), torch.int32)
    ids_p, vals_p, y_p, r_p = dev((M, K), torch.int32), dev((M, K), torch.int16), dev((M,), torch.int32), dev((M,), torch.int8)
    z = torch.randn((M, V), device="cuda", generator=torch.Generator(device="cuda").manual_seed(5))
    row_kl, loss, grad = dev((M,), torch.float32), dev((5,), torch.float32), dev((M, V), torch.float32)
    outs = (ids, vals, y, r, n_out, row_index, ids_p, vals_p, y_p, r_p, row_kl, loss, grad)

    def sequence(stream=None):
        dv.verify(stream=stream)
        av.aurora_trace_emit(td, lp, dv.draft_tokens, dv.parents, dv.next_token, dv.accept_mask, ids, vals, y, r, stream=stream)
        av.aurora_trace_pack(pd, r.view(-1), None, ids, vals, None, y.view(-1), n_out, row_index, None, ids_p, vals_p, None, y_p,
                             r_p, stream=stream)
        av.aurora_draft_loss(ld, z, ids, vals, r.view(-1), row_kl, loss, grad, stream=stream)

    sequence()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]
    assert 0 < int(n_out.item()) <= M and torch.isfinite(loss).all()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sequence(stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for i in range(3):
        for t in outs:
            t.fill_(1)
        graph.replay()
        torch.cuda.synchronize()
        n = int(n_out.item())
        for k, (a, b) in enumerate(zip(ref, outs)):
            if k in (6, 7, 8, 9):   # packed arrays: positions from n on are not written
                a, b = a[:n], b[:n]
            elif k == 5:
                a, b = a[:n], b[:n]
            assert torch.equal(a, b), (i, k)
        dv.accept()  # eager work on the verify workspace between replays
        torch.cuda.synchronize()
