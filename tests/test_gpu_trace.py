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
