"""Parity of the attention backward pass (paper section 3.1: the speculative tree goes through one batched forward and
backward pass) against the float64 oracle, through the C ABI.

Tolerances.  bf16 storage: p and the dot products are formed in fp32 from the bf16 inputs; delta uses the forward
output rounded to bf16 (relative 2^-9), so dS carries a relative error of that order on top of the fp32 sums;
gradients are compared like the forward output - absolute 2e-2 of the tensor's largest magnitude and relative RMS
1e-2.  fp32 storage: 2e-5 of the largest magnitude."""
import numpy as np
import pytest
import torch

import gen
import oracle

pytestmark = pytest.mark.gpu


def _run(w, dout):
    import paper_2602_06932_amd as av
    from paper_2602_06932_amd.device import DeviceVerify, _to_dev
    dv = DeviceVerify(w)
    d_dout = _to_dev(dout, w.dtype)
    dq = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device="cuda")
    dk = torch.zeros(dv.k_pages.shape, dtype=torch.float32, device="cuda")
    dvp = torch.zeros(dv.v_pages.shape, dtype=torch.float32, device="cuda")
    ws = torch.empty(av.aurora_attn_backward_workspace_bytes(dv.attn_desc), dtype=torch.uint8, device="cuda")
    av.aurora_attn_backward(dv.attn_desc, dv.q, dv.k_pages, dv.v_pages, dv.block_table, dv.seq_lens, dv.parents, d_dout,
                            dq, dk, dvp, ws)
    torch.cuda.synchronize()
    return dq.cpu().numpy(), dk.cpu().numpy(), dvp.cpu().numpy()


def _check(w, seed=0):
    print(f"[case] {w.name} B={w.batch} Nq={w.num_q} heads={w.num_q_heads}/{w.num_kv_heads}/{w.head_dim} "
          f"L={int(w.seq_lens.min())}..{int(w.seq_lens.max())} page={w.page_size} {w.dtype}", flush=True)
    rng = np.random.default_rng(seed)
    g32 = rng.standard_normal(w.q.shape).astype(np.float32)
    if w.dtype == "bf16":
        dout = (g32.view(np.uint32) >> 16).astype(np.uint16)          # bf16 storage of the upstream gradient
        g = (dout.astype(np.uint32) << 16).view(np.float32)
    else:
        dout, g = g32, g32
    _, rq, rk, rv = oracle.attn_backward(gen.as_f32(w.q, w.dtype), gen.as_f32(w.k_pages, w.dtype),
                                         gen.as_f32(w.v_pages, w.dtype), w.host_block_table(), w.seq_lens, w.parents, g)
    dq, dk, dv = _run(w, dout)
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        assert np.isfinite(got).all(), name
        err = np.abs(got - ref)
        top = np.abs(ref).max()
        if w.dtype == "bf16":
            assert err.max() <= 2e-2 * top, f"{name} abs err {err.max()} vs max {top}"
            assert np.sqrt((err ** 2).mean()) <= 1e-2 * np.sqrt((ref ** 2).mean()), name
        else:
            assert err.max() <= 2e-5 * top, f"{name} abs err {err.max()} vs max {top}"
    return dq, dk, dv


def test_chain_bf16(gpu_lib):
    _check(gen.llama_chain(131, batch=4, len_lo=40, len_hi=500, vocab=64, hidden_size=64), 1)


def test_tree_bf16_many_query_rows(gpu_lib):
    """A 16-node tree with four query heads per KV head: 64 query rows per pair, two passes over the pair's positions."""
    _check(gen.llama_tree(132, batch=3, num_q=16, context=150, vocab=64, hidden_size=64, num_q_heads=8, num_kv_heads=2), 2)


def test_tree_bf16_128_query_rows(gpu_lib):
    """A 32-node tree with four query heads per KV head (the tree workload's shape): four row tiles per pair, a ragged last
    tile, several runs of tiles per pair; then 24 rows (one tile) as a tree."""
    _check(gen.llama_tree(138, batch=5, num_q=32, context=700, vocab=64, hidden_size=64, num_q_heads=8, num_kv_heads=2), 7)
    _check(gen.llama_tree(139, batch=2, num_q=24, context=90, vocab=64, hidden_size=64, num_q_heads=4, num_kv_heads=1), 8)


@pytest.mark.parametrize("num_q,context", [(18, 33), (25, 40), (25, 257), (32, 32), (20, 700)])
def test_tree_bf16_partly_filled_row_tiles_and_short_runs(gpu_lib, num_q, context):
    """65 .. 128 query rows per KV head with a last row tile that is partly or wholly empty, on sequences of one or
    two tiles (runs shorter than the tile pipeline), a one-token last tile, and a prefix of zero length."""
    _check(gen.llama_tree(150 + num_q, batch=3, num_q=num_q, context=context, vocab=64, hidden_size=64, num_q_heads=8,
                          num_kv_heads=2), 20 + num_q)


def test_more_requests_than_the_in_lds_plan_holds(gpu_lib):
    """1030 short requests: past the 1024 requests whose tile prefix the kernels build in LDS, a planning kernel
    writes it to memory (one row tile; then a 70-row tree batch through the shared-tile kernel)."""
    _check(gen.llama_chain(160, batch=1030, num_q=3, num_q_heads=4, num_kv_heads=2, len_lo=3, len_hi=40, vocab=64,
                           hidden_size=64), 30)
    _check(gen.llama_tree(161, batch=1027, num_q=35, context=36, vocab=64, hidden_size=64, num_q_heads=2, num_kv_heads=1),
           31)


def test_fp32_head_dim_64_and_large_pages(gpu_lib):
    _check(gen.tiny_chain(133), 3)
    _check(gen.llama_chain(134, batch=2, len_lo=30, len_hi=200, vocab=64, hidden_size=64, page_size=24, head_dim=64,
                           num_q_heads=4, num_kv_heads=2, dtype=gen.F32), 4)


def test_single_position_and_repeatability(gpu_lib):
    w = gen.llama_chain(135, batch=2, num_q=1, len_lo=70, len_hi=90, vocab=64, hidden_size=64)
    a = _check(w, 5)
    rng = np.random.default_rng(5)
    dout = (rng.standard_normal(w.q.shape).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    b = _run(w, dout)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_unused_pool_positions_are_left_alone_and_host_errors(gpu_lib):
    import paper_2602_06932_amd as av
    from paper_2602_06932_amd.device import DeviceVerify
    w = gen.llama_chain(136, batch=2, len_lo=20, len_hi=50, vocab=64, hidden_size=64)
    dq, dk, dv = _check(w, 6)
    used = np.zeros(dk.shape[:3], bool)
    for b in range(w.batch):
        for j in range(int(w.seq_lens[b])):
            used[w.block_table[b, j // w.page_size], :, j % w.page_size] = True
    assert (~used).any() and not dk[~used].any() and not dv[~used].any()
    w8 = gen.llama_chain(137, batch=2, len_lo=20, len_hi=50, vocab=64, hidden_size=64, kv_fp8=True)
    d8 = DeviceVerify(w8)
    with pytest.raises(av.AuroraError) as e:
        av.aurora_attn_backward_workspace_bytes(d8.attn_desc)
    assert e.value.status == av.AURORA_ERR_UNSUPPORTED


def _forward_lse(w):
    import paper_2602_06932_amd as av
    from paper_2602_06932_amd.device import DeviceVerify
    dv = DeviceVerify(w)
    out = torch.empty_like(dv.q)
    lse = torch.full(w.q.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(av.aurora_verify_workspace_bytes(dv.attn_desc, None), dtype=torch.uint8, device="cuda")
    av.aurora_attn_forward(dv.attn_desc, dv.q, dv.k_pages, dv.v_pages, dv.block_table, dv.seq_lens, dv.parents, out, lse, ws)
    torch.cuda.synchronize()
    return dv, out, lse


def test_forward_with_logsumexp(gpu_lib):
    """aurora_attn_forward: the output is the verify step's, lse against the float64 oracle.  bf16 inputs are exact in
    the products and the sums run in fp32 over at most a few thousand terms of either path: absolute 1e-3 (lse is of
    order log L); fp32 storage 2e-5."""
    from parity_util import check_attention
    cases = [gen.llama_chain(140, batch=3, len_lo=40, len_hi=600, vocab=64, hidden_size=64),
             gen.llama_tree(141, batch=2, num_q=32, context=300, vocab=64, hidden_size=64, num_q_heads=8, num_kv_heads=2),
             gen.tiny_chain(142),
             gen.llama_chain(143, batch=2, len_lo=40, len_hi=300, vocab=64, hidden_size=64, kv_fp8=True)]
    for w in cases:
        print(f"[case] {w.name} {w.dtype} kv={w.kv_dtype}", flush=True)
        dv, out, lse = _forward_lse(w)
        check_attention(out.float().cpu().numpy(), oracle.attn_workload(w), w.dtype)
        if w.kv_dtype == "fp8":
            kf = gen.e4m3_rows_to_f32(w.k_pages.reshape(-1, w.head_dim), np.ones(1, np.float32)).reshape(w.k_pages.shape)
            kf = kf * w.k_scale[None, :, None, None]
        else:
            kf = gen.as_f32(w.k_pages, w.dtype)
        ref = oracle.attn_lse(gen.as_f32(w.q, w.dtype), kf, w.host_block_table(), w.seq_lens, w.parents)
        got = lse.cpu().numpy()
        assert np.isfinite(got).all()
        assert np.abs(got - ref).max() <= (2e-5 if w.dtype == "f32" else 1e-3), np.abs(got - ref).max()


def test_backward_from_saved_forward_is_bit_identical(gpu_lib):
    import paper_2602_06932_amd as av
    from paper_2602_06932_amd.device import _to_dev
    for w, seed in ((gen.llama_chain(144, batch=3, len_lo=40, len_hi=400, vocab=64, hidden_size=64), 9),
                    (gen.llama_tree(145, batch=2, num_q=32, context=200, vocab=64, hidden_size=64, num_q_heads=8,
                                    num_kv_heads=2), 10),
                    (gen.tiny_chain(146), 11)):
        rng = np.random.default_rng(seed)
        g32 = rng.standard_normal(w.q.shape).astype(np.float32)
        dout = (g32.view(np.uint32) >> 16).astype(np.uint16) if w.dtype == "bf16" else g32
        ref = _run(w, dout)
        dv, out, lse = _forward_lse(w)
        dq = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device="cuda")
        dk = torch.zeros(dv.k_pages.shape, dtype=torch.float32, device="cuda")
        dvp = torch.zeros(dv.v_pages.shape, dtype=torch.float32, device="cuda")
        ws = torch.empty(av.aurora_attn_backward_workspace_bytes(dv.attn_desc), dtype=torch.uint8, device="cuda")
        av.aurora_attn_backward_saved(dv.attn_desc, dv.q, dv.k_pages, dv.v_pages, dv.block_table, dv.seq_lens, dv.parents,
                                      out, lse, _to_dev(dout, w.dtype), dq, dk, dvp, ws)
        torch.cuda.synchronize()
        for x, y in zip(ref, (dq.cpu().numpy(), dk.cpu().numpy(), dvp.cpu().numpy())):
            assert np.array_equal(x, y)


def _sampled_check(w, sample, seed):
    """The whole batch runs on the GPU; the oracle differentiates the requests in `sample` one by one (pages are not
    shared between requests, so their dK / dV rows depend on nothing else)."""
    print(f"[case] full size {w.name} B={w.batch} Nq={w.num_q} L={int(w.seq_lens.min())}..{int(w.seq_lens.max())} "
          f"sample={list(sample)}", flush=True)
    rng = np.random.default_rng(seed)
    g32 = rng.standard_normal(w.q.shape).astype(np.float32)
    dout = (g32.view(np.uint32) >> 16).astype(np.uint16)
    g = (dout.astype(np.uint32) << 16).view(np.float32)
    dq, dk, dv = _run(w, dout)
    kf, vf = gen.as_f32(w.k_pages, w.dtype), gen.as_f32(w.v_pages, w.dtype)
    bt = w.host_block_table()
    for b in sample:
        ws = w.take_requests([b])
        _, rq, rk, rv = oracle.attn_backward(gen.as_f32(ws.q, w.dtype), kf, vf, bt[b:b + 1], ws.seq_lens, ws.parents,
                                             g[b:b + 1])
        L = int(w.seq_lens[b])
        pos = np.arange(L)
        pg, off = bt[b][pos // w.page_size], pos % w.page_size
        for name, got, ref in (("dq", dq[b], rq[0]), ("dk", dk[pg, :, off], rk[pg, :, off]),
                               ("dv", dv[pg, :, off], rv[pg, :, off])):
            assert np.isfinite(got).all(), (name, b)
            err = np.abs(got - ref)
            assert err.max() <= 2e-2 * np.abs(ref).max(), f"{name} request {b}: abs err {err.max()} vs max {np.abs(ref).max()}"
            assert np.sqrt((err ** 2).mean()) <= 1e-2 * np.sqrt((ref ** 2).mean()), (name, b)


@pytest.mark.timeout(300)
def test_full_size_chain_and_tree_sampled(gpu_lib):
    """The two shapes bench.py --stage attn_bwd times (config 2's chain batch, config 4's tree batch), whole batch on
    the GPU, sampled requests against the oracle."""
    w = gen.llama_chain(1, vocab=64, hidden_size=64)
    order = np.argsort(w.seq_lens, kind="stable")
    _sampled_check(w, [int(order[0]), int(order[len(order) // 2]), int(order[-1])], 12)
    _sampled_check(gen.llama_tree(1, vocab=64, hidden_size=64), [0, 11], 13)


@pytest.mark.parametrize("tree", [False, True])
def test_backward_replays_from_a_captured_graph(gpu_lib, tree):
    """The backward call (forward recomputed, delta, backward kernel, dq merge) is plain kernel launches on the caller's
    stream - no allocation, no memset: captured once and replayed, with eager work on the same workspace between
    the replays, it gives the eager call's bits every time."""
    import paper_2602_06932_amd as av
    from paper_2602_06932_amd.device import DeviceVerify, _to_dev
    if tree:
        w = gen.llama_tree(170, batch=3, num_q=32, context=300, vocab=64, hidden_size=64, num_q_heads=8, num_kv_heads=2)
    else:
        w = gen.llama_chain(171, batch=4, len_lo=40, len_hi=500, vocab=64, hidden_size=64)
    rng = np.random.default_rng(40)
    dout = (rng.standard_normal(w.q.shape).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    ref = _run(w, dout)
    dv = DeviceVerify(w)
    d_dout = _to_dev(dout, w.dtype)
    dq = torch.zeros(w.q.shape, dtype=torch.float32, device="cuda")
    dk = torch.zeros(dv.k_pages.shape, dtype=torch.float32, device="cuda")
    dvp = torch.zeros(dv.v_pages.shape, dtype=torch.float32, device="cuda")
    ws = torch.empty(av.aurora_attn_backward_workspace_bytes(dv.attn_desc), dtype=torch.uint8, device="cuda")
    call = lambda stream=None: av.aurora_attn_backward(dv.attn_desc, dv.q, dv.k_pages, dv.v_pages, dv.block_table,
                                                       dv.seq_lens, dv.parents, d_dout, dq, dk, dvp, ws, stream=stream)
    call()  # the first call of a kernel also sets its LDS attribute: not part of the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for i in range(3):
        dq.fill_(float("nan"))
        dk.zero_()
        dvp.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for name, x, y in zip(("dq", "dk", "dv"), ref, (dq, dk, dvp)):
            assert np.array_equal(x, y.cpu().numpy()), (i, name)
        ws.fill_(0xff)  # eager work on the workspace between the replays
        torch.cuda.synchronize()
