"""Parity of the trace-record packing (appendix A.1, eq. 4) against the oracle: bit-exact."""
import numpy as np
import pytest
import torch

import gen
import oracle

pytestmark = pytest.mark.gpu


def _run(traj, h=None, ids=None, lg=None, x=None, y=None, want_traj=True):
    import paper_2602_06932_amd as av
    M = traj.shape[0]
    K = 0 if ids is None else ids.shape[1]
    hb = 0 if h is None else h.shape[1] * h.dtype.itemsize
    d = av.aurora_pack_desc(rows=M, top_k=K, h_row_bytes=hb)
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(a.shape[0], -1) if a.ndim > 1
                                                            else np.ascontiguousarray(a)).cuda()
    like = lambda a: None if a is None else torch.full_like(dev(a), 0x5A if a.dtype == np.uint8 else 0)
    t_traj = torch.from_numpy(traj).cuda()
    n_out = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    row_index = torch.full((max(M, 1),), -1, dtype=torch.int32, device="cuda")
    ins = [dev(h), dev(ids), dev(lg), dev(x), dev(y)]
    outs = [like(h), like(ids), like(lg), like(x), like(y)]
    traj_out = torch.full((max(M, 1),), 9, dtype=torch.int8, device="cuda") if want_traj else None
    av.aurora_trace_pack(d, t_traj if M else None, ins[0], ins[1], ins[2], ins[3], ins[4], n_out, row_index if M else None,
                         outs[0], outs[1], outs[2], outs[3], outs[4], traj_out)
    torch.cuda.synchronize()
    n = int(n_out.item())
    back = lambda t, a: None if t is None else t.cpu().numpy()[:n].view(a.dtype).reshape((n,) + a.shape[1:])
    return dict(n=n, row_index=row_index.cpu().numpy()[:n], h=back(outs[0], h) if h is not None else None,
                topk_ids=back(outs[1], ids) if ids is not None else None,
                topk_logits=back(outs[2], lg) if lg is not None else None,
                x_in=back(outs[3], x) if x is not None else None, y_out=back(outs[4], y) if y is not None else None,
                traj=None if traj_out is None else traj_out.cpu().numpy()[:n])


def _check(traj, **kw):
    names = dict(h="h", ids="topk_ids", lg="topk_logits", x="x_in", y="y_out")
    ref = oracle.trace_pack(traj, **{names[k]: v for k, v in kw.items()})
    got = _run(traj, **kw)
    assert got["n"] == ref["n"] and np.array_equal(got["row_index"], ref["row_index"])
    for k, v in kw.items():
        assert np.array_equal(got[names[k]], ref[names[k]]), k
    assert np.array_equal(got["traj"], ref["traj"])


@pytest.mark.parametrize("rows,hdim,k", [(160, 12288, 1024), (512, 4096, 256), (5000, 24, 3), (1, 8, 1), (1025, 100, 7)])
def test_packing_matches_the_oracle(gpu_lib, rows, hdim, k):
    rng = np.random.default_rng(rows)
    traj = rng.integers(0, 3, rows).astype(np.int8)
    h = rng.integers(0, 65536, (rows, hdim)).astype(np.uint16)          # bf16 bit patterns: 3 x hidden of the target
    ids = rng.integers(-1, 32000, (rows, k)).astype(np.int32)
    lg = rng.integers(0, 65536, (rows, k)).astype(np.uint16)
    x = rng.integers(0, 128256, rows).astype(np.int32)
    y = rng.integers(-1, 128256, rows).astype(np.int32)
    _check(traj, h=h, ids=ids, lg=lg, x=x, y=y)


def test_subsets_of_the_arrays_odd_row_sizes_and_degenerate_masks(gpu_lib):
    rng = np.random.default_rng(9)
    traj = rng.integers(0, 3, 300).astype(np.int8)
    h = rng.integers(0, 256, (300, 37)).astype(np.uint8)               # 37-byte rows: the byte-wise copy
    _check(traj, h=h)
    _check(traj, x=rng.integers(0, 9, 300).astype(np.int32))
    _check(np.zeros(300, np.int8), h=h)                                  # nothing kept
    _check(np.full(300, 2, np.int8), h=h)                                # everything kept
    h6 = rng.integers(0, 65536, (300, 3)).astype(np.uint16)             # 6-byte rows
    _check(traj, h=h6, y=rng.integers(-1, 9, 300).astype(np.int32))


def test_records_of_a_verify_step_are_packed(gpu_lib):
    """verify -> trace emission -> packing, with the step's hidden rows as h."""
    from paper_2602_06932_amd.device import DeviceVerify
    w = gen.llama_tree(111, batch=6, num_q=12, vocab=5000, hidden_size=128, context=80, num_q_heads=4, num_kv_heads=2)
    dv = DeviceVerify(w)
    dv.verify()
    dv.trace(top_k=64)
    torch.cuda.synchronize()
    traj = dv.traj.cpu().numpy().reshape(-1)
    ids = dv.topk_ids.cpu().numpy()
    lg = dv.topk_logits.cpu().numpy().view(np.uint16)
    x = w.draft_tokens.reshape(-1).astype(np.int32)
    y = dv.y_out.cpu().numpy().reshape(-1)
    h = w.hidden.reshape(-1, w.hidden_size)
    assert 0 < (traj != 0).sum() < traj.size
    _check(np.ascontiguousarray(traj), h=np.ascontiguousarray(h), ids=np.ascontiguousarray(ids), lg=np.ascontiguousarray(lg),
           x=np.ascontiguousarray(x), y=np.ascontiguousarray(y))


def test_empty_batch_and_host_errors(gpu_lib):
    import paper_2602_06932_amd as av
    n_out = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    av.aurora_trace_pack(av.aurora_pack_desc(rows=0, top_k=0, h_row_bytes=0), None, None, None, None, None, None, n_out,
                         None, None, None, None, None, None, None)
    torch.cuda.synchronize()
    assert n_out.item() == 0
    t = torch.zeros(4, dtype=torch.int8, device="cuda")
    ri = torch.zeros(4, dtype=torch.int32, device="cuda")
    x = torch.zeros(4, dtype=torch.int32, device="cuda")
    d = av.aurora_pack_desc(rows=4, top_k=0, h_row_bytes=0)
    st = av.aurora_trace_pack(d, t, None, None, None, x, None, n_out, ri, None, None, None, None, None, None, check=False)
    assert st == av.AURORA_ERR_INVALID_ARG   # an input without its output
    st = av.aurora_trace_pack(d, None, None, None, None, None, None, n_out, ri, None, None, None, None, None, None, check=False)
    assert st == av.AURORA_ERR_INVALID_ARG   # no trajectory codes
    st = av.aurora_trace_pack(d, t, None, x, None, None, None, n_out, ri, None, x, None, None, None, None, check=False)
    assert st == av.AURORA_ERR_INVALID_ARG   # ids without values
