"""The allocation-free attention entry point (aurora_verify_attn_static): same output, bit for bit, as
aurora_verify_attn with a caller's workspace, on two calls in a row through the C ABI, the second on a smaller
input; sizes beyond the fixed array are refused before anything is enqueued."""
import numpy as np
import pytest

import gen


def test_static_entry_point_refuses_sizes_beyond_its_array():
    """Host-side check only (runs without a GPU): the tree workload of 16 requests needs 84 MB of partials."""
    import ctypes as C
    import paper_2602_06932_amd as av
    lib = av.load()
    d = av.aurora_attn_desc(batch=16, num_q=32, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
                            max_pages_per_seq=256, num_pages=4096, dtype=av.AURORA_BF16, sm_scale=0.0)
    need = av.aurora_verify_workspace_bytes(d, None)
    assert need > av.AURORA_STATIC_SCRATCH_BYTES
    st = lib.aurora_verify_attn_static(C.byref(d), None, None, None, None, None, None, None, None)
    assert st == av.AURORA_ERR_TOO_LARGE
    assert b"AURORA_STATIC_SCRATCH_BYTES" in lib.aurora_status_string(st)


@pytest.mark.gpu
def test_static_entry_point_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    import torch
    import paper_2602_06932_amd as av
    from paper_2602_06932_amd.device import DeviceVerify
    assert torch.cuda.is_available()
    big = gen.llama_chain(1)                                  # the headline shape: 12.6 MiB of partials
    small = gen.llama_chain(2, batch=5, len_lo=40, len_hi=900)  # second call: fewer, shorter requests
    tiny = gen.tiny_chain(3)                                  # fp32 path (generic kernel), third call
    outs = []
    for w in (big, small, tiny):
        dv = DeviceVerify(w)
        need = av.aurora_verify_workspace_bytes(dv.attn_desc, None)
        assert need <= av.AURORA_STATIC_SCRATCH_BYTES, need
        dv.attn()                                             # the existing entry point, caller's workspace
        torch.cuda.synchronize()
        ref = dv.attn_out.clone()
        outs.append((dv, ref))
    for dv, ref in outs:                                      # big, then small, then tiny: calls in a row
        dv.attn_out.fill_(float("nan"))
        av.aurora_verify_attn_static(dv.attn_desc, dv.q, dv.k_pages, dv.v_pages, dv.block_table, dv.seq_lens,
                                     dv.parents, dv.attn_out)
        torch.cuda.synchronize()
        assert torch.equal(dv.attn_out.view(torch.uint8), ref.view(torch.uint8))
    # and once more in the opposite order without synchronising in between (one stream: ordered)
    for dv, _ in reversed(outs):
        dv.attn_out.fill_(float("nan"))
        av.aurora_verify_attn_static(dv.attn_desc, dv.q, dv.k_pages, dv.v_pages, dv.block_table, dv.seq_lens,
                                     dv.parents, dv.attn_out)
    torch.cuda.synchronize()
    for dv, ref in outs:
        assert torch.equal(dv.attn_out.view(torch.uint8), ref.view(torch.uint8))
    # against the oracle too, on the small case (the bar of the parity tests)
    import oracle
    from parity_util import check_attention
    dv, _ = outs[1]
    ref_o, _ = oracle.verify(small)
    check_attention(dv.attn_out_host(), ref_o, small.dtype)
