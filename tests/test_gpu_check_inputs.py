"""The debug check of device-resident inputs: clean workloads pass, and each kind of out-of-range value -
planted in the HOST copy of the inputs before upload; the checker only reads inside the declared shapes -
is reported with the lowest offending request."""
import dataclasses

import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu
INT_MAX = 0x7FFFFFFF


def _flags(w):
    from paper_2602_06932_amd.device import DeviceVerify
    return DeviceVerify(w).check_inputs()


def _chain():
    return gen.llama_chain(71, batch=9, len_lo=20, len_hi=300, vocab=900, hidden_size=128)


def _tree():
    return gen.llama_tree(72, batch=7, num_q=12, vocab=900, hidden_size=128, context=90, num_q_heads=4, num_kv_heads=2)


def test_clean_workloads_raise_no_flag(gpu_lib):
    for w in (_chain(), _tree(), gen.tiny_chain(3), gen.qwen_greedy_chain(2, batch=5, len_lo=30, len_hi=200, vocab=700,
                                                                          hidden_size=128)):
        f = _flags(w)
        assert f[0] == 0 and (f[1:] == INT_MAX).all(), f


@pytest.mark.parametrize("kind", ["short", "long", "page_neg", "page_big", "parent_root", "parent_fwd", "token_neg",
                                  "token_big", "uniform_one", "uniform_nan"])
def test_each_kind_of_bad_input_is_reported(gpu_lib, kind):
    import paper_2602_06932_amd as av
    w = _tree() if kind.startswith("parent") else _chain()
    req = 4
    f = {k: np.array(getattr(w, k), copy=True) if getattr(w, k) is not None else None
         for k in ("seq_lens", "block_table", "parents", "draft_tokens", "uniforms")}
    if kind == "short":
        f["seq_lens"][req] = w.num_q - 1
        want, slot = av.AURORA_CHECK_SEQ_LEN, 1
    elif kind == "long":
        f["seq_lens"][req] = w.block_table.shape[1] * w.page_size + 1
        want, slot = av.AURORA_CHECK_SEQ_LEN, 1
    elif kind == "page_neg":
        f["block_table"][req, 0] = -1
        want, slot = av.AURORA_CHECK_PAGE_ID, 2
    elif kind == "page_big":
        last = (int(w.seq_lens[req]) - 1) // w.page_size
        f["block_table"][req, last] = w.num_pages
        want, slot = av.AURORA_CHECK_PAGE_ID, 2
    elif kind == "parent_root":
        f["parents"][req, 0] = 0
        want, slot = av.AURORA_CHECK_PARENT, 3
    elif kind == "parent_fwd":
        f["parents"][req, 5] = 5
        want, slot = av.AURORA_CHECK_PARENT, 3
    elif kind == "token_neg":
        f["draft_tokens"][req, 2] = -3
        want, slot = av.AURORA_CHECK_TOKEN, 4
    elif kind == "token_big":
        f["draft_tokens"][req, w.num_q - 1] = w.vocab
        want, slot = av.AURORA_CHECK_TOKEN, 4
    elif kind == "uniform_one":
        f["uniforms"][req, 1, 1] = 1.0
        want, slot = av.AURORA_CHECK_UNIFORM, 5
    else:
        f["uniforms"][req, 0, 0] = np.nan
        want, slot = av.AURORA_CHECK_UNIFORM, 5
    # a second, later offender of the same kind must not displace the first
    got = _flags(dataclasses.replace(w, **f))
    assert got[0] == want, (kind, got)
    assert got[slot] == req
    assert all(got[i] == INT_MAX for i in range(1, 6) if i != slot)


def test_unused_table_entries_and_the_root_token_are_not_checked(gpu_lib):
    w = _chain()
    bt = w.block_table.copy()
    for b in range(w.batch):
        used = (int(w.seq_lens[b]) + w.page_size - 1) // w.page_size
        bt[b, used:] = -1
    tok = w.draft_tokens.copy()
    tok[:, 0] = -99
    f = _flags(dataclasses.replace(w, block_table=bt, draft_tokens=tok))
    assert f[0] == 0


def test_partial_calls_and_host_errors(gpu_lib):
    import paper_2602_06932_amd as av
    from paper_2602_06932_amd.device import DeviceVerify
    w = _chain()
    dv = DeviceVerify(w)
    flags = torch.full((6,), -1, dtype=torch.int32, device="cuda")
    av.aurora_verify_check_inputs(dv.attn_desc, None, dv.block_table, dv.seq_lens, None, None, None, flags)
    torch.cuda.synchronize()
    assert flags[0].item() == 0
    bad_tok = dv.draft_tokens.clone()
    bad_tok[1, 1] = w.vocab + 5
    bad_tok[6, 2] = -1
    av.aurora_verify_check_inputs(None, dv.accept_desc, None, None, None, bad_tok, dv.uniforms, flags)
    torch.cuda.synchronize()
    assert flags[0].item() == av.AURORA_CHECK_TOKEN and flags[4].item() == 1
    st = av.aurora_verify_check_inputs(None, dv.accept_desc, dv.block_table, dv.seq_lens, None, None, None, flags,
                                       check=False)
    assert st == av.AURORA_ERR_INVALID_ARG  # KV arrays without the attention descriptor
    st = av.aurora_verify_check_inputs(dv.attn_desc, dv.accept_desc, None, None, None, None, None, None, check=False)
    assert st == av.AURORA_ERR_INVALID_ARG
