"""The C-ABI library builds, loads without a GPU and exports every symbol the header declares;
host-side validation works without a device."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "aurora_verify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aurora_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2602_06932_amd as av
    if not os.path.exists(av.LIB_PATH):
        from paper_2602_06932_amd import build
        build.build()
    lib = av.load()
    names = _declared()
    assert {"aurora_verify", "aurora_verify_attn", "aurora_verify_accept", "aurora_verify_workspace_bytes",
            "aurora_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(av.EXPORTS) == set(names)


def test_host_validation_without_device():
    import paper_2602_06932_amd as av
    ad = av.aurora_attn_desc(batch=2, num_q=5, num_q_heads=8, num_kv_heads=2, head_dim=64, page_size=16,
                             max_pages_per_seq=4, num_pages=8, dtype=av.AURORA_F32, sm_scale=0.0)
    cd = av.aurora_accept_desc(batch=2, num_q=5, hidden=64, vocab=100, dtype=av.AURORA_F32, temperature=1.0)
    n = av.aurora_verify_workspace_bytes(ad, cd)
    assert n >= 2 * 5 * 100 * 4 and n % 256 == 0
    assert av.aurora_verify_workspace_bytes(ad, None) + av.aurora_verify_workspace_bytes(None, cd) == n
    bad = av.aurora_attn_desc.from_buffer_copy(ad)
    bad.num_kv_heads = 3
    with pytest.raises(av.AuroraError) as e:
        av.aurora_verify_workspace_bytes(bad, cd)
    assert e.value.status == av.AURORA_ERR_INVALID_ARG
    bad = av.aurora_accept_desc.from_buffer_copy(cd)
    bad.temperature = -1.0
    with pytest.raises(av.AuroraError):
        av.aurora_verify_workspace_bytes(None, bad)
    # an 8-bit KV cache needs both scale arrays; the flag is 0 or 1; the workspace does not depend on it here
    bad = av.aurora_attn_desc.from_buffer_copy(ad)
    bad.kv_fp8 = 1
    with pytest.raises(av.AuroraError) as e:
        av.aurora_verify_workspace_bytes(bad, None)
    assert e.value.status == av.AURORA_ERR_INVALID_ARG
    bad.k_scale, bad.v_scale = 256, 512
    assert av.aurora_verify_workspace_bytes(bad, None) == av.aurora_verify_workspace_bytes(ad, None)
    bad.kv_fp8 = 2
    with pytest.raises(av.AuroraError):
        av.aurora_verify_workspace_bytes(bad, None)
    # trace emission: descriptor and pointer checks come before any device is touched
    td = av.aurora_trace_desc(batch=2, num_q=5, vocab=100, top_k=8)
    assert av.aurora_trace_emit(None, 16, None, None, None, None, 16, 16, None, None, stream=0, check=False) \
        == av.AURORA_ERR_INVALID_ARG
    assert av.aurora_trace_emit(td, None, None, None, None, None, None, None, None, None, stream=0, check=False) \
        == av.AURORA_ERR_INVALID_ARG  # nothing requested
    assert av.aurora_trace_emit(td, 16, None, None, None, None, 16, None, None, None, stream=0, check=False) \
        == av.AURORA_ERR_INVALID_ARG  # ids without values
    assert av.aurora_trace_emit(td, 18, None, None, None, None, 16, 16, None, None, stream=0, check=False) \
        == av.AURORA_ERR_INVALID_ARG  # logits not 4-byte aligned
    assert av.aurora_trace_emit(td, None, None, None, None, None, None, None, 16, 16, stream=0, check=False) \
        == av.AURORA_ERR_INVALID_ARG  # records without the acceptance outputs
    big = av.aurora_trace_desc(batch=2, num_q=5, vocab=100, top_k=4096)
    assert av.aurora_trace_emit(big, 16, None, None, None, None, 16, 16, None, None, stream=0, check=False) \
        == av.AURORA_ERR_UNSUPPORTED
    assert av.status_string(av.AURORA_ERR_UNSUPPORTED) == "unsupported configuration"
    assert av.status_string(12345) == "unknown status"


def test_training_side_entry_points_validate_on_the_host():
    """aurora_attn_forward / aurora_attn_backward / aurora_attn_backward_saved: descriptor, pointer, alignment and
    workspace checks come before any device is touched (addresses below are never dereferenced)."""
    import torch
    import paper_2602_06932_amd as av
    ad = av.aurora_attn_desc(batch=2, num_q=5, num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16,
                             max_pages_per_seq=4, num_pages=8, dtype=av.AURORA_BF16, sm_scale=0.0)
    n = av.aurora_attn_backward_workspace_bytes(ad)
    assert n % 256 == 0 and n > av.aurora_verify_workspace_bytes(ad, None)
    big = av.aurora_attn_desc.from_buffer_copy(ad)
    big.batch = 64
    assert av.aurora_attn_backward_workspace_bytes(big) > n
    f8 = av.aurora_attn_desc.from_buffer_copy(ad)
    f8.kv_fp8, f8.k_scale, f8.v_scale = 1, 256, 512
    with pytest.raises(av.AuroraError) as e:
        av.aurora_attn_backward_workspace_bytes(f8)
    assert e.value.status == av.AURORA_ERR_UNSUPPORTED
    ws = torch.empty(n + 256, dtype=torch.uint8)
    ws = ws[(-ws.data_ptr()) % 256:][:n]                       # a 256-byte aligned host buffer standing in for the workspace
    P = 4096                                                    # any 16-byte aligned address
    args = (P, P, P, P, P, None)                                # q, k, v, block_table, seq_lens, parents
    assert av.aurora_attn_forward(ad, *args, P, None, ws, stream=0, check=False) == av.AURORA_ERR_INVALID_ARG      # no lse
    assert av.aurora_attn_forward(ad, *args, P, P + 2, ws, stream=0, check=False) == av.AURORA_ERR_INVALID_ARG     # lse misaligned
    bw = lambda **k: av.aurora_attn_backward_saved(ad, *args, k.get("out", P), k.get("lse", P), k.get("dout", P), k.get("dq", P),
                                                   P, P, k.get("ws", ws), stream=0, check=False)
    assert bw(out=None) == av.AURORA_ERR_INVALID_ARG
    assert bw(lse=None) == av.AURORA_ERR_INVALID_ARG
    assert bw(dout=P + 8) == av.AURORA_ERR_INVALID_ARG                                                                # misaligned
    assert bw(dq=None) == av.AURORA_ERR_INVALID_ARG
    assert bw(ws=ws[:n - 256]) == av.AURORA_ERR_WORKSPACE
    assert av.aurora_attn_backward(ad, *args, P, None, P, P, ws, stream=0, check=False) == av.AURORA_ERR_INVALID_ARG  # no dq
    assert av.aurora_attn_backward(f8, *args, P, P, P, P, ws, stream=0, check=False) == av.AURORA_ERR_UNSUPPORTED
    empty = av.aurora_attn_desc.from_buffer_copy(ad)
    empty.batch = 0
    assert av.aurora_attn_backward_saved(empty, *args, P, P, P, P, P, P, ws, stream=0, check=False) == av.AURORA_OK


def test_product_package_does_not_touch_the_oracle():
    """The product path must not import, read or call anything under oracle/."""
    pkg = os.path.join(ROOT, "paper_2602_06932_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_probe_rejects_bad_arguments_on_the_host():
    """The calibration probe validates on the host before anything is enqueued (no GPU needed for this)."""
    import ctypes as C
    import paper_2602_06932_amd as av
    lib = av.load()
    buf = (C.c_char * 64)()
    one = (C.c_float * 1)()
    assert lib.aurora_probe_contraction(5, buf, 1 << 24, 8, 8, one, None) == av.AURORA_ERR_INVALID_ARG    # mode
    assert lib.aurora_probe_contraction(0, None, 1 << 24, 8, 8, one, None) == av.AURORA_ERR_INVALID_ARG   # operands
    assert lib.aurora_probe_contraction(0, buf, 1 << 20, 8, 8, one, None) == av.AURORA_ERR_INVALID_ARG    # too small
    assert lib.aurora_probe_contraction(0, buf, 1 << 24, 0, 8, one, None) == av.AURORA_ERR_INVALID_ARG    # no work
    assert lib.aurora_probe_contraction(0, buf, 1 << 24, 8, 8, None, None) == av.AURORA_ERR_INVALID_ARG   # sink
