"""MI355X-native verification step of speculative decoding (chunk attention over a paged GQA KV
cache; LM head + softmax + rejection-sampling acceptance; trace emission for the training side)
behind a C ABI.

`binding` mirrors the C entry points; `device.DeviceVerify` is memory plumbing for tests and the
benchmark.  The package never falls back to a CPU implementation.
"""
from .binding import (AURORA_BF16, AURORA_FP8_E4M3, AURORA_ERR_HIP, AURORA_ERR_INVALID_ARG, AURORA_ERR_UNSUPPORTED,  # noqa: F401
                      AURORA_ERR_WORKSPACE, AURORA_F32, AURORA_OK, EXPORTS, LIB_PATH, AuroraError,
                      aurora_accept_desc, aurora_attn_desc, aurora_trace_desc, aurora_trace_emit, aurora_verify,
                      aurora_verify_accept, aurora_verify_accept_logits,
                      aurora_verify_attn, aurora_verify_lmhead, aurora_verify_logits_ptr, aurora_verify_workspace_bytes, load,
                      status_string, aurora_verify_check_inputs, aurora_draft_loss, aurora_loss_desc, aurora_trace_pack, aurora_pack_desc, aurora_attn_backward, aurora_attn_backward_workspace_bytes, aurora_attn_forward, aurora_attn_backward_saved, aurora_debug_set_tree_spin_limit, aurora_verify_attn_static, aurora_verify_group_max_ptr, aurora_probe_contraction, AURORA_ERR_TOO_LARGE, AURORA_STATIC_SCRATCH_BYTES, AURORA_CHECK_SEQ_LEN, AURORA_CHECK_PAGE_ID,
                      AURORA_CHECK_PARENT, AURORA_CHECK_TOKEN, AURORA_CHECK_UNIFORM)
