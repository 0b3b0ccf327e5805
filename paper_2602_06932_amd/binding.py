"""ctypes binding of libaurora_verify.so: the same names as the C ABI, argument marshalling only.

PyTorch supplies device memory and streams; every step of the verify path runs in the HIP
kernels behind the C entry points.  There is no fallback: if the library is not built, or no
GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

AURORA_OK = 0
AURORA_ERR_INVALID_ARG = -1
AURORA_ERR_UNSUPPORTED = -2
AURORA_ERR_WORKSPACE = -3
AURORA_ERR_HIP = -4
AURORA_ERR_TOO_LARGE = -5
AURORA_STATIC_SCRATCH_BYTES = 16 << 20
AURORA_F32 = 0
AURORA_BF16 = 1
AURORA_FP8_E4M3 = 2

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libaurora_verify.so")

EXPORTS = ("aurora_verify_workspace_bytes", "aurora_verify_attn", "aurora_verify_accept", "aurora_verify",
           "aurora_verify_lmhead", "aurora_verify_accept_logits", "aurora_trace_emit",
           "aurora_verify_logits_ptr", "aurora_status_string", "aurora_verify_check_inputs", "aurora_draft_loss", "aurora_trace_pack", "aurora_attn_backward",
           "aurora_attn_backward_workspace_bytes", "aurora_attn_forward", "aurora_attn_backward_saved", "aurora_debug_set_tree_spin_limit", "aurora_verify_attn_static",
           "aurora_verify_group_max_ptr", "aurora_probe_contraction")


class aurora_attn_desc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("num_q", C.c_int32), ("num_q_heads", C.c_int32),
                ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("page_size", C.c_int32),
                ("max_pages_per_seq", C.c_int32), ("num_pages", C.c_int64), ("dtype", C.c_int32),
                ("sm_scale", C.c_float), ("kv_fp8", C.c_int32), ("k_scale", C.c_void_p), ("v_scale", C.c_void_p)]


class aurora_accept_desc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("num_q", C.c_int32), ("hidden", C.c_int32), ("vocab", C.c_int32),
                ("dtype", C.c_int32), ("temperature", C.c_float), ("draft_vocab", C.c_int32),
                ("target_to_draft", C.c_void_p), ("hidden_scale", C.c_void_p), ("lm_head_scale", C.c_void_p),
                ("temperatures", C.c_void_p), ("tree_without_replacement", C.c_int32)]


class aurora_trace_desc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("num_q", C.c_int32), ("vocab", C.c_int32), ("top_k", C.c_int32),
                ("draft_vocab", C.c_int32), ("draft_to_target", C.c_void_p), ("n_groups", C.c_int32),
                ("group_max", C.c_void_p)]


class aurora_pack_desc(C.Structure):
    _fields_ = [("rows", C.c_int32), ("top_k", C.c_int32), ("h_row_bytes", C.c_int64)]


class aurora_loss_desc(C.Structure):
    _fields_ = [("rows", C.c_int32), ("draft_vocab", C.c_int32), ("top_k", C.c_int32), ("discard_top_k", C.c_int32),
                ("lambda_discard", C.c_float)]


class AuroraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load():
    """Load the built library (raises if it is missing) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2602_06932_amd.build` "
                          "(or __graft_entry__.build()) first")
    # One HIP runtime per process: PyTorch ships its own copy of the runtime library, and device pointers and
    # streams made by one copy mean nothing to another.  Importing torch first makes the loader resolve this
    # library's dependency to the copy torch has already mapped, whatever order the caller imports things in.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    vp, i32p, f32p, u8p = C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p
    ad, cd = C.POINTER(aurora_attn_desc), C.POINTER(aurora_accept_desc)
    lib.aurora_verify_workspace_bytes.argtypes = [ad, cd, C.POINTER(C.c_size_t)]
    lib.aurora_verify_workspace_bytes.restype = C.c_int
    lib.aurora_verify_attn.argtypes = [ad, vp, vp, vp, i32p, i32p, i32p, vp, vp, C.c_size_t, vp]
    lib.aurora_verify_attn.restype = C.c_int
    lib.aurora_probe_contraction.argtypes = [C.c_int, vp, C.c_size_t, C.c_int, C.c_int, vp, vp]
    lib.aurora_probe_contraction.restype = C.c_int
    lib.aurora_verify_group_max_ptr.argtypes = [ad, cd, vp, C.POINTER(C.c_int32)]
    lib.aurora_verify_group_max_ptr.restype = C.c_void_p
    lib.aurora_verify_attn_static.argtypes = [ad, vp, vp, vp, i32p, i32p, i32p, vp, vp]
    lib.aurora_verify_attn_static.restype = C.c_int
    lib.aurora_verify_accept.argtypes = [cd, vp, vp, i32p, f32p, f32p, i32p, i32p, i32p, u8p, f32p, f32p, vp,
                                         C.c_size_t, vp]
    lib.aurora_verify_accept.restype = C.c_int
    lib.aurora_verify_lmhead.argtypes = [cd, vp, vp, vp, C.c_size_t, vp]
    lib.aurora_verify_lmhead.restype = C.c_int
    lib.aurora_verify.argtypes = [ad, cd, vp, vp, vp, i32p, i32p, i32p, vp, vp, vp, i32p, f32p, f32p, i32p, i32p,
                                  u8p, f32p, f32p, vp, C.c_size_t, vp]
    lib.aurora_verify.restype = C.c_int
    lib.aurora_verify_accept_logits.argtypes = [cd, i32p, f32p, f32p, i32p, i32p, i32p, u8p, f32p, f32p, vp, C.c_size_t, vp]
    lib.aurora_verify_accept_logits.restype = C.c_int
    lib.aurora_trace_emit.argtypes = [C.POINTER(aurora_trace_desc), vp, i32p, i32p, i32p, u8p, i32p, vp, i32p, vp, vp]
    lib.aurora_trace_emit.restype = C.c_int
    lib.aurora_verify_check_inputs.argtypes = [ad, cd, i32p, i32p, i32p, i32p, f32p, i32p, vp]
    lib.aurora_verify_check_inputs.restype = C.c_int
    lib.aurora_attn_backward_workspace_bytes.argtypes = [ad, C.POINTER(C.c_size_t)]
    lib.aurora_attn_backward_workspace_bytes.restype = C.c_int
    lib.aurora_attn_backward.argtypes = [ad, vp, vp, vp, i32p, i32p, i32p, vp, f32p, f32p, f32p, vp, C.c_size_t, vp]
    lib.aurora_attn_backward.restype = C.c_int
    lib.aurora_debug_set_tree_spin_limit.argtypes = [C.c_int]
    lib.aurora_debug_set_tree_spin_limit.restype = None
    lib.aurora_attn_forward.argtypes = [ad, vp, vp, vp, i32p, i32p, i32p, vp, f32p, vp, C.c_size_t, vp]
    lib.aurora_attn_forward.restype = C.c_int
    lib.aurora_attn_backward_saved.argtypes = [ad, vp, vp, vp, i32p, i32p, i32p, vp, f32p, vp, f32p, f32p, f32p, vp,
                                               C.c_size_t, vp]
    lib.aurora_attn_backward_saved.restype = C.c_int
    lib.aurora_trace_pack.argtypes = [C.POINTER(aurora_pack_desc)] + [vp] * 15
    lib.aurora_trace_pack.restype = C.c_int
    lib.aurora_draft_loss.argtypes = [C.POINTER(aurora_loss_desc), f32p, i32p, vp, vp, f32p, f32p, f32p, vp]
    lib.aurora_draft_loss.restype = C.c_int
    lib.aurora_verify_logits_ptr.argtypes = [ad, cd, vp]
    lib.aurora_verify_logits_ptr.restype = C.c_void_p
    lib.aurora_status_string.argtypes = [C.c_int]
    lib.aurora_status_string.restype = C.c_char_p
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().aurora_status_string(int(status)).decode()


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (or a raw integer address, or None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ref(d):
    return None if d is None else C.byref(d)


def aurora_verify_workspace_bytes(attn: Optional[aurora_attn_desc], accept: Optional[aurora_accept_desc]) -> int:
    out = C.c_size_t(0)
    st = load().aurora_verify_workspace_bytes(_ref(attn), _ref(accept), C.byref(out))
    if st != AURORA_OK:
        raise AuroraError(st, "aurora_verify_workspace_bytes")
    return int(out.value)


def aurora_verify_attn(desc, q, k_pages, v_pages, block_table, seq_lens, parents, out, workspace, stream=None,
                       workspace_bytes=None, check=True) -> int:
    wb = workspace_bytes if workspace_bytes is not None else (workspace.numel() * workspace.element_size())
    st = load().aurora_verify_attn(_ref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                   _ptr(seq_lens), _ptr(parents), _ptr(out), _ptr(workspace), wb, _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_verify_attn")
    return st


def aurora_verify_attn_static(desc, q, k_pages, v_pages, block_table, seq_lens, parents, out, stream=None,
                              check=True) -> int:
    st = load().aurora_verify_attn_static(_ref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                          _ptr(seq_lens), _ptr(parents), _ptr(out), _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_verify_attn_static")
    return st


def aurora_verify_accept(desc, hidden, lm_head, draft_tokens, draft_probs, uniforms, parents, accept_len,
                         next_token, accept_mask, p_at_draft, row_lse, workspace, stream=None,
                         workspace_bytes=None, check=True) -> int:
    wb = workspace_bytes if workspace_bytes is not None else (workspace.numel() * workspace.element_size())
    st = load().aurora_verify_accept(_ref(desc), _ptr(hidden), _ptr(lm_head), _ptr(draft_tokens),
                                     _ptr(draft_probs), _ptr(uniforms), _ptr(parents), _ptr(accept_len),
                                     _ptr(next_token), _ptr(accept_mask), _ptr(p_at_draft), _ptr(row_lse),
                                     _ptr(workspace), wb, _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_verify_accept")
    return st


def aurora_verify_lmhead(desc, hidden, lm_head, workspace, stream=None, workspace_bytes=None, check=True) -> int:
    wb = workspace_bytes if workspace_bytes is not None else (workspace.numel() * workspace.element_size())
    st = load().aurora_verify_lmhead(_ref(desc), _ptr(hidden), _ptr(lm_head), _ptr(workspace), wb, _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_verify_lmhead")
    return st


def aurora_verify_accept_logits(desc, draft_tokens, draft_probs, uniforms, parents, accept_len, next_token, accept_mask,
                                p_at_draft, row_lse, workspace, stream=None, workspace_bytes=None, check=True) -> int:
    wb = workspace_bytes if workspace_bytes is not None else (workspace.numel() * workspace.element_size())
    st = load().aurora_verify_accept_logits(_ref(desc), _ptr(draft_tokens), _ptr(draft_probs), _ptr(uniforms),
                                            _ptr(parents), _ptr(accept_len), _ptr(next_token), _ptr(accept_mask),
                                            _ptr(p_at_draft), _ptr(row_lse), _ptr(workspace), wb, _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_verify_accept_logits")
    return st


def aurora_trace_emit(desc, logits, draft_tokens, parents, next_token, accept_mask, topk_ids, topk_logits, y_out, traj,
                      stream=None, check=True) -> int:
    """`logits` may be a tensor or a raw device address (int), e.g. from aurora_verify_logits_ptr()."""
    lp = logits if isinstance(logits, int) or logits is None else _ptr(logits)
    st = load().aurora_trace_emit(_ref(desc), lp, _ptr(draft_tokens), _ptr(parents), _ptr(next_token),
                                  _ptr(accept_mask), _ptr(topk_ids), _ptr(topk_logits), _ptr(y_out), _ptr(traj),
                                  _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_trace_emit")
    return st


def aurora_verify(attn_desc, accept_desc, q, k_pages, v_pages, block_table, seq_lens, parents, attn_out, hidden,
                  lm_head, draft_tokens, draft_probs, uniforms, accept_len, next_token, accept_mask, p_at_draft,
                  row_lse, workspace, stream=None, workspace_bytes=None, check=True) -> int:
    wb = workspace_bytes if workspace_bytes is not None else (workspace.numel() * workspace.element_size())
    st = load().aurora_verify(_ref(attn_desc), _ref(accept_desc), _ptr(q), _ptr(k_pages), _ptr(v_pages),
                              _ptr(block_table), _ptr(seq_lens), _ptr(parents), _ptr(attn_out), _ptr(hidden),
                              _ptr(lm_head), _ptr(draft_tokens), _ptr(draft_probs), _ptr(uniforms),
                              _ptr(accept_len), _ptr(next_token), _ptr(accept_mask), _ptr(p_at_draft),
                              _ptr(row_lse), _ptr(workspace), wb, _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_verify")
    return st


AURORA_CHECK_SEQ_LEN, AURORA_CHECK_PAGE_ID, AURORA_CHECK_PARENT, AURORA_CHECK_TOKEN, AURORA_CHECK_UNIFORM = 1, 2, 4, 8, 16


def aurora_verify_check_inputs(attn_desc, accept_desc, block_table, seq_lens, parents, draft_tokens, uniforms, flags,
                               stream=None, check=True) -> int:
    """Debug check of device-resident inputs; `flags` is an int32 device tensor of 6 entries."""
    st = load().aurora_verify_check_inputs(_ref(attn_desc), _ref(accept_desc), _ptr(block_table), _ptr(seq_lens),
                                           _ptr(parents), _ptr(draft_tokens), _ptr(uniforms), _ptr(flags),
                                           _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_verify_check_inputs")
    return st


def aurora_attn_backward_workspace_bytes(desc) -> int:
    out = C.c_size_t(0)
    st = load().aurora_attn_backward_workspace_bytes(_ref(desc), C.byref(out))
    if st != AURORA_OK:
        raise AuroraError(st, "aurora_attn_backward_workspace_bytes")
    return int(out.value)


def aurora_attn_backward(desc, q, k_pages, v_pages, block_table, seq_lens, parents, dout, dq, dk_pages, dv_pages,
                         workspace, stream=None, check=True) -> int:
    wb = workspace.numel() * workspace.element_size()
    st = load().aurora_attn_backward(_ref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                     _ptr(seq_lens), _ptr(parents), _ptr(dout), _ptr(dq), _ptr(dk_pages),
                                     _ptr(dv_pages), _ptr(workspace), wb, _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_attn_backward")
    return st


def aurora_trace_pack(desc, traj, h, topk_ids, topk_logits, x_in, y_out, n_out, row_index, h_out, topk_ids_out,
                      topk_logits_out, x_in_out, y_out_out, traj_out, stream=None, check=True) -> int:
    st = load().aurora_trace_pack(_ref(desc), _ptr(traj), _ptr(h), _ptr(topk_ids), _ptr(topk_logits), _ptr(x_in),
                                  _ptr(y_out), _ptr(n_out), _ptr(row_index), _ptr(h_out), _ptr(topk_ids_out),
                                  _ptr(topk_logits_out), _ptr(x_in_out), _ptr(y_out_out), _ptr(traj_out),
                                  _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_trace_pack")
    return st


def aurora_draft_loss(desc, draft_logits, topk_ids, topk_logits, traj, row_kl, loss_out, grad, stream=None,
                      check=True) -> int:
    st = load().aurora_draft_loss(_ref(desc), _ptr(draft_logits), _ptr(topk_ids), _ptr(topk_logits), _ptr(traj),
                                  _ptr(row_kl), _ptr(loss_out), _ptr(grad), _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_draft_loss")
    return st


def aurora_verify_logits_ptr(attn_desc, accept_desc, workspace) -> int:
    p = load().aurora_verify_logits_ptr(_ref(attn_desc), _ref(accept_desc), _ptr(workspace))
    return int(p or 0)


def aurora_probe_contraction(mode, operands, workgroups, stages, sink, stream=None, check=True) -> int:
    st = load().aurora_probe_contraction(int(mode), _ptr(operands), operands.numel() * operands.element_size(),
                                         int(workgroups), int(stages), _ptr(sink), _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_probe_contraction")
    return st


def aurora_verify_group_max_ptr(attn_desc, accept_desc, workspace):
    """(device address, n_groups) of the group maxima the LM head left in the workspace; (0, 0) when it wrote none."""
    n = C.c_int32(0)
    p = load().aurora_verify_group_max_ptr(_ref(attn_desc), _ref(accept_desc), _ptr(workspace), C.byref(n))
    return int(p or 0), int(n.value)


def aurora_attn_forward(desc, q, k_pages, v_pages, block_table, seq_lens, parents, out, lse, workspace, stream=None,
                        check=True) -> int:
    wb = workspace.numel() * workspace.element_size()
    st = load().aurora_attn_forward(_ref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _ptr(seq_lens),
                                    _ptr(parents), _ptr(out), _ptr(lse), _ptr(workspace), wb, _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_attn_forward")
    return st


def aurora_attn_backward_saved(desc, q, k_pages, v_pages, block_table, seq_lens, parents, out, lse, dout, dq, dk_pages,
                               dv_pages, workspace, stream=None, check=True) -> int:
    wb = workspace.numel() * workspace.element_size()
    st = load().aurora_attn_backward_saved(_ref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                           _ptr(seq_lens), _ptr(parents), _ptr(out), _ptr(lse), _ptr(dout), _ptr(dq),
                                           _ptr(dk_pages), _ptr(dv_pages), _ptr(workspace), wb, _stream(stream))
    if check and st != AURORA_OK:
        raise AuroraError(st, "aurora_attn_backward_saved")
    return st


def aurora_debug_set_tree_spin_limit(polls: int) -> None:
    load().aurora_debug_set_tree_spin_limit(int(polls))
