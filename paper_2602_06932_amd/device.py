"""Device-memory plumbing around the binding: upload a host workload (any object with the
attribute names of the generator's Workload), allocate outputs and workspace, call the C ABI.
Nothing here computes; torch is used for allocation, copies and streams only."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _to_dev(a, dtype_tag):
    """Host array -> device tensor; uint16 arrays holding bf16 bits become torch.bfloat16."""
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if a.dtype == np.uint16:
        t = t.view(torch.int16).cuda().view(torch.bfloat16)
    else:
        t = t.cuda()
    return t


class DeviceVerify:
    """A workload resident in HBM plus the buffers one verify call needs."""

    def __init__(self, w, pool_pages_on_device=None):
        self.w = w
        bf16 = w.dtype == "bf16"
        self.dt = B.AURORA_BF16 if bf16 else B.AURORA_F32
        self.q = _to_dev(w.q, w.dtype)
        page_ids = getattr(w, "page_ids", None)
        kv_fp8 = getattr(w, "kv_dtype", "") == "fp8"    # uint8 E4M3 codes with one scale per KV head
        self.k_scale = _to_dev(w.k_scale, None) if kv_fp8 else None
        self.v_scale = _to_dev(w.v_scale, None) if kv_fp8 else None
        if page_ids is None:
            self.k_pages = _to_dev(w.k_pages, w.dtype)
            self.v_pages = _to_dev(w.v_pages, w.dtype)
        else:
            # sparse pool: allocate the whole pool, fill only the referenced pages
            shape = (int(w.num_pages),) + tuple(w.k_pages.shape[1:])
            tdt = torch.uint8 if kv_fp8 else torch.bfloat16 if bf16 else torch.float32
            self.k_pages = torch.empty(shape, dtype=tdt, device="cuda")
            self.v_pages = torch.empty(shape, dtype=tdt, device="cuda")
            idx = torch.from_numpy(np.asarray(page_ids, dtype=np.int64)).cuda()
            step = 8192
            for s in range(0, len(page_ids), step):
                self.k_pages[idx[s:s + step]] = _to_dev(w.k_pages[s:s + step], w.dtype)
                self.v_pages[idx[s:s + step]] = _to_dev(w.v_pages[s:s + step], w.dtype)
        self.block_table = _to_dev(w.block_table, None)
        self.seq_lens = _to_dev(w.seq_lens, None)
        self.parents = _to_dev(w.parents, None)
        self.hidden = _to_dev(w.hidden, w.dtype)    # uint8 codes stay uint8 (8-bit floating-point head)
        self.lm_head = _to_dev(w.lm_head, w.dtype)
        head_fp8 = getattr(w, "head_dtype", "") == "fp8"
        self.hidden_scale = _to_dev(w.hidden_scale, None) if head_fp8 else None
        self.lm_head_scale = _to_dev(w.lm_head_scale, None) if head_fp8 else None
        self.draft_tokens = _to_dev(w.draft_tokens, None)
        self.draft_probs = _to_dev(w.draft_probs, None)
        self.uniforms = _to_dev(w.uniforms, None)

        self.attn_desc = B.aurora_attn_desc(
            batch=w.batch, num_q=w.num_q, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads,
            head_dim=w.head_dim, page_size=w.page_size, max_pages_per_seq=int(w.block_table.shape[1]),
            num_pages=int(w.num_pages), dtype=self.dt, sm_scale=0.0, kv_fp8=1 if kv_fp8 else 0,
            k_scale=self.k_scale.data_ptr() if kv_fp8 else None, v_scale=self.v_scale.data_ptr() if kv_fp8 else None)
        # a draft model with its own vocabulary: the target -> draft index map goes with the descriptor
        t2d = w.target_to_draft() if getattr(w, "draft_to_target", None) is not None else None
        self.target_to_draft = _to_dev(t2d, None)
        temps = getattr(w, "temperatures", None)     # one temperature per request, or None
        self.temperatures = _to_dev(None if temps is None else np.asarray(temps, np.float32), None)
        self.accept_desc = B.aurora_accept_desc(
            batch=w.batch, num_q=w.num_q, hidden=w.hidden_size, vocab=w.vocab,
            dtype=B.AURORA_FP8_E4M3 if head_fp8 else self.dt,
            temperature=w.temperature, draft_vocab=int(getattr(w, "draft_vocab", 0) or 0),
            target_to_draft=None if t2d is None else self.target_to_draft.data_ptr(),
            hidden_scale=self.hidden_scale.data_ptr() if head_fp8 else None,
            lm_head_scale=self.lm_head_scale.data_ptr() if head_fp8 else None,
            temperatures=None if temps is None else self.temperatures.data_ptr(),
            tree_without_replacement=1 if getattr(w, "tree_without_replacement", False) else 0)
        self.ws_bytes = B.aurora_verify_workspace_bytes(self.attn_desc, self.accept_desc)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        assert self.workspace.data_ptr() % 256 == 0

        Bn, Nq = w.batch, w.num_q
        self.attn_out = torch.empty_like(self.q)
        self.accept_len = torch.full((Bn,), -7, dtype=torch.int32, device="cuda")
        self.next_token = torch.full((Bn,), -7, dtype=torch.int32, device="cuda")
        self.accept_mask = torch.full((Bn, Nq), 9, dtype=torch.uint8, device="cuda")
        self.p_at_draft = torch.full((Bn, Nq), float("nan"), dtype=torch.float32, device="cuda")
        self.row_lse = torch.full((Bn, Nq), float("nan"), dtype=torch.float32, device="cuda")

        # argument lists marshalled once: the buffers of a DeviceVerify never move
        import ctypes as C
        lib = B.load()
        P = B._ptr
        ws, wsb = P(self.workspace), self.ws_bytes
        attn_args = (P(self.q), P(self.k_pages), P(self.v_pages), P(self.block_table), P(self.seq_lens),
                     P(self.parents))
        acc_in = (P(self.hidden), P(self.lm_head), P(self.draft_tokens), P(self.draft_probs), P(self.uniforms))
        acc_out = (P(self.accept_len), P(self.next_token), P(self.accept_mask), P(self.p_at_draft), P(self.row_lse))
        ad, cd = C.byref(self.attn_desc), C.byref(self.accept_desc)
        self._fast = {
            "attn": (lib.aurora_verify_attn, (ad,) + attn_args + (P(self.attn_out), ws, wsb)),
            "accept": (lib.aurora_verify_accept, (cd,) + acc_in + (P(self.parents),) + acc_out + (ws, wsb)),
            "lmhead": (lib.aurora_verify_lmhead, (cd, P(self.hidden), P(self.lm_head), ws, wsb)),
            "accept_logits": (lib.aurora_verify_accept_logits,
                              (cd,) + acc_in[2:] + (P(self.parents),) + acc_out + (ws, wsb)),
            "verify": (lib.aurora_verify, (ad, cd) + attn_args + (P(self.attn_out),) + acc_in + acc_out + (ws, wsb)),
        }

    def _call(self, name, stream):
        fn, args = self._fast[name]
        st = fn(*args, B._stream(stream))
        if st != B.AURORA_OK:
            raise B.AuroraError(st, fn.__name__)
        return st

    # -- calls through the C ABI (the *_via_binding forms marshal through binding.py on every call) ----------
    def attn(self, stream=None):
        return self._call("attn", stream)

    def accept(self, stream=None):
        return self._call("accept", stream)

    def lmhead(self, stream=None):
        return self._call("lmhead", stream)

    def accept_logits(self, stream=None):
        """Second stage of accept() on the logits a preceding lmhead() left in the workspace."""
        return self._call("accept_logits", stream)

    def verify(self, stream=None):
        return self._call("verify", stream)

    def check_inputs(self, stream=None):
        """Debug check of the device-resident inputs; returns the six flags as a host array after a sync."""
        flags = torch.full((6,), -1, dtype=torch.int32, device="cuda")
        B.aurora_verify_check_inputs(self.attn_desc, self.accept_desc, self.block_table, self.seq_lens, self.parents,
                                     self.draft_tokens, self.uniforms, flags, stream)
        torch.cuda.synchronize()
        return flags.cpu().numpy()

    def trace(self, top_k=1024, after="verify", stream=None, group_max=True):
        """Trace emission from the logits and acceptance outputs the last verify / accept call left (with the group
        maxima of the same call's LM head, unless group_max is False or the call wrote none)."""
        w = self.w
        if getattr(self, "_trace_k", None) != (top_k, after, group_max):
            rows = w.batch * w.num_q
            gptr, ng = B.aurora_verify_group_max_ptr(self.attn_desc if after == "verify" else None, self.accept_desc,
                                                     self.workspace) if group_max else (0, 0)
            self.trace_desc = B.aurora_trace_desc(batch=w.batch, num_q=w.num_q, vocab=w.vocab, top_k=top_k,
                                                  n_groups=ng, group_max=gptr or None)
            self.topk_ids = torch.empty((rows, top_k), dtype=torch.int32, device="cuda")
            self.topk_logits = torch.empty((rows, top_k), dtype=torch.int16, device="cuda")
            self.y_out = torch.empty((w.batch, w.num_q), dtype=torch.int32, device="cuda")
            self.traj = torch.empty((w.batch, w.num_q), dtype=torch.int8, device="cuda")
            self._trace_logits = B.aurora_verify_logits_ptr(self.attn_desc if after == "verify" else None,
                                                            self.accept_desc, self.workspace)
            self._trace_k = (top_k, after, group_max)
            import ctypes as C
            P = B._ptr
            # marshalled once, like the verify calls: the buffers never move
            self._trace_args = (C.byref(self.trace_desc), self._trace_logits, P(self.draft_tokens), P(self.parents),
                                P(self.next_token), P(self.accept_mask), P(self.topk_ids), P(self.topk_logits),
                                P(self.y_out), P(self.traj))
        st = B.load().aurora_trace_emit(*self._trace_args, B._stream(stream))
        if st != B.AURORA_OK:
            raise B.AuroraError(st, "aurora_trace_emit")
        return st

    def attn_via_binding(self, stream=None):
        return B.aurora_verify_attn(self.attn_desc, self.q, self.k_pages, self.v_pages, self.block_table,
                                    self.seq_lens, self.parents, self.attn_out, self.workspace, stream)

    def accept_via_binding(self, stream=None):
        return B.aurora_verify_accept(self.accept_desc, self.hidden, self.lm_head, self.draft_tokens,
                                      self.draft_probs, self.uniforms, self.parents, self.accept_len,
                                      self.next_token, self.accept_mask, self.p_at_draft, self.row_lse,
                                      self.workspace, stream)

    def lmhead_via_binding(self, stream=None):
        return B.aurora_verify_lmhead(self.accept_desc, self.hidden, self.lm_head, self.workspace, stream)

    def verify_via_binding(self, stream=None):
        return B.aurora_verify(self.attn_desc, self.accept_desc, self.q, self.k_pages, self.v_pages,
                               self.block_table, self.seq_lens, self.parents, self.attn_out, self.hidden,
                               self.lm_head, self.draft_tokens, self.draft_probs, self.uniforms, self.accept_len,
                               self.next_token, self.accept_mask, self.p_at_draft, self.row_lse, self.workspace,
                               stream)

    # -- results back on the host --------------------------------------------------------------
    def attn_out_host(self) -> np.ndarray:
        return self.attn_out.float().cpu().numpy()

    def logits_host(self, after="verify") -> np.ndarray:
        """fp32 logits [B, Nq, V] left in the workspace by the last accept / verify call."""
        ad = self.attn_desc if after == "verify" else None
        ptr = B.aurora_verify_logits_ptr(ad, self.accept_desc, self.workspace)
        off = ptr - self.workspace.data_ptr()
        n = self.w.batch * self.w.num_q * self.w.vocab
        flat = self.workspace[off:off + 4 * n].view(torch.float32)
        return flat.cpu().numpy().reshape(self.w.batch, self.w.num_q, self.w.vocab)

    def results_host(self):
        torch.cuda.synchronize()
        return dict(accept_len=self.accept_len.cpu().numpy(), next_token=self.next_token.cpu().numpy(),
                    accept_mask=self.accept_mask.cpu().numpy(), p_at_draft=self.p_at_draft.cpu().numpy(),
                    row_lse=self.row_lse.cpu().numpy())
