"""ctypes front end of the C oracle (oracle/aurora_oracle.c).

TEST INFRASTRUCTURE ONLY: importable from tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py; never from the product package.  Marshals NumPy
host arrays to the C entry points and back; no arithmetic happens here.
"""
from __future__ import annotations

import ctypes as C
import dataclasses
from typing import Optional

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
_DT = {"f32": F32, "bf16": BF16, F32: F32, BF16: BF16}
_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build(force=False))
        for name in ("oracle_attn", "oracle_logits", "oracle_accept_logits", "oracle_accept", "oracle_accept_logits_ex",
                     "oracle_num_threads", "oracle_trace_topk", "oracle_trace_records", "oracle_logits_fp8",
                     "oracle_decode_e4m3", "oracle_attn_fp8kv"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a: Optional[np.ndarray], dtype, shape=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def _elem_dtype(dt):
    return np.float32 if _DT[dt] == F32 else np.uint16


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def attn(*, q, k_pages, v_pages, block_table, seq_lens, parents=None, dtype, sm_scale=0.0,
         k_scale=None, v_scale=None) -> np.ndarray:
    """Chunk attention; returns float64 [B, Nq, Hq, D].  With k_scale / v_scale (float32 [Hkv]) the pools
    hold uint8 E4M3 codes and a value is scale[head] * decode(code); q stays in `dtype`."""
    ed = _elem_dtype(dtype)
    fp8kv = k_scale is not None
    kvd = np.uint8 if fp8kv else ed
    q = _chk(q, ed)
    B, Nq, Hq, D = q.shape
    k_pages = _chk(k_pages, kvd)
    P, Hkv, page, D2 = k_pages.shape
    assert D2 == D
    v_pages = _chk(v_pages, kvd, k_pages.shape)
    block_table = _chk(block_table, np.int32)
    assert block_table.shape[0] == B
    seq_lens = _chk(seq_lens, np.int32, (B,))
    parents = _chk(parents, np.int32, (B, Nq))
    out = np.empty((B, Nq, Hq, D), dtype=np.float64)
    head = (C.c_int(B), C.c_int(Nq), C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int(page),
            C.c_int(block_table.shape[1]), C.c_int64(P), C.c_int(_DT[dtype]), C.c_double(sm_scale))
    if fp8kv:
        k_scale = _chk(k_scale, np.float32, (Hkv,))
        v_scale = _chk(v_scale, np.float32, (Hkv,))
        st = lib().oracle_attn_fp8kv(*head, _p(q), _p(k_pages), _p(v_pages), _p(k_scale), _p(v_scale),
                                     _p(block_table), _p(seq_lens), _p(parents), _p(out))
    else:
        st = lib().oracle_attn(*head, _p(q), _p(k_pages), _p(v_pages), _p(block_table), _p(seq_lens),
                               _p(parents), _p(out))
    if st != 0:
        raise ValueError(f"oracle_attn status {st}")
    return out


def logits(*, hidden, lm_head, dtype) -> np.ndarray:
    """LM-head projection; hidden [..., H], lm_head [V, H] -> float64 [..., V]."""
    ed = _elem_dtype(dtype)
    hidden = _chk(hidden, ed)
    lm_head = _chk(lm_head, ed)
    H = hidden.shape[-1]
    V = lm_head.shape[0]
    assert lm_head.shape[1] == H
    rows = int(np.prod(hidden.shape[:-1]))
    out = np.empty((rows, V), dtype=np.float64)
    st = lib().oracle_logits(C.c_int64(rows), C.c_int(H), C.c_int(V), C.c_int(_DT[dtype]),
                             _p(hidden), _p(lm_head), _p(out))
    if st != 0:
        raise ValueError(f"oracle_logits status {st}")
    return out.reshape(hidden.shape[:-1] + (V,))


def decode_e4m3(codes: np.ndarray) -> np.ndarray:
    """OCP E4M3 codes (uint8) -> float64."""
    codes = _chk(codes, np.uint8)
    out = np.empty(codes.shape, np.float64)
    lib().oracle_decode_e4m3(C.c_int64(codes.size), _p(codes), _p(out))
    return out


def logits_fp8(*, hidden, hidden_scale, lm_head, lm_head_scale) -> np.ndarray:
    """LM head on E4M3 operands: hidden [..., H] uint8 codes with one float32 scale per row, lm_head [V, H]
    codes with one scale per vocabulary row -> float64 [..., V]."""
    hidden = _chk(hidden, np.uint8)
    lm_head = _chk(lm_head, np.uint8)
    H = hidden.shape[-1]
    V = lm_head.shape[0]
    rows = int(np.prod(hidden.shape[:-1]))
    hs = _chk(np.asarray(hidden_scale, np.float32).reshape(rows), np.float32, (rows,))
    ws = _chk(lm_head_scale, np.float32, (V,))
    out = np.empty((rows, V), dtype=np.float64)
    st = lib().oracle_logits_fp8(C.c_int64(rows), C.c_int(H), C.c_int(V), _p(hidden), _p(hs), _p(lm_head), _p(ws),
                                 _p(out))
    if st != 0:
        raise ValueError(f"oracle_logits_fp8 status {st}")
    return out.reshape(hidden.shape[:-1] + (V,))


@dataclasses.dataclass
class AcceptResult:
    accept_len: np.ndarray      # [B] int32
    next_token: np.ndarray      # [B] int32
    accept_mask: np.ndarray     # [B, Nq] uint8
    p_at_draft: np.ndarray      # [B, Nq] float64
    row_lse: np.ndarray         # [B, Nq] float64
    test_margin: np.ndarray     # [B, Nq] float64 (NaN where no test was evaluated)
    top_gap: np.ndarray         # [B, Nq] float64
    stop_node: np.ndarray       # [B] int32
    final_cdf: Optional[np.ndarray]  # [B, V] float64 or None
    logits: Optional[np.ndarray]     # [B, Nq, V] float64 or None


def _alloc_results(B, Nq, V, want_cdf):
    return dict(
        accept_len=np.empty(B, np.int32), next_token=np.empty(B, np.int32),
        accept_mask=np.empty((B, Nq), np.uint8), p_at_draft=np.empty((B, Nq), np.float64),
        row_lse=np.empty((B, Nq), np.float64), test_margin=np.empty((B, Nq), np.float64),
        top_gap=np.empty((B, Nq), np.float64), stop_node=np.empty(B, np.int32),
        final_cdf=np.empty((B, V), np.float64) if want_cdf else None)


def _dense_draft_probs(draft_probs, draft_to_target, V):
    """A draft model with a smaller vocabulary (paper section 4.1: a 32K-entry draft head) gives
    q over its own vocabulary; on the target vocabulary q(v) = q_sub[j] where v = draft_to_target[j]
    and 0 everywhere else.  The oracle works on that dense form: the definition, written out."""
    if draft_to_target is None or draft_probs is None:
        return draft_probs
    d2t = np.asarray(draft_to_target, dtype=np.int64)
    B, Nq, Vd = draft_probs.shape
    assert d2t.shape == (Vd,) and len(np.unique(d2t)) == Vd and d2t.min() >= 0 and d2t.max() < V
    dense = np.zeros((B, Nq, V), np.float32)
    dense[:, :, d2t] = draft_probs
    return dense


def accept_from_logits(*, logits, draft_tokens, draft_probs=None, uniforms=None, parents=None,
                       temperature, want_cdf=False, draft_to_target=None, without_replacement=False) -> AcceptResult:
    """Acceptance on given float64 logits [B, Nq, V].  without_replacement: the children of a tree node were drawn
    one after the other without replacement (see oracle_accept_logits_ex in aurora_oracle.c)."""
    lg = _chk(logits, np.float64)
    B, Nq, V = lg.shape
    draft_probs = _dense_draft_probs(draft_probs, draft_to_target, V)
    draft_tokens = _chk(draft_tokens, np.int32, (B, Nq))
    draft_probs = _chk(draft_probs, np.float32, (B, Nq, V))
    uniforms = _chk(uniforms, np.float32, (B, Nq, 2))
    parents = _chk(parents, np.int32, (B, Nq))
    r = _alloc_results(B, Nq, V, want_cdf and temperature > 0)
    st = lib().oracle_accept_logits_ex(
        C.c_int(B), C.c_int(Nq), C.c_int(V), C.c_double(float(np.float32(temperature))), _p(lg),
        _p(draft_tokens), _p(draft_probs), _p(uniforms), _p(parents), _p(r["accept_len"]),
        _p(r["next_token"]), _p(r["accept_mask"]), _p(r["p_at_draft"]), _p(r["row_lse"]),
        _p(r["test_margin"]), _p(r["top_gap"]), _p(r["stop_node"]), _p(r["final_cdf"]),
        C.c_int(1 if without_replacement else 0))
    if st != 0:
        raise ValueError(f"oracle_accept_logits status {st}")
    return AcceptResult(logits=None, **r)


def accept(*, hidden, lm_head, draft_tokens, draft_probs=None, uniforms=None, parents=None, dtype,
           temperature, want_cdf=False, want_logits=False, draft_to_target=None) -> AcceptResult:
    """LM head + acceptance.  hidden [B, Nq, H], lm_head [V, H].  The temperature is first
    rounded to float32 (the type it has at the library boundary), then widened."""
    ed = _elem_dtype(dtype)
    hidden = _chk(hidden, ed)
    B, Nq, H = hidden.shape
    lm_head = _chk(lm_head, ed)
    V = lm_head.shape[0]
    assert lm_head.shape[1] == H
    draft_tokens = _chk(draft_tokens, np.int32, (B, Nq))
    draft_probs = _chk(_dense_draft_probs(draft_probs, draft_to_target, V), np.float32, (B, Nq, V))
    uniforms = _chk(uniforms, np.float32, (B, Nq, 2))
    parents = _chk(parents, np.int32, (B, Nq))
    r = _alloc_results(B, Nq, V, want_cdf and temperature > 0)
    lg = np.empty((B, Nq, V), np.float64) if want_logits else None
    st = lib().oracle_accept(
        C.c_int(B), C.c_int(Nq), C.c_int(H), C.c_int(V), C.c_int(_DT[dtype]),
        C.c_double(float(np.float32(temperature))), _p(hidden), _p(lm_head), _p(draft_tokens),
        _p(draft_probs), _p(uniforms), _p(parents), _p(r["accept_len"]), _p(r["next_token"]),
        _p(r["accept_mask"]), _p(r["p_at_draft"]), _p(r["row_lse"]), _p(r["test_margin"]),
        _p(r["top_gap"]), _p(r["stop_node"]), _p(r["final_cdf"]), _p(lg))
    if st != 0:
        raise ValueError(f"oracle_accept status {st}")
    return AcceptResult(logits=lg, **r)


def verify(w, want_cdf=False, want_logits=False):
    """Both halves on a gen.Workload; returns (attention float64, AcceptResult)."""
    o = attn_workload(w)
    a = accept_workload(w, want_cdf=want_cdf, want_logits=want_logits)
    return o, a


def attn_workload(w) -> np.ndarray:
    """The attention half on a gen.Workload (K/V in the workload's dtype, or E4M3 codes with per-head scales)."""
    fp8 = getattr(w, "kv_dtype", "") == "fp8"
    return attn(q=w.q, k_pages=w.k_pages, v_pages=w.v_pages, block_table=w.host_block_table(),
                seq_lens=w.seq_lens, parents=w.parents, dtype=w.dtype,
                k_scale=w.k_scale if fp8 else None, v_scale=w.v_scale if fp8 else None)


def accept_workload(w, want_cdf=False, want_logits=False) -> AcceptResult:
    """The acceptance half on a gen.Workload (bf16 / f32 operands, or E4M3 operands with scales).  A workload with
    one temperature per request is verified request by request, each at its own temperature (0 = greedy):
    requests are independent, so that is the definition."""
    temps = getattr(w, "temperatures", None)
    if temps is not None:
        import dataclasses as _dc
        parts = []
        for b in range(w.batch):
            wb = _dc.replace(w.take_requests([b]), temperatures=None, temperature=float(np.float32(temps[b])))
            if wb.temperature == 0.0:   # a greedy call reads neither of them
                wb = _dc.replace(wb, draft_probs=None, uniforms=None)
            parts.append(accept_workload(wb, want_cdf=want_cdf and wb.temperature > 0, want_logits=want_logits))
        V = w.vocab
        def cat(name):
            vals = [getattr(p_, name) for p_ in parts]
            if name == "final_cdf":
                if not want_cdf:
                    return None
                return np.concatenate([v if v is not None else np.full((1, V), np.nan) for v in vals], axis=0)
            if any(v is None for v in vals):
                return None
            return np.concatenate(vals, axis=0)
        return AcceptResult(**{f.name: cat(f.name) for f in dataclasses.fields(AcceptResult)})
    wor = bool(getattr(w, "tree_without_replacement", False))
    if getattr(w, "head_dtype", "") == "fp8" or wor:
        if getattr(w, "head_dtype", "") == "fp8":
            lg = logits_fp8(hidden=w.hidden, hidden_scale=w.hidden_scale, lm_head=w.lm_head,
                            lm_head_scale=w.lm_head_scale)
        else:
            lg = logits(hidden=w.hidden, lm_head=w.lm_head, dtype=w.dtype)
        a = accept_from_logits(logits=lg, draft_tokens=w.draft_tokens, draft_probs=w.draft_probs,
                               uniforms=w.uniforms, parents=w.parents, temperature=w.temperature, want_cdf=want_cdf,
                               draft_to_target=getattr(w, "draft_to_target", None), without_replacement=wor)
        if want_logits:
            a.logits = lg
        return a
    return accept(hidden=w.hidden, lm_head=w.lm_head, draft_tokens=w.draft_tokens,
                  draft_probs=w.draft_probs, uniforms=w.uniforms, parents=w.parents, dtype=w.dtype,
                  temperature=w.temperature, want_cdf=want_cdf, want_logits=want_logits,
                  draft_to_target=getattr(w, "draft_to_target", None))


def trace_topk(logits: np.ndarray, top_k: int, draft_to_target=None):
    """K largest entries of each row of float32 logits [rows, V]: (ids int32 [rows, K], bf16 bits uint16 [rows, K]).
    With draft_to_target the selection runs over logits[:, draft_to_target] (the logits of the draft
    vocabulary, paper appendix A.2) and the ids are positions in that list."""
    if draft_to_target is not None:
        logits = np.ascontiguousarray(np.asarray(logits)[:, np.asarray(draft_to_target, dtype=np.int64)])
    logits = _chk(logits, np.float32)
    rows, V = logits.shape
    ids = np.empty((rows, top_k), np.int32)
    vals = np.empty((rows, top_k), np.uint16)
    st = lib().oracle_trace_topk(C.c_int64(rows), V, int(top_k), _p(logits), _p(ids), _p(vals))
    if st != 0:
        raise ValueError(f"oracle_trace_topk status {st}")
    return ids, vals


def trace_records(*, draft_tokens, parents, next_token, accept_mask):
    """(y_out int32 [B, Nq], trajectory codes int8 [B, Nq]) from the acceptance outputs."""
    draft_tokens = _chk(draft_tokens, np.int32)
    B, Nq = draft_tokens.shape
    parents = _chk(parents, np.int32, (B, Nq))
    next_token = _chk(next_token, np.int32, (B,))
    accept_mask = _chk(accept_mask, np.uint8, (B, Nq))
    y = np.empty((B, Nq), np.int32)
    r = np.empty((B, Nq), np.int8)
    st = lib().oracle_trace_records(B, Nq, _p(draft_tokens), _p(parents), _p(next_token), _p(accept_mask), _p(y), _p(r))
    if st != 0:
        raise ValueError(f"oracle_trace_records status {st}")
    return y, r


def draft_loss(*args, **kw):
    """Drafter training loss of paper eq. 3 on a batch of trace rows (see oracle/loss_oracle.py)."""
    from .loss_oracle import draft_loss as _impl
    return _impl(*args, **kw)


def trace_pack(*args, **kw):
    """Packing of the trace records of the rows that carry a training signal (see oracle/pack_oracle.py)."""
    from .pack_oracle import trace_pack as _impl
    return _impl(*args, **kw)


def attn_lse(*args, **kw):
    """Logsumexp of every attention row (see oracle/attn_bwd_oracle.py)."""
    from .attn_bwd_oracle import attn_lse as _impl
    return _impl(*args, **kw)


def attn_backward(*args, **kw):
    """Backward pass of the chunk / tree attention (see oracle/attn_bwd_oracle.py)."""
    from .attn_bwd_oracle import attn_backward as _impl
    return _impl(*args, **kw)
