"""Seeded synthetic inputs for the speculative-verification step.

This module only *draws inputs*; it holds none of the verification method's
arithmetic (no attention, no acceptance test, no residual sampling).  Both the
CPU oracle and the HIP path consume exactly the arrays produced here.

The draft model is an input of the method.  Where a workload needs a draft
distribution that is correlated with the target model (so that acceptance is
partial, as in serving), the stand-in draft model is "a float32 library matmul
of the already rounded hidden states and LM-head weight, plus Gaussian noise,
soft-maxed".  Those float32 logits are used for nothing but drawing
`draft_probs` / `draft_tokens`; neither verification path ever sees them.

Shapes follow the serving settings the paper reports (Appendix B, Table 3:
5 speculative steps / 6 draft tokens per step; lookahead 3-5 in Tables 4-5;
vocabularies of 128K and 152K in Appendix A.2), on Llama-3-8B / Qwen3-8B head
geometry.

Array conventions (all NumPy, C-contiguous):
  q            [B, Nq, Hq, D]          float32, or uint16 holding bf16 bits
  k_pages      [P, Hkv, page, D]       same dtype as q
  v_pages      [P, Hkv, page, D]       same dtype as q
  block_table  [B, max_pages] int32    page ids, unused entries -1
  seq_lens     [B] int32               KV length including the Nq chunk tokens
  parents      [B, Nq] int32 or None   None => chain (parent[i] = i - 1)
  hidden       [B, Nq, H]              same dtype as q
  lm_head      [V, H]                  same dtype as q
  draft_tokens [B, Nq] int32           entry 0 (root) unused
  draft_probs  [B, Nq, V] float32      row n = distribution node n's children
                                       were drawn from; None when greedy
  uniforms     [B, Nq, 2] float32      in [0, 1), exactly k * 2**-24; None when greedy
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"

_CHUNK = 1 << 22  # elements per independently seeded chunk of a big tensor


# --------------------------------------------------------------------------
# dtype plumbing (storage format only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize_e4m3_rows(x: np.ndarray):
    """Per-row 8-bit storage of a float32 matrix: codes (uint8, OCP E4M3) and one float32 scale per
    row with scale = max|row| / 448, so that scale * decode(code) approximates x.  The rounding is the
    library's float32 -> float8_e4m3fn conversion.  Storage format only: both sides of a parity test
    consume the codes and scales this returns."""
    import torch
    x = np.ascontiguousarray(x, dtype=np.float32)
    amax = np.abs(x).max(axis=-1, keepdims=True)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    q = torch.from_numpy(x / scale).to(torch.float8_e4m3fn)
    return q.view(torch.uint8).numpy(), scale.reshape(x.shape[:-1])


def e4m3_rows_to_f32(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """The values a per-row quantised matrix stands for, as float32 (library decode times the scale)."""
    import torch
    v = torch.from_numpy(np.ascontiguousarray(codes)).view(torch.float8_e4m3fn).float().numpy()
    return v * np.asarray(scale, dtype=np.float32)[..., None]


def quantize_e4m3_heads(x: np.ndarray):
    """8-bit storage of a paged pool [P, Hkv, page, D] (float32): uint8 E4M3 codes and one float32 scale
    per KV head, scale[h] = max|x[:, h]| / 448.  Same rounding as quantize_e4m3_rows."""
    import torch
    x = np.ascontiguousarray(x, dtype=np.float32)
    amax = np.abs(x).max(axis=(0, 2, 3))
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    q = torch.from_numpy(x / scale[None, :, None, None]).to(torch.float8_e4m3fn)
    return q.view(torch.uint8).numpy(), scale


def as_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    """The values a stored tensor holds, as float32 (exact for both dtypes)."""
    return bf16_bits_to_f32(x) if dtype == BF16 else np.asarray(x, dtype=np.float32)


# --------------------------------------------------------------------------
# random tensors
# --------------------------------------------------------------------------
def _normal_tensor(seed_seq: np.random.SeedSequence, shape, std: float, dtype: str,
                   threads: int = 8) -> np.ndarray:
    """N(0, std^2) drawn in float32 and rounded once to `dtype`.

    The tensor is cut into fixed-size chunks, each with its own child seed, so
    the result does not depend on the number of threads.
    """
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16 if dtype == BF16 else np.float32)
    nchunks = (n + _CHUNK - 1) // _CHUNK
    children = seed_seq.spawn(max(nchunks, 1))

    def work(c):
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        g = np.random.Generator(np.random.PCG64(children[c]))
        v = g.standard_normal(hi - lo, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        out[lo:hi] = f32_to_bf16_bits(v) if dtype == BF16 else v

    if nchunks <= 1 or threads <= 1:
        for c in range(nchunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(nchunks)))
    return out.reshape(shape)


def _uniform24(rng: np.random.Generator, shape) -> np.ndarray:
    """Uniforms in [0,1) that float32 holds exactly: (32 random bits >> 8) * 2**-24."""
    bits = rng.integers(0, 1 << 32, size=shape, dtype=np.uint64).astype(np.uint32)
    return ((bits >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)).astype(np.float32)


def _softmax_rows_f32(z: np.ndarray) -> np.ndarray:
    """Row softmax used only to turn stand-in draft logits into draft_probs (float64 inside)."""
    z = z.astype(np.float64)
    z -= z.max(axis=-1, keepdims=True)
    np.exp(z, out=z)
    z /= z.sum(axis=-1, keepdims=True)
    return z.astype(np.float32)


def _draw_from_rows(rng: np.random.Generator, probs: np.ndarray) -> np.ndarray:
    """One categorical draw per row of `probs` ([R, V] float32)."""
    cdf = np.cumsum(probs.astype(np.float64), axis=-1)
    u = rng.random(probs.shape[0]) * cdf[:, -1]
    idx = np.array([np.searchsorted(cdf[r], u[r], side="right") for r in range(probs.shape[0])])
    return np.minimum(idx, probs.shape[1] - 1).astype(np.int32)


# --------------------------------------------------------------------------
# workload container
# --------------------------------------------------------------------------
@dataclasses.dataclass
class Workload:
    name: str
    seed: int
    dtype: str
    batch: int
    num_q: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    max_pages_per_seq: int
    num_pages: int
    hidden_size: int
    vocab: int
    temperature: float
    q: np.ndarray
    k_pages: np.ndarray
    v_pages: np.ndarray
    block_table: np.ndarray
    seq_lens: np.ndarray
    parents: Optional[np.ndarray]
    hidden: np.ndarray
    lm_head: np.ndarray
    draft_tokens: np.ndarray
    draft_probs: Optional[np.ndarray]
    uniforms: Optional[np.ndarray]
    recipe: str = ""
    # sparse pools only: k_pages/v_pages hold one compact slot per referenced page and
    # page_ids[i] is the pool id (the value block_table uses) of compact slot i
    page_ids: Optional[np.ndarray] = None
    # draft model with its own, smaller vocabulary: draft_probs is [B, Nq, draft_vocab] and
    # draft_to_target[j] is the target id of draft entry j (ascending); 0 / None otherwise
    draft_vocab: int = 0
    draft_to_target: Optional[np.ndarray] = None
    # LM-head operands in 8-bit floating point: head_dtype == "fp8" => hidden / lm_head hold uint8 E4M3
    # codes and hidden_scale [B, Nq] / lm_head_scale [V] the per-row float32 scales ("" = as `dtype`)
    head_dtype: str = ""
    hidden_scale: Optional[np.ndarray] = None
    lm_head_scale: Optional[np.ndarray] = None
    # KV cache in 8-bit floating point: kv_dtype == "fp8" => k_pages / v_pages hold uint8 E4M3 codes and
    # k_scale / v_scale [num_kv_heads] the float32 scale of each KV head ("" = as `dtype`)
    kv_dtype: str = ""
    k_scale: Optional[np.ndarray] = None
    v_scale: Optional[np.ndarray] = None
    # one temperature per request (float32 [B]; 0 = that request is verified greedily), or None: `temperature`
    temperatures: Optional[np.ndarray] = None
    # tree drafts whose siblings were drawn one after the other without replacement
    tree_without_replacement: bool = False

    def target_to_draft(self) -> Optional[np.ndarray]:
        """Inverse of draft_to_target over the target vocabulary, -1 where the draft model has no entry."""
        if self.draft_to_target is None:
            return None
        inv = np.full(self.vocab, -1, dtype=np.int32)
        inv[self.draft_to_target] = np.arange(len(self.draft_to_target), dtype=np.int32)
        return inv

    @property
    def num_draft(self) -> int:
        """Draft tokens per request (k for a chain, nodes-1 for a tree)."""
        return self.num_q - 1

    def host_block_table(self) -> np.ndarray:
        """Block table that indexes the host copy of the pools (differs from block_table only
        for sparse pools, where it points at compact slots)."""
        if self.page_ids is None:
            return self.block_table
        order = np.argsort(self.page_ids)
        pos = np.searchsorted(self.page_ids[order], np.maximum(self.block_table, 0))
        pos = np.minimum(pos, len(order) - 1)
        return np.where(self.block_table >= 0, order[pos], -1).astype(np.int32)

    def take_requests(self, idx) -> "Workload":
        """A workload holding only requests `idx` (page pool kept whole)."""
        idx = np.asarray(idx, dtype=np.int64)
        sl = lambda a: None if a is None else np.ascontiguousarray(a[idx])
        return dataclasses.replace(
            self, batch=len(idx), q=sl(self.q), block_table=sl(self.block_table),
            seq_lens=sl(self.seq_lens), parents=sl(self.parents), hidden=sl(self.hidden),
            draft_tokens=sl(self.draft_tokens), draft_probs=sl(self.draft_probs),
            uniforms=sl(self.uniforms), hidden_scale=sl(self.hidden_scale), temperatures=sl(self.temperatures))


# --------------------------------------------------------------------------
# pieces
# --------------------------------------------------------------------------
def make_kv(ss: np.random.SeedSequence, rng: np.random.Generator, seq_lens: np.ndarray,
            num_kv_heads: int, head_dim: int, page_size: int, dtype: str,
            slack: float = 0.10, shuffle: bool = True, pool_pages: Optional[int] = None, kv_fp8: bool = False):
    """Paged K/V pools and a block table.

    kv_fp8: the pools are drawn as float32 N(0,1), KV head h scaled by 2^(h mod 3 - 1) (so that the heads'
    scales differ), and stored as E4M3 codes with one scale per head; two more values are returned.

    pool_pages=None: the pool holds the referenced pages plus `slack` spare
    ones and the block table is a random permutation of pool ids (shuffle) or
    the identity.  pool_pages=P: referenced pages are drawn without
    replacement from a pool of P ids, and only a *compact* pool (one slot per
    referenced page) is returned together with `page_ids`, the pool id of each
    compact slot; the caller scatters compact slot i to device page
    page_ids[i].
    """
    B = len(seq_lens)
    pages_per = (seq_lens.astype(np.int64) + page_size - 1) // page_size
    used = int(pages_per.sum())
    max_pages = int(pages_per.max())
    if pool_pages is None:
        P = used + int(np.ceil(used * slack)) if shuffle else used
        ids = rng.permutation(P)[:used] if shuffle else np.arange(used)
        page_ids = None
    else:
        P = int(pool_pages)
        ids = rng.choice(P, size=used, replace=False)
        page_ids = ids.astype(np.int64)
    block_table = np.full((B, max_pages), -1, dtype=np.int32)
    o = 0
    for b in range(B):
        n = int(pages_per[b])
        block_table[b, :n] = ids[o:o + n]
        o += n
    kss, vss = ss.spawn(2)
    n_store = P if pool_pages is None else used
    shape = (n_store, num_kv_heads, page_size, head_dim)
    if kv_fp8:
        gain = np.exp2((np.arange(num_kv_heads) % 3 - 1).astype(np.float32))[None, :, None, None]
        k_pages, k_scale = quantize_e4m3_heads(_normal_tensor(kss, shape, 1.0, F32) * gain)
        v_pages, v_scale = quantize_e4m3_heads(_normal_tensor(vss, shape, 1.0, F32) * gain[:, ::-1])
        return k_pages, v_pages, block_table, P, max_pages, page_ids, k_scale, v_scale
    k_pages = _normal_tensor(kss, shape, 1.0, dtype)
    v_pages = _normal_tensor(vss, shape, 1.0, dtype)
    return k_pages, v_pages, block_table, P, max_pages, page_ids


def random_tree_parents(rng: np.random.Generator, batch: int, nodes: int,
                        max_children: int = 4, max_depth: int = 6) -> np.ndarray:
    """parents[b, n] for a draft tree: node 0 is the root (-1); node n's parent is uniform over
    earlier nodes that still have fewer than `max_children` children and depth < max_depth."""
    parents = np.full((batch, nodes), -1, dtype=np.int32)
    for b in range(batch):
        depth = np.zeros(nodes, dtype=np.int64)
        nchild = np.zeros(nodes, dtype=np.int64)
        for n in range(1, nodes):
            cand = [m for m in range(n) if depth[m] <= max_depth - 1 and nchild[m] < max_children]
            m = int(cand[rng.integers(0, len(cand))])
            parents[b, n] = m
            depth[n] = depth[m] + 1
            nchild[m] += 1
    return parents


def chain_parents(batch: int, num_q: int) -> np.ndarray:
    p = np.arange(-1, num_q - 1, dtype=np.int32)
    return np.ascontiguousarray(np.broadcast_to(p, (batch, num_q)))


def _standin_target_logits(hidden: np.ndarray, lm_head: np.ndarray, dtype: str) -> np.ndarray:
    """float32 BLAS product hidden . lm_head^T of the rounded inputs, vocab-chunked.
    Input synthesis for the stand-in draft model only."""
    h = as_f32(hidden, dtype).reshape(-1, hidden.shape[-1])
    V = lm_head.shape[0]
    out = np.empty((h.shape[0], V), dtype=np.float32)
    step = 16384
    for v0 in range(0, V, step):
        v1 = min(V, v0 + step)
        out[:, v0:v1] = h @ as_f32(lm_head[v0:v1], dtype).T
    return out


# --------------------------------------------------------------------------
# the general builder
# --------------------------------------------------------------------------
def make_workload(*, name: str, seed: int, dtype: str, batch: int, num_q: int,
                  num_q_heads: int, num_kv_heads: int, head_dim: int, page_size: int,
                  hidden_size: int, vocab: int, temperature: float,
                  seq_lens, draft: str, draft_noise: float = 1.0,
                  tree: bool = False, greedy_hit: float = 0.7,
                  shuffle_pages: bool = True, pool_pages: Optional[int] = None,
                  distinct_siblings: bool = False, draft_vocab: Optional[int] = None,
                  head_fp8: bool = False, kv_fp8: bool = False, temperatures=None,
                  siblings_without_replacement: bool = False, recipe: str = "") -> Workload:
    """Build one workload.

    draft = "independent": draft logits ~ N(0,1), draft tokens uniform over the vocab.
    draft = "noisy_target": draft logits = stand-in target logits / T + N(0, draft_noise)/T,
            i.e. softmax((target + noise)/T); each draft token is drawn from its parent's row.
    draft = "greedy_mix": token = argmax of the stand-in target logits of the parent row with
            probability `greedy_hit`, else uniform; draft_probs/uniforms are None.
    draft_vocab (with "noisy_target"): the draft model's vocabulary is a random subset of that many
            target ids; draft_probs is over the subset, tokens are drawn from it and stored as target ids.
    siblings_without_replacement (trees with "noisy_target"): the children of a node are drawn one after the
            other, each from the parent's row with the earlier siblings' tokens removed and renormalised.
    head_fp8: hidden and lm_head are drawn as float32 with the same recipe, then stored as E4M3 codes
            with one scale per row; the stand-in target logits use the values the codes stand for.
    kv_fp8: the K/V pools are stored as E4M3 codes with one scale per KV head (see make_kv).
    temperatures (with "noisy_target"): one temperature per request; the draft distribution of request b is
            softmax((target + noise) / T_b), with T_b = 1 standing in for a greedy request (T_b = 0).
    """
    ss = np.random.SeedSequence([int(seed), 0x2602_06932 & 0xFFFFFFFF])
    s_q, s_kv, s_h, s_w, s_misc = ss.spawn(5)
    rng = np.random.Generator(np.random.PCG64(s_misc))
    B, Nq, V = batch, num_q, vocab
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    assert seq_lens.shape == (B,) and int(seq_lens.min()) >= Nq

    q = _normal_tensor(s_q, (B, Nq, num_q_heads, head_dim), 1.0, dtype)
    k_scale = v_scale = None
    kv = make_kv(s_kv, rng, seq_lens, num_kv_heads, head_dim, page_size, dtype,
                 shuffle=shuffle_pages, pool_pages=pool_pages, kv_fp8=kv_fp8)
    if kv_fp8:
        k_pages, v_pages, block_table, P, max_pages, page_ids, k_scale, v_scale = kv
    else:
        k_pages, v_pages, block_table, P, max_pages, page_ids = kv
    hidden_scale = lm_head_scale = None
    head_values = None  # (hidden, lm_head) as float32 when they are not stored in `dtype`
    if head_fp8:
        hidden, hidden_scale = quantize_e4m3_rows(_normal_tensor(s_h, (B, Nq, hidden_size), 1.0, F32))
        lm_head, lm_head_scale = quantize_e4m3_rows(_normal_tensor(s_w, (V, hidden_size), 0.02, F32))
        head_values = (e4m3_rows_to_f32(hidden, hidden_scale), e4m3_rows_to_f32(lm_head, lm_head_scale))
    else:
        hidden = _normal_tensor(s_h, (B, Nq, hidden_size), 1.0, dtype)
        lm_head = _normal_tensor(s_w, (V, hidden_size), 0.02, dtype)

    def standin():
        if head_values is not None:
            return _standin_target_logits(head_values[0], head_values[1], F32)
        return _standin_target_logits(hidden, lm_head, dtype)

    parents = random_tree_parents(rng, B, Nq) if tree else None
    par = parents if tree else chain_parents(B, Nq)

    draft_tokens = np.zeros((B, Nq), dtype=np.int32)
    draft_probs = None
    uniforms = None
    d2t = None
    assert not draft_vocab or draft == "noisy_target"
    if draft == "independent":
        draft_tokens[:, 1:] = rng.integers(0, V, size=(B, Nq - 1), dtype=np.int64)
        z = rng.standard_normal((B * Nq, V), dtype=np.float32)
        draft_probs = _softmax_rows_f32(z).reshape(B, Nq, V)
        uniforms = _uniform24(rng, (B, Nq, 2))
    elif draft == "noisy_target":
        t = standin()
        T = np.float32(temperature if temperature > 0 else 1.0)
        if temperatures is not None:
            tb = np.asarray(temperatures, dtype=np.float32)
            assert tb.shape == (B,) and (tb >= 0).all()
            T = np.repeat(np.where(tb > 0, tb, np.float32(1.0)).astype(np.float32), Nq)[:, None]
        if draft_vocab:
            d2t = np.sort(rng.choice(V, size=int(draft_vocab), replace=False)).astype(np.int32)
            t = np.ascontiguousarray(t[:, d2t])
        noise = rng.standard_normal(t.shape, dtype=np.float32) * np.float32(draft_noise)
        draft_probs = _softmax_rows_f32((t + noise) / T).reshape(B, Nq, t.shape[1])
        del t, noise
        drawn = np.full((B, Nq), -1, dtype=np.int64)   # index within the draft vocabulary of node n's token
        for n in range(1, Nq):
            rows = draft_probs[np.arange(B), par[:, n]]
            if siblings_without_replacement:
                # the drafter draws the children of a node one after the other, each from q with the earlier
                # siblings' tokens removed and the rest renormalised
                rows = rows.copy()
                for m in range(1, n):
                    same = np.flatnonzero(par[:, m] == par[:, n])
                    rows[same, drawn[same, m]] = 0.0
                rows /= rows.sum(axis=1, keepdims=True, dtype=np.float64).astype(np.float32)
            idx = _draw_from_rows(rng, rows)
            drawn[:, n] = idx
            draft_tokens[:, n] = d2t[idx] if draft_vocab else idx
        uniforms = _uniform24(rng, (B, Nq, 2))
    elif draft == "greedy_mix":
        t = standin().reshape(B, Nq, V)
        top = t.argmax(axis=-1).astype(np.int32)
        del t
        for n in range(1, Nq):
            hit = rng.random(B) < greedy_hit
            rnd = rng.integers(0, V, size=B, dtype=np.int64).astype(np.int32)
            draft_tokens[:, n] = np.where(hit, top[np.arange(B), par[:, n]], rnd)
        if distinct_siblings and tree:
            for b in range(B):
                for n in range(1, Nq):
                    sib = [m for m in range(1, n) if par[b, m] == par[b, n]]
                    while any(draft_tokens[b, m] == draft_tokens[b, n] for m in sib):
                        draft_tokens[b, n] = (draft_tokens[b, n] + 1) % V
    else:
        raise ValueError(draft)

    w = Workload(name=name, seed=seed, dtype=dtype, batch=B, num_q=Nq, num_q_heads=num_q_heads,
                 num_kv_heads=num_kv_heads, head_dim=head_dim, page_size=page_size,
                 max_pages_per_seq=max_pages, num_pages=P, hidden_size=hidden_size, vocab=V,
                 temperature=float(temperature), q=q, k_pages=k_pages, v_pages=v_pages,
                 block_table=block_table, seq_lens=seq_lens, parents=parents, hidden=hidden,
                 lm_head=lm_head, draft_tokens=draft_tokens, draft_probs=draft_probs,
                 uniforms=uniforms, recipe=recipe, page_ids=page_ids,
                 draft_vocab=int(draft_vocab or 0), draft_to_target=d2t,
                 head_dtype="fp8" if head_fp8 else "", hidden_scale=hidden_scale, lm_head_scale=lm_head_scale,
                 kv_dtype="fp8" if kv_fp8 else "", k_scale=k_scale, v_scale=v_scale,
                 temperatures=None if temperatures is None else np.asarray(temperatures, dtype=np.float32),
                 tree_without_replacement=bool(siblings_without_replacement and tree))
    return w


# --------------------------------------------------------------------------
# the five named benchmark configurations, with size overrides
# for reduced parity cases
# --------------------------------------------------------------------------
def tiny_chain(seed: int = 1, **kw) -> Workload:
    """Config 1: fp32, B 4, k 4, context 256 held in one contiguous page per request."""
    p = dict(batch=4, num_q=5, num_q_heads=8, num_kv_heads=2, head_dim=64, page_size=256,
             hidden_size=256, vocab=1024, temperature=1.0, dtype=F32)
    seq = kw.pop("seq_lens", None)
    p.update(kw)
    if seq is None:
        seq = np.full(p["batch"], 256, dtype=np.int32)
    return make_workload(name="tiny_chain_f32", seed=seed, seq_lens=seq, draft="independent",
                         shuffle_pages=False,
                         recipe="config 1: tiny chain verify, fp32, contiguous KV", **p)


def llama_chain(seed: int = 1, len_lo: int = 1024, len_hi: int = 4096, **kw) -> Workload:
    """Config 2: Llama-3-8B shape, bf16, B 32, k 4, L ~ U{1024..4096}, page 16, shuffled table,
    draft = target + N(0,1) noise, T 1."""
    p = dict(batch=32, num_q=5, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
             hidden_size=4096, vocab=128256, temperature=1.0, dtype=BF16, draft_noise=1.0)
    p.update(kw)
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 2])))
    seq = rng.integers(len_lo, len_hi + 1, size=p["batch"]).astype(np.int32)
    return make_workload(name="llama3_8b_chain_k4", seed=seed, seq_lens=seq, draft="noisy_target",
                         recipe="config 2: Llama-3-8B-shaped chain verify, bf16", **p)


def qwen_greedy_chain(seed: int = 1, len_lo: int = 512, len_hi: int = 8192, **kw) -> Workload:
    """Config 3: greedy (T 0), Qwen3-8B vocab, B 64, k 6, L ~ U{512..8192}."""
    p = dict(batch=64, num_q=7, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
             hidden_size=4096, vocab=151936, temperature=0.0, dtype=BF16)
    p.update(kw)
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 3])))
    seq = rng.integers(len_lo, len_hi + 1, size=p["batch"]).astype(np.int32)
    return make_workload(name="qwen3_8b_greedy_k6", seed=seed, seq_lens=seq, draft="greedy_mix",
                         recipe="config 3: greedy chain verify, Qwen3-8B vocab, bf16", **p)


def llama_tree(seed: int = 1, context: int = 4096, **kw) -> Workload:
    """Config 4: 32-node draft tree per request (branching <= 4, depth <= 6), B 16, context 4096."""
    p = dict(batch=16, num_q=32, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
             hidden_size=4096, vocab=128256, temperature=1.0, dtype=BF16, draft_noise=1.0)
    p.update(kw)
    seq = np.full(p["batch"], context, dtype=np.int32)
    return make_workload(name="llama3_8b_tree32", seed=seed, seq_lens=seq, draft="noisy_target",
                         tree=True, recipe="config 4: tree-draft verify, bf16", **p)


def stress_chain(seed: int = 1, len_lo: int = 256, len_hi: int = 32768,
                 pool_pages: Optional[int] = None, **kw) -> Workload:
    """Config 5: B 256, k 4, L log-uniform in [256, 32768], 48/8/128 heads, H 6144, V 200064,
    draft = target + N(0, 0.5), T 0.7.  pool_pages selects a sparse pool (see make_kv)."""
    p = dict(batch=256, num_q=5, num_q_heads=48, num_kv_heads=8, head_dim=128, page_size=16,
             hidden_size=6144, vocab=200064, temperature=0.7, dtype=BF16, draft_noise=0.5)
    p.update(kw)
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 5])))
    seq = np.rint(np.exp(rng.uniform(np.log(len_lo), np.log(len_hi), size=p["batch"]))).astype(np.int32)
    return make_workload(name="stress_b256_longctx", seed=seed, seq_lens=seq, draft="noisy_target",
                         pool_pages=pool_pages,
                         recipe="config 5: large-batch long-context stress, bf16", **p)
