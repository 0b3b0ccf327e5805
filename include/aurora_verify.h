/*
 * aurora_verify.h - C ABI of the MI355X (gfx950) implementation of the target-model
 * verification step of speculative decoding, the step of the Aurora serving loop that
 * checks the drafted tokens and emits the accept / reject outcome the speculator is
 * trained on (paper sections 2.1, 3.1, 3.3; tree form: section 3.2 and figure 2;
 * logits l in R^{T x V}: appendix A.1, eq. 4).
 *
 * Conventions for every entry point
 *   - Every data pointer is CALLER-OWNED DEVICE memory on the current HIP device.
 *     Descriptors are host structs, read during the call and not retained.
 *     q, k_pages, v_pages, out, hidden and lm_head must be 16-byte aligned
 *     (AURORA_ERR_INVALID_ARG otherwise).
 *   - The library allocates nothing and keeps no state that changes results between calls.  What it does keep,
 *     per process: the test knob aurora_debug_set_tree_spin_limit, per-device facts looked up once (compute-unit
 *     count, "large LDS enabled for this kernel"), and the fixed scratch array of aurora_verify_attn_static.
 *     All other scratch lives in the
 *     caller's `workspace` (device memory, 256-byte aligned, at least
 *     aurora_verify_workspace_bytes() bytes).  No pointer is retained after the
 *     enqueued work completes.  Calls with distinct workspaces may overlap.
 *   - Calls are asynchronous: they enqueue kernels on `hip_stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and return.  Outputs are valid
 *     once the caller has synchronised that stream.
 *   - Return value: AURORA_OK or a negative AURORA_ERR_* code.  Validation is done on
 *     the host from the descriptors and pointers only (null pointers, head-count
 *     divisibility, supported head_dim / dtype / num_q, workspace size); when it fails
 *     nothing is enqueued.  Device-side contents (page ids in range, seq_lens >= num_q,
 *     parents[n] < n, token ids in range) are NOT checked.
 *   - Deterministic: the same inputs give bit-identical outputs from run to run.
 *   - There is no CPU fallback: without a HIP device every compute entry point
 *     returns AURORA_ERR_HIP.
 */
#ifndef AURORA_VERIFY_H
#define AURORA_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  AURORA_OK = 0,
  AURORA_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, Hq % Hkv != 0, ...      */
  AURORA_ERR_UNSUPPORTED = -2, /* well-formed but outside what the kernels cover           */
  AURORA_ERR_WORKSPACE = -3,   /* workspace null, misaligned or too small                  */
  AURORA_ERR_HIP = -4,         /* a HIP runtime call or kernel launch failed               */
  AURORA_ERR_TOO_LARGE = -5    /* aurora_verify_attn_static: needs more than AURORA_STATIC_SCRATCH_BYTES */
};

/* Size of the fixed scratch array behind aurora_verify_attn_static (bytes, per GPU the library runs on). */
#define AURORA_STATIC_SCRATCH_BYTES (16u << 20)

enum { AURORA_F32 = 0, AURORA_BF16 = 1, AURORA_FP8_E4M3 = 2 /* LM-head operands only, see aurora_accept_desc */ };

/* Attention half.  Nq query positions per request (k+1 for a chain of k drafts, or the
 * number of nodes of a draft tree, root included) attend to a paged GQA KV cache. */
typedef struct {
  int32_t batch;             /* B >= 0 (0: nothing is enqueued)                              */
  int32_t num_q;             /* Nq, 1..64                                                    */
  int32_t num_q_heads;       /* Hq                                                           */
  int32_t num_kv_heads;      /* Hkv, Hq % Hkv == 0                                           */
  int32_t head_dim;          /* D: 64 or 128                                                 */
  int32_t page_size;         /* tokens per KV page (any value >= 1; 16 is the tuned case)    */
  int32_t max_pages_per_seq; /* row stride of block_table                                    */
  int64_t num_pages;         /* P, pages in each of the K and V pools                        */
  int32_t dtype;             /* AURORA_F32 / AURORA_BF16: type of q, k_pages, v_pages, out   */
  float sm_scale;            /* softmax scale; 0 => 1/sqrt(head_dim)                         */
  /* KV cache in 8-bit floating point (the paper serves its frontier targets in FP8, sections 1 and 4.3;
   * what is stored in 8 bits, the format and the scaling are this library's choice).  kv_fp8 = 0: k_pages
   * and v_pages are of type `dtype`.  kv_fp8 = 1: they hold OCP E4M3 codes, one byte per element, same
   * [P, Hkv, page_size, D] layout, and a stored element of KV head h stands for k_scale[h] * decode(code)
   * (v_scale[h] for V); k_scale and v_scale are DEVICE pointers to float32 [Hkv].  q and out stay of type
   * `dtype`.  The codes are widened exactly to the type the products run in, so the only rounding this
   * adds is the one the caller made when it quantised the cache. */
  int32_t kv_fp8;
  const float* k_scale;
  const float* v_scale;
} aurora_attn_desc;

/* Acceptance half: LM head, softmax statistics, acceptance walk, residual / bonus draw. */
typedef struct {
  int32_t batch;     /* B                                                                    */
  int32_t num_q;     /* Nq, 1..64                                                            */
  int32_t hidden;    /* H (bf16: multiple of 8)                                              */
  int32_t vocab;     /* V (tree sampling, i.e. parents != NULL with T > 0: V <= 2^20)           */
  int32_t dtype;     /* type of hidden and lm_head: AURORA_F32, AURORA_BF16 or AURORA_FP8_E4M3      */
  float temperature; /* 0 => greedy (arg-max prefix); > 0 => speculative rejection sampling  */
  /* Draft model with a smaller vocabulary than the target (section 4.1: a 32K-entry draft head;
   * appendix A.2: 32K vs 128K / 152K).  draft_vocab = 0: draft_probs rows are dense over V.
   * draft_vocab = Vd in 1..V: draft_probs is [B, Nq, Vd] over the draft vocabulary and
   * target_to_draft (DEVICE pointer, [V] int32) gives for every target id its index in a row of
   * draft_probs, or -1 for ids the draft model cannot emit - there q = 0, so the residual
   * max(0, p - q) keeps all of p's mass.  draft_tokens stay target ids.  Ignored when T == 0. */
  int32_t draft_vocab;
  const int32_t* target_to_draft;
  /* dtype == AURORA_FP8_E4M3 (the paper serves its frontier targets in FP8, sections 1 and 4.3; format
   * and scaling are this library's choice): hidden and lm_head hold OCP E4M3 codes, one byte per element
   * (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities), and a stored element stands
   * for scale * decode(code) with one float32 scale per token row, hidden_scale [B*Nq], and one per
   * vocabulary row, lm_head_scale [V] (DEVICE pointers).  H must be a multiple of 128.  Logits and
   * everything after them are fp32 / fp64 as for the other types. */
  const float* hidden_scale;
  const float* lm_head_scale;
  /* One temperature per request (a serving batch mixes sampling settings; the paper's formulation has one).
   * NULL: `temperature` applies to every request.  Otherwise a DEVICE pointer to float32 [B]; `temperature`
   * is ignored, request b is verified at temperatures[b] > 0, or greedily if temperatures[b] == 0 (its
   * draft_probs / uniforms rows are then not read, row_lse is that of the raw logits and p_at_draft is
   * 1 / 0 as in a greedy call).  draft_probs and uniforms must be given. */
  const float* temperatures;
  /* Tree drafts at a temperature > 0: how the children of a node were drawn (the paper's tree verification does
   * not say).  0: independently from the parent's draft distribution q - after a rejection q stays as it is.
   * Non-zero: one after the other without replacement - a rejected child's token is removed from q (set to 0,
   * the rest divided by the mass that is left, the row being taken to sum to 1) for the tests and residuals of
   * its later siblings.  Ignored for chains and greedy requests. */
  int32_t tree_without_replacement;
} aurora_accept_desc;

/* Bytes of workspace needed by aurora_verify / _attn / _accept for these descriptors.
 * Either descriptor may be NULL (that half then needs nothing).  Host only. */
int aurora_verify_workspace_bytes(const aurora_attn_desc* attn, const aurora_accept_desc* accept,
                                  size_t* out_bytes);

/*
 * Chunk attention of the draft positions over the cached context (sections 3.1, 3.2).
 *
 *   out[b, n, hq, :] = sum_j softmax_j( sm_scale * <q[b, n, hq, :], K_j> ) V_j
 *
 * over the KV positions j of request b that node n may see: the whole prefix
 * j < L_b - Nq, plus the chunk slots L_b - Nq + a of a in {n and its ancestors}.  For a
 * chain (parents == NULL, parent[i] = i-1) that is plain causal masking.  Query head hq
 * reads KV head hq / (Hq / Hkv).  KV position j of request b is stored in page
 * block_table[b][j / page_size] at in-page offset j % page_size.
 * Numerics: fp32 path - everything in fp32.  bf16 path - scores and softmax in fp32, the
 * probabilities rounded to bf16 for the P.V product, fp32 accumulation, output rounded to bf16.
 */
int aurora_verify_attn(const aurora_attn_desc* desc,
                       const void* q,              /* [B, Nq, Hq, D]                          */
                       const void* k_pages,        /* [P, Hkv, page_size, D] (E4M3 codes if kv_fp8) */
                       const void* v_pages,        /* [P, Hkv, page_size, D]                  */
                       const int32_t* block_table, /* [B, max_pages_per_seq]; unused = -1     */
                       const int32_t* seq_lens,    /* [B] KV length INCLUDING the Nq chunk tokens */
                       const int32_t* parents,     /* [B, Nq], parents[b,0] = -1, parents[b,n] < n; or NULL */
                       void* out,                  /* [B, Nq, Hq, D], same dtype as q         */
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * aurora_verify_attn for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * `out`; the partial results the kernels exchange live in a fixed array of AURORA_STATIC_SCRATCH_BYTES (16 MiB)
 * inside the library instead of a caller's workspace - one copy per GPU, held until the process ends.  The call
 * allocates and frees nothing (the array's device address is looked up once per device, on the first call there).
 *   - Returns AURORA_ERR_TOO_LARGE, with nothing enqueued, when aurora_verify_workspace_bytes(desc, NULL) exceeds
 *     AURORA_STATIC_SCRATCH_BYTES (the headline shape - 32 requests, 8 KV heads, 20 query rows per KV head - needs
 *     12.6 MiB; 32-node trees of 16 requests do not fit).
 *   - Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two threads) race.
 *     Calls on one stream, or otherwise ordered, are safe; nothing of a previous call's contents is relied upon.
 */
int aurora_verify_attn_static(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                              const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents, void* out,
                              void* hip_stream);

/*
 * LM head + softmax + acceptance (sections 2.1, 3.1, 3.3; appendix A.1).
 *
 *   logits[m, v] = sum_h hidden[m, h] * lm_head[v, h]          (fp32 results, kept in workspace)
 *   T > 0 : p_n(v) = softmax_v(logits[b, n, :] / T).  Walk from the root: the children c of the
 *           current node, in ascending node index, are tested with
 *                 uniforms[b, c, 0] * q_cur(tok_c) < p(tok_c)        (q_cur = draft_probs[b, cur, :])
 *           an accepted child becomes the current node (p = p_c); after a rejected child
 *           p <- max(0, p - q_cur) renormalised (left unchanged if that is identically 0).
 *           When no child is left, next_token is drawn from p by inverse CDF in ascending
 *           token order with uniforms[b, cur, 1]: the first v whose running sum exceeds u * sum.
 *           A chain is the one-child case: the first rejection ends the walk.
 *   T == 0: a child is accepted iff its token equals the arg-max (lowest index on ties) of the
 *           current row; next_token is the arg-max of the row the walk stops at.
 *
 * Tree walks at T > 0 over large vocabularies are split over several workgroups per request that wait for each
 * other between vocabulary sweeps.  They fit the device together when nothing else occupies it; the wait is
 * bounded all the same: when the workgroups of a request do not meet in time (a GPU shared with other work), one
 * of them finishes the request alone inside the same call, with the same result bit for bit, only later.  The
 * outputs are therefore always complete and valid once the stream is synchronised.  Chains and greedy calls
 * never wait.
 */
int aurora_verify_accept(const aurora_accept_desc* desc,
                         const void* hidden,          /* [B, Nq, H]                           */
                         const void* lm_head,         /* [V, H] row-major                     */
                         const int32_t* draft_tokens, /* [B, Nq]; entry 0 (root) ignored      */
                         const float* draft_probs,    /* [B, Nq, V] fp32 (or [B, Nq, Vd], see desc), row n =
                                                         distribution of n's children; NULL allowed iff T == 0 */
                         const float* uniforms,       /* [B, Nq, 2] in [0,1); NULL allowed iff T == 0 */
                         const int32_t* parents,      /* [B, Nq] or NULL => chain             */
                         int32_t* accept_len,         /* [B] accepted draft tokens = depth of the stop node */
                         int32_t* next_token,         /* [B] corrected token, or bonus token if all accepted */
                         uint8_t* accept_mask,        /* [B, Nq] 1 on the accepted path (root always 1) */
                         float* p_at_draft,           /* [B, Nq] optional (NULL ok): p_parent(n)(tok_n) of the
                                                         unmodified target distribution; root 0; T == 0: 1/0 */
                         float* row_lse,              /* [B, Nq] optional: logsumexp(logits / T); T == 0: T = 1 */
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * First stage of aurora_verify_accept on its own: the LM-head projection (appendix A.1, eq. 4:
 * logits l in R^{T x V}) fused with the per-vocab-tile softmax statistics.  Leaves the fp32
 * logits [B*Nq, V] and the statistics in `workspace` (sized as for aurora_verify_accept); the
 * logits are found with aurora_verify_logits_ptr(NULL, desc, workspace).  Used to time and to
 * inspect the vocabulary sweep separately from the acceptance walk.
 */
int aurora_verify_lmhead(const aurora_accept_desc* desc,
                         const void* hidden,  /* [B, Nq, H]       */
                         const void* lm_head, /* [V, H] row-major */
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Second stage of aurora_verify_accept on its own: the acceptance walk and the residual / bonus draw
 * (section 2.1's rule, as specified at aurora_verify_accept) on the logits and statistics that a
 * preceding aurora_verify_lmhead call with the same descriptor left in `workspace`.
 * aurora_verify_lmhead followed by this call enqueues exactly the kernels of aurora_verify_accept;
 * the split exists so that a caller can put its own events (or other work) between the two stages.
 */
int aurora_verify_accept_logits(const aurora_accept_desc* desc, const int32_t* draft_tokens,
                                const float* draft_probs, const float* uniforms, const int32_t* parents,
                                int32_t* accept_len, int32_t* next_token, uint8_t* accept_mask,
                                float* p_at_draft, float* row_lse,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/* Both halves on the same stream: attention, then acceptance.  The halves share no data
 * (the hidden states entering the LM head are an independent input). */
int aurora_verify(const aurora_attn_desc* attn_desc, const aurora_accept_desc* accept_desc,
                  const void* q, const void* k_pages, const void* v_pages,
                  const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents,
                  void* attn_out,
                  const void* hidden, const void* lm_head, const int32_t* draft_tokens,
                  const float* draft_probs, const float* uniforms,
                  int32_t* accept_len, int32_t* next_token, uint8_t* accept_mask,
                  float* p_at_draft, float* row_lse,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* After aurora_verify_accept / aurora_verify has been enqueued with `workspace`, the fp32
 * logits [B*Nq, V] it computed live at this device address until the workspace is reused
 * (the target-logit payload of appendix A.1).  Host only; returns NULL on invalid descriptors. */
const float* aurora_verify_logits_ptr(const aurora_attn_desc* attn_desc, const aurora_accept_desc* accept_desc,
                                      const void* workspace);

/* After aurora_verify_accept / aurora_verify_lmhead / aurora_verify has been enqueued with `workspace`: the largest
 * logit of every 32 consecutive vocabulary ids of every token row, float32 [B*Nq, *n_groups] (group g = ids 32 g ..
 * 32 g + 31; -inf for groups past the vocabulary), valid like the logits above - what aurora_trace_desc.group_max
 * takes.  Host only.  Returns NULL and *n_groups = 0 for
 * configurations whose LM head runs outside the matrix-core kernels (float32 operands, hidden sizes they do not
 * take), which write none. */
const float* aurora_verify_group_max_ptr(const aurora_attn_desc* attn_desc, const aurora_accept_desc* accept_desc,
                                         const void* workspace, int32_t* n_groups);

/*
 * Debug check of the device-resident inputs of a verify step.  The calls above validate descriptors and
 * pointers on the host only; what the device arrays hold is trusted, and a page id, length, parent or
 * token id out of range would make a kernel read or write outside its buffers.  This call (for callers
 * who want to find such an input first; it is not part of the verify step and costs two small launches)
 * reads the arrays - never outside the shapes the descriptors declare - and writes, asynchronously on
 * `hip_stream`, to flags (DEVICE pointer, int32 [6]):
 *   flags[0]  OR of AURORA_CHECK_* bits, 0 if everything is in range
 *   flags[1 + i], i = 0..4: the lowest request index with an error of kind (1 << i), or INT32_MAX
 * Checked, each only if its array is given (NULL arrays are skipped; attn / accept may each be NULL when
 * none of its arrays is given):
 *   AURORA_CHECK_SEQ_LEN   seq_lens[b] >= num_q and ceil(seq_lens[b] / page_size) <= max_pages_per_seq
 *   AURORA_CHECK_PAGE_ID   block_table[b, i] in [0, num_pages) for the pages seq_lens[b] uses
 *                          (skipped for a request whose length failed)
 *   AURORA_CHECK_PARENT    parents[b, 0] == -1 and 0 <= parents[b, n] < n
 *   AURORA_CHECK_TOKEN     draft_tokens[b, n] in [0, vocab) for n >= 1
 *   AURORA_CHECK_UNIFORM   uniforms in [0, 1) (NaN fails)
 * Returns AURORA_ERR_INVALID_ARG for a NULL flags pointer, an array without the descriptor that gives its
 * shape, or descriptors that disagree on batch / num_q.
 */
enum {
  AURORA_CHECK_SEQ_LEN = 1, AURORA_CHECK_PAGE_ID = 2, AURORA_CHECK_PARENT = 4, AURORA_CHECK_TOKEN = 8,
  AURORA_CHECK_UNIFORM = 16
};
int aurora_verify_check_inputs(const aurora_attn_desc* attn_desc, const aurora_accept_desc* accept_desc,
                               const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents,
                               const int32_t* draft_tokens, const float* uniforms, int32_t* flags,
                               void* hip_stream);

/*
 * Trace emission: what the inference server hands to the training side after a verify step
 * (paper section 3.1: outcomes of accepted and rejected tokens are both streamed; appendix A.1,
 * eq. 4: a record is (h, l, x_in, y_out, R); appendix A.2: only the K largest target logits of a
 * token are kept, K = 1024, 2 bytes each instead of the whole vocabulary row).  h (the hidden rows)
 * and x_in (the draft tokens) are the caller's own buffers and are not copied; this call produces
 * the filtered logits, y_out and R.
 *
 *   top-K half (skipped when topk_ids and topk_logits are both NULL; one NULL alone is an error):
 *     for every token row m of `logits`, topk_ids[m, 0..K) are the ids of its K largest entries,
 *     ordered by value descending, equal values (-0.0 and +0.0 are equal) by ascending id;
 *     topk_logits[m, j] is the value rounded to bfloat16 (nearest, ties to even), stored as its
 *     16-bit pattern.  If V < K the tail holds id -1 / value -inf (0xFF80).  -inf entries are
 *     ordinary smallest values; NaN entries are not allowed (order unspecified).  The result is
 *     unique, so it is bit-reproducible.
 *   record half (skipped when y_out and traj are both NULL; one NULL alone is an error):
 *     y_out[b, n] = token emitted after node n: the token of n's accepted child, next_token[b] for
 *     the last node of the accepted path, -1 for nodes off the path.
 *     traj[b, n] (R) = 1 for nodes on the accepted path (root included); 2 for drafts that were
 *     tested and rejected - the acceptance step tries the children of a path node in index order
 *     until one is kept, so these are the children before the kept one, or all of them if none is
 *     kept; 0 for nodes that were never tested.
 *
 * No workspace.  Returns AURORA_ERR_INVALID_ARG for null / inconsistent pointers or a `logits`
 * pointer that is not 4-byte aligned, AURORA_ERR_UNSUPPORTED for top_k > 1024 or num_q > 64.
 */
typedef struct {
  int32_t batch; /* B >= 0 (0: nothing is enqueued)   */
  int32_t num_q; /* Nq, 1..64                         */
  int32_t vocab; /* V >= 1                            */
  int32_t top_k; /* K, 1..1024 (the paper uses 1024)  */
  /* Logits over the draft vocabulary only (appendix A.2: the draft model's vocabulary is 4-5 x smaller,
   * so only those logits are transmitted).  draft_vocab = 0: select over all V entries.  draft_vocab =
   * Vd in 1..V: select over logits[m, draft_to_target[j]], j < Vd (DEVICE pointer, [Vd] int32 target
   * ids, distinct); topk_ids then hold draft indices j, ties by ascending j, padding when Vd < K. */
  int32_t draft_vocab;
  const int32_t* draft_to_target;
  /* Optional, from the vocabulary sweep of the verify step (appendix A.2 reduces 256 KB of logits per token to
   * 2 KB; with this the reduction reads only the 128-byte groups that can hold a kept logit, about a quarter of the
   * row, instead of sampling and then streaming all of it).  n_groups = 0: not given.  Otherwise group_max is a
   * DEVICE pointer to float32 [B*Nq, n_groups] and entry (m, g) MUST be the largest of logits[m, 32 g .. 32 g + 31]
   * (ids below V) for every g < ceil(V / 32); further entries of a row are ignored.  aurora_verify_group_max_ptr()
   * hands out what the LM head wrote.  Used when K <= ceil(V / 32) <= 8192, V > 4096 and draft_vocab = 0, ignored
   * otherwise.  An entry larger than the true maximum only costs time; a smaller one may hide that group's logits
   * from the selection. */
  int32_t n_groups;
  const float* group_max;
} aurora_trace_desc;

int aurora_trace_emit(const aurora_trace_desc* desc,
                      const float* logits,         /* [B*Nq, V] fp32 target logits, e.g. aurora_verify_logits_ptr() */
                      const int32_t* draft_tokens, /* [B, Nq]; entry 0 (root) ignored          */
                      const int32_t* parents,      /* [B, Nq] or NULL => chain                 */
                      const int32_t* next_token,   /* [B]     from the acceptance step         */
                      const uint8_t* accept_mask,  /* [B, Nq] from the acceptance step         */
                      int32_t* topk_ids,           /* [B*Nq, K]                                */
                      uint16_t* topk_logits,       /* [B*Nq, K] bfloat16 bit patterns          */
                      int32_t* y_out,              /* [B, Nq]                                  */
                      int8_t* traj,                /* [B, Nq]                                  */
                      void* hip_stream);

/* For tests of the bounded wait described at aurora_verify_accept: the number of polls of the arrival counter a
 * workgroup of a split tree walk makes before it stops waiting (process-wide, applies to later calls; negative
 * restores the default of 2^15, some tens of milliseconds).  0 makes every wait fail at once unless the others have
 * already arrived, which forces the finish-alone path; results do not depend on the setting. */
void aurora_debug_set_tree_spin_limit(int polls);

/*
 * Calibration probe for the roofline of the LM head (appendix A.1's projection is a dense contraction): the inner
 * structure of the many-row LM-head kernel with its parts switched on one at a time, on operands the caller provides,
 * so that a benchmark can say what a bf16 contraction reaches on the device at hand - and how much that depends on
 * the values multiplied.  mode 0: matrix cores only (operands in registers); 1: + operand reads from LDS; 2: + the
 * LDS-direct loads that refill a stage, issued as that kernel issues them (L2 resident, no HBM traffic); 3: those loads alone; 4: the vocabulary
 * sweep alone - all of `operands` (whole multiples of 2 MiB; e.g. the LM head itself) streamed once from HBM through a
 * three-stage LDS ring in the LM head's tile shape, one workgroup per 256 rows of 8 KB, `workgroups` and `stages`
 * ignored.  `operands`:
 * DEVICE memory, 16-byte aligned, at least 16 MiB (operand_bytes says how much there is), read as bf16 - fill it with
 * values like the workload's, or zeros.  `workgroups` x `stages` is the amount of work (a stage is 256 x 256 x 64
 * multiply-adds per workgroup and 64 KB loaded); results are discarded; `sink` is one DEVICE float that is never
 * written in practice.  Asynchronous on hip_stream; the caller times it.  Not part of the verify step.
 */
int aurora_probe_contraction(int mode, const void* operands, size_t operand_bytes, int workgroups, int stages,
                             float* sink, void* hip_stream);

/* Human-readable name of a status code; never NULL. */
const char* aurora_status_string(int status);

/*
 * Backward pass of the chunk / tree attention above (section 3.1, "Efficient Tree Attention": the training side
 * puts the whole speculative tree - accepted and rejected branches - through one batched forward and backward
 * pass under the tree's mask).  With out = aurora_verify_attn(q, K, V) and dout = dLoss / dout:
 *
 *   p_ij = softmax_j(sm_scale <q_i, k_j>) over the positions row i sees,  delta_i = <dout_i, out_i>
 *   dS_ij = p_ij (<dout_i, v_j> - delta_i)
 *   dq_i = sm_scale sum_j dS_ij k_j      dk_j = sm_scale sum_i dS_ij q_i      dv_j = sum_i p_ij dout_i
 *
 * (dk_j, dv_j sum over every node and every query head of the KV head's group that sees position j: the cached
 * prefix receives gradient as well).  dq is float32 [B, Nq, Hq, D]; dk_pages / dv_pages are float32 pools in the
 * layout of k_pages / v_pages - the positions the batch's block tables address are written, every other element
 * is left as it is.  A page must belong to ONE request of the batch: dk / dv of a position are written, not
 * accumulated, per block-table entry, so a page that two requests share (a common prefix) would keep the gradient
 * of whichever wrote last - give such requests their own copies, or add the per-request results outside.
 * dout has the type of q.  All sums run in a fixed order: bit-reproducible.
 * bf16 caches with head_dim 128, power-of-two pages >= 16 and at most 128 query rows per KV head run on the
 * matrix cores (P and dS rounded to bf16 for the products, fp32 accumulation); every other
 * shape takes a plain fp32 vector kernel.  An 8-bit KV cache is not supported (AURORA_ERR_UNSUPPORTED).
 *
 *   aurora_attn_backward        runs the forward pass itself (into the workspace): nothing is kept from a forward call
 *   aurora_attn_forward         aurora_verify_attn that also writes lse [B, Nq, Hq] float32, the natural logarithm of
 *                               each row's softmax denominator sum_j exp(sm_scale <q_i, k_j>) - what a training
 *                               step keeps for the backward pass.  Workspace as for aurora_verify_attn
 *                               (aurora_verify_workspace_bytes(desc, NULL)); 8-bit KV caches are accepted.
 *   aurora_attn_backward_saved  the backward pass on `out` (type of q) and `lse` saved from aurora_attn_forward
 *                               with the same inputs; results are bit-identical to aurora_attn_backward.
 * Workspace of both backward calls: aurora_attn_backward_workspace_bytes().
 */
int aurora_attn_backward_workspace_bytes(const aurora_attn_desc* desc, size_t* out_bytes);
int aurora_attn_backward(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                         const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents,
                         const void* dout, float* dq, float* dk_pages, float* dv_pages,
                         void* workspace, size_t workspace_bytes, void* hip_stream);
int aurora_attn_forward(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                        const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents, void* out,
                        float* lse, void* workspace, size_t workspace_bytes, void* hip_stream);
int aurora_attn_backward_saved(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                               const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents,
                               const void* out, const float* lse, const void* dout, float* dq, float* dk_pages,
                               float* dv_pages, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Packing of the trace records that are shipped to the training side (appendix A.1, eq. 4: a record is
 * (h, l, x_in, y_out, R); section 3.3: accepted and rejected tokens both carry a training signal).  Of the
 * `rows` token rows of a verify step (or of several) only those with traj[m] != 0 - on the accepted path, or
 * tested and rejected - are kept; rows that were never tested are dropped.  Kept rows are copied in ascending
 * row order into dense arrays:
 *   n_out     [1]       number of kept rows n
 *   row_index [rows]    row_index[p], p < n: the source row of packed position p (entries from n on are not written)
 *   for every input that is given (a NULL input skips its output; topk_ids / topk_logits come as a pair), its
 *   packed copy, position p holding source row row_index[p]:
 *     h            [rows, h_row_bytes] bytes  -> h_out          the hidden row(s) of the token, any element type
 *     topk_ids     [rows, K] int32            -> topk_ids_out
 *     topk_logits  [rows, K] bf16 bits        -> topk_logits_out
 *     x_in, y_out  [rows] int32               -> x_in_out, y_out_out
 *     traj         [rows] int8                -> traj_out (may be NULL)
 * Output arrays are sized for `rows` rows by the caller.  All pointers are DEVICE pointers; asynchronous on
 * hip_stream; no workspace; the result is unique, hence bit-reproducible.  AURORA_ERR_INVALID_ARG for missing
 * traj / n_out / row_index, an input without its output (or the reverse), or negative sizes.
 */
typedef struct {
  int32_t rows;        /* M >= 0                                              */
  int32_t top_k;       /* K >= 0 entries per row of topk_ids / topk_logits    */
  int64_t h_row_bytes; /* bytes of one row of h (0 if h is not packed)        */
} aurora_pack_desc;

int aurora_trace_pack(const aurora_pack_desc* desc, const int8_t* traj, const void* h, const int32_t* topk_ids,
                      const uint16_t* topk_logits, const int32_t* x_in, const int32_t* y_out,
                      int32_t* n_out, int32_t* row_index, void* h_out, int32_t* topk_ids_out,
                      uint16_t* topk_logits_out, int32_t* x_in_out, int32_t* y_out_out, int8_t* traj_out,
                      void* hip_stream);

/*
 * Drafter training loss on a batch of trace rows (paper section 3.3, eq. 3) - the first thing the training
 * side computes from what aurora_trace_emit produced:
 *
 *   L = mean over accepted rows of KL(p_target || p_draft)
 *       + lambda_discard * mean over discarded rows of KL(p_target || p_draft)
 *
 * Row m is one token position; traj[m] (the record's R) is its class: 1 accepted, 2 discarded (tested and
 * rejected), anything else unused.  The means are over the rows of the class in this batch (an empty class
 * contributes 0).  p_target of a row is the softmax over the kept target logits topk_logits[m, 0..K) (bf16
 * bit patterns) on the tokens topk_ids[m, 0..K) - indices into the drafter's vocabulary, distinct, ordered
 * by value with the largest first, as aurora_trace_emit writes them with a draft_to_target map - and zero
 * elsewhere; entries with id -1 or value -inf carry no mass.  On discarded rows only the first
 * discard_top_k entries are used (the paper's top-k filtering of discarded tokens; 0 = all K).  p_draft is
 * the softmax of draft_logits[m, 0..Vd).  A row without any kept target logit has KL 0 and no gradient.
 * Outputs (all DEVICE pointers):
 *   row_kl   [rows] float32   KL of every row (also of unused rows)
 *   loss_out [5]    float32   L, the accepted-rows mean, the discarded-rows mean, N_accept, N_discard
 *   grad     [rows, Vd] float32 or NULL: dL / d draft_logits = w_m (p_draft - p_target),
 *            w_m = 1 / N_accept, lambda_discard / N_discard or 0 by class
 * Arithmetic: exponentials in fp32, every sum in fp64 in a fixed order (bit-reproducible).  No workspace;
 * asynchronous on hip_stream.  AURORA_ERR_INVALID_ARG for null pointers, non-positive sizes, negative or
 * non-finite lambda; AURORA_ERR_UNSUPPORTED for top_k > 1024.
 */
typedef struct {
  int32_t rows;          /* M >= 0 (0: only loss_out is written, with zeros)  */
  int32_t draft_vocab;   /* Vd >= 1                                            */
  int32_t top_k;         /* K, 1..1024: entries per row of topk_ids / topk_logits */
  int32_t discard_top_k; /* 0 => K, else 1..K                                  */
  float lambda_discard;  /* >= 0                                               */
} aurora_loss_desc;

int aurora_draft_loss(const aurora_loss_desc* desc, const float* draft_logits, const int32_t* topk_ids,
                      const uint16_t* topk_logits, const int8_t* traj, float* row_kl, float* loss_out, float* grad,
                      void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* AURORA_VERIFY_H */
