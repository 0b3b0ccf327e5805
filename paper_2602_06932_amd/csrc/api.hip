// C-ABI layer: host-side validation, workspace planning and kernel dispatch.
#include "../../include/aurora_verify.h"
#include "common.hpp"
#include "launch.hpp"

#include <mutex>

using namespace aurora;

namespace {

int check_attn_desc(const aurora_attn_desc* d) {
  if (!d) return AURORA_ERR_INVALID_ARG;
  if (d->batch < 0 || d->num_q < 1 || d->num_q_heads < 1 || d->num_kv_heads < 1 || d->head_dim < 1 ||
      d->page_size < 1 || d->max_pages_per_seq < 1 || d->num_pages < 1)
    return AURORA_ERR_INVALID_ARG;
  if (d->num_q_heads % d->num_kv_heads) return AURORA_ERR_INVALID_ARG;
  if (d->dtype != AURORA_F32 && d->dtype != AURORA_BF16) return AURORA_ERR_INVALID_ARG;
  if (!(d->sm_scale >= 0.f)) return AURORA_ERR_INVALID_ARG;
  if (d->kv_fp8 != 0 && d->kv_fp8 != 1) return AURORA_ERR_INVALID_ARG;
  if (d->kv_fp8 && (!d->k_scale || !d->v_scale)) return AURORA_ERR_INVALID_ARG;
  if (d->num_q > kMaxNq) return AURORA_ERR_UNSUPPORTED;
  if (d->head_dim != 64 && d->head_dim != 128) return AURORA_ERR_UNSUPPORTED;
  if ((int64_t)d->batch * d->num_q > 65535 || d->num_q_heads > 65535) return AURORA_ERR_UNSUPPORTED;
  if ((int64_t)d->max_pages_per_seq * d->page_size > (int64_t)1 << 30) return AURORA_ERR_UNSUPPORTED;
  return AURORA_OK;
}

int check_accept_desc(const aurora_accept_desc* d) {
  if (!d) return AURORA_ERR_INVALID_ARG;
  if (d->batch < 0 || d->num_q < 1 || d->hidden < 1 || d->vocab < 1) return AURORA_ERR_INVALID_ARG;
  if (d->dtype != AURORA_F32 && d->dtype != AURORA_BF16 && d->dtype != AURORA_FP8_E4M3) return AURORA_ERR_INVALID_ARG;
  if (!(d->temperature >= 0.f)) return AURORA_ERR_INVALID_ARG;
  if (d->num_q > kMaxNq) return AURORA_ERR_UNSUPPORTED;
  if ((int64_t)d->batch * d->num_q > 65535) return AURORA_ERR_UNSUPPORTED;
  if (d->dtype == AURORA_BF16 && d->hidden % 8) return AURORA_ERR_UNSUPPORTED;
  if (d->dtype == AURORA_FP8_E4M3) {
    if (!d->hidden_scale || !d->lm_head_scale) return AURORA_ERR_INVALID_ARG;
    if (d->hidden % 128) return AURORA_ERR_UNSUPPORTED;  // only the matrix-core kernel takes 8-bit operands
  }
  if (d->draft_vocab < 0 || d->draft_vocab > d->vocab) return AURORA_ERR_INVALID_ARG;
  if (d->draft_vocab > 0 && (d->temperature > 0.f || d->temperatures) && !d->target_to_draft) return AURORA_ERR_INVALID_ARG;
  return AURORA_OK;
}

AttnLaunch attn_launch_from(const aurora_attn_desc* d) {
  AttnLaunch a = {};
  a.B = d->batch; a.Nq = d->num_q; a.Hq = d->num_q_heads; a.Hkv = d->num_kv_heads; a.D = d->head_dim;
  a.page = d->page_size; a.max_pages = d->max_pages_per_seq; a.bf16 = d->dtype == AURORA_BF16;
  a.scale = d->sm_scale > 0.f ? d->sm_scale : 1.0f / sqrtf((float)d->head_dim);
  a.kv_fp8 = d->kv_fp8 != 0; a.k_scale = d->k_scale; a.v_scale = d->v_scale;
  return a;
}

// KV tokens per split: large enough that a split amortises its prologue, small enough that the
// longest request is cut into many workgroups; the number of splits is bounded so that the
// partial buffers stay modest.
AttnPlan plan_attn(const aurora_attn_desc* d) {
  AttnPlan p = {};
  p.rows_per_group = d->num_q_heads / d->num_kv_heads * d->num_q;
  AttnLaunch probe = attn_launch_from(d);
  p.mfma = attn_mfma_supported(probe);
  p.pb_off = 0;
  const size_t pb_bytes = align_up(((size_t)d->batch + 1) * sizeof(int32_t));
  p.part_o_off = pb_bytes;
  if (p.mfma) {
    p.row_tiles = (p.rows_per_group + 31) / 32;
    // the wide-row kernel (more than one row tile) writes two partials per segment
    p.slots = (kAttnWorkgroups + d->batch * d->num_kv_heads) * (p.row_tiles > 1 ? 2 : 1);
    const size_t nrows = (size_t)p.slots * p.row_tiles * 32;
    p.part_ml_off = p.part_o_off + align_up(nrows * d->head_dim * sizeof(float));
    p.bytes = p.part_ml_off + align_up(nrows * 2 * sizeof(float));
  } else {
    const int64_t max_len = (int64_t)d->max_pages_per_seq * d->page_size;
    int split = 512;
    while ((max_len + split - 1) / split > 64 && split < 4096) split *= 2;
    p.split_len = split;
    int64_t ms = (max_len + split - 1) / split;
    p.max_splits = (int)(ms < 1 ? 1 : ms);
    const size_t nrows = (size_t)d->batch * d->num_q * d->num_q_heads * p.max_splits;
    p.part_ml_off = p.part_o_off + align_up(nrows * d->head_dim * sizeof(float));
    p.bytes = p.part_ml_off + align_up(nrows * 2 * sizeof(float));
  }
  return p;
}

AcceptLaunch accept_launch_from(const aurora_accept_desc* d) {
  AcceptLaunch a = {};
  a.B = d->batch; a.Nq = d->num_q; a.H = d->hidden; a.V = d->vocab; a.bf16 = d->dtype == AURORA_BF16;
  a.fp8 = d->dtype == AURORA_FP8_E4M3;
  a.hidden_scale = d->hidden_scale; a.lm_scale = d->lm_head_scale;
  a.temperature = d->temperature;
  a.temps = d->temperatures;
  a.wor = d->tree_without_replacement;
  if (d->draft_vocab > 0 && (d->temperature > 0.f || d->temperatures)) { a.Vd = d->draft_vocab; a.target_to_draft = d->target_to_draft; }
  return a;
}

AcceptPlan plan_accept(const aurora_accept_desc* d) {
  AcceptPlan p = {};
  p.rows = (int64_t)d->batch * d->num_q;
  AcceptLaunch probe = accept_launch_from(d);
  p.stat_tile = lmhead_mfma_supported(probe) ? lmhead_mfma_stat_tile() : 1024;
  p.n_tiles = (d->vocab + p.stat_tile - 1) / p.stat_tile;
  const size_t rows = (size_t)p.rows;
  p.logits_off = 0;
  p.pmax_off = align_up(rows * d->vocab * sizeof(float));
  p.psum_off = p.pmax_off + align_up(rows * p.n_tiles * sizeof(float));
  p.parg_off = p.psum_off + align_up(rows * p.n_tiles * sizeof(float));
  accept_chain_geometry(d->batch, d->vocab, &p.slices, &p.gmul, &p.ngroups);
  const size_t B = (size_t)d->batch;
  // maxima of groups of 32 vocabulary entries, written by the matrix-core LM-head kernels for the top-K emission
  p.n_half = lmhead_mfma_supported(probe) ? p.n_tiles * kLmHalfPerTile : 0;
  p.hmax_off = p.parg_off + align_up(rows * p.n_tiles * sizeof(int32_t));
  p.st_lse_off = p.hmax_off + align_up(rows * p.n_half * sizeof(float));
  p.st_row_off = p.st_lse_off + align_up(B * sizeof(double));
  p.st_rej_off = p.st_row_off + align_up(B * sizeof(int32_t));
  p.gsum_off = p.st_rej_off + align_up(B * sizeof(int32_t));
  // the tree walk keeps two copies of the group sums and of the per-slice last positions (alternating by sweep)
  p.lastpos_off = p.gsum_off + align_up(2 * B * p.ngroups * sizeof(double));
  const size_t lp_slices = (size_t)std::max(p.slices, 2 * accept_tree_max_slices());
  p.tree_bar_off = p.lastpos_off + align_up(B * lp_slices * sizeof(int32_t));
  p.bytes = p.tree_bar_off + align_up(B * sizeof(int32_t));
  return p;
}

bool misaligned(const void* p) { return ((uintptr_t)p & 255u) != 0; }

int run_attn(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
             const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents, void* out,
             void* workspace, size_t workspace_bytes, hipStream_t st, float* lse_out = nullptr) {
  int rc = check_attn_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (desc->batch == 0) return AURORA_OK;
  if (!q || !k_pages || !v_pages || !block_table || !seq_lens || !out) return AURORA_ERR_INVALID_ARG;
  if (((uintptr_t)q | (uintptr_t)k_pages | (uintptr_t)v_pages | (uintptr_t)out) & 15) return AURORA_ERR_INVALID_ARG;
  AttnPlan plan = plan_attn(desc);
  if (!workspace || misaligned(workspace) || workspace_bytes < plan.bytes) return AURORA_ERR_WORKSPACE;
  AttnLaunch a = attn_launch_from(desc);
  a.q = q; a.k = k_pages; a.v = v_pages; a.block_table = block_table; a.seq_lens = seq_lens; a.parents = parents;
  a.out = out;
  a.lse_out = lse_out;
  a.plan_pb = (int32_t*)((char*)workspace + plan.pb_off);
  a.part_o = (float*)((char*)workspace + plan.part_o_off);
  a.part_ml = (float*)((char*)workspace + plan.part_ml_off);
  a.plan = plan;
  hipError_t e = plan.mfma ? launch_attn_mfma(a, st) : launch_attn_generic(a, st);
  return e == hipSuccess ? AURORA_OK : AURORA_ERR_HIP;
}

int run_accept(const aurora_accept_desc* desc, const void* hidden, const void* lm_head, const int32_t* draft_tokens,
               const float* draft_probs, const float* uniforms, const int32_t* parents, int32_t* accept_len,
               int32_t* next_token, uint8_t* accept_mask, float* p_at_draft, float* row_lse, void* workspace,
               size_t workspace_bytes, hipStream_t st, bool with_lmhead = true) {
  int rc = check_accept_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (desc->batch == 0) return AURORA_OK;
  if (!draft_tokens || !accept_len || !next_token || !accept_mask) return AURORA_ERR_INVALID_ARG;
  if (with_lmhead && (!hidden || !lm_head)) return AURORA_ERR_INVALID_ARG;
  if ((desc->temperature > 0.f || desc->temperatures) && (!draft_probs || !uniforms)) return AURORA_ERR_INVALID_ARG;
  if (with_lmhead && (((uintptr_t)hidden | (uintptr_t)lm_head) & 15)) return AURORA_ERR_INVALID_ARG;
  // the one-workgroup tree walk keeps one partial sum per 256 tokens in LDS
  if ((desc->temperature > 0.f || desc->temperatures) && parents && desc->vocab > (1 << 20)) return AURORA_ERR_UNSUPPORTED;
  AcceptPlan plan = plan_accept(desc);
  if (!workspace || misaligned(workspace) || workspace_bytes < plan.bytes) return AURORA_ERR_WORKSPACE;
  AcceptLaunch a = accept_launch_from(desc);
  a.hidden = hidden; a.lm_head = lm_head; a.draft_tokens = draft_tokens; a.draft_probs = draft_probs;
  a.uniforms = uniforms; a.parents = parents; a.accept_len = accept_len; a.next_token = next_token;
  a.accept_mask = accept_mask; a.p_at_draft = p_at_draft; a.row_lse = row_lse;
  char* ws = (char*)workspace;
  a.logits = (float*)(ws + plan.logits_off);
  a.pmax = (float*)(ws + plan.pmax_off);
  a.psum = (float*)(ws + plan.psum_off);
  a.parg = (int32_t*)(ws + plan.parg_off);
  a.hmax = (float*)(ws + plan.hmax_off);
  a.st_lse = (double*)(ws + plan.st_lse_off);
  a.st_row = (int32_t*)(ws + plan.st_row_off);
  a.st_rej = (int32_t*)(ws + plan.st_rej_off);
  a.gsum = (double*)(ws + plan.gsum_off);
  a.lastpos = (int32_t*)(ws + plan.lastpos_off);
  a.tree_bar = (int32_t*)(ws + plan.tree_bar_off);
  a.plan = plan;
  if (with_lmhead) {
    hipError_t e = lmhead_mfma_supported(a) ? launch_lmhead_mfma(a, st) : launch_lmhead_generic(a, st);
    if (e != hipSuccess) return AURORA_ERR_HIP;
  }
  return launch_accept(a, st) == hipSuccess ? AURORA_OK : AURORA_ERR_HIP;
}

int run_lmhead(const aurora_accept_desc* desc, const void* hidden, const void* lm_head, void* workspace,
               size_t workspace_bytes, hipStream_t st) {
  int rc = check_accept_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (desc->batch == 0) return AURORA_OK;
  if (!hidden || !lm_head) return AURORA_ERR_INVALID_ARG;
  if (((uintptr_t)hidden | (uintptr_t)lm_head) & 15) return AURORA_ERR_INVALID_ARG;
  AcceptPlan plan = plan_accept(desc);
  if (!workspace || misaligned(workspace) || workspace_bytes < plan.bytes) return AURORA_ERR_WORKSPACE;
  AcceptLaunch a = accept_launch_from(desc);
  a.hidden = hidden; a.lm_head = lm_head;
  char* ws = (char*)workspace;
  a.logits = (float*)(ws + plan.logits_off);
  a.pmax = (float*)(ws + plan.pmax_off);
  a.psum = (float*)(ws + plan.psum_off);
  a.parg = (int32_t*)(ws + plan.parg_off);
  a.hmax = (float*)(ws + plan.hmax_off);
  a.plan = plan;
  hipError_t e = lmhead_mfma_supported(a) ? launch_lmhead_mfma(a, st) : launch_lmhead_generic(a, st);
  return e == hipSuccess ? AURORA_OK : AURORA_ERR_HIP;
}

// ---- the allocation-free attention entry point's scratch -------------------------------------------------
// One array per GPU the library is loaded on, held until the process ends.  In host code the name `scratch` is
// only a handle for the symbol: the device address is looked up once per device and kept in g_scratch_ptr.
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[AURORA_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up on the first call per device).
hipError_t static_scratch(void** out) {
  int dev = -1;
  if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

bool have_device() {
  static int cached = -1;  // the answer does not change during a process's life
  if (cached < 0) {
    int n = 0;
    cached = (hipGetDeviceCount(&n) == hipSuccess && n > 0) ? 1 : 0;
  }
  return cached == 1;
}

}  // namespace

extern "C" {

int aurora_verify_workspace_bytes(const aurora_attn_desc* attn, const aurora_accept_desc* accept, size_t* out_bytes) {
  if (!out_bytes || (!attn && !accept)) return AURORA_ERR_INVALID_ARG;
  size_t total = 0;
  if (attn) {
    int rc = check_attn_desc(attn);
    if (rc != AURORA_OK) return rc;
    total += plan_attn(attn).bytes;
  }
  if (accept) {
    int rc = check_accept_desc(accept);
    if (rc != AURORA_OK) return rc;
    total += plan_accept(accept).bytes;
  }
  *out_bytes = total < 256 ? 256 : total;
  return AURORA_OK;
}

int aurora_verify_attn(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                       const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents, void* out,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_attn_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (!have_device()) return AURORA_ERR_HIP;
  return run_attn(desc, q, k_pages, v_pages, block_table, seq_lens, parents, out, workspace, workspace_bytes,
                  (hipStream_t)hip_stream);
}

int aurora_verify_attn_static(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                              const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents, void* out,
                              void* hip_stream) {
  int rc = check_attn_desc(desc);
  if (rc != AURORA_OK) return rc;
  const size_t need = plan_attn(desc).bytes;
  if (need > (size_t)AURORA_STATIC_SCRATCH_BYTES) return AURORA_ERR_TOO_LARGE;
  if (!have_device()) return AURORA_ERR_HIP;
  void* ws = nullptr;
  if (static_scratch(&ws) != hipSuccess) return AURORA_ERR_HIP;
  // the kernels write every partial they later read, so nothing of the previous call's contents needs clearing
  return run_attn(desc, q, k_pages, v_pages, block_table, seq_lens, parents, out, ws, AURORA_STATIC_SCRATCH_BYTES,
                  (hipStream_t)hip_stream);
}

int aurora_verify_accept(const aurora_accept_desc* desc, const void* hidden, const void* lm_head,
                         const int32_t* draft_tokens, const float* draft_probs, const float* uniforms,
                         const int32_t* parents, int32_t* accept_len, int32_t* next_token, uint8_t* accept_mask,
                         float* p_at_draft, float* row_lse, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  int rc = check_accept_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (!have_device()) return AURORA_ERR_HIP;
  return run_accept(desc, hidden, lm_head, draft_tokens, draft_probs, uniforms, parents, accept_len, next_token,
                    accept_mask, p_at_draft, row_lse, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

int aurora_verify_lmhead(const aurora_accept_desc* desc, const void* hidden, const void* lm_head, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  int rc = check_accept_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (!have_device()) return AURORA_ERR_HIP;
  return run_lmhead(desc, hidden, lm_head, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

int aurora_verify_accept_logits(const aurora_accept_desc* desc, const int32_t* draft_tokens, const float* draft_probs,
                                const float* uniforms, const int32_t* parents, int32_t* accept_len,
                                int32_t* next_token, uint8_t* accept_mask, float* p_at_draft, float* row_lse,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_accept_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (!have_device()) return AURORA_ERR_HIP;
  return run_accept(desc, nullptr, nullptr, draft_tokens, draft_probs, uniforms, parents, accept_len, next_token,
                    accept_mask, p_at_draft, row_lse, workspace, workspace_bytes, (hipStream_t)hip_stream, false);
}

int aurora_verify(const aurora_attn_desc* attn_desc, const aurora_accept_desc* accept_desc, const void* q,
                  const void* k_pages, const void* v_pages, const int32_t* block_table, const int32_t* seq_lens,
                  const int32_t* parents, void* attn_out, const void* hidden, const void* lm_head,
                  const int32_t* draft_tokens, const float* draft_probs, const float* uniforms, int32_t* accept_len,
                  int32_t* next_token, uint8_t* accept_mask, float* p_at_draft, float* row_lse, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  int rc = check_attn_desc(attn_desc);
  if (rc != AURORA_OK) return rc;
  rc = check_accept_desc(accept_desc);
  if (rc != AURORA_OK) return rc;
  if (attn_desc->batch != accept_desc->batch || attn_desc->num_q != accept_desc->num_q)
    return AURORA_ERR_INVALID_ARG;
  if (!have_device()) return AURORA_ERR_HIP;
  const size_t attn_bytes = plan_attn(attn_desc).bytes;
  const size_t acc_bytes = plan_accept(accept_desc).bytes;
  if (!workspace || misaligned(workspace) || workspace_bytes < attn_bytes + acc_bytes) return AURORA_ERR_WORKSPACE;
  // validate the second half's pointers before anything is enqueued
  if (accept_desc->batch > 0) {
    if (!hidden || !lm_head || !draft_tokens || !accept_len || !next_token || !accept_mask)
      return AURORA_ERR_INVALID_ARG;
    if ((accept_desc->temperature > 0.f || accept_desc->temperatures) && (!draft_probs || !uniforms)) return AURORA_ERR_INVALID_ARG;
  }
  rc = run_attn(attn_desc, q, k_pages, v_pages, block_table, seq_lens, parents, attn_out, workspace, attn_bytes,
                (hipStream_t)hip_stream);
  if (rc != AURORA_OK) return rc;
  return run_accept(accept_desc, hidden, lm_head, draft_tokens, draft_probs, uniforms, parents, accept_len,
                    next_token, accept_mask, p_at_draft, row_lse, (char*)workspace + attn_bytes, acc_bytes,
                    (hipStream_t)hip_stream);
}

const float* aurora_verify_logits_ptr(const aurora_attn_desc* attn_desc, const aurora_accept_desc* accept_desc,
                                      const void* workspace) {
  if (!workspace || check_accept_desc(accept_desc) != AURORA_OK) return nullptr;
  size_t off = 0;
  if (attn_desc) {
    if (check_attn_desc(attn_desc) != AURORA_OK) return nullptr;
    off = plan_attn(attn_desc).bytes;
  }
  return (const float*)((const char*)workspace + off + plan_accept(accept_desc).logits_off);
}

const float* aurora_verify_group_max_ptr(const aurora_attn_desc* attn_desc, const aurora_accept_desc* accept_desc,
                                         const void* workspace, int32_t* n_groups) {
  if (n_groups) *n_groups = 0;
  if (!workspace || !n_groups || check_accept_desc(accept_desc) != AURORA_OK) return nullptr;
  size_t off = 0;
  if (attn_desc) {
    if (check_attn_desc(attn_desc) != AURORA_OK) return nullptr;
    off = plan_attn(attn_desc).bytes;
  }
  const AcceptPlan plan = plan_accept(accept_desc);
  if (plan.n_half == 0) return nullptr;
  *n_groups = plan.n_half;
  return (const float*)((const char*)workspace + off + plan.hmax_off);
}

int aurora_verify_check_inputs(const aurora_attn_desc* attn_desc, const aurora_accept_desc* accept_desc,
                               const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents,
                               const int32_t* draft_tokens, const float* uniforms, int32_t* flags,
                               void* hip_stream) {
  if (!flags || (!attn_desc && !accept_desc)) return AURORA_ERR_INVALID_ARG;
  if (attn_desc) { int rc = check_attn_desc(attn_desc); if (rc != AURORA_OK) return rc; }
  if (accept_desc) { int rc = check_accept_desc(accept_desc); if (rc != AURORA_OK) return rc; }
  if (attn_desc && accept_desc && (attn_desc->batch != accept_desc->batch || attn_desc->num_q != accept_desc->num_q))
    return AURORA_ERR_INVALID_ARG;
  if ((block_table || seq_lens) && !attn_desc) return AURORA_ERR_INVALID_ARG;
  if (block_table && !seq_lens) return AURORA_ERR_INVALID_ARG;  // which pages are in use comes from the lengths
  if ((draft_tokens || uniforms) && !accept_desc) return AURORA_ERR_INVALID_ARG;
  CheckLaunch c = {};
  c.B = attn_desc ? attn_desc->batch : accept_desc->batch;
  c.Nq = attn_desc ? attn_desc->num_q : accept_desc->num_q;
  if (attn_desc) { c.page = attn_desc->page_size; c.max_pages = attn_desc->max_pages_per_seq; c.num_pages = attn_desc->num_pages; }
  if (accept_desc) c.V = accept_desc->vocab;
  c.block_table = block_table; c.seq_lens = seq_lens; c.parents = parents; c.draft_tokens = draft_tokens;
  c.uniforms = uniforms; c.flags = flags;
  return launch_check_inputs(c, (hipStream_t)hip_stream) == hipSuccess ? AURORA_OK : AURORA_ERR_HIP;
}

namespace {
struct BwdPlan { size_t fwd_bytes, out_off, lse_off, delta_off, pb_off, part_dq_off, bytes; };
BwdPlan plan_bwd(const aurora_attn_desc* d) {
  BwdPlan p = {};
  p.fwd_bytes = plan_attn(d).bytes;
  const size_t rows = (size_t)d->batch * d->num_q * d->num_q_heads;
  const size_t esz = d->dtype == AURORA_BF16 ? 2 : 4;
  p.out_off = align_up(p.fwd_bytes);
  p.lse_off = p.out_off + align_up(rows * d->head_dim * esz);
  p.delta_off = p.lse_off + align_up(rows * sizeof(float));
  p.pb_off = p.delta_off + align_up(rows * sizeof(float));
  // matrix-core kernel: one partial dq (the pair's query rows x 128 columns) per run of tiles
  p.part_dq_off = p.pb_off + align_up(((size_t)d->batch + 1) * sizeof(int32_t));
  p.bytes = p.part_dq_off + align_up(attn_bwd_mfma_partial_bytes(d->batch, d->num_kv_heads, d->num_q_heads / d->num_kv_heads * d->num_q));
  return p;
}
}  // namespace

int aurora_attn_backward_workspace_bytes(const aurora_attn_desc* desc, size_t* out_bytes) {
  if (!out_bytes) return AURORA_ERR_INVALID_ARG;
  int rc = check_attn_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (desc->kv_fp8) return AURORA_ERR_UNSUPPORTED;
  *out_bytes = plan_bwd(desc).bytes;
  return AURORA_OK;
}

namespace {
// delta, the backward kernel and the dq merge on a forward output and logsumexp that are already there
int run_attn_bwd(const aurora_attn_desc* desc, const BwdPlan& bp, const void* q, const void* k_pages, const void* v_pages,
                 const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents, const void* out,
                 const float* lse, const void* dout, float* dq, float* dk_pages, float* dv_pages, char* ws, hipStream_t st) {
  AttnBwdLaunch a = {};
  a.B = desc->batch; a.Nq = desc->num_q; a.Hq = desc->num_q_heads; a.Hkv = desc->num_kv_heads; a.D = desc->head_dim;
  a.page = desc->page_size; a.max_pages = desc->max_pages_per_seq; a.bf16 = desc->dtype == AURORA_BF16;
  a.scale = desc->sm_scale > 0.f ? desc->sm_scale : 1.0f / sqrtf((float)desc->head_dim);
  a.q = q; a.k = k_pages; a.v = v_pages; a.out = out; a.dout = dout;
  a.block_table = block_table; a.seq_lens = seq_lens; a.parents = parents;
  a.lse = lse; a.delta = (float*)(ws + bp.delta_off); a.dq = dq; a.dk = dk_pages; a.dv = dv_pages;
  a.plan_pb = (int32_t*)(ws + bp.pb_off); a.part_dq = (float*)(ws + bp.part_dq_off);
  return launch_attn_backward(a, st) == hipSuccess ? AURORA_OK : AURORA_ERR_HIP;
}

int check_bwd_args(const aurora_attn_desc* desc, const void* dout, const float* dq, const float* dk_pages,
                   const float* dv_pages, const void* workspace, size_t workspace_bytes, const BwdPlan& bp) {
  if (!dout || !dq || !dk_pages || !dv_pages) return AURORA_ERR_INVALID_ARG;
  if (((uintptr_t)dout | (uintptr_t)dq | (uintptr_t)dk_pages | (uintptr_t)dv_pages) & 15) return AURORA_ERR_INVALID_ARG;
  if (!workspace || misaligned(workspace) || workspace_bytes < bp.bytes) return AURORA_ERR_WORKSPACE;
  return AURORA_OK;
}
}  // namespace

int aurora_attn_backward(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                         const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents,
                         const void* dout, float* dq, float* dk_pages, float* dv_pages,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_attn_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (desc->kv_fp8) return AURORA_ERR_UNSUPPORTED;
  if (desc->batch == 0) return AURORA_OK;
  const BwdPlan bp = plan_bwd(desc);
  rc = check_bwd_args(desc, dout, dq, dk_pages, dv_pages, workspace, workspace_bytes, bp);
  if (rc != AURORA_OK) return rc;
  if (!have_device()) return AURORA_ERR_HIP;
  char* ws = (char*)workspace;
  hipStream_t st = (hipStream_t)hip_stream;
  // forward pass into the workspace: out and the rows' logsumexp
  float* lse = (float*)(ws + bp.lse_off);
  rc = run_attn(desc, q, k_pages, v_pages, block_table, seq_lens, parents, ws + bp.out_off, workspace, bp.fwd_bytes, st, lse);
  if (rc != AURORA_OK) return rc;
  return run_attn_bwd(desc, bp, q, k_pages, v_pages, block_table, seq_lens, parents, ws + bp.out_off, lse, dout, dq,
                      dk_pages, dv_pages, ws, st);
}

void aurora_debug_set_tree_spin_limit(int polls) { set_tree_spin_limit(polls); }

int aurora_attn_forward(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                        const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents, void* out,
                        float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_attn_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (desc->batch > 0 && (!lse || ((uintptr_t)lse & 3))) return AURORA_ERR_INVALID_ARG;
  if (!have_device()) return AURORA_ERR_HIP;
  return run_attn(desc, q, k_pages, v_pages, block_table, seq_lens, parents, out, workspace, workspace_bytes,
                  (hipStream_t)hip_stream, lse);
}

int aurora_attn_backward_saved(const aurora_attn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                               const int32_t* block_table, const int32_t* seq_lens, const int32_t* parents,
                               const void* out, const float* lse, const void* dout, float* dq, float* dk_pages,
                               float* dv_pages, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_attn_desc(desc);
  if (rc != AURORA_OK) return rc;
  if (desc->kv_fp8) return AURORA_ERR_UNSUPPORTED;
  if (desc->batch == 0) return AURORA_OK;
  if (!q || !k_pages || !v_pages || !block_table || !seq_lens || !out || !lse) return AURORA_ERR_INVALID_ARG;
  if (((uintptr_t)q | (uintptr_t)k_pages | (uintptr_t)v_pages | (uintptr_t)out) & 15) return AURORA_ERR_INVALID_ARG;
  const BwdPlan bp = plan_bwd(desc);
  rc = check_bwd_args(desc, dout, dq, dk_pages, dv_pages, workspace, workspace_bytes, bp);
  if (rc != AURORA_OK) return rc;
  if (!have_device()) return AURORA_ERR_HIP;
  return run_attn_bwd(desc, bp, q, k_pages, v_pages, block_table, seq_lens, parents, out, lse, dout, dq, dk_pages,
                      dv_pages, (char*)workspace, (hipStream_t)hip_stream);
}

int aurora_trace_pack(const aurora_pack_desc* d, const int8_t* traj, const void* h, const int32_t* topk_ids,
                      const uint16_t* topk_logits, const int32_t* x_in, const int32_t* y_out,
                      int32_t* n_out, int32_t* row_index, void* h_out, int32_t* topk_ids_out,
                      uint16_t* topk_logits_out, int32_t* x_in_out, int32_t* y_out_out, int8_t* traj_out,
                      void* hip_stream) {
  if (!d || d->rows < 0 || d->top_k < 0 || d->h_row_bytes < 0) return AURORA_ERR_INVALID_ARG;
  if (!n_out || (d->rows > 0 && (!traj || !row_index))) return AURORA_ERR_INVALID_ARG;
  if ((h != nullptr) != (h_out != nullptr) || (h && d->h_row_bytes == 0)) return AURORA_ERR_INVALID_ARG;
  if ((topk_ids != nullptr) != (topk_logits != nullptr)) return AURORA_ERR_INVALID_ARG;
  if ((topk_ids != nullptr) != (topk_ids_out != nullptr) || (topk_logits != nullptr) != (topk_logits_out != nullptr))
    return AURORA_ERR_INVALID_ARG;
  if (topk_ids && d->top_k == 0) return AURORA_ERR_INVALID_ARG;
  if ((x_in != nullptr) != (x_in_out != nullptr) || (y_out != nullptr) != (y_out_out != nullptr))
    return AURORA_ERR_INVALID_ARG;
  PackLaunch P = {};
  P.M = d->rows; P.K = d->top_k; P.h_bytes = (size_t)d->h_row_bytes;
  P.traj = traj; P.h = h; P.ids = topk_ids; P.vals = topk_logits; P.x_in = x_in; P.y = y_out;
  P.n_out = n_out; P.row_index = row_index; P.h_out = h_out; P.ids_out = topk_ids_out; P.vals_out = topk_logits_out;
  P.x_out = x_in_out; P.y_packed = y_out_out; P.traj_out = traj_out;
  return launch_trace_pack(P, (hipStream_t)hip_stream) == hipSuccess ? AURORA_OK : AURORA_ERR_HIP;
}

int aurora_draft_loss(const aurora_loss_desc* d, const float* draft_logits, const int32_t* topk_ids,
                      const uint16_t* topk_logits, const int8_t* traj, float* row_kl, float* loss_out, float* grad,
                      void* hip_stream) {
  if (!d || d->rows < 0 || d->draft_vocab < 1 || d->top_k < 1 || d->discard_top_k < 0 ||
      d->discard_top_k > d->top_k || !(d->lambda_discard >= 0.f) || !(d->lambda_discard < INFINITY))
    return AURORA_ERR_INVALID_ARG;
  if (d->top_k > loss_max_k()) return AURORA_ERR_UNSUPPORTED;
  if (!loss_out) return AURORA_ERR_INVALID_ARG;
  if (d->rows > 0 && (!draft_logits || !topk_ids || !topk_logits || !traj || !row_kl)) return AURORA_ERR_INVALID_ARG;
  if (((uintptr_t)draft_logits | (uintptr_t)grad | (uintptr_t)row_kl | (uintptr_t)loss_out | (uintptr_t)topk_ids) & 3)
    return AURORA_ERR_INVALID_ARG;
  if ((uintptr_t)topk_logits & 1) return AURORA_ERR_INVALID_ARG;
  LossLaunch P = {};
  P.M = d->rows; P.Vd = d->draft_vocab; P.K = d->top_k; P.discard_k = d->discard_top_k; P.lambda = d->lambda_discard;
  P.draft_logits = draft_logits; P.topk_ids = topk_ids; P.topk_logits = topk_logits; P.traj = traj;
  P.row_kl = row_kl; P.loss_out = loss_out; P.grad = grad;
  return launch_draft_loss(P, (hipStream_t)hip_stream) == hipSuccess ? AURORA_OK : AURORA_ERR_HIP;
}

int aurora_trace_emit(const aurora_trace_desc* d, const float* logits, const int32_t* draft_tokens,
                      const int32_t* parents, const int32_t* next_token, const uint8_t* accept_mask,
                      int32_t* topk_ids, uint16_t* topk_logits, int32_t* y_out, int8_t* traj, void* hip_stream) {
  if (!d || d->batch < 0 || d->num_q < 1 || d->vocab < 1 || d->top_k < 1) return AURORA_ERR_INVALID_ARG;
  if (d->draft_vocab < 0 || d->draft_vocab > d->vocab || (d->draft_vocab > 0 && !d->draft_to_target))
    return AURORA_ERR_INVALID_ARG;
  if (d->n_groups < 0 || (d->n_groups > 0 && !d->group_max)) return AURORA_ERR_INVALID_ARG;
  if (d->num_q > kMaxNq || d->top_k > trace_max_k()) return AURORA_ERR_UNSUPPORTED;
  const bool want_topk = topk_ids || topk_logits, want_rec = y_out || traj;
  if (!want_topk && !want_rec) return AURORA_ERR_INVALID_ARG;
  if (want_topk && (!topk_ids || !topk_logits || !logits || ((uintptr_t)logits & 3))) return AURORA_ERR_INVALID_ARG;
  if (want_rec && (!y_out || !traj || !draft_tokens || !next_token || !accept_mask)) return AURORA_ERR_INVALID_ARG;
  if (!have_device()) return AURORA_ERR_HIP;
  if (d->batch == 0) return AURORA_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  RecArgs rec = {};
  if (want_rec) {
    rec.B = d->batch; rec.Nq = d->num_q; rec.draft_tokens = draft_tokens; rec.parents = parents;
    rec.next_token = next_token; rec.accept_mask = accept_mask; rec.y_out = y_out; rec.traj = traj;
  }
  if (want_topk) {
    // the records ride in the same launch as the top-K rows
    if (launch_trace_topk(logits, (int64_t)d->batch * d->num_q, d->vocab, d->top_k,
                          d->draft_vocab > 0 ? d->draft_to_target : nullptr, d->draft_vocab,
                          d->n_groups > 0 ? d->group_max : nullptr, d->n_groups, topk_ids, topk_logits,
                          want_rec ? &rec : nullptr, st) != hipSuccess)
      return AURORA_ERR_HIP;
  } else if (launch_trace_records(rec, st) != hipSuccess) {
    return AURORA_ERR_HIP;
  }
  return AURORA_OK;
}

int aurora_probe_contraction(int mode, const void* operands, size_t operand_bytes, int workgroups, int stages,
                             float* sink, void* hip_stream) {
  if (mode < 0 || mode > 4 || !operands || !sink || workgroups < 1 || stages < 1) return AURORA_ERR_INVALID_ARG;
  if (operand_bytes < probe_operand_bytes() || ((uintptr_t)operands & 15)) return AURORA_ERR_INVALID_ARG;
  if (!have_device()) return AURORA_ERR_HIP;
  if (mode == 4)
    return launch_probe_stream(operands, operand_bytes, (hipStream_t)hip_stream) == hipSuccess ? AURORA_OK : AURORA_ERR_HIP;
  return launch_probe(mode, operands, workgroups, stages, sink, (hipStream_t)hip_stream) == hipSuccess ? AURORA_OK
                                                                                                          : AURORA_ERR_HIP;
}

const char* aurora_status_string(int status) {
  switch (status) {
    case AURORA_OK: return "ok";
    case AURORA_ERR_INVALID_ARG: return "invalid argument";
    case AURORA_ERR_UNSUPPORTED: return "unsupported configuration";
    case AURORA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case AURORA_ERR_HIP: return "HIP runtime error or no device";
    case AURORA_ERR_TOO_LARGE:
      return "problem needs more scratch than the allocation-free entry point's fixed array (AURORA_STATIC_SCRATCH_BYTES) "
             "holds; use the entry point that takes a workspace";
    default: return "unknown status";
  }
}

}  // extern "C"
