// Host-side launcher interfaces between the C-ABI layer and the kernel translation units.
#pragma once
#include "common.hpp"

namespace aurora {

struct AttnLaunch {
  int B, Nq, Hq, Hkv, D, page, max_pages;
  bool bf16;
  bool kv_fp8;                     // k / v hold E4M3 codes; a value of KV head h is k_scale[h] * decode(code)
  const float *k_scale, *v_scale;  // [Hkv] when kv_fp8
  float scale;
  const void *q, *k, *v;
  const int32_t *block_table, *seq_lens, *parents;
  void* out;
  float* lse_out;  // [B, Nq, Hq] natural-log logsumexp of the scaled scores of every row, or NULL (the backward pass asks for it)
  float *part_o, *part_ml;
  int32_t* plan_pb;
  AttnPlan plan;
};

struct AcceptLaunch {
  int B, Nq, H, V;
  int Vd;                          // draft vocabulary (entries per row of draft_probs) when target_to_draft is set
  const int32_t* target_to_draft;  // or NULL: draft_probs rows are dense over V
  bool bf16;
  bool fp8;                              // hidden / lm_head are E4M3 codes with per-row scales
  const float *hidden_scale, *lm_scale;  // [B*Nq], [V] when fp8
  float temperature;
  const float* temps;  // [B] one temperature per request (0 = greedy request), or NULL: `temperature` for all
  int wor;             // tree siblings were drawn without replacement
  const void *hidden, *lm_head;
  const int32_t *draft_tokens, *parents;
  const float *draft_probs, *uniforms;
  int32_t *accept_len, *next_token;
  uint8_t* accept_mask;
  float *p_at_draft, *row_lse;
  float *logits, *pmax, *psum;
  int32_t* parg;
  float* hmax;  // [rows, n_tiles * kLmHalfPerTile] maxima of groups of 32 vocabulary entries (matrix-core LM head only)
  double *st_lse, *gsum;
  int32_t *st_row, *st_rej, *lastpos;
  int32_t* tree_bar;  // [B] arrival counters of the several-workgroups-per-request tree walk
  AcceptPlan plan;
};

// attention
bool attn_mfma_supported(const AttnLaunch& a);
hipError_t launch_attn_mfma(const AttnLaunch& a, hipStream_t st);
hipError_t launch_attn_generic(const AttnLaunch& a, hipStream_t st);
hipError_t launch_attn_combine(const AttnLaunch& a, hipStream_t st);

// LM head + softmax statistics
bool lmhead_mfma_supported(const AcceptLaunch& a);
int lmhead_mfma_stat_tile();
hipError_t launch_lmhead_mfma(const AcceptLaunch& a, hipStream_t st);  // picks the small- or large-M kernel
constexpr int kLmHalfPerTile = 8;     // groups of 32 vocabulary rows per 256-row statistics tile
constexpr int kLmBigFromRows = 384;  // token rows from which the tiled many-row kernel takes the LM head
bool lmhead_mfma_big_supported(const AcceptLaunch& a);
hipError_t launch_lmhead_mfma_big(const AcceptLaunch& a, hipStream_t st);
hipError_t launch_lmhead_generic(const AcceptLaunch& a, hipStream_t st);

// acceptance walk + residual / bonus draw
void accept_chain_geometry(int batch, int vocab, int* slices, int* gmul, int* ngroups);
int accept_tree_max_slices();  // workgroups per request the tree walk may use (sizes its exchange buffers)
hipError_t launch_accept(const AcceptLaunch& a, hipStream_t st);

// trace emission: top-K target logits per token row, y_out and rejection trajectory
int trace_max_k();
// calibration probe (see probe.hip)
size_t probe_operand_bytes();
hipError_t launch_probe_stream(const void* operands, size_t operand_bytes, hipStream_t st);
hipError_t launch_probe(int mode, const void* operands, int workgroups, int stages, float* sink, hipStream_t st);

// records of the acceptance outcome (y_out, rejection trajectory); B = 0: none wanted
struct RecArgs {
  int B, Nq;  // B = 0: no records wanted
  const int32_t* draft_tokens;
  const int32_t* parents;
  const int32_t* next_token;
  const uint8_t* accept_mask;
  int32_t* y_out;
  int8_t* traj;
};
hipError_t launch_trace_topk(const float* logits, int64_t rows, int V, int K, const int32_t* map, int n_map,
                             const float* group_max, int n_groups, int32_t* ids, uint16_t* vals, const RecArgs* rec,
                             hipStream_t st);
hipError_t launch_trace_records(const RecArgs& R, hipStream_t st);

// backward pass of the chunk / tree attention (see attn_bwd.hip); out / lse come from the forward kernels
struct AttnBwdLaunch {
  int B, Nq, Hq, Hkv, D, page, max_pages;
  bool bf16;
  float scale;
  const void *q, *k, *v, *out, *dout;
  const int32_t *block_table, *seq_lens, *parents;
  const float* lse;
  float *delta, *dq, *dk, *dv;
  // matrix-core kernel only: tile prefix per request [B + 1] and the per-run partial dq
  int32_t* plan_pb;
  float* part_dq;
};
hipError_t launch_attn_backward(const AttnBwdLaunch& a, hipStream_t st);
// matrix-core kernel (attn_bwd_mfma.hip): shapes it takes, its resident workgroups, and its launch (delta is ready)
void set_tree_spin_limit(int polls);  // accept.hip: bounded wait of the split tree walk (negative: default)
// tile prefix per request, PB[0 .. B], by one workgroup (attn_mfma.hip): for batches past the in-LDS plan
hipError_t launch_attn_plan(const int32_t* seq_lens, int B, int Hkv, int32_t* PB, hipStream_t st);
bool attn_bwd_mfma_supported(const AttnBwdLaunch& a);
int attn_bwd_mfma_workgroups();
size_t attn_bwd_mfma_partial_bytes(int batch, int kv_heads, int rows_per_group);
hipError_t launch_attn_backward_mfma(const AttnBwdLaunch& a, hipStream_t st);

// packing of trace records (see pack.hip)
struct PackLaunch {
  int M, K;
  size_t h_bytes;           // bytes of one hidden row
  const int8_t* traj;
  const void* h;            // or NULL
  const int32_t* ids;       // [M, K] or NULL (then vals is NULL too)
  const uint16_t* vals;
  const int32_t *x_in, *y;  // [M] or NULL
  int32_t *n_out, *row_index;
  void* h_out;
  int32_t* ids_out;
  uint16_t* vals_out;
  int32_t *x_out, *y_packed;
  int8_t* traj_out;
};
hipError_t launch_trace_pack(const PackLaunch& P, hipStream_t st);

// drafter training loss on trace rows (see loss.hip)
struct LossLaunch {
  int M, Vd, K, discard_k;
  float lambda;
  const float* draft_logits;
  const int32_t* topk_ids;
  const uint16_t* topk_logits;
  const int8_t* traj;
  float *row_kl, *loss_out, *grad;
};
int loss_max_k();
hipError_t launch_draft_loss(const LossLaunch& P, hipStream_t st);

// debug check of device-resident inputs (see check.hip); bits of flags[0]
constexpr unsigned kCheckSeqLen = 1, kCheckPageId = 2, kCheckParent = 4, kCheckToken = 8, kCheckUniform = 16;
constexpr int kCheckKinds = 5;
struct CheckLaunch {
  int B, Nq, page, max_pages, V;
  long long num_pages;
  const int32_t *block_table, *seq_lens, *parents, *draft_tokens;
  const float* uniforms;
  int32_t* flags;  // [1 + kCheckKinds]
};
hipError_t launch_check_inputs(const CheckLaunch& c, hipStream_t st);

}  // namespace aurora
