// bf16 LM-head projection on the matrix cores, fused with per-tile softmax statistics
// (appendix A.1, eq. 4 of the paper: target logits l in R^{T x V}; the acceptance step needs
// their row-wise softmax).
//
//   logits[m, v] = sum_h hidden[m, h] * W[v, h]      hidden [M, H] bf16, W [V, H] bf16, fp32 out
//
// The weight matrix is streamed from HBM exactly once; it is the dominant traffic of the whole
// verify step.  One workgroup (4 multiplying + 4 loading wavefronts) owns 256 vocabulary rows and up to 160 token rows
// and walks the hidden dimension in steps of 64.  Each step's operands are brought in with
// direct global->LDS loads (16 B per lane, fully coalesced 128-B rows) into a 3-deep ring of
// LDS stages, so two steps are always in flight while one is being multiplied.  The 16-byte
// chunks of every row are XOR-swizzled by (row mod 8) on the way in - the global address a lane
// reads is permuted, the LDS slot is fixed by the lane id - which makes the 128-bit operand
// reads of v_mfma_f32_32x32x16_bf16 bank-conflict free.
// Vocabulary rows are the MFMA "A" rows and tokens its "B" columns: a lane then holds 16 vocab
// entries of ONE token per accumulator tile, so row statistics (max, arg-max, sum exp) reduce
// inside a lane and need a single cross-lane step.
#include "launch.hpp"
#include "lmhead_tile.hpp"

namespace aurora {

constexpr int kLmThreads = 512;                // 4 consumer + 4 producer wavefronts
constexpr int kLmRowBytes = 128;               // bytes of a row segment per stage: 64 bf16 or 128 fp8 elements
constexpr int kLmVTile = 256;                  // vocab rows per workgroup
constexpr int kLmWaveV = 64;                   // vocab rows per wavefront (= statistics tile)
constexpr int kLmStages = 3;
constexpr int kLmWBytes = kLmVTile * kLmRowBytes;  // 32 KB
// cache-policy operand of the LDS-direct load: "non-temporal".  W is read exactly once, so it should
// not displace the hidden-state rows that every workgroup re-reads from L2.
constexpr int kCpolNT = 2;

#define WAIT_VMCNT(n) LM_WAIT_VMCNT(n)

// kFp8: operands are OCP E4M3 codes (1 byte) with one float32 scale per token row and per vocabulary
// row; the products run on v_mfma_scale_f32_32x32x64_f8f6f4 (K = 64: twice the products per cycle of the
// K = 16 fp8 form, which runs at the bf16 rate), and the scales are applied to the fp32 accumulators in the
// epilogue.  A stage then holds 128 hidden elements per row instead of 64 - the same 128 bytes.
template <int NT, bool kFp8>
__global__ __launch_bounds__(kLmThreads, 1) void lmhead_mfma_kernel(
    const char* __restrict__ hidden, const char* __restrict__ w, const float* __restrict__ h_scale,
    const float* __restrict__ w_scale, float* __restrict__ logits, float* __restrict__ pmax,
    float* __restrict__ psum, int32_t* __restrict__ parg, float* __restrict__ hmax, int M, int H, int V, int n_tiles,
    int m_tiles,
    float exp_scale /* log2(e) / T */, const float* __restrict__ temps /* per-request T, or NULL */, int Nq) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  constexpr int kEsz = kFp8 ? 1 : 2;             // bytes per operand element
  constexpr int kLmBK = kLmRowBytes / kEsz;      // hidden elements per stage
  constexpr int kStageBytes = kLmWBytes + NT * 32 * kLmRowBytes;
  constexpr int kLoadsPerStage = 8 + NT;  // global->LDS instructions per producer wavefront per stage

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool producer = wave >= 4;
  const int wv = wave & 3;  // vocab slice: consumer wv multiplies the rows producer wv + 4 brings in
  // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  The m_tiles token passes
  // over one vocab tile get ids 8 apart: same XCD, launched together, walking k in the same order - so
  // the W tile comes from HBM once and from L2 for the other passes.
  const int wg = blockIdx.x;
  const int vt = (wg / (8 * m_tiles)) * 8 + (wg & 7);
  const int mt = (wg >> 3) % m_tiles;
  if (vt >= n_tiles) return;
  const int vbase = vt * kLmVTile;
  const int m0 = mt * (NT * 32);
  const int nk = H / kLmBK;
  // Workgroups start their walk over the hidden dimension at different offsets (and wrap around):
  // rows are a multiple of the memory-channel interleave apart, so workgroups marching through k
  // in lockstep would all hit the same few HBM channels at any moment.
  const int ks0 = (int)((vt * 13u) % (unsigned)nk);

  if (producer) {
    // ---- producer wavefronts: nothing but address arithmetic, LDS-direct loads and barriers ----------
    // rows are clamped into range; out-of-range rows are masked in the epilogue
    const int sub = lane >> 3;  // row within an 8-row load instruction
    // 16-byte chunk c of row r lives in LDS slot c ^ ((r >> 1) & 7): sixteen consecutive rows then
    // put one chunk index into sixteen different 16-byte bank groups of the 64-bank LDS
    const int chunk_even = (lane & 7) ^ (sub >> 1);        // instructions whose first row is 0 mod 16
    const int chunk_odd = (lane & 7) ^ (4 + (sub >> 1));   // ... 8 mod 16
    const char* wsrc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int row = vbase + wv * kLmWaveV + 8 * j + sub;
      row = row < V ? row : V - 1;
      wsrc[j] = w + (size_t)row * H * kEsz + ((j & 1) ? chunk_odd : chunk_even) * 16;
    }
    const char* hsrc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int q8 = wv * NT + j;  // 8-row group of the hidden tile
      int row = m0 + 8 * q8 + sub;
      row = row < M ? row : M - 1;
      hsrc[j] = hidden + (size_t)row * H * kEsz + ((q8 & 1) ? chunk_odd : chunk_even) * 16;
    }
    auto issue = [&](int ks, int buf) {
      char* base = lds + buf * kStageBytes;
      int kk = ks + ks0;
      kk = kk >= nk ? kk - nk : kk;
      const int koff = kk * kLmRowBytes;  // bytes
#pragma unroll
      for (int j = 0; j < 8; ++j)
        __builtin_amdgcn_global_load_lds(GLB_PTR(wsrc[j] + koff),
                                         LDS_PTR(base + (wv * kLmWaveV + 8 * j) * kLmRowBytes), 16, 0, kCpolNT);
#pragma unroll
      for (int j = 0; j < NT; ++j)
        __builtin_amdgcn_global_load_lds(GLB_PTR(hsrc[j] + koff),
                                         LDS_PTR(base + kLmWBytes + 8 * (wv * NT + j) * kLmRowBytes), 16, 0, 0);
    };
    issue(0, 0);
    if (nk > 1) issue(1, 1);
    for (int ks = 0; ks < nk; ++ks) {
      // stage ks has landed once at most one younger stage's loads are still outstanding
      if (ks + 1 < nk) WAIT_VMCNT(kLoadsPerStage); else WAIT_VMCNT(0);
      __builtin_amdgcn_s_barrier();  // stage ks visible to the consumers; stage ks-1's buffer is free
      if (ks + 2 < nk) issue(ks + 2, (ks + 2) % kLmStages);
    }
    __builtin_amdgcn_s_barrier();  // pairs with the consumers' statistics exchange below
    return;
  }

  // ---- consumer wavefronts ------------------------------------------------------------------------
  f32x16_t acc[2][NT];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;

  const int li = lane & 31, lh = lane >> 5;
  // byte offsets of this lane's operand rows inside a stage (the chunk term is added per step)
  const int wrow_off = (wv * kLmWaveV + li) * kLmRowBytes;
  const int hrow_off = kLmWBytes + li * kLmRowBytes;
  const int sw = (li >> 1) & 7;

  // A stage is walked in four steps of one 16-byte chunk pair per row: lane half lh takes chunk 2s + lh.
  // For bf16 that is one MFMA step (k = 16); the 8-bit path further down joins two steps into one K = 64
  // MFMA.  The operands of step s+1 are read from LDS while the MFMAs of step s run (fragments
  // double-buffered in registers), and the barrier that opens the next stage sits before the last step
  // of the current one, so that the matrix pipe never waits for LDS latency or for the barrier.
  typedef __attribute__((ext_vector_type(2))) long i64x2_t;
  struct Frag { i64x2_t w[2], h[NT]; };
  auto load_frag = [&](int stage, int s, Frag& f) {
    const char* base = lds + stage * kStageBytes;
    const int coff = ((2 * s + lh) ^ sw) * 16;
#pragma unroll
    for (int a = 0; a < 2; ++a) f.w[a] = *(const i64x2_t*)(base + wrow_off + a * 32 * kLmRowBytes + coff);
#pragma unroll
    for (int t = 0; t < NT; ++t) f.h[t] = *(const i64x2_t*)(base + hrow_off + t * 32 * kLmRowBytes + coff);
  };
  auto multiply = [&](const Frag& f) {  // bf16 operands
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int t = 0; t < NT; ++t)
        acc[a][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, f.w[a]),
                                                            __builtin_bit_cast(bf16x8_t, f.h[t]), acc[a][t], 0, 0, 0);
  };
  constexpr int kMfmaPerStep = 2 * NT;
  // pins "this step's LDS reads, then the previous step's MFMAs" against the compiler's own ordering
#define LM_STEP_ORDER()                                                 \
  do {                                                                  \
    __builtin_amdgcn_sched_group_barrier(0x100, 2 + NT, 0);             \
    __builtin_amdgcn_sched_group_barrier(0x008, kMfmaPerStep, 0);       \
    __builtin_amdgcn_sched_barrier(0);                                  \
  } while (0)

  if constexpr (kFp8) {
    // 8-bit operands: the K = 16 fp8 MFMA runs at the bf16 rate; the K = 64 form (v_mfma_scale_f32_32x32x64_f8f6f4,
    // both formats E4M3, unit scales) delivers twice the products per cycle.  It takes 32 bytes per lane and operand:
    // the lane's 16-byte chunks of two consecutive steps (which hidden elements meet in which MFMA does not matter
    // as long as both operands are read the same way).  A stage is two such double steps.
    typedef __attribute__((ext_vector_type(8))) int i32x8_t;
    typedef __attribute__((ext_vector_type(4))) int i32x4_t;
    // Operands roll through the registers: the two W operands of the next double step are read into a second pair
    // (16 registers), and a token-row operand is re-read for the next double step right after the two MFMAs that
    // consumed it - so the LDS reads of a double step run under the MFMAs of the previous one without a second full
    // fragment set (which would not fit beside the 32 NT accumulator registers).
    auto ld_w = [&](int stg, int s2, i32x8_t (&wf)[2]) {
      const char* base = lds + stg * kStageBytes + wrow_off;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int coff = ((2 * (2 * s2 + e) + lh) ^ sw) * 16;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          const i32x4_t v = *(const i32x4_t*)(base + a * 32 * kLmRowBytes + coff);
#pragma unroll
          for (int i = 0; i < 4; ++i) wf[a][4 * e + i] = v[i];
        }
      }
    };
    auto ld_h = [&](int stg, int s2, int t, i32x8_t& hf) {
      const char* base = lds + stg * kStageBytes + hrow_off + t * 32 * kLmRowBytes;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int coff = ((2 * (2 * s2 + e) + lh) ^ sw) * 16;
        const i32x4_t v = *(const i32x4_t*)(base + coff);
#pragma unroll
        for (int i = 0; i < 4; ++i) hf[4 * e + i] = v[i];
      }
    };
    auto mul_t = [&](const i32x8_t (&wf)[2], const i32x8_t& hf, int t) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
        acc[a][t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[a], hf, acc[a][t], 0, 0, 0, 127, 0, 127);
    };
    // First double step of a stage, rolling in its second.  Pinned order: two MFMAs; the next W pair's four reads, the two
    // that refill the first token operand and the two of the last token operand of THIS double step (held back from
    // the previous roll, so that a loop iteration ends on MFMAs and the wait at its head finds every read returned);
    // then per further token tile two MFMAs and the two reads that refill its operand.
    constexpr bool kDefer = NT >= 2;
    i32x8_t wA[2], wB[2], hf[NT];
    auto phase_a = [&](int stg_) {
      ld_w(stg_, 1, wB);
      if (kDefer) ld_h(stg_, 0, NT - 1, hf[NT - 1]);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        mul_t(wA, hf[t], t);
        ld_h(stg_, 1, t, hf[t]);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, kDefer ? 8 : 6, 0);
      for (int t_ = 1; t_ < NT; ++t_) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    __builtin_amdgcn_s_barrier();  // stage 0 visible
    asm volatile("" ::: "memory");
    int stg = 0;
    ld_w(0, 0, wA);
#pragma unroll
    for (int t = 0; t < NT; ++t) ld_h(0, 0, t, hf[t]);
    for (int ks = 0; ks + 1 < nk; ++ks) {
      phase_a(stg);
      // second double step, rolling in the first of the next stage: the barrier that opens that stage comes after
      // the first pair of MFMAs, which covers the return of this stage's last reads
      mul_t(wB, hf[0], 0);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt((7 << 4) | (3 << 14) | 15);  // lgkmcnt(0) only: every read of this stage is back
      __builtin_amdgcn_s_barrier();  // stage ks+1 visible; this stage's buffer may be refilled
      asm volatile("" ::: "memory");
      stg = stg + 1 == kLmStages ? 0 : stg + 1;
      ld_w(stg, 0, wA);
      ld_h(stg, 0, 0, hf[0]);
#pragma unroll
      for (int t = 1; t < NT; ++t) {
        mul_t(wB, hf[t], t);
        if (!kDefer || t < NT - 1) ld_h(stg, 0, t, hf[t]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
      for (int t_ = 1; t_ < NT; ++t_) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        if (!kDefer || t_ < NT - 1) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // the last stage: nothing left to roll in behind its second double step
    phase_a(stg);
#pragma unroll
    for (int t = 0; t < NT; ++t) mul_t(wB, hf[t], t);
    // the epilogue's work stays behind the last MFMAs: mixed in with them it would need registers the operands still hold
#pragma unroll
    for (int t = 0; t < NT; ++t) asm volatile("" : "+v"(acc[0][t]), "+v"(acc[1][t])::"memory");
  } else {
  Frag f0, f1;
  __builtin_amdgcn_s_barrier();  // stage 0 visible
  asm volatile("" ::: "memory");
  load_frag(0, 0, f0);
  int stage = 0;
  for (int ks = 0; ks < nk; ++ks) {
    load_frag(stage, 1, f1);
    multiply(f0);
    LM_STEP_ORDER();
    load_frag(stage, 2, f0);
    multiply(f1);
    LM_STEP_ORDER();
    load_frag(stage, 3, f1);
    multiply(f0);
    LM_STEP_ORDER();
    if (ks + 1 < nk) {
      // every LDS read of this stage has returned before the producers are told its buffer may be refilled
      __builtin_amdgcn_s_waitcnt((7 << 4) | (3 << 14) | 15);  // lgkmcnt(0) only
      __builtin_amdgcn_s_barrier();  // stage ks+1 visible
      asm volatile("" ::: "memory");
      stage = stage + 1 == kLmStages ? 0 : stage + 1;
      load_frag(stage, 0, f0);
    }
    multiply(f1);
    LM_STEP_ORDER();
  }
  }
#undef LM_STEP_ORDER

  // ---- epilogue: logits out, and (max, arg-max, sum exp) of the workgroup's 256 vocab rows ---------
  // Each wavefront reduces its 64 rows per token in registers and parks the triple in an LDS stage
  // that the main loop no longer touches; after one barrier the first 32*NT threads merge the four
  // wavefronts.  The logits go out through this wavefront's own W rows of stage 0 (idle now).
  float* st_max = (float*)(lds + (nk % kLmStages) * kStageBytes + kLmWBytes);  // hidden part of an idle stage
  float* st_sum = st_max + 4 * NT * 32;
  int* st_arg = (int*)(st_sum + 4 * NT * 32);
  float* st_half = (float*)(st_arg + 4 * NT * 32);  // [8][NT * 32]: maxima of the eight groups of 32 vocab rows
  const int vrow0 = vbase + wv * kLmWaveV;
  const bool vec_ok = (V & 3) == 0;
  char* tb = lds + wv * (kLmWaveV * kLmRowBytes);
  if constexpr (kFp8) {
    // dequantise: accumulator (vocab row v, token m) times w_scale[v] * h_scale[m]
    float hs[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int m = m0 + 32 * t + li;
      hs[t] = h_scale[m < M ? m : M - 1];
    }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        // four consecutive vocabulary rows: 8(r/4) + 4 lh + r%4 for r = 4g .. 4g+3
        const int v = vrow0 + 32 * a + 8 * g + 4 * lh;
        float wsc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) wsc[e] = w_scale[v + e < V ? v + e : V - 1];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[a][t][4 * g + e] *= wsc[e] * hs[t];
      }
  }
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    float mx, sum, half;
    int arg;
    lm_tile_out(acc[0][t], acc[1][t], vrow0, V, m0 + 32 * t, M, lm_row_scale(exp_scale, temps, Nq, m0 + 32 * t + li, M), tb,
                logits, vec_ok, lane, mx, sum, arg, half);
    if (lh == 0) {
      st_max[wv * NT * 32 + t * 32 + li] = mx;
      st_sum[wv * NT * 32 + t * 32 + li] = sum;
      st_arg[wv * NT * 32 + t * 32 + li] = arg;
    }
    st_half[(2 * wv + lh) * NT * 32 + t * 32 + li] = half;
  }
  __syncthreads();  // the producers' last barrier pairs with this one
  if (tid < NT * 32) {
    const int m = m0 + tid;
    if (m < M) {
      float mx, sum;
      int arg;
      lm_merge_waves(st_max, st_sum, st_arg, NT * 32, tid, lm_row_scale(exp_scale, temps, Nq, m, M), mx, sum, arg);
      const size_t o = (size_t)m * n_tiles + vt;
      pmax[o] = mx;
      psum[o] = sum;
      parg[o] = arg;
      // the eight group maxima of this tile, 32 contiguous bytes per token row
      f32x4_t h0, h1;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        h0[j] = st_half[j * NT * 32 + tid];
        h1[j] = st_half[(4 + j) * NT * 32 + tid];
      }
      f32x4_t* hd = (f32x4_t*)(hmax + ((size_t)m * n_tiles + vt) * kLmHalfPerTile);
      hd[0] = h0;
      hd[1] = h1;
    }
  }
}

bool lmhead_mfma_supported(const AcceptLaunch& a) {
  const int bk = a.fp8 ? kLmRowBytes : kLmRowBytes / 2;  // hidden elements per stage
  return (a.bf16 || a.fp8) && a.H % bk == 0 && a.H >= bk && a.V >= 1;
}

int lmhead_mfma_stat_tile() { return kLmVTile; }

template <int NT, bool kFp8>
static hipError_t launch_nt_t(const AcceptLaunch& a, hipStream_t st, int m_tiles) {
  constexpr int lds_bytes = kLmStages * (kLmWBytes + NT * 32 * kLmRowBytes);
  static LdsAttrOnce attr;
  if (hipError_t e = attr.ensure((const void*)lmhead_mfma_kernel<NT, kFp8>, lds_bytes); e != hipSuccess) return e;
  const float exp_scale = 1.4426950408889634f / (a.temperature > 0.f ? a.temperature : 1.f);
  const int v_tiles = (a.V + kLmVTile - 1) / kLmVTile;
  dim3 grid((v_tiles + 7) / 8 * 8 * m_tiles);
  hipLaunchKernelGGL((lmhead_mfma_kernel<NT, kFp8>), grid, dim3(kLmThreads), lds_bytes, st, (const char*)a.hidden,
                     (const char*)a.lm_head, a.hidden_scale, a.lm_scale, a.logits, a.pmax, a.psum, a.parg, a.hmax,
                     (int)a.plan.rows, a.H, a.V, a.plan.n_tiles, m_tiles, exp_scale, a.temps, a.Nq);
  return hipGetLastError();
}

template <int NT>
static hipError_t launch_nt(const AcceptLaunch& a, hipStream_t st, int m_tiles) {
  return a.fp8 ? launch_nt_t<NT, true>(a, st, m_tiles) : launch_nt_t<NT, false>(a, st, m_tiles);
}

hipError_t launch_lmhead_mfma(const AcceptLaunch& a, hipStream_t st) {
  const int M = (int)a.plan.rows;
  // From 384 token rows on the contraction is bound by the matrix cores and the tiled kernel, in which all
  // wavefronts multiply and whose workgroup columns are sized to the token rows, is the faster one (measured on
  // 128256 x 4096: 448 rows 0.52 against 0.55 ms, 1280 rows 1.33 against 1.44 ms; 320 rows 0.43 against 0.37 ms).
  if (M >= kLmBigFromRows && lmhead_mfma_big_supported(a)) return launch_lmhead_mfma_big(a, st);
  // token rows per workgroup: the fewest 160-row passes over W, each as narrow as the rows allow
  const int passes = (M + 159) / 160;
  const int per = (M + passes - 1) / passes;
  const int nt = (per + 31) / 32;
  const int m_tiles = (M + nt * 32 - 1) / (nt * 32);
  switch (nt) {
    case 1: return launch_nt<1>(a, st, m_tiles);
    case 2: return launch_nt<2>(a, st, m_tiles);
    case 3: return launch_nt<3>(a, st, m_tiles);
    case 4: return launch_nt<4>(a, st, m_tiles);
    default: return launch_nt<5>(a, st, m_tiles);
  }
}

}  // namespace aurora
