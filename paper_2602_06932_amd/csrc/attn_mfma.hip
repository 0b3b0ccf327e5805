// bf16 chunk attention on the matrix cores (paper sections 3.1 / 3.2: the Nq draft positions of a
// request - a chain, or a tree under its ancestor mask - are verified in one pass over the cached
// context).  head_dim 128, KV pages of 16 * 2^i tokens.
//
// The KV sweep is cut into 32-token tiles of one (request, KV head) pair; the tiles of the whole batch,
// numbered request-major, are dealt out in equal contiguous runs to a fixed number of resident
// workgroups (two per compute unit), whatever the mix of sequence lengths.  A workgroup's run meets
// one or a few pairs; for each it produces one partial (m, l, O) - a "segment" - that a small merge
// kernel folds.  The G*Nq query rows that share a KV head form the 32-wide N side of
// v_mfma_f32_32x32x16_bf16, so a KV byte is read once for the whole GQA group.  Inside a segment the
// four wavefronts are independent: wavefront w owns every 4th tile, with private LDS buffers, a
// private online-softmax state, and no workgroup barrier until the segment's merge.
//
//   S^T = K Q^T   tokens are MFMA rows, query rows MFMA columns: a lane owns ONE query row and
//                 16 tokens, so max / sum reduce inside the lane plus one cross-half exchange, and
//                 the exp'd scores are already laid out as the B operand of the next product;
//   O^T = V^T P^T again one query row per lane, so the running rescale is lane-local.
//
// K and V tiles (32 tokens x 256 B) come in by direct global->LDS loads, 16 B per lane, each
// instruction covering four whole token rows (fully coalesced); chunks are XOR-swizzled by
// (row mod 8) so that both the 128-bit K operand reads and the 16-bit strided V^T reads are
// bank-conflict free.  K(t+1) is requested as soon as S(t) has consumed K(t), V(t+1) after
// O += P V(t), so HBM requests stay in flight through the softmax and MFMA phases.
#include "common.hpp"
#include "launch.hpp"

namespace aurora {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) unsigned short u16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

constexpr int kAtThreads = 256;
constexpr int kAtD = 128;
constexpr int kAtTile = 32;                       // tokens per tile
constexpr int kAtRowBytes = kAtD * 2;             // 256
constexpr int kAtTileBytes = kAtTile * kAtRowBytes;  // 8 KB
constexpr float kLog2e = 1.4426950408889634f;

// Direct global->LDS load of 16 bytes per lane: lane i's data lands at lds_base + 16*i.  Written as
// inline assembly so that the compiler's own wait-count bookkeeping does not see it (it would make
// every later LDS read wait for ALL such loads); the explicit s_waitcnt vmcnt(n) below do the
// waiting.  Waits the compiler inserts for its own vector memory operations can only become more
// conservative, because the counter retires in order.
__device__ __forceinline__ void load_to_lds_16(const void* gptr, const void* lds_base) {
  const unsigned base = (unsigned)(uintptr_t)lds_base;  // LDS pointers are 32-bit offsets
  // m0 holds the LDS base; one wait state is required between writing m0 and the load that reads it.
  // Nothing else in this kernel uses m0.
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(__builtin_amdgcn_readfirstlane(base)),
               "v"(gptr)
               : "memory");
}
#define WAIT_VMCNT(n)                                                                              \
  do {                                                                                             \
    __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8));            \
    asm volatile("" ::: "memory");                                                                 \
  } while (0)

// Units of work are 32-token tiles of one (request, KV head) pair, numbered request-major.  PB[b] is
// the number of units before request b; PB[B] the total.
__global__ __launch_bounds__(256) void attn_plan_kernel(const int32_t* __restrict__ seq_lens, int B, int Hkv,
                                                        int32_t* __restrict__ PB) {
  __shared__ int s_part[256];
  __shared__ int s_carry;
  const int tid = threadIdx.x;
  if (tid == 0) { s_carry = 0; PB[0] = 0; }
  __syncthreads();
  for (int b0 = 0; b0 < B; b0 += 256) {
    const int b = b0 + tid;
    const int mine = b < B ? ((seq_lens[b] + kAtTile - 1) / kAtTile) * Hkv : 0;
    s_part[tid] = mine;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {  // inclusive scan
      const int v = tid >= o ? s_part[tid - o] : 0;
      __syncthreads();
      s_part[tid] += v;
      __syncthreads();
    }
    if (b < B) PB[b + 1] = s_carry + s_part[tid];
    __syncthreads();
    if (tid == 255) s_carry += s_part[255];
    __syncthreads();
  }
}

__device__ __forceinline__ int units_per_wg(int U, int wgs) {
  const int c = (U + wgs - 1) / wgs;
  return (c + 3) & ~3;  // a multiple of four tiles: the four wavefronts of a workgroup stay balanced
}

// ---- pieces shared by the two sweep kernels -----------------------------------------------------------
struct SoftmaxState {
  f32x16_t o[4];   // O^T accumulators: block db, register r <-> column 32 db + 8(r/4) + 4*lh + r%4
  float m_run;     // running max of the scaled scores of this lane's query row, log2 units
  float l_half;    // running sum over the tokens this half-lane owns
};

__device__ __forceinline__ void softmax_state_reset(SoftmaxState& st) {
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) st.o[db][r] = 0.f;
  st.m_run = -INFINITY;
  st.l_half = 0.f;
}

// S^T = K Q^T for one 32-token tile: tokens are MFMA rows, the 32 query rows MFMA columns
__device__ __forceinline__ f32x16_t tile_scores(const char* kbuf, const char* qtile, int li, int lh) {
  f32x16_t s_acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) s_acc[r] = 0.f;
  const int sw = li & 15;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const int coff = li * kAtRowBytes + (((2 * s + lh) ^ sw) * 16);
    const bf16x8_t ka = *(const bf16x8_t*)(kbuf + coff);
    const bf16x8_t qa = *(const bf16x8_t*)(qtile + coff);
    s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qa, s_acc, 0, 0, 0);
  }
  return s_acc;
}

// online softmax of the tile (register r holds token j0 + 8(r/4) + 4*lh + r%4 of this lane's row);
// returns the exp'd scores rounded to bf16, already laid out as the B operand of the P.V product
__device__ __forceinline__ void tile_softmax(f32x16_t s_acc, SoftmaxState& st, u16x8_t pb2[2], float scale_log2, int j0,
                                             int prefix, int L, unsigned long long anc, int lh) {
  const bool need_mask = j0 + kAtTile > prefix;
  float tmax = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float x = s_acc[r] * scale_log2;
    if (need_mask) {
      const int j = j0 + 8 * (r >> 2) + 4 * lh + (r & 3);
      const bool seen = j < prefix || (j < L && ((anc >> (j - prefix)) & 1ull));
      x = seen ? x : -INFINITY;
    }
    s_acc[r] = x;
    tmax = fmaxf(tmax, x);
  }
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
  const float m_new = fmaxf(st.m_run, tmax);
  const float m_safe = m_new == -INFINITY ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(st.m_run - m_safe);
  st.m_run = m_new;
  float psum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const float pexp = __builtin_amdgcn_exp2f(s_acc[r] - m_safe);
    psum += pexp;
    pb2[r >> 3][r & 7] = f32_to_bf16(pexp);
  }
  st.l_half = st.l_half * alpha + psum;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
}

// O^T += V^T P^T
__device__ __forceinline__ void tile_pv(const char* vbuf, const u16x8_t pb2[2], SoftmaxState& st, int li, int lh) {
#pragma unroll
  for (int uu = 0; uu < 2; ++uu) {
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      // slot j of this half-lane is token 16u + 8(j/4) + 4*lh + j%4, column d = 32 db + li
      const int d = 32 * db + li;
      u16x8_t va;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int t = 16 * uu + 8 * (j >> 2) + 4 * lh + (j & 3);
        va[j] = *(const unsigned short*)(vbuf + t * kAtRowBytes + (((d >> 3) ^ (t & 15)) * 16) + (d & 7) * 2);
      }
      st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, va),
                                                         __builtin_bit_cast(bf16x8_t, pb2[uu]), st.o[db], 0, 0, 0);
    }
  }
}

// one of the 8 load instructions of a K or V tile: token rows 4j .. 4j+3 of the tile starting at j0
__device__ __forceinline__ void issue_rows(const bf16_t* pool, char* buf, int j, int j0, int L, int page_shift, int Hkv,
                                           int hk, int pid_a, int pid_b, int lane) {
  const int lrow = lane >> 4, lpos = lane & 15;
  const int pa = j0 >> page_shift;
  const int tok = min(j0 + 4 * j + lrow, L - 1);
  const int pid = (tok >> page_shift) == pa ? pid_a : pid_b;
  const int r = 4 * j + lrow;
  const int chunk = lpos ^ (r & 15);
  const bf16_t* src =
      pool + ((((size_t)pid * Hkv + hk) << page_shift) + (tok & ((1 << page_shift) - 1))) * kAtD + chunk * 8;
  load_to_lds_16(src, buf + j * 1024);
}

// prefix of tiles per request (see attn_plan_kernel) built by the whole workgroup into s_pb[0..B], B <= 1024
__device__ __forceinline__ void build_prefix(const int32_t* __restrict__ seq_lens, int B, int Hkv, int* s_pb,
                                             int* s_wsum) {
  const int t4 = threadIdx.x * 4;
  int un[4], loc = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    un[i] = t4 + i < B ? ((seq_lens[t4 + i] + kAtTile - 1) / kAtTile) * Hkv : 0;
    loc += un[i];
  }
  int incl = loc;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int y = __shfl_up(incl, o, kWave);
    if ((int)(threadIdx.x & 63) >= o) incl += y;
  }
  if ((threadIdx.x & 63) == 63) s_wsum[threadIdx.x >> 6] = incl;
  __syncthreads();
  int run = incl - loc;
  for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) run += s_wsum[w];
  if (threadIdx.x == 0) s_pb[0] = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    run += un[i];
    if (t4 + i < B) s_pb[t4 + i + 1] = run;
  }
  __syncthreads();
}

constexpr int kLocalPlanMax = 1024;  // up to this many requests every workgroup builds the prefix itself

template <bool kLocalPlan>
__global__ __launch_bounds__(kAtThreads, 2) void attn_mfma_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kp, const bf16_t* __restrict__ vp,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ parents, int32_t* __restrict__ PB, float* __restrict__ part_o,
    float* __restrict__ part_ml, int B, int Nq, int Hq, int Hkv, int page_shift, int max_pages, float scale_log2) {
  // K and V tiles live in separate LDS objects: the compiler tracks pending LDS-direct loads per object,
  // so a read of a K tile does not wait for the V tile still in flight (and vice versa)
  __shared__ __attribute__((aligned(1024))) char kbuf_all[4 * kAtTileBytes];
  __shared__ __attribute__((aligned(1024))) char vbuf_all[4 * kAtTileBytes];
  __shared__ __attribute__((aligned(1024))) char qbuf[32 * kAtRowBytes];  // the segment's 32 query rows
  __shared__ float s_m[4][32];
  __shared__ float s_l[4][32];

  __shared__ int s_pb[kLocalPlan ? kLocalPlanMax + 1 : 1];
  __shared__ int s_wsum[4];
  if (kLocalPlan) {
    // every workgroup builds the prefix itself; workgroup (0,0) also publishes it for the merge kernel
    build_prefix(seq_lens, B, Hkv, s_pb, s_wsum);
    if (blockIdx.x == 0 && blockIdx.y == 0)
      for (int i = threadIdx.x; i <= B; i += kAtThreads) PB[i] = s_pb[i];
  }
  auto pbv = [&](int i) -> int { return kLocalPlan ? s_pb[i] : PB[i]; };

  const int rt = blockIdx.y, row_tiles = gridDim.y;
  const int U = pbv(B);
  const int c = units_per_wg(U, gridDim.x);
  int u = blockIdx.x * c;
  const int u_end = min(U, u + c);
  if (u >= u_end) return;

  const int G = Hq / Hkv;
  const int R = G * Nq;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, lh = lane >> 5;
  char* kbuf = kbuf_all + wv * kAtTileBytes;
  char* vbuf = vbuf_all + wv * kAtTileBytes;

  // this lane's query row (MFMA column li) within the group: node n, head g
  const int mrow = rt * 32 + li;
  const bool row_ok = mrow < R;
  const int node = row_ok ? mrow / G : 0;
  // the query row this thread stages into LDS at the start of a segment (8 threads per row, 32 B each)
  const int qs_row = tid >> 3;
  const int qs_m = rt * 32 + qs_row;
  const bool qs_ok = qs_m < R;
  const int qs_node = qs_ok ? qs_m / G : 0;
  const int qs_g = qs_ok ? qs_m % G : 0;

  // request holding unit u: largest b with PB[b] <= u
  int b = 0;
  {
    int lo = 0, hi = B - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (pbv(mid) <= u) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }

  // ---- one segment per (request, KV head) pair this workgroup's unit range touches --------------------
  while (u < u_end) {
    while (pbv(b + 1) <= u) ++b;
    const int L = seq_lens[b];
    const int n_b = (L + kAtTile - 1) / kAtTile;
    const int rel = u - pbv(b);
    const int hk = __builtin_amdgcn_readfirstlane(rel / n_b);
    const int t0 = rel - hk * n_b;
    const int t1 = min(n_b, t0 + (u_end - u));
    const int slot = blockIdx.x + b * Hkv + hk;  // segments are a monotone path in (workgroup, pair): unique
    u += t1 - t0;

    const int start = t0 * kAtTile;
    const int prefix = L - Nq;
    {
      // 32 query rows -> LDS, 16-byte chunks swizzled like the K rows (they are read the same way)
      const u32x4_t* qp = (const u32x4_t*)(q + (((size_t)b * Nq + qs_node) * Hq + hk * G + qs_g) * kAtD);
      const int c0 = (tid & 7) * 2;
      u32x4_t z = {0u, 0u, 0u, 0u};
      const u32x4_t v0 = qs_ok ? qp[c0] : z;
      const u32x4_t v1 = qs_ok ? qp[c0 + 1] : z;
      *(u32x4_t*)(qbuf + qs_row * kAtRowBytes + ((c0 ^ (qs_row & 15)) * 16)) = v0;
      *(u32x4_t*)(qbuf + qs_row * kAtRowBytes + (((c0 + 1) ^ (qs_row & 15)) * 16)) = v1;
    }
    // chunk slots this node may see: itself and its ancestors (chain: every slot up to its own)
    unsigned long long anc;
    if (parents) {
      anc = 0;
      for (int a = node, hops = 0; a >= 0 && hops <= Nq; a = parents[(size_t)b * Nq + a], ++hops) anc |= 1ull << a;
    } else {
      anc = node == 63 ? ~0ull : ((1ull << (node + 1)) - 1);
    }

    const int ntile = t1 - t0;
    const int32_t* bt = block_table + (size_t)b * max_pages;

    // Tile loads: always exactly 8 instructions of 4 token rows each (the s_waitcnt bookkeeping below
    // counts them).  Rows past the end of the sequence re-read the last valid token; their scores are
    // masked to -inf, so their (finite) values are multiplied by exact zeros.  A 32-token tile touches
    // at most two pages, whose ids are fetched with scalar loads.
    auto tile_pages = [&](int tt, int& pid_a, int& pid_b) {
      const int j0 = start + tt * kAtTile;
      pid_a = bt[j0 >> page_shift];
      pid_b = bt[min(j0 + 16, L - 1) >> page_shift];
    };
    auto issue_tile = [&](const bf16_t* pool, char* buf, int tt, int pid_a, int pid_b) {
      const int j0 = start + tt * kAtTile;
#pragma unroll
      for (int j = 0; j < 8; ++j) issue_rows(pool, buf, j, j0, L, page_shift, Hkv, hk, pid_a, pid_b, lane);
    };

    SoftmaxState st;
    softmax_state_reset(st);

    __syncthreads();  // query rows staged (nothing is in flight yet, so the fence costs nothing)
    int tt = wv;
    if (tt < ntile) {
      int pa0, pb0;
      tile_pages(tt, pa0, pb0);
      issue_tile(kp, kbuf, tt, pa0, pb0);
      issue_tile(vp, vbuf, tt, pa0, pb0);
    }
    for (; tt < ntile; tt += 4) {
      const bool more = tt + 4 < ntile;
      // page ids of the next tile: scalar loads issued a whole tile ahead of their use
      int npa = 0, npb = 0;
      if (more) tile_pages(tt + 4, npa, npb);
      WAIT_VMCNT(8);  // K(t) landed (V(t) may still be in flight)
      const f32x16_t s_acc = tile_scores(kbuf, qbuf, li, lh);
      // the K buffer is free once the products above have their operands; the memory clobber keeps
      // the compiler from moving the LDS reads below the overwrite
      asm volatile("" ::: "memory");
      if (more) issue_tile(kp, kbuf, tt + 4, npa, npb);
      u16x8_t pb2[2];
      tile_softmax(s_acc, st, pb2, scale_log2, start + tt * kAtTile, prefix, L, anc, lh);
      if (more) WAIT_VMCNT(8); else WAIT_VMCNT(0);  // V(t) landed (K(t+1) may be in flight)
      tile_pv(vbuf, pb2, st, li, lh);
      asm volatile("" ::: "memory");
      if (more) issue_tile(vp, vbuf, tt + 4, npa, npb);
    }
    f32x16_t(&o_acc)[4] = st.o;
    const float m_run = st.m_run, l_half = st.l_half;

    // ---- merge the four wavefronts and write this segment's partial (m, l, O) -------------------------
    float l_row = l_half + __shfl_xor(l_half, 32, kWave);
    if (lh == 0) { s_m[wv][li] = m_run; s_l[wv][li] = l_row; }
    __syncthreads();  // also: every wavefront is done with its K/V buffers
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, s_m[w][li]);
    const float M_safe = M == -INFINITY ? 0.f : M;
    float l_tot = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) l_tot += s_l[w][li] * __builtin_amdgcn_exp2f(s_m[w][li] - M_safe);
    const float f_own = __builtin_amdgcn_exp2f(m_run - M_safe);
    // each wavefront parks its rescaled O^T as [row li][64 d] floats in its K buffer (columns 0..63)
    // and its V buffer (columns 64..127)
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      float* obuf = (float*)((db < 2 ? kbuf_all : vbuf_all) + wv * kAtTileBytes);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int dd = 32 * (db & 1) + 8 * g + 4 * lh;  // column within the 64-wide half
        f32x4_t o = {o_acc[db][4 * g] * f_own, o_acc[db][4 * g + 1] * f_own, o_acc[db][4 * g + 2] * f_own,
                     o_acc[db][4 * g + 3] * f_own};
        // rotate the 16-byte slot by the row so that the 32 rows of a column group spread over banks
        *(f32x4_t*)(obuf + li * 64 + ((dd / 4 + li) & 15) * 4) = o;
      }
    }
    __syncthreads();
    // wavefront w sums and stores d-block w (32 columns) of all rows
    {
      const int db = wv;
      const size_t prow = ((size_t)slot * row_tiles + rt) * 32 + li;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int dd = 32 * (db & 1) + 8 * g + 4 * lh;
        f32x4_t sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float* ob = (const float*)((db < 2 ? kbuf_all : vbuf_all) + w * kAtTileBytes);
          sum += *(const f32x4_t*)(ob + li * 64 + ((dd / 4 + li) & 15) * 4);
        }
        if (row_ok) *(f32x4_t*)(part_o + prow * kAtD + 32 * db + 8 * g + 4 * lh) = sum;
      }
      if (row_ok && wv == 0 && lh == 0) {
        part_ml[prow * 2 + 0] = M * (1.0f / kLog2e);  // natural-log units
        part_ml[prow * 2 + 1] = l_tot;
      }
    }
    __syncthreads();  // the K/V buffers are about to be refilled for the next segment
  }
}

// Merge the partials of one output row (request b, node n, query head hq): the segments of its
// (request, KV head) pair sit in slots w + pair for the workgroups w whose unit range meets the pair's.
__global__ __launch_bounds__(kAtD) void attn_mfma_combine(const float* __restrict__ part_o,
                                                          const float* __restrict__ part_ml,
                                                          const int32_t* __restrict__ seq_lens,
                                                          const int32_t* __restrict__ PB, bf16_t* __restrict__ out, int B,
                                                          int Nq, int Hq, int Hkv, int wgs, int row_tiles) {
  const size_t row = blockIdx.x;  // (b*Nq + n)*Hq + hq
  const int hq = (int)(row % Hq);
  const int n = (int)((row / Hq) % Nq);
  const int b = (int)(row / ((size_t)Hq * Nq));
  const int G = Hq / Hkv;
  const int hk = hq / G;
  const int mrow = n * G + hq % G;
  const int rt = mrow >> 5, li = mrow & 31;
  const int n_b = (seq_lens[b] + kAtTile - 1) / kAtTile;
  const int c = units_per_wg(PB[B], wgs);
  const int u0 = PB[b] + hk * n_b, u1 = u0 + n_b;
  const int w0 = u0 / c, w1 = (u1 - 1) / c;
  const int pair = b * Hkv + hk;
  const int d = threadIdx.x;
  // online merge, four segments' loads in flight at a time
  float M = -INFINITY, num = 0.f, den = 0.f;
  for (int w = w0; w <= w1; w += 4) {
    float ms[4], ls[4], os[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool ok = w + i <= w1;
      const size_t prow = ((size_t)(ok ? w + i + pair : w + pair) * row_tiles + rt) * 32 + li;
      ms[i] = ok ? part_ml[prow * 2] : -INFINITY;
      ls[i] = ok ? part_ml[prow * 2 + 1] : 0.f;
      os[i] = ok ? part_o[prow * kAtD + d] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (ms[i] == -INFINITY) continue;
      const float nm = fmaxf(M, ms[i]);
      const float fo = M == -INFINITY ? 0.f : __expf(M - nm);
      const float fn = __expf(ms[i] - nm);
      num = num * fo + fn * os[i];
      den = den * fo + fn * ls[i];
      M = nm;
    }
  }
  out[row * kAtD + d] = f32_to_bf16(den > 0.f ? num / den : 0.f);
}

bool attn_mfma_supported(const AttnLaunch& a) {
  return a.bf16 && a.D == kAtD && a.page >= 16 && (a.page & (a.page - 1)) == 0;
}

hipError_t launch_attn_mfma(const AttnLaunch& a, hipStream_t st) {
  const int R = a.Hq / a.Hkv * a.Nq;
  const int row_tiles = (R + 31) / 32;
  hipError_t e;
  if (a.B <= kLocalPlanMax) {
    hipLaunchKernelGGL(attn_mfma_kernel<true>, dim3(kAttnWorkgroups, row_tiles), dim3(kAtThreads), 0, st,
                       (const bf16_t*)a.q, (const bf16_t*)a.k, (const bf16_t*)a.v, a.block_table, a.seq_lens, a.parents,
                       a.plan_pb, a.part_o, a.part_ml, a.B, a.Nq, a.Hq, a.Hkv, __builtin_ctz(a.page), a.max_pages,
                       a.scale * kLog2e);
  } else {
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(256), 0, st, a.seq_lens, a.B, a.Hkv, a.plan_pb);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attn_mfma_kernel<false>, dim3(kAttnWorkgroups, row_tiles), dim3(kAtThreads), 0, st,
                       (const bf16_t*)a.q, (const bf16_t*)a.k, (const bf16_t*)a.v, a.block_table, a.seq_lens, a.parents,
                       a.plan_pb, a.part_o, a.part_ml, a.B, a.Nq, a.Hq, a.Hkv, __builtin_ctz(a.page), a.max_pages,
                       a.scale * kLog2e);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const unsigned rows = (unsigned)((size_t)a.B * a.Nq * a.Hq);
  hipLaunchKernelGGL(attn_mfma_combine, dim3(rows), dim3(kAtD), 0, st, a.part_o, a.part_ml, a.seq_lens, a.plan_pb,
                     (bf16_t*)a.out, a.B, a.Nq, a.Hq, a.Hkv, kAttnWorkgroups, row_tiles);
  return hipGetLastError();
}

}  // namespace aurora
