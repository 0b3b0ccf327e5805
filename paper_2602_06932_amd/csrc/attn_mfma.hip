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
#include "launch.hpp"
#include "attn_tile.hpp"

namespace aurora {

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

hipError_t launch_attn_plan(const int32_t* seq_lens, int B, int Hkv, int32_t* PB, hipStream_t st) {
  hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(256), 0, st, seq_lens, B, Hkv, PB);
  return hipGetLastError();
}

// kFp8KV: kp_ / vp_ hold E4M3 codes and k_scale / v_scale [Hkv] their per-head scales (see Tile8 above);
// otherwise bf16 pools, loaded straight into LDS.
template <bool kLocalPlan, bool kFp8KV>
__global__ __launch_bounds__(kAtThreads, 2) void attn_mfma_kernel(
    const bf16_t* __restrict__ q, const void* __restrict__ kp_, const void* __restrict__ vp_,
    const float* __restrict__ k_scale, const float* __restrict__ v_scale,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ parents, int32_t* __restrict__ PB, float* __restrict__ part_o,
    float* __restrict__ part_ml, int B, int Nq, int Hq, int Hkv, int page_shift, int max_pages, float scale_log2_q) {
  const bf16_t* kp = (const bf16_t*)kp_;
  const bf16_t* vp = (const bf16_t*)vp_;
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
  int u = unit_begin(U, gridDim.x, blockIdx.x);
  const int u_end = unit_begin(U, gridDim.x, blockIdx.x + 1);
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
    const float scale_log2 = kFp8KV ? scale_log2_q * k_scale[hk] : scale_log2_q;
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
    auto issue_k = [&](int tt, int pid_a, int pid_b) {
      const int j0 = start + tt * kAtTile;
#pragma unroll
      for (int j = 0; j < 8; ++j) issue_rows<false>(kp, kbuf, j, j0, L, page_shift, Hkv, hk, pid_a, pid_b, lane);
    };
    auto issue_v = [&](int tt, int pid_a, int pid_b) {
      const int j0 = start + tt * kAtTile;
#pragma unroll
      for (int j = 0; j < 8; ++j) issue_rows<true>(vp, vbuf, j, j0, L, page_shift, Hkv, hk, pid_a, pid_b, lane);
    };

    SoftmaxState st;
    softmax_state_reset(st);

    __syncthreads();  // query rows staged (nothing is in flight yet, so the fence costs nothing)
    if constexpr (kFp8KV) {
      // This wavefront's tiles are wv, wv + 4, ...; two of them are always on their way into registers.
      // Loads past the wavefront's last tile re-read that tile (cache hits), so the loop body is straight
      // code and the compiler's wait counts leave the younger tile in flight.
      const int n_my = ntile > wv ? (ntile - wv + 3) >> 2 : 0;
      if (n_my > 0) {
        const uint8_t* kp8 = (const uint8_t*)kp_;
        const uint8_t* vp8 = (const uint8_t*)vp_;
        auto fetch = [&](Tile8& t, int i) {
          const int tile = wv + 4 * min(i, n_my - 1);
          int pa, pb;
          tile_pages(tile, pa, pb);
          load_tile8(t, kp8, vp8, start + tile * kAtTile, L, page_shift, Hkv, hk, pa, pb, lane);
        };
        // `live` is wave-uniform; a dead turn (odd tile count) still spills and fetches, so that the order
        // of loads and waits is the same on every path
        auto consume = [&](Tile8& t, int i, bool live) {
          spill_tile8(t, kbuf, vbuf, lane);
          fetch(t, i + 2);
          if (live) {
            const f32x16_t s_acc = tile_scores(kbuf, qbuf, li, lh);
            bf16x8_t pb2[2];
            tile_softmax(s_acc, st, pb2, scale_log2, start + (wv + 4 * i) * kAtTile, prefix, L, anc, lh);
            tile_pv(vbuf, pb2, st, lane);
          }
        };
        Tile8 ta, tb;
        fetch(ta, 0);
        fetch(tb, 1);
        for (int i = 0; i < n_my; i += 2) {
          consume(ta, i, true);
          consume(tb, i + 1, i + 1 < n_my);
        }
      }
    } else {
    int tt = wv;
    if (tt < ntile) {
      int pa0, pb0;
      tile_pages(tt, pa0, pb0);
      issue_k(tt, pa0, pb0);
      issue_v(tt, pa0, pb0);
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
      if (more) issue_k(tt + 4, npa, npb);
      bf16x8_t pb2[2];
      tile_softmax(s_acc, st, pb2, scale_log2, start + tt * kAtTile, prefix, L, anc, lh);
      if (more) WAIT_VMCNT(8); else WAIT_VMCNT(0);  // V(t) landed (K(t+1) may be in flight)
      tile_pv(vbuf, pb2, st, lane);
      asm volatile("" ::: "memory");
      if (more) issue_v(tt + 4, npa, npb);
    }
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
    const float f_own = __builtin_amdgcn_exp2f(m_run - M_safe) * (kFp8KV ? v_scale[hk] : 1.f);
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

// ---- wide-row variant: more than 32 query rows per (request, KV head) pair (draft trees) ----------------
// Eight wavefronts: wavefront (g, w) owns the 32-row query tile w and the KV tiles of parity g, so a KV
// byte is still read once per pair while two wavefronts per SIMD hide each other's latencies.  K/V
// tiles go through a ring of LDS stages of two tiles each (every wavefront loads an eighth of both),
// one workgroup barrier per step; one workgroup per compute unit.  Work is dealt out exactly as in the
// narrow kernel; each wavefront writes its own partial, two per segment and query tile.
constexpr int kWideThreads = 512;
constexpr int kWideStages = 3;
constexpr int kWideStageBytes = 2 * 2 * kAtTileBytes;                // two tiles, K and V
constexpr int kWideQBytes = 4 * 32 * kAtRowBytes;                    // four query tiles
constexpr int kWideLdsBytes = kWideQBytes + kWideStages * kWideStageBytes;

// kFp8KV: the cache holds E4M3 codes (see Tile8 above).  A wavefront then fetches its eighth of a step - four
// token rows of K in lanes 0..31, of V in lanes 32..63, for each of the step's two tiles - into registers
// two steps ahead, and widens it into the ring stage right before the step's barrier.
template <bool kLocalPlan, bool kFp8KV>
__global__ __launch_bounds__(kWideThreads, 1) void attn_mfma_wide_kernel(
    const bf16_t* __restrict__ q, const void* __restrict__ kp_, const void* __restrict__ vp_,
    const float* __restrict__ k_scale, const float* __restrict__ v_scale,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ parents, int32_t* __restrict__ PB, float* __restrict__ part_o,
    float* __restrict__ part_ml, int B, int Nq, int Hq, int Hkv, int page_shift, int max_pages, int row_tiles,
    float scale_log2_q) {
  const bf16_t* kp = (const bf16_t*)kp_;
  const bf16_t* vp = (const bf16_t*)vp_;
  extern __shared__ __attribute__((aligned(1024))) char wlds[];
  char* qall = wlds;
  char* ring = wlds + kWideQBytes;
  __shared__ int s_pb[kLocalPlan ? kLocalPlanMax + 1 : 1];
  __shared__ int s_wsum[kWideThreads / kWave];
  if (kLocalPlan) {
    // as build_prefix, for 512 threads (threads 256.. own requests beyond 1024: none)
    {
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
    if (blockIdx.x == 0 && blockIdx.y == 0)
      for (int i = threadIdx.x; i <= B; i += kWideThreads) PB[i] = s_pb[i];
  }
  auto pbv = [&](int i) -> int { return kLocalPlan ? s_pb[i] : PB[i]; };

  const int U = pbv(B);
  int u = unit_begin(U, gridDim.x, blockIdx.x);
  const int u_end = unit_begin(U, gridDim.x, blockIdx.x + 1);
  if (u >= u_end) return;

  const int G = Hq / Hkv;
  const int R = G * Nq;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2, wq = wave & 3;
  const int li = lane & 31, lh = lane >> 5;
  const int rt = blockIdx.y * 4 + wq;          // this wavefront's query tile
  const bool rt_ok = rt < row_tiles;           // wave-uniform
  const int mrow = rt * 32 + li;
  const bool row_ok = rt_ok && mrow < R;
  const int node = row_ok ? mrow / G : 0;
  const char* qtile = qall + wq * (32 * kAtRowBytes);
  const int qs_row = (tid & 255) >> 3;  // staging: 8 threads per query row, 32 B each
  const int qs_half = tid >> 8;         // threads 0..255 stage tiles 0 and 1, threads 256..511 tiles 2 and 3

  int b = 0;
  {
    int lo = 0, hi = B - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (pbv(mid) <= u) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }

  while (u < u_end) {
    while (pbv(b + 1) <= u) ++b;
    const int L = seq_lens[b];
    const int n_b = (L + kAtTile - 1) / kAtTile;
    const int rel = u - pbv(b);
    const int hk = __builtin_amdgcn_readfirstlane(rel / n_b);
    const int t0 = rel - hk * n_b;
    const int t1 = min(n_b, t0 + (u_end - u));
    const int slot = blockIdx.x + b * Hkv + hk;
    u += t1 - t0;
    const int start = t0 * kAtTile;
    const int prefix = L - Nq;
    const int ntile = t1 - t0;
    const int nstep = (ntile + 1) >> 1;
    const int last_tile_start = ((L - 1) >> 5) << 5;
    const int32_t* bt = block_table + (size_t)b * max_pages;
    const float scale_log2 = kFp8KV ? scale_log2_q * k_scale[hk] : scale_log2_q;

    // the four query tiles -> LDS
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int ti = qs_half * 2 + i;
      const int m = (blockIdx.y * 4 + ti) * 32 + qs_row;
      const bool ok = m < R;
      const int nd = ok ? m / G : 0, g = ok ? m % G : 0;
      const u32x4_t* qp = (const u32x4_t*)(q + (((size_t)b * Nq + nd) * Hq + hk * G + g) * kAtD);
      const int c0 = (tid & 7) * 2;
      u32x4_t z = {0u, 0u, 0u, 0u};
      const u32x4_t v0 = ok ? qp[c0] : z;
      const u32x4_t v1 = ok ? qp[c0 + 1] : z;
      char* dst = qall + ti * (32 * kAtRowBytes) + qs_row * kAtRowBytes;
      *(u32x4_t*)(dst + ((c0 ^ (qs_row & 15)) * 16)) = v0;
      *(u32x4_t*)(dst + (((c0 + 1) ^ (qs_row & 15)) * 16)) = v1;
    }
    unsigned long long anc;
    if (parents) {
      anc = 0;
      for (int a = node, hops = 0; a >= 0 && hops <= Nq; a = parents[(size_t)b * Nq + a], ++hops) anc |= 1ull << a;
    } else {
      anc = node == 63 ? ~0ull : ((1ull << (node + 1)) - 1);
    }

    // this wavefront's eighth of a step: load instruction `wave` of K and of V, for both tiles of the step
    // (a tile past the end of the sequence re-reads the last one; it is never multiplied)
    auto issue_step = [&](int sidx) {
      char* stage = ring + (sidx % kWideStages) * kWideStageBytes;
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const int j0 = min(start + (2 * sidx + g) * kAtTile, last_tile_start);
        const int pid_a = bt[j0 >> page_shift];
        const int pid_b = bt[min(j0 + 16, L - 1) >> page_shift];
        char* kb = stage + g * (2 * kAtTileBytes);
        issue_rows<false>(kp, kb, wave, j0, L, page_shift, Hkv, hk, pid_a, pid_b, lane);
        issue_rows<true>(vp, kb + kAtTileBytes, wave, j0, L, page_shift, Hkv, hk, pid_a, pid_b, lane);
      }
    };

    SoftmaxState st;
    softmax_state_reset(st);
    __syncthreads();  // query tiles staged; the ring is idle
    QFrags qf;  // this wavefront's query tile as MFMA operand fragments, for the whole run
    load_q_frags(qf, qtile, li, lh);
    auto compute_step = [&](int sidx) {
      const int tt = 2 * sidx + grp;
      if (rt_ok && tt < ntile) {
        const char* kb = ring + (sidx % kWideStages) * kWideStageBytes + grp * (2 * kAtTileBytes);
        const f32x16_t s_acc = tile_scores_qreg(kb, qf, li, lh);
        bf16x8_t pb2[2];
        tile_softmax(s_acc, st, pb2, scale_log2, start + tt * kAtTile, prefix, L, anc, lh);
        tile_pv(kb + kAtTileBytes, pb2, st, lane);
      }
    };
    if constexpr (kFp8KV) {
      struct Step8 { u32x4_t t[2]; };
      const bool is_v = lane >= 32;
      const int r8 = 4 * wave + ((lane & 31) >> 3), f8 = lane & 7;  // token row of the tile, 16-byte chunk of its codes
      const uint8_t* pool8 = (const uint8_t*)(is_v ? vp_ : kp_);
      // steps past the segment's last re-read it: every turn of the loop below has the same loads and waits
      auto fetch = [&](Step8& r, int sidx) {
        const int sc = min(sidx, nstep - 1);
#pragma unroll
        for (int g = 0; g < 2; ++g) {
          const int j0 = min(start + (2 * sc + g) * kAtTile, last_tile_start);
          const int pid_a = bt[j0 >> page_shift];
          const int pid_b = bt[min(j0 + 16, L - 1) >> page_shift];
          const int tok = min(j0 + r8, L - 1);
          const int pid = (tok >> page_shift) == (j0 >> page_shift) ? pid_a : pid_b;
          const size_t off = ((((size_t)pid * Hkv + hk) << page_shift) + (tok & ((1 << page_shift) - 1))) * kAtD + f8 * 16;
          r.t[g] = __builtin_nontemporal_load((const u32x4_t*)(pool8 + off));
        }
      };
      auto spill = [&](const Step8& r, int sidx) {
        char* stage = ring + (sidx % kWideStages) * kWideStageBytes + (is_v ? kAtTileBytes : 0);
        const int key = is_v ? v_key(r8) : (r8 & 15);
#pragma unroll
        for (int g = 0; g < 2; ++g) {
          u32x4_t lo, hi;
          widen16(r.t[g], lo, hi);
          char* row = stage + g * (2 * kAtTileBytes) + r8 * kAtRowBytes;
          *(u32x4_t*)(row + (((2 * f8) ^ key) * 16)) = lo;
          *(u32x4_t*)(row + (((2 * f8 + 1) ^ key) * 16)) = hi;
        }
      };
      // A turn writes stage sidx % 3 while slower wavefronts may still read stage (sidx - 1) % 3; the stage it
      // overwrites was last read two barriers ago.
      auto turn = [&](Step8& r, int sidx, bool live) {
        spill(r, sidx);
        // LDS writes done, then the bare barrier: a fenced one would also wait for the loads in flight
        __builtin_amdgcn_s_waitcnt((7 << 4) | (3 << 14) | 15);  // lgkmcnt(0) only
        __builtin_amdgcn_s_barrier();  // the step's stage is complete from all eight wavefronts
        asm volatile("" ::: "memory");
        fetch(r, sidx + 2);
        if (live) compute_step(sidx);
      };
      Step8 ra, rb;
      fetch(ra, 0);
      __builtin_amdgcn_sched_barrier(0);  // issue order = use order, or the first wait covers both steps
      fetch(rb, 1);
      for (int sidx = 0; sidx < nstep; sidx += 2) {
        turn(ra, sidx, true);
        turn(rb, sidx + 1, sidx + 1 < nstep);  // nstep is the same for the whole workgroup
      }
    } else {
      for (int i = 0; i < kWideStages - 1 && i < nstep; ++i) issue_step(i);
      for (int sidx = 0; sidx < nstep; ++sidx) {
        // steps sidx+1 .. sidx+kWideStages-2 may stay in flight; near the end of the segment fewer were issued
        if (nstep - 1 - sidx >= kWideStages - 2) WAIT_VMCNT(4 * (kWideStages - 2)); else WAIT_VMCNT(0);
        __builtin_amdgcn_s_barrier();  // step complete from all eight wavefronts; the previous step's stage is free
        asm volatile("" ::: "memory");
        if (sidx + kWideStages - 1 < nstep) issue_step(sidx + kWideStages - 1);
        compute_step(sidx);
        asm volatile("" ::: "memory");
      }
    }

    pin_accumulators(st);
    // each wavefront writes the partial of its own query tile and tile parity
    const float l_row = st.l_half + __shfl_xor(st.l_half, 32, kWave);
    if (row_ok) {
      const size_t prow = (((size_t)slot * 2 + grp) * row_tiles + rt) * 32 + li;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4_t o = {st.o[db][4 * g], st.o[db][4 * g + 1], st.o[db][4 * g + 2], st.o[db][4 * g + 3]};
          if constexpr (kFp8KV) o *= v_scale[hk];
          *(f32x4_t*)(part_o + prow * kAtD + 32 * db + 8 * g + 4 * lh) = o;
        }
      if (lh == 0) {
        part_ml[prow * 2 + 0] = st.m_run * (1.0f / kLog2e);  // natural-log units (-inf if nothing was visible)
        part_ml[prow * 2 + 1] = l_row;
      }
    }
    __syncthreads();  // the query tiles and the ring are about to be rewritten
  }
}

// Merge the partials of one output row (request b, node n, query head hq): the segments of its
// (request, KV head) pair sit in slots w + pair for the workgroups w whose unit range meets the pair's.
// Thirty-two threads per row (four output columns each), eight rows per workgroup: the merge is a short chain
// of dependent loads, so what counts is how many rows a compute unit has in flight.
constexpr int kCombineRows = 8;
__global__ __launch_bounds__(32 * kCombineRows) void attn_mfma_combine(const float* __restrict__ part_o,
                                                                       const float* __restrict__ part_ml,
                                                                       const int32_t* __restrict__ seq_lens,
                                                                       const int32_t* __restrict__ PB,
                                                                       bf16_t* __restrict__ out, int B, int Nq, int Hq,
                                                                       int Hkv, int wgs, int row_tiles, int groups,
                                                                       unsigned n_rows, float* __restrict__ lse_out) {
  const size_t row = (size_t)blockIdx.x * kCombineRows + (threadIdx.x >> 5);  // (b*Nq + n)*Hq + hq
  if (row >= n_rows) return;
  const int hq = (int)(row % Hq);
  const int n = (int)((row / Hq) % Nq);
  const int b = (int)(row / ((size_t)Hq * Nq));
  const int G = Hq / Hkv;
  const int hk = hq / G;
  const int mrow = n * G + hq % G;
  const int rt = mrow >> 5, li = mrow & 31;
  const int n_b = (seq_lens[b] + kAtTile - 1) / kAtTile;
  const int u0 = PB[b] + hk * n_b, u1 = u0 + n_b;
  // (a sequence of length 0 has no unit and no partial: w1 < w0, nothing is merged and the row comes out as zeros)
  const int w0 = n_b > 0 ? unit_owner(PB[B], wgs, u0) : 0, w1 = n_b > 0 ? unit_owner(PB[B], wgs, u1 - 1) : -1;
  const int pair = b * Hkv + hk;
  const int d4 = threadIdx.x & 31;  // columns 4 d4 .. 4 d4 + 3
  // online merge, four partials' loads in flight at a time; partial p of the pair is segment
  // (w0 + p / groups), tile parity p % groups
  float M = -INFINITY, den = 0.f;
  f32x4_t num = {0.f, 0.f, 0.f, 0.f};
  const int np = (w1 - w0 + 1) * groups;
  for (int p0 = 0; p0 < np; p0 += 4) {
    float ms[4], ls[4];
    f32x4_t os[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int pp = p0 + i < np ? p0 + i : 0;
      const bool ok = p0 + i < np;
      const size_t sl = (size_t)(w0 + pp / groups + pair) * groups + pp % groups;
      const size_t prow = (sl * row_tiles + rt) * 32 + li;
      const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
      ms[i] = ok ? part_ml[prow * 2] : -INFINITY;
      ls[i] = ok ? part_ml[prow * 2 + 1] : 0.f;
      os[i] = ok ? *(const f32x4_t*)(part_o + prow * kAtD + 4 * d4) : z;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (ms[i] == -INFINITY) continue;
      const float nm = fmaxf(M, ms[i]);
      const float fo = M == -INFINITY ? 0.f : __expf(M - nm);
      const float fn = __expf(ms[i] - nm);
      num = num * fo + os[i] * fn;
      den = den * fo + fn * ls[i];
      M = nm;
    }
  }
  if (lse_out && d4 == 0) lse_out[row] = den > 0.f ? M + __logf(den) : -INFINITY;
  typedef __attribute__((ext_vector_type(4))) unsigned short u16x4_t;
  u16x4_t o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = f32_to_bf16(den > 0.f ? num[e] / den : 0.f);
  *(u16x4_t*)(out + row * kAtD + 4 * d4) = o;
}

bool attn_mfma_supported(const AttnLaunch& a) {
  return a.bf16 && a.D == kAtD && a.page >= 16 && (a.page & (a.page - 1)) == 0;
}

constexpr int kWideWorkgroups = 256;  // one per compute unit

hipError_t launch_attn_mfma(const AttnLaunch& a, hipStream_t st) {
  const int R = a.Hq / a.Hkv * a.Nq;
  const int row_tiles = (R + 31) / 32;
  const bool local_plan = a.B <= kLocalPlanMax;
  hipError_t e;
  if (!local_plan) {
    e = launch_attn_plan(a.seq_lens, a.B, a.Hkv, a.plan_pb, st);
    if (e != hipSuccess) return e;
  }
  const int shift = __builtin_ctz(a.page);
  const float sc = a.scale * kLog2e;
  int wgs;
  if (row_tiles == 1) {
    wgs = kAttnWorkgroups;
    dim3 grid(wgs, 1);
#define AURORA_LAUNCH_NARROW(LOCAL, FP8)                                                                            \
  hipLaunchKernelGGL((attn_mfma_kernel<LOCAL, FP8>), grid, dim3(kAtThreads), 0, st, (const bf16_t*)a.q, a.k, a.v,    \
                     a.k_scale, a.v_scale, a.block_table, a.seq_lens, a.parents, a.plan_pb, a.part_o, a.part_ml, a.B, \
                     a.Nq, a.Hq, a.Hkv, shift, a.max_pages, sc)
    if (local_plan) {
      if (a.kv_fp8) AURORA_LAUNCH_NARROW(true, true); else AURORA_LAUNCH_NARROW(true, false);
    } else {
      if (a.kv_fp8) AURORA_LAUNCH_NARROW(false, true); else AURORA_LAUNCH_NARROW(false, false);
    }
#undef AURORA_LAUNCH_NARROW
  } else {
    wgs = kWideWorkgroups;
    dim3 grid(wgs, (row_tiles + 3) / 4);
#define AURORA_LAUNCH_WIDE(LOCAL, FP8)                                                                             \
  do {                                                                                                              \
    static LdsAttrOnce attr;                                                                                        \
    e = attr.ensure((const void*)attn_mfma_wide_kernel<LOCAL, FP8>, kWideLdsBytes);                                 \
    if (e != hipSuccess) return e;                                                                                  \
    hipLaunchKernelGGL((attn_mfma_wide_kernel<LOCAL, FP8>), grid, dim3(kWideThreads), kWideLdsBytes, st,            \
                       (const bf16_t*)a.q, a.k, a.v, a.k_scale, a.v_scale, a.block_table, a.seq_lens, a.parents,    \
                       a.plan_pb, a.part_o, a.part_ml, a.B, a.Nq, a.Hq, a.Hkv, shift, a.max_pages, row_tiles, sc);  \
  } while (0)
    if (local_plan) {
      if (a.kv_fp8) AURORA_LAUNCH_WIDE(true, true); else AURORA_LAUNCH_WIDE(true, false);
    } else {
      if (a.kv_fp8) AURORA_LAUNCH_WIDE(false, true); else AURORA_LAUNCH_WIDE(false, false);
    }
#undef AURORA_LAUNCH_WIDE
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const unsigned rows = (unsigned)((size_t)a.B * a.Nq * a.Hq);
  hipLaunchKernelGGL(attn_mfma_combine, dim3((rows + kCombineRows - 1) / kCombineRows), dim3(32 * kCombineRows), 0, st,
                     a.part_o, a.part_ml, a.seq_lens, a.plan_pb, (bf16_t*)a.out, a.B, a.Nq, a.Hq, a.Hkv, wgs, row_tiles,
                     row_tiles == 1 ? 1 : 2, rows, a.lse_out);
  return hipGetLastError();
}

}  // namespace aurora
