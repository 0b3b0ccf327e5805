// bf16 chunk attention on the matrix cores (paper sections 3.1 / 3.2: the Nq draft positions of a
// request - a chain, or a tree under its ancestor mask - are verified in one pass over the cached
// context).  head_dim 128, KV pages of 16 * 2^i tokens.
//
// One workgroup (4 wavefronts) per (request, KV head, KV split, tile of 32 query rows).  The G*Nq
// query rows that share a KV head form the 32-wide N side of v_mfma_f32_32x32x16_bf16, so a KV
// byte is read once for the whole GQA group.  Inside a workgroup the wavefronts are independent:
// wavefront w owns every 4th 32-token tile of the split, with private LDS buffers, a private
// online-softmax state, and no workgroup barrier until the final merge.
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
constexpr int kAtWaveLds = 2 * kAtTileBytes;      // K + V
constexpr float kLog2e = 1.4426950408889634f;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define WAIT_VMCNT(n)                                                                              \
  do {                                                                                             \
    __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8));            \
    asm volatile("" ::: "memory");                                                                 \
  } while (0)

__global__ __launch_bounds__(kAtThreads, 2) void attn_mfma_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kp, const bf16_t* __restrict__ vp,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ parents, float* __restrict__ part_o, float* __restrict__ part_ml, int Nq, int Hq,
    int Hkv, int page_shift, int max_pages, int split_len, int max_splits, int row_tiles, float scale_log2) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * kAtWaveLds];
  __shared__ float s_m[4][32];
  __shared__ float s_l[4][32];

  const int split = blockIdx.x / row_tiles, rt = blockIdx.x % row_tiles;
  const int hk = blockIdx.y, b = blockIdx.z;
  const int L = seq_lens[b];
  const int start = split * split_len;
  if (start >= L) return;
  const int end = min(L, start + split_len);
  const int prefix = L - Nq;
  const int G = Hq / Hkv;
  const int R = G * Nq;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, lh = lane >> 5;
  char* kbuf = lds + wv * kAtWaveLds;
  char* vbuf = kbuf + kAtTileBytes;

  // ---- this lane's query row (MFMA column li): node n, head g -------------------------------------
  const int mrow = rt * 32 + li;
  const bool row_ok = mrow < R;
  const int node = row_ok ? mrow / G : 0;
  const int hq = hk * G + (row_ok ? mrow % G : 0);
  u32x4_t qreg[8];
  {
    const u32x4_t* qp = (const u32x4_t*)(q + (((size_t)b * Nq + node) * Hq + hq) * kAtD);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      u32x4_t z = {0u, 0u, 0u, 0u};
      qreg[s] = row_ok ? qp[2 * s + lh] : z;
    }
  }
  // chunk slots this node may see: itself and its ancestors (chain: every slot up to its own)
  unsigned long long anc;
  if (parents) {
    anc = 0;
    for (int a = node, hops = 0; a >= 0 && hops <= Nq; a = parents[(size_t)b * Nq + a], ++hops) anc |= 1ull << a;
  } else {
    anc = node == 63 ? ~0ull : ((1ull << (node + 1)) - 1);
  }

  const int ntile = (end - start + kAtTile - 1) / kAtTile;
  const int32_t* bt = block_table + (size_t)b * max_pages;

  // ---- tile loads: always exactly 8 instructions of 4 token rows each (the s_waitcnt bookkeeping
  // below counts them).  Rows past the end of the sequence re-read the last valid token; their
  // scores are masked to -inf, so their (finite) values are multiplied by exact zeros.
  const int lrow = lane >> 4;    // token row within a 4-row instruction
  const int lpos = lane & 15;    // 16-byte slot within the row
  const int page_mask = (1 << page_shift) - 1;
  auto issue_tile = [&](const bf16_t* pool, char* buf, int tt) {
    const int j0 = start + tt * kAtTile;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int tok0 = min(j0 + 4 * j, L - 1);  // wave-uniform
      const int tok = min(tok0 + lrow, L - 1);  // same page as tok0
      const int pid = bt[tok0 >> page_shift];
      const int r = 4 * j + lrow;
      const int chunk = lpos ^ (r & 7);
      const bf16_t* src =
          pool + ((((size_t)pid * Hkv + hk) << page_shift) + (tok & page_mask)) * kAtD + chunk * 8;
      __builtin_amdgcn_global_load_lds(GLB_PTR(src), LDS_PTR(buf + j * 1024), 16, 0, 0);
    }
  };

  f32x16_t o_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
  float m_run = -INFINITY;  // running max of scaled scores, log2 units
  float l_half = 0.f;       // running sum over the tokens this half-lane owns

  int tt = wv;
  if (tt < ntile) {
    issue_tile(kp, kbuf, tt);
    issue_tile(vp, vbuf, tt);
  }
  const int sw = li & 7;
  for (; tt < ntile; tt += 4) {
    const bool more = tt + 4 < ntile;
    // ---- S^T = K Q^T ------------------------------------------------------------------------------
    WAIT_VMCNT(8);  // K(t) landed (V(t) may still be in flight)
    f32x16_t s_acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) s_acc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8_t ka = *(const bf16x8_t*)(kbuf + li * kAtRowBytes + (((2 * s + lh) ^ sw) * 16));
      s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, __builtin_bit_cast(bf16x8_t, qreg[s]), s_acc, 0, 0, 0);
    }
    // the K buffer is free once the products above have their operands; the memory clobber keeps
    // the compiler from moving the LDS reads below the overwrite
    asm volatile("" ::: "memory");
    if (more) issue_tile(kp, kbuf, tt + 4);

    // ---- online softmax (register r holds token j0 + 8(r/4) + 4*lh + r%4 of this lane's row) ----
    const int j0 = start + tt * kAtTile;
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
    const float m_new = fmaxf(m_run, tmax);
    const float m_safe = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
    m_run = m_new;
    float psum = 0.f;
    u16x8_t pb[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = __builtin_amdgcn_exp2f(s_acc[r] - m_safe);
      psum += p;
      pb[r >> 3][r & 7] = f32_to_bf16(p);
    }
    l_half = l_half * alpha + psum;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;

    // ---- O^T += V^T P^T ---------------------------------------------------------------------------
    if (more) WAIT_VMCNT(8); else WAIT_VMCNT(0);  // V(t) landed (K(t+1) may be in flight)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        // slot j of this half-lane is token 16u + 8(j/4) + 4*lh + j%4, column d = 32 db + li
        const int d = 32 * db + li;
        u16x8_t va;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int t = 16 * u + 8 * (j >> 2) + 4 * lh + (j & 3);
          va[j] = *(const unsigned short*)(vbuf + t * kAtRowBytes + (((d >> 3) ^ (t & 7)) * 16) + (d & 7) * 2);
        }
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, va),
                                                            __builtin_bit_cast(bf16x8_t, pb[u]), o_acc[db], 0, 0, 0);
      }
    }
    asm volatile("" ::: "memory");
    if (more) issue_tile(vp, vbuf, tt + 4);
  }

  // ---- merge the four wavefronts and write this split's partial (m, l, O) ---------------------------
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
  // each wavefront parks its rescaled O^T in its own 16 KB of LDS as [row li][128 d] floats
  float* obuf = (float*)(lds + wv * kAtWaveLds);
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d = 32 * db + 8 * g + 4 * lh;
      f32x4_t o = {o_acc[db][4 * g] * f_own, o_acc[db][4 * g + 1] * f_own, o_acc[db][4 * g + 2] * f_own,
                   o_acc[db][4 * g + 3] * f_own};
      // rotate the 16-byte slot by the row so that the 32 rows of a column group spread over banks
      *(f32x4_t*)(obuf + li * kAtD + ((d / 4 + li) & 31) * 4) = o;
    }
  __syncthreads();
  // wavefront w sums and stores d-block w (32 columns) of all rows
  if (row_ok) {
    const int db = wv;
    const size_t pidx = (((size_t)b * Nq + node) * Hq + hq) * max_splits + split;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d = 32 * db + 8 * g + 4 * lh;
      f32x4_t sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float* ob = (const float*)(lds + w * kAtWaveLds);
        sum += *(const f32x4_t*)(ob + li * kAtD + ((d / 4 + li) & 31) * 4);
      }
      *(f32x4_t*)(part_o + pidx * kAtD + d) = sum;
    }
    if (wv == 0 && lh == 0) {
      part_ml[pidx * 2 + 0] = M * (1.0f / kLog2e);  // back to natural-log units for the merge kernel
      part_ml[pidx * 2 + 1] = l_tot;
    }
  }
}

bool attn_mfma_supported(const AttnLaunch& a) {
  return a.bf16 && a.D == kAtD && a.page >= 16 && (a.page & (a.page - 1)) == 0 && a.plan.split_len % (4 * kAtTile) == 0 &&
         (((uintptr_t)a.q | (uintptr_t)a.k | (uintptr_t)a.v) & 15) == 0;
}

hipError_t launch_attn_mfma(const AttnLaunch& a, hipStream_t st) {
  const int R = a.Hq / a.Hkv * a.Nq;
  const int row_tiles = (R + 31) / 32;
  dim3 grid(a.plan.max_splits * row_tiles, a.Hkv, a.B);
  hipLaunchKernelGGL(attn_mfma_kernel, grid, dim3(kAtThreads), 0, st, (const bf16_t*)a.q, (const bf16_t*)a.k,
                     (const bf16_t*)a.v, a.block_table, a.seq_lens, a.parents, a.part_o, a.part_ml, a.Nq, a.Hq, a.Hkv,
                     __builtin_ctz(a.page), a.max_pages, a.plan.split_len, a.plan.max_splits, row_tiles, a.scale * kLog2e);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_attn_combine(a, st);
}

}  // namespace aurora
