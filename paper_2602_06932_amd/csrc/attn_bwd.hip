// Backward pass of the chunk / tree attention (paper section 3.1: the speculative tree - accepted and
// rejected branches - goes through one batched forward and backward pass under the tree's mask).
//
//   p_ij = exp(scale <q_i, k_j> - lse_i),  delta_i = <dO_i, O_i>,  dP_ij = <dO_i, v_j>,  dS_ij = p_ij (dP_ij - delta_i)
//   dq_i = scale sum_j dS_ij k_j      dk_j = scale sum_i dS_ij q_i      dv_j = sum_i p_ij dO_i
//
// The forward pass comes first (the library's own kernels; its merge kernel also writes lse), or its saved
// output and lse are handed in.  Then one
// workgroup per (request, KV head) pair walks the pair's KV positions in blocks of 64 with fp32 vector
// arithmetic: in the token-major half a thread owns a quarter of one token's K and V row, forms the scores and
// dP against the group's query rows (kept in LDS, 32 at a time), and accumulates its share of dk_j and dv_j over
// the rows; dS goes to LDS, and in the row-major half a thread owns 16 columns of one query row and adds the
// block's dS_ij k_j to dq_i.  Every K / V element is read once per 32 query rows; all sums run in a fixed order.
// This is the kernel for the shapes the matrix-core kernels (attn_bwd_mfma.hip) do not take: vector fp32 arithmetic.
#include "launch.hpp"

namespace aurora {

constexpr int kBwThreads = 256;
constexpr int kBwTok = 64;    // KV positions per block: four threads per position
constexpr int kBwRows = 32;   // query rows per pass over the pair's positions

// delta[row] = <dout[row], out[row]> ; one wavefront per row
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(const T* __restrict__ out, const T* __restrict__ dout,
                                                             float* __restrict__ delta, int rows, int D) {
  const int row = blockIdx.x * 4 + threadIdx.x / kWave, lane = threadIdx.x % kWave;
  if (row >= rows) return;
  float s = 0.f;
  for (int d = lane; d < D; d += kWave) s = fmaf(to_f32<T>(out[(size_t)row * D + d]), to_f32<T>(dout[(size_t)row * D + d]), s);
  s = wave_sum(s);
  if (lane == 0) delta[row] = s;
}

template <typename T, int kQuarter /* D / 4 */>
__global__ __launch_bounds__(kBwThreads) void attn_bwd_kernel(
    const T* __restrict__ q, const T* __restrict__ kp, const T* __restrict__ vp, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ parents, const T* __restrict__ dout,
    const float* __restrict__ lse, const float* __restrict__ delta, float* __restrict__ dq, float* __restrict__ dk,
    float* __restrict__ dv, int Nq, int Hq, int Hkv, int page, int max_pages, float scale) {
  constexpr int D = 4 * kQuarter;
  constexpr int kCols = D / 8;  // columns of a query row a thread owns in the row-major half
  // more than 64 KB of LDS in all: carved out of the dynamic allocation
  extern __shared__ __attribute__((aligned(16))) char bw_lds[];
  float(*s_q)[D] = (float(*)[D])bw_lds;
  float(*s_do)[D] = (float(*)[D])(bw_lds + sizeof(float) * kBwRows * D);
  float(*s_k)[D + 4] = (float(*)[D + 4])(bw_lds + sizeof(float) * 2 * kBwRows * D);
  float(*s_ds)[kBwTok + 1] = (float(*)[kBwTok + 1])(bw_lds + sizeof(float) * (2 * kBwRows * D + kBwTok * (D + 4)));
  __shared__ float s_lse[kBwRows], s_delta[kBwRows];
  __shared__ unsigned long long s_anc[kBwRows];
  const int b = blockIdx.x / Hkv, hk = blockIdx.x % Hkv;
  const int tid = threadIdx.x;
  const int G = Hq / Hkv, R = G * Nq;
  const int L = seq_lens[b], prefix = L - Nq;
  const int tl = tid >> 2, qd = tid & 3;       // token-major half: position within the block, quarter of its row
  const int ri = tid >> 3, dc = tid & 7;       // row-major half: query row of the chunk, column group
  const int32_t* bt = block_table + (size_t)b * max_pages;

  for (int r0 = 0; r0 < R; r0 += kBwRows) {
    const int nrows = min(kBwRows, R - r0);
    __syncthreads();  // the previous pass is done with the row tables
    // ---- the pass's query rows: group row m = n * G + g  <->  (node n, query head hk * G + g) ----------
    for (int idx = tid; idx < kBwRows * D; idx += kBwThreads) {
      const int i = idx / D, d = idx % D;
      float qv = 0.f, gv = 0.f;
      if (i < nrows) {
        const int m = r0 + i, n = m / G, g = m % G;
        const size_t at = (((size_t)b * Nq + n) * Hq + hk * G + g) * D + d;
        qv = to_f32<T>(q[at]);
        gv = to_f32<T>(dout[at]);
      }
      s_q[i][d] = qv;
      s_do[i][d] = gv;
    }
    if (tid < kBwRows) {
      float l = 0.f, de = 0.f;
      unsigned long long anc = 0;
      if (tid < nrows) {
        const int m = r0 + tid, n = m / G, g = m % G;
        const size_t row = ((size_t)b * Nq + n) * Hq + hk * G + g;
        l = lse[row];
        de = delta[row];
        if (parents) {
          for (int a = n, hops = 0; a >= 0 && hops <= Nq; a = parents[(size_t)b * Nq + a], ++hops) anc |= 1ull << a;
        } else {
          anc = n == 63 ? ~0ull : ((1ull << (n + 1)) - 1);
        }
      }
      s_lse[tid] = l;
      s_delta[tid] = de;
      s_anc[tid] = anc;
    }
    float dq_acc[kCols];
#pragma unroll
    for (int e = 0; e < kCols; ++e) dq_acc[e] = 0.f;
    __syncthreads();

    for (int j0 = 0; j0 < L; j0 += kBwTok) {
      // ---- token-major half ------------------------------------------------------------------------------
      const int j = j0 + tl;
      const bool valid = j < L;
      float kr[kQuarter], vr[kQuarter], dkr[kQuarter], dvr[kQuarter];
      size_t at = 0;
      if (valid) {
        const int pg = bt[j / page];
        at = (((size_t)pg * Hkv + hk) * page + j % page) * D + qd * kQuarter;
      }
#pragma unroll
      for (int d = 0; d < kQuarter; ++d) {
        kr[d] = valid ? to_f32<T>(kp[at + d]) : 0.f;
        vr[d] = valid ? to_f32<T>(vp[at + d]) : 0.f;
        dkr[d] = 0.f;
        dvr[d] = 0.f;
        s_k[tl][qd * kQuarter + d] = kr[d];
      }
      for (int i = 0; i < nrows; ++i) {
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int d = 0; d < kQuarter; ++d) {
          s = fmaf(kr[d], s_q[i][qd * kQuarter + d], s);
          dp = fmaf(vr[d], s_do[i][qd * kQuarter + d], dp);
        }
        s += __shfl_xor(s, 1, kWave);
        s += __shfl_xor(s, 2, kWave);
        dp += __shfl_xor(dp, 1, kWave);
        dp += __shfl_xor(dp, 2, kWave);
        const bool seen = valid && (j < prefix || ((s_anc[i] >> (j - prefix)) & 1ull));
        const float p = seen ? __expf(s * scale - s_lse[i]) : 0.f;
        const float ds = p * (dp - s_delta[i]);
        if (qd == 0) s_ds[i][tl] = ds;
#pragma unroll
        for (int d = 0; d < kQuarter; ++d) {
          dkr[d] = fmaf(ds, s_q[i][qd * kQuarter + d], dkr[d]);
          dvr[d] = fmaf(p, s_do[i][qd * kQuarter + d], dvr[d]);
        }
      }
      if (valid) {
#pragma unroll
        for (int d = 0; d < kQuarter; ++d) {
          // later passes (more than 32 query rows per KV head) add to what the earlier ones wrote
          const float k0 = r0 > 0 ? dk[at + d] : 0.f, v0 = r0 > 0 ? dv[at + d] : 0.f;
          dk[at + d] = k0 + dkr[d] * scale;
          dv[at + d] = v0 + dvr[d];
        }
      }
      __syncthreads();
      // ---- row-major half: dq_i += sum_j dS_ij k_j over the block ------------------------------------------
      if (ri < nrows) {
        const int nt = min(kBwTok, L - j0);
        for (int t = 0; t < nt; ++t) {
          const float ds = s_ds[ri][t];
#pragma unroll
          for (int e = 0; e < kCols; ++e) dq_acc[e] = fmaf(ds, s_k[t][dc * kCols + e], dq_acc[e]);
        }
      }
      __syncthreads();
    }
    if (ri < nrows) {
      const int m = r0 + ri, n = m / G, g = m % G;
      const size_t at = (((size_t)b * Nq + n) * Hq + hk * G + g) * D + dc * kCols;
#pragma unroll
      for (int e = 0; e < kCols; ++e) dq[at + e] = dq_acc[e] * scale;
    }
  }
}

template <typename T>
static hipError_t launch_bwd_t(const AttnBwdLaunch& a, hipStream_t st) {
  if (attn_bwd_mfma_supported(a)) return launch_attn_backward_mfma(a, st);  // forms delta itself
  const int rows = a.B * a.Nq * a.Hq;
  hipLaunchKernelGGL(attn_bwd_delta_kernel<T>, dim3((rows + 3) / 4), dim3(256), 0, st, (const T*)a.out, (const T*)a.dout,
                     a.delta, rows, a.D);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid(a.B * a.Hkv);
  const int lds = (int)sizeof(float) * (2 * kBwRows * a.D + kBwTok * (a.D + 4) + kBwRows * (kBwTok + 1));
  static LdsAttrOnce attr128, attr64;
  e = a.D == 128 ? attr128.ensure((const void*)attn_bwd_kernel<T, 32>, lds) : attr64.ensure((const void*)attn_bwd_kernel<T, 16>, lds);
  if (e != hipSuccess) return e;
  if (a.D == 128)
    hipLaunchKernelGGL((attn_bwd_kernel<T, 32>), grid, dim3(kBwThreads), lds, st, (const T*)a.q, (const T*)a.k, (const T*)a.v,
                       a.block_table, a.seq_lens, a.parents, (const T*)a.dout, a.lse, a.delta, a.dq, a.dk, a.dv, a.Nq, a.Hq,
                       a.Hkv, a.page, a.max_pages, a.scale);
  else
    hipLaunchKernelGGL((attn_bwd_kernel<T, 16>), grid, dim3(kBwThreads), lds, st, (const T*)a.q, (const T*)a.k, (const T*)a.v,
                       a.block_table, a.seq_lens, a.parents, (const T*)a.dout, a.lse, a.delta, a.dq, a.dk, a.dv, a.Nq, a.Hq,
                       a.Hkv, a.page, a.max_pages, a.scale);
  return hipGetLastError();
}

hipError_t launch_attn_backward(const AttnBwdLaunch& a, hipStream_t st) {
  return a.bf16 ? launch_bwd_t<bf16_t>(a, st) : launch_bwd_t<float>(a, st);
}

}  // namespace aurora
