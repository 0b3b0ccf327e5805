// Drafter training loss on a batch of trace rows (paper section 3.3, eq. 3):
//
//   L = mean_{accepted rows} KL(p_target || p_draft) + lambda_discard * mean_{discarded rows} KL(p_target || p_draft)
//
// with its gradient with respect to the drafter's logits, w_m (p_draft - p_target).  p_target of a row is
// the softmax over the target logits kept for it (the K largest, appendix A.2; on discarded rows only the
// first discard_top_k of them - the paper's top-k filtering of discarded tokens), p_draft the softmax of
// the drafter's logits over its whole vocabulary.  Row classes are the trajectory codes of the trace
// record (appendix A.1): 1 accepted, 2 discarded, 0 unused.
//
// Three small kernels: class counts, one workgroup per row, and a fixed-order fp64 reduction of the row values.
#include "launch.hpp"

namespace aurora {

constexpr int kLossThreads = 1024;
constexpr int kLossWaves = kLossThreads / kWave;

template <int kWaves = kLossWaves>
__device__ __forceinline__ float block_max(float v, float* s_red) {
  v = wave_max(v);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();  // s_red may still be read from the previous reduction
  if (lane == 0) s_red[wv] = v;
  __syncthreads();
  float r = s_red[0];
#pragma unroll
  for (int i = 1; i < kWaves; ++i) r = fmaxf(r, s_red[i]);
  return r;
}

template <int kWaves = kLossWaves>
__device__ __forceinline__ double block_sum(double v, double* s_red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) s_red[wv] = v;
  __syncthreads();
  double r = 0.0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) r += s_red[i];  // fixed order
  return r;
}

__global__ __launch_bounds__(kLossThreads) void loss_count_kernel(const int8_t* __restrict__ traj, int M,
                                                                   float* __restrict__ loss_out) {
  __shared__ double s_red[kLossWaves];
  double na = 0.0, nd = 0.0;
  for (int m = threadIdx.x; m < M; m += kLossThreads) {
    const int c = traj[m];
    na += c == 1;
    nd += c == 2;
  }
  na = block_sum(na, s_red);
  nd = block_sum(nd, s_red);
  if (threadIdx.x == 0) {
    loss_out[3] = (float)na;
    loss_out[4] = (float)nd;
  }
}

// One workgroup of four wavefronts per row.  kInRegs: the row is 16-byte aligned and at most kRowRegVals values
// long, so every thread keeps its share (up to 32 x 4 values) in registers: the row is read once, each exponential
// is taken once, and the gradient is that exponential times w / sum.  Four-wavefront workgroups at this register
// count put three rows on a compute unit at a time, so one row's loads and stores overlap another's reductions.
// Otherwise three passes over the row (the second and third hit L2).
constexpr int kRowThreads = 256;
constexpr int kRowWaves = kRowThreads / kWave;
constexpr int kRowRounds = 32;
constexpr int kRowRegVals = kRowThreads * 4 * kRowRounds;  // 32768
constexpr int kRowKept = 1024 / kRowThreads;               // kept target logits per thread
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

template <bool kInRegs>
__global__ __launch_bounds__(kRowThreads) void loss_rows_kernel(LossLaunch P) {
  __shared__ float s_redf[kRowWaves];
  __shared__ double s_redd[kRowWaves];
  const int m = blockIdx.x, tid = threadIdx.x;
  const int Vd = P.Vd, K = P.K;
  const float* z = P.draft_logits + (size_t)m * Vd;
  const int n4 = Vd / 4;

  // the row first: its loads are in flight while the target side is worked out
  f32x4_t r[kInRegs ? kRowRounds : 1];
  if constexpr (kInRegs) {
#pragma unroll
    for (int j = 0; j < kRowRounds; ++j) {
      const int i = tid + j * kRowThreads;
      const f32x4_t ninf = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      r[j] = i < n4 ? *((const f32x4_t*)z + i) : ninf;
    }
  }
  const int cls = P.traj[m];

  // ---- the row's target distribution: thread t holds kept entries t, t + 256, ... ------------------------
  const int k_eff = (cls == 2 && P.discard_k > 0) ? min(P.discard_k, K) : K;
  int id[kRowKept];
  float lt[kRowKept], zt_at[kRowKept];
  bool kept[kRowKept];
  float tmax = -INFINITY;
#pragma unroll
  for (int e = 0; e < kRowKept; ++e) {
    const int t = tid + e * kRowThreads;
    id[e] = -1;
    lt[e] = -INFINITY;
    if (t < k_eff) {
      id[e] = P.topk_ids[(size_t)m * K + t];
      lt[e] = __uint_as_float((uint32_t)P.topk_logits[(size_t)m * K + t] << 16);
    }
    kept[e] = id[e] >= 0 && id[e] < Vd && lt[e] > -INFINITY;
    tmax = fmaxf(tmax, kept[e] ? lt[e] : -INFINITY);
  }
#pragma unroll
  for (int e = 0; e < kRowKept; ++e) zt_at[e] = kept[e] ? z[id[e]] : 0.f;  // the drafter's logit of the kept token
  tmax = block_max<kRowWaves>(tmax, s_redf);
  const bool any = tmax > -INFINITY;  // a row without a kept target logit contributes nothing
  double tsum = 0.0;
#pragma unroll
  for (int e = 0; e < kRowKept; ++e) tsum += kept[e] ? (double)__expf(lt[e] - tmax) : 0.0;
  tsum = block_sum<kRowWaves>(tsum, s_redd);
  const double lse_t = (double)tmax + log(tsum);

  // ---- the drafter's logsumexp over its whole vocabulary ---------------------------------------------------
  const bool vec_ok = (Vd & 3) == 0 && ((uintptr_t)P.draft_logits & 15) == 0;
  float zmax = -INFINITY;
  double zsum = 0.0;
  if constexpr (kInRegs) {
#pragma unroll
    for (int j = 0; j < kRowRounds; ++j) zmax = fmaxf(zmax, fmaxf(fmaxf(r[j][0], r[j][1]), fmaxf(r[j][2], r[j][3])));
    zmax = block_max<kRowWaves>(zmax, s_redf);
#pragma unroll
    for (int j = 0; j < kRowRounds; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) r[j][e] = __expf(r[j][e] - zmax);  // exp(-inf) = 0 past the end of the row
      zsum += ((double)r[j][0] + (double)r[j][1]) + ((double)r[j][2] + (double)r[j][3]);
    }
  } else {
    if (vec_ok) {
      const float4* z4 = (const float4*)z;
      for (int i = tid; i < n4; i += kRowThreads) {
        const float4 x = z4[i];
        zmax = fmaxf(zmax, fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w)));
      }
    } else {
      for (int v = tid; v < Vd; v += kRowThreads) zmax = fmaxf(zmax, z[v]);
    }
    zmax = block_max<kRowWaves>(zmax, s_redf);
    if (vec_ok) {
      const float4* z4 = (const float4*)z;
      for (int i = tid; i < n4; i += kRowThreads) {
        const float4 x = z4[i];
        zsum += (double)__expf(x.x - zmax) + (double)__expf(x.y - zmax) + (double)__expf(x.z - zmax) +
                (double)__expf(x.w - zmax);
      }
    } else {
      for (int v = tid; v < Vd; v += kRowThreads) zsum += (double)__expf(z[v] - zmax);
    }
  }
  zsum = block_sum<kRowWaves>(zsum, s_redd);
  const double lse_d = (double)zmax + log(zsum);
  const float lse_df = (float)lse_d;

  // ---- KL(p_target || p_draft) of the row --------------------------------------------------------------------
  float pt[kRowKept];
  double term = 0.0;
#pragma unroll
  for (int e = 0; e < kRowKept; ++e) {
    const double logpt = (double)lt[e] - lse_t;
    pt[e] = kept[e] ? __expf((float)logpt) : 0.f;
    term += kept[e] ? (double)pt[e] * (logpt - ((double)zt_at[e] - lse_d)) : 0.0;
  }
  const double kl = block_sum<kRowWaves>(term, s_redd);
  if (tid == 0) P.row_kl[m] = any ? (float)kl : 0.f;

  // ---- gradient: w (p_draft - p_target) ------------------------------------------------------------------------
  if (!P.grad) return;
  const float n_acc = P.loss_out[3], n_disc = P.loss_out[4];
  float w = 0.f;
  if (any && cls == 1) w = 1.f / n_acc;
  if (any && cls == 2) w = P.lambda / n_disc;
  float* g = P.grad + (size_t)m * Vd;
  if constexpr (kInRegs) {
    const float scale = w * (float)(1.0 / zsum);
#pragma unroll
    for (int j = 0; j < kRowRounds; ++j) {
      const int i = tid + j * kRowThreads;
      if (i < n4) *((f32x4_t*)g + i) = r[j] * scale;
    }
  } else {
    const bool gvec = vec_ok && ((uintptr_t)P.grad & 15) == 0;
    if (gvec) {
      const float4* z4 = (const float4*)z;
      float4* g4 = (float4*)g;
      for (int i = tid; i < n4; i += kRowThreads) {
        const float4 x = z4[i];
        float4 o;
        o.x = w * __expf(x.x - lse_df);
        o.y = w * __expf(x.y - lse_df);
        o.z = w * __expf(x.z - lse_df);
        o.w = w * __expf(x.w - lse_df);
        g4[i] = o;
      }
    } else {
      for (int v = tid; v < Vd; v += kRowThreads) g[v] = w * __expf(z[v] - lse_df);
    }
  }
  __syncthreads();  // the kept tokens' entries are rewritten by other threads than those that wrote them above
#pragma unroll
  for (int e = 0; e < kRowKept; ++e)
    if (kept[e]) g[id[e]] = w * (__expf(zt_at[e] - lse_df) - pt[e]);
}

__global__ __launch_bounds__(kLossThreads) void loss_reduce_kernel(const float* __restrict__ row_kl,
                                                                    const int8_t* __restrict__ traj, int M, float lambda,
                                                                    float* __restrict__ loss_out) {
  __shared__ double s_red[kLossWaves];
  double sa = 0.0, sd = 0.0;
  for (int m = threadIdx.x; m < M; m += kLossThreads) {
    const int c = traj[m];
    const double x = (double)row_kl[m];
    if (c == 1) sa += x;
    if (c == 2) sd += x;
  }
  sa = block_sum(sa, s_red);
  sd = block_sum(sd, s_red);
  if (threadIdx.x == 0) {
    const double na = loss_out[3], nd = loss_out[4];
    const double ma = na > 0 ? sa / na : 0.0, md = nd > 0 ? sd / nd : 0.0;
    loss_out[0] = (float)(ma + (double)lambda * md);
    loss_out[1] = (float)ma;
    loss_out[2] = (float)md;
  }
}

int loss_max_k() { return kRowKept * kRowThreads; }

hipError_t launch_draft_loss(const LossLaunch& P, hipStream_t st) {
  hipLaunchKernelGGL(loss_count_kernel, dim3(1), dim3(kLossThreads), 0, st, P.traj, P.M, P.loss_out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (P.M > 0) {
    const bool in_regs = (P.Vd & 3) == 0 && P.Vd <= kRowRegVals && ((uintptr_t)P.draft_logits & 15) == 0 &&
                         (!P.grad || ((uintptr_t)P.grad & 15) == 0);
    if (in_regs)
      hipLaunchKernelGGL(loss_rows_kernel<true>, dim3(P.M), dim3(kRowThreads), 0, st, P);
    else
      hipLaunchKernelGGL(loss_rows_kernel<false>, dim3(P.M), dim3(kRowThreads), 0, st, P);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(kLossThreads), 0, st, P.row_kl, P.traj, P.M, P.lambda, P.loss_out);
  return hipGetLastError();
}

}  // namespace aurora
