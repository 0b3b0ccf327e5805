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
// Three small kernels: class counts, one workgroup per row (three passes over the row's 4 * Vd bytes, which
// stay in L2: maximum, sum of exponentials, gradient), and a fixed-order fp64 reduction of the row values.
#include "launch.hpp"

namespace aurora {

constexpr int kLossThreads = 1024;
constexpr int kLossWaves = kLossThreads / kWave;

__device__ __forceinline__ float block_max(float v, float* s_red) {
  v = wave_max(v);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();  // s_red may still be read from the previous reduction
  if (lane == 0) s_red[wv] = v;
  __syncthreads();
  float r = s_red[0];
#pragma unroll
  for (int i = 1; i < kLossWaves; ++i) r = fmaxf(r, s_red[i]);
  return r;
}

__device__ __forceinline__ double block_sum(double v, double* s_red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) s_red[wv] = v;
  __syncthreads();
  double r = 0.0;
#pragma unroll
  for (int i = 0; i < kLossWaves; ++i) r += s_red[i];  // fixed order
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

__global__ __launch_bounds__(kLossThreads) void loss_rows_kernel(LossLaunch P) {
  __shared__ float s_redf[kLossWaves];
  __shared__ double s_redd[kLossWaves];
  const int m = blockIdx.x, tid = threadIdx.x;
  const int Vd = P.Vd, K = P.K;
  const int cls = P.traj[m];
  const float* z = P.draft_logits + (size_t)m * Vd;

  // ---- the row's target distribution: thread t holds kept entry t --------------------------------------
  const int k_eff = (cls == 2 && P.discard_k > 0) ? min(P.discard_k, K) : K;
  int id = -1;
  float lt = -INFINITY;
  if (tid < k_eff) {
    id = P.topk_ids[(size_t)m * K + tid];
    lt = __uint_as_float((uint32_t)P.topk_logits[(size_t)m * K + tid] << 16);
  }
  const bool kept = id >= 0 && id < Vd && lt > -INFINITY;
  const float zt_at = kept ? z[id] : 0.f;  // the drafter's logit of this thread's token
  const float tmax = block_max(kept ? lt : -INFINITY, s_redf);
  const bool any = tmax > -INFINITY;  // a row without a kept target logit contributes nothing
  const double tsum = block_sum(kept ? (double)__expf(lt - tmax) : 0.0, s_redd);
  const double lse_t = (double)tmax + log(tsum);

  // ---- the drafter's logsumexp over its whole vocabulary ---------------------------------------------------
  const bool vec_ok = (Vd & 3) == 0 && ((uintptr_t)P.draft_logits & 15) == 0;
  float zmax = -INFINITY;
  if (vec_ok) {
    const float4* z4 = (const float4*)z;
    for (int i = tid; i < Vd / 4; i += kLossThreads) {
      const float4 x = z4[i];
      zmax = fmaxf(zmax, fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w)));
    }
  } else {
    for (int v = tid; v < Vd; v += kLossThreads) zmax = fmaxf(zmax, z[v]);
  }
  zmax = block_max(zmax, s_redf);
  double zsum = 0.0;
  if (vec_ok) {
    const float4* z4 = (const float4*)z;
    for (int i = tid; i < Vd / 4; i += kLossThreads) {
      const float4 x = z4[i];
      zsum += (double)__expf(x.x - zmax) + (double)__expf(x.y - zmax) + (double)__expf(x.z - zmax) +
              (double)__expf(x.w - zmax);
    }
  } else {
    for (int v = tid; v < Vd; v += kLossThreads) zsum += (double)__expf(z[v] - zmax);
  }
  zsum = block_sum(zsum, s_redd);
  const double lse_d = (double)zmax + log(zsum);
  const float lse_df = (float)lse_d;

  // ---- KL(p_target || p_draft) of the row --------------------------------------------------------------------
  const double logpt = (double)lt - lse_t;
  const float pt = kept ? __expf((float)logpt) : 0.f;
  const double term = kept ? (double)pt * (logpt - ((double)zt_at - lse_d)) : 0.0;
  const double kl = block_sum(term, s_redd);
  if (tid == 0) P.row_kl[m] = any ? (float)kl : 0.f;

  // ---- gradient: w (p_draft - p_target) ------------------------------------------------------------------------
  if (!P.grad) return;
  const float n_acc = P.loss_out[3], n_disc = P.loss_out[4];
  float w = 0.f;
  if (any && cls == 1) w = 1.f / n_acc;
  if (any && cls == 2) w = P.lambda / n_disc;
  float* g = P.grad + (size_t)m * Vd;
  const bool gvec = vec_ok && ((uintptr_t)P.grad & 15) == 0;
  if (gvec) {
    const float4* z4 = (const float4*)z;
    float4* g4 = (float4*)g;
    for (int i = tid; i < Vd / 4; i += kLossThreads) {
      const float4 x = z4[i];
      float4 o;
      o.x = w * __expf(x.x - lse_df);
      o.y = w * __expf(x.y - lse_df);
      o.z = w * __expf(x.z - lse_df);
      o.w = w * __expf(x.w - lse_df);
      g4[i] = o;
    }
  } else {
    for (int v = tid; v < Vd; v += kLossThreads) g[v] = w * __expf(z[v] - lse_df);
  }
  __syncthreads();  // the kept tokens' entries are rewritten by other threads than those that wrote them above
  if (kept) g[id] = w * (__expf(zt_at - lse_df) - pt);
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

int loss_max_k() { return kLossThreads; }

hipError_t launch_draft_loss(const LossLaunch& P, hipStream_t st) {
  hipLaunchKernelGGL(loss_count_kernel, dim3(1), dim3(kLossThreads), 0, st, P.traj, P.M, P.loss_out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (P.M > 0) {
    hipLaunchKernelGGL(loss_rows_kernel, dim3(P.M), dim3(kLossThreads), 0, st, P);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(kLossThreads), 0, st, P.row_kl, P.traj, P.M, P.lambda, P.loss_out);
  return hipGetLastError();
}

}  // namespace aurora
