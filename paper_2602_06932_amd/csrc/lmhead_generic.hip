// Generic LM-head projection (fp32 FMA, fp32 or bf16 storage) followed by per-tile softmax
// statistics.  It is the fp32 path of the library and the fallback for shapes the MFMA kernel
// does not cover.  logits[m, v] = sum_h hidden[m, h] * W[v, h]  (appendix A.1, eq. 4: l in R^{T x V}).
#include "common.hpp"
#include "launch.hpp"

namespace aurora {

constexpr int kTM = 64, kTN = 64, kTK = 16;

template <typename T>
__global__ __launch_bounds__(256) void lmhead_generic(const T* __restrict__ hidden, const T* __restrict__ w,
                                                      float* __restrict__ logits, int64_t M, int H, int V) {
  __shared__ float As[kTK][kTM + 4];
  __shared__ float Bs[kTK][kTN + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int64_t m0 = (int64_t)blockIdx.y * kTM;
  const int64_t v0 = (int64_t)blockIdx.x * kTN;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < H; k0 += kTK) {
    for (int i = tid; i < kTM * kTK; i += 256) {
      const int r = i / kTK, c = i % kTK;
      const int64_t m = m0 + r;
      const int k = k0 + c;
      As[c][r] = (m < M && k < H) ? to_f32<T>(hidden[m * H + k]) : 0.f;
      const int64_t v = v0 + r;
      Bs[c][r] = (v < V && k < H) ? to_f32<T>(w[v * H + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kTK; ++kk) {
      float a[4], bcol[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bcol[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], bcol[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t v = v0 + tx * 4 + j;
      if (v < V) logits[m * V + v] = acc[i][j];
    }
  }
}

// One workgroup per (vocab tile, row): max, arg-max (lowest index on ties) and
// sum exp((l - max) * inv_t) over the tile's columns.
__global__ __launch_bounds__(256) void row_tile_stats(const float* __restrict__ logits, float* __restrict__ pmax,
                                                      float* __restrict__ psum, int32_t* __restrict__ parg, int V,
                                                      int stat_tile, int n_tiles, float inv_t,
                                                      const float* __restrict__ temps, int Nq) {
  __shared__ float smax[4];
  __shared__ int sarg[4];
  __shared__ float ssum[4];
  const int tile = blockIdx.x;
  const int64_t row = blockIdx.y;
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  const int v0 = tile * stat_tile, v1 = min(V, v0 + stat_tile);
  const float* lr = logits + row * V;
  if (temps) {  // one temperature per request; 0 = greedy, statistics at T = 1
    const float T = temps[row / Nq];
    inv_t = T > 0.f ? 1.f / T : 1.f;
  }
  float mx = -INFINITY;
  int arg = 0x7fffffff;
  for (int v = v0 + tid; v < v1; v += 256) {
    const float x = lr[v];
    if (x > mx) { mx = x; arg = v; }  // ascending v per thread: first occurrence kept
  }
  // wave reduce (max, lowest index among equals)
  for (int o = 32; o > 0; o >>= 1) {
    const float om = __shfl_xor(mx, o, kWave);
    const int oa = __shfl_xor(arg, o, kWave);
    if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
  }
  if (lane == 0) { smax[wv] = mx; sarg[wv] = arg; }
  __syncthreads();
  mx = smax[0]; arg = sarg[0];
  for (int i = 1; i < 4; ++i)
    if (smax[i] > mx || (smax[i] == mx && sarg[i] < arg)) { mx = smax[i]; arg = sarg[i]; }
  float s = 0.f;
  for (int v = v0 + tid; v < v1; v += 256) s += __expf((lr[v] - mx) * inv_t);
  s = wave_sum(s);
  if (lane == 0) ssum[wv] = s;
  __syncthreads();
  if (tid == 0) {
    pmax[row * n_tiles + tile] = mx;
    psum[row * n_tiles + tile] = ssum[0] + ssum[1] + ssum[2] + ssum[3];
    parg[row * n_tiles + tile] = arg;
  }
}

hipError_t launch_lmhead_generic(const AcceptLaunch& a, hipStream_t st) {
  const int64_t M = a.plan.rows;
  dim3 grid((unsigned)((a.V + kTN - 1) / kTN), (unsigned)((M + kTM - 1) / kTM));
  if (a.bf16)
    hipLaunchKernelGGL(lmhead_generic<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)a.hidden,
                       (const bf16_t*)a.lm_head, a.logits, M, a.H, a.V);
  else
    hipLaunchKernelGGL(lmhead_generic<float>, grid, dim3(256), 0, st, (const float*)a.hidden,
                       (const float*)a.lm_head, a.logits, M, a.H, a.V);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const float inv_t = a.temperature > 0.f ? 1.f / a.temperature : 1.f;
  hipLaunchKernelGGL(row_tile_stats, dim3(a.plan.n_tiles, (unsigned)M), dim3(256), 0, st, a.logits, a.pmax, a.psum,
                     a.parg, a.V, a.plan.stat_tile, a.plan.n_tiles, inv_t, a.temps, a.Nq);
  return hipGetLastError();
}

}  // namespace aurora
