// Generic chunk attention (any head_dim <= 256, any page size, fp32 or bf16 storage - or a KV cache of
// E4M3 codes with one scale per KV head - fp32 arithmetic).  It is the fp32 path of the library and the fallback for bf16 shapes the MFMA
// kernel does not cover.  One workgroup per (split, query head, request x node): scores for
// the split's visible KV positions, a block-wide max / sum, then the weighted value sum; a
// second kernel merges the splits (sections 3.1 and 3.2 of the paper define what is computed:
// the draft positions are verified in one pass, a tree under its ancestor mask).
#include "common.hpp"
#include "launch.hpp"

namespace aurora {

constexpr int kGenThreads = 256;
constexpr int kGenMaxSplit = 4096;

// TKV = T, or e4m3_t with k_scale / v_scale [Hkv]: the scale of the KV head multiplies the scores and
// the weighted value sum (both are linear in it).
template <typename T, typename TKV>
__global__ __launch_bounds__(kGenThreads) void attn_generic_partial(
    const T* __restrict__ q, const TKV* __restrict__ kp, const TKV* __restrict__ vp,
    const float* __restrict__ k_scale, const float* __restrict__ v_scale,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ parents, float* __restrict__ part_o, float* __restrict__ part_ml,
    int Nq, int Hq, int Hkv, int D, int page, int max_pages, int split_len, int max_splits, float scale) {
  __shared__ float q_s[256];
  __shared__ float sc[kGenMaxSplit];
  __shared__ float red[kGenThreads];
  __shared__ unsigned long long anc_s;

  const int split = blockIdx.x, hq = blockIdx.y, bn = blockIdx.z;
  const int b = bn / Nq, n = bn % Nq;
  const int tid = threadIdx.x;
  const int L = seq_lens[b];
  const int start = split * split_len;
  if (start >= L) return;
  const int end = min(L, start + split_len);
  const int prefix = L - Nq;
  const int hk = hq / (Hq / Hkv);
  if (k_scale) scale *= k_scale[hk];
  const float vs = v_scale ? v_scale[hk] : 1.f;

  if (tid == 0) {
    unsigned long long m = 0;
    if (parents) {
      for (int a = n, hops = 0; a >= 0 && hops <= Nq; a = parents[b * Nq + a], ++hops) m |= 1ull << a;
    } else {
      m = n == 63 ? ~0ull : ((1ull << (n + 1)) - 1);
    }
    anc_s = m;
  }
  const size_t qoff = ((size_t)bn * Hq + hq) * D;
  for (int d = tid; d < D; d += kGenThreads) q_s[d] = to_f32<T>(q[qoff + d]);
  __syncthreads();
  const unsigned long long anc = anc_s;

  float lmax = -INFINITY;
  for (int j = start + tid; j < end; j += kGenThreads) {
    const bool seen = j < prefix || ((anc >> (j - prefix)) & 1ull);
    float s = -INFINITY;
    if (seen) {
      const int pg = block_table[(size_t)b * max_pages + j / page];
      const TKV* kr = kp + (((size_t)pg * Hkv + hk) * page + j % page) * D;
      float acc = 0.f;
      for (int d = 0; d < D; ++d) acc = fmaf(q_s[d], to_f32<TKV>(kr[d]), acc);
      s = acc * scale;
    }
    sc[j - start] = s;
    lmax = fmaxf(lmax, s);
  }
  red[tid] = lmax;
  __syncthreads();
  for (int o = kGenThreads / 2; o > 0; o >>= 1) {
    if (tid < o) red[tid] = fmaxf(red[tid], red[tid + o]);
    __syncthreads();
  }
  const float m = red[0];
  __syncthreads();
  float lsum = 0.f;
  for (int j = start + tid; j < end; j += kGenThreads) {
    const float s = sc[j - start];
    const float p = (s == -INFINITY) ? 0.f : __expf(s - m);
    sc[j - start] = p;
    lsum += p;
  }
  red[tid] = lsum;
  __syncthreads();
  for (int o = kGenThreads / 2; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  const float l = red[0];
  __syncthreads();

  // weighted value sum: thread (d, g) adds the positions j == g (mod groups)
  const int groups = kGenThreads / D > 0 ? kGenThreads / D : 1;
  const size_t pidx = ((size_t)bn * Hq + hq) * max_splits + split;
  for (int d0 = 0; d0 < D; d0 += kGenThreads) {
    const int d = d0 + tid % (D < kGenThreads ? D : kGenThreads);
    const int g = tid / D;
    float acc = 0.f;
    if (g < groups && d < D) {
      for (int j = start + g; j < end; j += groups) {
        const float p = sc[j - start];
        if (p != 0.f) {
          const int pg = block_table[(size_t)b * max_pages + j / page];
          acc = fmaf(p, to_f32<TKV>(vp[(((size_t)pg * Hkv + hk) * page + j % page) * D + d]), acc);
        }
      }
    }
    red[tid] = acc;
    __syncthreads();
    if (g == 0 && d < D) {
      float tot = 0.f;
      for (int gg = 0; gg < groups; ++gg) tot += red[gg * D + tid];
      part_o[pidx * D + d] = tot * vs;
    }
    __syncthreads();
  }
  if (tid == 0) {
    part_ml[pidx * 2 + 0] = m;
    part_ml[pidx * 2 + 1] = l;
  }
}

// Merge the per-split partials of one (request, node, query head): out = sum_s e^{m_s-M} O_s / sum_s e^{m_s-M} l_s.
template <typename T>
__global__ void attn_combine(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                             const int32_t* __restrict__ seq_lens, T* __restrict__ out, int Nq, int Hq, int D,
                             int split_len, int max_splits, float* __restrict__ lse_out) {
  const size_t row = blockIdx.x;  // (b*Nq + n)*Hq + hq
  const int b = (int)(row / ((size_t)Nq * Hq));
  const int L = seq_lens[b];
  const int ns = min(max_splits, (L + split_len - 1) / split_len);
  const size_t base = row * max_splits;
  float M = -INFINITY;
  for (int s = 0; s < ns; ++s) M = fmaxf(M, part_ml[(base + s) * 2]);
  if (lse_out && threadIdx.x == 0) {
    float den = 0.f;
    for (int s = 0; s < ns; ++s) {
      const float ms = part_ml[(base + s) * 2];
      if (ms > -INFINITY) den = fmaf(__expf(ms - M), part_ml[(base + s) * 2 + 1], den);
    }
    lse_out[row] = den > 0.f ? M + __logf(den) : -INFINITY;
  }
  for (int d = threadIdx.x; d < D; d += blockDim.x) {
    float num = 0.f, den = 0.f;
    for (int s = 0; s < ns; ++s) {
      const float ms = part_ml[(base + s) * 2];
      const float w = (ms == -INFINITY) ? 0.f : __expf(ms - M);
      num = fmaf(w, part_o[(base + s) * D + d], num);
      den = fmaf(w, part_ml[(base + s) * 2 + 1], den);
    }
    out[row * D + d] = from_f32<T>(den > 0.f ? num / den : 0.f);
  }
}

template <typename T>
static hipError_t launch_generic_t(const AttnLaunch& a, hipStream_t st) {
  dim3 grid(a.plan.max_splits, a.Hq, a.B * a.Nq);
  if (a.kv_fp8)
    hipLaunchKernelGGL((attn_generic_partial<T, e4m3_t>), grid, dim3(kGenThreads), 0, st, (const T*)a.q,
                       (const e4m3_t*)a.k, (const e4m3_t*)a.v, a.k_scale, a.v_scale, a.block_table, a.seq_lens,
                       a.parents, a.part_o, a.part_ml, a.Nq, a.Hq, a.Hkv, a.D, a.page, a.max_pages, a.plan.split_len,
                       a.plan.max_splits, a.scale);
  else
    hipLaunchKernelGGL((attn_generic_partial<T, T>), grid, dim3(kGenThreads), 0, st, (const T*)a.q, (const T*)a.k,
                       (const T*)a.v, (const float*)nullptr, (const float*)nullptr, a.block_table, a.seq_lens,
                       a.parents, a.part_o, a.part_ml, a.Nq, a.Hq, a.Hkv, a.D, a.page, a.max_pages, a.plan.split_len,
                       a.plan.max_splits, a.scale);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_attn_combine(a, st);
}

hipError_t launch_attn_combine(const AttnLaunch& a, hipStream_t st) {
  const unsigned rows = (unsigned)((size_t)a.B * a.Nq * a.Hq);
  if (a.bf16)
    hipLaunchKernelGGL(attn_combine<bf16_t>, dim3(rows), dim3(a.D <= 64 ? 64 : 128), 0, st, a.part_o, a.part_ml,
                       a.seq_lens, (bf16_t*)a.out, a.Nq, a.Hq, a.D, a.plan.split_len, a.plan.max_splits, a.lse_out);
  else
    hipLaunchKernelGGL(attn_combine<float>, dim3(rows), dim3(a.D <= 64 ? 64 : 128), 0, st, a.part_o, a.part_ml,
                       a.seq_lens, (float*)a.out, a.Nq, a.Hq, a.D, a.plan.split_len, a.plan.max_splits, a.lse_out);
  return hipGetLastError();
}

hipError_t launch_attn_generic(const AttnLaunch& a, hipStream_t st) {
  return a.bf16 ? launch_generic_t<bf16_t>(a, st) : launch_generic_t<float>(a, st);
}

}  // namespace aurora
