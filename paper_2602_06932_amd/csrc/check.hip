// Debug check of the device-resident inputs of a verify step.  The kernels of the library trust what
// they are given (page ids, lengths, tree parents, token ids index memory directly); this kernel reads
// the same arrays - only inside their declared shapes - and reports what is out of range, so that a caller
// can find a bad input before it turns into a memory fault.  Not on the hot path.
#include "launch.hpp"

namespace aurora {

// one 256-thread workgroup per request; error bits are OR-ed into flags[0], and for each kind the lowest
// offending request index is kept in flags[1 + bit] (initialised to INT_MAX by the clear kernel)
__global__ __launch_bounds__(256) void check_inputs_kernel(CheckLaunch c) {
  const int b = blockIdx.x, tid = threadIdx.x;
  unsigned bad = 0;
  if (c.seq_lens) {
    const int L = c.seq_lens[b];
    const long long need = ((long long)L + c.page - 1) / c.page;
    const bool len_ok = L >= c.Nq && need <= c.max_pages;
    if (!len_ok) bad |= kCheckSeqLen;
    if (c.block_table && len_ok)
      for (long long i = tid; i < need; i += 256) {
        const int pid = c.block_table[(size_t)b * c.max_pages + i];
        if (pid < 0 || pid >= c.num_pages) bad |= kCheckPageId;
      }
  }
  if (c.parents)
    for (int n = tid; n < c.Nq; n += 256) {
      const int p = c.parents[(size_t)b * c.Nq + n];
      if (n == 0 ? p != -1 : (p < 0 || p >= n)) bad |= kCheckParent;
    }
  if (c.draft_tokens)
    for (int n = 1 + tid; n < c.Nq; n += 256) {
      const int t = c.draft_tokens[(size_t)b * c.Nq + n];
      if (t < 0 || t >= c.V) bad |= kCheckToken;
    }
  if (c.uniforms)
    for (int i = tid; i < 2 * c.Nq; i += 256) {
      const float u = c.uniforms[(size_t)b * c.Nq * 2 + i];
      if (!(u >= 0.f && u < 1.f)) bad |= kCheckUniform;  // NaN fails too
    }
  // fold over the workgroup
  __shared__ unsigned s_bad;
  if (tid == 0) s_bad = 0;
  __syncthreads();
  if (bad) atomicOr(&s_bad, bad);
  __syncthreads();
  if (tid == 0 && s_bad) {
    atomicOr((unsigned*)&c.flags[0], s_bad);
    for (int bit = 0; bit < kCheckKinds; ++bit)
      if (s_bad & (1u << bit)) atomicMin(&c.flags[1 + bit], b);
  }
}

__global__ void check_clear_kernel(int32_t* flags) {
  const int i = threadIdx.x;
  if (i == 0) flags[0] = 0;
  else if (i <= kCheckKinds) flags[i] = 0x7fffffff;
}

hipError_t launch_check_inputs(const CheckLaunch& c, hipStream_t st) {
  hipLaunchKernelGGL(check_clear_kernel, dim3(1), dim3(64), 0, st, c.flags);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || c.B == 0) return e;
  hipLaunchKernelGGL(check_inputs_kernel, dim3(c.B), dim3(256), 0, st, c);
  return hipGetLastError();
}

}  // namespace aurora
