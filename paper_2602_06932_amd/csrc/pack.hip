// Packing of trace records (paper appendix A.1, eq. 4: the inference server ships (h, l, x_in, y_out, R) per
// token; section 3.3: accepted and rejected tokens both carry a training signal).  Rows whose trajectory code
// is 0 were never tested and are dropped; the others are copied, in row order, into dense arrays.
//
//   pack_index_kernel   one workgroup: stable compaction of the row numbers with R != 0 (chunks of 1024 rows,
//                       a ballot / prefix count per wavefront and a running base), and the count
//   pack_rows_kernel    one workgroup per packed position: copies the source row's hidden bytes, kept logits
//                       (ids and values) and scalars; positions past the count leave at once
#include "launch.hpp"

namespace aurora {

constexpr int kPackThreads = 1024;
constexpr int kPackWaves = kPackThreads / kWave;

__global__ __launch_bounds__(kPackThreads) void pack_index_kernel(const int8_t* __restrict__ traj, int M,
                                                                   int32_t* __restrict__ row_index,
                                                                   int32_t* __restrict__ n_out) {
  __shared__ int s_cnt[kPackWaves];
  __shared__ int s_base;
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  if (tid == 0) s_base = 0;
  __syncthreads();
  for (int m0 = 0; m0 < M; m0 += kPackThreads) {
    const int m = m0 + tid;
    const bool keep = m < M && traj[m] != 0;
    const unsigned long long mask = __ballot(keep);
    const int before = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) s_cnt[wv] = __popcll(mask);
    __syncthreads();
    int off = s_base;
    for (int i = 0; i < wv; ++i) off += s_cnt[i];
    if (keep) row_index[off + before] = m;
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
      for (int i = 0; i < kPackWaves; ++i) tot += s_cnt[i];
      s_base += tot;
    }
    __syncthreads();
  }
  if (tid == 0) n_out[0] = s_base;
}

// copies `bytes` from src to dst with the widest loads the three of them allow
__device__ __forceinline__ void copy_row(const char* __restrict__ src, char* __restrict__ dst, size_t bytes, int tid,
                                         int nthreads) {
  if ((((uintptr_t)src | (uintptr_t)dst | bytes) & 15) == 0) {
    typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
    for (size_t i = tid; i < bytes / 16; i += nthreads) ((u32x4_t*)dst)[i] = ((const u32x4_t*)src)[i];
  } else if ((((uintptr_t)src | (uintptr_t)dst | bytes) & 3) == 0) {
    for (size_t i = tid; i < bytes / 4; i += nthreads) ((uint32_t*)dst)[i] = ((const uint32_t*)src)[i];
  } else {
    for (size_t i = tid; i < bytes; i += nthreads) dst[i] = src[i];
  }
}

__global__ __launch_bounds__(256) void pack_rows_kernel(PackLaunch P) {
  const int p = blockIdx.x, tid = threadIdx.x;
  if (p >= P.n_out[0]) return;
  const size_t m = (size_t)P.row_index[p];
  if (P.h) copy_row((const char*)P.h + m * P.h_bytes, (char*)P.h_out + (size_t)p * P.h_bytes, P.h_bytes, tid, 256);
  if (P.ids) {
    copy_row((const char*)(P.ids + m * P.K), (char*)(P.ids_out + (size_t)p * P.K), (size_t)P.K * 4, tid, 256);
    copy_row((const char*)(P.vals + m * P.K), (char*)(P.vals_out + (size_t)p * P.K), (size_t)P.K * 2, tid, 256);
  }
  if (tid == 0) {
    if (P.x_in) P.x_out[p] = P.x_in[m];
    if (P.y) P.y_packed[p] = P.y[m];
    if (P.traj_out) P.traj_out[p] = P.traj[m];
  }
}

hipError_t launch_trace_pack(const PackLaunch& P, hipStream_t st) {
  hipLaunchKernelGGL(pack_index_kernel, dim3(1), dim3(kPackThreads), 0, st, P.traj, P.M, P.row_index, P.n_out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || P.M == 0) return e;
  hipLaunchKernelGGL(pack_rows_kernel, dim3(P.M), dim3(256), 0, st, P);
  return hipGetLastError();
}

}  // namespace aurora
