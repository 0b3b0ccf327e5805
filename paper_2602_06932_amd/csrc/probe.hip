// Calibration probe: what a dense bf16 contraction can reach on this device, stripped of everything specific to
// the LM head.  One workgroup per compute unit slot runs the many-row LM-head kernel's inner structure - eight
// wavefronts, 2 x 4 accumulator tiles of v_mfma_f32_32x32x16_bf16 each, four steps per stage, 64 KB of operands per
// stage - with its parts switched on one at a time:
//   mode 0  matrix cores only, operands fixed in registers
//   mode 1  + the operand reads from LDS (six 16-byte reads per lane and step, the LM head's swizzled layout)
//   mode 2  + the LDS-direct loads that refill the stage (row slivers of 128 bytes at an 8 KB pitch, L2
//             resident: no HBM traffic), issued by the multiplying wavefronts as in that kernel: through a buffer
//             descriptor, two after every step
//   mode 3  the loads alone
//   mode 4  the W sweep alone: every workgroup streams its own 256 rows x 8 KB of `operands` once from HBM through a
//           three-stage LDS ring in the LM head's tile shape (row slivers of 128 bytes per stage), four loading
//           wavefronts, nothing multiplied - the ceiling of the vocabulary sweep's access pattern
// Nothing waits for data and the results are discarded: the probe measures rates, and how they depend on the VALUES
// multiplied (the caller fills `operands`: random LM-head-like values, or zeros).  The time of a matrix-core
// kernel on this part depends on them - the signature of a power limit - and the numbers this gives are the
// ceiling the LM-head kernels are priced against beside the published peak.
#include "launch.hpp"
#include "lmhead_tile.hpp"

namespace aurora {

constexpr int kPrThreads = 512;
constexpr int kPrLds = 65536;
constexpr size_t kPrOperandBytes = (size_t)4 * 512 * 8192;  // four tiles of 512 rows at an 8 KB pitch

__device__ __forceinline__ void probe_dma16(const void* g, unsigned l) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(l), "v"(g) : "memory");
}
// the same through a buffer descriptor: descriptor base + 32-bit lane offset + scalar offset, range-checked by the hardware
typedef __attribute__((ext_vector_type(4))) int probe_i32x4_t;
__device__ __forceinline__ void probe_bdma16(probe_i32x4_t rsrc, unsigned voff, unsigned soff, unsigned l) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(l), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}

template <int MODE>
__global__ __launch_bounds__(kPrThreads, 1) void probe_kernel(const char* __restrict__ base, int stages, float* __restrict__ sink) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned lds0 = (unsigned)(uintptr_t)lds;
  const char* tile = base + (size_t)(blockIdx.x & 3) * (512 * 8192);
  f32x16_t acc[2][4];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;
  bf16x8_t wa[2], hb[4];
  // register operands of mode 0: the first bytes of the caller's buffer, so that they are random or zero with it
  {
    const bf16x8_t* p = (const bf16x8_t*)(base + (size_t)lane * 128);
    wa[0] = p[0]; wa[1] = p[1];
#pragma unroll
    for (int t = 0; t < 4; ++t) hb[t] = p[2 + t];
  }
  if (MODE >= 1) {
    // fill the LDS stage once (plain stores), so that mode 1 multiplies the caller's values too
    for (int i = threadIdx.x; i < kPrLds / 16; i += kPrThreads)
      ((f32x4_t*)lds)[i] = ((const f32x4_t*)tile)[i];
    __syncthreads();
  }
  const int li = lane & 31, lh = lane >> 5;
  // descriptor over this workgroup's 512-row tile; wavefront w, instruction j: rows 64 w + 8 j .. + 7, 128 bytes at k offset s
  probe_i32x4_t rsrc;
  {
    const uint64_t a = (uint64_t)(uintptr_t)tile;
    rsrc[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    rsrc[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((a >> 32) & 0xffffu));
    rsrc[2] = 512 * 8192;
    rsrc[3] = 0x00020000;
  }
  const unsigned voff = (unsigned)((wave * 64 + (lane >> 3)) * 8192 + (lane & 7) * 16);
  auto refill = [&](int s, int j) {
    probe_bdma16(rsrc, voff, (unsigned)(j * 8 * 8192 + (s & 63) * 128), lds0 + wave * 8192 + j * 1024);
  };
  for (int s = 0; s < stages; ++s) {
    if (MODE == 2) LM_WAIT_VMCNT(8);  // at most one stage's loads of this wavefront in flight
    if (MODE != 3) {
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        if (MODE >= 1) {
          const int chunk = ((2 * st + lh) ^ ((li >> 1) & 7)) * 16;
#pragma unroll
          for (int a = 0; a < 2; ++a) wa[a] = *(const bf16x8_t*)(lds + ((wave & 3) * 64 + a * 32 + li) * 128 + chunk);
#pragma unroll
          for (int t = 0; t < 4; ++t) hb[t] = *(const bf16x8_t*)(lds + 32768 + (((wave >> 2) * 4 + t) * 32 + li) * 128 + chunk);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int a = 0; a < 2; ++a) acc[a][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[a], hb[t], acc[a][t], 0, 0, 0);
        if (MODE == 2) {  // two of the stage's eight loads after every step
          __builtin_amdgcn_sched_barrier(0);
          refill(s, 2 * st);
          refill(s, 2 * st + 1);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (MODE == 3) {
      LM_WAIT_VMCNT(8);
#pragma unroll
      for (int j = 0; j < 8; ++j) refill(s, j);
    }
    __builtin_amdgcn_s_barrier();
  }
  LM_WAIT_VMCNT(0);  // every load has landed before the workgroup's LDS is given back
  float x = 0.f;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) x += acc[a][t][r];
  if (x == 12345.678f) sink[0] = x;  // keeps the products alive; practically never true
}

// mode 4: workgroup i streams rows 256 i .. 256 i + 255 (8 KB each); the walk over k starts at a staggered offset
__global__ __launch_bounds__(256, 1) void probe_stream_kernel(const char* __restrict__ base, int n_tiles) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned lds0 = (unsigned)(uintptr_t)lds;
  const int vt = blockIdx.x;
  if (vt >= n_tiles) return;
  constexpr int nk = 64;
  const int k0 = (vt * 13) % nk;
  const char* src[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
    src[j] = base + ((size_t)vt * 256 + wave * 64 + j * 8 + (lane >> 3)) * 8192 + (lane & 7) * 16;
  auto issue = [&](int s) {
    const int k = (k0 + s) % nk;
#pragma unroll
    for (int j = 0; j < 8; ++j) probe_dma16(src[j] + k * 128, lds0 + (s % 3) * 32768 + wave * 8192 + j * 1024);
  };
  issue(0); issue(1); issue(2);
  for (int s = 0; s < nk; ++s) {
    const int rem = nk - 1 - s;  // stages after this one
    if (rem >= 2) LM_WAIT_VMCNT(16); else if (rem == 1) LM_WAIT_VMCNT(8); else LM_WAIT_VMCNT(0);
    __builtin_amdgcn_s_barrier();  // stage s has landed for every wavefront; its slot may be refilled
    if (s + 3 < nk) issue(s + 3);
  }
}

size_t probe_operand_bytes() { return kPrOperandBytes; }

hipError_t launch_probe_stream(const void* operands, size_t operand_bytes, hipStream_t st) {
  static LdsAttrOnce attr;
  if (hipError_t e = attr.ensure((const void*)probe_stream_kernel, 3 * 32768); e != hipSuccess) return e;
  const int n_tiles = (int)(operand_bytes / ((size_t)256 * 8192));
  if (n_tiles < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(probe_stream_kernel, dim3(n_tiles), dim3(256), 3 * 32768, st, (const char*)operands, n_tiles);
  return hipGetLastError();
}

hipError_t launch_probe(int mode, const void* operands, int workgroups, int stages, float* sink, hipStream_t st) {
  static LdsAttrOnce attr[4];
  const void* fn[4] = {(const void*)probe_kernel<0>, (const void*)probe_kernel<1>, (const void*)probe_kernel<2>,
                       (const void*)probe_kernel<3>};
  if (mode < 0 || mode > 3) return hipErrorInvalidValue;
  if (hipError_t e = attr[mode].ensure(fn[mode], kPrLds); e != hipSuccess) return e;
  const char* b = (const char*)operands;
  switch (mode) {
    case 0: hipLaunchKernelGGL(probe_kernel<0>, dim3(workgroups), dim3(kPrThreads), kPrLds, st, b, stages, sink); break;
    case 1: hipLaunchKernelGGL(probe_kernel<1>, dim3(workgroups), dim3(kPrThreads), kPrLds, st, b, stages, sink); break;
    case 2: hipLaunchKernelGGL(probe_kernel<2>, dim3(workgroups), dim3(kPrThreads), kPrLds, st, b, stages, sink); break;
    default: hipLaunchKernelGGL(probe_kernel<3>, dim3(workgroups), dim3(kPrThreads), kPrLds, st, b, stages, sink); break;
  }
  return hipGetLastError();
}

}  // namespace aurora
