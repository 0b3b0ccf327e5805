// Shared device/host helpers of the verify-step library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aurora {

constexpr int kWave = 64;
constexpr int kMaxNq = 64;

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round to nearest, ties to even (finite inputs; NaN stays NaN)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }

// One byte of an 8-bit floating-point tensor: OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa
// bits; exponent field 0 is subnormal, no infinities).  Decoded with integer operations here; the
// matrix-core kernels use the hardware conversion.
struct e4m3_t { uint8_t bits; };
__device__ __forceinline__ float e4m3_to_f32(uint8_t c) {
  const uint32_t sign = (uint32_t)(c & 0x80u) << 24;
  const uint32_t e = (c >> 3) & 15u, m = c & 7u;
  if (e == 15u && m == 7u) return __uint_as_float(sign | 0x7fc00000u);  // the format's only NaN
  if (e == 0u) return __uint_as_float(sign | __float_as_uint((float)m * 0.001953125f));  // m * 2^-9
  return __uint_as_float(sign | ((e + 120u) << 23) | (m << 20));
}
template <> __device__ __forceinline__ float to_f32<e4m3_t>(e4m3_t v) { return e4m3_to_f32(v.bits); }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// butterfly reductions over the 64 lanes of a wavefront; every lane gets the result
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ int wave_max(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, kWave));
  return v;
}

// --- launch plans shared by the API layer and the launchers (host) ----------------------
constexpr int kAttnWorkgroups = 512;  // resident workgroups of the MFMA attention kernel (2 per compute unit)

struct AttnPlan {
  int rows_per_group;  // G * Nq query rows that share one KV head
  bool mfma;           // the bf16 MFMA kernel takes this shape
  // generic kernel: fixed-length KV splits
  int split_len;       // KV tokens per split (multiple of 128)
  int max_splits;      // ceil(max_len / split_len)
  // MFMA kernel: one partial per (workgroup, pair) segment
  int slots;           // kAttnWorkgroups + B * Hkv
  int row_tiles;       // ceil(G * Nq / 32)
  size_t pb_off, part_o_off, part_ml_off, bytes;
};

struct AcceptPlan {
  int64_t rows;     // M = B * Nq
  int stat_tile;    // vocab columns per softmax-statistics partial
  int n_tiles;      // ceil(V / stat_tile)
  int slices;       // chain draw: workgroups per request in the vocabulary sweep
  int gmul;         // chain draw: a group is 64 * gmul consecutive tokens
  int ngroups;      // chain draw: ceil(V / (64 * gmul))
  int n_half;       // group maxima per row kept for the top-K emission (0: the LM-head kernel in use writes none)
  size_t hmax_off;
  size_t logits_off, pmax_off, psum_off, parg_off, st_lse_off, st_row_off, st_rej_off, gsum_off, lastpos_off, tree_bar_off, bytes;
};

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Kernels that use more than 64 KB of dynamic LDS need hipFuncSetAttribute once per device (the
// attribute belongs to the device's copy of the function).  One of these per kernel, function-local
// static; the flags only ever go from false to true, so a race between host threads repeats the call.
struct LdsAttrOnce {
  bool done[64] = {};
  hipError_t ensure(const void* fn, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool track = dev >= 0 && dev < 64;
    if (track && done[dev]) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && track) done[dev] = true;
    return e;
  }
};

// Number of compute units of the current device (cached per device).
inline hipError_t device_cu_count(int* out) {
  static int count[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool track = dev >= 0 && dev < 64;
  if (track && count[dev] > 0) { *out = count[dev]; return hipSuccess; }
  int n = 0;
  e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  if (track) count[dev] = n;
  *out = n;
  return hipSuccess;
}

}  // namespace aurora
