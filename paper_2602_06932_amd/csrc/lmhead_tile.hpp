// Pieces shared by the two matrix-core LM-head kernels: operand types, the direct global->LDS load,
// and the epilogue of one 64-vocab x 32-token accumulator pair (softmax statistics of appendix A.1's
// logits l and the fp32 logits store).
#pragma once
#include "common.hpp"

namespace aurora {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14])
#define LM_WAIT_VMCNT(n)                                                                            \
  do {                                                                                             \
    __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8));            \
    asm volatile("" ::: "memory");                                                                 \
  } while (0)

// Accumulator register r of a 32x32 MFMA tile holds row 8(r/4) + 4(lane/32) + r%4, column lane%32.
// a0 / a1 are the tiles of vocab rows vrow0.. and vrow0+32.. for the 32 tokens mrow0.. (column = token).
// Entries past the vocabulary are set to -inf in place.  Returns this token's (max, arg-max, sum of
// exp2((x - max) * exp_scale)) over the 64 vocab rows in every lane of the token's lane pair, in half_max_out the
// largest of the 32 consecutive vocab rows vrow0 + 32 (lane / 32) .., and
// writes the 64 x 32 logits through `tb`, 8 KB of LDS private to the calling wavefront, so that each
// store instruction covers four token rows of 256 contiguous bytes.  LDS operations of one wavefront
// execute in order, so consecutive calls may reuse `tb` without a barrier.
__device__ __forceinline__ void lm_tile_out(f32x16_t& a0, f32x16_t& a1, int vrow0, int V, int mrow0, int M,
                                            float exp_scale, char* tb, float* __restrict__ logits, bool vec_ok, int lane,
                                            float& mx_out, float& sum_out, int& arg_out, float& half_max_out) {
  const int li = lane & 31, lh = lane >> 5;
  float m01[2] = {-INFINITY, -INFINITY};  // this lane's largest entry among vocab rows vrow0 .. +31 and vrow0 + 32 .. +63
  const bool v_whole = vrow0 + 64 <= V;  // wave-uniform: only the vocabulary's last tile has rows to mask
  if (!v_whole) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        f32x16_t& acc = a ? a1 : a0;
        const int v = vrow0 + 32 * a + 8 * (r >> 2) + 4 * lh + (r & 3);
        if (v >= V) acc[r] = -INFINITY;
      }
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const f32x16_t& acc = a ? a1 : a0;
      m01[a] = fmaxf(m01[a], acc[r]);
    }
  float mx = fmaxf(m01[0], m01[1]);
  // largest of 32 consecutive vocab rows (the two lane halves hold interleaved runs of four): lane half 0 keeps the
  // group vrow0 .. +31, lane half 1 the group vrow0 + 32 .. +63
  {
    const float o0 = __shfl_xor(m01[0], 32, kWave), o1 = __shfl_xor(m01[1], 32, kWave);
    half_max_out = lh ? fmaxf(m01[1], o1) : fmaxf(m01[0], o0);
  }
  int arg = 0x7fffffff;
#pragma unroll
  for (int a = 1; a >= 0; --a)
#pragma unroll
    for (int r = 15; r >= 0; --r) {
      const f32x16_t& acc = a ? a1 : a0;
      const int v = vrow0 + 32 * a + 8 * (r >> 2) + 4 * lh + (r & 3);
      arg = (acc[r] == mx) ? v : arg;
    }
  // merge the two lane halves (they hold interleaved groups of 4 rows of the same token)
  const float omx = __shfl_xor(mx, 32, kWave);
  const int oarg = __shfl_xor(arg, 32, kWave);
  if (omx > mx || (omx == mx && oarg < arg)) { mx = omx; arg = oarg; }
  const float mx_safe = mx == -INFINITY ? 0.f : mx;
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f((a0[r] - mx_safe) * exp_scale);
#pragma unroll
  for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f((a1[r] - mx_safe) * exp_scale);
  sum += __shfl_xor(sum, 32, kWave);
  mx_out = mx;
  sum_out = sum;
  arg_out = arg;

  // Logits out.  A lane holds 4 consecutive vocab entries of ONE token, so a direct store would touch 64
  // different rows per instruction; the tile is turned through LDS instead.  16-byte slots are
  // XOR-swizzled by the token row on both sides: no bank conflicts.
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x16_t& acc = a ? a1 : a0;
      const int slot = 8 * a + 2 * g + lh;  // 16-byte slot of vocab 32a + 8g + 4lh within the 64-wide row
      f32x4_t o = {acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
      *(f32x4_t*)(tb + li * 256 + ((slot ^ (li & 15)) * 16)) = o;
    }
  const int srow = lane >> 4, sslot = lane & 15;
  if (vec_ok && v_whole && mrow0 + 32 <= M) {
    // the common case, decided once per wavefront: every row and column of the tile exists - eight plain vector stores
    float* dst = logits + (size_t)(mrow0 + srow) * V + (vrow0 + 4 * sslot);
    const size_t step = (size_t)4 * V;  // four token rows further
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int n = 4 * j + srow;
      const f32x4_t o = *(const f32x4_t*)(tb + n * 256 + ((sslot ^ (n & 15)) * 16));
      __builtin_nontemporal_store(o, (f32x4_t*)(dst + j * step));  // written once, read much later: keep it out of the way of W
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int n = 4 * j + srow;  // token row of the tile
    const f32x4_t o = *(const f32x4_t*)(tb + n * 256 + ((sslot ^ (n & 15)) * 16));
    const int mm = mrow0 + n;
    const int v = vrow0 + 4 * sslot;
    if (mm < M) {
      float* dst = logits + (size_t)mm * V + v;
      if (vec_ok && v + 3 < V) {
        __builtin_nontemporal_store(o, (f32x4_t*)dst);  // written once, read much later: keep it out of the way of W
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (v + e < V) dst[e] = o[e];
      }
    }
  }
}

// exp2 scale log2(e) / T of token row m: the call's scalar, or - with one temperature per request (temps[b],
// b = m / Nq; 0 stands for a greedy request, whose statistics are taken at T = 1) - the request's own.
__device__ __forceinline__ float lm_row_scale(float exp_scale, const float* __restrict__ temps, int Nq, int m, int M) {
  if (!temps) return exp_scale;
  const float T = temps[(m < M ? m : M - 1) / Nq];
  return 1.4426950408889634f / (T > 0.f ? T : 1.f);
}

// Merge of the four wavefronts' statistics of one token (ascending vocab order, so ties keep the lowest
// index).  st_* are laid out [4][stride].
__device__ __forceinline__ void lm_merge_waves(const float* st_max, const float* st_sum, const int* st_arg, int stride,
                                               int col, float exp_scale, float& mx_out, float& sum_out, int& arg_out) {
  float mx = -INFINITY;
  int arg = 0x7fffffff;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float x = st_max[w * stride + col];
    if (x > mx) { mx = x; arg = st_arg[w * stride + col]; }
  }
  float sum = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float x = st_max[w * stride + col];
    if (x > -INFINITY) sum += st_sum[w * stride + col] * __builtin_amdgcn_exp2f((x - mx) * exp_scale);
  }
  mx_out = mx;
  sum_out = sum;
  arg_out = arg;
}

}  // namespace aurora
