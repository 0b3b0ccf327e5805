// Pieces shared by the matrix-core attention kernels (forward and backward): operand types, the direct
// global->LDS tile loads, the work split into 32-token tiles, and the per-tile products.
#pragma once
#include "common.hpp"

namespace aurora {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) unsigned short u16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

constexpr int kAtThreads = 256;
constexpr int kAtD = 128;
constexpr int kAtTile = 32;                       // tokens per tile
constexpr int kAtRowBytes = kAtD * 2;             // 256
constexpr int kAtTileBytes = kAtTile * kAtRowBytes;  // 8 KB
constexpr float kLog2e = 1.4426950408889634f;

// Direct global->LDS load of 16 bytes per lane: lane i's data lands at lds_base + 16*i.  Written as
// inline assembly so that the compiler's own wait-count bookkeeping does not see it (it would make
// every later LDS read wait for ALL such loads); the explicit s_waitcnt vmcnt(n) below do the
// waiting.  Waits the compiler inserts for its own vector memory operations can only become more
// conservative, because the counter retires in order.
__device__ __forceinline__ void load_to_lds_16(const void* gptr, const void* lds_base) {
  const unsigned base = (unsigned)(uintptr_t)lds_base;  // LDS pointers are 32-bit offsets
  // m0 holds the LDS base; one wait state is required between writing m0 and the load that reads it.
  // Nothing else in this kernel uses m0.
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(__builtin_amdgcn_readfirstlane(base)),
               "v"(gptr)
               : "memory");
}
#define WAIT_VMCNT(n)                                                                              \
  do {                                                                                             \
    __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8));            \
    asm volatile("" ::: "memory");                                                                 \
  } while (0)

__device__ __forceinline__ int units_per_wg(int U, int wgs) {
  const int c = (U + wgs - 1) / wgs;
  return (c + 3) & ~3;  // a multiple of four tiles: the four wavefronts of a workgroup stay balanced
}

// The forward sweeps deal the U units to the workgroups as evenly as they divide: contiguous runs of U / wgs units, one
// more for the first U % wgs workgroups - every resident workgroup has work and no compute unit holds more than its share.
__device__ __forceinline__ int unit_begin(int U, int wgs, int w) {
  const int q = U / wgs, r = U % wgs;
  return w * q + (w < r ? w : r);
}
// the workgroup whose run holds unit u (0 <= u < U)
__device__ __forceinline__ int unit_owner(int U, int wgs, int u) {
  const int q = U / wgs, r = U % wgs;
  const int edge = r * (q + 1);  // units below it sit in runs of q + 1
  return u < edge ? u / (q + 1) : r + (u - edge) / q;  // u >= edge implies q >= 1
}

// ---- pieces shared by the two sweep kernels -----------------------------------------------------------
struct SoftmaxState {
  f32x16_t o[4];   // O^T accumulators: block db, register r <-> column 32 db + 8(r/4) + 4*lh + r%4
  float m_run;     // running max of the scaled scores of this lane's query row, log2 units
  float l_half;    // running sum over the tokens this half-lane owns
};

__device__ __forceinline__ void softmax_state_reset(SoftmaxState& st) {
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) st.o[db][r] = 0.f;
  st.m_run = -INFINITY;
  st.l_half = 0.f;
}

// Placed between a tile loop and the code that consumes the accumulators piecewise: the accumulators leave the
// loop as four whole 16-register values.  Without it the compiler keeps a second, scattered copy of all 64
// registers for the later piecewise reads and refreshes it after the MFMAs of EVERY tile (64 moves per tile,
// and 36 more registers).
__device__ __forceinline__ void pin_accumulators(SoftmaxState& st) {
  asm volatile("" : "+v"(st.o[0]), "+v"(st.o[1]), "+v"(st.o[2]), "+v"(st.o[3]));
}

// S^T = K Q^T for one 32-token tile: tokens are MFMA rows, the 32 query rows MFMA columns
__device__ __forceinline__ f32x16_t tile_scores(const char* kbuf, const char* qtile, int li, int lh) {
  f32x16_t s_acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) s_acc[r] = 0.f;
  const int sw = li & 15;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const int coff = li * kAtRowBytes + (((2 * s + lh) ^ sw) * 16);
    const bf16x8_t ka = *(const bf16x8_t*)(kbuf + coff);
    const bf16x8_t qa = *(const bf16x8_t*)(qtile + coff);
    s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qa, s_acc, 0, 0, 0);
  }
  return s_acc;
}

// The same product with the query tile's operand fragments already in registers (32 VGPRs, loaded once per run of
// tiles by load_q_frags): a third less LDS traffic per tile.
struct QFrags { bf16x8_t f[8]; };
__device__ __forceinline__ void load_q_frags(QFrags& qf, const char* qtile, int li, int lh) {
  const int sw = li & 15;
#pragma unroll
  for (int s = 0; s < 8; ++s) qf.f[s] = *(const bf16x8_t*)(qtile + li * kAtRowBytes + (((2 * s + lh) ^ sw) * 16));
}
__device__ __forceinline__ f32x16_t tile_scores_qreg(const char* kbuf, const QFrags& qf, int li, int lh) {
  f32x16_t s_acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) s_acc[r] = 0.f;
  const int sw = li & 15;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const bf16x8_t ka = *(const bf16x8_t*)(kbuf + li * kAtRowBytes + (((2 * s + lh) ^ sw) * 16));
    s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf.f[s], s_acc, 0, 0, 0);
  }
  return s_acc;
}

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;

// The running reference of a row's scaled scores only moves when a tile's maximum exceeds it by more
// than 2^kLazyBits: exp'd scores stay below 2^kLazyBits (exact in fp32, same relative rounding in
// bf16), and on most tiles no accumulator needs rescaling.
constexpr float kLazyBits = 8.0f;

// LDS position of 16-byte chunk c of V-tile row r: chunk ^ v_key(r).  Four consecutive token rows land in
// four different 64-byte groups, which is what the transposing reads below need to be conflict-free.
__device__ __forceinline__ int v_key(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// online softmax of the tile (register r holds token j0 + 8(r/4) + 4*lh + r%4 of this lane's row);
// returns the exp'd scores rounded to bf16 (hardware round-to-nearest-even), already laid out as the
// B operand of the P.V product
__device__ __forceinline__ void tile_softmax(f32x16_t s_acc, SoftmaxState& st, bf16x8_t pb2[2], float scale_log2, int j0,
                                             int prefix, int L, unsigned long long anc, int lh) {
  const bool need_mask = j0 + kAtTile > prefix;
  float tmax = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float x = s_acc[r];
    if (need_mask) {
      const int j = j0 + 8 * (r >> 2) + 4 * lh + (r & 3);
      const bool seen = j < prefix || (j < L && ((anc >> (j - prefix)) & 1ull));
      x = seen ? x : -INFINITY;
      s_acc[r] = x;
    }
    tmax = fmaxf(tmax, x);
  }
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave)) * scale_log2;  // scale > 0: the max commutes with it
  if (__any(tmax > st.m_run + kLazyBits)) {  // wave-uniform branch
    const float m_new = tmax > st.m_run + kLazyBits ? tmax : st.m_run;
    const float alpha = __builtin_amdgcn_exp2f(st.m_run - (m_new == -INFINITY ? 0.f : m_new));
    st.m_run = m_new;
    st.l_half *= alpha;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
  }
  const float neg_m = st.m_run == -INFINITY ? 0.f : -st.m_run;
  float psum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; r += 2) {
    const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[r], scale_log2, neg_m));
    const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[r + 1], scale_log2, neg_m));
    psum += p0 + p1;
    const f32x2_t pp = {p0, p1};
    const bf16x2_t pk = __builtin_convertvector(pp, bf16x2_t);
    pb2[r >> 3][r & 7] = pk[0];
    pb2[r >> 3][(r & 7) + 1] = pk[1];
  }
  st.l_half += psum;
}

// O^T += V^T P^T.  The A operand needs, per lane, one column of V for eight tokens: two transposing LDS
// reads (ds_read_b64_tr_b16: within 16 lanes, lane i receives element i%4 of the 8-byte vectors
// addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4) fetch four tokens each.  Lane k of a 16-lane group
// therefore addresses token row tb + k/4, columns 4(k%4)..4(k%4)+3 of the group's 16 columns.
__device__ __forceinline__ void tile_pv(const char* vbuf, const bf16x8_t pb2[2], SoftmaxState& st, int lane) {
  const int lh = lane >> 5, k = lane & 15, kq = k >> 2;
  const int g1 = (lane >> 4) & 1;  // which 16 of the 32 columns of a block
  // byte address = row*256 + ((chunk ^ v_key(row)) * 16) + (col % 8) * 2 with
  //   row = 16u + 8e + 4lh + kq,  col = 32db + 16g1 + 4(k%4)   (see v_key; derivation in comments below)
  // v_key(row) = (kq << 2) | ((2e + lh) & 3);  chunk = 4db + 2g1 + (k%4)/2
  const int lo0 = ((2 * g1 + ((k & 3) >> 1)) ^ (lh & 3)) * 16;
  const int lo1 = ((2 * g1 + ((k & 3) >> 1)) ^ ((2 + lh) & 3)) * 16;
  const int common = lh * 1024 + kq * 256 + (k & 1) * 8 + kq * 64;
  const int base0 = common + lo0;          // e = 0
  const int base1 = common + lo1 + 2048;   // e = 1 (token rows + 8)
#pragma unroll
  for (int uu = 0; uu < 2; ++uu) {
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      typedef __attribute__((address_space(3))) s16x4_t* lds_v4;
      const s16x4_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(vbuf + uu * 4096 + (base0 ^ (db * 64))));
      const s16x4_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(vbuf + uu * 4096 + (base1 ^ (db * 64))));
      const u16x8_t va = {(unsigned short)r0[0], (unsigned short)r0[1], (unsigned short)r0[2], (unsigned short)r0[3],
                          (unsigned short)r1[0], (unsigned short)r1[1], (unsigned short)r1[2], (unsigned short)r1[3]};
      st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, va), pb2[uu], st.o[db], 0, 0, 0);
    }
  }
}

// one of the 8 load instructions of a K or V tile: token rows 4j .. 4j+3 of the tile starting at j0
template <bool kIsV>
__device__ __forceinline__ void issue_rows(const bf16_t* pool, char* buf, int j, int j0, int L, int page_shift, int Hkv,
                                           int hk, int pid_a, int pid_b, int lane) {
  const int lrow = lane >> 4, lpos = lane & 15;
  const int pa = j0 >> page_shift;
  const int tok = min(j0 + 4 * j + lrow, L - 1);
  const int pid = (tok >> page_shift) == pa ? pid_a : pid_b;
  const int r = 4 * j + lrow;
  const int chunk = lpos ^ (kIsV ? v_key(r) : (r & 15));
  const bf16_t* src =
      pool + ((((size_t)pid * Hkv + hk) << page_shift) + (tok & ((1 << page_shift) - 1))) * kAtD + chunk * 8;
  load_to_lds_16(src, buf + j * 1024);
}

// ---- KV cache held as E4M3 codes (one byte per element, one scale per KV head) ----------------------------
// A 32-token tile of codes is 32 rows x 128 B.  It is loaded into registers (four 16-byte loads per lane for
// K, four for V: 8 lanes cover a token row, so an instruction covers 8 rows = 1 KB of a page), widened
// exactly to bf16 in registers and written to the wavefront's LDS tile in the layout the LDS-direct loads
// of the bf16 path produce, so that the score and P.V code is shared.  The scales are applied outside the
// products: K's folds into the softmax scale, V's multiplies the segment's partial O.
struct Tile8 { u32x4_t k[4], v[4]; };

// row of a V load instruction's lane group g: consecutive groups take rows four apart, whose swizzle keys
// have different parity, so that the sixteen lanes an LDS write instruction serves at a time hit distinct banks
__device__ __forceinline__ int v_row_of_group(int g) { return ((g & 1) << 2) | (g >> 1); }

__device__ __forceinline__ void load_tile8(Tile8& t, const uint8_t* __restrict__ kp, const uint8_t* __restrict__ vp, int j0,
                                           int L, int page_shift, int Hkv, int hk, int pid_a, int pid_b, int lane) {
  const int pa = j0 >> page_shift;
  const int g = lane >> 3, f = lane & 7;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int tok_k = min(j0 + 8 * i + g, L - 1);
    const int tok_v = min(j0 + 8 * i + v_row_of_group(g), L - 1);
    const int pid_k = (tok_k >> page_shift) == pa ? pid_a : pid_b;
    const int pid_v = (tok_v >> page_shift) == pa ? pid_a : pid_b;
    const size_t ok = ((((size_t)pid_k * Hkv + hk) << page_shift) + (tok_k & ((1 << page_shift) - 1))) * kAtD + f * 16;
    const size_t ov = ((((size_t)pid_v * Hkv + hk) << page_shift) + (tok_v & ((1 << page_shift) - 1))) * kAtD + f * 16;
    t.k[i] = __builtin_nontemporal_load((const u32x4_t*)(kp + ok));
    t.v[i] = __builtin_nontemporal_load((const u32x4_t*)(vp + ov));
  }
}

// sixteen E4M3 codes -> sixteen bf16 (exact: 3 mantissa bits and the exponent range fit), as two 16-byte chunks
__device__ __forceinline__ void widen16(const u32x4_t c, u32x4_t& lo, u32x4_t& hi) {
  unsigned int out[8];
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8((int)c[w], false);  // bytes 0, 1
    const f32x2_t b = __builtin_amdgcn_cvt_pk_f32_fp8((int)c[w], true);   // bytes 2, 3
    out[2 * w] = __builtin_bit_cast(unsigned int, __builtin_convertvector(a, bf16x2_t));
    out[2 * w + 1] = __builtin_bit_cast(unsigned int, __builtin_convertvector(b, bf16x2_t));
  }
  lo = u32x4_t{out[0], out[1], out[2], out[3]};
  hi = u32x4_t{out[4], out[5], out[6], out[7]};
}

__device__ __forceinline__ void spill_tile8(const Tile8& t, char* kbuf, char* vbuf, int lane) {
  const int g = lane >> 3, f = lane & 7;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    u32x4_t lo, hi;
    const int rk = 8 * i + g;
    widen16(t.k[i], lo, hi);
    *(u32x4_t*)(kbuf + rk * kAtRowBytes + (((2 * f) ^ (rk & 15)) * 16)) = lo;
    *(u32x4_t*)(kbuf + rk * kAtRowBytes + (((2 * f + 1) ^ (rk & 15)) * 16)) = hi;
    const int rv = 8 * i + v_row_of_group(g);
    widen16(t.v[i], lo, hi);
    *(u32x4_t*)(vbuf + rv * kAtRowBytes + (((2 * f) ^ v_key(rv)) * 16)) = lo;
    *(u32x4_t*)(vbuf + rv * kAtRowBytes + (((2 * f + 1) ^ v_key(rv)) * 16)) = hi;
  }
}

// prefix of tiles per request (see attn_plan_kernel) built by the whole workgroup into s_pb[0..B], B <= 1024
__device__ __forceinline__ void build_prefix(const int32_t* __restrict__ seq_lens, int B, int Hkv, int* s_pb,
                                             int* s_wsum) {
  const int t4 = threadIdx.x * 4;
  int un[4], loc = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    un[i] = t4 + i < B ? ((seq_lens[t4 + i] + kAtTile - 1) / kAtTile) * Hkv : 0;
    loc += un[i];
  }
  int incl = loc;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int y = __shfl_up(incl, o, kWave);
    if ((int)(threadIdx.x & 63) >= o) incl += y;
  }
  if ((threadIdx.x & 63) == 63) s_wsum[threadIdx.x >> 6] = incl;
  __syncthreads();
  int run = incl - loc;
  for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) run += s_wsum[w];
  if (threadIdx.x == 0) s_pb[0] = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    run += un[i];
    if (t4 + i < B) s_pb[t4 + i + 1] = run;
  }
  __syncthreads();
}

constexpr int kLocalPlanMax = 1024;  // up to this many requests every workgroup builds the prefix itself


}  // namespace aurora
