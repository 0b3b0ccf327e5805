// bf16 LM-head projection for many token rows (M > 160: large batches, draft trees), where the
// contraction is bound by the matrix cores rather than by the sweep over W (appendix A.1, eq. 4 of the
// paper: target logits l in R^{T x V}; softmax statistics fused as in the small-M kernel).
//
// One workgroup of 8 wavefronts owns 256 vocabulary rows x 64 NT token rows (NT = 1..4); wavefront (v, m) owns
// 64 vocab rows x 32 NT tokens (2 x NT accumulator tiles of v_mfma_f32_32x32x16_bf16).  The token rows of a call
// are cut into pairs of 32-row tiles and the pairs dealt evenly to the fewest workgroup columns, so a launch uses
// at most two values of NT, one apart (448 rows: 7 pairs = 4 + 3), and no matrix-core work is spent on padding
// beyond the last pair.  Every
// wavefront multiplies; wavefronts 0-3 also load W and 4-7 the token rows, each operand into its own
// LDS ring (W: 3 stages of 32 KB, it comes from HBM; token rows: 2 stages, they come from L2), by direct
// global->LDS loads of 128-byte row segments through a buffer descriptor that covers exactly the tile's rows; a
// stage's loads leave in two halves, a matrix-core step apart, rather than in one burst (a burst stalls the
// matrix cores of the issuing wavefronts' SIMDs).  A stage is 64 hidden elements = 4 MFMA steps; operand
// fragments are double-buffered in registers one step ahead, and the barrier that opens the next
// stage sits before the last step of the current one, so the matrix pipe never waits on it.
// The eight 16-byte chunks of a row segment are XOR-swizzled by (row / 2) mod 8 on the way in, which
// makes the 128-bit operand reads conflict free on the 64-bank LDS.
// kFp8: operands are E4M3 codes with one float32 scale per token row and per vocabulary row (as in the small-M
// kernel): a stage of 128 bytes per row is then 128 hidden elements, multiplied by two K = 64 MFMAs per accumulator
// tile (v_mfma_scale_f32_32x32x64_f8f6f4, unit scales); the scales are applied to the accumulators in the epilogue.
#include "launch.hpp"
#include "lmhead_tile.hpp"

namespace aurora {

constexpr int kBgThreads = 512;
constexpr int kBgRowBytes = 128;                // bytes of a row segment per stage: 64 bf16 or 128 fp8 elements
constexpr int kBgVTile = 256;                   // vocab rows per workgroup (= statistics tile)
constexpr int kBgMTile = 256;                   // token rows per workgroup, at most
constexpr int kBgWBytes = kBgVTile * kBgRowBytes;  // 32 KB: one stage of W rows
constexpr int kBgHBytes = kBgMTile * kBgRowBytes;  // 32 KB: one stage of token rows
constexpr int kBgWStages = 3;
constexpr int kBgHStages = 2;
constexpr int kBgWRing = kBgWStages * kBgWBytes;
constexpr int kBgLdsBytes = kBgWRing + kBgHStages * kBgHBytes;  // 160 KB
constexpr int kBgLoads = 8;                     // global->LDS instructions per wavefront per stage

// Direct global->LDS load of 16 bytes per lane through a buffer descriptor; lane i's data lands at lds_base + 16 i.
// The address is descriptor base + voff (per lane, 32 bits) + soff (scalar); the hardware checks voff + soff against
// the descriptor's byte count (out-of-range lanes read zero and touch nothing).  Written as
// inline assembly so that the compiler does not order every later LDS read behind all such loads;
// the explicit vmcnt waits below do the waiting.  m0 holds the LDS base; one wait state is required
// between writing m0 and the load that reads it.
typedef __attribute__((ext_vector_type(4))) int i32x4_t;
__device__ __forceinline__ void dma16(i32x4_t rsrc, unsigned voff, unsigned soff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}
// Raw buffer descriptor (stride 0) over `bytes` bytes at p; the words are made wave-uniform.
__device__ __forceinline__ i32x4_t bg_rsrc(const void* p, unsigned bytes) {
  const uint64_t a = (uint64_t)(uintptr_t)p;
  i32x4_t r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((a >> 32) & 0xffffu));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;  // 32-bit data format, no swizzle, no index stride
  return r;
}

struct BgArgs {
  const char* hidden;
  const char* w;
  const float* h_scale;
  const float* w_scale;
  float* logits;
  float* pmax;
  float* psum;
  int32_t* parg;
  float* hmax;
  int M, H, V, n_tiles;
  float exp_scale;     // log2(e) / T
  const float* temps;  // per-request T, or NULL
  int Nq;
};

// One workgroup's tile: vocabulary tile vt, token rows m0 .. m0 + 64 NT.
template <bool kFp8, int NT>
__device__ __forceinline__ void bg_tile(const BgArgs& A, char* lds, int vt, int m0) {
  const char* __restrict__ hidden = A.hidden;
  const char* __restrict__ w = A.w;
  const float* __restrict__ h_scale = A.h_scale;
  const float* __restrict__ w_scale = A.w_scale;
  float* __restrict__ logits = A.logits;
  const int M = A.M, H = A.H, V = A.V, n_tiles = A.n_tiles, Nq = A.Nq;
  const float exp_scale = A.exp_scale;
  const float* __restrict__ temps = A.temps;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wvv = wave & 3;   // vocab slice of 64 rows
  const int wm = wave >> 2;   // token half
  const int vbase = vt * kBgVTile;
  const int tb0 = wm * NT;  // first 32-token tile of this wavefront; rows past M are loaded clamped and never stored
  constexpr int kEsz = kFp8 ? 1 : 2;  // bytes per operand element
  const int nk = H * kEsz / kBgRowBytes;
  const unsigned lds0 = (unsigned)(uintptr_t)lds;  // LDS pointers are 32-bit offsets

  // ---- loader role: 64 rows of one operand per wavefront and stage.  A wavefront's vmcnt queue holds one
  // operand only, so the deeper W ring is not held up behind token-row loads.
  // A W loader brings 64 vocabulary rows per stage (8 instructions), a token-row loader 16 NT rows (2 NT).
  const bool w_loader = wave < 4;
  const int depth = w_loader ? kBgWStages : kBgHStages;
  constexpr int kHLoads = 2 * NT;
  const int lrow = lane >> 3, lslot = lane & 7;
  const int row0 = (w_loader ? 64 : 8 * kHLoads) * (wave & 3);  // first row of the wavefront's share, within the tile
  // the descriptor covers exactly the tile's rows that exist; rows past the end are loaded clamped and never stored
  const int rows_here = w_loader ? (V - vbase < kBgVTile ? V - vbase : kBgVTile) : (M - m0 < 64 * NT ? M - m0 : 64 * NT);
  const size_t row_bytes = (size_t)H * kEsz;
  const i32x4_t rsrc = bg_rsrc(w_loader ? w + (size_t)vbase * row_bytes : hidden + (size_t)m0 * row_bytes,
                               (unsigned)(rows_here * row_bytes));
  unsigned voff[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    int r = row0 + 8 * j + lrow;
    const int chunk = lslot ^ ((r >> 1) & 7);
    r = r < rows_here ? r : rows_here - 1;
    voff[j] = (unsigned)(r * row_bytes + chunk * 16);
  }
  const unsigned ring0 = lds0 + (w_loader ? 0 : kBgWRing) + row0 * kBgRowBytes;
  // A stage's loads are cut into four parts (a W loader: two instructions each; a token-row loader: NT each in the first two
  // parts), so that they can be placed between the matrix-core work instead of leaving in one burst.
  auto issue_part = [&](int ks, int slot, int part) {
    const unsigned base = ring0 + slot * kBgWBytes;
    const unsigned koff = (unsigned)(ks * kBgRowBytes);
    if (w_loader) {
#pragma unroll
      for (int j = 0; j < 2; ++j) dma16(rsrc, voff[2 * part + j], koff, base + 8 * (2 * part + j) * kBgRowBytes);
    } else if (part < 2) {
#pragma unroll
      for (int j = 0; j < NT; ++j) dma16(rsrc, voff[NT * part + j], koff, base + 8 * (NT * part + j) * kBgRowBytes);
    }
  };
  auto issue = [&](int ks, int slot) {
#pragma unroll
    for (int part = 0; part < 4; ++part) issue_part(ks, slot, part);
  };

  f32x16_t acc[2][NT];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;

  const int li = lane & 31, lh = lane >> 5;
  const int sw = (li >> 1) & 7;
  const int wrow_off = (wvv * 64 + li) * kBgRowBytes;
  const int hrow_off = kBgWRing + (tb0 * 32 + li) * kBgRowBytes;

  auto load_frag = [&](int wslot, int hslot, int s, bf16x8_t (&wa)[2], bf16x8_t (&hb)[NT]) {
    const int coff = ((2 * s + lh) ^ sw) * 16;
    const char* wb = lds + wslot * kBgWBytes + wrow_off + coff;
    const char* hbp = lds + hslot * kBgHBytes + hrow_off + coff;
#pragma unroll
    for (int a = 0; a < 2; ++a) wa[a] = *(const bf16x8_t*)(wb + a * 32 * kBgRowBytes);
#pragma unroll
    for (int t = 0; t < NT; ++t)
      hb[t] = *(const bf16x8_t*)(hbp + t * 32 * kBgRowBytes);
  };
  auto multiply = [&](const bf16x8_t (&wa)[2], const bf16x8_t (&hb)[NT]) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int a = 0; a < 2; ++a)
        acc[a][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[a], hb[t], acc[a][t], 0, 0, 0);
  };
  // one MFMA (its wait covers only reads issued a step ago), then this step's reads, then the other MFMAs
#define BG_STEP_ORDER()                                  \
  do {                                                   \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   \
    __builtin_amdgcn_sched_group_barrier(0x100, 2 + NT, 0);   \
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * NT - 1, 0);   \
    __builtin_amdgcn_sched_barrier(0);                   \
  } while (0)
  auto wait_younger = [&](int groups) {  // wait until at most `groups` stages' loads of this wavefront are outstanding
    if (groups <= 0) LM_WAIT_VMCNT(0);
    else if (w_loader) {
      if (groups >= 2) LM_WAIT_VMCNT(2 * kBgLoads); else LM_WAIT_VMCNT(kBgLoads);
    } else {
      if (groups >= 2) LM_WAIT_VMCNT(2 * kHLoads); else LM_WAIT_VMCNT(kHLoads);
    }
  };
  static_assert(kBgWStages <= 3 && kBgHStages <= 3, "wait_younger covers at most 2 younger stages");

  for (int s = 0; s < depth && s < nk; ++s) issue(s, s);
  wait_younger(nk - 1 < depth - 1 ? nk - 1 : depth - 1);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  int wslot = 0, hslot = 0;  // ring slots of the stage being multiplied
  int myslot = 0;            // the same for this wavefront's loader ring
  if constexpr (kFp8) {
    // a double step = the lane's 16-byte chunks of two consecutive steps = 32 bytes per operand = one K = 64 MFMA per
    // accumulator tile; one fragment set at a time (a second set spills into the main loop: five times slower)
    typedef __attribute__((ext_vector_type(8))) int i32x8_t;
    typedef __attribute__((ext_vector_type(4))) int i32x4_t;
    // Operands roll through the registers as in the small-M kernel: a second pair of W operands, and a token-row operand
    // is re-read for the next double step right after the two MFMAs that consumed it; the last one's refill is held back
    // to the head of the next double step, so that a loop iteration ends on MFMAs.
    i32x8_t wA[2], wB[2], hf[NT];
    auto ld_w = [&](int slot, int s2, i32x8_t (&wf)[2]) {
      const char* base = lds + slot * kBgWBytes + wrow_off;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int coff = ((2 * (2 * s2 + e) + lh) ^ sw) * 16;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          const i32x4_t v = *(const i32x4_t*)(base + a * 32 * kBgRowBytes + coff);
#pragma unroll
          for (int i = 0; i < 4; ++i) wf[a][4 * e + i] = v[i];
        }
      }
    };
    auto ld_h = [&](int slot, int s2, int t, i32x8_t& f) {
      const char* base = lds + slot * kBgHBytes + hrow_off + t * 32 * kBgRowBytes;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int coff = ((2 * (2 * s2 + e) + lh) ^ sw) * 16;
        const i32x4_t v = *(const i32x4_t*)(base + coff);
#pragma unroll
        for (int i = 0; i < 4; ++i) f[4 * e + i] = v[i];
      }
    };
    auto mul_t = [&](const i32x8_t (&wf)[2], const i32x8_t& f, int t) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
        acc[a][t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[a], f, acc[a][t], 0, 0, 0, 127, 0, 127);
    };
    // first double step of a stage, rolling in its second: two MFMAs; the next W pair's four reads, the two that refill the
    // first token operand and the two held back for the last one of this double step; then two MFMAs and two reads per tile
    auto phase_a = [&](int ws, int hs) {
      ld_w(ws, 1, wB);
      ld_h(hs, 0, NT - 1, hf[NT - 1]);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        mul_t(wA, hf[t], t);
        ld_h(hs, 1, t, hf[t]);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
      for (int t_ = 1; t_ < NT; ++t_) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    // an empty statement that "uses" every accumulator and clobbers memory: the MFMAs before it cannot sink below it
    // (into or past the conditional blocks of the loads), LDS reads cannot cross it
    auto pin_acc = [&]() {
#pragma unroll
      for (int t = 0; t < NT; ++t) asm volatile("" : "+v"(acc[0][t]), "+v"(acc[1][t])::"memory");
    };
    ld_w(0, 0, wA);
#pragma unroll
    for (int t = 0; t < NT; ++t) ld_h(0, 0, t, hf[t]);
    int pend = -1, pslot = 0;  // stage whose second half of the loads is still to be issued, and its slot
    for (int ks = 0; ks + 1 < nk; ++ks) {
      phase_a(wslot, hslot);
      pin_acc();  // the MFMAs above stay above the branches below
      if (pend >= 0) {  // the second half of the loads of stage ks - 1 + depth, between the two double steps
        issue_part(pend, pslot, 2);
        issue_part(pend, pslot, 3);
      }
      __builtin_amdgcn_sched_barrier(0);
      // second double step, rolling in the first of the next stage; the barrier that opens it comes after the first pair
      // of MFMAs, which covers the return of this stage's last reads
      mul_t(wB, hf[0], 0);
      asm volatile("" : "+v"(acc[0][0]), "+v"(acc[1][0])::"memory");
      __builtin_amdgcn_s_waitcnt((7 << 4) | (3 << 14) | 15);  // lgkmcnt(0) only: every read of stage ks is back
      wait_younger(nk - 2 - ks < depth - 2 ? nk - 2 - ks : depth - 2);
      __builtin_amdgcn_s_barrier();  // stage ks+1 visible to all; nobody reads stage ks's slots again
      asm volatile("" ::: "memory");
      pend = ks + depth < nk ? ks + depth : -1;
      pslot = myslot;
      if (pend >= 0) {
        issue_part(pend, pslot, 0);
        issue_part(pend, pslot, 1);
      }
      __builtin_amdgcn_sched_barrier(0);
      myslot = myslot + 1 == depth ? 0 : myslot + 1;
      wslot = wslot + 1 == kBgWStages ? 0 : wslot + 1;
      hslot = hslot + 1 == kBgHStages ? 0 : hslot + 1;
      ld_w(wslot, 0, wA);
      ld_h(hslot, 0, 0, hf[0]);
#pragma unroll
      for (int t = 1; t < NT; ++t) {
        mul_t(wB, hf[t], t);
        if (t < NT - 1) ld_h(hslot, 0, t, hf[t]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
      for (int t_ = 1; t_ < NT; ++t_) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        if (t_ < NT - 1) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // the last stage: nothing left to roll in behind its second double step
    phase_a(wslot, hslot);
#pragma unroll
    for (int t = 0; t < NT; ++t) mul_t(wB, hf[t], t);
    // the epilogue's work stays behind the last MFMAs
#pragma unroll
    for (int t = 0; t < NT; ++t) asm volatile("" : "+v"(acc[0][t]), "+v"(acc[1][t])::"memory");
  } else {
  bf16x8_t wa0[2], hb0[NT], wa1[2], hb1[NT];
  load_frag(0, 0, 0, wa0, hb0);
  // The loads of stage ks + depth leave in two halves: one right after the barrier that frees their slot (below), the
  // other after the first step of the next stage (later than that and the W rows that come from HBM arrive too late for
  // the stage that needs them; all at once and the burst holds up the matrix cores).  All of a stage's loads are out before
  // the next vmcnt wait, so the counts waited for are the same as with one burst.
  int pend = -1, pslot = 0;  // stage whose second half is still to be issued, and its slot
#define BG_HALF(h)                                       \
  do {                                                   \
    if (pend >= 0) {                                     \
      issue_part(pend, pslot, 2 * (h));                  \
      issue_part(pend, pslot, 2 * (h) + 1);              \
    }                                                    \
    __builtin_amdgcn_sched_barrier(0);                   \
  } while (0)
  for (int ks = 0; ks + 1 < nk; ++ks) {
    load_frag(wslot, hslot, 1, wa1, hb1);
    multiply(wa0, hb0);
    BG_STEP_ORDER();
    BG_HALF(1);
    load_frag(wslot, hslot, 2, wa0, hb0);
    multiply(wa1, hb1);
    BG_STEP_ORDER();
    load_frag(wslot, hslot, 3, wa1, hb1);
    multiply(wa0, hb0);
    BG_STEP_ORDER();
    // every read of stage ks by this wavefront has returned before it says so to the others
    __builtin_amdgcn_s_waitcnt((7 << 4) | (3 << 14) | 15);  // lgkmcnt(0) only
    wait_younger(nk - 2 - ks < depth - 2 ? nk - 2 - ks : depth - 2);
    __builtin_amdgcn_s_barrier();  // stage ks+1 visible to all; nobody reads stage ks's slots again
    asm volatile("" ::: "memory");
    pend = ks + depth < nk ? ks + depth : -1;
    pslot = myslot;
    BG_HALF(0);
    myslot = myslot + 1 == depth ? 0 : myslot + 1;
    wslot = wslot + 1 == kBgWStages ? 0 : wslot + 1;
    hslot = hslot + 1 == kBgHStages ? 0 : hslot + 1;
    load_frag(wslot, hslot, 0, wa0, hb0);
    multiply(wa1, hb1);
    BG_STEP_ORDER();
  }
#undef BG_HALF
  load_frag(wslot, hslot, 1, wa1, hb1);
  multiply(wa0, hb0);
  load_frag(wslot, hslot, 2, wa0, hb0);
  multiply(wa1, hb1);
  load_frag(wslot, hslot, 3, wa1, hb1);
  multiply(wa0, hb0);
  multiply(wa1, hb1);
  }
#undef BG_STEP_ORDER
  __syncthreads();  // every wavefront is done with the ring; it becomes epilogue scratch

  // ---- epilogue ---------------------------------------------------------------------------------------
  // wavefront-private 8 KB each for turning the logits tiles, then [4][256] statistics of the four vocab slices
  char* tb = lds + wave * 8192;
  float* st_max = (float*)(lds + 8 * 8192);
  float* st_sum = st_max + 4 * kBgMTile;
  int* st_arg = (int*)(st_sum + 4 * kBgMTile);
  float* st_half = (float*)(st_arg + 4 * kBgMTile);  // [8][256]: maxima of the eight groups of 32 vocab rows
  const int vrow0 = vbase + wvv * 64;
  const bool vec_ok = (V & 3) == 0;
  if constexpr (kFp8) {
    // dequantise: accumulator (vocab row v, token m) times w_scale[v] * h_scale[m]
    float hs[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int m = m0 + (tb0 + t) * 32 + li;
      hs[t] = h_scale[m < M ? m : M - 1];
    }
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        // four consecutive vocabulary rows: 8(r/4) + 4 lh + r%4 for r = 4g .. 4g+3
        const int v = vrow0 + 32 * a + 8 * g + 4 * lh;
        float wsc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) wsc[e] = w_scale[v + e < V ? v + e : V - 1];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[a][t][4 * g + e] *= wsc[e] * hs[t];
      }
  }
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int col0 = (tb0 + t) * 32;
    if (m0 + col0 < M) {  // tiles wholly past the last token row hold nothing
      float mx, sum, half;
      int arg;
      lm_tile_out(acc[0][t], acc[1][t], vrow0, V, m0 + col0, M, lm_row_scale(exp_scale, temps, Nq, m0 + col0 + li, M), tb,
                  logits, vec_ok, lane, mx, sum, arg, half);
      if (lh == 0) {
        st_max[wvv * kBgMTile + col0 + li] = mx;
        st_sum[wvv * kBgMTile + col0 + li] = sum;
        st_arg[wvv * kBgMTile + col0 + li] = arg;
      }
      st_half[(2 * wvv + lh) * kBgMTile + col0 + li] = half;
    }
  }
  __syncthreads();
  if (tid < 64 * NT) {
    const int m = m0 + tid;
    if (m < M) {
      float mx, sum;
      int arg;
      lm_merge_waves(st_max, st_sum, st_arg, kBgMTile, tid, lm_row_scale(exp_scale, temps, Nq, m, M), mx, sum, arg);
      const size_t o = (size_t)m * n_tiles + vt;
      A.pmax[o] = mx;
      A.psum[o] = sum;
      A.parg[o] = arg;
      // the eight group maxima of this tile, 32 contiguous bytes per token row
      f32x4_t h0, h1;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        h0[j] = st_half[j * kBgMTile + tid];
        h1[j] = st_half[(4 + j) * kBgMTile + tid];
      }
      f32x4_t* hd = (f32x4_t*)(A.hmax + o * kLmHalfPerTile);
      hd[0] = h0;
      hd[1] = h1;
    }
  }
}

// Workgroup columns [0, n_a) hold 64 NTA token rows each, the others 64 NTB (NTB = NTA or NTA - 1).
template <bool kFp8, int NTA, int NTB>
__global__ __launch_bounds__(kBgThreads, 1) void lmhead_mfma_big_kernel(BgArgs A, int m_tiles, int n_a) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  The m_tiles token tiles
  // of one vocab tile get ids 8 apart: same XCD, launched together - the W tile comes from HBM once and
  // from L2 for the others.  Every workgroup walks the hidden dimension in the same order: the
  // workgroups resident on one XCD then want the same slices of the token tiles at about the same time
  // and its L2 serves all but the first.
  const int wg = blockIdx.x;
  const int vt = (wg / (8 * m_tiles)) * 8 + (wg & 7);
  const int mt = (wg >> 3) % m_tiles;
  if (vt >= A.n_tiles) return;
  if constexpr (NTA == NTB) {
    bg_tile<kFp8, NTA>(A, lds, vt, mt * 64 * NTA);
  } else {
    if (mt < n_a) bg_tile<kFp8, NTA>(A, lds, vt, mt * 64 * NTA);
    else bg_tile<kFp8, NTB>(A, lds, vt, n_a * 64 * NTA + (mt - n_a) * 64 * NTB);
  }
}

bool lmhead_mfma_big_supported(const AcceptLaunch& a) {
  const int esz = a.fp8 ? 1 : 2;
  return a.plan.rows >= kLmBigFromRows && (a.bf16 || a.fp8) && (a.H * esz) % kBgRowBytes == 0 && a.H * esz >= kBgRowBytes &&
         a.H * esz <= (1 << 20) /* 256 rows of a tile within a 32-bit buffer offset */ && a.V >= 1 &&
         a.plan.stat_tile == kBgVTile;
}

template <bool kFp8, int NTA, int NTB>
static hipError_t launch_big_t(const AcceptLaunch& a, hipStream_t st, int m_tiles, int n_a) {
  static LdsAttrOnce attr;
  if (hipError_t e = attr.ensure((const void*)lmhead_mfma_big_kernel<kFp8, NTA, NTB>, kBgLdsBytes); e != hipSuccess)
    return e;
  BgArgs A = {};
  A.hidden = (const char*)a.hidden; A.w = (const char*)a.lm_head; A.h_scale = a.hidden_scale; A.w_scale = a.lm_scale;
  A.logits = a.logits; A.pmax = a.pmax; A.psum = a.psum; A.parg = a.parg; A.hmax = a.hmax;
  A.M = (int)a.plan.rows; A.H = a.H; A.V = a.V; A.n_tiles = a.plan.n_tiles;
  A.exp_scale = 1.4426950408889634f / (a.temperature > 0.f ? a.temperature : 1.f);
  A.temps = a.temps; A.Nq = a.Nq;
  const int v_tiles = (a.V + kBgVTile - 1) / kBgVTile;
  dim3 grid((v_tiles + 7) / 8 * 8 * m_tiles);
  hipLaunchKernelGGL((lmhead_mfma_big_kernel<kFp8, NTA, NTB>), grid, dim3(kBgThreads), kBgLdsBytes, st, A, m_tiles, n_a);
  return hipGetLastError();
}

// Pairs of 32-row tiles dealt evenly to the fewest workgroup columns of at most four pairs.
void lmhead_mfma_big_geometry(int M, int* m_tiles, int* nt_a, int* nt_b, int* n_a) {
  const int pairs = (M + 63) / 64;
  const int cols = (pairs + 3) / 4;
  const int base = pairs / cols, rem = pairs % cols;
  *m_tiles = cols;
  *nt_a = rem ? base + 1 : base;
  *nt_b = base;
  *n_a = rem ? rem : cols;
}

template <bool kFp8>
static hipError_t launch_big_dt(const AcceptLaunch& a, hipStream_t st) {
  int m_tiles, nta, ntb, n_a;
  lmhead_mfma_big_geometry((int)a.plan.rows, &m_tiles, &nta, &ntb, &n_a);
  // from kLmBigFromRows (six pairs) on, every column holds three or four pairs
  switch (nta * 10 + ntb) {
    case 44: return launch_big_t<kFp8, 4, 4>(a, st, m_tiles, n_a);
    case 43: return launch_big_t<kFp8, 4, 3>(a, st, m_tiles, n_a);
    case 33: return launch_big_t<kFp8, 3, 3>(a, st, m_tiles, n_a);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_lmhead_mfma_big(const AcceptLaunch& a, hipStream_t st) {
  return a.fp8 ? launch_big_dt<true>(a, st) : launch_big_dt<false>(a, st);
}

}  // namespace aurora
