// bf16 LM-head projection for many token rows (M > 160: large batches, draft trees), where the
// contraction is bound by the matrix cores rather than by the sweep over W (appendix A.1, eq. 4 of the
// paper: target logits l in R^{T x V}; softmax statistics fused as in the small-M kernel).
//
// One workgroup of 8 wavefronts owns 256 vocabulary rows x up to 256 token rows; wavefront (v, m) owns
// 64 vocab rows x up to 128 tokens (2 x 4 accumulator tiles of v_mfma_f32_32x32x16_bf16).  Every
// wavefront multiplies; wavefronts 0-3 also load W and 4-7 the token rows, each operand into its own
// LDS ring (W: 3 stages of 32 KB, it comes from HBM; token rows: 2 stages, they come from L2), by direct
// global->LDS loads of 128-byte row segments.  A stage is 64 hidden elements = 4 MFMA steps; operand
// fragments are double-buffered in registers one step ahead, and the barrier that opens the next
// stage sits before the last step of the current one, so the matrix pipe never waits on it.
// The eight 16-byte chunks of a row segment are XOR-swizzled by (row / 2) mod 8 on the way in, which
// makes the 128-bit operand reads conflict free on the 64-bank LDS.
#include "launch.hpp"
#include "lmhead_tile.hpp"

namespace aurora {

constexpr int kBgThreads = 512;
constexpr int kBgBK = 64;                       // hidden elements per stage
constexpr int kBgRowBytes = kBgBK * 2;          // 128
constexpr int kBgVTile = 256;                   // vocab rows per workgroup (= statistics tile)
constexpr int kBgMTile = 256;                   // token rows per workgroup, at most
constexpr int kBgWBytes = kBgVTile * kBgRowBytes;  // 32 KB: one stage of W rows
constexpr int kBgHBytes = kBgMTile * kBgRowBytes;  // 32 KB: one stage of token rows
constexpr int kBgWStages = 3;
constexpr int kBgHStages = 2;
constexpr int kBgWRing = kBgWStages * kBgWBytes;
constexpr int kBgLdsBytes = kBgWRing + kBgHStages * kBgHBytes;  // 160 KB
constexpr int kBgLoads = 8;                     // global->LDS instructions per wavefront per stage

// Direct global->LDS load of 16 bytes per lane; lane i's data lands at lds_base + 16 i.  Written as
// inline assembly so that the compiler does not order every later LDS read behind all such loads;
// the explicit vmcnt waits below do the waiting.  m0 holds the LDS base; one wait state is required
// between writing m0 and the load that reads it.
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}

__global__ __launch_bounds__(kBgThreads, 1) void lmhead_mfma_big_kernel(
    const bf16_t* __restrict__ hidden, const bf16_t* __restrict__ w, float* __restrict__ logits,
    float* __restrict__ pmax, float* __restrict__ psum, int32_t* __restrict__ parg, int M, int H, int V, int n_tiles,
    int m_tiles, float exp_scale /* log2(e) / T */, const float* __restrict__ temps /* per-request T, or NULL */,
    int Nq) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wvv = wave & 3;   // vocab slice of 64 rows
  const int wm = wave >> 2;   // token half
  // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  The m_tiles token tiles
  // of one vocab tile get ids 8 apart: same XCD, launched together - the W tile comes from HBM once and
  // from L2 for the others.  Every workgroup walks the hidden dimension in the same order: the
  // workgroups resident on one XCD then want the same slices of the token tiles at about the same time
  // and its L2 serves all but the first.
  const int wg = blockIdx.x;
  const int vt = (wg / (8 * m_tiles)) * 8 + (wg & 7);
  const int mt = (wg >> 3) % m_tiles;
  if (vt >= n_tiles) return;
  const int vbase = vt * kBgVTile;
  const int m0 = mt * kBgMTile;
  const int tb0 = wm * 4;  // first 32-token tile of this wavefront; rows past M are loaded clamped and never stored
  const int nk = H / kBgBK;
  const unsigned lds0 = (unsigned)(uintptr_t)lds;  // LDS pointers are 32-bit offsets

  // ---- loader role: 64 rows of one operand per wavefront and stage.  A wavefront's vmcnt queue holds one
  // operand only, so the deeper W ring is not held up behind token-row loads.
  const bool w_loader = wave < 4;
  const int depth = w_loader ? kBgWStages : kBgHStages;
  const int lrow = lane >> 3, lslot = lane & 7;
  const bf16_t* src[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int r = 64 * (wave & 3) + 8 * j + lrow;
    const int chunk = lslot ^ ((r >> 1) & 7);
    int vrow = vbase + r;
    vrow = vrow < V ? vrow : V - 1;
    int hrow = m0 + r;
    hrow = hrow < M ? hrow : M - 1;
    src[j] = w_loader ? w + (size_t)vrow * H + chunk * 8 : hidden + (size_t)hrow * H + chunk * 8;
  }
  const unsigned ring0 = lds0 + (w_loader ? 0 : kBgWRing) + 64 * (wave & 3) * kBgRowBytes;
  auto issue = [&](int ks, int slot) {
    const unsigned base = ring0 + slot * kBgWBytes;
    const int koff = ks * kBgBK;
#pragma unroll
    for (int j = 0; j < 8; ++j) dma16(src[j] + koff, base + 8 * j * kBgRowBytes);
  };

  f32x16_t acc[2][4];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;

  const int li = lane & 31, lh = lane >> 5;
  const int sw = (li >> 1) & 7;
  const int wrow_off = (wvv * 64 + li) * kBgRowBytes;
  const int hrow_off = kBgWRing + (tb0 * 32 + li) * kBgRowBytes;

  auto load_frag = [&](int wslot, int hslot, int s, bf16x8_t (&wa)[2], bf16x8_t (&hb)[4]) {
    const int coff = ((2 * s + lh) ^ sw) * 16;
    const char* wb = lds + wslot * kBgWBytes + wrow_off + coff;
    const char* hbp = lds + hslot * kBgHBytes + hrow_off + coff;
#pragma unroll
    for (int a = 0; a < 2; ++a) wa[a] = *(const bf16x8_t*)(wb + a * 32 * kBgRowBytes);
#pragma unroll
    for (int t = 0; t < 4; ++t)
      hb[t] = *(const bf16x8_t*)(hbp + t * 32 * kBgRowBytes);
  };
  auto multiply = [&](const bf16x8_t (&wa)[2], const bf16x8_t (&hb)[4]) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int a = 0; a < 2; ++a)
        acc[a][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[a], hb[t], acc[a][t], 0, 0, 0);
  };
  // one MFMA (its wait covers only reads issued a step ago), then this step's reads, then the other MFMAs
#define BG_STEP_ORDER()                                  \
  do {                                                   \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   \
    __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);   \
    __builtin_amdgcn_sched_group_barrier(0x008, 7, 0);   \
    __builtin_amdgcn_sched_barrier(0);                   \
  } while (0)
  auto wait_younger = [&](int groups) {  // wait until at most `groups` stages' loads of this wavefront are outstanding
    if (groups >= 2) LM_WAIT_VMCNT(2 * kBgLoads);
    else if (groups == 1) LM_WAIT_VMCNT(kBgLoads);
    else LM_WAIT_VMCNT(0);
  };
  static_assert(kBgWStages <= 3 && kBgHStages <= 3, "wait_younger covers at most 2 younger stages");

  for (int s = 0; s < depth && s < nk; ++s) issue(s, s);
  wait_younger(nk - 1 < depth - 1 ? nk - 1 : depth - 1);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  bf16x8_t wa0[2], hb0[4], wa1[2], hb1[4];
  load_frag(0, 0, 0, wa0, hb0);
  int wslot = 0, hslot = 0;  // ring slots of the stage being multiplied
  int myslot = 0;            // the same for this wavefront's loader ring
  for (int ks = 0; ks + 1 < nk; ++ks) {
    load_frag(wslot, hslot, 1, wa1, hb1);
    multiply(wa0, hb0);
    BG_STEP_ORDER();
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
    if (ks + depth < nk) issue(ks + depth, myslot);
    myslot = myslot + 1 == depth ? 0 : myslot + 1;
    wslot = wslot + 1 == kBgWStages ? 0 : wslot + 1;
    hslot = hslot + 1 == kBgHStages ? 0 : hslot + 1;
    load_frag(wslot, hslot, 0, wa0, hb0);
    multiply(wa1, hb1);
    BG_STEP_ORDER();
  }
  load_frag(wslot, hslot, 1, wa1, hb1);
  multiply(wa0, hb0);
  load_frag(wslot, hslot, 2, wa0, hb0);
  multiply(wa1, hb1);
  load_frag(wslot, hslot, 3, wa1, hb1);
  multiply(wa0, hb0);
  multiply(wa1, hb1);
#undef BG_STEP_ORDER
  __syncthreads();  // every wavefront is done with the ring; it becomes epilogue scratch

  // ---- epilogue ---------------------------------------------------------------------------------------
  // wavefront-private 8 KB each for turning the logits tiles, then [4][256] statistics of the four vocab slices
  char* tb = lds + wave * 8192;
  float* st_max = (float*)(lds + 8 * 8192);
  float* st_sum = st_max + 4 * kBgMTile;
  int* st_arg = (int*)(st_sum + 4 * kBgMTile);
  const int vrow0 = vbase + wvv * 64;
  const bool vec_ok = (V & 3) == 0;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int col0 = (tb0 + t) * 32;
    if (m0 + col0 < M) {  // tiles wholly past the last token row hold nothing
      float mx, sum;
      int arg;
      lm_tile_out(acc[0][t], acc[1][t], vrow0, V, m0 + col0, M, lm_row_scale(exp_scale, temps, Nq, m0 + col0 + li, M), tb,
                  logits, vec_ok, lane, mx, sum, arg);
      if (lh == 0) {
        st_max[wvv * kBgMTile + col0 + li] = mx;
        st_sum[wvv * kBgMTile + col0 + li] = sum;
        st_arg[wvv * kBgMTile + col0 + li] = arg;
      }
    }
  }
  __syncthreads();
  if (tid < kBgMTile) {
    const int m = m0 + tid;
    if (m < M) {
      float mx, sum;
      int arg;
      lm_merge_waves(st_max, st_sum, st_arg, kBgMTile, tid, lm_row_scale(exp_scale, temps, Nq, m, M), mx, sum, arg);
      const size_t o = (size_t)m * n_tiles + vt;
      pmax[o] = mx;
      psum[o] = sum;
      parg[o] = arg;
    }
  }
}

bool lmhead_mfma_big_supported(const AcceptLaunch& a) {
  return a.bf16 && a.H % kBgBK == 0 && a.H >= kBgBK && a.V >= 1 && a.plan.stat_tile == kBgVTile;
}

hipError_t launch_lmhead_mfma_big(const AcceptLaunch& a, hipStream_t st) {
  static LdsAttrOnce attr;
  if (hipError_t e = attr.ensure((const void*)lmhead_mfma_big_kernel, kBgLdsBytes); e != hipSuccess) return e;
  const int M = (int)a.plan.rows;
  const int m_tiles = (M + kBgMTile - 1) / kBgMTile;
  const float exp_scale = 1.4426950408889634f / (a.temperature > 0.f ? a.temperature : 1.f);
  const int v_tiles = (a.V + kBgVTile - 1) / kBgVTile;
  dim3 grid((v_tiles + 7) / 8 * 8 * m_tiles);
  hipLaunchKernelGGL(lmhead_mfma_big_kernel, grid, dim3(kBgThreads), kBgLdsBytes, st, (const bf16_t*)a.hidden,
                     (const bf16_t*)a.lm_head, a.logits, a.pmax, a.psum, a.parg, M, a.H, a.V, a.plan.n_tiles, m_tiles,
                     exp_scale, a.temps, a.Nq);
  return hipGetLastError();
}

}  // namespace aurora
