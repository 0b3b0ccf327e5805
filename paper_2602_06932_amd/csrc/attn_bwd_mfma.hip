// Backward pass of the chunk / tree attention on the matrix cores (paper section 3.1: the speculative tree goes
// through one batched forward and backward pass under the tree's mask), for up to 32 query rows per KV head
// (chains, small trees), head_dim 128, bf16.  Work is split exactly as in the forward kernel: 32-token tiles
// of a (request, KV head) pair, dealt in contiguous runs to one resident workgroup per compute unit; the four
// wavefronts of a workgroup take every fourth tile of a run with private LDS tiles.
//
// Per tile (tokens are the rows of the first two products, so a lane owns one query row and 16 tokens):
//   S^T  = K Q^T,  dP^T = V dO^T                      two 32x32x128 products, operands read like the forward scores
//   P^T  = exp2(S^T scale - lse),  dS^T = P^T o (dP^T - delta)          lane-local (lse, delta belong to the row)
//   dQ^T += K^T dS^T                                   like the forward's V^T P^T: transposing LDS reads of the K tile
//   dV    = P^T dO,  dK = dS^T Q                       contraction over the query rows: P and dS go through a small
//                                                      transposed LDS tile to become operands; a lane ends up with one
//                                                      column of 16 tokens, so a store instruction writes whole
//                                                      128-byte lines of the fp32 pools (partial lines cost 2.5x)
// K and V tiles come in by direct global->LDS loads in the layout of the forward kernel's V tiles (it serves
// the 128-bit row reads and the transposing reads alike); the next tile's V is requested once dP is formed,
// its K once dQ is updated.  delta = <dO, O> of a row is formed by the threads that stage the row.  dq is summed
// over the wavefronts at the end of a run and over the runs of a pair by a second kernel; dK / dV tiles are written
// once, by the wavefront that owns the tile.
#include "launch.hpp"
#include "attn_tile.hpp"

namespace aurora {

constexpr int kBmThreads = 256;
constexpr int kBmXtStride = 80;                       // bytes per token row of a transposed 32 x 32 bf16 tile
constexpr int kBmXtBytes = 32 * kBmXtStride;          // 2560
constexpr int kBmWaveBytes = 2 * kAtTileBytes + 2 * kBmXtBytes;
constexpr int bm_lds_bytes(int rt) { return 2 * rt * kAtTileBytes + 4 * kBmWaveBytes; }  // Q and dO tiles + four wavefronts

// S^T-type product: rows of `abuf` against the rows of `btile` (both in the V-tile layout, chunk ^ v_key(row):
// v_key is a permutation of 0..15 over any 16 consecutive rows, so the 128-bit row reads are conflict-free as
// well), contraction over the 128 columns
__device__ __forceinline__ f32x16_t tile_scores_v(const char* abuf, const char* btile, int li, int lh) {
  f32x16_t acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  const int key = v_key(li);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const bf16x8_t a = *(const bf16x8_t*)(abuf + li * kAtRowBytes + (((2 * s + lh) ^ key) * 16));
    const bf16x8_t b = *(const bf16x8_t*)(btile + li * kAtRowBytes + (((2 * s + lh) ^ key) * 16));
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
  }
  return acc;
}

// acc[db] += (A^T)(128 x 32) B(32 x 32): A is a 32-row tile in the V-tile layout read with transposing loads
// (as in the forward's P V product), b[uu] the B operand of contraction step uu.  kSwap exchanges the operands,
// which transposes the output: acc[db] += B^T A (block db of A's columns)
template <bool kSwap = false>
__device__ __forceinline__ void tile_tmm(const char* abuf, const bf16x8_t b[2], f32x16_t acc[4], int lane) {
  const int lh = lane >> 5, k = lane & 15, kq = k >> 2;
  const int g1 = (lane >> 4) & 1;
  const int lo0 = ((2 * g1 + ((k & 3) >> 1)) ^ (lh & 3)) * 16;
  const int lo1 = ((2 * g1 + ((k & 3) >> 1)) ^ ((2 + lh) & 3)) * 16;
  const int common = lh * 1024 + kq * 256 + (k & 1) * 8 + kq * 64;
  const int base0 = common + lo0;
  const int base1 = common + lo1 + 2048;
#pragma unroll
  for (int uu = 0; uu < 2; ++uu) {
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      typedef __attribute__((address_space(3))) s16x4_t* lds_v4;
      const s16x4_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(abuf + uu * 4096 + (base0 ^ (db * 64))));
      const s16x4_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(abuf + uu * 4096 + (base1 ^ (db * 64))));
      const u16x8_t va = {(unsigned short)r0[0], (unsigned short)r0[1], (unsigned short)r0[2], (unsigned short)r0[3],
                          (unsigned short)r1[0], (unsigned short)r1[1], (unsigned short)r1[2], (unsigned short)r1[3]};
      if (kSwap)
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[uu], __builtin_bit_cast(bf16x8_t, va), acc[db], 0, 0, 0);
      else
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, va), b[uu], acc[db], 0, 0, 0);
    }
  }
}

// Accumulator register r of lane (li, lh) holds tile row t(r) = 8(r/4) + 4 lh + r%4, column li.  The values are
// rounded to bf16 and (1) packed as the B operand of a product that contracts over the tile rows (x_b, as the
// forward does with P), (2) written to xt[row t][column li] so that they can be read back with the roles swapped.
__device__ __forceinline__ void pack_and_transpose(const float x[16], bf16x8_t x_b[2], char* xt, int li, int lh) {
#pragma unroll
  for (int r = 0; r < 16; r += 2) {
    const f32x2_t pp = {x[r], x[r + 1]};
    const bf16x2_t pk = __builtin_convertvector(pp, bf16x2_t);
    x_b[r >> 3][r & 7] = pk[0];
    x_b[r >> 3][(r & 7) + 1] = pk[1];
    const int t0 = 8 * (r >> 2) + 4 * lh + (r & 3);
    *(__bf16*)(xt + t0 * kBmXtStride + li * 2) = pk[0];
    *(__bf16*)(xt + (t0 + 1) * kBmXtStride + li * 2) = pk[1];
  }
}

// B operand of a product that contracts over the 32 columns of xt (the query rows) for output column li (a token):
// contraction step uu, element i of lane half lh  <->  column 16 uu + 8 (i / 4) + 4 lh + i % 4 - the order in which
// tile_tmm's transposing reads deliver the rows of its A tile
__device__ __forceinline__ void read_transposed(const char* xt, bf16x8_t b[2], int li, int lh) {
  typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
#pragma unroll
  for (int uu = 0; uu < 2; ++uu) {
    const bf16x4_t lo = *(const bf16x4_t*)(xt + li * kBmXtStride + (16 * uu + 4 * lh) * 2);
    const bf16x4_t hi = *(const bf16x4_t*)(xt + li * kBmXtStride + (16 * uu + 8 + 4 * lh) * 2);
    b[uu] = bf16x8_t{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  }
}

// <a, b> over eight bf16 pairs held as four 32-bit words each, accumulated in fp32
__device__ __forceinline__ float dot8_bf16(const u32x4_t a, const u32x4_t b, float acc) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    acc = fmaf(__uint_as_float(a[w] << 16), __uint_as_float(b[w] << 16), acc);
    acc = fmaf(__uint_as_float(a[w] & 0xffff0000u), __uint_as_float(b[w] & 0xffff0000u), acc);
  }
  return acc;
}

// P^T and dS^T of a tile for this lane's query row (register r <-> token j0 + 8(r/4) + 4 lh + r%4).  Only tiles
// that reach into the draft positions need the mask (a wavefront-uniform test); masked scores become -inf, and a
// row past the group has lse = +inf, so both give p = 0 without a select.
__device__ __forceinline__ void tile_p_ds(f32x16_t s_acc, const f32x16_t dp_acc, float p[16], float ds[16], float scale_log2,
                                          float lse2, float dlt, unsigned long long anc, int j0, int prefix, int L, int lh) {
  if (j0 + kAtTile > prefix) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = j0 + 8 * (r >> 2) + 4 * lh + (r & 3);
      const bool seen = j < prefix || (j < L && ((anc >> (j - prefix)) & 1ull));
      s_acc[r] = seen ? s_acc[r] : -INFINITY;
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    p[r] = __builtin_amdgcn_exp2f(fmaf(s_acc[r], scale_log2, -lse2));
    ds[r] = p[r] * (dp_acc[r] - dlt);
  }
}

// kLocalPlan: every workgroup builds the tile prefix per request in LDS (up to kLocalPlanMax requests; workgroup 0
// also writes it to PB for the dq merge); otherwise PB was filled by the planning kernel and is read from memory.
template <int kRT /* 32-row tiles of query rows per KV head: 1 or 2 */, bool kLocalPlan>
__global__ __launch_bounds__(kBmThreads, 1) void attn_bwd_mfma_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kp, const bf16_t* __restrict__ vp,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ parents,
    const bf16_t* __restrict__ dout, const float* __restrict__ lse, const bf16_t* __restrict__ out,
    int32_t* __restrict__ PB, float* __restrict__ part_dq, float* __restrict__ dk, float* __restrict__ dv, int B, int Nq,
    int Hq, int Hkv, int page_shift, int max_pages, float scale) {
  extern __shared__ __attribute__((aligned(1024))) char bm_lds[];
  char* qV = bm_lds;                          // the pair's query rows, kRT tiles in the V-tile layout
  char* doV = bm_lds + kRT * kAtTileBytes;    // their upstream gradients
  char* waves = bm_lds + 2 * kRT * kAtTileBytes;
  __shared__ int s_pb[kLocalPlan ? kLocalPlanMax + 1 : 1];
  __shared__ int s_wsum[4];
  __shared__ float s_delta[32 * kRT];  // delta_i = <dO_i, O_i> of the pair's query rows, formed while they are staged
  if (kLocalPlan) {
    build_prefix(seq_lens, B, Hkv, s_pb, s_wsum);
    if (blockIdx.x == 0)
      for (int i = threadIdx.x; i <= B; i += kBmThreads) PB[i] = s_pb[i];
  }
  auto pbv = [&](int i) -> int { return kLocalPlan ? s_pb[i] : PB[i]; };

  const int U = pbv(B);
  const int c = units_per_wg(U, gridDim.x);
  int u = blockIdx.x * c;
  const int u_end = min(U, u + c);
  if (u >= u_end) return;

  const int G = Hq / Hkv, R = G * Nq;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, lh = lane >> 5;
  char* kbuf = waves + wv * kBmWaveBytes;
  char* vbuf = kbuf + kAtTileBytes;
  char* pt = kbuf + 2 * kAtTileBytes;
  char* dst = pt + kBmXtBytes;
  const float scale_log2 = scale * kLog2e;

  int b = 0;
  {
    int lo = 0, hi = B - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (pbv(mid) <= u) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }

  while (u < u_end) {
    while (pbv(b + 1) <= u) ++b;
    const int L = seq_lens[b];
    const int n_b = (L + kAtTile - 1) / kAtTile;
    const int rel = u - pbv(b);
    const int hk = __builtin_amdgcn_readfirstlane(rel / n_b);
    const int t0 = rel - hk * n_b;
    const int t1 = min(n_b, t0 + (u_end - u));
    const int slot = blockIdx.x + b * Hkv + hk;
    u += t1 - t0;
    const int start = t0 * kAtTile;
    const int prefix = L - Nq;
    const int ntile = t1 - t0;
    const int32_t* bt = block_table + (size_t)b * max_pages;
    // the pair's query rows and their upstream gradients: group row m = n * G + g <-> (node n, head hk * G + g);
    // 8 threads per row, 32 bytes each, 32 rows per turn
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt) {
      const int m = 32 * rt + (tid >> 3);
      const bool ok = m < R;
      const int n = ok ? m / G : 0, g = ok ? m % G : 0;
      const size_t at = (((size_t)b * Nq + n) * Hq + hk * G + g) * kAtD;
      const u32x4_t* qp = (const u32x4_t*)(q + at);
      const u32x4_t* gp = (const u32x4_t*)(dout + at);
      const u32x4_t* op = (const u32x4_t*)(out + at);
      const int c0 = (tid & 7) * 2, row = tid >> 3;
      const u32x4_t z = {0u, 0u, 0u, 0u};
      float dpart = 0.f;  // this thread's share of delta = <dO, O> of the row
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int cv = ((c0 + i) ^ v_key(row)) * 16;
        const u32x4_t gv = ok ? gp[c0 + i] : z;
        *(u32x4_t*)(qV + rt * kAtTileBytes + row * kAtRowBytes + cv) = ok ? qp[c0 + i] : z;
        *(u32x4_t*)(doV + rt * kAtTileBytes + row * kAtRowBytes + cv) = gv;
        dpart = dot8_bf16(gv, ok ? op[c0 + i] : z, dpart);
      }
      dpart += __shfl_xor(dpart, 1, kWave);
      dpart += __shfl_xor(dpart, 2, kWave);
      dpart += __shfl_xor(dpart, 4, kWave);
      if ((tid & 7) == 0) s_delta[32 * rt + row] = dpart;
    }
    // this lane's query row of every row tile: logsumexp (log2 units), delta and the set of tree nodes it sees;
    // rows past the group see nothing
    float lse2[kRT], dlt[kRT];
    unsigned long long anc[kRT];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt) {
      const int m = 32 * rt + li;
      lse2[rt] = INFINITY;
      dlt[rt] = 0.f;
      anc[rt] = 0;
      if (m < R) {
        const int node = m / G;
        const size_t row = ((size_t)b * Nq + node) * Hq + hk * G + m % G;
        lse2[rt] = lse[row] * kLog2e;
        if (parents) {
          for (int a = node, hops = 0; a >= 0 && hops <= Nq; a = parents[(size_t)b * Nq + a], ++hops) anc[rt] |= 1ull << a;
        } else {
          anc[rt] = node == 63 ? ~0ull : ((1ull << (node + 1)) - 1);
        }
      }
    }

    auto tile_pages = [&](int tt, int& pid_a, int& pid_b) {
      const int j0 = start + tt * kAtTile;
      pid_a = bt[j0 >> page_shift];
      pid_b = bt[min(j0 + 16, L - 1) >> page_shift];
    };
    auto issue_tile = [&](const bf16_t* pool, char* buf, int tt, int pid_a, int pid_b) {
      const int j0 = start + tt * kAtTile;
#pragma unroll
      for (int j = 0; j < 8; ++j) issue_rows<true>(pool, buf, j, j0, L, page_shift, Hkv, hk, pid_a, pid_b, lane);
    };

    f32x16_t dq_acc[kRT][4];
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt)
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dq_acc[rt][db][r] = 0.f;

    __syncthreads();  // query rows staged
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt) dlt[rt] = 32 * rt + li < R ? s_delta[32 * rt + li] : 0.f;
    int tt = wv;
    int pa = 0, pb = 0;
    if (tt < ntile) {
      tile_pages(tt, pa, pb);
      issue_tile(kp, kbuf, tt, pa, pb);
      issue_tile(vp, vbuf, tt, pa, pb);
    }
    for (; tt < ntile; tt += 4) {
      const bool more = tt + 4 < ntile;
      int npa = 0, npb = 0;
      if (more) tile_pages(tt + 4, npa, npb);
      WAIT_VMCNT(0);  // this tile's K and V have landed (and the previous tile's stores have left)
      const int j0 = start + tt * kAtTile;
      f32x16_t dv_acc[4], dk_acc[4];
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dv_acc[db][r] = 0.f; dk_acc[db][r] = 0.f; }
#pragma unroll
      for (int rt = 0; rt < kRT; ++rt) {
        const f32x16_t s_acc = tile_scores_v(kbuf, qV + rt * kAtTileBytes, li, lh);
        const f32x16_t dp_acc = tile_scores_v(vbuf, doV + rt * kAtTileBytes, li, lh);
        if (rt == kRT - 1) {
          asm volatile("" ::: "memory");
          if (more) issue_tile(vp, vbuf, tt + 4, npa, npb);  // V is not read again
        }
        float p[16], ds[16];
        tile_p_ds(s_acc, dp_acc, p, ds, scale_log2, lse2[rt], dlt[rt], anc[rt], j0, prefix, L, lh);
        bf16x8_t p_b[2], ds_b[2];
        pack_and_transpose(p, p_b, pt, li, lh);
        pack_and_transpose(ds, ds_b, dst, li, lh);
        tile_tmm(kbuf, ds_b, dq_acc[rt], lane);  // dQ^T += K^T dS^T
        if (rt == kRT - 1) {
          asm volatile("" ::: "memory");
          if (more) issue_tile(kp, kbuf, tt + 4, npa, npb);  // K is not read again
        }
        // dV += P^T dO and dK += dS^T Q over this row tile.  The transposed tile is the A operand: the output has
        // one column per lane (32 db + li) and 16 tokens in the registers.
        bf16x8_t pt_b[2], dst_b[2];
        read_transposed(pt, pt_b, li, lh);
        read_transposed(dst, dst_b, li, lh);
        tile_tmm<true>(doV + rt * kAtTileBytes, pt_b, dv_acc, lane);
        tile_tmm<true>(qV + rt * kAtTileBytes, dst_b, dk_acc, lane);
      }
      {
        // a store instruction writes two whole 128-byte lines; the gradients are not read again
        const int mask = (1 << page_shift) - 1;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int tok = j0 + 8 * (r >> 2) + 4 * lh + (r & 3);
          if (tok < L) {
            const int pid = r < 8 ? pa : pb;  // tokens 0..15 of the tile lie in its first page, 16..31 in the page of token 16
            const size_t at = ((((size_t)pid * Hkv + hk) << page_shift) + (tok & mask)) * kAtD + li;
#pragma unroll
            for (int db = 0; db < 4; ++db) {
              __builtin_nontemporal_store(dv_acc[db][r], dv + at + 32 * db);
              __builtin_nontemporal_store(dk_acc[db][r] * scale, dk + at + 32 * db);
            }
          }
        }
      }
      pa = npa;
      pb = npb;
    }

    // ---- sum dQ^T over the four wavefronts and write the run's partial, one row tile at a time ----------------
    WAIT_VMCNT(0);
    __syncthreads();  // every wavefront is done with its tiles
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        float* obuf = (float*)(db < 2 ? kbuf : vbuf);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int dd = 32 * (db & 1) + 8 * g + 4 * lh;
          f32x4_t o = {dq_acc[rt][db][4 * g], dq_acc[rt][db][4 * g + 1], dq_acc[rt][db][4 * g + 2], dq_acc[rt][db][4 * g + 3]};
          *(f32x4_t*)(obuf + li * 64 + ((dd / 4 + li) & 15) * 4) = o;
        }
      }
      __syncthreads();
      {
        const int db = wv;  // wavefront w sums and stores d-block w of all rows
        const size_t prow = ((size_t)slot * kRT + rt) * 32 + li;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int dd = 32 * (db & 1) + 8 * g + 4 * lh;
          f32x4_t sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const char* wb = waves + w * kBmWaveBytes;
            const float* ob = (const float*)(db < 2 ? wb : wb + kAtTileBytes);
            sum += *(const f32x4_t*)(ob + li * 64 + ((dd / 4 + li) & 15) * 4);
          }
          if (32 * rt + li < R) *(f32x4_t*)(part_dq + prow * kAtD + 32 * db + 8 * g + 4 * lh) = sum;
        }
      }
      __syncthreads();  // the tiles are about to be overwritten (next row tile, or the next run's K and V)
    }
  }
}

// ---- 65 .. 128 query rows per KV head: one row tile per wavefront, K / V tiles shared by the workgroup -----------
// Four dq accumulator sets per wavefront do not fit the register file next to the dK / dV accumulators, so the
// work of a tile is cut the other way.  The workgroup walks the tiles of its run together (a K / V tile pair is
// loaded once for everybody); wavefront w of a group of four forms S^T, dP^T, P, dS and dQ for row tile w and
// publishes its transposed P and dS tiles; after a barrier it contracts over ALL row tiles for column block w of
// dV and dK (16 accumulator registers each) and stores those columns.
constexpr int kBsKvBytes = 2 * kAtTileBytes;   // K tile, then V tile
constexpr int kBsXtBytes = 2 * kBmXtBytes;     // transposed P, then dS, of one wavefront

// block db of tile_tmm<true>: acc += B^T A[:, 32 db .. 32 db + 31]
__device__ __forceinline__ void tile_tmm_block(const char* abuf, const bf16x8_t b[2], f32x16_t& acc, int lane, int db) {
  const int lh = lane >> 5, k = lane & 15, kq = k >> 2;
  const int g1 = (lane >> 4) & 1;
  const int lo0 = ((2 * g1 + ((k & 3) >> 1)) ^ (lh & 3)) * 16;
  const int lo1 = ((2 * g1 + ((k & 3) >> 1)) ^ ((2 + lh) & 3)) * 16;
  const int common = lh * 1024 + kq * 256 + (k & 1) * 8 + kq * 64;
  const int base0 = (common + lo0) ^ (db * 64);
  const int base1 = (common + lo1 + 2048) ^ (db * 64);
#pragma unroll
  for (int uu = 0; uu < 2; ++uu) {
    typedef __attribute__((address_space(3))) s16x4_t* lds_v4;
    const s16x4_t r0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(abuf + uu * 4096 + base0));
    const s16x4_t r1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(abuf + uu * 4096 + base1));
    const u16x8_t va = {(unsigned short)r0[0], (unsigned short)r0[1], (unsigned short)r0[2], (unsigned short)r0[3],
                        (unsigned short)r1[0], (unsigned short)r1[1], (unsigned short)r1[2], (unsigned short)r1[3]};
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[uu], __builtin_bit_cast(bf16x8_t, va), acc, 0, 0, 0);
  }
}

// Eight wavefronts: two groups of four, half a tile apart.  Group g = wavefront / 4 takes the tiles of the run
// with parity g.  The workgroup advances in steps separated by one barrier: in step s group s % 2 does the first half of tile s (S^T, dP^T, P, dS, dQ for row tile w, transposed
// tiles published to the group's own buffer) while the other group does the second half of tile s - 1 (column
// block w of dV and dK over all row tiles, stores).  Each SIMD thus holds one wavefront that mostly multiplies
// and one that mostly moves data, and there is one barrier per tile instead of two.  K / V tile pairs rotate
// through three buffers: tile s + 2 is requested at the top of step s (every wavefront issues one row group of K
// and one of V), into the buffer that tile s - 1 left at the end of step s - 1.  The requests are issued for
// clamped tile numbers up to the last step, so that every wavefront's queue of outstanding memory operations looks
// the same at every step top: [loads of tile s] [2 loads, 32 stores in either order] - hence vmcnt(34), and
// vmcnt(2) in the first three steps, where the stores are not there yet.
constexpr int kB8Threads = 512;
constexpr int kB8LdsBytes = 8 * kAtTileBytes + 3 * kBsKvBytes + 2 * 4 * kBsXtBytes;

template <bool kLocalPlan>
__global__ __launch_bounds__(kB8Threads, 1) void attn_bwd_mfma_shared_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kp, const bf16_t* __restrict__ vp,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ parents,
    const bf16_t* __restrict__ dout, const float* __restrict__ lse, const bf16_t* __restrict__ out,
    int32_t* __restrict__ PB, float* __restrict__ part_dq, float* __restrict__ dk, float* __restrict__ dv, int B, int Nq,
    int Hq, int Hkv, int page_shift, int max_pages, float scale) {
  extern __shared__ __attribute__((aligned(1024))) char bm_lds[];
  char* qV = bm_lds;                        // four row tiles of the pair's query rows (V-tile layout)
  char* doV = bm_lds + 4 * kAtTileBytes;    // their upstream gradients
  char* kv = bm_lds + 8 * kAtTileBytes;     // three K / V tile pairs
  char* xt = kv + 3 * kBsKvBytes;           // per group: four transposed (P, dS) tiles
  __shared__ int s_pb[kLocalPlan ? kLocalPlanMax + 1 : 1];
  __shared__ int s_wsum[8];
  __shared__ float s_delta[128];  // delta_i = <dO_i, O_i> of the pair's query rows, formed while they are staged
  if (kLocalPlan) {
    build_prefix(seq_lens, B, Hkv, s_pb, s_wsum);
    if (blockIdx.x == 0)
      for (int i = threadIdx.x; i <= B; i += kB8Threads) PB[i] = s_pb[i];
  }
  auto pbv = [&](int i) -> int { return kLocalPlan ? s_pb[i] : PB[i]; };

  const int U = pbv(B);
  const int c = units_per_wg(U, gridDim.x);
  int u = blockIdx.x * c;
  const int u_end = min(U, u + c);
  if (u >= u_end) return;

  const int G = Hq / Hkv, R = G * Nq;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wv8 >> 2, wv = wv8 & 3;  // group; row tile and column block within the group
  const int li = lane & 31, lh = lane >> 5;
  const float scale_log2 = scale * kLog2e;
  const int mask = (1 << page_shift) - 1;
  char* xts = xt + grp * 4 * kBsXtBytes;

  int b = 0;
  {
    int lo = 0, hi = B - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (pbv(mid) <= u) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }

  while (u < u_end) {
    while (pbv(b + 1) <= u) ++b;
    const int L = seq_lens[b];
    const int n_b = (L + kAtTile - 1) / kAtTile;
    const int rel = u - pbv(b);
    const int hk = __builtin_amdgcn_readfirstlane(rel / n_b);
    const int t0 = rel - hk * n_b;
    const int t1 = min(n_b, t0 + (u_end - u));
    const int slot = blockIdx.x + b * Hkv + hk;
    u += t1 - t0;
    const int start = t0 * kAtTile;
    const int prefix = L - Nq;
    const int ntile = t1 - t0;
    const int32_t* bt = block_table + (size_t)b * max_pages;
    // the pair's query rows and upstream gradients: 8 threads per row, 32 bytes each, 64 rows per turn
#pragma unroll
    for (int turn = 0; turn < 2; ++turn) {
      const int m = 64 * turn + (tid >> 3);
      const bool ok = m < R;
      const int n = ok ? m / G : 0, g = ok ? m % G : 0;
      const size_t at = (((size_t)b * Nq + n) * Hq + hk * G + g) * kAtD;
      const u32x4_t* qp = (const u32x4_t*)(q + at);
      const u32x4_t* gp = (const u32x4_t*)(dout + at);
      const u32x4_t* op = (const u32x4_t*)(out + at);
      const int c0 = (tid & 7) * 2, row = m & 31, rt = m >> 5;
      const u32x4_t z = {0u, 0u, 0u, 0u};
      float dpart = 0.f;  // this thread's share of delta = <dO, O> of the row
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int cv = ((c0 + i) ^ v_key(row)) * 16;
        const u32x4_t gv = ok ? gp[c0 + i] : z;
        *(u32x4_t*)(qV + rt * kAtTileBytes + row * kAtRowBytes + cv) = ok ? qp[c0 + i] : z;
        *(u32x4_t*)(doV + rt * kAtTileBytes + row * kAtRowBytes + cv) = gv;
        dpart = dot8_bf16(gv, ok ? op[c0 + i] : z, dpart);
      }
      dpart += __shfl_xor(dpart, 1, kWave);
      dpart += __shfl_xor(dpart, 2, kWave);
      dpart += __shfl_xor(dpart, 4, kWave);
      if ((tid & 7) == 0) s_delta[m] = dpart;
    }
    // this lane's query row (row tile = wavefront within the group)
    const int m_row = 32 * wv + li;
    float lse2 = INFINITY, dlt = 0.f;
    unsigned long long anc = 0;
    if (m_row < R) {
      const int node = m_row / G;
      const size_t row = ((size_t)b * Nq + node) * Hq + hk * G + m_row % G;
      lse2 = lse[row] * kLog2e;
      if (parents) {
        for (int a = node, hops = 0; a >= 0 && hops <= Nq; a = parents[(size_t)b * Nq + a], ++hops) anc |= 1ull << a;
      } else {
        anc = node == 63 ? ~0ull : ((1ull << (node + 1)) - 1);
      }
    }

    // this wavefront's eighth of a tile pair's loads: one row group (four token rows) of K and one of V
    auto issue_eighth = [&](int tt) {
      const int tl = min(tt, ntile - 1);
      const int j0 = start + tl * kAtTile;
      const int pid_a = bt[j0 >> page_shift];
      const int pid_b = bt[min(j0 + 16, L - 1) >> page_shift];
      char* kb = kv + (tt % 3) * kBsKvBytes;
      issue_rows<true>(kp, kb, wv8, j0, L, page_shift, Hkv, hk, pid_a, pid_b, lane);
      issue_rows<true>(vp, kb + kAtTileBytes, wv8, j0, L, page_shift, Hkv, hk, pid_a, pid_b, lane);
    };

    f32x16_t dq_acc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) dq_acc[db][r] = 0.f;

    __syncthreads();  // query rows staged; the previous run is done with every buffer
    dlt = m_row < R ? s_delta[m_row] : 0.f;
    issue_eighth(0);
    issue_eighth(1);
    for (int s = 0; s <= ntile; ++s) {
      if (s <= 2) WAIT_VMCNT(2); else WAIT_VMCNT(34);            // tile s has landed (this wavefront's part)
      __builtin_amdgcn_s_waitcnt((7 << 4) | (3 << 14) | 15);      // lgkmcnt(0): LDS reads and writes of the last step
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      issue_eighth(s + 2);  // into the buffer tile s - 1 used
      if ((s & 1) == grp) {
        if (s < ntile) {
          const char* kb = kv + (s % 3) * kBsKvBytes;
          const char* vb = kb + kAtTileBytes;
          const int j0 = start + s * kAtTile;
          const f32x16_t s_acc = tile_scores_v(kb, qV + wv * kAtTileBytes, li, lh);
          const f32x16_t dp_acc = tile_scores_v(vb, doV + wv * kAtTileBytes, li, lh);
          float p[16], ds[16];
          tile_p_ds(s_acc, dp_acc, p, ds, scale_log2, lse2, dlt, anc, j0, prefix, L, lh);
          bf16x8_t p_b[2], ds_b[2];
          pack_and_transpose(p, p_b, xts + wv * kBsXtBytes, li, lh);
          pack_and_transpose(ds, ds_b, xts + wv * kBsXtBytes + kBmXtBytes, li, lh);
          tile_tmm(kb, ds_b, dq_acc, lane);  // dQ^T += K^T dS^T for this wavefront's row tile
        }
      } else if (s >= 1) {
        // columns 32 wv .. 32 wv + 31 of dV = P^T dO and dK = dS^T Q of tile s - 1, contraction over all four row tiles
        const int j0 = start + (s - 1) * kAtTile;
        const int pa = bt[j0 >> page_shift];
        const int pb = bt[min(j0 + 16, L - 1) >> page_shift];
        f32x16_t dv_acc, dk_acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) { dv_acc[r] = 0.f; dk_acc[r] = 0.f; }
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
          bf16x8_t pt_b[2], dst_b[2];
          read_transposed(xts + rt * kBsXtBytes, pt_b, li, lh);
          read_transposed(xts + rt * kBsXtBytes + kBmXtBytes, dst_b, li, lh);
          tile_tmm_block(doV + rt * kAtTileBytes, pt_b, dv_acc, lane, wv);
          tile_tmm_block(qV + rt * kAtTileBytes, dst_b, dk_acc, lane, wv);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int tok = j0 + 8 * (r >> 2) + 4 * lh + (r & 3);
          if (tok < L) {
            const int pid = r < 8 ? pa : pb;
            const size_t at = ((((size_t)pid * Hkv + hk) << page_shift) + (tok & mask)) * kAtD + 32 * wv + li;
            __builtin_nontemporal_store(dv_acc[r], dv + at);
            __builtin_nontemporal_store(dk_acc[r] * scale, dk + at);
          }
        }
      }
    }
    // ---- the two groups' dq of a row tile are summed through LDS; group 0 writes the run's partial -----------
    WAIT_VMCNT(0);  // the clamped requests of the last steps have landed: the tile buffers can be reused
    __syncthreads();
    float* park = (float*)kv + wv * (64 * 64);  // 16 KB per row tile, inside the K / V and transposed-tile buffers
    if (grp == 1) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) park[(db * 16 + r) * 64 + lane] = dq_acc[db][r];
    }
    __syncthreads();
    if (grp == 0 && m_row < R) {
      const size_t prow = (size_t)slot * 128 + m_row;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4_t o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = dq_acc[db][4 * g + e] + park[(db * 16 + 4 * g + e) * 64 + lane];
          *(f32x4_t*)(part_dq + prow * kAtD + 32 * db + 8 * g + 4 * lh) = o;
        }
    }
    __syncthreads();  // the query tiles and the parked sums are overwritten by the next run
  }
}

// dq of one output row = scale * sum of the partials of the runs that met its (request, KV head) pair
__global__ __launch_bounds__(256) void attn_bwd_dq_combine(const float* __restrict__ part_dq,
                                                           const int32_t* __restrict__ seq_lens,
                                                           const int32_t* __restrict__ PB, float* __restrict__ dq, int B,
                                                           int Nq, int Hq, int Hkv, int wgs, int row_tiles, unsigned n_rows, float scale) {
  const size_t row = (size_t)blockIdx.x * 8 + (threadIdx.x >> 5);
  if (row >= n_rows) return;
  const int hq = (int)(row % Hq);
  const int n = (int)((row / Hq) % Nq);
  const int b = (int)(row / ((size_t)Hq * Nq));
  const int G = Hq / Hkv, hk = hq / G;
  const int mrow = n * G + hq % G;
  const int n_b = (seq_lens[b] + kAtTile - 1) / kAtTile;
  const int c = units_per_wg(PB[B], wgs);
  const int u0 = PB[b] + hk * n_b, u1 = u0 + n_b;
  const int w0 = u0 / c, w1 = (u1 - 1) / c;
  const int pair = b * Hkv + hk;
  const int d4 = threadIdx.x & 31;
  f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
  for (int w = w0; w <= w1; ++w) acc += *(const f32x4_t*)(part_dq + ((size_t)(w + pair) * 32 * row_tiles + mrow) * kAtD + 4 * d4);
  *(f32x4_t*)(dq + row * kAtD + 4 * d4) = acc * scale;
}

bool attn_bwd_mfma_supported(const AttnBwdLaunch& a) {
  return a.bf16 && a.D == kAtD && a.page >= 16 && (a.page & (a.page - 1)) == 0 && a.Hq / a.Hkv * a.Nq <= 128;
}

int attn_bwd_mfma_workgroups() { return 256; }

// row tiles of the pair: 1 or 2 (wavefront-private tiles), 4 (shared tiles)
static int bwd_row_tiles(const AttnBwdLaunch& a) {
  const int R = a.Hq / a.Hkv * a.Nq;
  return R <= 32 ? 1 : R <= 64 ? 2 : 4;
}
size_t attn_bwd_mfma_partial_bytes(int batch, int kv_heads, int rows_per_group) {
  const int rt = rows_per_group <= 32 ? 1 : rows_per_group <= 64 ? 2 : 4;
  return ((size_t)attn_bwd_mfma_workgroups() + (size_t)batch * kv_heads) * 32 * rt * kAtD * sizeof(float);
}

template <int kRT, bool kLocalPlan>
static hipError_t launch_bwd_mfma_t(const AttnBwdLaunch& a, hipStream_t st) {
  static LdsAttrOnce attr;
  if (hipError_t e = attr.ensure((const void*)attn_bwd_mfma_kernel<kRT, kLocalPlan>, bm_lds_bytes(kRT)); e != hipSuccess)
    return e;
  hipLaunchKernelGGL((attn_bwd_mfma_kernel<kRT, kLocalPlan>), dim3(attn_bwd_mfma_workgroups()), dim3(kBmThreads), bm_lds_bytes(kRT), st,
                     (const bf16_t*)a.q, (const bf16_t*)a.k, (const bf16_t*)a.v, a.block_table, a.seq_lens, a.parents,
                     (const bf16_t*)a.dout, a.lse, (const bf16_t*)a.out, a.plan_pb, a.part_dq, a.dk, a.dv, a.B, a.Nq, a.Hq, a.Hkv,
                     __builtin_ctz(a.page), a.max_pages, a.scale);
  return hipGetLastError();
}

template <bool kLocalPlan>
static hipError_t launch_bwd_mfma_shared(const AttnBwdLaunch& a, hipStream_t st) {
  static LdsAttrOnce attr;
  if (hipError_t e = attr.ensure((const void*)attn_bwd_mfma_shared_kernel<kLocalPlan>, kB8LdsBytes); e != hipSuccess)
    return e;
  hipLaunchKernelGGL(attn_bwd_mfma_shared_kernel<kLocalPlan>, dim3(attn_bwd_mfma_workgroups()), dim3(kB8Threads), kB8LdsBytes, st,
                     (const bf16_t*)a.q, (const bf16_t*)a.k, (const bf16_t*)a.v, a.block_table, a.seq_lens, a.parents,
                     (const bf16_t*)a.dout, a.lse, (const bf16_t*)a.out, a.plan_pb, a.part_dq, a.dk, a.dv, a.B, a.Nq, a.Hq, a.Hkv,
                     __builtin_ctz(a.page), a.max_pages, a.scale);
  return hipGetLastError();
}

hipError_t launch_attn_backward_mfma(const AttnBwdLaunch& a, hipStream_t st) {
  const int rows = a.B * a.Nq * a.Hq;
  const int rt = bwd_row_tiles(a);
  hipError_t e = hipSuccess;
  if (a.B <= kLocalPlanMax) {
    e = rt == 1 ? launch_bwd_mfma_t<1, true>(a, st) : rt == 2 ? launch_bwd_mfma_t<2, true>(a, st)
                                                              : launch_bwd_mfma_shared<true>(a, st);
  } else {
    e = launch_attn_plan(a.seq_lens, a.B, a.Hkv, a.plan_pb, st);
    if (e != hipSuccess) return e;
    e = rt == 1 ? launch_bwd_mfma_t<1, false>(a, st) : rt == 2 ? launch_bwd_mfma_t<2, false>(a, st)
                                                               : launch_bwd_mfma_shared<false>(a, st);
  }
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_bwd_dq_combine, dim3((rows + 7) / 8), dim3(256), 0, st, a.part_dq, a.seq_lens, a.plan_pb, a.dq,
                     a.B, a.Nq, a.Hq, a.Hkv, attn_bwd_mfma_workgroups(), rt, (unsigned)rows, a.scale);
  return hipGetLastError();
}

}  // namespace aurora
