// Trace emission after a verify step (paper section 3.1: accepted and rejected outcomes are both
// streamed to the training side; appendix A.1 eq. 4: a record is (h, l, x_in, y_out, R); appendix A.2:
// only the K = 1024 largest target logits of a token are kept, 2 bytes each).
//
//   trace_topk_kernel     one workgroup per token row: the K largest logits, ids ordered by value
//                         descending (equal values by ascending id), values rounded to bfloat16.
//   trace_records_kernel  y_out and the rejection trajectory R from the acceptance outputs.
//
// Selection.  A float is mapped to an unsigned key with the same order (-0.0 folded onto +0.0); an
// entry is the 64-bit word (key << 32 | ~id): words are distinct, and descending word order is value
// order with the lowest id first among equals.  "The K largest words" is therefore a unique set, and
// a radix select (8 bits per pass, histogram in LDS, stop as soon as the threshold bin is taken whole)
// finds the threshold word T with exactly K words >= T.
// Common case, one pass over the row: a cut-off key is selected from a sample of 4096 entries (1024
// evenly spaced 16-byte vectors) so that
// about 2K entries reach it; the row is streamed once (16-byte loads, eight in flight per thread) and
// the few entries at or above the cut-off are appended to a list in LDS; the list is cut to exactly K
// by a radix select inside LDS, compacted, sorted (bitonic, 1024 words) and written out.  If the list
// comes out shorter than K or longer than its capacity (heavily repeated values, adversarial rows),
// the radix select runs over the whole row in global memory instead.  Both routes give the same set.
#include "common.hpp"
#include "launch.hpp"

namespace aurora {

constexpr int kTrThreads = 1024;
constexpr int kTrCap = 4096;     // capacity of the candidate list (and size of the sample)
constexpr int kTrMaxK = 1024;

__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0;  // -0.0 compares equal to +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t entry_word(float x, int id) {
  return ((uint64_t)order_key(x) << 32) | (uint32_t)~id;
}

__device__ __forceinline__ uint16_t bf16_rne_bits(float f) {
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) == 0x7f800000u) return (uint16_t)(u >> 16);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// Descending bitonic sort of n (a power of two, 2..kTrCap) words in LDS by the whole workgroup.  A
// wavefront's 64 pairs of a step span 128 consecutive words whenever the step's stride is at most 64,
// so those steps need no workgroup barrier: LDS operations of one wavefront execute in order.
template <typename T>
__device__ __forceinline__ void bitonic_desc(T* a, int n) {
  for (int size = 2, lsize = 1; size <= n; size <<= 1, ++lsize) {
    for (int ls = lsize - 1; ls >= 0; --ls) {
      const int stride = 1 << ls;
      if (stride >= 64 || ls == lsize - 1) __syncthreads();  // the step reads words other wavefronts wrote
      else __builtin_amdgcn_wave_barrier();
      for (int t = threadIdx.x; t < (n >> 1); t += kTrThreads) {
        const int lo = ((t >> ls) << (ls + 1)) + (t & (stride - 1));
        const int hi = lo + stride;
        const bool desc = ((lo & size) == 0);
        const T x = a[lo], y = a[hi];
        if ((x < y) == desc) { a[lo] = y; a[hi] = x; }
      }
    }
  }
  __syncthreads();
}

struct SelectShared {
  int hist[256];
  int digit, remaining, whole;  // written by pick_digit
};

// One histogram increment per calling lane (inactive lanes pass valid = false).  Lanes of a wavefront
// that hit the same bin are first combined (up to four distinct bins), because same-address LDS
// atomics serialise and the high digits of similar values are nearly all equal.
__device__ __forceinline__ void hist_add(int* hist, int digit, bool valid) {
  unsigned long long active = __ballot(valid);
  const int lane = threadIdx.x & 63;
#pragma unroll 1
  for (int round = 0; round < 4 && active; ++round) {
    const int leader = __ffsll((long long)active) - 1;
    const int v = __shfl(digit, leader, kWave);
    const unsigned long long same = __ballot(valid && digit == v) & active;
    if (lane == leader) atomicAdd(&hist[v], __popcll(same));
    active &= ~same;
  }
  if (valid && ((active >> lane) & 1ull)) atomicAdd(&hist[digit], 1);
}

// Called by every thread of wavefront 0 after the histogram is complete (and a barrier).  Finds the
// highest digit d whose bins d..255 hold at least `rem` entries; remaining = entries still to take from
// bin d, whole = that is all of bin d.
__device__ __forceinline__ void pick_digit(SelectShared& sh, int rem) {
  const int lane = threadIdx.x & 63;
  int c[4], tot = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) { c[j] = sh.hist[4 * lane + j]; tot += c[j]; }
  int suffix = tot;  // entries in the bins of lanes >= this one
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int y = __shfl_down(suffix, o, kWave);
    if (lane + o < kWave) suffix += y;
  }
  int above = suffix - tot;
  if (above < rem && rem <= suffix) {
#pragma unroll
    for (int j = 3; j >= 0; --j) {
      if (above < rem && rem <= above + c[j]) {
        sh.digit = 4 * lane + j;
        sh.remaining = rem - above;
        sh.whole = (rem - above) == c[j];
      }
      above += c[j];
    }
  }
}

// Threshold word T such that exactly `want` of the n words produced by word(i), i in [0, n), are >= T
// (1 <= want <= n; the words are distinct).  kBits = 32 or 64: the width that carries information.
// With kStop > 0 the digits below bit kStop are not examined: the result is then the threshold's prefix,
// zero-extended, and at least `want` words are >= it (the whole last bin is included).
// Whole workgroup; `word` is evaluated once per pass and entry.
template <int kBits, int kStop, typename F>
__device__ __forceinline__ uint64_t radix_threshold(SelectShared& sh, int n, int want, F word) {
  uint64_t prefix = 0, mask = 0;
  int rem = want;
  for (int shift = kBits - 8; shift >= kStop; shift -= 8) {
    __syncthreads();
    if (threadIdx.x < 256) sh.hist[threadIdx.x] = 0;
    __syncthreads();
    for (int i0 = 0; i0 < n; i0 += kTrThreads) {
      const int i = i0 + threadIdx.x;
      uint64_t w = 0;
      const bool in = i < n;
      if (in) w = word(i);
      hist_add(sh.hist, (int)((w >> shift) & 255), in && (w & mask) == prefix);
    }
    __syncthreads();
    if (threadIdx.x < kWave) pick_digit(sh, rem);
    __syncthreads();
    prefix |= (uint64_t)sh.digit << shift;
    mask |= 255ull << shift;
    rem = sh.remaining;
    if (sh.whole) break;  // every word that shares the prefix is taken: prefix, zero-extended, is the threshold
  }
  return prefix;
}

// kMapped: the selection runs over the V entries row[map[0]], .., row[map[V-1]] of a row of Vrow logits
// (the draft vocabulary, appendix A.2) and the ids written are positions in that list.
template <bool kMapped>
__global__ __launch_bounds__(kTrThreads, 2) void trace_topk_kernel(const float* __restrict__ logits, int Vrow, int V, int K,
                                                               const int32_t* __restrict__ map,
                                                               int32_t* __restrict__ out_ids,
                                                               uint16_t* __restrict__ out_vals) {
  __shared__ uint64_t s_cand[kTrCap];   // 32 KB: the sample (as 32-bit keys), then the candidate list
  __shared__ uint64_t s_top[kTrMaxK];   // 8 KB: the K selected words, sorted at the end
  __shared__ SelectShared s_sel;
  __shared__ unsigned s_count;
  const int tid = threadIdx.x;
  const float* row = logits + (size_t)blockIdx.x * Vrow;
  auto at = [&](int i) -> float { return kMapped ? row[map[i]] : row[i]; };
  int32_t* ids = out_ids + (size_t)blockIdx.x * K;
  uint16_t* vals = out_vals + (size_t)blockIdx.x * K;
  const int want = K < V ? K : V;  // entries that exist
  int count;                       // entries in the candidate list
  bool from_row = false;           // select over the whole row instead of the list

  if (V <= kTrCap) {
    for (int i = tid; i < V; i += kTrThreads) s_cand[i] = entry_word(at(i), i);
    count = V;
  } else {
    // entries before the first 16-byte boundary (of the row, or of the index list when mapped)
    const uintptr_t vec_base = kMapped ? (uintptr_t)map : (uintptr_t)row;
    const int head = (int)(((16 - (vec_base & 15)) & 15) >> 2);
    const int h = head < V ? head : V;
    const int nvec = (V - h) >> 2;  // >= 1023 here
    typedef __attribute__((ext_vector_type(4))) float f32x4_t;
    typedef __attribute__((ext_vector_type(4))) int i32x4_t;
    auto load4 = [&](int i) -> f32x4_t {  // entries h + 4i .. h + 4i + 3
      if (!kMapped) return ((const f32x4_t*)(row + h))[i];
      const i32x4_t j = ((const i32x4_t*)(map + h))[i];
      return f32x4_t{row[j[0]], row[j[1]], row[j[2]], row[j[3]]};
    };
    // ---- cut-off key from a sample ---------------------------------------------------------------------
    // 1024 evenly spaced 16-byte vectors (one 128-byte line in several is touched, not every line)
    uint32_t* s_sample = (uint32_t*)s_cand;
    {
      const int vstride = nvec / (kTrCap / 4);
      const int vi = vstride ? tid * vstride : (tid < nvec ? tid : nvec - 1);
      const f32x4_t x = load4(vi);
#pragma unroll
      for (int j = 0; j < 4; ++j) s_sample[4 * tid + j] = order_key(x[j]);
    }
    // sample rank whose key is expected to have about 2K row entries at or above it (always < kTrCap); the
    // cut-off only needs the key's upper 16 bits (sign, exponent, 7 mantissa bits): a few more entries pass
    const int r = (int)((2ll * K * kTrCap + V - 1) / V) + 8;
    const uint32_t cut = (uint32_t)radix_threshold<32, 16>(s_sel, kTrCap, r + 1, [&](int i) { return (uint64_t)s_sample[i]; });
    __syncthreads();
    if (tid == 0) s_count = 0;
    __syncthreads();
    // ---- one pass over the row: keep what reaches the cut-off ------------------------------------------
    // The pass compares floats: key(x) >= cut  <=>  x >= cut_f for the float cut_f whose key is `cut` (keys
    // are monotone, and -0.0 >= +0.0 holds just as their keys are equal); only survivors pay for a key.
    float cut_f;
    {
      const uint32_t u = (cut & 0x80000000u) ? (cut ^ 0x80000000u) : ~cut;
      cut_f = __uint_as_float(u);
      if (cut_f != cut_f) cut_f = -INFINITY;  // a prefix below every finite key: everything passes
    }
    if (tid < h) {
      const float x = at(tid);
      if (x >= cut_f) {
        const unsigned slot = atomicAdd(&s_count, 1u);
        if (slot < (unsigned)kTrCap) s_cand[slot] = entry_word(x, tid);
      }
    }
    // sixteen 16-byte loads in flight per thread: the pass is bound by memory latency otherwise
    constexpr int kU = 8;
    for (int i0 = tid; i0 < nvec; i0 += kU * kTrThreads) {
      f32x4_t x[kU];
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int i = i0 + u * kTrThreads;
        x[u] = i < nvec ? load4(i) : f32x4_t{0.f, 0.f, 0.f, 0.f};
      }
#pragma unroll
      for (int u = 0; u < kU; ++u) {
        const int i = i0 + u * kTrThreads;
        if (i < nvec) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (x[u][j] >= cut_f) {
              const unsigned slot = atomicAdd(&s_count, 1u);
              if (slot < (unsigned)kTrCap) s_cand[slot] = entry_word(x[u][j], h + 4 * i + j);
            }
          }
        }
      }
    }
    for (int i = h + 4 * nvec + tid; i < V; i += kTrThreads) {
      const float x = at(i);
      if (x >= cut_f) {
        const unsigned slot = atomicAdd(&s_count, 1u);
        if (slot < (unsigned)kTrCap) s_cand[slot] = entry_word(x, i);
      }
    }
    __syncthreads();
    count = (int)s_count;
    from_row = count < want || count > kTrCap;
  }

  // ---- cut to exactly `want` words and compact them into s_top ------------------------------------------
  __syncthreads();
  if (tid == 0) s_count = 0;
  if (!from_row) {
    uint64_t thr = 0;  // count == want: everything is taken
    if (count > want) thr = radix_threshold<64, 0>(s_sel, count, want, [&](int i) { return s_cand[i]; });
    __syncthreads();
    for (int i = tid; i < count; i += kTrThreads) {
      const uint64_t w = s_cand[i];
      if (w >= thr) {
        const unsigned slot = atomicAdd(&s_count, 1u);
        if (slot < (unsigned)kTrMaxK) s_top[slot] = w;
      }
    }
  } else {
    const uint64_t thr = radix_threshold<64, 0>(s_sel, V, want, [&](int i) { return entry_word(at(i), i); });
    __syncthreads();
    for (int i = tid; i < V; i += kTrThreads) {
      const uint64_t w = entry_word(at(i), i);
      if (w >= thr) {
        const unsigned slot = atomicAdd(&s_count, 1u);
        if (slot < (unsigned)kTrMaxK) s_top[slot] = w;  // exactly `want` of these exist
      }
    }
  }
  // ---- sort and write out ------------------------------------------------------------------------------------
  int n2 = 2;
  while (n2 < want) n2 <<= 1;
  for (int i = want + tid; i < n2; i += kTrThreads) s_top[i] = 0ull;  // sorts last: no entry word is zero
  bitonic_desc(s_top, n2);
  for (int k = tid; k < K; k += kTrThreads) {
    if (k < want) {
      const int id = (int)~(uint32_t)(s_top[k] & 0xffffffffull);
      ids[k] = id;
      vals[k] = bf16_rne_bits(at(id));
    } else {
      ids[k] = -1;
      vals[k] = 0xff80u;  // -inf
    }
  }
}

// One wavefront per request, lane n = node n (Nq <= 64).  Children of a path node are tried in index order
// until one is kept (the acceptance step's order), so those before the kept one - or all, if none is kept -
// were tested and rejected (code 2); path nodes get code 1 and the token emitted after them; everything
// else 0 / -1.  The walk from the root is written per node: kc[p] is the first child of p whose mask is set;
// a node is on the path iff it is the root, or it is kc of a parent that is on the path (parents precede
// their children, so Nq rounds of that rule reach every node).
constexpr int kRecWaves = 4;
__global__ __launch_bounds__(kRecWaves * kWave) void trace_records_kernel(
    int B, int Nq, const int32_t* __restrict__ draft_tokens, const int32_t* __restrict__ parents,
    const int32_t* __restrict__ next_token, const uint8_t* __restrict__ accept_mask, int32_t* __restrict__ y_out,
    int8_t* __restrict__ traj) {
  __shared__ int s_par[kRecWaves][kMaxNq], s_kc[kRecWaves][kMaxNq];
  __shared__ unsigned char s_mask[kRecWaves][kMaxNq], s_on[kRecWaves][kMaxNq];
  const int wv = threadIdx.x / kWave, n = threadIdx.x % kWave;
  const int b = blockIdx.x * kRecWaves + wv;
  if (b >= B) return;  // whole wavefronts leave; the rest of the kernel has no workgroup barrier
  const bool node = n < Nq;
  const size_t at = (size_t)b * Nq + n;
  const int par = node ? (parents ? parents[at] : n - 1) : -1;
  const int tok = node ? draft_tokens[at] : -1;
  const int msk = node ? (accept_mask[at] != 0) : 0;
  const int nxt = next_token[b];
  if (node) {
    s_par[wv][n] = par;
    s_mask[wv][n] = (unsigned char)msk;
    s_on[wv][n] = n == 0;
  }
  __builtin_amdgcn_wave_barrier();  // LDS operations of one wavefront execute in order
  int kc = Nq;  // first kept child of node n
  if (node)
    for (int c = Nq - 1; c > n; --c)
      if (s_par[wv][c] == n && s_mask[wv][c]) kc = c;
  if (node) s_kc[wv][n] = kc;
  const int tok_kc = __shfl(tok, kc < Nq ? kc : 0, kWave);  // all 64 lanes are still active here
  __builtin_amdgcn_wave_barrier();
  bool on = n == 0;
  for (int round = 1; round < Nq; ++round) {
    if (node && n > 0 && !on && par >= 0 && par < n) on = msk && s_on[wv][par] && s_kc[wv][par] == n;
    if (node) s_on[wv][n] = on;
    __builtin_amdgcn_wave_barrier();
  }
  if (!node) return;
  int code = 0, y = -1;
  if (on) {
    code = 1;
    y = kc < Nq ? tok_kc : nxt;
  } else if (n > 0 && par >= 0 && par < n && s_on[wv][par] && n < s_kc[wv][par]) {
    code = 2;
  }
  y_out[at] = y;
  traj[at] = (int8_t)code;
}

hipError_t launch_trace_topk(const float* logits, int64_t rows, int V, int K, const int32_t* map, int n_map,
                             int32_t* ids, uint16_t* vals, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  if (map)
    hipLaunchKernelGGL(trace_topk_kernel<true>, dim3((unsigned)rows), dim3(kTrThreads), 0, st, logits, V, n_map, K, map,
                       ids, vals);
  else
    hipLaunchKernelGGL(trace_topk_kernel<false>, dim3((unsigned)rows), dim3(kTrThreads), 0, st, logits, V, V, K,
                       (const int32_t*)nullptr, ids, vals);
  return hipGetLastError();
}

hipError_t launch_trace_records(int B, int Nq, const int32_t* draft_tokens, const int32_t* parents,
                                const int32_t* next_token, const uint8_t* accept_mask, int32_t* y_out, int8_t* traj,
                                hipStream_t st) {
  if (B <= 0) return hipSuccess;
  hipLaunchKernelGGL(trace_records_kernel, dim3((B + kRecWaves - 1) / kRecWaves), dim3(kRecWaves * kWave), 0, st, B, Nq, draft_tokens, parents,
                     next_token, accept_mask, y_out, traj);
  return hipGetLastError();
}

int trace_max_k() { return kTrMaxK; }

}  // namespace aurora
