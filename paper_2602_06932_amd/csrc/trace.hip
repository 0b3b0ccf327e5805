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
// With group maxima from the LM-head sweep (the largest logit of every 32 consecutive ids): the K-th largest of
// those maxima is a cut-off that at least K entries of the row reach - the maxima themselves are K distinct
// entries - and only about 1.2 K do.  Entries at or above it can only sit in the groups whose maximum reaches it,
// about K of them: those 128-byte groups are gathered and the rest of the row is never read (a quarter of the
// bytes, and nothing is sampled).
// Without them, one pass over the whole row: a cut-off key is selected from a sample of 4096 entries (1024
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
  if (x != x) return 0u;        // NaN ranks below everything on every route (the streamed pass never keeps one)
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

__device__ __forceinline__ unsigned wave_umax(unsigned v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v = max(v, (unsigned)__shfl_xor((int)v, o, kWave));
  return v;
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

// One wavefront per request, lane n = node n (Nq <= 64).  Children of a path node are tried in index order
// until one is kept (the acceptance step's order), so those before the kept one - or all, if none is kept -
// were tested and rejected (code 2); path nodes get code 1 and the token emitted after them; everything
// else 0 / -1.  The walk from the root is written per node: kc[p] is the first child of p whose mask is set;
// a node is on the path iff it is the root, or it is kc of a parent that is on the path (parents precede
// their children, so Nq rounds of that rule reach every node).

// One wavefront: request b, lane n = node n.  `lds` is kRecLds bytes private to the wavefront.
constexpr int kRecLds = kMaxNq * (4 + 4 + 1 + 1);
__device__ __forceinline__ void trace_records_wave(const RecArgs& R, int b, int n, char* lds) {
  int* s_par = (int*)lds;
  int* s_kc = s_par + kMaxNq;
  unsigned char* s_mask = (unsigned char*)(s_kc + kMaxNq);
  unsigned char* s_on = s_mask + kMaxNq;
  const int Nq = R.Nq;
  const bool node = n < Nq;
  const size_t at = (size_t)b * Nq + n;
  const int par = node ? (R.parents ? R.parents[at] : n - 1) : -1;
  const int tok = node ? R.draft_tokens[at] : -1;
  const int msk = node ? (R.accept_mask[at] != 0) : 0;
  const int nxt = R.next_token[b];
  if (node) {
    s_par[n] = par;
    s_mask[n] = (unsigned char)msk;
    s_on[n] = n == 0;
  }
  __builtin_amdgcn_wave_barrier();  // LDS operations of one wavefront execute in order
  int kc = Nq;  // first kept child of node n
  if (node)
    for (int c = Nq - 1; c > n; --c)
      if (s_par[c] == n && s_mask[c]) kc = c;
  if (node) s_kc[n] = kc;
  const int tok_kc = __shfl(tok, kc < Nq ? kc : 0, kWave);  // all 64 lanes are still active here
  __builtin_amdgcn_wave_barrier();
  bool on = n == 0;
  for (int round = 1; round < Nq; ++round) {
    if (node && n > 0 && !on && par >= 0 && par < n) on = msk && s_on[par] && s_kc[par] == n;
    if (node) s_on[n] = on;
    __builtin_amdgcn_wave_barrier();
  }
  if (!node) return;
  int code = 0, y = -1;
  if (on) {
    code = 1;
    y = kc < Nq ? tok_kc : nxt;
  } else if (n > 0 && par >= 0 && par < n && s_on[par] && n < s_kc[par]) {
    code = 2;
  }
  R.y_out[at] = y;
  R.traj[at] = (int8_t)code;
}

constexpr int kRecWaves = 4;
__global__ __launch_bounds__(kRecWaves * kWave) void trace_records_kernel(RecArgs R) {
  __shared__ __attribute__((aligned(16))) char s_rec[kRecWaves][kRecLds];
  const int wv = threadIdx.x / kWave, n = threadIdx.x % kWave;
  const int b = blockIdx.x * kRecWaves + wv;
  if (b >= R.B) return;  // whole wavefronts leave; the rest of the kernel has no workgroup barrier
  trace_records_wave(R, b, n, s_rec[wv]);
}

// kMapped: the selection runs over the V entries row[map[0]], .., row[map[V-1]] of a row of Vrow logits
// (the draft vocabulary, appendix A.2) and the ids written are positions in that list.
// kGroups: group_max[row][g] is the largest of the row's entries 32 g .. 32 g + 31 (those below V), for every
// g < ceil(V / 32); K <= n_groups <= 2 kTrCap, n_groups the row pitch of group_max (not with kMapped: maxima
// over the whole row say nothing about a subset of it).
// kOcc: workgroups per compute unit the kernel is built for.  Up to one row per compute unit (kOcc = 1) a thread
// keeps sixteen 16-byte loads of the row in flight; with more rows than units two workgroups share a unit.
template <bool kMapped, bool kGroups, int kOcc>
__global__ __launch_bounds__(kTrThreads, kOcc) void trace_topk_kernel(const float* __restrict__ logits, int Vrow, int V, int K,
                                                               const int32_t* __restrict__ map,
                                                               const float* __restrict__ group_max, int n_groups,
                                                               int32_t* __restrict__ out_ids,
                                                               uint16_t* __restrict__ out_vals, int rows, RecArgs R) {
  __shared__ uint64_t s_cand[kTrCap];   // 32 KB: the sample (as 32-bit keys), then the candidate list
  __shared__ uint64_t s_buck[kTrCap];   // 32 KB: the list regrouped by value range (bucket ranking)
  // workgroups past the token rows write the records (y_out, rejection trajectory): one wavefront per request
  if ((int)blockIdx.x >= rows) {
    const int wv = threadIdx.x / kWave;
    const int b = ((int)blockIdx.x - rows) * (kTrThreads / kWave) + wv;
    if (b < R.B) trace_records_wave(R, b, threadIdx.x % kWave, (char*)s_cand + wv * ((kRecLds + 15) & ~15));
    return;
  }
  uint64_t* s_top = s_buck;             // the whole-row route keeps its K selected words here
  __shared__ SelectShared s_sel;
  __shared__ unsigned s_count;
  __shared__ unsigned s_kmax, s_nkmin, s_big;
  __shared__ unsigned long long s_scale;
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
    uint32_t cut;
    if constexpr (kGroups) {
      // the K-th largest group maximum: K distinct entries of the row are at or above it
      const int used = (V + 31) >> 5;  // groups that hold entries; the others are padding
      const float* gm = group_max + (size_t)blockIdx.x * n_groups;
      for (int i = tid; i < used; i += kTrThreads) s_sample[i] = order_key(gm[i]);
      cut = (uint32_t)radix_threshold<32, 16>(s_sel, used, want, [&](int i) { return (uint64_t)s_sample[i]; });
      __syncthreads();
      if (tid == 0) s_count = 0;
      __syncthreads();
      // the groups that can hold an entry at or above the cut-off
      int* s_list = (int*)s_buck;  // up to 2 kTrCap group numbers
      for (int i = tid; i < used; i += kTrThreads)
        if (s_sample[i] >= cut) s_list[atomicAdd(&s_count, 1u)] = i;
      __syncthreads();
      const int ngl = (int)s_count;
      __syncthreads();
      if (tid == 0) s_count = 0;
      __syncthreads();  // the keys are dead from here on: s_cand takes the candidates
      float cut_f;
      {
        const uint32_t u = (cut & 0x80000000u) ? (cut ^ 0x80000000u) : ~cut;
        cut_f = __uint_as_float(u);
        if (cut_f != cut_f) cut_f = -INFINITY;
      }
      // eight lanes per group, 16 bytes each; eight groups in flight per lane
      const int oct = tid >> 3, ol = tid & 7;
      const bool vec_ok = (((uintptr_t)row | ((size_t)V * sizeof(float))) & 15) == 0;
      constexpr int kG = 8, kOcts = kTrThreads / 8;
      for (int j0 = oct; j0 < ngl; j0 += kG * kOcts) {
        f32x4_t x[kG];
        int e0[kG];
#pragma unroll
        for (int u = 0; u < kG; ++u) {
          const int j = j0 + u * kOcts;
          e0[u] = j < ngl ? s_list[j] * 32 + ol * 4 : V;  // first of this lane's four entries (V: nothing to read)
          if (e0[u] + 3 < V && vec_ok) {
            x[u] = *(const f32x4_t*)(row + e0[u]);
          } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) x[u][q] = e0[u] + q < V ? row[e0[u] + q] : -INFINITY;
          }
        }
#pragma unroll
        for (int u = 0; u < kG; ++u)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            if (e0[u] + q < V && x[u][q] >= cut_f) {
              const unsigned slot = atomicAdd(&s_count, 1u);
              if (slot < (unsigned)kTrCap) s_cand[slot] = entry_word(x[u][q], e0[u] + q);
            }
      }
      __syncthreads();
      count = (int)s_count;
      from_row = count < want || count > kTrCap;
    } else {
      const int vstride = nvec / (kTrCap / 4);
      const int vi = vstride ? tid * vstride : (tid < nvec ? tid : nvec - 1);
      const f32x4_t x = load4(vi);
#pragma unroll
      for (int j = 0; j < 4; ++j) s_sample[4 * tid + j] = order_key(x[j]);
      // sample rank whose key is expected to have about 2K row entries at or above it (always < kTrCap); the
      // cut-off only needs the key's upper 16 bits (sign, exponent, 7 mantissa bits): a few more entries pass
      const int r = (int)((2ll * K * kTrCap + V - 1) / V) + 8;
      cut = (uint32_t)radix_threshold<32, 16>(s_sel, kTrCap, r + 1, [&](int i) { return (uint64_t)s_sample[i]; });
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
    constexpr int kU = kOcc == 1 ? 16 : 8;
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
    }  // without group maxima
  }

  // ---- a list that fits is ranked in place: bucket by value range, count the larger words inside the bucket ----
  // Words are distinct, so the rank of a word (how many are larger) is its position in the output.  The upper 32
  // bits of a word are an order-preserving key of the value: a monotone map of the key onto 256 buckets (linear
  // between the smallest and the largest key of the list, highest values first) keeps the order between buckets,
  // and inside a bucket - a few dozen words for logits of an LM head - ranks come from direct comparison.  A bucket
  // of more than 256 words (heavy ties) sends the list to the radix select and bitonic sort below instead.
  __syncthreads();
  if (!from_row) {
    constexpr int kPer = kTrCap / kTrThreads;  // list entries per thread
    if (tid < 256) s_sel.hist[tid] = 0;
    if (tid == 0) { s_kmax = 0u; s_nkmin = 0u; s_big = 0u; }
    __syncthreads();
    uint64_t w[kPer];
    unsigned kmin_l = 0xffffffffu, kmax_l = 0u;
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const int i = tid + e * kTrThreads;
      w[e] = i < count ? s_cand[i] : 0ull;
      if (i < count) {
        const unsigned k = (unsigned)(w[e] >> 32);
        kmin_l = min(kmin_l, k);
        kmax_l = max(kmax_l, k);
      }
    }
    // the smallest key is found as the largest of the complements: one atomicMax per wavefront each
    kmax_l = wave_umax(kmax_l);
    const unsigned nkmin_l = wave_umax(~kmin_l);
    if ((tid & 63) == 0) { atomicMax(&s_kmax, kmax_l); atomicMax(&s_nkmin, nkmin_l); }
    __syncthreads();
    const unsigned kmax = s_kmax, kmin = ~s_nkmin;
    if (tid == 0) {
      const unsigned long long range = (unsigned long long)(kmax - kmin) + 1ull;
      s_scale = range <= 256ull ? 0ull : ((256ull << 32) / range);  // 0: the key offset is the bucket
    }
    __syncthreads();
    const unsigned long long scale = s_scale;
    int bucket[kPer], pos[kPer];
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
      const int i = tid + e * kTrThreads;
      bucket[e] = 0; pos[e] = 0;
      if (i < count) {
        const unsigned d = (unsigned)(w[e] >> 32) - kmin;
        const unsigned up = scale ? (unsigned)(((unsigned long long)d * scale) >> 32) : d;  // 0 .. 255, rising with the value
        bucket[e] = 255 - (int)up;                                                           // highest values first
        pos[e] = atomicAdd(&s_sel.hist[bucket[e]], 1);
      }
    }
    __syncthreads();
    if (tid < kWave) {
      // exclusive scan of the 256 bucket sizes (four per lane), in place; remember whether a bucket is too large
      int c[4], tot = 0, big = 0;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) { c[jj] = s_sel.hist[4 * tid + jj]; tot += c[jj]; big |= c[jj] > 256; }
      int incl = tot;
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const int y = __shfl_up(incl, o, kWave);
        if (tid >= o) incl += y;
      }
      int run = incl - tot;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) { s_sel.hist[4 * tid + jj] = run; run += c[jj]; }
      if (big) s_big = 1u;
    }
    __syncthreads();
    if (!s_big) {
      // bucket b occupies s_buck[hist[b] .. hist[b + 1]) (the last one ends at count)
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        const int i = tid + e * kTrThreads;
        if (i < count) s_buck[s_sel.hist[bucket[e]] + pos[e]] = w[e];
      }
      __syncthreads();
#pragma unroll
      for (int e = 0; e < kPer; ++e) {
        const int i = tid + e * kTrThreads;
        if (i < count) {
          const int lo = s_sel.hist[bucket[e]];
          const int hi = bucket[e] == 255 ? count : s_sel.hist[bucket[e] + 1];
          int rank = lo;
          for (int jj = lo; jj < hi; ++jj) rank += s_buck[jj] > w[e];
          if (rank < want) {
            const int id = (int)~(uint32_t)(w[e] & 0xffffffffull);
            const uint32_t key = (uint32_t)(w[e] >> 32);
            const uint32_t bits = (key & 0x80000000u) ? (key ^ 0x80000000u) : ~key;  // the value, but for the sign of a zero
            ids[rank] = id;
            vals[rank] = bf16_rne_bits((bits << 1) ? __uint_as_float(bits) : at(id));
          }
        }
      }
      for (int k = want + tid; k < K; k += kTrThreads) {
        ids[k] = -1;
        vals[k] = 0xff80u;  // -inf
      }
      return;
    }
    __syncthreads();
  }
  // ---- cut to exactly `want` words and compact them into s_top ------------------------------------------
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

// Top-K rows and, when `rec` is given, the records in the same launch (extra workgroups at the end of the grid).
hipError_t launch_trace_topk(const float* logits, int64_t rows, int V, int K, const int32_t* map, int n_map,
                             const float* group_max, int n_groups, int32_t* ids, uint16_t* vals, const RecArgs* rec,
                             hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  const int want = K < V ? K : V;
  int cus = 0;
  if (hipError_t e = device_cu_count(&cus); e != hipSuccess) return e;
  const bool one_per_unit = rows <= cus;
  const int used = (V + 31) / 32;  // groups of 32 consecutive ids that hold entries
  const bool groups = !map && group_max && V > kTrCap && used >= want && n_groups >= used && used <= 2 * kTrCap;
  RecArgs R = {};
  if (rec) R = *rec;
  constexpr int per_wg = kTrThreads / kWave;
  const unsigned grid = (unsigned)rows + (unsigned)((R.B + per_wg - 1) / per_wg);
#define AURORA_TOPK_LAUNCH(M_, G_, O_, Vsel, MAP, GM, NG)                                                            \
  hipLaunchKernelGGL((trace_topk_kernel<M_, G_, O_>), dim3(grid), dim3(kTrThreads), 0, st, logits, V, Vsel, K, MAP, GM, NG, \
                     ids, vals, (int)rows, R)
  if (map) {
    if (one_per_unit) AURORA_TOPK_LAUNCH(true, false, 1, n_map, map, (const float*)nullptr, 0);
    else AURORA_TOPK_LAUNCH(true, false, 2, n_map, map, (const float*)nullptr, 0);
  } else if (groups) {
    if (one_per_unit) AURORA_TOPK_LAUNCH(false, true, 1, V, (const int32_t*)nullptr, group_max, n_groups);
    else AURORA_TOPK_LAUNCH(false, true, 2, V, (const int32_t*)nullptr, group_max, n_groups);
  } else {
    if (one_per_unit) AURORA_TOPK_LAUNCH(false, false, 1, V, (const int32_t*)nullptr, (const float*)nullptr, 0);
    else AURORA_TOPK_LAUNCH(false, false, 2, V, (const int32_t*)nullptr, (const float*)nullptr, 0);
  }
#undef AURORA_TOPK_LAUNCH
  return hipGetLastError();
}

hipError_t launch_trace_records(const RecArgs& R, hipStream_t st) {
  if (R.B <= 0) return hipSuccess;
  hipLaunchKernelGGL(trace_records_kernel, dim3((R.B + kRecWaves - 1) / kRecWaves), dim3(kRecWaves * kWave), 0, st, R);
  return hipGetLastError();
}

int trace_max_k() { return kTrMaxK; }

}  // namespace aurora
