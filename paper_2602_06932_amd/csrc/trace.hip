// Trace emission after a verify step (paper section 3.1: accepted and rejected outcomes are both
// streamed to the training side; appendix A.1 eq. 4: a record is (h, l, x_in, y_out, R); appendix A.2:
// only the K = 1024 largest target logits of a token are kept, 2 bytes each).
//
//   trace_topk_kernel     one workgroup per token row: the K largest logits, ids ordered by value
//                         descending (equal values by ascending id), values rounded to bfloat16.
//   trace_records_kernel  y_out and the rejection trajectory R from the acceptance outputs.
//
// Selection.  A float is mapped to an unsigned key with the same order (-0.0 folded onto +0.0); a
// candidate is the 64-bit word (key << 32 | ~id), so one descending sort gives value order with the
// lowest id first among equals.  Common case, one pass over the row: a cut-off is taken from a sorted
// sample of 4096 entries so that about 2K entries pass it; the row is streamed once (16-byte loads),
// the few entries at or above the cut-off are appended to a list in LDS, the list is sorted there
// (bitonic) and its first K entries are the answer.  If the list comes out shorter than K or longer
// than its capacity (heavily repeated values, adversarial rows), an exact radix select over the keys
// (four passes of 8 bits, LDS histograms) finds the K-th key, and the entries above it plus the first
// ones equal to it in id order are collected instead.  Both routes give the same, unique answer.
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

__device__ __forceinline__ uint16_t bf16_rne_bits(float f) {
  const uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) == 0x7f800000u) return (uint16_t)(u >> 16);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

// descending bitonic sort of n (a power of two, <= kTrCap) 64-bit words in LDS by the whole workgroup
__device__ __forceinline__ void bitonic_desc(uint64_t* a, int n) {
  for (int size = 2; size <= n; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      __syncthreads();
      for (int t = threadIdx.x; t < (n >> 1); t += kTrThreads) {
        const int lo = ((t / stride) * stride << 1) + (t % stride);
        const int hi = lo + stride;
        const bool desc = ((lo & size) == 0);
        const uint64_t x = a[lo], y = a[hi];
        if ((x < y) == desc) { a[lo] = y; a[hi] = x; }
      }
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(kTrThreads) void trace_topk_kernel(const float* __restrict__ logits, int V, int K,
                                                               int32_t* __restrict__ out_ids,
                                                               uint16_t* __restrict__ out_vals) {
  __shared__ uint64_t s_cand[kTrCap];  // 32 KB
  __shared__ int s_hist[256];
  __shared__ int s_scan[kTrThreads / 64];
  __shared__ unsigned s_count;
  __shared__ uint32_t s_prefix;
  __shared__ int s_remaining, s_eq_base;
  const int tid = threadIdx.x;
  const float* row = logits + (size_t)blockIdx.x * V;
  int32_t* ids = out_ids + (size_t)blockIdx.x * K;
  uint16_t* vals = out_vals + (size_t)blockIdx.x * K;
  const int want = K < V ? K : V;  // entries that exist
  int count;                       // entries in s_cand, sorted, after the selection below (>= want)

  if (V <= kTrCap) {
    // the whole row fits the list
    for (int i = tid; i < kTrCap; i += kTrThreads)
      s_cand[i] = i < V ? ((uint64_t)order_key(row[i]) << 32) | (uint32_t)~i : 0ull;
    count = V;
  } else {
    // ---- cut-off from a sorted sample --------------------------------------------------------------
    // the sample is sorted as 64-bit words with the key in the high half
    const int stride = V / kTrCap;
    for (int i = tid; i < kTrCap; i += kTrThreads) s_cand[i] = (uint64_t)order_key(row[(size_t)i * stride]) << 32;
    bitonic_desc(s_cand, kTrCap);
    // rank in the sample whose key is expected to have about 2K row entries at or above it
    long long r = (2ll * K * kTrCap + V - 1) / V + 8;
    uint32_t cut = 0;  // 0: below every key, everything passes (the list then overflows and the exact route runs)
    if (r < kTrCap) cut = (uint32_t)(s_cand[r] >> 32);
    __syncthreads();
    if (tid == 0) s_count = 0;
    __syncthreads();
    // ---- one pass over the row: keep what reaches the cut-off ------------------------------------------
    const int head = (int)(((16 - ((uintptr_t)row & 15)) & 15) >> 2);  // entries before the first 16-byte boundary
    const int h = head < V ? head : V;
    if (tid < h) {
      const uint32_t k = order_key(row[tid]);
      if (k >= cut) {
        const unsigned slot = atomicAdd(&s_count, 1u);
        if (slot < (unsigned)kTrCap) s_cand[slot] = ((uint64_t)k << 32) | (uint32_t)~tid;
      }
    }
    const int nvec = (V - h) >> 2;
    const float4* rv = (const float4*)(row + h);
    for (int i = tid; i < nvec; i += kTrThreads) {
      const float4 x = rv[i];
      const float e[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t k = order_key(e[j]);
        if (k >= cut) {
          const unsigned slot = atomicAdd(&s_count, 1u);
          if (slot < (unsigned)kTrCap) s_cand[slot] = ((uint64_t)k << 32) | (uint32_t) ~(h + 4 * i + j);
        }
      }
    }
    for (int i = h + 4 * nvec + tid; i < V; i += kTrThreads) {
      const uint32_t k = order_key(row[i]);
      if (k >= cut) {
        const unsigned slot = atomicAdd(&s_count, 1u);
        if (slot < (unsigned)kTrCap) s_cand[slot] = ((uint64_t)k << 32) | (uint32_t)~i;
      }
    }
    __syncthreads();
    count = (int)s_count;
    __syncthreads();
    if (count < want || count > kTrCap) {
      // ---- exact route: radix select of the want-th largest key, 8 bits per pass -----------------------
      if (tid == 0) { s_prefix = 0; s_remaining = want; }
      uint32_t mask = 0;
      for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) s_hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        for (int i = tid; i < V; i += kTrThreads) {
          const uint32_t k = order_key(row[i]);
          if ((k & mask) == prefix) atomicAdd(&s_hist[(k >> shift) & 255], 1);
        }
        __syncthreads();
        if (tid == 0) {
          int rem = s_remaining, d = 255;
          while (d > 0 && s_hist[d] < rem) { rem -= s_hist[d]; --d; }
          s_remaining = rem;  // entries still to take from digit d (>= 1, <= s_hist[d])
          s_prefix = prefix | ((uint32_t)d << shift);
        }
        mask |= 255u << shift;
        __syncthreads();
      }
      const uint32_t kth = s_prefix;      // the want-th largest key
      const int need_eq = s_remaining;    // entries equal to it that belong to the answer: the lowest ids
      if (tid == 0) { s_count = 0; s_eq_base = 0; }
      __syncthreads();
      // entries above the K-th key in any order; entries equal to it ranked in id order by a running scan
      for (int base = 0; base < V; base += kTrThreads) {
        const int i = base + tid;
        uint32_t k = 0;
        bool gt = false, eq = false;
        if (i < V) {
          k = order_key(row[i]);
          gt = k > kth;
          eq = k == kth;
        }
        if (gt) {
          const unsigned slot = atomicAdd(&s_count, 1u);
          // fewer than want <= kTrMaxK of these exist; the bound only guards the list against a broken row (NaN)
          if (slot < (unsigned)kTrCap) s_cand[slot] = ((uint64_t)k << 32) | (uint32_t)~i;
        }
        const unsigned long long bal = __ballot(eq);
        const int lane = tid & 63, wv = tid >> 6;
        if (lane == 0) s_scan[wv] = __popcll(bal);
        __syncthreads();
        int before = s_eq_base;
        for (int w2 = 0; w2 < wv; ++w2) before += s_scan[w2];
        const int rank = before + __popcll(bal & ((1ull << lane) - 1ull));
        if (eq && rank < need_eq) {
          const unsigned slot = atomicAdd(&s_count, 1u);
          if (slot < (unsigned)kTrCap) s_cand[slot] = ((uint64_t)k << 32) | (uint32_t)~i;
        }
        __syncthreads();
        if (tid == 0) {
          int tot = 0;
          for (int w2 = 0; w2 < kTrThreads / 64; ++w2) tot += s_scan[w2];
          s_eq_base += tot;
        }
        __syncthreads();
      }
      count = (int)s_count;  // == want
      if (count > kTrCap) count = kTrCap;
    }
  }
  // sort the list (padded to a power of two with words that sort last)
  int n2 = 2;
  while (n2 < count) n2 <<= 1;
  for (int i = count + tid; i < n2; i += kTrThreads) s_cand[i] = 0ull;
  bitonic_desc(s_cand, n2);
  for (int k = tid; k < K; k += kTrThreads) {
    if (k < want) {
      const int id = (int)~(uint32_t)(s_cand[k] & 0xffffffffull);
      ids[k] = id;
      vals[k] = bf16_rne_bits(row[id]);
    } else {
      ids[k] = -1;
      vals[k] = 0xff80u;  // -inf
    }
  }
}

// One thread per request: walk the accepted path from the root.  Children of a path node are tried in
// index order until one is kept (the acceptance step's order), so those before the kept one - or all,
// if none is kept - were tested and rejected (code 2); path nodes get code 1 and the token emitted
// after them; everything else 0 / -1.
__global__ void trace_records_kernel(int B, int Nq, const int32_t* __restrict__ draft_tokens,
                                     const int32_t* __restrict__ parents, const int32_t* __restrict__ next_token,
                                     const uint8_t* __restrict__ accept_mask, int32_t* __restrict__ y_out,
                                     int8_t* __restrict__ traj) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int32_t* tok = draft_tokens + (size_t)b * Nq;
  const uint8_t* mask = accept_mask + (size_t)b * Nq;
  int32_t* y = y_out + (size_t)b * Nq;
  int8_t* r = traj + (size_t)b * Nq;
  for (int n = 0; n < Nq; ++n) { y[n] = -1; r[n] = 0; }
  int cur = 0;
  r[0] = 1;
  for (;;) {
    int kept = -1;
    for (int c = cur + 1; c < Nq; ++c) {
      const int par = parents ? parents[(size_t)b * Nq + c] : c - 1;
      if (par != cur) continue;
      if (mask[c]) { kept = c; break; }
      r[c] = 2;
    }
    if (kept < 0) break;
    r[kept] = 1;
    y[cur] = tok[kept];
    cur = kept;
  }
  y[cur] = next_token[b];
}

hipError_t launch_trace_topk(const float* logits, int64_t rows, int V, int K, int32_t* ids, uint16_t* vals,
                             hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(trace_topk_kernel, dim3((unsigned)rows), dim3(kTrThreads), 0, st, logits, V, K, ids, vals);
  return hipGetLastError();
}

hipError_t launch_trace_records(int B, int Nq, const int32_t* draft_tokens, const int32_t* parents,
                                const int32_t* next_token, const uint8_t* accept_mask, int32_t* y_out, int8_t* traj,
                                hipStream_t st) {
  if (B <= 0) return hipSuccess;
  hipLaunchKernelGGL(trace_records_kernel, dim3((B + 127) / 128), dim3(128), 0, st, B, Nq, draft_tokens, parents,
                     next_token, accept_mask, y_out, traj);
  return hipGetLastError();
}

int trace_max_k() { return kTrMaxK; }

}  // namespace aurora
