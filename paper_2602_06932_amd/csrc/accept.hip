// Acceptance walk and residual / bonus draw of the verification step (paper sections 2.1, 3.1,
// 3.3: the target keeps a prefix of the drafted chain - or a root-to-node path of the drafted
// tree - and emits one more token; accepted and rejected positions are both reported).
//
// One workgroup of 1024 threads per request.  Inputs are the fp32 logits written by the LM-head
// kernel and the per-(row, vocab tile) softmax statistics (max, sum exp, arg-max).
//   1. merge the tile statistics of each of the request's Nq rows into (max, logsumexp, arg-max);
//   2. walk: children of the current node in ascending index; the test u * q(tok) < p(tok) is
//      evaluated by thread 0 in fp64; after a rejection the whole workgroup sweeps the row pair
//      (logits, q) once to get the residual mass Z of max(0, p - q) and its sums over groups of
//      consecutive tokens;
//   3. inverse-CDF draw: exclusive scan of the group sums, pick the group the threshold u * total
//      falls in, rescan that group with a wavefront prefix sum to find the token.
// All sums are fp64 with a fixed reduction order, so results are reproducible bit for bit.
#include "common.hpp"
#include "launch.hpp"

namespace aurora {

constexpr int kAccThreads = 1024;
constexpr int kAccWaves = kAccThreads / kWave;
constexpr int kMaxGroups = 4096;  // group sums kept in LDS (32 KB of doubles)

// Probability mass of token v at the current node after `nres` residual steps.
// p0 = exp(l / T - lse);  p_{s+1} = max(0, p_s - q) / Z_s.  skip_last leaves the last step
// unnormalised (the weights whose sum is Z_{nres-1}).
__device__ __forceinline__ double node_weight(float l, float qv, double lse, double T, int nres, const double* Zs,
                                              bool skip_last) {
  double x = exp((double)l / T - lse);
  for (int s = 0; s < nres; ++s) {
    x = fmax(0.0, x - (double)qv);
    if (!(skip_last && s == nres - 1)) x /= Zs[s];
  }
  return x;
}

__device__ __forceinline__ double wave_incl_scan(double x, int lane) {
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const double y = __shfl_up(x, o, kWave);
    if (lane >= o) x += y;
  }
  return x;
}

// Sum over the workgroup in a fixed order; result returned to every thread.  `buf` holds kAccWaves doubles.
__device__ __forceinline__ double block_sum(double x, double* buf, int lane, int wv) {
  x = wave_sum(x);
  __syncthreads();
  if (lane == 0) buf[wv] = x;
  __syncthreads();
  double t = 0.0;
  for (int i = 0; i < kAccWaves; ++i) t += buf[i];
  return t;
}

struct AcceptParams {
  int Nq, V, n_tiles;
  float temperature;
  const float* logits;
  const float* pmax;
  const float* psum;
  const int32_t* parg;
  const int32_t* tok;
  const float* q;
  const float* un;
  const int32_t* parents;
  int32_t* accept_len;
  int32_t* next_token;
  uint8_t* accept_mask;
  float* p_at_draft;
  float* row_lse;
};

__global__ __launch_bounds__(kAccThreads) void accept_kernel(AcceptParams P) {
  __shared__ double s_lse[kMaxNq];
  __shared__ float s_max[kMaxNq];
  __shared__ int s_arg[kMaxNq];
  __shared__ double s_Z[kMaxNq];
  __shared__ double s_gsum[kMaxGroups];
  __shared__ double s_wtot[kAccWaves];
  __shared__ double s_red[kAccWaves];
  __shared__ int s_cur, s_depth, s_nres, s_last_child, s_state, s_have_gsum, s_exact_node, s_pick, s_lastpos;
  __shared__ double s_lse_cur, s_pick_prefix;

  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  const int Nq = P.Nq, V = P.V, nt = P.n_tiles;
  const bool greedy = !(P.temperature > 0.f);
  const double T = greedy ? 1.0 : (double)P.temperature;
  const size_t row0 = (size_t)b * Nq;

  // ---- 1. per-row (max, logsumexp, arg-max) from the tile statistics -----------------------
  for (int n = wv; n < Nq; n += kAccWaves) {
    const float* pm = P.pmax + (row0 + n) * nt;
    const float* ps = P.psum + (row0 + n) * nt;
    float mx = -INFINITY;
    int mt = 0x7fffffff;
    for (int t = lane; t < nt; t += kWave) {
      const float x = pm[t];
      if (x > mx) { mx = x; mt = t; }
    }
    for (int o = 32; o > 0; o >>= 1) {
      const float om = __shfl_xor(mx, o, kWave);
      const int ot = __shfl_xor(mt, o, kWave);
      if (om > mx || (om == mx && ot < mt)) { mx = om; mt = ot; }
    }
    double s = 0.0;
    for (int t = lane; t < nt; t += kWave) s += (double)ps[t] * exp(((double)pm[t] - (double)mx) / T);
    s = wave_sum(s);
    if (lane == 0) {
      s_max[n] = mx;
      s_arg[n] = P.parg[(row0 + n) * nt + mt];
      s_lse[n] = (double)mx / T + log(s);
    }
  }
  __syncthreads();

  // ---- optional per-node outputs ---------------------------------------------------------------
  if (tid < Nq) {
    const int n = tid;
    if (P.row_lse) P.row_lse[row0 + n] = (float)s_lse[n];
    if (P.p_at_draft) {
      float pv = 0.f;
      if (n > 0) {
        const int par = P.parents ? P.parents[row0 + n] : n - 1;
        const int tk = P.tok[row0 + n];
        if (greedy) pv = (tk == s_arg[par]) ? 1.f : 0.f;
        else pv = (float)exp((double)P.logits[(row0 + par) * V + tk] / T - s_lse[par]);
      }
      P.p_at_draft[row0 + n] = pv;
    }
    P.accept_mask[row0 + n] = n == 0 ? 1 : 0;
  }
  __syncthreads();

  // ---- 2a. greedy walk: thread 0 only -----------------------------------------------------------
  if (greedy) {
    if (tid == 0) {
      int cur = 0, depth = 0;
      for (;;) {
        int moved = 0;
        for (int c = cur + 1; c < Nq && !moved; ++c) {
          const int par = P.parents ? P.parents[row0 + c] : c - 1;
          if (par == cur && P.tok[row0 + c] == s_arg[cur]) {
            cur = c;
            ++depth;
            P.accept_mask[row0 + c] = 1;
            moved = 1;
          }
        }
        if (!moved) break;
      }
      P.accept_len[b] = depth;
      P.next_token[b] = s_arg[cur];
    }
    return;
  }

  // ---- 2b. sampling walk ------------------------------------------------------------------------
  const int gmul = (V + kWave * kMaxGroups - 1) / (kWave * kMaxGroups);
  const int GE = kWave * gmul;               // tokens per group
  const int ngroups = (V + GE - 1) / GE;     // <= kMaxGroups
  if (tid == 0) {
    s_cur = 0; s_depth = 0; s_nres = 0; s_last_child = 0; s_have_gsum = 0; s_exact_node = -1;
    s_lse_cur = s_lse[0];
  }
  enum { ST_DONE = 0, ST_ACCEPTED = 1, ST_REJECTED = 2 };
  for (;;) {
    __syncthreads();
    if (tid == 0) {
      const int cur = s_cur;
      int c = s_last_child + 1;
      for (; c < Nq; ++c) {
        const int par = P.parents ? P.parents[row0 + c] : c - 1;
        if (par == cur) break;
      }
      if (c >= Nq) {
        s_state = ST_DONE;
      } else {
        const int tk = P.tok[row0 + c];
        const float l = P.logits[(row0 + cur) * V + tk];
        const float qv = P.q[(row0 + cur) * V + tk];
        const double p = node_weight(l, qv, s_lse_cur, T, s_nres, s_Z, false);
        const double u = (double)P.un[(row0 + c) * 2 + 0];
        s_last_child = c;
        if (u * (double)qv < p) {
          s_cur = c;
          s_depth = s_depth + 1;
          s_nres = 0;
          s_have_gsum = 0;
          s_lse_cur = s_lse[c];
          s_exact_node = -1;
          P.accept_mask[row0 + c] = 1;
          s_state = ST_ACCEPTED;
        } else {
          s_state = ST_REJECTED;
        }
      }
    }
    __syncthreads();
    const int state = s_state;
    if (state == ST_ACCEPTED) continue;

    const int cur = s_cur;
    const float* lrow = P.logits + (row0 + cur) * V;
    const float* qrow = P.q + (row0 + cur) * V;
    const bool need_sweep = state == ST_REJECTED || !s_have_gsum;

    if (need_sweep && s_exact_node != cur) {
      // logsumexp of this row again, now in fp64 straight from the fp32 logits, so that the
      // row's probabilities sum to one to fp64 accuracy before differences with q are taken
      const double mx = (double)s_max[cur];
      double acc = 0.0;
      for (int v = tid; v < V; v += kAccThreads) acc += exp(((double)lrow[v] - mx) / T);
      const double tot = block_sum(acc, s_red, lane, wv);
      if (tid == 0) {
        s_lse_cur = mx / T + log(tot);
        s_exact_node = cur;
      }
      __syncthreads();
    }

    if (need_sweep) {
      // group sums of the weights: after a rejection the unnormalised next residual level,
      // otherwise (nothing rejected at this node, or its residual vanished) the current level
      const int nres = state == ST_REJECTED ? s_nres + 1 : s_nres;
      const bool skip_last = state == ST_REJECTED;
      const double lse = s_lse_cur;
      int lastpos = -1;
      for (int g = wv; g < ngroups; g += kAccWaves) {
        double acc = 0.0;
        for (int it = 0; it < gmul; ++it) {
          const int v = g * GE + it * kWave + lane;
          if (v < V) {
            const double x = node_weight(lrow[v], qrow[v], lse, T, nres, s_Z, skip_last);
            acc += x;
            if (x > 0.0) lastpos = v;
          }
        }
        acc = wave_sum(acc);
        if (lane == 0) s_gsum[g] = acc;
      }
      lastpos = wave_max(lastpos);
      if (tid == 0) s_lastpos = -1;
      __syncthreads();
      if (lane == 0) atomicMax(&s_lastpos, lastpos);
      __syncthreads();
    }

    // exclusive scan of the group sums: thread t owns groups 4t .. 4t+3
    double mine[4];
    double loc = 0.0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int g = tid * 4 + i;
      mine[i] = g < ngroups ? s_gsum[g] : 0.0;
      loc += mine[i];
    }
    const double incl = wave_incl_scan(loc, lane);
    if (lane == kWave - 1) s_wtot[wv] = incl;
    __syncthreads();
    double wbase = 0.0, total = 0.0;
    for (int i = 0; i < kAccWaves; ++i) {
      if (i < wv) wbase += s_wtot[i];
      total += s_wtot[i];
    }
    const double excl = wbase + incl - loc;

    if (state == ST_REJECTED) {
      __syncthreads();
      if (tid == 0) {
        if (total > 0.0) {
          s_Z[s_nres] = total;
          s_nres = s_nres + 1;
          s_have_gsum = 1;
        } else {
          s_have_gsum = 0;  // residual vanished: the distribution is left as it was
        }
      }
      continue;
    }

    // ---- 3. state == ST_DONE: inverse-CDF draw --------------------------------------------------
    const double u = (double)P.un[(row0 + cur) * 2 + 1];
    const double thr = u * total;
    if (tid == 0) s_pick = 0x7fffffff;
    __syncthreads();
    {
      double run = excl;
      int found = 0x7fffffff;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int g = tid * 4 + i;
        run += mine[i];
        if (g < ngroups && found == 0x7fffffff && run > thr) found = g;
      }
      if (found != 0x7fffffff) atomicMin(&s_pick, found);
    }
    __syncthreads();
    const int pick = s_pick;
    if (pick != 0x7fffffff && pick / 4 == tid) {
      double run = excl;
      for (int i = 0; i < pick % 4; ++i) run += mine[i];
      s_pick_prefix = run;
    }
    __syncthreads();
    if (wv == 0) {
      int token = s_lastpos;  // rounding left no crossing: the largest token with positive weight
      if (pick != 0x7fffffff) {
        const bool have = s_have_gsum;
        const int nres = s_nres;
        const double lse = s_lse_cur;
        double run = s_pick_prefix;
        int last_in_group = -1;
        bool done = false;
        for (int it = 0; it < gmul && !done; ++it) {
          const int v = pick * GE + it * kWave + lane;
          const double x = v < V ? node_weight(lrow[v], qrow[v], lse, T, nres, s_Z, have) : 0.0;
          const double inc = wave_incl_scan(x, lane) + run;
          const unsigned long long hit = __ballot(v < V && inc > thr);
          const unsigned long long pos = __ballot(x > 0.0);
          if (hit) {
            token = pick * GE + it * kWave + (__ffsll((long long)hit) - 1);
            done = true;
          } else {
            if (pos) last_in_group = pick * GE + it * kWave + (63 - __clzll((long long)pos));
            run = __shfl(inc, kWave - 1, kWave);
          }
        }
        if (!done && last_in_group >= 0) token = last_in_group;
      }
      if (lane == 0) {
        P.next_token[b] = token;
        P.accept_len[b] = s_depth;
      }
    }
    return;
  }
}

hipError_t launch_accept(const AcceptLaunch& a, hipStream_t st) {
  AcceptParams P;
  P.Nq = a.Nq; P.V = a.V; P.n_tiles = a.plan.n_tiles; P.temperature = a.temperature;
  P.logits = a.logits; P.pmax = a.pmax; P.psum = a.psum; P.parg = a.parg;
  P.tok = a.draft_tokens; P.q = a.draft_probs; P.un = a.uniforms; P.parents = a.parents;
  P.accept_len = a.accept_len; P.next_token = a.next_token; P.accept_mask = a.accept_mask;
  P.p_at_draft = a.p_at_draft; P.row_lse = a.row_lse;
  hipLaunchKernelGGL(accept_kernel, dim3(a.B), dim3(kAccThreads), 0, st, P);
  return hipGetLastError();
}

}  // namespace aurora
