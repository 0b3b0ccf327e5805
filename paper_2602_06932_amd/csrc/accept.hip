// Acceptance walk and residual / bonus draw of the verification step (paper sections 2.1, 3.1,
// 3.3: the target keeps a prefix of the drafted chain - or a root-to-node path of the drafted
// tree - and emits one more token; accepted and rejected positions are both reported).
//
// Inputs are the fp32 logits written by the LM-head kernel and the per-(row, vocab tile) softmax
// statistics (max, sum exp, arg-max) of its epilogue.
//
// Chains at T > 0 (the serving default) take two small kernels so that the one vocabulary sweep a
// request needs is spread over the whole chip instead of one compute unit:
//   accept_chain_sweep  S workgroups per request.  Each repeats the cheap part - merge the tile
//                       statistics of the request's rows, evaluate the k accept tests
//                       u * q(d) < p(d) in parallel (fp64), find the first failure - and then sums
//                       the draw weights - max(0, p - q) after a rejection, p itself when every
//                       draft was kept - over groups of 256 tokens of its slice; slice 0 writes
//                       accept_len / accept_mask / p_at_draft / row_lse;
//   accept_chain_pick   one workgroup per request: scan the group sums, find the group holding
//                       u * total, rescan that group with a wavefront prefix sum for the token.
// Trees at T > 0 may need one sweep per rejected sibling, each depending on the previous one:
// accept_tree_kernel walks a request in up to 16 workgroups that split every sweep and exchange their
// partial sums behind a counting barrier.  The same kernel, one workgroup per request, serves every
// greedy (T = 0) call, where no sweep exists.
// All sums are fp64 in a fixed order: results are reproducible bit for bit.
#include "common.hpp"
#include "launch.hpp"

namespace aurora {

constexpr int kAccThreads = 1024;
constexpr int kAccWaves = kAccThreads / kWave;
constexpr int kMaxGroups = 4096;  // group sums kept in LDS by the tree kernel (32 KB of doubles): V <= 2^20
constexpr int kSmallThreads = 256;
constexpr int kSweepThreads = 512;  // chain sweep: eight wavefronts, so five rows merge and a 32-group slice sweeps in one round
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// Probability of token v at the current node after `nres` residual steps, in fp64 throughout (used
// for the accept tests).  p0 = exp(l / T - lse);  p_{s+1} = max(0, p_s - q) / Z_s.
__device__ __forceinline__ double node_weight(float l, float qv, double lse, double T, int nres, const double* Zs) {
  double x = exp((double)l / T - lse);
  for (int s = 0; s < nres; ++s) x = fmax(0.0, x - (double)qv) / Zs[s];
  return x;
}

// The same quantity for the vocabulary sweeps.  The exponent is formed in fp64 (so the row's
// logsumexp enters unrounded), rounded once to fp32 and exponentiated by the hardware exp2, the
// function the LM-head epilogue used for the statistics lse was merged from - a bias of that
// function cancels between the two.  The fp32 rounding is an independent ~1e-7 relative
// perturbation per token and averages out of the running sums.  skip_last leaves the last residual
// step unnormalised (weights whose sum is Z_{nres-1}).  The normalisers enter as reciprocals: a
// multiplication per token and level instead of an fp64 division.
__device__ __forceinline__ double sweep_weight(float l, float qv, double lse, double inv_t, int nres,
                                               const double* invZs, bool skip_last) {
  const double a = ((double)l * inv_t - lse) * 1.4426950408889634;
  double x = (double)__builtin_amdgcn_exp2f((float)a);
  for (int s = 0; s < nres; ++s) {
    x = fmax(0.0, x - (double)qv);
    if (!(skip_last && s == nres - 1)) x *= invZs[s];
  }
  return x;
}

// Siblings drawn without replacement: the children of a node were drawn one after the other, each from the
// parent's q with the earlier siblings' tokens removed.  The draft distribution that residual level s was formed
// with is then q with the tokens rej[0 .. len[s]) set to zero, times fac[s] = 1 / (1 - their mass).
struct QLevels {
  const int* rej;
  const int* len;
  const double* fac;
};
__device__ __forceinline__ bool in_list(int v, const int* list, int n) {
  bool hit = false;
  for (int i = 0; i < n; ++i) hit |= list[i] == v;
  return hit;
}
__device__ __forceinline__ double node_weight_wor(float l, float qv, int v, double lse, double T, int nres, const double* Zs,
                                                  const QLevels& ql) {
  double x = exp((double)l / T - lse);
  for (int s = 0; s < nres; ++s) {
    const double qs = in_list(v, ql.rej, ql.len[s]) ? 0.0 : (double)qv * ql.fac[s];
    x = fmax(0.0, x - qs) / Zs[s];
  }
  return x;
}
__device__ __forceinline__ double sweep_weight_wor(float l, float qv, int v, double lse, double inv_t, int nres,
                                                   const double* invZs, bool skip_last, const QLevels& ql) {
  const double a = ((double)l * inv_t - lse) * 1.4426950408889634;
  double x = (double)__builtin_amdgcn_exp2f((float)a);
  for (int s = 0; s < nres; ++s) {
    const double qs = in_list(v, ql.rej, ql.len[s]) ? 0.0 : (double)qv * ql.fac[s];
    x = fmax(0.0, x - qs);
    if (!(skip_last && s == nres - 1)) x *= invZs[s];
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

struct AcceptParams {
  int Nq, V, n_tiles, slices, gmul, ngroups;
  float temperature;
  const float* logits;
  const float* pmax;
  const float* psum;
  const int32_t* parg;
  const int32_t* tok;
  const float* q;       // draft probabilities, row stride Vq
  const int32_t* t2d;   // target id -> index into a row of q, or -1 (q = 0 there); NULL: q rows are dense over V
  int Vq;               // entries per row of q: the draft vocabulary, or V
  const float* un;
  const int32_t* parents;
  int32_t* accept_len;
  int32_t* next_token;
  uint8_t* accept_mask;
  float* p_at_draft;
  float* row_lse;
  // scratch of the chain path
  double* st_lse;     // [B] logsumexp of the row the draw happens on
  int32_t* st_row;    // [B] that row (= accept_len)
  int32_t* st_rej;    // [B] 1: draw from max(0, p - q); 0: draw from p
  double* gsum;       // [B, ngroups]
  int32_t* lastpos;   // [B, slices] largest token with positive weight per slice, or -1
  // tree path with several workgroups per request: gsum is [B, 2, ngroups] and lastpos [B, 2, tree_slices]
  // (two copies, alternating by sweep), tree_bar [B] counts workgroup arrivals (zero at launch)
  int tree_slices;
  int32_t* tree_bar;
  const float* temps;  // [B] one temperature per request (0 = that request is verified greedily), or NULL
  int wor;             // tree walk: siblings were drawn without replacement
  int spin_limit;      // tree walk with several workgroups: polls of the arrival counter before giving up
};

// the temperature of request b: its own, or the call's
__device__ __forceinline__ float request_temperature(const AcceptParams& P, int b) {
  return P.temps ? P.temps[b] : P.temperature;
}

// (max, logsumexp(l / T), arg-max) of one logits row, merged from its tile statistics by one
// wavefront; result valid in every lane.  Each lane folds its tiles into a running (max, scaled
// sum) pair - the loads of eight tiles are issued together - then the lanes are folded by
// butterfly exchanges.  Scale factors go through the hardware exp2 of an fp64-formed exponent.
// kLanes = 32: the two halves of the wavefront merge two different rows at the same time (`row` then
// differs between the halves), so a workgroup gets through twice as many rows per round of loads.
template <int kLanes = kWave>
__device__ __forceinline__ void merge_row_stats(const AcceptParams& P, size_t row, double T, int lane, float* out_max,
                                                double* out_lse, int* out_arg, bool want_arg = true) {
  const int nt = P.n_tiles;
  const float* pm = P.pmax + row * nt;
  const float* ps = P.psum + row * nt;
  const double c = 1.4426950408889634 / T;
  const int sub = lane & (kLanes - 1);
  float m = -INFINITY;
  double s = 0.0;
  int mt = 0x7fffffff;
  for (int t0 = 0; t0 < nt; t0 += kLanes * 8) {
    float xm[8], xs[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int t = t0 + u * kLanes + sub;
      xm[u] = t < nt ? pm[t] : -INFINITY;
      xs[u] = t < nt ? ps[t] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (xm[u] > m) {
        s = s * (double)__builtin_amdgcn_exp2f((float)(((double)m - (double)xm[u]) * c)) + (double)xs[u];
        m = xm[u];
        mt = t0 + u * kLanes + sub;
      } else if (xm[u] > -INFINITY) {
        s += (double)xs[u] * (double)__builtin_amdgcn_exp2f((float)(((double)xm[u] - (double)m) * c));
      }
    }
  }
#pragma unroll
  for (int o = kLanes / 2; o > 0; o >>= 1) {
    const float om = __shfl_xor(m, o, kWave);
    const double os = __shfl_xor(s, o, kWave);
    const int ot = __shfl_xor(mt, o, kWave);
    const float nm = fmaxf(m, om);
    if (nm > -INFINITY) {
      const double fa = m > -INFINITY ? (double)__builtin_amdgcn_exp2f((float)(((double)m - (double)nm) * c)) : 0.0;
      const double fb = om > -INFINITY ? (double)__builtin_amdgcn_exp2f((float)(((double)om - (double)nm) * c)) : 0.0;
      s = s * fa + os * fb;
    }
    if (om > m || (om == m && ot < mt)) mt = ot;
    m = nm;
  }
  *out_max = m;
  *out_lse = (double)m / T + log(s);
  // the arg-max id sits behind one more dependent load; only greedy verification reads it
  *out_arg = want_arg ? P.parg[row * nt + mt] : 0;
}

// ============================================================================================
// Chain path.  A group is 256 consecutive tokens: lane i of the wavefront that owns it holds tokens
// 4i .. 4i+3 (one 16-byte load per row when the row is 16-byte aligned).
// ============================================================================================
constexpr int kGroup = 256;

// the logits and draft probabilities of the four tokens v0 .. v0+3 a lane owns
struct Lane4 { float l[4], q[4]; };
// One row of draft probabilities: dense over the target vocabulary, or compact over the draft vocabulary
// with the target -> draft index map (entries off the draft vocabulary have probability 0).
struct QRow {
  const float* row;
  const int32_t* t2d;
};
// 16-byte loads of the logits row and of the q row (or of the index map) are possible
__device__ __forceinline__ bool rows_vec_ok(const AcceptParams& P) {
  const uintptr_t qa = P.t2d ? (uintptr_t)P.t2d : (uintptr_t)P.q;
  return (P.V & 3) == 0 && ((qa | (uintptr_t)P.logits) & 15) == 0;
}
__device__ __forceinline__ QRow q_row(const AcceptParams& P, size_t r) { return QRow{P.q + r * (size_t)P.Vq, P.t2d}; }
__device__ __forceinline__ float q_at(const QRow& q, int v) {
  if (!q.t2d) return q.row[v];
  const int j = q.t2d[v];
  return j >= 0 ? q.row[j] : 0.f;
}
typedef __attribute__((ext_vector_type(4))) int i32x4_t;
__device__ __forceinline__ Lane4 lane_load(const float* __restrict__ lrow, const QRow& q, int v0, int V, bool vec_ok) {
  Lane4 r;
  if (vec_ok && v0 + 3 < V) {
    const f32x4_t lv = *(const f32x4_t*)(lrow + v0);
#pragma unroll
    for (int e = 0; e < 4; ++e) r.l[e] = lv[e];
    if (!q.t2d) {
      const f32x4_t qv = *(const f32x4_t*)(q.row + v0);
#pragma unroll
      for (int e = 0; e < 4; ++e) r.q[e] = qv[e];
    } else {
      const i32x4_t jv = *(const i32x4_t*)(q.t2d + v0);
#pragma unroll
      for (int e = 0; e < 4; ++e) r.q[e] = jv[e] >= 0 ? q.row[jv[e]] : 0.f;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      r.l[e] = v0 + e < V ? lrow[v0 + e] : -INFINITY;
      r.q[e] = v0 + e < V ? q_at(q, v0 + e) : 0.f;
    }
  }
  return r;
}
// their draw weights (0 past the end of the vocabulary)
__device__ __forceinline__ void lane_weights(const Lane4& r, int v0, int V, double lse, double inv_t, int nres,
                                             double x[4], const double* invZs = nullptr, bool skip_last = true) {
#pragma unroll
  for (int e = 0; e < 4; ++e)
    x[e] = v0 + e < V ? sweep_weight(r.l[e], r.q[e], lse, inv_t, nres, invZs, skip_last) : 0.0;
}

__device__ __forceinline__ void lane_weights_wor(const Lane4& r, int v0, int V, double lse, double inv_t, int nres,
                                                 double x[4], const double* invZs, bool skip_last, const QLevels& ql) {
#pragma unroll
  for (int e = 0; e < 4; ++e)
    x[e] = v0 + e < V ? sweep_weight_wor(r.l[e], r.q[e], v0 + e, lse, inv_t, nres, invZs, skip_last, ql) : 0.0;
}

// Kernel 1: S workgroups per request.  Every workgroup repeats the (cheap) walk - merge the tile
// statistics of the request's rows, evaluate the k accept tests in parallel in fp64, find the first
// failure - then sums the draw weights over its slice of the vocabulary.  Slice 0 writes the
// per-request outputs and the state the draw kernel needs.
__global__ __launch_bounds__(kSweepThreads) void accept_chain_sweep(AcceptParams P) {
  __shared__ double s_lse[kMaxNq];
  __shared__ int s_ok[kMaxNq], s_arg[kMaxNq];
  __shared__ int s_last[kSweepThreads / kWave];
  const int slice = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  const int Nq = P.Nq, V = P.V;
  // with one temperature per request, a request at T = 0 is verified greedily inside this kernel
  const float Tf = request_temperature(P, b);
  const bool greedy = !(Tf > 0.f);
  const double T = greedy ? 1.0 : (double)Tf;
  const size_t row0 = (size_t)b * Nq;
  // operands of the accept tests: their addresses are known up front, so the loads fly during the merge
  float t_l = 0.f, t_q = 0.f, t_u = 0.f;
  int t_tok = -1;
  if (tid > 0 && tid < Nq) {
    t_tok = P.tok[row0 + tid];
    t_l = P.logits[(row0 + tid - 1) * V + t_tok];
    t_q = q_at(q_row(P, row0 + tid - 1), t_tok);
    t_u = P.un[(row0 + tid) * 2 + 0];
  }
  for (int n = wv; n < Nq; n += kSweepThreads / kWave) {
    float mx; double lse; int arg;
    merge_row_stats(P, row0 + n, T, lane, &mx, &lse, &arg, greedy);
    if (lane == 0) { s_lse[n] = lse; s_arg[n] = arg; }
  }
  __syncthreads();
  if (tid < Nq) {
    const int n = tid;
    float pv = 0.f;
    int ok = 1;
    if (n > 0 && greedy) {
      ok = t_tok == s_arg[n - 1];
      pv = ok ? 1.f : 0.f;
    } else if (n > 0) {
      const double p = exp((double)t_l / T - s_lse[n - 1]);
      ok = ((double)t_u * (double)t_q < p) ? 1 : 0;
      pv = (float)p;
    }
    s_ok[n] = ok;
    if (slice == 0) {
      if (P.p_at_draft) P.p_at_draft[row0 + n] = pv;
      if (P.row_lse) P.row_lse[row0 + n] = (float)s_lse[n];
    }
  }
  __syncthreads();
  int first_fail = Nq;
  for (int n = 1; n < Nq; ++n)
    if (!s_ok[n]) { first_fail = n; break; }
  const int row = first_fail - 1;          // accepted drafts = index of the row the draw happens on
  const int nres = first_fail < Nq ? 1 : 0;  // 1: draw from max(0, p - q); 0: all kept, draw from p
  const double lse = s_lse[row];
  if (slice == 0) {
    if (tid < Nq) P.accept_mask[row0 + tid] = tid <= row ? 1 : 0;
    if (tid == 0) {
      P.accept_len[b] = row;
      P.st_row[b] = row;
      P.st_rej[b] = greedy ? 2 : nres;  // 2: nothing left for the draw kernel
      P.st_lse[b] = lse;
      if (greedy) P.next_token[b] = s_arg[row];
    }
  }
  if (greedy) return;  // the whole workgroup: a greedy request has no sweep

  const double inv_t = 1.0 / T;
  const float* lrow = P.logits + (row0 + row) * V;
  const QRow qrow = q_row(P, row0 + row);
  const bool vec_ok = rows_vec_ok(P);
  const int per = (P.ngroups + P.slices - 1) / P.slices;
  const int g0 = slice * per, g1 = min(P.ngroups, g0 + per);
  int lastpos = -1;
  constexpr int kBatch = 4;  // groups whose loads a wavefront keeps in flight together
  constexpr int kStep = kSweepThreads / kWave;
  for (int g = g0 + wv; g < g1; g += kBatch * kStep) {
    Lane4 r[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int gi = g + i * kStep;
      if (gi < g1) r[i] = lane_load(lrow, qrow, gi * kGroup + lane * 4, V, vec_ok);
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int gi = g + i * kStep;
      if (gi < g1) {  // wave-uniform
        const int v0 = gi * kGroup + lane * 4;
        double x[4];
        lane_weights(r[i], v0, V, lse, inv_t, nres, x);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (x[e] > 0.0) lastpos = max(lastpos, v0 + e);
        const double sg = wave_sum((x[0] + x[1]) + (x[2] + x[3]));
        if (lane == 0) P.gsum[(size_t)b * P.ngroups + gi] = sg;
      }
    }
  }
  lastpos = wave_max(lastpos);
  if (lane == 0) s_last[wv] = lastpos;
  __syncthreads();
  if (tid == 0) {
    int m = -1;
    for (int i = 0; i < kSweepThreads / kWave; ++i) m = max(m, s_last[i]);
    P.lastpos[(size_t)b * P.slices + slice] = m;
  }
}

// Kernel 2: inverse-CDF draw from the group sums, one workgroup per request.
// A residual that vanished (sum 0) falls back to the row's p: rare enough for one workgroup.
__global__ __launch_bounds__(kSmallThreads) void accept_chain_pick(AcceptParams P) {
  __shared__ double s_wtot[kSmallThreads / kWave];
  __shared__ int s_pick;
  __shared__ double s_prefix;
  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  const int V = P.V, ng = P.ngroups;
  const int row = P.st_row[b];
  int nres = P.st_rej[b];
  if (nres == 2) return;  // a greedy request (one temperature per request): its token is already written
  const double lse = P.st_lse[b];
  const double inv_t = 1.0 / (double)request_temperature(P, b);
  const float* lrow = P.logits + ((size_t)b * P.Nq + row) * V;
  const QRow qrow = q_row(P, (size_t)b * P.Nq + row);
  const bool vec_ok = rows_vec_ok(P);
  double* gs = P.gsum + (size_t)b * ng;
  const int per = (ng + kSmallThreads - 1) / kSmallThreads;
  const int ga = min(ng, tid * per), gb = min(ng, ga + per);

  for (int attempt = 0; attempt < 2; ++attempt) {
    double loc = 0.0;
    for (int g = ga; g < gb; ++g) loc += gs[g];
    const double incl = wave_incl_scan(loc, lane);
    if (lane == kWave - 1) s_wtot[wv] = incl;
    if (tid == 0) s_pick = 0x7fffffff;
    __syncthreads();
    double wbase = 0.0, total = 0.0;
    for (int i = 0; i < kSmallThreads / kWave; ++i) {
      if (i < wv) wbase += s_wtot[i];
      total += s_wtot[i];
    }
    if (total > 0.0 || nres == 0) {
      const double thr = (double)P.un[((size_t)b * P.Nq + row) * 2 + 1] * total;
      double run = wbase + incl - loc;
      int found = 0x7fffffff;
      double before = 0.0;
      for (int g = ga; g < gb; ++g) {
        const double nxt = run + gs[g];
        if (found == 0x7fffffff && nxt > thr) { found = g; before = run; }
        run = nxt;
      }
      if (found != 0x7fffffff) atomicMin(&s_pick, found);
      __syncthreads();
      const int pick = s_pick;
      if (pick == found && found != 0x7fffffff) s_prefix = before;
      __syncthreads();
      if (wv == 0) {
        int token = -1;
        if (pick != 0x7fffffff) {
          const int v0 = pick * kGroup + lane * 4;
          double x[4];
          lane_weights(lane_load(lrow, qrow, v0, V, vec_ok), v0, V, lse, inv_t, nres, x);
          const double lane_tot = (x[0] + x[1]) + (x[2] + x[3]);
          const double lane_incl = wave_incl_scan(lane_tot, lane) + s_prefix;
          const unsigned long long hit = __ballot(lane_incl > thr);
          const unsigned long long pos = __ballot(lane_tot > 0.0);
          if (hit) {
            const int hl = __ffsll((long long)hit) - 1;  // first lane whose running sum crosses
            double r0 = __shfl(lane_incl - lane_tot, hl, kWave);
            int e_hit = 3;
            const double y0 = __shfl(x[0], hl, kWave), y1 = __shfl(x[1], hl, kWave), y2 = __shfl(x[2], hl, kWave);
            if (r0 + y0 > thr) e_hit = 0;
            else if (r0 + y0 + y1 > thr) e_hit = 1;
            else if (r0 + y0 + y1 + y2 > thr) e_hit = 2;
            token = pick * kGroup + hl * 4 + e_hit;
            if (token >= V) token = -1;
          } else if (pos) {
            // rounding left no crossing inside the group: its last token with positive weight
            const int pl = 63 - __clzll((long long)pos);
            int e_last = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (__shfl(x[e], pl, kWave) > 0.0) e_last = e;
            token = pick * kGroup + pl * 4 + e_last;
          }
        }
        if (token < 0) {  // no crossing at all: the largest token with positive weight
          int m = -1;
          for (int i = lane; i < P.slices; i += kWave) m = max(m, P.lastpos[(size_t)b * P.slices + i]);
          token = wave_max(m);
        }
        if (lane == 0) P.next_token[b] = token;
      }
      return;
    }
    // residual identically zero: recompute the group sums of p itself with this workgroup, then draw
    __syncthreads();
    nres = 0;
    int lastpos = -1;
    for (int g = wv; g < ng; g += kSmallThreads / kWave) {
      const int v0 = g * kGroup + lane * 4;
      double x[4];
      lane_weights(lane_load(lrow, qrow, v0, V, vec_ok), v0, V, lse, inv_t, 0, x);
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (x[e] > 0.0) lastpos = max(lastpos, v0 + e);
      const double acc = wave_sum((x[0] + x[1]) + (x[2] + x[3]));
      if (lane == 0) gs[g] = acc;
    }
    lastpos = wave_max(lastpos);
    if (lane == 0) atomicMax(&P.lastpos[(size_t)b * P.slices], lastpos);
    __threadfence_block();
    __syncthreads();
  }
}

// ============================================================================================
// Trees at T > 0, and every greedy call.  Grid (S, B): S workgroups per request.  With S = 1 the
// request's walk and all its vocabulary sweeps run in one workgroup.  With S > 1 every workgroup of a
// request repeats the walk (the same inputs give the same decisions, bit for bit) and sweeps only its
// slice of the vocabulary; after each sweep the group sums are exchanged through global memory behind a
// counting barrier, and every workgroup scans all of them in the same order as the one-workgroup form -
// so both forms return identical results.  The launcher keeps S * B within the number of compute units,
// so all workgroups of a request are resident together; the wait on the counter is bounded all the same.
// ============================================================================================
constexpr int kTreeMaxSlices = 16;
constexpr int kSpinLimit = 1 << 15;  // default number of polls of the arrival counter (tens of milliseconds) before a workgroup stops waiting

// The values exchanged between the workgroups of a request are written and read with device-scope
// atomic accesses: on this multi-die part they go past the die-local L2 to the point all dies see, so the
// hand-over needs no L2 write-back or invalidate - only "my stores have been acknowledged" before the
// arrival is counted.
__device__ __forceinline__ void store_agent(int32_t* p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent(double* p, double v) {
  __hip_atomic_store((unsigned long long*)p, __builtin_bit_cast(unsigned long long, v), __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_stores_acknowledged() {
  __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));  // vmcnt(0), nothing else
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ int load_agent(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double load_agent(const double* p) {
  const unsigned long long u = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return __builtin_bit_cast(double, u);
}

__global__ __launch_bounds__(kAccThreads) void accept_tree_kernel(AcceptParams P) {
  __shared__ double s_lse[kMaxNq];
  __shared__ int s_arg[kMaxNq];
  __shared__ double s_Z[kMaxNq], s_invZ[kMaxNq];
  __shared__ double s_gsum[kMaxGroups];
  __shared__ double s_wtot[kAccWaves];
  __shared__ int s_cur, s_depth, s_nres, s_last_child, s_state, s_have_gsum, s_pick, s_lastpos, s_fail;
  __shared__ double s_pick_prefix;
  // the request's tree, tokens and uniforms: the walk below is one thread chasing them, so they are
  // staged once instead of being fetched from global memory one dependent load at a time
  __shared__ int s_par[kMaxNq], s_tok[kMaxNq];
  __shared__ float s_u0[kMaxNq], s_u1[kMaxNq];
  __shared__ float s_ltok[kMaxNq], s_qtok[kMaxNq];  // logit and draft probability of node n's token in its parent's row
  // siblings without replacement: tokens rejected at the current node, the draft distribution each residual level
  // was formed with (see QLevels), and the one the next sibling was drawn from
  __shared__ int s_rej[kMaxNq], s_qlen[kMaxNq], s_cur_len;
  __shared__ double s_qfac[kMaxNq], s_cur_fac, s_rej_mass;

  const int b = blockIdx.y;
  const int S = (int)gridDim.x, slice = blockIdx.x;  // S > 1 only for sampling walks
  const bool writer = slice == 0;                     // the workgroup that stores the request's outputs
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  const int Nq = P.Nq, V = P.V;
  const float Tf = request_temperature(P, b);
  const bool greedy = !(Tf > 0.f);
  const double T = greedy ? 1.0 : (double)Tf;
  const double inv_t = 1.0 / T;
  const size_t row0 = (size_t)b * Nq;
  if (tid < Nq) {
    s_par[tid] = P.parents ? P.parents[row0 + tid] : tid - 1;
    s_tok[tid] = P.tok[row0 + tid];
    s_u0[tid] = greedy ? 0.f : P.un[(row0 + tid) * 2 + 0];
    s_u1[tid] = greedy ? 0.f : P.un[(row0 + tid) * 2 + 1];
  }

  // ---- 1. per-row (logsumexp, arg-max) from the tile statistics ---------------------------------
  // half a wavefront per row: 32 rows per round
  for (int n0 = 0; n0 < Nq; n0 += 2 * kAccWaves) {
    const int n = n0 + 2 * wv + (lane >> 5);
    const int nc = n < Nq ? n : Nq - 1;  // idle halves repeat the last row (the shuffles need every lane)
    float mx; double lse; int arg;
    merge_row_stats<32>(P, row0 + nc, T, lane, &mx, &lse, &arg, greedy);
    if ((lane & 31) == 0 && n < Nq) { s_lse[n] = lse; s_arg[n] = arg; }
  }
  __syncthreads();

  // ---- per-node outputs ------------------------------------------------------------------------
  if (tid < Nq) {
    const int n = tid;
    if (P.row_lse && writer) P.row_lse[row0 + n] = (float)s_lse[n];
    float pv = 0.f;
    if (n > 0) {
      const int par = s_par[n];
      const int tk = s_tok[n];
      if (greedy) {
        pv = (tk == s_arg[par]) ? 1.f : 0.f;
      } else {
        const float l = P.logits[(row0 + par) * V + tk];
        s_ltok[n] = l;
        s_qtok[n] = q_at(q_row(P, row0 + par), tk);
        pv = (float)exp((double)l / T - s_lse[par]);
      }
    }
    if (writer) {
      if (P.p_at_draft) P.p_at_draft[row0 + n] = pv;
      P.accept_mask[row0 + n] = n == 0 ? 1 : 0;
    }
  }
  __syncthreads();

  // ---- 2a. greedy walk: thread 0 only -----------------------------------------------------------
  if (greedy) {
    if (tid == 0 && writer) {
      int cur = 0, depth = 0;
      for (;;) {
        int moved = 0;
        for (int c = cur + 1; c < Nq && !moved; ++c) {
          if (s_par[c] == cur && s_tok[c] == s_arg[cur]) {
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
  const int ngroups = (V + kGroup - 1) / kGroup;  // <= kMaxGroups (checked by the launcher)
  const bool vec_ok = rows_vec_ok(P);
  const int per_slice = (ngroups + S - 1) / S;
  int g_lo = slice * per_slice;
  int g_hi = min(ngroups, g_lo + per_slice);
  bool split = S > 1;  // false once the writer has stopped waiting for the others and carries on alone
  int sweeps = 0;      // sweeps done so far: the same in every workgroup of the request
  const bool wor = P.wor != 0;
  const QLevels ql = {s_rej, s_qlen, s_qfac};
  if (tid == 0) {
    s_cur = 0; s_depth = 0; s_nres = 0; s_last_child = 0; s_have_gsum = 0; s_fail = 0;
    s_cur_len = 0; s_cur_fac = 1.0; s_rej_mass = 0.0;
  }
  enum { ST_DONE = 0, ST_ACCEPTED = 1, ST_REJECTED = 2 };
  for (;;) {
    __syncthreads();
    if (tid == 0) {
      const int cur = s_cur;
      int c = s_last_child + 1;
      for (; c < Nq; ++c)
        if (s_par[c] == cur) break;
      if (c >= Nq) {
        s_state = ST_DONE;
      } else {
        const float l = s_ltok[c];
        const float qv = s_qtok[c];
        const int tk = s_tok[c];
        const double p = wor ? node_weight_wor(l, qv, tk, s_lse[cur], T, s_nres, s_Z, ql)
                             : node_weight(l, qv, s_lse[cur], T, s_nres, s_Z);
        // the probability this sibling was drawn with
        const double qd = !wor ? (double)qv : in_list(tk, s_rej, s_cur_len) ? 0.0 : (double)qv * s_cur_fac;
        const double u = (double)s_u0[c];
        s_last_child = c;
        if (u * qd < p) {
          s_cur = c;
          s_depth = s_depth + 1;
          s_nres = 0;
          s_have_gsum = 0;
          s_cur_len = 0; s_cur_fac = 1.0; s_rej_mass = 0.0;
          if (writer) P.accept_mask[row0 + c] = 1;
          s_state = ST_ACCEPTED;
        } else {
          // the residual level that the sweep below forms subtracts the distribution this sibling was drawn from
          s_qlen[s_nres] = s_cur_len;
          s_qfac[s_nres] = s_cur_fac;
          s_state = ST_REJECTED;
        }
      }
    }
    __syncthreads();
    const int state = s_state;
    if (state == ST_ACCEPTED) continue;

    const int cur = s_cur;
    const float* lrow = P.logits + (row0 + cur) * V;
    const QRow qrow = q_row(P, row0 + cur);
    const double lse = s_lse[cur];

    if (state == ST_REJECTED || !s_have_gsum) {
      // group sums of the weights: after a rejection the unnormalised next residual level,
      // otherwise (nothing rejected at this node, or its residual vanished) the current level
      const int nres = state == ST_REJECTED ? s_nres + 1 : s_nres;
      const bool skip_last = state == ST_REJECTED;
      int lastpos = -1;
      constexpr int kBatch = 5;  // groups whose loads a wavefront keeps in flight together (160 KB per workgroup)
      double* gs_out = P.gsum + ((size_t)b * 2 + (sweeps & 1)) * ngroups;  // used while split
    sweep_again:
      for (int g = g_lo + wv; g < g_hi; g += kBatch * kAccWaves) {
        Lane4 r[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
          const int gi = g + i * kAccWaves;
          if (gi < g_hi) r[i] = lane_load(lrow, qrow, gi * kGroup + lane * 4, V, vec_ok);
        }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
          const int gi = g + i * kAccWaves;
          if (gi < g_hi) {  // wave-uniform
            const int v0 = gi * kGroup + lane * 4;
            double x[4];
            if (wor) lane_weights_wor(r[i], v0, V, lse, inv_t, nres, x, s_invZ, skip_last, ql);
            else lane_weights(r[i], v0, V, lse, inv_t, nres, x, s_invZ, skip_last);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (x[e] > 0.0) lastpos = max(lastpos, v0 + e);
            const double sg = wave_sum((x[0] + x[1]) + (x[2] + x[3]));
            if (lane == 0) {
              if (split) store_agent(&gs_out[gi], sg); else s_gsum[gi] = sg;
            }
          }
        }
      }
      lastpos = wave_max(lastpos);
      if (tid == 0) s_lastpos = -1;
      __syncthreads();
      if (lane == 0) atomicMax(&s_lastpos, lastpos);
      if (split) {
        // ---- exchange with the request's other workgroups ----------------------------------------
        wait_stores_acknowledged();  // this thread's group sums, before the arrival is counted
        __syncthreads();
        int32_t* lp = P.lastpos + ((size_t)b * 2 + (sweeps & 1)) * S;
        if (tid == 0) {
          store_agent(&lp[slice], s_lastpos);
          wait_stores_acknowledged();
          // release: everything this workgroup stored (ordered before this thread by the barrier above) is
          // visible device-wide before the arrival is
          __hip_atomic_fetch_add(&P.tree_bar[b], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
          const int target = S * (sweeps + 1);
          int polls = 0;
          while (load_agent(&P.tree_bar[b]) < target) {
            if (++polls > P.spin_limit) { s_fail = 1; break; }
            __builtin_amdgcn_s_sleep(4);
          }
          // acquire: pairs with the release of every arrival counted above
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        __syncthreads();
        if (s_fail) {
          // A workgroup of the request has not arrived within the bound (the GPU is shared and they are not all
          // resident, or one of them gave up earlier).  The others leave; the writer, which holds the whole walk
          // state like every workgroup, repeats this sweep over the entire vocabulary by itself and finishes the
          // request as the one-workgroup form would: same sums in the same order, so the same result.
          if (!writer) return;
          split = false;
          g_lo = 0;
          g_hi = ngroups;
          lastpos = -1;
          goto sweep_again;
        }
        // loads that bypass this compute unit's L1, which may still hold the copy of two sweeps ago
        for (int g = tid; g < ngroups; g += kAccThreads) s_gsum[g] = load_agent(&gs_out[g]);
        if (tid < S) atomicMax(&s_lastpos, load_agent(&lp[tid]));
        ++sweeps;
      }
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
          s_invZ[s_nres] = 1.0 / total;
          s_nres = s_nres + 1;
          s_have_gsum = 1;
        } else {
          s_have_gsum = 0;  // residual vanished: the distribution is left as it was
        }
        if (wor) {
          // the rejected token leaves the distribution the later siblings were drawn from
          const int c = s_last_child, tk = s_tok[c];
          if (!in_list(tk, s_rej, s_cur_len)) {
            s_rej[s_cur_len] = tk;
            s_cur_len = s_cur_len + 1;
            s_rej_mass = s_rej_mass + (double)s_qtok[c];
            const double left = 1.0 - s_rej_mass;
            s_cur_fac = left > 0.0 ? 1.0 / left : 0.0;
          }
        }
      }
      continue;
    }

    // ---- 3. state == ST_DONE: inverse-CDF draw --------------------------------------------------
    const double u = (double)s_u1[cur];
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
    if (!writer) return;  // no barrier between workgroups follows
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
        const int v0 = pick * kGroup + lane * 4;
        double x[4];
        if (wor) lane_weights_wor(lane_load(lrow, qrow, v0, V, vec_ok), v0, V, lse, inv_t, nres, x, s_invZ, have, ql);
        else lane_weights(lane_load(lrow, qrow, v0, V, vec_ok), v0, V, lse, inv_t, nres, x, s_invZ, have);
        const double lane_tot = (x[0] + x[1]) + (x[2] + x[3]);
        const double lane_incl = wave_incl_scan(lane_tot, lane) + s_pick_prefix;
        const unsigned long long hit = __ballot(lane_incl > thr);
        const unsigned long long pos = __ballot(lane_tot > 0.0);
        if (hit) {
          const int hl = __ffsll((long long)hit) - 1;  // first lane whose running sum crosses
          const double r0 = __shfl(lane_incl - lane_tot, hl, kWave);
          const double y0 = __shfl(x[0], hl, kWave), y1 = __shfl(x[1], hl, kWave), y2 = __shfl(x[2], hl, kWave);
          int e_hit = 3;
          if (r0 + y0 > thr) e_hit = 0;
          else if (r0 + y0 + y1 > thr) e_hit = 1;
          else if (r0 + y0 + y1 + y2 > thr) e_hit = 2;
          const int cand = pick * kGroup + hl * 4 + e_hit;
          if (cand < V) token = cand;
        } else if (pos) {
          const int pl = 63 - __clzll((long long)pos);
          int e_last = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (__shfl(x[e], pl, kWave) > 0.0) e_last = e;
          token = pick * kGroup + pl * 4 + e_last;
        }
      }
      if (lane == 0) {
        P.next_token[b] = token;
        P.accept_len[b] = s_depth;
      }
    }
    return;
  }
}

void accept_chain_geometry(int batch, int vocab, int* slices, int* gmul, int* ngroups) {
  const int ng = (vocab + kGroup - 1) / kGroup;
  // enough slices that a wavefront sweeps its share in two batches of four groups, within about two
  // workgroups per compute unit over the whole batch
  int s = (ng + 31) / 32;
  const int cap = (512 + batch - 1) / (batch > 0 ? batch : 1);
  if (s > cap) s = cap;
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  *slices = s;
  *gmul = kGroup / kWave;
  *ngroups = ng;
}

// polls before a workgroup of a split tree walk gives up waiting for the others (host-side setting, see the header)
static int g_tree_spin_limit = kSpinLimit;
void set_tree_spin_limit(int polls) { g_tree_spin_limit = polls < 0 ? kSpinLimit : polls; }

__global__ void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

int accept_tree_max_slices() { return kTreeMaxSlices; }

// Workgroups per request for a sampling tree walk: as many as leave every workgroup at least 16 groups
// to sweep, at most kTreeMaxSlices, and S * B within the number of compute units (all of them resident
// at once); 1 when that leaves fewer than two.
static int tree_slices_for(int B, int ngroups, int cus) {
  int s = ngroups / 16;
  if (s > kTreeMaxSlices) s = kTreeMaxSlices;
  if (B > 0 && s > cus / B) s = cus / B;
  return s >= 2 ? s : 1;
}

hipError_t launch_accept(const AcceptLaunch& a, hipStream_t st) {
  AcceptParams P = {};
  P.Nq = a.Nq; P.V = a.V; P.n_tiles = a.plan.n_tiles; P.temperature = a.temperature;
  P.logits = a.logits; P.pmax = a.pmax; P.psum = a.psum; P.parg = a.parg;
  P.tok = a.draft_tokens; P.q = a.draft_probs; P.un = a.uniforms; P.parents = a.parents;
  P.t2d = a.target_to_draft; P.Vq = a.target_to_draft ? a.Vd : a.V;
  P.accept_len = a.accept_len; P.next_token = a.next_token; P.accept_mask = a.accept_mask;
  P.p_at_draft = a.p_at_draft; P.row_lse = a.row_lse;
  P.slices = a.plan.slices; P.gmul = a.plan.gmul; P.ngroups = a.plan.ngroups;
  P.st_lse = a.st_lse; P.st_row = a.st_row; P.st_rej = a.st_rej; P.gsum = a.gsum; P.lastpos = a.lastpos;
  P.tree_bar = a.tree_bar;
  P.temps = a.temps;
  P.wor = a.wor;
  P.spin_limit = g_tree_spin_limit;
  const bool sampling = a.temperature > 0.f || a.temps != nullptr;  // per-request temperatures: the sampling kernels
  const bool chain_sampling = sampling && a.parents == nullptr;
  if (!chain_sampling) {
    const int ngroups = (a.V + kGroup - 1) / kGroup;
    if (sampling && ngroups > kMaxGroups) return hipErrorInvalidValue;
    int S = 1;
    if (sampling) {
      int cus = 0;
      if (hipError_t e = device_cu_count(&cus); e != hipSuccess) return e;
      S = tree_slices_for(a.B, ngroups, cus);
    }
    if (S > 1) {
      hipLaunchKernelGGL(zero_i32_kernel, dim3((a.B + 255) / 256), dim3(256), 0, st, a.tree_bar, a.B);
      if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    P.tree_slices = S;
    hipLaunchKernelGGL(accept_tree_kernel, dim3(S, a.B), dim3(kAccThreads), 0, st, P);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(accept_chain_sweep, dim3(P.slices, a.B), dim3(kSweepThreads), 0, st, P);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(accept_chain_pick, dim3(a.B), dim3(kSmallThreads), 0, st, P);
  return hipGetLastError();
}

}  // namespace aurora
