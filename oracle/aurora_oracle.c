/*
 * CPU oracle for the target-model verification step of speculative decoding.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may include, link or
 * call this file; it exists so that tests, the smoke check and the benchmark's
 * cpu_baseline leg have an independent answer to compare the HIP kernels with.
 * It shares no code with them.
 *
 * What it computes (paper section 2.1: the draft proposes several tokens, the
 * target verifies them in one pass and accepts a prefix; section 3.1: accepted
 * and rejected outcomes are both emitted; section 3.2 / figure 2: a tree of
 * candidates is verified in one batched pass under an ancestor mask; appendix
 * A.1 eq. 4: target logits l in R^{T x V}):
 *
 *   oracle_attn          chunk attention of the Nq draft-query positions of each
 *                        request over its paged GQA KV cache, chain-causal or
 *                        tree (ancestor) masked: the plain definition
 *                        softmax(scale * Q K^T + mask) V.
 *   oracle_logits        l[m, v] = sum_h hidden[m, h] * W[v, h].
 *   oracle_logits_fp8    the same with E4M3 operands and per-row scales.
 *   oracle_accept_logits target distribution per row, acceptance walk over the
 *                        chain or tree, residual / bonus sampling.
 *   oracle_accept        oracle_logits followed by oracle_accept_logits.
 *
 * The acceptance rule is the speculative-sampling rule the paper refers to in
 * section 2.1 (reference [leviathan2023fast] there): token d drawn from q is
 * kept iff u * q(d) < p(d); on rejection the replacement is drawn from
 * max(0, p - q) renormalised; if every draft is kept one more token is drawn
 * from the last row's p.  At temperature 0 it degenerates to "keep the longest
 * prefix whose tokens equal the target arg-max" (section 2.1's wording).
 *
 * All arithmetic is IEEE double on inputs widened exactly from float32 or
 * bfloat16, every sum runs in ascending index order, and nothing is blocked,
 * fused or reordered.  OpenMP only distributes independent requests / vocab
 * rows over threads.
 *
 * Pins (tests/test_oracle_*.py): library dense attention on tiny inputs,
 * closed forms (equal keys => mean of visible V), permutation / paging /
 * chain-vs-tree invariances; float64 library matmul; greedy = longest arg-max
 * prefix; q == p => everything accepted; Monte-Carlo on a 16-token vocabulary
 * (emitted-token law equals p, chain and tree); E[L] closed form of eq. 1;
 * rejection probability equals residual mass; a hand-worked 3-token example.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_OK = 0, ORACLE_BAD_ARG = -1, ORACLE_BAD_PAGE = -2, ORACLE_BAD_TREE = -3, ORACLE_NOMEM = -4 };

static double widen(const void *base, int64_t i, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* parent of node n in request b: explicit table, or n-1 for a chain */
static int parent_of(const int32_t *parents, int64_t b, int num_q, int n)
{
    return parents ? parents[b * num_q + n] : n - 1;
}

/* ------------------------------------------------------------------------
 * Chunk attention (sections 3.1, 3.2 / figure 2).
 *
 * Query position n of request b sits at absolute KV position L_b - Nq + n.
 * It sees the whole cached prefix j < L_b - Nq and, inside the chunk, the
 * slots of itself and of its ancestors (chain: all slots <= its own).
 * KV position j lives in page block_table[b][j / page] at offset j % page.
 * Query head hq reads KV head hq / (Hq / Hkv).
 * out: double [B, Nq, Hq, D].
 * ---------------------------------------------------------------------- */
static double decode_e4m3(uint8_t c);

/* Element i of a K or V pool of KV head hk.  kv_dtype ORACLE_KV_E4M3: the pool holds 8-bit E4M3 codes and
 * the value is scale[hk] * decode(code) (the cache is kept in 8-bit floating point with one float32 scale
 * per KV head, separately for K and V; queries, scores and the output stay as before). */
#define ORACLE_KV_E4M3 2
static double widen_kv(const void *base, int64_t i, int kv_dtype, const float *scale, int hk)
{
    if (kv_dtype == ORACLE_KV_E4M3) return (double)scale[hk] * decode_e4m3(((const uint8_t *)base)[i]);
    return widen(base, i, kv_dtype);
}

static int attn_impl(int batch, int num_q, int num_q_heads, int num_kv_heads, int head_dim,
                     int page_size, int max_pages_per_seq, int64_t num_pages, int dtype, int kv_dtype,
                     double sm_scale, const void *q, const void *k_pages, const void *v_pages,
                     const float *k_scale, const float *v_scale,
                     const int32_t *block_table, const int32_t *seq_lens, const int32_t *parents,
                     double *out)
{
    if (batch < 0 || num_q < 1 || num_kv_heads < 1 || num_q_heads % num_kv_heads || head_dim < 1 ||
        page_size < 1)
        return ORACLE_BAD_ARG;
    const int group = num_q_heads / num_kv_heads;
    if (sm_scale == 0.0)
        sm_scale = 1.0 / sqrt((double)head_dim);
    int status = ORACLE_OK;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < batch; ++b) {
        const int L = seq_lens[b];
        const int prefix = L - num_q;
        if (prefix < 0 || (int64_t)(L + page_size - 1) / page_size > max_pages_per_seq) {
#pragma omp atomic write
            status = ORACLE_BAD_ARG;
            continue;
        }
        double *score = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        unsigned char *visible = (unsigned char *)malloc((size_t)num_q);
        if (!score || !visible) {
#pragma omp atomic write
            status = ORACLE_NOMEM;
            free(score);
            free(visible);
            continue;
        }
        for (int n = 0; n < num_q; ++n) {
            /* visible[c] = 1 iff chunk slot c is node n itself or one of its ancestors */
            memset(visible, 0, (size_t)num_q);
            int bad = 0;
            for (int a = n, hops = 0; a >= 0; a = parent_of(parents, b, num_q, a), ++hops) {
                if (a >= num_q || hops > num_q) { bad = 1; break; }
                visible[a] = 1;
            }
            if (bad) {
#pragma omp atomic write
                status = ORACLE_BAD_TREE;
                continue;
            }
            for (int hq = 0; hq < num_q_heads; ++hq) {
                const int hk = hq / group;
                const int64_t qoff = (((int64_t)b * num_q + n) * num_q_heads + hq) * head_dim;
                double smax = -INFINITY;
                for (int j = 0; j < L; ++j) {
                    int seen = j < prefix ? 1 : visible[j - prefix];
                    if (!seen) { score[j] = -INFINITY; continue; }
                    const int32_t page = block_table[b * (int64_t)max_pages_per_seq + j / page_size];
                    if (page < 0 || page >= num_pages) {
#pragma omp atomic write
                        status = ORACLE_BAD_PAGE;
                        score[j] = -INFINITY;
                        continue;
                    }
                    const int64_t koff =
                        (((int64_t)page * num_kv_heads + hk) * page_size + j % page_size) * head_dim;
                    double dot = 0.0;
                    for (int d = 0; d < head_dim; ++d)
                        dot += widen(q, qoff + d, dtype) * widen_kv(k_pages, koff + d, kv_dtype, k_scale, hk);
                    score[j] = sm_scale * dot;
                    if (score[j] > smax) smax = score[j];
                }
                double denom = 0.0;
                for (int j = 0; j < L; ++j) {
                    score[j] = score[j] == -INFINITY ? 0.0 : exp(score[j] - smax);
                    denom += score[j];
                }
                double *o = out + qoff;
                for (int d = 0; d < head_dim; ++d) o[d] = 0.0;
                for (int j = 0; j < L; ++j) {
                    if (score[j] == 0.0) continue;
                    const int32_t page = block_table[b * (int64_t)max_pages_per_seq + j / page_size];
                    if (page < 0 || page >= num_pages) continue;
                    const int64_t voff =
                        (((int64_t)page * num_kv_heads + hk) * page_size + j % page_size) * head_dim;
                    const double w = score[j] / denom;
                    for (int d = 0; d < head_dim; ++d) o[d] += w * widen_kv(v_pages, voff + d, kv_dtype, v_scale, hk);
                }
            }
        }
        free(score);
        free(visible);
    }
    return status;
}

int oracle_attn(int batch, int num_q, int num_q_heads, int num_kv_heads, int head_dim,
                int page_size, int max_pages_per_seq, int64_t num_pages, int dtype, double sm_scale,
                const void *q, const void *k_pages, const void *v_pages,
                const int32_t *block_table, const int32_t *seq_lens, const int32_t *parents,
                double *out)
{
    return attn_impl(batch, num_q, num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq, num_pages,
                     dtype, dtype, sm_scale, q, k_pages, v_pages, NULL, NULL, block_table, seq_lens, parents, out);
}

/* The same attention over a cache held as E4M3 codes: k_scale / v_scale are float32 [num_kv_heads]. */
int oracle_attn_fp8kv(int batch, int num_q, int num_q_heads, int num_kv_heads, int head_dim,
                      int page_size, int max_pages_per_seq, int64_t num_pages, int dtype, double sm_scale,
                      const void *q, const uint8_t *k_pages, const uint8_t *v_pages,
                      const float *k_scale, const float *v_scale,
                      const int32_t *block_table, const int32_t *seq_lens, const int32_t *parents,
                      double *out)
{
    if (!k_scale || !v_scale) return ORACLE_BAD_ARG;
    return attn_impl(batch, num_q, num_q_heads, num_kv_heads, head_dim, page_size, max_pages_per_seq, num_pages,
                     dtype, ORACLE_KV_E4M3, sm_scale, q, k_pages, v_pages, k_scale, v_scale, block_table, seq_lens,
                     parents, out);
}

/* ------------------------------------------------------------------------
 * LM-head projection (appendix A.1, eq. 4: logits l in R^{T x V}).
 * logits[m, v] = sum_h hidden[m, h] * W[v, h], W stored [V, H] row-major.
 * out: double [M, V].
 * ---------------------------------------------------------------------- */
int oracle_logits(int64_t rows, int hidden_size, int vocab, int dtype,
                  const void *hidden, const void *lm_head, double *out)
{
    if (rows < 0 || hidden_size < 1 || vocab < 1) return ORACLE_BAD_ARG;
    double *hid = (double *)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * hidden_size);
    if (!hid) return ORACLE_NOMEM;
    for (int64_t i = 0; i < rows * hidden_size; ++i) hid[i] = widen(hidden, i, dtype);
    int status = ORACLE_OK;
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)hidden_size);
        if (!wrow) {
#pragma omp atomic write
            status = ORACLE_NOMEM;
        }
#pragma omp for schedule(static)
        for (int64_t v = 0; v < vocab; ++v) {
            if (!wrow) continue;
            for (int h = 0; h < hidden_size; ++h) wrow[h] = widen(lm_head, v * hidden_size + h, dtype);
            for (int64_t m = 0; m < rows; ++m) {
                const double *x = hid + m * hidden_size;
                double acc = 0.0;
                for (int h = 0; h < hidden_size; ++h) acc += x[h] * wrow[h];
                out[m * vocab + v] = acc;
            }
        }
        free(wrow);
    }
    free(hid);
    return status;
}

/* ------------------------------------------------------------------------
 * LM head with 8-bit floating-point operands (the paper serves its frontier
 * targets in FP8, sections 1 and 4.3; it does not give a quantisation recipe).
 * Reading taken: OCP E4M3 codes (1 sign, 4 exponent bits with bias 7, 3
 * mantissa bits; no infinities, S.1111.111 is NaN) with one float32 scale per
 * token row of `hidden` and one per vocabulary row of `lm_head`; a stored
 * element stands for scale * decode(code), and the logit is the plain dot
 * product of the dequantised rows.
 * ---------------------------------------------------------------------- */
static double decode_e4m3(uint8_t c)
{
    const int sign = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

int oracle_decode_e4m3(int64_t n, const uint8_t *codes, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = decode_e4m3(codes[i]);
    return ORACLE_OK;
}

int oracle_logits_fp8(int64_t rows, int hidden_size, int vocab, const uint8_t *hidden, const float *hidden_scale,
                      const uint8_t *lm_head, const float *lm_scale, double *out)
{
    if (rows < 0 || hidden_size < 1 || vocab < 1 || !hidden_scale || !lm_scale) return ORACLE_BAD_ARG;
    double *hid = (double *)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * hidden_size);
    if (!hid) return ORACLE_NOMEM;
    for (int64_t m = 0; m < rows; ++m)
        for (int h = 0; h < hidden_size; ++h)
            hid[m * hidden_size + h] = (double)hidden_scale[m] * decode_e4m3(hidden[m * hidden_size + h]);
    int status = ORACLE_OK;
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)hidden_size);
        if (!wrow) {
#pragma omp atomic write
            status = ORACLE_NOMEM;
        }
#pragma omp for schedule(static)
        for (int64_t v = 0; v < vocab; ++v) {
            if (!wrow) continue;
            for (int h = 0; h < hidden_size; ++h)
                wrow[h] = (double)lm_scale[v] * decode_e4m3(lm_head[v * hidden_size + h]);
            for (int64_t m = 0; m < rows; ++m) {
                const double *x = hid + m * hidden_size;
                double acc = 0.0;
                for (int h = 0; h < hidden_size; ++h) acc += x[h] * wrow[h];
                out[m * vocab + v] = acc;
            }
        }
        free(wrow);
    }
    free(hid);
    return status;
}

/* ------------------------------------------------------------------------
 * Target distribution of one row.
 * T > 0: p(v) = exp(l(v)/T - lse), lse = log sum_v exp(l(v)/T), max-subtracted.
 * Returns lse.  p may be NULL.
 * ---------------------------------------------------------------------- */
static double row_softmax(const double *logit, int vocab, double T, double *p)
{
    double mx = -INFINITY;
    for (int v = 0; v < vocab; ++v) {
        double x = logit[v] / T;
        if (x > mx) mx = x;
    }
    double s = 0.0;
    for (int v = 0; v < vocab; ++v) s += exp(logit[v] / T - mx);
    const double lse = mx + log(s);
    if (p)
        for (int v = 0; v < vocab; ++v) p[v] = exp(logit[v] / T - lse);
    return lse;
}

/* arg-max, lowest index on exact ties; also the gap to the runner-up */
static int row_argmax(const double *logit, int vocab, double *gap)
{
    int best = 0;
    for (int v = 1; v < vocab; ++v)
        if (logit[v] > logit[best]) best = v;
    if (gap) {
        double second = -INFINITY;
        for (int v = 0; v < vocab; ++v)
            if (v != best && logit[v] > second) second = logit[v];
        *gap = logit[best] - second;
    }
    return best;
}

/* Inverse-CDF draw from the unnormalised non-negative weights r[0..V):
 * Z = sum r, t = u * Z, result = first v whose running sum exceeds t;
 * if rounding leaves none, the largest v with r(v) > 0.
 * cdf (optional, [V]) receives the normalised running sums. */
static int draw_inverse_cdf(const double *r, int vocab, double u, double *cdf)
{
    double Z = 0.0;
    for (int v = 0; v < vocab; ++v) Z += r[v];
    const double t = u * Z;
    double run = 0.0;
    int pick = -1, last_pos = -1;
    for (int v = 0; v < vocab; ++v) {
        run += r[v];
        if (r[v] > 0.0) last_pos = v;
        if (pick < 0 && run > t) pick = v;
        if (cdf) cdf[v] = run / Z;
    }
    return pick >= 0 ? pick : last_pos;
}

/* ------------------------------------------------------------------------
 * Chain acceptance of one request, written out on its own (section 2.1: the
 * target keeps a prefix of the drafted chain and emits one more token).
 *
 * T > 0:  for i = 1..k in order: keep d_i iff u_i * q_{i-1}(d_i) < p_{i-1}(d_i); stop at the
 *         first failure.  j = number kept.  If j < k the next token is drawn from
 *         max(0, p_j - q_j) (from p_j itself if that is identically 0); if j == k from p_k.
 * T == 0: keep d_i iff d_i == argmax l_{i-1}; next token = argmax l_j.
 * The draw uses uniforms[j][1].  Returns j.
 * lg [Nq, V], tok [Nq], q [Nq, V], un [Nq, 2], mask [Nq] (pre-zeroed, may be NULL),
 * margin [Nq] (pre-filled NaN, may be NULL), p / r scratch [V], cdf [V] or NULL.
 * ---------------------------------------------------------------------- */
static int accept_chain(int num_q, int vocab, double T, const double *lg, const int32_t *tok,
                        const float *q, const float *un, uint8_t *mask, double *margin,
                        double *p, double *r, double *cdf, int32_t *next)
{
    const int k = num_q - 1;
    int j = 0;
    if (mask) mask[0] = 1;
    if (T == 0.0) {
        for (int i = 1; i <= k; ++i) {
            if (tok[i] != row_argmax(lg + (int64_t)(i - 1) * vocab, vocab, NULL)) break;
            if (mask) mask[i] = 1;
            j = i;
        }
        *next = row_argmax(lg + (int64_t)j * vocab, vocab, NULL);
        return j;
    }
    for (int i = 1; i <= k; ++i) {
        row_softmax(lg + (int64_t)(i - 1) * vocab, vocab, T, p);
        const double u = (double)un[i * 2 + 0];
        const double qd = (double)q[(int64_t)(i - 1) * vocab + tok[i]];
        const double pd = p[tok[i]];
        if (margin) margin[i] = qd > 0.0 ? fabs(pd / qd - u) : INFINITY;
        if (!(u * qd < pd)) break;
        if (mask) mask[i] = 1;
        j = i;
    }
    row_softmax(lg + (int64_t)j * vocab, vocab, T, p);
    const double *weights = p;
    if (j < k) {
        double Z = 0.0;
        for (int v = 0; v < vocab; ++v) {
            const double d = p[v] - (double)q[(int64_t)j * vocab + v];
            r[v] = d > 0.0 ? d : 0.0;
            Z += r[v];
        }
        if (Z > 0.0) weights = r;
    }
    *next = draw_inverse_cdf(weights, vocab, (double)un[j * 2 + 1], cdf);
    return j;
}

/* ------------------------------------------------------------------------
 * Acceptance from given logits.
 *
 * logits        double [B, Nq, V]
 * draft_tokens  [B, Nq], entry 0 unused
 * draft_probs   float  [B, Nq, V]; row n = distribution the children of n were drawn from
 * uniforms      float  [B, Nq, 2]; [.,n,0] accept test of node n, [.,n,1] draw when the walk stops at n
 * parents       [B, Nq] or NULL (chain)
 *
 * parents == NULL: each request goes through accept_chain above.
 * parents != NULL: tree walk (a chain given as parents[n] = n-1 must and does give the same
 * result; a test checks it): cur = root, p = p_root.
 *   for each child c of cur in ascending node index:
 *       accept iff u_c * q_cur(tok_c) < p(tok_c)
 *       accepted: mark c, cur = c, p = p_c, continue with c's children
 *       rejected: p <- max(0, p - q_cur) / sum max(0, p - q_cur)   (q_cur unchanged:
 *                 siblings are independent draws from q_cur); if that sum is 0, p is kept
 *   siblings_without_replacement != 0 (oracle_accept_logits_ex): the children of a node were drawn one after
 *   the other, each from q_cur with the tokens of the earlier siblings removed.  Then the test and the residual
 *   of a child use q' = that distribution, q'(v) = 0 for v in X, else q_cur(v) / (1 - sum_{x in X} q_cur(x)),
 *   X = the set of tokens rejected at this node so far (the row q_cur is taken to sum to 1; a remaining mass
 *   <= 0 makes q' identically 0).
 *   no child left: next_token ~ p by inverse CDF with uniforms[b, cur, 1].
 * T == 0: accept c iff tok_c == argmax_cur; next_token = argmax_cur.
 *
 * Outputs (any may be NULL):
 *   accept_len [B]      depth of the last accepted node = number of accepted draft tokens
 *   next_token [B]
 *   accept_mask[B, Nq]  1 on the accepted path (root included), else 0
 *   p_at_draft [B, Nq]  target probability p_parent(n)(tok_n) of every non-root node
 *                       (T == 0: 1 if tok_n is the parent's arg-max else 0); root 0
 *   row_lse    [B, Nq]  logsumexp(l / T) per row (T == 0: logsumexp(l))
 * Diagnostics for near-tie bookkeeping in parity tests (any may be NULL):
 *   test_margin[B, Nq]  |p/q - u| of each evaluated accept test (NaN where none was
 *                       evaluated; +inf when q == 0)
 *   top_gap    [B, Nq]  top-1 minus top-2 logit of each row
 *   stop_node  [B]      node the walk stopped at
 *   final_cdf  [B, V]   normalised running sums of the distribution next_token was drawn from
 *                       (T == 0: not written)
 * ---------------------------------------------------------------------- */
int oracle_accept_logits_ex(int batch, int num_q, int vocab, double temperature,
                            const double *logits, const int32_t *draft_tokens,
                            const float *draft_probs, const float *uniforms, const int32_t *parents,
                            int32_t *accept_len, int32_t *next_token, uint8_t *accept_mask,
                            double *p_at_draft, double *row_lse,
                            double *test_margin, double *top_gap, int32_t *stop_node, double *final_cdf,
                            int siblings_without_replacement)
{
    if (batch < 0 || num_q < 1 || vocab < 1 || temperature < 0.0) return ORACLE_BAD_ARG;
    const int greedy = temperature == 0.0;
    if (!greedy && (!draft_probs || !uniforms)) return ORACLE_BAD_ARG;
    int status = ORACLE_OK;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < batch; ++b) {
        const double *lg = logits + b * (int64_t)num_q * vocab;
        const int32_t *tok = draft_tokens + b * (int64_t)num_q;
        int bad = 0;
        for (int n = 1; n < num_q; ++n) {
            int par = parent_of(parents, b, num_q, n);
            if (par < 0 || par >= n || tok[n] < 0 || tok[n] >= vocab) bad = 1;
        }
        if (bad) {
#pragma omp atomic write
            status = ORACLE_BAD_TREE;
            continue;
        }
        double *p = (double *)malloc(sizeof(double) * (size_t)vocab);
        double *r = (double *)malloc(sizeof(double) * (size_t)vocab);
        if (!p || !r) {
#pragma omp atomic write
            status = ORACLE_NOMEM;
            free(p);
            free(r);
            continue;
        }
        /* per-row statistics that do not depend on the walk */
        for (int n = 0; n < num_q; ++n) {
            double gap;
            (void)row_argmax(lg + (int64_t)n * vocab, vocab, &gap);
            if (top_gap) top_gap[b * num_q + n] = gap;
            if (row_lse)
                row_lse[b * num_q + n] = row_softmax(lg + (int64_t)n * vocab, vocab, greedy ? 1.0 : temperature, NULL);
            if (test_margin) test_margin[b * num_q + n] = NAN;
            if (accept_mask) accept_mask[b * num_q + n] = 0;
            if (p_at_draft) p_at_draft[b * num_q + n] = 0.0;
        }
        if (p_at_draft)
            for (int n = 1; n < num_q; ++n) {
                const int par = parent_of(parents, b, num_q, n);
                const double *lrow = lg + (int64_t)par * vocab;
                if (greedy) {
                    p_at_draft[b * num_q + n] = row_argmax(lrow, vocab, NULL) == tok[n] ? 1.0 : 0.0;
                } else {
                    const double lse = row_softmax(lrow, vocab, temperature, NULL);
                    p_at_draft[b * num_q + n] = exp(lrow[tok[n]] / temperature - lse);
                }
            }

        int cur = 0, depth = 0;
        if (!parents) {
            int32_t nt = -1;
            depth = cur = accept_chain(num_q, vocab, temperature, lg, tok,
                                       draft_probs ? draft_probs + b * (int64_t)num_q * vocab : NULL,
                                       uniforms ? uniforms + b * (int64_t)num_q * 2 : NULL,
                                       accept_mask ? accept_mask + b * num_q : NULL,
                                       test_margin ? test_margin + b * num_q : NULL, p, r,
                                       final_cdf && !greedy ? final_cdf + b * (int64_t)vocab : NULL, &nt);
            if (next_token) next_token[b] = nt;
            if (accept_len) accept_len[b] = depth;
            if (stop_node) stop_node[b] = cur;
            free(p);
            free(r);
            continue;
        }
        if (accept_mask) accept_mask[b * num_q] = 1;
        if (greedy) {
            for (;;) {
                const int best = row_argmax(lg + (int64_t)cur * vocab, vocab, NULL);
                int moved = 0;
                for (int c = cur + 1; c < num_q && !moved; ++c) {
                    if (parent_of(parents, b, num_q, c) != cur) continue;
                    if (tok[c] == best) {
                        cur = c;
                        ++depth;
                        if (accept_mask) accept_mask[b * num_q + c] = 1;
                        moved = 1;
                    }
                }
                if (!moved) {
                    if (next_token) next_token[b] = best;
                    break;
                }
            }
        } else {
            row_softmax(lg + (int64_t)cur * vocab, vocab, temperature, p);
            /* removed[v] != 0: token v was rejected at the current node (only used without replacement) */
            unsigned char *removed = siblings_without_replacement ? (unsigned char *)calloc((size_t)vocab, 1) : NULL;
            if (siblings_without_replacement && !removed) {
#pragma omp atomic write
                status = ORACLE_NOMEM;
                free(p);
                free(r);
                continue;
            }
            for (;;) {
                const float *qrow = draft_probs + (b * (int64_t)num_q + cur) * vocab;
                double removed_mass = 0.0; /* sum of q_cur over the removed tokens */
                if (removed) memset(removed, 0, (size_t)vocab);
                int moved = 0;
                for (int c = cur + 1; c < num_q && !moved; ++c) {
                    if (parent_of(parents, b, num_q, c) != cur) continue;
                    const double u = (double)uniforms[(b * (int64_t)num_q + c) * 2 + 0];
                    /* the distribution this sibling was drawn from: q_cur, or q_cur without the removed tokens */
                    const double left = 1.0 - removed_mass;
                    const double qscale = !removed ? 1.0 : (left > 0.0 ? 1.0 / left : 0.0);
                    const double qc = removed && removed[tok[c]] ? 0.0 : (double)qrow[tok[c]] * qscale;
                    const double pc = p[tok[c]];
                    if (test_margin)
                        test_margin[b * num_q + c] = qc > 0.0 ? fabs(pc / qc - u) : INFINITY;
                    if (u * qc < pc) {
                        cur = c;
                        ++depth;
                        if (accept_mask) accept_mask[b * num_q + c] = 1;
                        row_softmax(lg + (int64_t)cur * vocab, vocab, temperature, p);
                        moved = 1;
                    } else {
                        double Z = 0.0;
                        for (int v = 0; v < vocab; ++v) {
                            const double qv = removed && removed[v] ? 0.0 : (double)qrow[v] * qscale;
                            const double d = p[v] - qv;
                            r[v] = d > 0.0 ? d : 0.0;
                            Z += r[v];
                        }
                        if (Z > 0.0)
                            for (int v = 0; v < vocab; ++v) p[v] = r[v] / Z;
                        if (removed && !removed[tok[c]]) {
                            removed[tok[c]] = 1;
                            removed_mass += (double)qrow[tok[c]];
                        }
                    }
                }
                if (!moved) break;
            }
            free(removed);
            const double us = (double)uniforms[(b * (int64_t)num_q + cur) * 2 + 1];
            const int t = draw_inverse_cdf(p, vocab, us, final_cdf ? final_cdf + b * (int64_t)vocab : NULL);
            if (next_token) next_token[b] = t;
        }
        if (accept_len) accept_len[b] = depth;
        if (stop_node) stop_node[b] = cur;
        free(p);
        free(r);
    }
    return status;
}

int oracle_accept_logits(int batch, int num_q, int vocab, double temperature,
                         const double *logits, const int32_t *draft_tokens,
                         const float *draft_probs, const float *uniforms, const int32_t *parents,
                         int32_t *accept_len, int32_t *next_token, uint8_t *accept_mask,
                         double *p_at_draft, double *row_lse,
                         double *test_margin, double *top_gap, int32_t *stop_node, double *final_cdf)
{
    return oracle_accept_logits_ex(batch, num_q, vocab, temperature, logits, draft_tokens, draft_probs, uniforms,
                                   parents, accept_len, next_token, accept_mask, p_at_draft, row_lse, test_margin,
                                   top_gap, stop_node, final_cdf, 0);
}

/* LM head, then acceptance.  logits_out (optional) receives double [B*Nq, V]. */
int oracle_accept(int batch, int num_q, int hidden_size, int vocab, int dtype, double temperature,
                  const void *hidden, const void *lm_head, const int32_t *draft_tokens,
                  const float *draft_probs, const float *uniforms, const int32_t *parents,
                  int32_t *accept_len, int32_t *next_token, uint8_t *accept_mask,
                  double *p_at_draft, double *row_lse,
                  double *test_margin, double *top_gap, int32_t *stop_node, double *final_cdf,
                  double *logits_out)
{
    const int64_t rows = (int64_t)batch * num_q;
    double *logits = logits_out ? logits_out
                                : (double *)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * vocab);
    if (!logits) return ORACLE_NOMEM;
    int st = oracle_logits(rows, hidden_size, vocab, dtype, hidden, lm_head, logits);
    if (st == ORACLE_OK)
        st = oracle_accept_logits(batch, num_q, vocab, temperature, logits, draft_tokens, draft_probs,
                                  uniforms, parents, accept_len, next_token, accept_mask, p_at_draft,
                                  row_lse, test_margin, top_gap, stop_node, final_cdf);
    if (!logits_out) free(logits);
    return st;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
