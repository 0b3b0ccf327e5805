/*
 * CPU oracle for trace emission: what the inference server hands to the training
 * side after a verify step.
 *
 * TEST INFRASTRUCTURE ONLY (see aurora_oracle.c).  Shares no code with the HIP path.
 *
 * What it computes (paper section 3.1: the outcomes of accepted and rejected
 * tokens are both streamed to the data buffer; appendix A.1, eq. 4: a record is
 * (h, l, x_in, y_out, R) with l the target logits and R the rejection trajectory;
 * appendix A.2: only the K most informative target logits per token are kept,
 * K = 1024, which turns 256 KB of logits per token into 2 KB):
 *
 *   oracle_trace_topk     per row of l, the K largest entries: ids ordered by value
 *                         descending, equal values by ascending id; values stored
 *                         as bfloat16 (round to nearest even).  Written out as the
 *                         definition: sort every (value, id) pair of the row, keep
 *                         the first K.
 *   oracle_trace_records  y_out and R from the acceptance outputs (integer logic).
 *
 * The paper fixes K and the 2-bytes-per-logit budget, not the order, tie rule, the
 * layout of y_out or the encoding of R; those are this build's readings:
 *   - order: value descending, ties (including -0.0 vs +0.0, which compare equal)
 *     by ascending id; -inf is an ordinary smallest value; NaN is an error;
 *   - rows shorter than K are padded with id -1 and value -inf;
 *   - y_out[b, n] = the token emitted after node n: the token of n's accepted child,
 *     next_token[b] for the last node of the accepted path, -1 for nodes off it;
 *   - R[b, n] = 1 for nodes on the accepted path (root included), 2 for drafts that
 *     were tested and rejected (under the sequential rule the children of a path
 *     node are tried in index order until one is kept: those before the kept one,
 *     or all of them if none is kept), 0 for nodes never tested.
 *
 * Pins (tests/test_oracle_trace.py): repeated arg-max extraction by brute force on
 * small rows, rows that are permutations of known values (closed form), ties,
 * signed zeros, -inf, K >= V; bfloat16 rounding against hand-computed bit patterns
 * and the halfway cases; hand-worked chain and tree trajectories.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { TRACE_OK = 0, TRACE_BAD_ARG = -1, TRACE_NAN = -5, TRACE_NOMEM = -4 };

typedef struct {
    float v;
    int32_t id;
} pair_t;

static int cmp_pair(const void *pa, const void *pb)
{
    const pair_t *a = (const pair_t *)pa, *b = (const pair_t *)pb;
    if (a->v > b->v) return -1;
    if (a->v < b->v) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

/* float32 -> bfloat16 bits, round to nearest, ties to even; infinities kept */
static uint16_t to_bf16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) == 0x7f800000u) return (uint16_t)(u >> 16);
    const uint32_t lower = u & 0xffffu, keep = u >> 16;
    uint32_t out = keep;
    if (lower > 0x8000u || (lower == 0x8000u && (keep & 1u))) out = keep + 1u;
    return (uint16_t)out;
}

int oracle_trace_topk(int64_t rows, int vocab, int top_k, const float *logits, int32_t *ids, uint16_t *vals)
{
    if (rows < 0 || vocab < 1 || top_k < 1 || !logits || !ids || !vals) return TRACE_BAD_ARG;
    int status = TRACE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t m = 0; m < rows; ++m) {
        pair_t *row = (pair_t *)malloc(sizeof(pair_t) * (size_t)vocab);
        if (!row) {
#pragma omp critical
            status = TRACE_NOMEM;
            continue;
        }
        int bad = 0;
        for (int v = 0; v < vocab; ++v) {
            row[v].v = logits[m * vocab + v];
            row[v].id = v;
            if (isnan(row[v].v)) bad = 1;
        }
        if (bad) {
#pragma omp critical
            status = TRACE_NAN;
        } else {
            qsort(row, (size_t)vocab, sizeof(pair_t), cmp_pair);
            for (int k = 0; k < top_k; ++k) {
                if (k < vocab) {
                    ids[m * top_k + k] = row[k].id;
                    vals[m * top_k + k] = to_bf16_bits(row[k].v);
                } else {
                    ids[m * top_k + k] = -1;
                    vals[m * top_k + k] = 0xff80u; /* -inf */
                }
            }
        }
        free(row);
    }
    return status;
}

int oracle_trace_records(int batch, int num_q, const int32_t *draft_tokens, const int32_t *parents,
                         const int32_t *next_token, const uint8_t *accept_mask, int32_t *y_out, int8_t *traj)
{
    if (batch < 0 || num_q < 1 || !draft_tokens || !next_token || !accept_mask || !y_out || !traj)
        return TRACE_BAD_ARG;
    for (int b = 0; b < batch; ++b) {
        const int32_t *tok = draft_tokens + (int64_t)b * num_q;
        const uint8_t *mask = accept_mask + (int64_t)b * num_q;
        int32_t *y = y_out + (int64_t)b * num_q;
        int8_t *r = traj + (int64_t)b * num_q;
        for (int n = 0; n < num_q; ++n) {
            y[n] = -1;
            r[n] = 0;
        }
        /* walk the accepted path from the root */
        int cur = 0;
        r[0] = 1;
        for (;;) {
            int kept = -1;
            for (int c = cur + 1; c < num_q; ++c) {
                const int par = parents ? parents[(int64_t)b * num_q + c] : c - 1;
                if (par != cur) continue;
                if (mask[c]) {
                    kept = c;
                    break;
                }
                r[c] = 2; /* tried before the kept sibling (or no sibling was kept) */
            }
            if (kept < 0) break;
            r[kept] = 1;
            y[cur] = tok[kept];
            cur = kept;
        }
        y[cur] = next_token[b];
    }
    return TRACE_OK;
}
