/*
 * CPU oracle for the budget-constrained MoE layer forward of Alloc-MoE.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * single-threaded restatement of the paper's definitions, in double precision,
 * used only by the tests, the smoke check and the benchmark's cpu_baseline leg
 * to judge the HIP library.  It shares no code, header, table or helper with
 * the HIP path and must never be called from it.
 *
 * Every function cites the passage of the paper it follows.  Notation follows
 * the paper: T tokens, H (here d) hidden size, N (here E) experts, K_orig
 * (here K) candidates per token, K_base (here Kb), layer budget T*K_l (here B,
 * taken as any integer number of activations).
 *
 * Element types: dtype 0 = IEEE fp32, dtype 1 = bfloat16 bit patterns in
 * uint16_t (widened exactly to fp32 by placing them in the upper 16 bits).
 * All matrices are row-major.  Expert e's matrices: W1[e] and W3[e] are
 * [d, I], W2[e] is [I, d]; the expert network is
 *     E_e(x) = ( silu(x W1_e) (*) (x W3_e) ) W2_e ,  silu(a) = a / (1 + exp(-a))
 * (the paper speaks only of a feed-forward execution per activation; the SwiGLU
 * form, with W1 on the gated branch, is the workload definition of the evaluated
 * models).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (brute
 * force of the selection problem, reduction to plain Top-K, budget
 * conservation, dense-vs-dispatched Eq. (2), closed forms and a library fp64
 * re-computation).  No function here is left without a pin.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ helpers */

static double load_elem(const void *p, int dtype, size_t i)
{
    if (dtype == 0)
        return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static size_t elem_size(int dtype) { return dtype == 0 ? 4u : 2u; }

static const void *offset_elems(const void *p, int dtype, size_t n)
{
    return (const void *)((const char *)p + n * elem_size(dtype));
}

/* ---------------------------------------------------- Eq. (1): gate, softmax */

/* logits[t,e] = sum_h X[t,h] * W_gate[h,e] (+ bias[e]);  Section 3.1, Eq. (1):
 * the hidden state times the gate matrix of shape [H, N].  The additive per-expert bias is
 * not in the paper; it is the synthetic workload's popularity skew and is
 * applied to the logits before the softmax.  bias may be NULL. */
void oracle_gate_logits(const void *X, const void *Wg, const float *bias,
                        int T, int d, int E, int dtype, double *logits)
{
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int h = 0; h < d; ++h)
                acc += load_elem(X, dtype, (size_t)t * d + h) *
                       load_elem(Wg, dtype, (size_t)h * E + e);
            if (bias)
                acc += (double)bias[e];
            logits[(size_t)t * E + e] = acc;
        }
}

/* scores[t,:] = Softmax(logits[t,:]) over all N experts; Eq. (1).  The softmax
 * is taken over every expert before any Top-K, exactly as the equation nests
 * them.  Computed in double (max-subtracted), stored as fp32. */
void oracle_softmax(const double *logits, int T, int E, float *scores)
{
    for (int t = 0; t < T; ++t) {
        const double *l = logits + (size_t)t * E;
        double m = l[0];
        for (int e = 1; e < E; ++e)
            if (l[e] > m)
                m = l[e];
        double den = 0.0;
        for (int e = 0; e < E; ++e)
            den += exp(l[e] - m);
        for (int e = 0; e < E; ++e)
            scores[(size_t)t * E + e] = (float)(exp(l[e] - m) / den);
    }
}

/* Optional sigmoid gate of a shared expert: g[t] = 1/(1+exp(-x_t . w_sg)).
 * Not in the paper; part of the Qwen-shaped workload definition. */
void oracle_shared_gate(const void *X, const void *w_sg, int T, int d, int dtype,
                        double *g)
{
    for (int t = 0; t < T; ++t) {
        double acc = 0.0;
        for (int h = 0; h < d; ++h)
            acc += load_elem(X, dtype, (size_t)t * d + h) * load_elem(w_sg, dtype, h);
        g[t] = 1.0 / (1.0 + exp(-acc));
    }
}

/* ---------------------------------- Eq. (6): candidate set, sorted per token */

typedef struct {
    float s;
    int32_t id;
} cand_t;

static int cmp_cand(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    return (a->id > b->id) - (a->id < b->id); /* equal scores: lower expert id first */
}

/* Per-token Top-K_orig candidates in descending order of score (Section 3.3,
 * Eq. (6) and the paragraph after Eq. (9)).  Whole row sorted by (score down,
 * expert id up); the first K entries are the candidates. */
void oracle_topk(const float *scores, int T, int E, int K, int32_t *ids, float *s)
{
    cand_t *row = (cand_t *)malloc((size_t)E * sizeof *row);
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            row[e].s = scores[(size_t)t * E + e];
            row[e].id = e;
        }
        qsort(row, (size_t)E, sizeof *row, cmp_cand);
        for (int j = 0; j < K; ++j) {
            ids[(size_t)t * K + j] = row[j].id;
            s[(size_t)t * K + j] = row[j].s;
        }
    }
    free(row);
}

/* ------------------------------------------- Section 3.3: Alloc-T selection */

typedef struct {
    float s;
    int32_t t, j;
} pool_t;

static int cmp_pool(const void *pa, const void *pb)
{
    const pool_t *a = (const pool_t *)pa, *b = (const pool_t *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    if (a->t != b->t) return (a->t > b->t) - (a->t < b->t); /* lower token first */
    return (a->j > b->j) - (a->j < b->j);                   /* then lower rank   */
}

/* Alloc-T as the paper states the procedure (paragraph after Eq. (9)):
 *   1. keep the Top-K_base entries (ranks j < Kb) of every token;
 *   2. pool the remaining K_orig - K_base candidates of all tokens and keep the
 *      globally largest B - T*Kb of them.
 * Equal scores are ordered by lower token, then lower rank (the paper is
 * silent on ties).  kept[t,j] in {0,1}; keep_count[t] = sum_j kept[t,j].
 * Returns 0, or -1 if the budget is infeasible (B < T*Kb violates Eq. (9),
 * B > T*K exceeds the candidate set). */
int oracle_alloc_t(const float *topk_s, int T, int K, int Kb, int64_t B,
                   uint8_t *kept, int32_t *keep_count)
{
    if (Kb < 0 || Kb > K || B < (int64_t)T * Kb || B > (int64_t)T * K)
        return -1;
    memset(kept, 0, (size_t)T * K);
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < Kb; ++j)
            kept[(size_t)t * K + j] = 1;

    size_t n_pool = (size_t)T * (size_t)(K - Kb);
    int64_t extra = B - (int64_t)T * Kb;
    if (n_pool > 0) {
        pool_t *pool = (pool_t *)malloc(n_pool * sizeof *pool);
        size_t n = 0;
        for (int t = 0; t < T; ++t)
            for (int j = Kb; j < K; ++j) {
                pool[n].s = topk_s[(size_t)t * K + j];
                pool[n].t = t;
                pool[n].j = j;
                ++n;
            }
        qsort(pool, n_pool, sizeof *pool, cmp_pool);
        for (int64_t i = 0; i < extra; ++i)
            kept[(size_t)pool[i].t * K + pool[i].j] = 1;
        free(pool);
    }
    for (int t = 0; t < T; ++t) {
        int32_t c = 0;
        for (int j = 0; j < K; ++j)
            c += kept[(size_t)t * K + j];
        keep_count[t] = c;
    }
    return 0;
}

/* --------------------------------------------------- expert-sorted dispatch */

/* Rows of the selected (token, expert) pairs in the order (expert up, token
 * up).  Not in the paper (it is how the feed-forward executions of the activated
 * experts, Section 3.1, are batched); the order is unique because a token
 * selects an expert at most once.
 *   expert_offsets[e] .. expert_offsets[e+1]  = rows of expert e
 *   row_token[r], row_rank[r]                  = the pair behind row r
 *   inv_row[t,j]                               = row of pair (t,j), -1 if dropped
 * A pair (t,j) is selected iff kept[t,j] != 0.  Returns the number of rows. */
int64_t oracle_dispatch(const int32_t *topk_ids, const uint8_t *kept, int T, int K,
                        int E, int32_t *expert_offsets, int32_t *row_token,
                        int32_t *row_rank, int32_t *inv_row)
{
    int64_t r = 0;
    for (size_t i = 0; i < (size_t)T * K; ++i)
        inv_row[i] = -1;
    for (int e = 0; e < E; ++e) {
        expert_offsets[e] = (int32_t)r;
        for (int t = 0; t < T; ++t)
            for (int j = 0; j < K; ++j)
                if (kept[(size_t)t * K + j] && topk_ids[(size_t)t * K + j] == e) {
                    row_token[r] = t;
                    row_rank[r] = j;
                    inv_row[(size_t)t * K + j] = (int32_t)r;
                    ++r;
                }
    }
    expert_offsets[E] = (int32_t)r;
    return r;
}

/* ------------------------------------------------- expert network, Eq. (2) */

/* out[0..d) = ( silu(x W1) (*) (x W3) ) W2 for one token x[0..d) (double).
 * W1, W3: [d, I]; W2: [I, d]; element type dtype.  hbuf: scratch of 3*I
 * doubles.  Every sum runs over its index in ascending order; the loops walk
 * the row-major matrices row by row. */
static void swiglu_ffn(const double *x, const void *W1, const void *W3,
                       const void *W2, int d, int I, int dtype, double *hbuf,
                       double *out)
{
    double *a = hbuf + I, *b = hbuf + 2 * (size_t)I;
    for (int i = 0; i < I; ++i)
        a[i] = b[i] = 0.0;
    for (int h = 0; h < d; ++h)
        for (int i = 0; i < I; ++i) {
            a[i] += x[h] * load_elem(W1, dtype, (size_t)h * I + i);
            b[i] += x[h] * load_elem(W3, dtype, (size_t)h * I + i);
        }
    for (int i = 0; i < I; ++i)
        hbuf[i] = (a[i] / (1.0 + exp(-a[i]))) * b[i];
    for (int c = 0; c < d; ++c)
        out[c] = 0.0;
    for (int i = 0; i < I; ++i)
        for (int c = 0; c < d; ++c)
            out[c] += hbuf[i] * load_elem(W2, dtype, (size_t)i * d + c);
}

/* Exported single-expert evaluation (used by the closed-form pins). */
void oracle_expert_ffn(const void *x, const void *W1, const void *W3, const void *W2,
                       int d, int I, int dtype, double *out)
{
    double *xd = (double *)malloc((size_t)d * sizeof *xd);
    double *hb = (double *)malloc(3 * (size_t)I * sizeof *hb);
    for (int h = 0; h < d; ++h)
        xd[h] = load_elem(x, dtype, (size_t)h);
    swiglu_ffn(xd, W1, W3, W2, d, I, dtype, hb, out);
    free(hb);
    free(xd);
}

/* Layer output by the literal Eq. (2):  y_t = sum_{i=1..N} w_{t,i} E_i(x_t),
 * with w_{t,i} the retained routing score of a selected pair and 0 otherwise
 * (no renormalisation), plus the always-on shared expert of the workload:
 *   y_t += g_t * Shared(x_t),  g_t = 1 or the sigmoid gate (sgate != NULL).
 * dense != 0: every one of the N experts is evaluated and multiplied by its
 * weight, zeros included (tiny sizes only).  dense == 0: zero-weight terms are
 * skipped.  Only the tokens listed in tok[0..n_tok) are computed;
 * Y[q*d .. q*d+d) is the output of token tok[q].  W1/W3/W2 hold all E experts
 * back to back.  Ws1/Ws3/Ws2 may be NULL (I_sh = 0). */
void oracle_moe_eq2(const void *X, const void *W1, const void *W3, const void *W2,
                    const void *Ws1, const void *Ws3, const void *Ws2,
                    const double *sgate, const int32_t *topk_ids, const float *topk_s,
                    const uint8_t *kept, int T, int d, int E, int I, int K, int I_sh,
                    int dtype, int dense, const int32_t *tok, int n_tok, double *Y)
{
    (void)T;
    int Imax = I > I_sh ? I : I_sh;
    double *xd = (double *)malloc((size_t)d * sizeof *xd);
    double *hb = (double *)malloc(3 * (size_t)(Imax > 0 ? Imax : 1) * sizeof *hb);
    double *eo = (double *)malloc((size_t)d * sizeof *eo);
    double *w = (double *)malloc((size_t)E * sizeof *w);
    for (int q = 0; q < n_tok; ++q) {
        int t = tok[q];
        double *y = Y + (size_t)q * d;
        for (int h = 0; h < d; ++h) {
            xd[h] = load_elem(X, dtype, (size_t)t * d + h);
            y[h] = 0.0;
        }
        for (int e = 0; e < E; ++e)
            w[e] = 0.0;
        for (int j = 0; j < K; ++j)
            if (kept[(size_t)t * K + j])
                w[topk_ids[(size_t)t * K + j]] = (double)topk_s[(size_t)t * K + j];
        for (int e = 0; e < E; ++e) {
            int selected = 0;
            for (int j = 0; j < K; ++j)
                if (kept[(size_t)t * K + j] && topk_ids[(size_t)t * K + j] == e)
                    selected = 1;
            if (!dense && !selected)
                continue;
            size_t w13 = (size_t)e * d * I, w2 = (size_t)e * I * d;
            swiglu_ffn(xd, offset_elems(W1, dtype, w13), offset_elems(W3, dtype, w13),
                       offset_elems(W2, dtype, w2), d, I, dtype, hb, eo);
            for (int h = 0; h < d; ++h)
                y[h] += w[e] * eo[h];
        }
        if (I_sh > 0 && Ws1) {
            swiglu_ffn(xd, Ws1, Ws3, Ws2, d, I_sh, dtype, hb, eo);
            double g = sgate ? sgate[t] : 1.0;
            for (int h = 0; h < d; ++h)
                y[h] += g * eo[h];
        }
    }
    free(w);
    free(eo);
    free(hb);
    free(xd);
}

/* The same layer output computed the way a dispatched implementation does it:
 * expert by expert over the rows of oracle_dispatch, one expert evaluation per
 * row, then per token the score-weighted sum over its rows via inv_row.  Its
 * agreement with oracle_moe_eq2(dense=1) pins the dispatch bookkeeping against
 * Eq. (2).  Computes all T tokens; Y is [T, d]. */
void oracle_moe_dispatched(const void *X, const void *W1, const void *W3,
                           const void *W2, const void *Ws1, const void *Ws3,
                           const void *Ws2, const double *sgate,
                           const float *topk_s, const int32_t *expert_offsets,
                           const int32_t *row_token, const int32_t *inv_row, int T,
                           int d, int E, int I, int K, int I_sh, int dtype, double *Y)
{
    int64_t R = expert_offsets[E];
    int Imax = I > I_sh ? I : I_sh;
    double *O = (double *)malloc((size_t)(R > 0 ? R : 1) * d * sizeof *O);
    double *xd = (double *)malloc((size_t)d * sizeof *xd);
    double *hb = (double *)malloc(3 * (size_t)(Imax > 0 ? Imax : 1) * sizeof *hb);
    double *eo = (double *)malloc((size_t)d * sizeof *eo);
    for (int e = 0; e < E; ++e)
        for (int64_t r = expert_offsets[e]; r < expert_offsets[e + 1]; ++r) {
            int t = row_token[r];
            for (int h = 0; h < d; ++h)
                xd[h] = load_elem(X, dtype, (size_t)t * d + h);
            size_t w13 = (size_t)e * d * I, w2 = (size_t)e * I * d;
            swiglu_ffn(xd, offset_elems(W1, dtype, w13), offset_elems(W3, dtype, w13),
                       offset_elems(W2, dtype, w2), d, I, dtype, hb, O + (size_t)r * d);
        }
    for (int t = 0; t < T; ++t) {
        double *y = Y + (size_t)t * d;
        for (int h = 0; h < d; ++h)
            y[h] = 0.0;
        for (int j = 0; j < K; ++j) {
            int32_t r = inv_row[(size_t)t * K + j];
            if (r < 0)
                continue;
            double wt = (double)topk_s[(size_t)t * K + j];
            for (int h = 0; h < d; ++h)
                y[h] += wt * O[(size_t)r * d + h];
        }
        if (I_sh > 0 && Ws1) {
            for (int h = 0; h < d; ++h)
                xd[h] = load_elem(X, dtype, (size_t)t * d + h);
            swiglu_ffn(xd, Ws1, Ws3, Ws2, d, I_sh, dtype, hb, eo);
            double g = sgate ? sgate[t] : 1.0;
            for (int h = 0; h < d; ++h)
                y[h] += g * eo[h];
        }
    }
    free(eo);
    free(hb);
    free(xd);
    free(O);
}
