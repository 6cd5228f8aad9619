/*
 * step_oracle.c -- plain, slow, obviously-correct CPU definitions of the three
 * operations of one STEP decode step.  TEST INFRASTRUCTURE ONLY: the product
 * path (the HIP library) never includes, links or calls anything in here, and
 * nothing in here includes or calls the product path.
 *
 * What each function follows in the paper (arxiv 2601.09093, "STEP"):
 *   oracle_paged_decode_attn  - the attention inside NextToken(t) of Algorithm 1.
 *                               The paper gives no formula for it; this is the
 *                               textbook definition softmax(q K^T * scale) V for
 *                               one query token per trace over a paged KV cache.
 *   oracle_step_score         - Section 4.1 "Model Architecture":
 *                               y = sigma(W2 act(W1 h + b1) + b2); Table 5 fixes
 *                               act = ReLU (GELU-erf is a caller-selected variant).
 *   oracle_running_mean       - Section 4.3: score_t = (1/n) sum_{i<=n} y_i^t,
 *                               "Update score_t" of Algorithm 1.
 *   oracle_prune_free         - Algorithm 1: t* = argmin score_t,
 *                               ReleaseKVCache(t*), T <- T \ {t*}, applied k times
 *                               (Section 4.2: prune lowest average score, release
 *                               its KV cache).
 *   oracle_reserve_pages      - Section 4.2's trigger: prune one trace at a time
 *                               while the next decode step cannot be scheduled,
 *                               then hand out the new pages.
 *   oracle_append_kv          - the KV-cache write of NextToken(t).
 *   oracle_weighted_vote      - Section 4.3 / WeightedVote of Algorithm 1.
 *
 * All floating-point work is float64 on the exact values of the bf16/fp32
 * inputs, except the running-mean state, which is fp32 by definition of the
 * boundary (sum fp32, count int32, IEEE fp32 divide).
 * No blocking, fusion, or reordering: every loop is the definition written out.
 * OpenMP only splits independent output units (one (trace, head) row, one
 * boundary); it never changes the order of any floating-point sum.
 *
 * Parity pins (tests/test_oracle_*.py): every function here is pinned against
 * closed forms, brute-force library evaluation and invariants; none is
 * "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum {
    ORACLE_OK = 0,
    ORACLE_EINVAL = 1,      /* bad dimensions / null pointer / k > live        */
    ORACLE_EPAGE = 2,       /* block-table entry outside [0, NP)               */
    ORACLE_ELEN = 3,        /* seq_len < 0 or > MAXB * P                        */
    ORACLE_EINDEX = 4,      /* boundary_idx outside [0, R) / trace_of outside N */
    ORACLE_ENAN = 5,        /* NaN score among live traces                     */
    ORACLE_EREFCOUNT = 6    /* refcount would drop below zero                  */
};

static inline double bf16_to_f64(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* ------------------------------------------------------------------------ */
/* Attention                                                                */
/* ------------------------------------------------------------------------ */

/* One output row: trace i, query head h.  Two passes over the trace's tokens.
 * out_row[D] (float64, not rounded), *lse = M + log(sum_t exp(x_t - M)) in
 * natural-log units (the log of the softmax denominator), used by the
 * split-and-merge pin.  L == 0 gives a zero row and lse = -inf. */
static int attn_row(int Hq, int Hkv, int D, int P, int MAXB, int NP, double scale,
                    const uint16_t *q, const uint16_t *k_pages, const uint16_t *v_pages,
                    const int32_t *block_tables, const int32_t *seq_lens,
                    int i, int h, double *out_row, double *lse, double *x /* scratch [MAXB*P] */)
{
    const int G = Hq / Hkv;
    const int g = h / G; /* consecutive query heads share one KV head */
    const int64_t L = seq_lens[i];
    for (int c = 0; c < D; ++c) out_row[c] = 0.0;
    if (lse) *lse = -INFINITY;
    if (L < 0 || L > (int64_t)MAXB * P) return ORACLE_ELEN;
    if (L == 0) return ORACLE_OK;

    const uint16_t *qrow = q + ((int64_t)i * Hq + h) * D;
    const int32_t *bt = block_tables + (int64_t)i * MAXB;

    /* pass 1: logits x_t = scale * <q, k_t>, and their maximum */
    double M = -INFINITY;
    for (int64_t t = 0; t < L; ++t) {
        const int32_t p = bt[t / P];
        if (p < 0 || p >= NP) return ORACLE_EPAGE;
        const int s = (int)(t % P);
        const uint16_t *krow = k_pages + (((int64_t)p * Hkv + g) * P + s) * D;
        double dot = 0.0;
        for (int c = 0; c < D; ++c) dot += bf16_to_f64(qrow[c]) * bf16_to_f64(krow[c]);
        x[t] = scale * dot;
        if (x[t] > M) M = x[t];
    }
    /* pass 2: weights w_t = exp(x_t - M), out = sum w_t v_t / sum w_t */
    double denom = 0.0;
    for (int64_t t = 0; t < L; ++t) {
        const int32_t p = bt[t / P];
        const int s = (int)(t % P);
        const uint16_t *vrow = v_pages + (((int64_t)p * Hkv + g) * P + s) * D;
        const double w = exp(x[t] - M);
        denom += w;
        for (int c = 0; c < D; ++c) out_row[c] += w * bf16_to_f64(vrow[c]);
    }
    for (int c = 0; c < D; ++c) out_row[c] /= denom;
    if (lse) *lse = M + log(denom);
    return ORACLE_OK;
}

/* Selected rows: for r < n_sel computes out[r][:] for (sel_trace[r], sel_head[r]).
 * lse may be NULL.  Returns the first (lowest r) error met, ORACLE_OK otherwise. */
int oracle_paged_decode_attn_rows(int N, int Hq, int Hkv, int D, int P, int MAXB, int NP, double scale,
                                  const uint16_t *q, const uint16_t *k_pages, const uint16_t *v_pages,
                                  const int32_t *block_tables, const int32_t *seq_lens,
                                  int n_sel, const int32_t *sel_trace, const int32_t *sel_head,
                                  double *out, double *lse)
{
    if (N < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || P <= 0 || MAXB < 0 || NP < 0 || n_sel < 0) return ORACLE_EINVAL;
    if (Hq % Hkv != 0) return ORACLE_EINVAL;
    if (!q || !k_pages || !v_pages || !block_tables || !seq_lens || !out) return ORACLE_EINVAL;
    for (int r = 0; r < n_sel; ++r)
        if (sel_trace[r] < 0 || sel_trace[r] >= N || sel_head[r] < 0 || sel_head[r] >= Hq) return ORACLE_EINVAL;

    int *err = (int *)calloc((size_t)(n_sel > 0 ? n_sel : 1), sizeof(int));
    if (!err) return ORACLE_EINVAL;
#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * ((size_t)MAXB * P + 1));
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_sel; ++r) {
            err[r] = attn_row(Hq, Hkv, D, P, MAXB, NP, scale, q, k_pages, v_pages, block_tables, seq_lens,
                              sel_trace[r], sel_head[r], out + (int64_t)r * D, lse ? lse + r : NULL, x);
        }
        free(x);
    }
    int rc = ORACLE_OK;
    for (int r = 0; r < n_sel; ++r)
        if (err[r] != ORACLE_OK) { rc = err[r]; break; }
    free(err);
    return rc;
}

/* All rows: out[N][Hq][D], lse[N][Hq] (nullable). */
int oracle_paged_decode_attn(int N, int Hq, int Hkv, int D, int P, int MAXB, int NP, double scale,
                             const uint16_t *q, const uint16_t *k_pages, const uint16_t *v_pages,
                             const int32_t *block_tables, const int32_t *seq_lens,
                             double *out, double *lse)
{
    if (N < 0 || Hq <= 0) return ORACLE_EINVAL;
    const int n_sel = N * Hq;
    int32_t *st = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_sel > 0 ? n_sel : 1));
    int32_t *sh = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_sel > 0 ? n_sel : 1));
    if (!st || !sh) { free(st); free(sh); return ORACLE_EINVAL; }
    for (int i = 0; i < N; ++i)
        for (int h = 0; h < Hq; ++h) { st[i * Hq + h] = i; sh[i * Hq + h] = h; }
    const int rc = oracle_paged_decode_attn_rows(N, Hq, Hkv, D, P, MAXB, NP, scale, q, k_pages, v_pages,
                                                 block_tables, seq_lens, n_sel, st, sh, out, lse);
    free(st);
    free(sh);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Step scorer                                                              */
/* ------------------------------------------------------------------------ */

/* act: 0 = ReLU (the paper's), 1 = GELU in its exact erf form. */
static inline double activation(double z, int act)
{
    if (act == 0) return z > 0.0 ? z : 0.0;
    return 0.5 * z * (1.0 + erf(z / sqrt(2.0)));
}

/* hidden [R][d] bf16; boundary_idx [B]; W1 [m][d] bf16 (row j = weights of
 * hidden unit j, i.e. W1 h is a matrix-vector product); b1 [m] fp32; W2 [m]
 * bf16; b2 fp32.  logits[B], probs[B] float64. */
int oracle_step_score(int R, int d, int m, int B, int act,
                      const uint16_t *hidden, const int32_t *boundary_idx,
                      const uint16_t *W1, const float *b1, const uint16_t *W2, float b2,
                      double *logits, double *probs)
{
    if (R < 0 || d <= 0 || m <= 0 || B < 0 || (act != 0 && act != 1)) return ORACLE_EINVAL;
    if (!hidden || !W1 || !b1 || !W2 || (B > 0 && (!boundary_idx || !logits || !probs))) return ORACLE_EINVAL;
    for (int b = 0; b < B; ++b)
        if (boundary_idx[b] < 0 || boundary_idx[b] >= R) return ORACLE_EINDEX;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const uint16_t *x = hidden + (int64_t)boundary_idx[b] * d;
        double logit = (double)b2;
        for (int j = 0; j < m; ++j) {
            const uint16_t *w = W1 + (int64_t)j * d;
            double z = (double)b1[j];
            for (int c = 0; c < d; ++c) z += bf16_to_f64(w[c]) * bf16_to_f64(x[c]);
            logit += bf16_to_f64(W2[j]) * activation(z, act);
        }
        logits[b] = logit;
        probs[b] = 1.0 / (1.0 + exp(-logit));
    }
    return ORACLE_OK;
}

/* Running mean of step scores per trace, boundaries taken in index order.
 * State is fp32/int32 (that is the boundary's definition of the state); a
 * trace with no scored step yet has score +inf (it is pruned last). */
int oracle_running_mean(int B, int N, const int32_t *trace_of, const float *probs,
                        float *score_sum, int32_t *score_cnt, float *scores)
{
    if (B < 0 || N < 0) return ORACLE_EINVAL;
    for (int b = 0; b < B; ++b)
        if (trace_of[b] < 0 || trace_of[b] >= N) return ORACLE_EINDEX;
    for (int b = 0; b < B; ++b) {
        const int t = trace_of[b];
        score_sum[t] = score_sum[t] + probs[b];
        score_cnt[t] = score_cnt[t] + 1;
    }
    for (int t = 0; t < N; ++t)
        scores[t] = score_cnt[t] > 0 ? score_sum[t] / (float)score_cnt[t] : INFINITY;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Prune + free                                                             */
/* ------------------------------------------------------------------------ */

/* k rounds of Algorithm 1's prune: take the live trace (seq_lens > 0) with the
 * lowest score (ties: lowest index), release every page it references
 * (refcount - 1; a page whose count reaches 0 is freed), clear its block-table
 * row to -1 and its seq_len to 0.  pruned[k] is in pruning order; freed_pages
 * is the set of freed page ids in ascending order, *n_freed its size.
 * On any error nothing is modified. */
int oracle_prune_free(int N, int MAXB, int NP, int P, const float *scores, int k,
                      int32_t *refcounts, int32_t *block_tables, int32_t *seq_lens,
                      int32_t *pruned, int32_t *freed_pages, int32_t *n_freed)
{
    if (N < 0 || MAXB < 0 || NP < 0 || P <= 0 || k < 0) return ORACLE_EINVAL;
    if (!scores || !refcounts || !block_tables || !seq_lens || !n_freed) return ORACLE_EINVAL;
    int live = 0;
    for (int i = 0; i < N; ++i) {
        if (seq_lens[i] < 0 || (int64_t)seq_lens[i] > (int64_t)MAXB * P) return ORACLE_ELEN;
        if (seq_lens[i] > 0) {
            ++live;
            if (isnan(scores[i])) return ORACLE_ENAN;
        }
    }
    if (k > live) return ORACLE_EINVAL;

    /* choose the victims first, on a scratch copy of the live mask */
    char *taken = (char *)calloc((size_t)(N > 0 ? N : 1), 1);
    int32_t *rc = (int32_t *)malloc(sizeof(int32_t) * (size_t)(NP > 0 ? NP : 1));
    if (!taken || !rc) { free(taken); free(rc); return ORACLE_EINVAL; }
    memcpy(rc, refcounts, sizeof(int32_t) * (size_t)NP);
    int err = ORACLE_OK;
    for (int r = 0; r < k; ++r) {
        int best = -1;
        for (int i = 0; i < N; ++i) {
            if (seq_lens[i] <= 0 || taken[i]) continue;
            if (best < 0 || scores[i] < scores[best]) best = i; /* strict <: lowest index wins ties */
        }
        taken[best] = 1;
        pruned[r] = best;
        const int nb = (seq_lens[best] + P - 1) / P;
        for (int j = 0; j < nb; ++j) {
            const int32_t p = block_tables[(int64_t)best * MAXB + j];
            if (p < 0 || p >= NP) { err = ORACLE_EPAGE; goto done; }
            if (rc[p] <= 0) { err = ORACLE_EREFCOUNT; goto done; }
            rc[p] -= 1;
        }
    }
    /* commit */
    {
        int nf = 0;
        for (int p = 0; p < NP; ++p) {
            if (rc[p] == 0 && refcounts[p] > 0) freed_pages[nf++] = p; /* ascending page id */
            refcounts[p] = rc[p];
        }
        *n_freed = nf;
        for (int r = 0; r < k; ++r) {
            const int t = pruned[r];
            for (int j = 0; j < MAXB; ++j) block_tables[(int64_t)t * MAXB + j] = -1;
            seq_lens[t] = 0;
        }
    }
done:
    free(taken);
    free(rc);
    return err;
}

/* ------------------------------------------------------------------------ */
/* Memory trigger + page allocation (Section 4.2; Algorithm 1's GPUMemoryFull) */
/* ------------------------------------------------------------------------ */

/* Before the next decode step: a live trace whose length is a multiple of P
 * opens a new page with its next token.  Section 4.2's trigger (memory is
 * full and the next step's KV cache does not fit) is read as:
 * fewer free pages (refcount 0) than traces that need one.  While that holds,
 * prune the live trace with the lowest score (ties: lowest index) and release
 * its pages, exactly as oracle_prune_free does for k = 1.  Then every trace
 * that still needs a page, in ascending trace index, takes the smallest free
 * page id: block_tables[i][L_i / P] = page, refcounts[page] = 1.
 * pruned[] (capacity N) lists the pruned traces in order, new_pages[i] is the
 * page given to trace i or -1.  On an error nothing is modified. */
int oracle_reserve_pages(int N, int MAXB, int NP, int P, const float *scores,
                         int32_t *refcounts, int32_t *block_tables, int32_t *seq_lens,
                         int32_t *pruned, int32_t *n_pruned, int32_t *new_pages)
{
    if (N < 0 || MAXB < 0 || NP < 0 || P <= 0) return ORACLE_EINVAL;
    int32_t *rc = (int32_t *)malloc(sizeof(int32_t) * (size_t)(NP > 0 ? NP : 1));
    int32_t *sl = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    if (!rc || !sl) { free(rc); free(sl); return ORACLE_EINVAL; }
    memcpy(rc, refcounts, sizeof(int32_t) * (size_t)NP);
    memcpy(sl, seq_lens, sizeof(int32_t) * (size_t)N);
    int err = ORACLE_OK, np = 0;
    for (int i = 0; i < N; ++i)
        if (sl[i] < 0 || (int64_t)sl[i] > (int64_t)MAXB * P) { err = ORACLE_ELEN; goto done; }
    for (;;) {
        int needed = 0, nfree = 0;
        for (int i = 0; i < N; ++i)
            if (sl[i] > 0 && sl[i] % P == 0) {
                if (sl[i] / P >= MAXB) { err = ORACLE_ELEN; goto done; } /* row has no entry left */
                ++needed;
            }
        for (int p = 0; p < NP; ++p)
            if (rc[p] == 0) ++nfree;
        if (nfree >= needed) break;
        int best = -1;
        for (int i = 0; i < N; ++i) {
            if (sl[i] <= 0) continue;
            if (isnan(scores[i])) { err = ORACLE_ENAN; goto done; }
            if (best < 0 || scores[i] < scores[best]) best = i;
        }
        /* needed > 0 implies a live trace exists */
        const int nb = (sl[best] + P - 1) / P;
        for (int j = 0; j < nb; ++j) {
            const int32_t p = block_tables[(int64_t)best * MAXB + j];
            if (p < 0 || p >= NP) { err = ORACLE_EPAGE; goto done; }
            if (rc[p] <= 0) { err = ORACLE_EREFCOUNT; goto done; }
            rc[p] -= 1;
        }
        sl[best] = 0;
        pruned[np++] = best;
    }
    /* commit: pruned rows, then allocation */
    for (int r = 0; r < np; ++r) {
        const int t = pruned[r];
        for (int j = 0; j < MAXB; ++j) block_tables[(int64_t)t * MAXB + j] = -1;
    }
    {
        int next = 0;
        for (int i = 0; i < N; ++i) {
            new_pages[i] = -1;
            if (sl[i] > 0 && sl[i] % P == 0) {
                while (rc[next] != 0) ++next; /* exists: nfree >= needed */
                rc[next] = 1;
                block_tables[(int64_t)i * MAXB + sl[i] / P] = next;
                new_pages[i] = next;
            }
        }
    }
    memcpy(refcounts, rc, sizeof(int32_t) * (size_t)NP);
    memcpy(seq_lens, sl, sizeof(int32_t) * (size_t)N);
    *n_pruned = np;
done:
    free(rc);
    free(sl);
    return err;
}

/* Append the newest token's K and V rows (k_new, v_new: [N][Hkv][D] bf16) to
 * every live trace: row L_i of trace i lives in page block_tables[i][L_i / P],
 * slot L_i % P; then L_i += 1.  This is the KV-cache write of NextToken(t) in
 * Algorithm 1 (the paper leaves it to the serving engine).  A page written to
 * must be private (refcount 1).  On an error nothing is modified. */
int oracle_append_kv(int N, int Hkv, int D, int P, int MAXB, int NP,
                     const uint16_t *k_new, const uint16_t *v_new, uint16_t *k_pages, uint16_t *v_pages,
                     const int32_t *block_tables, const int32_t *refcounts, int32_t *seq_lens)
{
    if (N < 0 || Hkv <= 0 || D <= 0 || P <= 0 || MAXB < 0 || NP < 0) return ORACLE_EINVAL;
    for (int i = 0; i < N; ++i) {
        const int64_t L = seq_lens[i];
        if (L < 0 || L > (int64_t)MAXB * P) return ORACLE_ELEN;
        if (L == 0) continue;
        if (L == (int64_t)MAXB * P) return ORACLE_ELEN;
        const int32_t p = block_tables[(int64_t)i * MAXB + L / P];
        if (p < 0 || p >= NP) return ORACLE_EPAGE;
        if (refcounts && refcounts[p] != 1) return ORACLE_EREFCOUNT;
    }
    for (int i = 0; i < N; ++i) {
        const int64_t L = seq_lens[i];
        if (L == 0) continue;
        const int32_t p = block_tables[(int64_t)i * MAXB + L / P];
        const int s = (int)(L % P);
        for (int g = 0; g < Hkv; ++g) {
            const int64_t dst = (((int64_t)p * Hkv + g) * P + s) * D;
            const int64_t src = ((int64_t)i * Hkv + g) * D;
            memcpy(k_pages + dst, k_new + src, sizeof(uint16_t) * (size_t)D);
            memcpy(v_pages + dst, v_new + src, sizeof(uint16_t) * (size_t)D);
        }
        seq_lens[i] = (int32_t)(L + 1);
    }
    return ORACLE_OK;
}

/* Weighted majority vote over the final answers (Section 4.3; WeightedVote in
 * Algorithm 1): answer[i] >= 0 is the answer id of a finished trace, -1 means
 * the trace has none (pruned or unfinished).  The weight of an answer is the
 * fp32 sum, in trace index order, of the scores of the traces that gave it;
 * the winner has the largest weight (ties: smallest answer id).  Returns -1 in
 * *winner when nobody answered. */
int oracle_weighted_vote(int N, const int32_t *answer, const float *scores, int32_t *winner, float *weight)
{
    if (N < 0) return ORACLE_EINVAL;
    int32_t best = -1;
    float best_w = 0.0f;
    for (int i = 0; i < N; ++i) {
        if (answer[i] < 0) continue;
        if (isnan(scores[i])) return ORACLE_ENAN;
        float w = 0.0f;
        for (int j = 0; j < N; ++j)
            if (answer[j] == answer[i]) w = w + scores[j];
        if (best < 0 || w > best_w || (w == best_w && answer[i] < best)) {
            best = answer[i];
            best_w = w;
        }
    }
    *winner = best;
    *weight = best_w;
    return ORACLE_OK;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
