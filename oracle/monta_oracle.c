/*
 * monta_oracle.c -- plain, slow CPU reference of the MoE token dispatch / combine
 * path of MoNTA (arxiv 2411.00662).  Built without OpenMP it is single-threaded:
 * that build is the parity reference.  A second build with -fopenmp runs the same
 * loops with the independent outer iterations (tokens, rows, blocks) of route,
 * pack, regather and combine dealt to all host cores; it exists only to time the
 * CPU baseline on every core, computes exactly the same bytes (no iteration reads
 * what another writes) and is checked against the first build by a test.  The plan
 * stays serial in both.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the HIP path can be checked
 * against something that is obviously the definition.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it; the product never does.
 * It shares no code, header, table or helper with the HIP path.
 *
 * The paper claims its transforms (TP-group split "Drop", chunking along the
 * sequence, intra-node gather, D2D copy to index offsets) are exact
 * rearrangements of the plain AllToAll (section "Pipelining": the gathered result
 * is equivalent to the original AllToAll; paragraph "AllGather and D2D copy
 * Pipelining": the final output equals the original data).  So the *result* is
 * defined by the plain MoE data flow of section "Expert Parallel" (Routing,
 * Permutation, Dispatch, Combine, Unpermutation) and tp / slices only decide the
 * intermediate send-buffer layout (STAGE).
 *
 * Floating point: gate weights and the combine sum are evaluated in double and
 * rounded once to the output type.  Everything else is integer / byte work.
 *
 * Readings where the paper is silent (listed with their reasons in the design
 * notes of the repository):
 *   - top-k ties go to the lower expert index; selection is on the raw logits;
 *   - capacity C = ceil(cf*T*k/E) (cf = 0: no drop), global over all tokens,
 *     the C lowest token indices of each expert are kept;
 *   - compact (unpadded) expert segments; expert order = (EP rank, local expert);
 *   - the TP split is over tokens: inside slice j virtual TP rank r owns the r-th
 *     run of T/(S*tp) tokens; STAGE is laid out [slice][tp rank][expert][rows];
 *   - dropped pairs contribute nothing to the combine, gates are not renormalised
 *     again after a drop.
 *
 * Parity pins (tests/, CPU only): brute-force sort routing, dense-softmax gates,
 * numpy stable argsort permutation, dense one-hot MoE combine, (tp,S)-independence,
 * round trip with identity experts, the 1/t volume closed form and Table 8 volumes.
 * STAGE layout itself: parity unpinned by the paper (its Fig. 7 is not available);
 * fixed by the reading above and checked through the regather post-condition.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#define ORACLE_PARALLEL_FOR _Pragma("omp parallel for schedule(static)")
#else
#define ORACLE_PARALLEL_FOR
#endif

/* threads the loops above run on: 1 in the plain build */
int monta_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)
#define ORACLE_NOMEM (-2)

/* ---------------------------------------------------------------- routing */

/* Section "Expert Parallel", Routing: per token the TopK expert indices and
 * probabilities.  Experts are ordered by (logit descending, index ascending);
 * slot j = 0 is the strongest choice.  Probabilities are the softmax of the
 * logits (section "MoE": linear, softmax, TopK gate); with renorm != 0 they are
 * renormalised over the k winners, which equals a softmax over the k winning
 * logits.  exp() is shifted by the largest logit, which changes nothing
 * mathematically. */
int monta_oracle_route(int64_t T, int E, int k, int renorm, const float *logits,
                       int32_t *topk_idx, float *gates)
{
    if (T < 0 || E < 1 || k < 1 || k > E || !logits || !topk_idx || !gates)
        return ORACLE_BAD_ARG;
    if (E > 4096) return ORACLE_BAD_ARG;       /* the per-token scratch below lives on the stack */
    ORACLE_PARALLEL_FOR
    for (int64_t t = 0; t < T; ++t) {
        char taken[4096];
        double w[4096];
        const float *l = logits + t * E;
        memset(taken, 0, (size_t)E);
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e; /* strict: first index wins a tie */
            }
            taken[best] = 1;
            topk_idx[t * k + j] = best;
        }
        const double top = (double)l[topk_idx[t * k]];
        double denom = 0.0;
        for (int j = 0; j < k; ++j) {
            w[j] = exp((double)l[topk_idx[t * k + j]] - top);
            if (renorm) denom += w[j];
        }
        if (!renorm)
            for (int e = 0; e < E; ++e) denom += exp((double)l[e] - top);
        for (int j = 0; j < k; ++j) gates[t * k + j] = (float)(w[j] / denom);
    }
    return ORACLE_OK;
}

/* Section "MoE": the gating network is a linear layer before the softmax and TopK.  logits[t][e] =
 * sum_h x[t][h] * w[e][h], with x [T][H] and w [E][H] in the activation type (0 = fp32, 1 = bf16 bits);
 * every product is exact in double, the sum runs over h in ascending order in double and is rounded
 * once to fp32. */
int monta_oracle_gate(int64_t T, int H, int E, int dtype, const void *x, const void *w, float *logits)
{
    if (T < 0 || H < 1 || E < 1 || (dtype != 0 && dtype != 1)) return ORACLE_BAD_ARG;
    for (int64_t t = 0; t < T; ++t)
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h) {
                double a, b;
                if (dtype == 0) {
                    a = (double)((const float *)x)[t * H + h];
                    b = (double)((const float *)w)[(int64_t)e * H + h];
                } else {
                    uint32_t ua = (uint32_t)((const uint16_t *)x)[t * H + h] << 16;
                    uint32_t ub = (uint32_t)((const uint16_t *)w)[(int64_t)e * H + h] << 16;
                    float fa, fb;
                    memcpy(&fa, &ua, 4);
                    memcpy(&fb, &ub, 4);
                    a = fa;
                    b = fb;
                }
                acc += a * b;
            }
            logits[t * E + e] = (float)acc;
        }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------- plan */

/* Capacity per expert.  The paper never drops tokens for capacity; the workloads
 * of this repository do, with the usual definition. */
int64_t monta_oracle_capacity(int64_t T, int E, int k, double cf)
{
    if (cf <= 0.0) return T;
    double c = ceil(cf * (double)T * (double)k / (double)E);
    if (c > (double)T) return T;
    if (c < 0.0) return 0;
    return (int64_t)c;
}

/* Section "Expert Parallel", Permutation: rows that chose the same expert are
 * grouped together.  Written out as the definition of a stable counting sort by
 * expert id over pairs (t, j) in token order: rank(t, e) is the number of earlier
 * tokens that chose e.  A pair is kept iff rank < C.
 *
 * Units: unit u = tokens [u*Tu, (u+1)*Tu), Tu = T/(S*tp); slice = u / tp (chunk j
 * of Eq. 4, taken along the sequence), virtual TP rank = u % tp (the "Drop" split
 * of section "Pipelining": each TP rank keeps 1/t of the identical activations).
 *
 * Outputs (all int32 unless noted):
 *   counts[E], kept[E], offsets[E+1]              expert histogram, after capacity, exclusive scan
 *   pos_final[T*k]   row of pair in the expert-major FINAL buffer, -1 if dropped
 *   n[U*E]           kept pairs of expert e whose token lies in unit u
 *   stage_off[U*E]   first STAGE row of block (u,e): exclusive scan of n in (u,e) order
 *   unit_base[U*E]   first FINAL row of block (u,e): offsets[e] + sum_{u'<u} n[u'][e]
 *   pos_stage[T*k]   row of pair in STAGE, -1 if dropped
 *   send_rows[U*ep]  rows unit u sends to EP rank d (experts d*E/ep .. (d+1)*E/ep - 1)
 *   *alive           tokens with at least one kept pair (int64)
 *
 * padded != 0 selects the capacity-padded layout [E][C][H] of FINAL (the dispatch tensor of
 * capacity-based MoE layers): expert e owns rows [e*C, (e+1)*C), its kept rows come first, the rest is
 * padding.  Then offsets[e] = e*C and offsets[E] = E*C; the number of kept pairs is returned in *R.
 * STAGE is compact in both layouts.
 */
int monta_oracle_plan(int64_t T, int E, int k, int ep, int tp, int S, double cf, int padded, int64_t *R,
                      const int32_t *topk_idx, int32_t *counts, int32_t *kept,
                      int32_t *offsets, int32_t *pos_final, int32_t *n,
                      int32_t *stage_off, int32_t *unit_base, int32_t *pos_stage,
                      int32_t *send_rows, int64_t *alive)
{
    if (T < 1 || E < 1 || k < 1 || k > E || ep < 1 || tp < 1 || S < 1) return ORACLE_BAD_ARG;
    if (E % ep != 0) return ORACLE_BAD_ARG;
    const int64_t U = (int64_t)S * tp;
    if (T % U != 0) return ORACLE_BAD_ARG;
    const int64_t Tu = T / U;
    const int E_loc = E / ep;
    const int64_t C = monta_oracle_capacity(T, E, k, cf);

    int32_t *rank = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T * k));
    int32_t *before = (int32_t *)malloc(sizeof(int32_t) * (size_t)(U * E)); /* sum_{u'<u} n[u'][e] */
    if (!rank || !before) { free(rank); free(before); return ORACLE_NOMEM; }

    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int64_t t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            int e = topk_idx[t * k + j];
            if (e < 0 || e >= E) { free(rank); free(before); return ORACLE_BAD_ARG; }
            rank[t * k + j] = counts[e]++;
        }
    offsets[0] = 0;
    int64_t rows = 0;
    for (int e = 0; e < E; ++e) {
        kept[e] = counts[e] < C ? counts[e] : (int32_t)C;
        rows += kept[e];
        offsets[e + 1] = padded ? (int32_t)((e + 1) * C) : offsets[e] + kept[e];
    }
    *R = rows;
    for (int64_t i = 0; i < U * E; ++i) n[i] = 0;
    int64_t live = 0;
    for (int64_t t = 0; t < T; ++t) {
        int any = 0;
        for (int j = 0; j < k; ++j) {
            int e = topk_idx[t * k + j];
            if (rank[t * k + j] < C) {
                pos_final[t * k + j] = offsets[e] + rank[t * k + j];
                n[(t / Tu) * E + e] += 1;
                any = 1;
            } else {
                pos_final[t * k + j] = -1;
            }
        }
        live += any;
    }
    *alive = live;
    int32_t run = 0;
    for (int64_t u = 0; u < U; ++u)
        for (int e = 0; e < E; ++e) {
            stage_off[u * E + e] = run;
            run += n[u * E + e];
            before[u * E + e] = (u == 0) ? 0 : before[(u - 1) * E + e] + n[(u - 1) * E + e];
            unit_base[u * E + e] = offsets[e] + before[u * E + e];
        }
    for (int64_t t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            int e = topk_idx[t * k + j];
            int64_t u = t / Tu;
            if (pos_final[t * k + j] >= 0)
                pos_stage[t * k + j] = stage_off[u * E + e] + (rank[t * k + j] - before[u * E + e]);
            else
                pos_stage[t * k + j] = -1;
        }
    for (int64_t u = 0; u < U; ++u)
        for (int d = 0; d < ep; ++d) {
            int32_t s = 0;
            for (int el = 0; el < E_loc; ++el) s += n[u * E + d * E_loc + el];
            send_rows[u * ep + d] = s;
        }
    free(rank);
    free(before);
    return ORACLE_OK;
}

/* ------------------------------------------------------------ pack / gather */

/* Dispatch send buffer: unit by unit (slice-major, then virtual TP rank, as in
 * Eq. 4 and the "Drop" split), every kept pair's token row is copied bit for bit
 * to its STAGE row.  slice < 0 packs every slice. */
int monta_oracle_pack(int64_t T, int k, int tp, int S, int64_t row_bytes, const void *x,
                      const int32_t *pos_stage, void *stage, int slice)
{
    if (T < 1 || k < 1 || tp < 1 || S < 1 || row_bytes < 1 || slice >= S) return ORACLE_BAD_ARG;
    const int64_t U = (int64_t)S * tp, Tu = T / U;
    if (T % U != 0) return ORACLE_BAD_ARG;
    for (int64_t u = 0; u < U; ++u) {
        if (slice >= 0 && u / tp != slice) continue;
        ORACLE_PARALLEL_FOR
        for (int64_t t = u * Tu; t < (u + 1) * Tu; ++t)
            for (int j = 0; j < k; ++j) {
                int32_t p = pos_stage[t * k + j];
                if (p >= 0)
                    memcpy((char *)stage + (int64_t)p * row_bytes,
                           (const char *)x + t * row_bytes, (size_t)row_bytes);
            }
    }
    return ORACLE_OK;
}

/* Intra-node gather + D2D copy to the rows' index offsets (paragraph "AllGather and
 * D2D copy Pipelining", Fig. 7-8): every (unit, expert) block of STAGE goes to its
 * place in the expert-major FINAL buffer. */
/* The padded layout's padding rows [offsets[e] + kept[e], offsets[e+1]) are zero-filled. */
int monta_oracle_pad(int E, int64_t row_bytes, const int32_t *kept, const int32_t *offsets, void *final_)
{
    if (E < 1 || row_bytes < 1) return ORACLE_BAD_ARG;
    for (int e = 0; e < E; ++e) {
        const int64_t a = (int64_t)offsets[e] + kept[e], b = offsets[e + 1];
        if (b > a) memset((char *)final_ + a * row_bytes, 0, (size_t)((b - a) * row_bytes));
    }
    return ORACLE_OK;
}

int monta_oracle_regather(int tp, int S, int E, int64_t row_bytes, const int32_t *n,
                          const int32_t *stage_off, const int32_t *unit_base,
                          const void *stage, void *final_, int slice)
{
    if (tp < 1 || S < 1 || E < 1 || row_bytes < 1 || slice >= S) return ORACLE_BAD_ARG;
    const int64_t U = (int64_t)S * tp;
    for (int64_t u = 0; u < U; ++u) {
        if (slice >= 0 && u / tp != slice) continue;
        ORACLE_PARALLEL_FOR
        for (int e = 0; e < E; ++e)
            memcpy((char *)final_ + (int64_t)unit_base[u * E + e] * row_bytes,
                   (const char *)stage + (int64_t)stage_off[u * E + e] * row_bytes,
                   (size_t)((int64_t)n[u * E + e] * row_bytes));
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------- combine */

static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* double -> bf16, one rounding, nearest with ties to even (no detour through
 * float, which would round twice). */
static uint16_t double_to_bf16(double d)
{
    if (isnan(d)) return 0x7FC0;
    uint16_t sign = signbit(d) ? 0x8000 : 0;
    double a = fabs(d);
    if (a == 0.0) return sign;
    if (isinf(a)) return sign | 0x7F80;
    int ex;
    (void)frexp(a, &ex);          /* a = m * 2^ex, m in [0.5, 1) => floor(log2 a) = ex - 1 */
    int e = ex - 1;
    if (e < -126) e = -126;       /* subnormal range: fixed spacing */
    double ulp = ldexp(1.0, e - 7);
    double q = nearbyint(a / ulp); /* default rounding mode: ties to even; division by 2^n is exact */
    double r = q * ulp;            /* exact */
    float f = (float)r;            /* representable, or overflow to inf */
    uint32_t u;
    memcpy(&u, &f, 4);
    return sign | (uint16_t)(u >> 16);
}

/* Section "Expert Parallel", Unpermutation: back in token order every token is the
 * scale-add of its experts' rows with its top-k probabilities:
 *   out[t,:] = sum over kept j (ascending) of gates[t,j] * y[pos_final[t,j], :]
 * A token whose pairs were all dropped yields zeros.  dtype 0 = fp32, 1 = bf16. */
int monta_oracle_combine(int64_t T, int H, int k, int dtype, const void *y,
                         const float *gates, const int32_t *pos_final, void *out)
{
    if (T < 0 || H < 1 || k < 1 || (dtype != 0 && dtype != 1)) return ORACLE_BAD_ARG;
    ORACLE_PARALLEL_FOR
    for (int64_t t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j) {
                int32_t p = pos_final[t * k + j];
                if (p < 0) continue;
                double v = dtype == 0 ? (double)((const float *)y)[(int64_t)p * H + h]
                                      : bf16_to_double(((const uint16_t *)y)[(int64_t)p * H + h]);
                acc += (double)gates[t * k + j] * v;
            }
            if (dtype == 0) ((float *)out)[t * H + h] = (float)acc;
            else ((uint16_t *)out)[t * H + h] = double_to_bf16(acc);
        }
    return ORACLE_OK;
}

/* The gather as a pass of its own (the O2 order of section "Pipelining": AllGather, then the D2D
 * copy): after the gather every TP rank of the group holds the pieces of all tp ranks of the slice
 * side by side, i.e. the slice's whole STAGE range, unchanged, in a second buffer.  The D2D copy
 * (monta_oracle_regather) then runs from that buffer.  slice < 0: all slices. */
int monta_oracle_allgather(int tp, int S, int E, int64_t row_bytes, const int32_t *n,
                           const int32_t *stage_off, const void *stage, void *gathered, int slice)
{
    if (tp < 1 || S < 1 || E < 1 || row_bytes < 1 || slice >= S) return ORACLE_BAD_ARG;
    const int64_t U = (int64_t)S * tp;
    for (int64_t u = 0; u < U; ++u) {
        if (slice >= 0 && u / tp != slice) continue;
        int64_t rows = 0;
        for (int e = 0; e < E; ++e) rows += n[u * E + e];
        memcpy((char *)gathered + (int64_t)stage_off[u * E] * row_bytes,
               (const char *)stage + (int64_t)stage_off[u * E] * row_bytes, (size_t)(rows * row_bytes));
    }
    return ORACLE_OK;
}

/* ------------------------------------------------- the second AllToAll, mirrored */

/* Section "Pipelining" (end of the Drop / AllGather paragraph: the split also applies to the second
 * AllToAll).  After the experts
 * the rows travel back: the expert output y (FINAL layout, expert-major) is cut into the same
 * (unit, expert) blocks and each block returns to its place in the unit-major layout of STAGE --
 * the inverse of the gather + D2D copy -- so that every virtual TP rank again carries only 1/t of a
 * slice.  slice < 0: all slices. */
int monta_oracle_unregather(int tp, int S, int E, int64_t row_bytes, const int32_t *n,
                            const int32_t *stage_off, const int32_t *unit_base, const void *y,
                            void *y_stage, int slice)
{
    if (tp < 1 || S < 1 || E < 1 || row_bytes < 1 || slice >= S) return ORACLE_BAD_ARG;
    const int64_t U = (int64_t)S * tp;
    for (int64_t u = 0; u < U; ++u) {
        if (slice >= 0 && u / tp != slice) continue;
        for (int e = 0; e < E; ++e)
            memcpy((char *)y_stage + (int64_t)stage_off[u * E + e] * row_bytes,
                   (const char *)y + (int64_t)unit_base[u * E + e] * row_bytes,
                   (size_t)((int64_t)n[u * E + e] * row_bytes));
    }
    return ORACLE_OK;
}

/* Unpermutation from the unit-major layout, for the tokens [t0, t1) only (one slice, or all):
 * the same scale-add as monta_oracle_combine, rows addressed through pos_stage. */
int monta_oracle_combine_staged(int64_t t0, int64_t t1, int H, int k, int dtype, const void *y_stage,
                                const float *gates, const int32_t *pos_stage, void *out)
{
    if (t0 < 0 || t1 < t0 || H < 1 || k < 1 || (dtype != 0 && dtype != 1)) return ORACLE_BAD_ARG;
    const int64_t bpe = dtype == 0 ? 4 : 2;
    return monta_oracle_combine(t1 - t0, H, k, dtype, y_stage, gates + t0 * k, pos_stage + t0 * k,
                                (char *)out + t0 * H * bpe);
}

/* ----------------------------------------------------------------- expert */

/* Expert computation (section "Expert Parallel": between Dispatch and Combine every expert processes
 * the tokens that were grouped to it; section "Pipelining": it may start once the D2D copies of the
 * chunks it needs are done).  One linear layer per expert stands in for the expert network: for
 * expert e and every row r in [seg_lo[e], seg_hi[e]) of the expert-major buffer,
 *   y[r][n] = sum_k x_final[r][k] * w[e][n][k],   w [E][N][H] (one row of H inputs per output feature),
 * products exact in double, summed over k ascending in double, rounded once to the activation type.
 * Rows outside every range are left untouched.  If only_rows is not NULL only the listed rows are
 * evaluated (rows outside every range are skipped). */
int monta_oracle_expert(int E, int H, int N, int dtype, const int32_t *seg_lo, const int32_t *seg_hi,
                        const void *x_final, const void *w, void *y, const int32_t *only_rows, int64_t n_only)
{
    if (E < 1 || H < 1 || N < 1 || (dtype != 0 && dtype != 1) || n_only < 0) return ORACLE_BAD_ARG;
    const int64_t count = only_rows ? n_only : -1;
    for (int e = 0; e < E; ++e) {
        const int64_t lo = seg_lo[e], hi = seg_hi[e];
        if (hi < lo || lo < 0) return ORACLE_BAD_ARG;
        const int64_t span = only_rows ? count : hi - lo;
        for (int64_t i = 0; i < span; ++i) {
            const int64_t r = only_rows ? only_rows[i] : lo + i;
            if (r < lo || r >= hi) continue;
            for (int n = 0; n < N; ++n) {
                const int64_t wbase = ((int64_t)e * N + n) * H;
                double acc = 0.0;
                for (int k = 0; k < H; ++k) {
                    double a, b;
                    if (dtype == 0) {
                        a = (double)((const float *)x_final)[r * H + k];
                        b = (double)((const float *)w)[wbase + k];
                    } else {
                        a = bf16_to_double(((const uint16_t *)x_final)[r * H + k]);
                        b = bf16_to_double(((const uint16_t *)w)[wbase + k]);
                    }
                    acc += a * b;
                }
                if (dtype == 0) ((float *)y)[r * N + n] = (float)acc;
                else ((uint16_t *)y)[r * N + n] = double_to_bf16(acc);
            }
        }
    }
    return ORACLE_OK;
}

/* ----------------------------------------------------------------- volume */

/* Byte accounting of the exchange (Eq. 3 traffic I = b*s*h*BPE; Eq. 8-10 per-chunk
 * volumes; Table 8).  unit_bytes[u] is what virtual TP rank u%tp puts on the wire
 * for slice u/tp; dest_bytes[u*ep+d] the part of it addressed to EP rank d;
 * slice_gather_bytes[j] the payload assembled by the gather + D2D copy of slice j. */
int monta_oracle_volume(int tp, int S, int E, int ep, int64_t row_bytes, const int32_t *n,
                        const int32_t *send_rows, int64_t *unit_bytes, int64_t *dest_bytes,
                        int64_t *slice_gather_bytes)
{
    if (tp < 1 || S < 1 || E < 1 || ep < 1 || row_bytes < 1) return ORACLE_BAD_ARG;
    const int64_t U = (int64_t)S * tp;
    for (int j = 0; j < S; ++j) slice_gather_bytes[j] = 0;
    for (int64_t u = 0; u < U; ++u) {
        int64_t rows = 0;
        for (int e = 0; e < E; ++e) rows += n[u * E + e];
        unit_bytes[u] = rows * row_bytes;
        slice_gather_bytes[u / tp] += rows * row_bytes;
        for (int d = 0; d < ep; ++d) dest_bytes[u * ep + d] = (int64_t)send_rows[u * ep + d] * row_bytes;
    }
    return ORACLE_OK;
}
