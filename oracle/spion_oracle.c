/*
 * CPU oracle for the SPION sparse-attention path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, by-the-definition implementation used to check the GPU library: it is called
 * only by the tests, the smoke check and the benchmark's CPU-baseline leg.  It shares no code,
 * headers, tables or helpers with the GPU library and must never be used as a fallback for it.
 *
 * What it follows (SPION: layer-wise sparse training via convolutional flood filling):
 *   - pattern generation: Algorithm 3 (generate_pattern), Eq. 3 (diagonal convolution),
 *     Eq. 4 (average pooling), Algorithm 4 (flood_fill), Section 4.2 (threshold = quantile of
 *     pool_out, diagonal forced to 1, nearest-neighbour upsampling), Section 4.3 (CSR conversion,
 *     kept here at block granularity: BSR and its transpose BSC);
 *   - attention: Eq. 1 (dense attention), Eq. 5 and Algorithm 5 lines 4-7 (SDDMM, sparse softmax,
 *     SpMM), Algorithm 6 (SparseSoftmax; its extra denominator term is available as a flag);
 *     the backward pass is the textbook gradient of Eq. 5 (the paper only states it exists);
 *   - producers of the pattern input: the mean of the heads' score maps (Section 3) and the
 *     Frobenius distance of Eq. 2.
 *
 * Arithmetic: attention in fp64.  Pattern in exact integers: every score is first quantised to
 * fixed point, a_q = rint(a * 2^40), so the sums of Eq. 3 and Eq. 4 are exact and independent of
 * summation order; the decisions of Algorithm 4 (== m, > t) are taken on those integer sums
 * (pool_sum = B^2 * 2^40 * pool_out, a positive rescaling that changes no comparison).
 *
 * Readings where the paper is silent or inconsistent are listed next to each function.
 *
 * Pins: every function here is pinned by the CPU tests against closed forms, library routines,
 * brute force or finite differences.  The paper's own worked flood-fill example exists only as a
 * figure that is not available, so agreement with the authors' output on that example is
 * "parity unpinned"; Algorithm 4's text is pinned by brute-force reachability instead.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG -1
#define ORACLE_ERR_NOMEM -3

#define FIXED_POINT_SCALE 1099511627776.0 /* 2^40 */

/* threshold modes */
#define T_ABS 0
#define T_QUANTILE 1
#define T_MEAN_KSTD 2

/* A threshold is either an exact integer (quantile mode) or a double (the other modes). */
typedef struct {
    int32_t is_int;
    int32_t pad;
    int64_t ti;
    double td;
} oracle_thresh;

int oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------------------------------------
 * Pattern generation
 * ------------------------------------------------------------------------------------------- */

/* Fixed-point quantisation of the score map: a_q = rint(a * 2^40), ties to even.
 * (Reading: the paper does not fix the arithmetic of Eq. 3 / Eq. 4; exact integers make the
 * equality and threshold tests of Algorithm 4 well defined.) */
int oracle_quantize(const float *a, int64_t n, int64_t *aq) {
    if (!a || !aq || n < 0) return ORACLE_ERR_ARG;
    for (int64_t k = 0; k < n; ++k) aq[k] = llrint((double)a[k] * FIXED_POINT_SCALE);
    return ORACLE_OK;
}

/* Eq. 3: conv_out(i,j) = sum over the F taps of the diagonal filter (weight 1 on its main
 * diagonal, 0 elsewhere) of the zero-padded input.  Reading: the filter is centred
 * ("same" padding, p = (F-1)/2, F odd) so that conv_out keeps the L x L size the text states. */
int oracle_conv_diag(const int64_t *aq, int32_t L, int32_t F, int64_t *conv) {
    if (!aq || !conv || L <= 0 || F < 1 || (F % 2) == 0) return ORACLE_ERR_ARG;
    const int32_t p = (F - 1) / 2;
    for (int32_t i = 0; i < L; ++i) {
        for (int32_t j = 0; j < L; ++j) {
            int64_t s = 0;
            for (int32_t f = 0; f < F; ++f) {
                const int32_t y = i + f - p, x = j + f - p;
                if (y >= 0 && y < L && x >= 0 && x < L) s += aq[(int64_t)y * L + x];
            }
            conv[(int64_t)i * L + j] = s;
        }
    }
    return ORACLE_OK;
}

/* Eq. 4 without the 1/B^2 factor: pool_sum(I,J) = sum of conv_out over the non-overlapping
 * B x B block (I,J).  pool_out = pool_sum / (B^2 * 2^40). */
int oracle_pool_sum(const int64_t *conv, int32_t L, int32_t bs, int64_t *pool_sum) {
    if (!conv || !pool_sum || L <= 0 || bs <= 0 || (L % bs) != 0) return ORACLE_ERR_ARG;
    const int32_t nb = L / bs;
    for (int32_t I = 0; I < nb; ++I) {
        for (int32_t J = 0; J < nb; ++J) {
            int64_t s = 0;
            for (int32_t u = 0; u < bs; ++u)
                for (int32_t v = 0; v < bs; ++v) s += conv[(int64_t)(I * bs + u) * L + (J * bs + v)];
            pool_sum[(int64_t)I * nb + J] = s;
        }
    }
    return ORACLE_OK;
}

static int cmp_i64(const void *a, const void *b) {
    const int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

/* Threshold t of Algorithm 4 in pool_sum units (Section 4.2 takes a quantile of the pooled map).
 *   T_QUANTILE  value = q in [0,1]: nearest-rank order statistic without interpolation,
 *               t = sorted[floor(q * (n-1))]; exact integer.
 *   T_MEAN_KSTD value = k: t = mean + k * std (population std); both sums run left to right in
 *               row-major order in fp64 on (double)pool_sum.
 *   T_ABS       value = a threshold on pool_out itself: t = value * B^2 * 2^40 in fp64.
 * An entry counts as above the threshold iff pool_sum > t (integer compare in quantile mode, fp64 otherwise). */
int oracle_threshold(const int64_t *pool_sum, int32_t nb, int32_t bs, int32_t mode, double value,
                     oracle_thresh *t) {
    if (!pool_sum || !t || nb <= 0 || bs <= 0) return ORACLE_ERR_ARG;
    const int64_t n = (int64_t)nb * nb;
    memset(t, 0, sizeof(*t));
    if (mode == T_QUANTILE) {
        if (!(value >= 0.0 && value <= 1.0)) return ORACLE_ERR_ARG;
        int64_t *s = (int64_t *)malloc((size_t)n * sizeof(int64_t));
        if (!s) return ORACLE_ERR_NOMEM;
        memcpy(s, pool_sum, (size_t)n * sizeof(int64_t));
        qsort(s, (size_t)n, sizeof(int64_t), cmp_i64);
        int64_t k = (int64_t)floor(value * (double)(n - 1));
        if (k < 0) k = 0;
        if (k > n - 1) k = n - 1;
        t->is_int = 1;
        t->ti = s[k];
        t->td = (double)s[k];
        free(s);
        return ORACLE_OK;
    }
    if (mode == T_MEAN_KSTD) {
        double sum = 0.0;
        for (int64_t k = 0; k < n; ++k) sum = sum + (double)pool_sum[k];
        const double mean = sum / (double)n;
        double ss = 0.0;
        for (int64_t k = 0; k < n; ++k) {
            const double dlt = (double)pool_sum[k] - mean;
            const double sq = dlt * dlt;
            ss = ss + sq;
        }
        const double var = ss / (double)n;
        const double sd = sqrt(var);
        const double ks = value * sd;
        t->td = mean + ks;
        return ORACLE_OK;
    }
    if (mode == T_ABS) {
        const double cells = (double)bs * (double)bs;
        const double scaled = value * cells;
        t->td = scaled * FIXED_POINT_SCALE;
        return ORACLE_OK;
    }
    return ORACLE_ERR_ARG;
}

static int above(int64_t x, const oracle_thresh *t) {
    return t->is_int ? (x > t->ti) : ((double)x > t->td);
}

/* Algorithm 4 driven the way Algorithm 3 drives it (zeroed fl_out; one walk from every cell of the
 * first row, then one from every cell of the first column; the diagonal forced afterwards),
 * restated as walks over an explicit stack.
 *
 * A walk that stands on cell (r, c) outside the last row and column looks at the cells below, to
 * the right and below-right of it; those equal to the largest of the three are its successors
 * (all of them when values tie).  A successor that is not marked yet is marked if it exceeds t,
 * and the walk continues from it whether it was marked or not; an already marked successor ends
 * that branch, and so does the last row or column.  A seed is not marked by its own walk.
 *
 * Moves never decrease r or c, so by the time a cell is met again everything reachable from it
 * has been visited: walking from it a second time can mark nothing new.  `walked` records the
 * cells a walk has continued from, each is expanded once, and the work is bounded by 3 nb^2
 * steps (re-expanding unmarked cells, as a literal recursion would, is exponential on plateaus
 * of equal sub-threshold values and gives the same fl_out). */
int oracle_fill(const int64_t *pool_sum, int32_t nb, const oracle_thresh *t, int32_t force_diag,
                uint8_t *fl_out) {
    if (!pool_sum || !t || !fl_out || nb <= 0) return ORACLE_ERR_ARG;
    const int64_t n = (int64_t)nb * nb;
    uint8_t *walked = (uint8_t *)calloc((size_t)n, 1);
    int64_t *stack = (int64_t *)malloc((size_t)(n + 2 * (int64_t)nb) * sizeof(int64_t));
    if (!walked || !stack) {
        free(walked);
        free(stack);
        return ORACLE_ERR_NOMEM;
    }
    memset(fl_out, 0, (size_t)n);
    static const int32_t step_r[3] = {1, 0, 1}, step_c[3] = {0, 1, 1}; /* below, right, below-right */
    for (int32_t s = 0; s < 2 * nb; ++s) {
        /* seeds in Algorithm 3's order: (0, 0..nb-1), then (0..nb-1, 0) */
        int64_t top = 0;
        stack[top++] = s < nb ? (int64_t)s : (int64_t)(s - nb) * nb;
        while (top > 0) {
            const int64_t cell = stack[--top];
            const int32_t r = (int32_t)(cell / nb), c = (int32_t)(cell % nb);
            if (r == nb - 1 || c == nb - 1) continue;
            int64_t best = INT64_MIN;
            for (int k = 0; k < 3; ++k) {
                const int64_t v = pool_sum[(int64_t)(r + step_r[k]) * nb + (c + step_c[k])];
                if (v > best) best = v;
            }
            for (int k = 0; k < 3; ++k) {
                const int64_t nxt = (int64_t)(r + step_r[k]) * nb + (c + step_c[k]);
                if (pool_sum[nxt] != best || fl_out[nxt]) continue;
                if (above(pool_sum[nxt], t)) fl_out[nxt] = 1;
                if (!walked[nxt]) {
                    walked[nxt] = 1;
                    stack[top++] = nxt;
                }
            }
        }
    }
    free(walked);
    free(stack);
    if (force_diag)
        for (int32_t k = 0; k < nb; ++k) fl_out[(int64_t)k * nb + k] = 1;
    return ORACLE_OK;
}

/* SPION-C variant (Section 5, "Models Compared"): no flood fill, keep the blocks of pool_out
 * above the threshold, plus the diagonal. */
int oracle_topk(const int64_t *pool_sum, int32_t nb, const oracle_thresh *t, int32_t force_diag,
                uint8_t *fl_out) {
    if (!pool_sum || !t || !fl_out || nb <= 0) return ORACLE_ERR_ARG;
    for (int64_t k = 0; k < (int64_t)nb * nb; ++k) fl_out[k] = above(pool_sum[k], t) ? 1 : 0;
    if (force_diag)
        for (int32_t k = 0; k < nb; ++k) fl_out[(int64_t)k * nb + k] = 1;
    return ORACLE_OK;
}

/* Nearest-neighbour upsampling of fl_out to the L x L pattern matrix P (Algorithm 3, last line). */
int oracle_upsample(const uint8_t *fl_out, int32_t nb, int32_t bs, uint8_t *P) {
    if (!fl_out || !P || nb <= 0 || bs <= 0) return ORACLE_ERR_ARG;
    const int64_t L = (int64_t)nb * bs;
    for (int64_t i = 0; i < L; ++i)
        for (int64_t j = 0; j < L; ++j) P[i * L + j] = fl_out[(i / bs) * nb + (j / bs)];
    return ORACLE_OK;
}

/* Compressed index of the pattern at block granularity (Section 4.3 converts P to CSR; a kept
 * block stands for its B x B entries).  BSR: rows in order, columns ascending.  BSC: columns in
 * order, rows ascending; bsr_pos[k] is the position in col_idx of the k-th BSC entry. */
int oracle_compact(const uint8_t *fl_out, int32_t nb, int32_t *row_ptr, int32_t *col_idx,
                   int32_t *col_ptr, int32_t *row_idx, int32_t *bsr_pos, int32_t *nnzb) {
    if (!fl_out || !row_ptr || !col_idx || !nnzb || nb <= 0) return ORACLE_ERR_ARG;
    int32_t n = 0;
    for (int32_t I = 0; I < nb; ++I) {
        row_ptr[I] = n;
        for (int32_t J = 0; J < nb; ++J)
            if (fl_out[(int64_t)I * nb + J]) col_idx[n++] = J;
    }
    row_ptr[nb] = n;
    *nnzb = n;
    if (col_ptr && row_idx && bsr_pos) {
        int32_t m = 0;
        for (int32_t J = 0; J < nb; ++J) {
            col_ptr[J] = m;
            for (int32_t I = 0; I < nb; ++I) {
                if (!fl_out[(int64_t)I * nb + J]) continue;
                int32_t pos = -1;
                for (int32_t k = row_ptr[I]; k < row_ptr[I + 1]; ++k)
                    if (col_idx[k] == J) pos = k;
                row_idx[m] = I;
                bsr_pos[m] = pos;
                ++m;
            }
        }
        col_ptr[nb] = m;
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Producers of the pattern input
 * ------------------------------------------------------------------------------------------- */

/* Section 3: the score maps of the heads of a layer are averaged (element-wise mean, fp64). */
int oracle_score_mean(const double *maps, int32_t n_maps, int64_t n, double *out) {
    if (!maps || !out || n_maps <= 0 || n <= 0) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int32_t m = 0; m < n_maps; ++m) s += maps[(int64_t)m * n + i];
        out[i] = s / (double)n_maps;
    }
    return ORACLE_OK;
}

/* Eq. 2: distance = | sqrt(sum a^2) - sqrt(sum b^2) |; out = {distance, ||a||_F, ||b||_F}. */
int oracle_frobenius_distance(const double *a, const double *b, int64_t n, double *out) {
    if (!a || !b || !out || n <= 0) return ORACLE_ERR_ARG;
    double sa = 0.0, sb = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        sa += a[i] * a[i];
        sb += b[i] * b[i];
    }
    out[1] = sqrt(sa);
    out[2] = sqrt(sb);
    out[0] = fabs(out[1] - out[2]);
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Attention (fp64).  Tensors are [BH, L, d] row-major; P is the L x L 0/1 pattern shared by all
 * batch items and heads (Section 4.3).
 *
 * Forward, per head (Eq. 5 / Algorithm 5 lines 5-7), default reading:
 *     s_ij = scale * <q_i, k_j> where P_ij > 0, -inf elsewhere
 *     p_ij = exp(s_ij - m_i) / sum_j exp(s_ij - m_i),  m_i = max_j s_ij      (kept entries only)
 *     o_i  = sum_j p_ij v_j,   lse_i = m_i + log(sum_j exp(s_ij - m_i))
 * With flag ORACLE_ATTN_PAPER_DENOM the denominator is the one Algorithm 6 prints:
 *     sum_j(kept) exp(s_ij - m_i) + exp(-m_i) * (L - kept_i)
 * (every masked entry counted as a score of 0); the two coincide for an all-ones pattern.
 * A row with no kept entry yields o_i = 0 and lse_i = -inf.
 * ------------------------------------------------------------------------------------------- */
#define ORACLE_ATTN_PAPER_DENOM 1

/* Softmax probabilities of row i of one head into p[L]; returns lse. */
static double prob_row(const double *Q, const double *K, const uint8_t *P, int32_t L, int32_t d,
                       double scale, int32_t flags, int32_t i, double *p) {
    const uint8_t *Pi = P + (int64_t)i * L;
    const double *qi = Q + (int64_t)i * d;
    double m = -INFINITY;
    int32_t kept = 0;
    for (int32_t j = 0; j < L; ++j) {
        const double *kj = K + (int64_t)j * d;
        double dot = 0.0;
        for (int32_t c = 0; c < d; ++c) dot += qi[c] * kj[c];
        const double s = Pi[j] ? scale * dot : -INFINITY;
        p[j] = s;
        if (Pi[j]) ++kept;
        if (s > m) m = s;
    }
    if (kept == 0) {
        for (int32_t j = 0; j < L; ++j) p[j] = 0.0;
        return -INFINITY;
    }
    double sum = 0.0;
    for (int32_t j = 0; j < L; ++j) {
        p[j] = exp(p[j] - m); /* exp(-inf) == 0 for masked entries */
        sum += p[j];
    }
    if (flags & ORACLE_ATTN_PAPER_DENOM) sum += exp(-m) * (double)(L - kept);
    for (int32_t j = 0; j < L; ++j) p[j] /= sum;
    return m + log(sum);
}

int oracle_attn_fwd(const double *Q, const double *K, const double *V, const uint8_t *P,
                    int32_t BH, int32_t L, int32_t d, double scale, int32_t flags, double *O,
                    double *LSE) {
    if (!Q || !K || !V || !P || !O || BH <= 0 || L <= 0 || d <= 0) return ORACLE_ERR_ARG;
    int err = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t bh = 0; bh < BH; ++bh) {
        const int64_t off = (int64_t)bh * L * d;
        double *p = (double *)malloc((size_t)L * sizeof(double));
        if (!p) {
            err = ORACLE_ERR_NOMEM;
            continue;
        }
        for (int32_t i = 0; i < L; ++i) {
            const double lse = prob_row(Q + off, K + off, P, L, d, scale, flags, i, p);
            if (LSE) LSE[(int64_t)bh * L + i] = lse;
            double *oi = O + off + (int64_t)i * d;
            for (int32_t c = 0; c < d; ++c) oi[c] = 0.0;
            for (int32_t j = 0; j < L; ++j) {
                const double *vj = V + off + (int64_t)j * d;
                for (int32_t c = 0; c < d; ++c) oi[c] += p[j] * vj[c];
            }
        }
        free(p);
    }
    return err;
}

/* Backward of the forward above (gradient of Eq. 5 w.r.t. Q, K, V given dO):
 *     dV = p^T dO;  dP = dO V^T;  delta_i = sum_j p_ij dP_ij;  dS = p .* (dP - delta)
 *     dQ = scale * dS K;  dK = scale * dS^T Q.
 * Masked entries have p_ij = 0 and so dS_ij = 0.  The same formula holds for the
 * ORACLE_ATTN_PAPER_DENOM variant (the extra denominator term is a constant score). */
int oracle_attn_bwd(const double *Q, const double *K, const double *V, const double *dO,
                    const uint8_t *P, int32_t BH, int32_t L, int32_t d, double scale,
                    int32_t flags, double *dQ, double *dK, double *dV) {
    if (!Q || !K || !V || !dO || !P || !dQ || !dK || !dV || BH <= 0 || L <= 0 || d <= 0)
        return ORACLE_ERR_ARG;
    int err = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t bh = 0; bh < BH; ++bh) {
        const int64_t off = (int64_t)bh * L * d;
        double *p = (double *)malloc((size_t)L * sizeof(double));
        double *ds = (double *)malloc((size_t)L * sizeof(double));
        if (!p || !ds) {
            err = ORACLE_ERR_NOMEM;
            free(p);
            free(ds);
            continue;
        }
        for (int64_t k = 0; k < (int64_t)L * d; ++k) {
            dQ[off + k] = 0.0;
            dK[off + k] = 0.0;
            dV[off + k] = 0.0;
        }
        for (int32_t i = 0; i < L; ++i) {
            prob_row(Q + off, K + off, P, L, d, scale, flags, i, p);
            const double *doi = dO + off + (int64_t)i * d;
            const double *qi = Q + off + (int64_t)i * d;
            double delta = 0.0;
            for (int32_t j = 0; j < L; ++j) {
                const double *vj = V + off + (int64_t)j * d;
                double dp = 0.0;
                for (int32_t c = 0; c < d; ++c) dp += doi[c] * vj[c];
                ds[j] = dp; /* dP_ij for now */
                delta += p[j] * dp;
            }
            for (int32_t j = 0; j < L; ++j) ds[j] = p[j] * (ds[j] - delta);
            double *dqi = dQ + off + (int64_t)i * d;
            for (int32_t j = 0; j < L; ++j) {
                const double *kj = K + off + (int64_t)j * d;
                double *dkj = dK + off + (int64_t)j * d;
                double *dvj = dV + off + (int64_t)j * d;
                for (int32_t c = 0; c < d; ++c) {
                    dqi[c] += scale * ds[j] * kj[c];
                    dkj[c] += scale * ds[j] * qi[c];
                    dvj[c] += p[j] * doi[c];
                }
            }
        }
        free(p);
        free(ds);
    }
    return err;
}

/* Row i of the probability matrix of head bh (for tests that look at p itself). */
int oracle_attn_probs_row(const double *Q, const double *K, const uint8_t *P, int32_t L, int32_t d,
                          double scale, int32_t flags, int32_t bh, int32_t i, double *p) {
    if (!Q || !K || !P || !p || i < 0 || i >= L) return ORACLE_ERR_ARG;
    const int64_t off = (int64_t)bh * L * d;
    prob_row(Q + off, K + off, P, L, d, scale, flags, i, p);
    return ORACLE_OK;
}
