/*
 * otf_oracle.c -- plain CPU oracle for the ranking hot path of "Efficient On-the-fly
 * Category Retrieval using ConvNets and GPUs" (arXiv 1407.4764).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or import this
 * file; it exists so that the HIP kernels have an independent definition to be compared
 * with.  It shares no code, header, table or helper with the HIP path.
 *
 * Every function is the textbook definition written out as scalar loops in double
 * precision.  The only parallelism is an OpenMP "parallel for" over independent dataset
 * rows; there is no blocking, no vectorisation by hand, no reordering of the sums (the
 * inner index always ascends).
 *
 * What each function follows in the paper:
 *   orc_dense_*        Sec. 3.2 "Implementation Details" (the linear predictor <w, phi(I)>)
 *                      and Sec. 4 "On-line (GPU back-end)", Ranking: every dataset feature
 *                      is scored with the current model.
 *   orc_pq_*           Sec. 3, paragraph "Product quantization (PQ)": the feature is split
 *                      into sub-blocks, each encoded with its own vocabulary of centres;
 *                      Table 2 gives one byte per sub-block.  The paper does not say how
 *                      coded features are scored; the reading taken is the score of the
 *                      centre-reconstructed vector (w itself is never quantised).
 *   orc_binary_scores  Sec. 3, paragraph "Binarization", Eq. (1) (codes in {0,1}^n), ranked
 *                      by a linear SVM (Sec. 3.1, discussion after Table 2).  A bit b
 *                      enters the model as 2b-1.
 *   orc_hamming_scores Sec. 3.1, discussion after Table 2: ranking binary codes by Hamming
 *                      distance, which the paper names as the way to speed their ranking up
 *                      and leaves for later.  The ranking model it needs in place of the linear
 *                      SVM is taken to be a query code; a row's score is minus its distance to it.
 *   orc_sparse_expand  Sec. 3.1, same discussion: ConvNet features are very sparse (the 128-D
 *                      ones over 60 % zeros), a compression the paper points at but does not
 *                      build.  The store keeps a presence mask and the non-zero values of a
 *                      row; expanding it gives back the dense row, which orc_dense_f32 scores.
 *   orc_topk           Sec. 4, Ranking: the scores are sorted and the head of the list goes
 *                      to the front-end.
 *   orc_sgd_step       Sec. 4, Training: mini-batch SGD with Pegasos updates, learning rate
 *                      1/(lambda t), batches of half positives and half negatives.
 *
 * Parity pins (tests/test_oracle_pins.py) tie each function to something outside this file:
 * numpy fp64 matmul, brute-force python loops, closed forms of the Pegasos update, and the
 * storage arithmetic of the paper's Table 2.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_BAD_ARG (-1)
#define ORC_NO_MEM (-2)
#define ORC_NOT_FINITE (-3)

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* IEEE binary16 -> double, exact (every half is representable). */
double orc_half_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);              /* zero and subnormals: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

/* ---------------------------------------------------------------- dense scoring
 * s[q][i] = bias[q] + sum_{d=0}^{D-1} W[q][d] * X[i][d],  d ascending, all in double.
 * X is N x D row-major with leading dimension ldx (elements); W is Q x D, contiguous.
 * bias may be NULL (all zero).  out is Q x N doubles.
 */
int orc_dense_f32(const float *X, int64_t N, int32_t D, int64_t ldx,
                  const float *W, int32_t Q, const float *bias, double *out) {
    if (!X || !W || !out || N < 0 || D < 1 || Q < 1 || ldx < D) return ORC_BAD_ARG;
    for (int32_t q = 0; q < Q; ++q) {
        const float *w = W + (int64_t)q * D;
        double b = bias ? (double)bias[q] : 0.0;
        double *s = out + (int64_t)q * N;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            const float *x = X + i * ldx;
            double acc = b;
            for (int32_t d = 0; d < D; ++d) acc += (double)w[d] * (double)x[d];
            s[i] = acc;
        }
    }
    return ORC_OK;
}

/* Same with X and W stored as IEEE half (raw 16-bit patterns); the stored values are
 * widened exactly, so the oracle sees the very numbers the GPU reads. */
int orc_dense_f16(const uint16_t *X, int64_t N, int32_t D, int64_t ldx,
                  const uint16_t *W, int32_t Q, const float *bias, double *out) {
    if (!X || !W || !out || N < 0 || D < 1 || Q < 1 || ldx < D) return ORC_BAD_ARG;
    double *wd = (double *)malloc(sizeof(double) * (size_t)D);
    if (!wd) return ORC_NO_MEM;
    for (int32_t q = 0; q < Q; ++q) {
        for (int32_t d = 0; d < D; ++d) wd[d] = orc_half_to_double(W[(int64_t)q * D + d]);
        double b = bias ? (double)bias[q] : 0.0;
        double *s = out + (int64_t)q * N;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            const uint16_t *x = X + i * ldx;
            double acc = b;
            for (int32_t d = 0; d < D; ++d) acc += wd[d] * orc_half_to_double(x[d]);
            s[i] = acc;
        }
    }
    free(wd);
    return ORC_OK;
}

/* Half-precision dataset, single-precision model (the single-query fp16 store). */
int orc_dense_f16x_f32w(const uint16_t *X, int64_t N, int32_t D, int64_t ldx,
                        const float *W, int32_t Q, const float *bias, double *out) {
    if (!X || !W || !out || N < 0 || D < 1 || Q < 1 || ldx < D) return ORC_BAD_ARG;
    for (int32_t q = 0; q < Q; ++q) {
        const float *w = W + (int64_t)q * D;
        double b = bias ? (double)bias[q] : 0.0;
        double *s = out + (int64_t)q * N;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            const uint16_t *x = X + i * ldx;
            double acc = b;
            for (int32_t d = 0; d < D; ++d) acc += (double)w[d] * orc_half_to_double(x[d]);
            s[i] = acc;
        }
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------- product quantisation
 * Store: codes[i][m] in [0,K) selects centre C[m][code][0..dsub) for sub-block m.
 * Reconstruction: xhat_i[m*dsub + j] = C[m][codes[i][m]][j].
 */

/* Score by explicit reconstruction: build xhat_i, then the dense definition on it. */
int orc_pq_scores_reconstruct(const uint8_t *codes, int64_t N, int32_t M, int32_t K,
                              int32_t dsub, const float *codebooks, const float *w,
                              double bias, double *out) {
    if (!codes || !codebooks || !w || !out || N < 0 || M < 1 || K < 1 || K > 256 || dsub < 1)
        return ORC_BAD_ARG;
    const int32_t D = M * dsub;
    int bad = 0;
#pragma omp parallel
    {
        float *xhat = (float *)malloc(sizeof(float) * (size_t)D);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            if (!xhat) { bad = 1; continue; }
            int row_ok = 1;
            for (int32_t m = 0; m < M; ++m) {
                int32_t c = codes[i * M + m];
                if (c >= K) { row_ok = 0; break; }
                const float *centre = codebooks + ((int64_t)m * K + c) * dsub;
                for (int32_t j = 0; j < dsub; ++j) xhat[m * dsub + j] = centre[j];
            }
            if (!row_ok) { bad = 2; out[i] = NAN; continue; }
            double acc = bias;
            for (int32_t d = 0; d < D; ++d) acc += (double)w[d] * (double)xhat[d];
            out[i] = acc;
        }
        free(xhat);
    }
    if (bad == 1) return ORC_NO_MEM;
    if (bad == 2) return ORC_BAD_ARG;
    return ORC_OK;
}

/* lut[m][k] = sum_{j<dsub} w[m*dsub+j] * C[m][k][j], in double. */
int orc_pq_lut(const float *codebooks, int32_t M, int32_t K, int32_t dsub,
               const float *w, double *lut) {
    if (!codebooks || !w || !lut || M < 1 || K < 1 || dsub < 1) return ORC_BAD_ARG;
    for (int32_t m = 0; m < M; ++m)
        for (int32_t k = 0; k < K; ++k) {
            const float *centre = codebooks + ((int64_t)m * K + k) * dsub;
            double acc = 0.0;
            for (int32_t j = 0; j < dsub; ++j) acc += (double)w[m * dsub + j] * (double)centre[j];
            lut[(int64_t)m * K + k] = acc;
        }
    return ORC_OK;
}

/* Score by table sums: s_i = bias + sum_m lut[m][codes[i][m]].  Must agree with
 * orc_pq_scores_reconstruct up to the rounding order of a double sum. */
int orc_pq_scores_lut(const uint8_t *codes, int64_t N, int32_t M, int32_t K,
                      const double *lut, double bias, double *out) {
    if (!codes || !lut || !out || N < 0 || M < 1 || K < 1 || K > 256) return ORC_BAD_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        double acc = bias;
        for (int32_t m = 0; m < M; ++m) {
            int32_t c = codes[i * M + m];
            if (c >= K) { bad = 1; c = 0; }
            acc += lut[(int64_t)m * K + c];
        }
        out[i] = acc;
    }
    return bad ? ORC_BAD_ARG : ORC_OK;
}

/* ---------------------------------------------------------------- binary codes
 * Dimension d of row i is bit (d mod 32), least significant first, of word (d div 32);
 * rows are ld_words words apart.  A bit b contributes w_d * (2b - 1).
 */
int orc_binary_scores(const uint32_t *bits, int64_t N, int32_t D, int64_t ld_words,
                      const float *w, double bias, double *out) {
    if (!bits || !w || !out || N < 0 || D < 1 || ld_words * 32 < D) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        const uint32_t *row = bits + i * ld_words;
        double acc = bias;
        for (int32_t d = 0; d < D; ++d) {
            uint32_t bit = (row[d >> 5] >> (d & 31)) & 1u;
            acc += bit ? (double)w[d] : -(double)w[d];
        }
        out[i] = acc;
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------- Hamming ranking
 * score[i] = -(number of dimensions d < D in which row i and the query differ), bit by bit.
 * Same bit layout as orc_binary_scores.  The larger (less negative) score is the nearer row.
 */
int orc_hamming_scores(const uint32_t *bits, int64_t N, int32_t D, int64_t ld_words,
                       const uint32_t *query, double *out) {
    if (!bits || !query || !out || N < 0 || D < 1 || ld_words * 32 < D) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        const uint32_t *row = bits + i * ld_words;
        int64_t differ = 0;
        for (int32_t d = 0; d < D; ++d) {
            uint32_t a = (row[d >> 5] >> (d & 31)) & 1u;
            uint32_t b = (query[d >> 5] >> (d & 31)) & 1u;
            if (a != b) ++differ;
        }
        out[i] = -(double)differ;
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------- sparse rows
 * A sparse row i of D dimensions is stored as a presence mask of D bits (dimension d = bit
 * d mod 32, least significant first, of word d div 32 of mask row i; rows ld_mask words apart)
 * and its non-zero values in ascending order of dimension, values[start[i]] onwards.
 * Expands N rows into the dense N x D matrix X (row-major, contiguous): a dimension whose mask
 * bit is clear is 0, the others take the stored values in order.  start has N + 1 entries
 * (start[N] = total number of stored values); it is checked against the masks.
 */
int orc_sparse_expand(const uint32_t *mask, int64_t ld_mask, const float *values, const int64_t *start,
                      int64_t N, int32_t D, float *X) {
    if (!mask || !values || !start || !X || N < 0 || D < 1 || ld_mask * 32 < D) return ORC_BAD_ARG;
    for (int64_t i = 0; i < N; ++i) {
        const uint32_t *mrow = mask + i * ld_mask;
        int64_t next = start[i];
        for (int32_t d = 0; d < D; ++d) {
            if ((mrow[d >> 5] >> (d & 31)) & 1u) X[i * D + d] = values[next++];
            else X[i * D + d] = 0.0f;
        }
        if (next != start[i + 1]) return ORC_BAD_ARG;   /* offsets and masks disagree */
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------- ranking
 * Full sort of all N (score, index) pairs, score descending, equal scores by ascending
 * index; the first k are returned.  Scores must be finite.
 */
typedef struct { double s; int64_t i; } orc_pair;

static int orc_pair_cmp(const void *pa, const void *pb) {
    const orc_pair *a = (const orc_pair *)pa, *b = (const orc_pair *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    if (a->i < b->i) return -1;
    if (a->i > b->i) return 1;
    return 0;
}

int orc_topk(const double *scores, int64_t N, int64_t k, int64_t *out_idx, double *out_scores) {
    if (!scores || !out_idx || !out_scores || N < 1 || k < 1 || k > N) return ORC_BAD_ARG;
    orc_pair *p = (orc_pair *)malloc(sizeof(orc_pair) * (size_t)N);
    if (!p) return ORC_NO_MEM;
    for (int64_t i = 0; i < N; ++i) {
        if (!isfinite(scores[i])) { free(p); return ORC_NOT_FINITE; }
        p[i].s = scores[i];
        p[i].i = i;
    }
    qsort(p, (size_t)N, sizeof(orc_pair), orc_pair_cmp);
    for (int64_t j = 0; j < k; ++j) { out_idx[j] = p[j].i; out_scores[j] = p[j].s; }
    free(p);
    return ORC_OK;
}

/* ---------------------------------------------------------------- Pegasos mini-batch step
 * Batch = the n_pos rows Xpos[idx_pos[.]] with label +1 followed by the n_neg rows
 * Xneg[idx_neg[.]] with label -1;  B = n_pos + n_neg.
 *   eta      = 1 / (lambda t)
 *   m_j      = y_j (<w_t, x_j> + b_t)              margins under the model BEFORE the step
 *   V        = { j : m_j < 1 }                     strict: no sub-gradient at the kink
 *   w_{t+1}  = (1 - eta lambda) w_t + (eta / B) sum_{j in V} y_j x_j
 *   b_{t+1}  = b_t + (eta / B) sum_{j in V} y_j    only if update_bias, else b_t
 * No projection step.  margins_out (B doubles, may be NULL) receives m_j.
 */
int orc_sgd_step(const float *w_in, double b_in, int32_t D,
                 const float *Xpos, int64_t ld_pos, const int32_t *idx_pos, int32_t n_pos,
                 const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int32_t n_neg,
                 double lambda, int64_t t, int32_t update_bias,
                 double *w_out, double *b_out, double *margins_out) {
    if (!w_in || !w_out || !b_out || D < 1 || n_pos < 0 || n_neg < 0 || n_pos + n_neg < 1 ||
        (n_pos > 0 && (!Xpos || !idx_pos)) || (n_neg > 0 && (!Xneg || !idx_neg)) ||
        !(lambda > 0.0) || t < 1)
        return ORC_BAD_ARG;
    const int32_t B = n_pos + n_neg;
    const double eta = 1.0 / (lambda * (double)t);
    double *grad = (double *)calloc((size_t)D, sizeof(double));
    if (!grad) return ORC_NO_MEM;
    double ysum = 0.0;
    for (int32_t j = 0; j < B; ++j) {
        const float *x;
        double y;
        if (j < n_pos) { x = Xpos + (int64_t)idx_pos[j] * ld_pos; y = 1.0; }
        else           { x = Xneg + (int64_t)idx_neg[j - n_pos] * ld_neg; y = -1.0; }
        double dot = b_in;
        for (int32_t d = 0; d < D; ++d) dot += (double)w_in[d] * (double)x[d];
        double margin = y * dot;
        if (margins_out) margins_out[j] = margin;
        if (margin < 1.0) {
            for (int32_t d = 0; d < D; ++d) grad[d] += y * (double)x[d];
            ysum += y;
        }
    }
    const double shrink = 1.0 - eta * lambda;
    for (int32_t d = 0; d < D; ++d) w_out[d] = shrink * (double)w_in[d] + (eta / (double)B) * grad[d];
    *b_out = update_bias ? b_in + (eta / (double)B) * ysum : b_in;
    free(grad);
    return ORC_OK;
}

/* Regularised hinge objective over two pools:
 *   lambda/2 |w|^2 + mean_j max(0, 1 - y_j (<w,x_j> + b)),  j over all pool rows. */
int orc_svm_objective(const double *w, double b, int32_t D,
                      const float *Xpos, int64_t ld_pos, int64_t n_pos,
                      const float *Xneg, int64_t ld_neg, int64_t n_neg,
                      double lambda, double *out) {
    if (!w || !out || D < 1 || n_pos < 0 || n_neg < 0 || n_pos + n_neg < 1) return ORC_BAD_ARG;
    double reg = 0.0;
    for (int32_t d = 0; d < D; ++d) reg += w[d] * w[d];
    double hinge = 0.0;
    for (int64_t j = 0; j < n_pos + n_neg; ++j) {
        const float *x = j < n_pos ? Xpos + j * ld_pos : Xneg + (j - n_pos) * ld_neg;
        double y = j < n_pos ? 1.0 : -1.0;
        double dot = b;
        for (int32_t d = 0; d < D; ++d) dot += w[d] * (double)x[d];
        double loss = 1.0 - y * dot;
        if (loss > 0.0) hinge += loss;
    }
    *out = 0.5 * lambda * reg + hinge / (double)(n_pos + n_neg);
    return ORC_OK;
}
