/*
 * Runs every function of oracle/otf_oracle.c on small inputs whose buffers are exactly as large as
 * the functions are entitled to touch (heap allocations, so that AddressSanitizer sees one byte
 * too many), over ragged sizes and padded rows, and prints a checksum per call.  Built twice by
 * tests/test_sanitizers.py: with -fsanitize=address,undefined and without; both must print the
 * same lines and the sanitized run must end without a report.  TEST INFRASTRUCTURE ONLY.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int orc_num_threads(void);
double orc_half_to_double(uint16_t h);
int orc_dense_f32(const float *X, int64_t N, int32_t D, int64_t ldx, const float *W, int32_t Q, const float *bias, double *out);
int orc_dense_f16(const uint16_t *X, int64_t N, int32_t D, int64_t ldx, const uint16_t *W, int32_t Q, const float *bias, double *out);
int orc_dense_f16x_f32w(const uint16_t *X, int64_t N, int32_t D, int64_t ldx, const float *W, int32_t Q, const float *bias, double *out);
int orc_pq_scores_reconstruct(const uint8_t *codes, int64_t N, int32_t M, int32_t K, int32_t dsub, const float *codebooks,
                              const float *w, double bias, double *out);
int orc_pq_lut(const float *codebooks, int32_t M, int32_t K, int32_t dsub, const float *w, double *lut);
int orc_pq_scores_lut(const uint8_t *codes, int64_t N, int32_t M, int32_t K, const double *lut, double bias, double *out);
int orc_binary_scores(const uint32_t *bits, int64_t N, int32_t D, int64_t ld_words, const float *w, double bias, double *out);
int orc_hamming_scores(const uint32_t *bits, int64_t N, int32_t D, int64_t ld_words, const uint32_t *query, double *out);
int orc_sparse_expand(const uint32_t *mask, int64_t ld_mask, const float *values, const int64_t *start, int64_t N, int32_t D, float *X);
int orc_topk(const double *scores, int64_t N, int64_t k, int64_t *out_idx, double *out_scores);
int orc_sgd_step(const float *w_in, double b_in, int32_t D, const float *Xpos, int64_t ld_pos, const int32_t *idx_pos,
                 int32_t n_pos, const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int32_t n_neg, double lambda,
                 int64_t t, int32_t update_bias, double *w_out, double *b_out, double *margins_out);
int orc_svm_objective(const double *w, double b, int32_t D, const float *Xpos, int64_t ld_pos, int64_t n_pos,
                      const float *Xneg, int64_t ld_neg, int64_t n_neg, double lambda, double *out);

static uint32_t state = 20140717u;
static uint32_t next_u32(void) {
    state = state * 1664525u + 1013904223u;
    return state >> 8;
}
static float next_float(void) { return (float)((int)(next_u32() & 0xffff) - 32768) / 4096.0f; }

static void *must(size_t bytes) {
    void *p = malloc(bytes ? bytes : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    return p;
}
static float *floats(size_t n) {
    float *p = (float *)must(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = next_float();
    return p;
}
/* half-precision patterns of finite values only (exponent field below 31) */
static uint16_t *halves(size_t n) {
    uint16_t *p = (uint16_t *)must(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) {
        uint16_t h = (uint16_t)next_u32();
        if (((h >> 10) & 0x1f) == 0x1f) h &= (uint16_t)~(1u << 14);
        p[i] = h;
    }
    return p;
}
static double checksum(const double *v, size_t n) {
    double s = 0.0;
    for (size_t i = 0; i < n; ++i) s += v[i] * (double)(1 + (i % 7));
    return s;
}
static void report(const char *what, int64_t a, int64_t b, int64_t c, int rc, double sum) {
    printf("%-24s %6lld %5lld %5lld rc=%d sum=%.17g\n", what, (long long)a, (long long)b, (long long)c, rc, sum);
}

static void dense_cases(void) {
    const int64_t Ns[] = {1, 7, 130};
    const int32_t Ds[] = {4, 36, 128};
    for (int a = 0; a < 3; ++a)
        for (int b = 0; b < 3; ++b)
            for (int32_t Q = 1; Q <= 3; Q += 2)
                for (int pad = 0; pad <= 8; pad += 8) {
                    const int64_t N = Ns[a], ldx = Ds[b] + pad;
                    const int32_t D = Ds[b];
                    /* the last row ends at its D-th element: no padding behind it */
                    float *X = floats((size_t)((N - 1) * ldx + D)), *W = floats((size_t)Q * D), *bias = floats((size_t)Q);
                    uint16_t *Xh = halves((size_t)((N - 1) * ldx + D)), *Wh = halves((size_t)Q * D);
                    double *out = (double *)must(sizeof(double) * (size_t)(Q * N));
                    int rc = orc_dense_f32(X, N, D, ldx, W, Q, pad ? bias : NULL, out);
                    report("dense_f32", N, D, Q, rc, checksum(out, (size_t)(Q * N)));
                    rc = orc_dense_f16(Xh, N, D, ldx, Wh, Q, bias, out);
                    report("dense_f16", N, D, Q, rc, checksum(out, (size_t)(Q * N)));
                    rc = orc_dense_f16x_f32w(Xh, N, D, ldx, W, Q, NULL, out);
                    report("dense_f16x_f32w", N, D, Q, rc, checksum(out, (size_t)(Q * N)));
                    free(X); free(W); free(bias); free(Xh); free(Wh); free(out);
                }
}

static void pq_cases(void) {
    const int32_t Ms[] = {1, 4, 16}, dsubs[] = {1, 4, 16}, Ks[] = {2, 256};
    for (int a = 0; a < 3; ++a)
        for (int b = 0; b < 3; ++b)
            for (int c = 0; c < 2; ++c) {
                const int32_t M = Ms[a], dsub = dsubs[b], K = Ks[c];
                const int64_t N = 33;
                uint8_t *codes = (uint8_t *)must((size_t)(N * M));
                for (int64_t i = 0; i < N * M; ++i) codes[i] = (uint8_t)(next_u32() % (uint32_t)K);
                codes[0] = (uint8_t)(K - 1);                       /* the last centre of the vocabulary */
                float *cb = floats((size_t)M * K * dsub), *w = floats((size_t)M * dsub);
                double *lut = (double *)must(sizeof(double) * (size_t)(M * K)), *out = (double *)must(sizeof(double) * (size_t)N);
                int rc = orc_pq_scores_reconstruct(codes, N, M, K, dsub, cb, w, 0.25, out);
                report("pq_reconstruct", M, dsub, K, rc, checksum(out, (size_t)N));
                rc = orc_pq_lut(cb, M, K, dsub, w, lut);
                report("pq_lut", M, dsub, K, rc, checksum(lut, (size_t)(M * K)));
                rc = orc_pq_scores_lut(codes, N, M, K, lut, 0.25, out);
                report("pq_scores_lut", M, dsub, K, rc, checksum(out, (size_t)N));
                if (K < 256) {                                     /* a code beyond the vocabulary is an error, not a read */
                    codes[N * M - 1] = (uint8_t)K;
                    report("pq_bad_code", M, dsub, K, orc_pq_scores_lut(codes, N, M, K, lut, 0.0, out), 0.0);
                    report("pq_bad_code_rec", M, dsub, K, orc_pq_scores_reconstruct(codes, N, M, K, dsub, cb, w, 0.0, out), 0.0);
                }
                free(codes); free(cb); free(w); free(lut); free(out);
            }
}

static void bit_cases(void) {
    const int32_t Ds[] = {1, 31, 32, 33, 128, 2048};
    for (int a = 0; a < 6; ++a)
        for (int pad = 0; pad <= 3; pad += 3) {
            const int32_t D = Ds[a];
            const int64_t N = 19, words = (D + 31) / 32, ld = words + pad;
            uint32_t *bits = (uint32_t *)must(sizeof(uint32_t) * (size_t)((N - 1) * ld + words));
            for (int64_t i = 0; i < (N - 1) * ld + words; ++i) bits[i] = next_u32() * 2654435761u;
            uint32_t *query = (uint32_t *)must(sizeof(uint32_t) * (size_t)words);
            for (int64_t i = 0; i < words; ++i) query[i] = next_u32() * 2246822519u;
            float *w = floats((size_t)D);
            double *out = (double *)must(sizeof(double) * (size_t)N);
            int rc = orc_binary_scores(bits, N, D, ld, w, -1.5, out);
            report("binary_scores", N, D, ld, rc, checksum(out, (size_t)N));
            rc = orc_hamming_scores(bits, N, D, ld, query, out);
            report("hamming_scores", N, D, ld, rc, checksum(out, (size_t)N));
            free(bits); free(query); free(w); free(out);
        }
}

static void sparse_cases(void) {
    const int32_t Ds[] = {5, 32, 128};
    for (int a = 0; a < 3; ++a) {
        const int32_t D = Ds[a];
        const int64_t N = 23, ld = (D + 31) / 32;
        uint32_t *mask = (uint32_t *)must(sizeof(uint32_t) * (size_t)(N * ld));
        int64_t *start = (int64_t *)must(sizeof(int64_t) * (size_t)(N + 1));
        int64_t total = 0;
        for (int64_t i = 0; i < N; ++i) {
            start[i] = total;
            for (int64_t j = 0; j < ld; ++j) mask[i * ld + j] = 0u;
            for (int32_t d = 0; d < D; ++d)
                if (i != 3 && (next_u32() % 5u) < 2u) {            /* row 3 stays empty */
                    mask[i * ld + (d >> 5)] |= 1u << (d & 31);
                    ++total;
                }
        }
        start[N] = total;
        float *values = floats((size_t)total), *X = (float *)must(sizeof(float) * (size_t)(N * D));
        double *as_double = (double *)must(sizeof(double) * (size_t)(N * D));
        int rc = orc_sparse_expand(mask, ld, values, start, N, D, X);
        for (int64_t i = 0; i < N * D; ++i) as_double[i] = (double)X[i];
        report("sparse_expand", N, D, total, rc, checksum(as_double, (size_t)(N * D)));
        start[N] = total + 1;                                      /* offsets that disagree with the masks */
        report("sparse_bad_offsets", N, D, total, orc_sparse_expand(mask, ld, values, start, N, D, X), 0.0);
        free(mask); free(start); free(values); free(X); free(as_double);
    }
}

static void topk_cases(void) {
    const int64_t Ns[] = {1, 2, 100, 1000};
    for (int a = 0; a < 4; ++a) {
        const int64_t N = Ns[a];
        double *s = (double *)must(sizeof(double) * (size_t)N);
        for (int64_t i = 0; i < N; ++i) s[i] = (double)(next_u32() % 17u);    /* many ties */
        const int64_t ks[] = {1, N / 2 > 0 ? N / 2 : 1, N};
        for (int b = 0; b < 3; ++b) {
            const int64_t k = ks[b];
            int64_t *idx = (int64_t *)must(sizeof(int64_t) * (size_t)k);
            double *val = (double *)must(sizeof(double) * (size_t)k), pos = 0.0;
            int rc = orc_topk(s, N, k, idx, val);
            for (int64_t i = 0; i < k; ++i) pos += (double)idx[i] * (double)(1 + (i % 5));
            report("topk", N, k, 0, rc, checksum(val, (size_t)k) + pos);
            free(idx); free(val);
        }
        free(s);
    }
}

static void sgd_cases(void) {
    const int32_t Ds[] = {3, 64, 130};
    for (int a = 0; a < 3; ++a)
        for (int32_t n_pos = 0; n_pos <= 5; n_pos += 5)
            for (int32_t n_neg = 0; n_neg <= 7; n_neg += 7) {
                if (n_pos + n_neg == 0) continue;
                const int32_t D = Ds[a];
                const int64_t pool = 11, ld = D + 2;
                float *Xp = floats((size_t)((pool - 1) * ld + D)), *Xn = floats((size_t)((pool - 1) * ld + D)), *w = floats((size_t)D);
                int32_t *ip = (int32_t *)must(sizeof(int32_t) * (size_t)n_pos), *in = (int32_t *)must(sizeof(int32_t) * (size_t)n_neg);
                for (int32_t i = 0; i < n_pos; ++i) ip[i] = (int32_t)(next_u32() % (uint32_t)pool);
                for (int32_t i = 0; i < n_neg; ++i) in[i] = (int32_t)(next_u32() % (uint32_t)pool);
                if (n_pos) ip[0] = (int32_t)pool - 1;              /* the last row of the pool */
                double *wo = (double *)must(sizeof(double) * (size_t)D), b = 0.0;
                double *margins = (double *)must(sizeof(double) * (size_t)(n_pos + n_neg));
                for (int64_t t = 1; t <= 3; t += 2) {
                    int rc = orc_sgd_step(w, 0.125, D, n_pos ? Xp : NULL, ld, n_pos ? ip : NULL, n_pos, n_neg ? Xn : NULL, ld,
                                          n_neg ? in : NULL, n_neg, 0.01, t, (int32_t)(t == 3), wo, &b, margins);
                    report("sgd_step", D, n_pos, n_neg, rc, checksum(wo, (size_t)D) + b + checksum(margins, (size_t)(n_pos + n_neg)));
                }
                double obj = 0.0;
                int rc = orc_svm_objective(wo, b, D, Xp, ld, pool, Xn, ld, pool, 0.01, &obj);
                report("svm_objective", D, n_pos, n_neg, rc, obj);
                free(Xp); free(Xn); free(w); free(ip); free(in); free(wo); free(margins);
            }
}

int main(void) {
    double h = 0.0;
    for (uint32_t v = 0; v < 65536u; v += 1u)
        if (((v >> 10) & 0x1f) != 0x1f) h += orc_half_to_double((uint16_t)v) * (double)(1 + v % 3);
    report("half_to_double", 65536, 0, 0, orc_num_threads() > 0 ? 0 : 1, h);
    dense_cases();
    pq_cases();
    bit_cases();
    sparse_cases();
    topk_cases();
    sgd_cases();
    /* argument errors: rejected before any pointer is followed */
    double out[1];
    report("null_args", 0, 0, 0, orc_dense_f32(NULL, 1, 4, 4, NULL, 1, NULL, out), 0.0);
    report("null_args", 1, 0, 0, orc_topk(NULL, 1, 1, NULL, NULL), 0.0);
    report("null_args", 2, 0, 0, orc_binary_scores(NULL, 1, 32, 1, NULL, 0.0, out), 0.0);
    report("null_args", 3, 0, 0, orc_pq_lut(NULL, 1, 1, 1, NULL, out), 0.0);
    return 0;
}
