/*
 * otf.h -- C ABI of the on-the-fly ranking hot path for MI355X (gfx950).
 *
 * The library ranks a large, GPU-resident store of compact image features by the score of
 * a linear SVM, s_i = <w, x_i> + b, and returns the k best rows; it also performs the
 * Pegasos mini-batch update of w.  These are the two operations the GPU back-end of
 * "Efficient On-the-fly Category Retrieval using ConvNets and GPUs" (arXiv 1407.4764)
 * alternates between (Sec. 4, "On-line (GPU back-end)").
 *
 * Conventions shared by every entry point
 *   - Every pointer is a DEVICE pointer unless its comment says "host".  The caller owns
 *     every buffer; the library allocates nothing and keeps no state between calls (the
 *     diagnostics at the end of this header are the exception and say so).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it and the call returns without synchronising; outputs are valid once
 *     the caller has synchronised the stream.
 *   - Matrices are row-major.  Row starts must be 16-byte aligned (base pointer and
 *     leading dimension), otherwise OTF_ERR_INVALID_ARG.
 *   - Row indices are int32: N must be below 2^31, otherwise OTF_ERR_UNSUPPORTED.
 *   - Ranked lists hold k entries, best first: score descending, equal scores by ascending
 *     row index.  1 <= k <= N, otherwise OTF_ERR_INVALID_ARG; k above OTF_MAX_K is a limit of
 *     this build: OTF_ERR_UNSUPPORTED.  A score of -0.0 is reported as +0.0.
 *     Scores must be finite; NaN/Inf inputs give unspecified (but in-range) rankings.
 *   - Return value: OTF_OK (0) or a negative otf_status.  Argument errors are detected on
 *     the host before anything is enqueued: then no buffer has been written.
 *   - A leading dimension (ldx, ld, ld_phi; in elements) is at least the row length and small
 *     enough that the whole store spans less than 2^48 bytes; otherwise OTF_ERR_INVALID_ARG.
 *   - `ws` is scratch device memory of at least otf_workspace_bytes(N, k, Q) bytes,
 *     256-byte aligned.  Its contents are undefined on entry and on exit.  Two calls that
 *     overlap in time (different streams) need different workspaces.
 */
#ifndef OTF_H_
#define OTF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OTF_OK = 0,
    OTF_ERR_INVALID_ARG = -1, /* NULL pointer, non-positive size, k out of range, misalignment */
    OTF_ERR_UNSUPPORTED = -2, /* a shape this build has no kernel for (see each function)   */
    OTF_ERR_WORKSPACE = -3,   /* ws is NULL, misaligned or smaller than otf_workspace_bytes */
    OTF_ERR_HIP = -4,         /* a HIP runtime call or kernel launch failed                 */
    OTF_ERR_SCRATCH = -5      /* the call needs more scratch than a no-allocation entry point owns */
} otf_status;

/* Element type of a dense store or model.  An integer at the boundary, so that a value that names
 * no type arrives as it was passed (and is answered with OTF_ERR_INVALID_ARG) in C and C++ alike. */
typedef int32_t otf_dtype;
enum { OTF_F32 = 0, OTF_F16 = 1 };

/* Largest k any ranking call accepts. */
#define OTF_MAX_K 8192

/* Host.  Name of a status code (static string). */
const char *otf_status_string(int status);

/* Host.  Upper bound on the scratch bytes any otf_rank_* / otf_topk call needs for N rows,
 * list length k and Q simultaneous classifiers.  Returns 0 for invalid arguments. */
size_t otf_workspace_bytes(int64_t N, int32_t k, int32_t Q);

/*
 * Dense store (paper Sec. 4: the pre-computed ConvNet features of the target dataset kept
 * in GPU memory, Table 2 rows "2048" / "128", 4 bytes per dimension; ranking = scoring all
 * of them with the current model, then sorting).
 *
 *   scores[q][i] = bias[q] + sum_d W[q][d] * X[i][d]      accumulated in fp32
 *
 *   X     N x D, dtype xdt, leading dimension ldx (elements, >= D).
 *   W     Q x D, dtype wdt, contiguous.  Q >= 1.
 *   bias  Q floats, or NULL for zero.
 *   out_scores, out_idx   Q x k, the ranked list of each classifier.
 *   all_scores            Q x N floats, or NULL when the caller wants only the lists.
 *
 * Supported: xdt = F32 with wdt = F32; xdt = F16 with wdt = F32 or F16.  D a multiple of 4
 * (F32) or 8 (F16), at most 16384.  With Q > 1 and F16/F16 inputs, Q a multiple of 32 and D
 * a multiple of 128, scoring runs as an MFMA matrix product (unless 127 row strides exceed
 * 4 GiB); other Q > 1 shapes are scored one classifier at a time (X is then read Q times).
 * Anything else: OTF_ERR_UNSUPPORTED.
 */
int otf_rank_dense(const void *X, otf_dtype xdt, int64_t N, int32_t D, int64_t ldx,
                   const void *W, otf_dtype wdt, int32_t Q, const float *bias,
                   int32_t k, float *out_scores, int32_t *out_idx,
                   float *all_scores, void *ws, size_t ws_bytes, void *stream);

/*
 * otf_rank_dense for callers that cannot allocate device memory and so cannot bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as otf_rank_dense without `ws`; the scratch is an array of
 * OTF_NOALLOC_SCRATCH_BYTES that is part of the library's device code (each GPU the library runs
 * on holds its own copy until the process ends).  The call allocates and frees nothing.
 *   - Sizes whose otf_workspace_bytes(N, k, Q) exceed OTF_NOALLOC_SCRATCH_BYTES (one classifier:
 *     above ~3.8 million rows) return OTF_ERR_SCRATCH and enqueue nothing.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *     streams or host threads) race and give undefined results; calls on one stream are safe.
 *     Every call clears the parts of the array that must start at zero itself.
 *   - The first call on a GPU looks up that GPU's copy of the array (hipGetSymbolAddress); make it
 *     outside a graph capture.
 */
#define OTF_NOALLOC_SCRATCH_BYTES (16u << 20)

int otf_rank_dense_noalloc(const void *X, otf_dtype xdt, int64_t N, int32_t D, int64_t ldx,
                           const void *W, otf_dtype wdt, int32_t Q, const float *bias,
                           int32_t k, float *out_scores, int32_t *out_idx,
                           float *all_scores, void *stream);

/*
 * Product-quantised store (paper Sec. 3, "Product quantization (PQ)": the feature is cut
 * into M sub-blocks of dsub dimensions, each replaced by the index of the nearest of K
 * centres of that sub-block's own vocabulary; Table 2: one byte per sub-block, so K = 256).
 * The paper does not say how coded rows are scored; this library scores the reconstructed
 * row, sum_m <w_m, C[m][code_m]>, through a table of the K partial products per sub-block.
 *
 * otf_pq_build_lut:  lut[m][k] = sum_{j<dsub} w[m*dsub + j] * codebooks[m][k][j]   (fp32)
 *   codebooks  M x K x dsub floats, contiguous.   w  M*dsub floats.   lut  M x K floats.
 *   Any M, K, dsub >= 1.
 *
 * otf_rank_pq:       scores[i] = bias + sum_m lut[m][codes[i][m]]                  (fp32)
 *   codes  N x M bytes, contiguous rows (leading dimension M).  lut as built above.
 *   K must be 256 and M a multiple of 16, at most 1024 (rows are read in 16-byte chunks; M = 512
 *   is the paper's 2048-D feature at 4 dimensions per sub-block); other shapes return
 *   OTF_ERR_UNSUPPORTED.
 */
int otf_pq_build_lut(const float *codebooks, int32_t M, int32_t K, int32_t dsub,
                     const float *w, float *lut, void *stream);

/*
 * otf_rank_pq_model: otf_pq_build_lut followed by otf_rank_pq in one call, for the on-line loop of
 * Sec. 4, where every ranking runs under a new model and nobody reads the table: the table goes
 * from the vocabularies and w straight into the layout the scan uses (one launch less).  Scores
 * and lists are bit-identical to the two calls.  Same shapes and errors as otf_rank_pq; dsub >= 1.
 */
int otf_rank_pq_model(const uint8_t *codes, int64_t N, int32_t M, int32_t K, int32_t dsub,
                      const float *codebooks, const float *w, float bias, int32_t k,
                      float *out_scores, int32_t *out_idx, float *all_scores,
                      void *ws, size_t ws_bytes, void *stream);

int otf_rank_pq(const uint8_t *codes, int64_t N, int32_t M, int32_t K, const float *lut,
                float bias, int32_t k, float *out_scores, int32_t *out_idx,
                float *all_scores, void *ws, size_t ws_bytes, void *stream);

/*
 * Binarised store (paper Sec. 3, "Binarization", Eq. (1): codes in {0,1}^D, ranked by a
 * linear SVM).  Dimension d of row i is bit (d mod 32), least significant first, of 32-bit
 * word (d div 32) of that row.  A bit enters the model as +1 (set) or -1 (clear):
 *
 *   scores[i] = bias + sum_d w[d] * (2 * bit_{i,d} - 1)                           (fp32)
 *
 *   bits  N x (D/32) uint32, contiguous rows.   w  D floats.
 *   D must be a multiple of 128 (rows are read in 16-byte chunks), at most 8192; other values
 *   return OTF_ERR_UNSUPPORTED.
 */
int otf_rank_binary(const uint32_t *bits, int64_t N, int32_t D, const float *w, float bias,
                    int32_t k, float *out_scores, int32_t *out_idx,
                    float *all_scores, void *ws, size_t ws_bytes, void *stream);

/*
 * Sparse-row store (paper Sec. 3.1, discussion after Table 2: the ConvNet features are very sparse,
 * the 128-D ones over 60 % zeros, and compression that exploits it could shrink the store further).
 * The scores are those of otf_rank_dense on the expanded rows; only the storage differs:
 *
 *   row i occupies the 32-bit words [start[i], start[i+1]) of `rows`: first D/32 words of presence
 *   mask (dimension d = bit d mod 32, least significant first, of word d div 32; set iff the value
 *   is stored), then the fp32 bit patterns of the stored values in ascending order of dimension.
 *
 *   scores[i] = bias + sum over stored d of w[d] * value_{i,d}                       (fp32)
 *
 *   rows   the word array, 16-byte aligned, readable up to start[N] rounded up to a multiple of 4 words.
 *   start  N + 1 int64 word offsets, ascending, start[i+1] - start[i] = D/32 + popcount(mask of row i).
 *   D must be 128 (the paper's compact feature); other values return OTF_ERR_UNSUPPORTED.
 */
int otf_rank_sparse(const uint32_t *rows, const int64_t *start, int64_t N, int32_t D, const float *w,
                    float bias, int32_t k, float *out_scores, int32_t *out_idx,
                    float *all_scores, void *ws, size_t ws_bytes, void *stream);

/*
 * Hamming ranking of the binarised store (paper Sec. 3.1, discussion after Table 2: binary codes
 * could be ranked faster still by Hamming distances, which the hardware computes cheaply; that
 * needs a ranking model other than the linear SVM and is left open there).  The model here
 * is a query code of D bits in the layout of the rows; nearer rows rank first:
 *
 *   scores[i] = -(number of dimensions d < D with bit_{i,d} != query bit d)      (exact)
 *
 *   bits   N x (D/32) uint32, contiguous rows.   query  D/32 uint32, 16-byte aligned.
 *   Equal distances rank by ascending row index, like every list of this library.
 *   D a multiple of 128, at most 8192; other values return OTF_ERR_UNSUPPORTED.
 */
int otf_rank_hamming(const uint32_t *bits, int64_t N, int32_t D, const uint32_t *query,
                     int32_t k, float *out_scores, int32_t *out_idx,
                     float *all_scores, void *ws, size_t ws_bytes, void *stream);

/*
 * Ranking alone (paper Sec. 4: the scores are sorted on the GPU and the head of the list is
 * handed to the front-end).  For each of the Q rows of `scores` (row stride ld floats,
 * ld >= N) returns the k largest entries, sorted.
 */
int otf_topk(const float *scores, int64_t N, int64_t ld, int32_t Q, int32_t k,
             float *out_scores, int32_t *out_idx, void *ws, size_t ws_bytes, void *stream);

/*
 * One Pegasos mini-batch step on the hinge loss with L2 regulariser lambda (paper Sec. 4,
 * "Training": learning rate 1/(lambda t), each batch half positives, half negatives).
 * The batch is rows Xpos[idx_pos[0..n_pos)] with label +1 and rows Xneg[idx_neg[0..n_neg)]
 * with label -1 (sampling is the caller's job); B = n_pos + n_neg.
 *
 *   eta  = 1 / (lambda * t)
 *   m_j  = y_j * (<w, x_j> + b)        with w, b as they are on entry
 *   V    = { j : m_j < 1 }
 *   w   <- (1 - eta*lambda) * w + (eta / B) * sum_{j in V} y_j * x_j
 *   b   <- b + (eta / B) * sum_{j in V} y_j      only if update_bias != 0
 *
 *   w  D floats, updated in place.  b  one float (may be NULL: bias 0, never updated).
 *   Xpos, Xneg  fp32 pools with leading dimensions ld_pos, ld_neg (elements, >= D).
 *   idx_pos, idx_neg  int32 row numbers into the pools (device memory).
 *   D a multiple of 4; 1 <= B <= 4096; t >= 1; lambda > 0.
 *   ws  at least otf_sgd_workspace_bytes(B) bytes.
 */
size_t otf_sgd_workspace_bytes(int32_t B);

int otf_svm_sgd_step(float *w, float *b, int32_t D,
                     const float *Xpos, int64_t ld_pos, const int32_t *idx_pos, int32_t n_pos,
                     const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int32_t n_neg,
                     float lambda, int64_t t, int32_t update_bias,
                     void *ws, size_t ws_bytes, void *stream);

/*
 * n_steps consecutive Pegasos steps (iterations t_first, t_first + 1, ...) from one call:
 * step s uses the batch idx_pos[s * n_pos .. (s+1) * n_pos), idx_neg[s * n_neg .. (s+1) * n_neg).
 * Same arguments, limits and errors as otf_svm_sgd_step; n_steps >= 1.  (Paper Sec. 4: between two
 * rankings the model takes as many steps as fit; one call keeps the host out of that loop.)
 *
 * The steps are enqueued back to back, two kernels each.  A second route runs the whole call as ONE
 * kernel (D <= 2048; diagnostic switch OTF_DEBUG_SGD_PASS_PATH): up to 32 workgroups share the batch
 * rows and meet once per step through a counter in `ws`.  It is not the default because on this
 * chip a step then costs a chain of round trips between dies, ~15 us against ~10 us.  Its waits
 * are bounded: if one expires (the workgroups could not all become resident, e.g. on a GPU that
 * other work keeps full for seconds) the kernel ends at once, w and b keep their values from before
 * the call, and the 32-bit word at the start of `ws` reads 1 after the call has completed.  After
 * any complete run, by either route, it reads 0.  The routes agree to rounding (the sums are
 * formed in another order).
 */
int otf_svm_sgd_pass(float *w, float *b, int32_t D,
                     const float *Xpos, int64_t ld_pos, const int32_t *idx_pos, int32_t n_pos,
                     const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int32_t n_neg,
                     float lambda, int64_t t_first, int32_t n_steps, int32_t update_bias,
                     void *ws, size_t ws_bytes, void *stream);

/*
 * Diagnostic: counts the entries of idx[0..n) that are not row numbers of a pool of `rows` rows into
 * *bad (one int32 in device memory, which the caller has set to 0).  The training calls read their
 * row numbers unchecked (they are not told the pools' sizes): check them once where they are made.
 */
int otf_check_indices(const int32_t *idx, int64_t n, int64_t rows, int32_t *bad, void *stream);

/*
 * Binarisation encoder (paper Sec. 3, "Binarization", Eq. (1)): a zero-centred descriptor phi in
 * R^m is coded as beta = sgn(U phi) in {0,1}^n, n > m, with sgn(a) = 1 iff a > 0 (a zero
 * projection codes as 0) and U the first m columns of the orthogonal factor of a QR
 * decomposition of a random n x n matrix.  The codes are the rows otf_rank_binary scans:
 * dimension d is bit (d mod 32), least significant first, of word (d div 32).
 *
 * otf_tight_frame:  U from the random matrix (set-up, once per frame).
 *   G   n x n floats, row-major, drawn by the caller.  Of the possible QR factorisations the one
 *       with a positive diagonal of R is taken, so U is a function of G (it depends on the
 *       first m columns of G only and is their Gram-Schmidt orthonormalisation, computed in fp64).
 *       A leading column that lies in the span of its predecessors (what orthogonalisation
 *       leaves of it is below n * 2^-52 of its length) gives a zero column in U, and the
 *       columns after it are orthogonalised against the non-zero ones only.
 *   U   n x m floats, row-major (row d = the frame vector of code bit d).
 *   ws  at least otf_tight_frame_workspace_bytes(n, m) bytes, 16-byte aligned.
 *   1 <= m <= n; n <= 4096 and m <= 256, otherwise OTF_ERR_UNSUPPORTED.
 *
 * otf_binarize:  bits[i][d] = ( sum_j U[d][j] * phi[i][j] > 0 ), evaluated on the matrix cores
 *   at fp32 accuracy (every value enters as three exact bf16 pieces, piece products below 2^-22 of
 *   |U[d][j] phi[i][j]| are left out, sums in fp32): a bit whose exact projection is within
 *   rounding of zero may differ from an evaluation in another precision.
 *   phi   N x m floats, leading dimension ld_phi (elements, >= m, a multiple of 4).
 *   U     n x m floats as above, contiguous.      bits  N x (n/32) uint32, contiguous rows.
 *   m a multiple of 4, at most 128; n a multiple of 32; otherwise OTF_ERR_UNSUPPORTED.
 */
size_t otf_tight_frame_workspace_bytes(int32_t n, int32_t m);

int otf_tight_frame(const float *G, int32_t n, int32_t m, float *U, void *ws, size_t ws_bytes, void *stream);

int otf_binarize(const float *phi, int64_t N, int32_t m, int64_t ld_phi, const float *U, int32_t n,
                 uint32_t *bits, void *stream);

/*
 * Product-quantisation encoder and vocabulary training (paper Sec. 3, "Product quantization (PQ)":
 * every sub-block has a vocabulary of its own, learned beforehand on training features, and is
 * stored as the index of one of its centres).  The codes are the rows otf_rank_pq scans.
 *
 * otf_pq_encode:  codes[i][m] = argmin_k || X[i][m*dsub .. (m+1)*dsub) - codebooks[m][k] ||^2, the
 *   lowest k among equal distances.  Evaluated as argmin_k ||c_k||^2 - 2 <x, c_k> on the matrix cores
 *   at fp32 accuracy (every value enters as three exact bf16 pieces and piece products below
 *   2^-22 of |x_j c_j| are left out; sums in fp32): where two centres are equally near to within
 *   rounding, either may be returned.
 *   X  N x (M*dsub) floats, leading dimension ldx (elements, a multiple of 4).
 *   codebooks  M x K x dsub floats, contiguous.   codes  N x M bytes, contiguous rows, 4-byte aligned.
 *   K must be 256, dsub 4, 8 or 16, M a multiple of 4; otherwise OTF_ERR_UNSUPPORTED.
 *
 * otf_pq_lloyd_step:  one k-means iteration on the training rows X.  The paper does not say how the
 *   centres are learned; the PQ method it cites uses k-means, taken here as Lloyd iterations from
 *   centres supplied by the caller: (1) codes = otf_pq_encode(X, codebooks); (2) every centre moves
 *   to the mean of the sub-vectors assigned to it, a centre with none stays.  The sums are taken
 *   in 64-bit fixed point, scaled from the largest sub-vector norm of X and from N so that no sum can
 *   overflow (resolution at most 2^-30 of that norm for N < 2^31, 2^-41 at a million rows): the
 *   new centres and the distortion are the same bits whatever the order the rows are added in, run
 *   after run.  X must be finite.  codebooks is updated in place; codes receives the assignment of
 *   step (1); *distortion (one double in device memory, may be NULL) the mean over rows of the
 *   summed squared distances to the assigned centres, measured before the move and evaluated in
 *   double precision as sum ||x||^2 + sum_k (n_k ||c_k||^2 - 2 <c_k, S_k>), S_k the sum and n_k the
 *   number of the sub-vectors assigned to centre k (exact up to ~1e-15 of sum ||x||^2).
 *
 *   ws  at least otf_pq_train_workspace_bytes(M, dsub) bytes, 256-byte aligned.
 */
size_t otf_pq_train_workspace_bytes(int32_t M, int32_t dsub);

int otf_pq_encode(const float *X, int64_t N, int64_t ldx, const float *codebooks, int32_t M, int32_t K,
                  int32_t dsub, uint8_t *codes, void *ws, size_t ws_bytes, void *stream);

int otf_pq_lloyd_step(const float *X, int64_t N, int64_t ldx, float *codebooks, int32_t M, int32_t K,
                      int32_t dsub, uint8_t *codes, double *distortion, void *ws, size_t ws_bytes, void *stream);

/*
 * Diagnostics (host, not part of the paper's method; for benchmarks that must time the
 * scoring kernel by itself).  Between otf_profile_begin and otf_profile_end every otf_rank_*
 * call brackets its scoring kernel(s), and every otf_pq_lloyd_step call the kernel of its
 * per-centre sums, with a pair of HIP events on the call's stream, at most max_records calls.  otf_profile_end waits for the recorded events, returns the summed
 * kernel time in milliseconds and the number of calls recorded, and releases the events.
 * Process-wide state, not thread-safe; returns OTF_ERR_INVALID_ARG when misused.
 */
int otf_profile_begin(int32_t max_records);
int otf_profile_end(double *scan_ms_total, int32_t *n_records);

/*
 * Diagnostic switches (host, not part of the paper's method; for tests that must force a code
 * path and for launch-shape sweeps).  otf_debug_set(key, value) sets one process-wide switch that
 * every later call reads; value 0 clears it (the built-in choice applies again).  The results of
 * the library do not depend on any switch, only which kernels produce them and how they are
 * launched.  Returns OTF_ERR_INVALID_ARG for an unknown key or a value the key does not accept.
 * Not thread-safe against calls that are being enqueued at the same time.
 */
typedef enum {
    OTF_DEBUG_RANK_PATH = 0,         /* 1: always rank by full selection over materialised scores */
    OTF_DEBUG_BINARIZE_FP32,         /* 1: otf_binarize with fp32 matrix instructions (comparison kernel) */
    OTF_DEBUG_PQENC_FP32,            /* 1: otf_pq_encode with fp32 matrix instructions (comparison kernel) */
    OTF_DEBUG_SCAN_THREADS,          /* threads per workgroup of the table scans: a multiple of 64, 64..1024 */
    OTF_DEBUG_SCAN_UNROLL,           /* 4 or 8 loads per lane and tile in the filtered table scan */
    OTF_DEBUG_BINARIZE_WAVES,        /* 4 or 8 waves per workgroup of otf_binarize */
    OTF_DEBUG_PQENC_RANGE,           /* sub-blocks per work unit of otf_pq_encode: a multiple of 4, 4..64 */
    OTF_DEBUG_DENSE_BLOCKS_PER_CU,   /* 1..8 workgroups per compute unit, wide dense scan */
    OTF_DEBUG_NARROW_BLOCKS_PER_CU,  /* 1..8, dense scan of rows up to 512 bytes */
    OTF_DEBUG_MFMA_BLOCKS_PER_CU,    /* 1..8, multi-classifier scan */
    OTF_DEBUG_PQENC_BLOCKS_PER_CU,   /* 1..8, otf_pq_encode */
    OTF_DEBUG_WALK_TILES,            /* 2, 4 or 8 tiles of 64 rows per wave and block, table scans of rows > 128 bytes */
    OTF_DEBUG_SGD_PASS_PATH,         /* 1: otf_svm_sgd_pass as one kernel for the whole run (D <= 2048) */
    OTF_DEBUG_SGD_SPIN_LIMIT,        /* polls after which a wait of the one-launch training run gives up (default 2^20) */
    OTF_DEBUG_MEET_SPIN_LIMIT,       /* polls after which a workgroup of the fallback selection stops waiting for the
                                        others between passes (default 2^14); then one workgroup finishes alone */
    OTF_DEBUG_KEYS
} otf_debug_key;

int otf_debug_set(int key, int value);

#ifdef __cplusplus
}
#endif
#endif /* OTF_H_ */
