// Host-side declarations shared by the translation units of libotf.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "otf.h"
#include "otf_device.h"

namespace otf {

// Where the selection state of the Q classifiers lives inside the workspace.
struct SelectWs {
    SelState *st;              // [Q]
    uint32_t *hist1;           // [Q][kHistShards][kBins1]
    uint32_t *hist2;           // [Q][kBins2]
    uint32_t *hist3;           // [Q][kBins3]
    uint32_t *blockhist3;      // [Q][kSelBlocks][kBins3]
    uint32_t *eqoff;           // [Q][kSelBlocks]
    unsigned long long *cand;  // [Q][kCandCap]   (key << 32 | ~index)
};

struct WsLayout {
    size_t st, hist1, hist2, hist3, blockhist3, eqoff, cand, sample_st, sample_scores,
        lut_image, short_store, scores, total;
    int64_t sample_ld;   // row stride (floats) of the sample score buffer
};
// Byte offsets of the workspace regions for N rows and Q classifiers (every offset 256-aligned).
WsLayout ws_layout(int64_t N, int32_t Q);
SelectWs select_ws(void *ws, const WsLayout &L);         // state of the full selection
SelectWs sample_select_ws(void *ws, const WsLayout &L);  // state used to threshold the sample

constexpr int kDenseMaxD = 16384;  // widest dense row any kernel takes (elements)
constexpr size_t kLutImageBytes = 8u * 128u * 1024u + 4096u;  // up to 8 table images of 128 KiB, or one + side table

// A table store of fewer rows than one tile of the multi-image scan is copied here first.
constexpr int kShortStoreRows = 64;
constexpr size_t kShortStoreBytes = (size_t)kShortStoreRows * 1024u;

// Rows of the strided sample of an N-row store (whole groups only).
inline int64_t sample_rows(int64_t N) {
    return N / ((int64_t)kSampleGroup * kSampleStride) * kSampleGroup;
}

// Zeroes the selection state and the pass-1/2 histograms of Q classifiers.
hipError_t launch_select_init(const SelectWs &sw, int Q, hipStream_t s);
// The same for the full selection's state and the sample's in one launch.
hipError_t launch_select_init_both(const SelectWs &sw, const SelectWs &sample_sw, int Q, hipStream_t s);
// Radix pass 1 over ready-made scores (rows of length N, stride ld).
hipError_t launch_hist1(const float *scores, int64_t N, int64_t ld, int Q, const SelectWs &sw, Gate gate,
                        hipStream_t s);
// Passes 2 and 3 (skipped on the device when pass 1 was decisive), gather and final sort.
//   kTailPlain       four launches
//   kTailBehindFlag  the fallback of filtered scans whose lists launch_filter_sort has judged (many
//                    classifiers): one launch that returns at once unless sw.st[0].fallback is set
//   kTailBehindScan  the end of ONE classifier's filtered scan, in one launch: when the scan's list
//                    serves (Gate{sw.st, k} shut) one workgroup sorts it into the outputs; otherwise
//                    the flag is raised (for whoever asks afterwards) and the full selection runs on the
//                    scores that the gated re-scan before this launch has written
enum SelectTail { kTailPlain = 0, kTailBehindFlag = 1, kTailBehindScan = 2 };
hipError_t launch_select_tail(const float *scores, int64_t N, int64_t ld, int Q, int k, const SelectWs &sw,
                              float *out_scores, int32_t *out_idx, SelectTail tail, hipStream_t s);
// Thresholds of the filtered scans of Q classifiers from the Nv sample scores of each (rank m):
// sample_sw.st[q].tau_key receives the top 24 bits of the m-th largest sample key, and
// main_st[0].fallback is raised when a classifier's threshold would let far more rows pass than the
// candidate list holds.  Only the states of sample_sw are used.
hipError_t launch_sample_threshold(const float *sample_scores, int64_t Nv, int64_t ld, int Q, int m,
                                   const SelectWs &sample_sw, SelState *main_st, hipStream_t s);
// otf_topk in one read of the scores (one classifier, N large enough for a sample): zeroes the states
// itself, sample -> threshold -> filter -> sort, the exact passes gated behind.
hipError_t launch_topk_filtered(const float *scores, int64_t N, int k, const SelectWs &sw, const SelectWs &sample_sw,
                                SampleSlot *slots, float *out_scores, int32_t *out_idx, hipStream_t s);
// End of a filtered scan: sort the appended candidates or raise sw.st[0].fallback.
hipError_t launch_filter_sort(const SelectWs &sw, int Q, int k, float *out_scores, int32_t *out_idx, hipStream_t s);

enum ScanEmit { kEmitScores = 0, kEmitSample = 1, kEmitFilter = 2 };

// Dense single-classifier scan: writes N scores (bias included) and accumulates the pass-1 histogram.
// chunk_ctr: a zeroed word in global memory (work counter of the dynamically scheduled kernels).
hipError_t launch_dense_scan(const void *X, int x_is_half, int64_t N, int D, int64_t ldx,
                             const void *w, int w_is_half, const float *bias_ptr, int bias_index,
                             float *scores, uint32_t *hist1, uint32_t *chunk_ctr, hipStream_t s);
// True for rows of at most 512 bytes: those scans also come as sample and filtered scans.
bool dense_scan_filters(int x_is_half, int D);
// The same scan in the three forms of the table scans (narrow rows only for the last two):
//   kEmitScores  as above; behind a gate (see Gate) the kernel returns at once unless the gate is open
//   kEmitSample  N = rows of the strided sample, numbered compactly: the waves' largest keys into `slots`,
//                their number into st (the sample's state)
//   kEmitFilter  rows at or above the threshold go to cand (cursor in st); every workgroup resolves the
//                threshold from `slots` (their number in tau->ncand); store_rows = rows of the whole store
hipError_t launch_dense_scan_emit(const void *X, int x_is_half, int64_t N, int D, int64_t ldx, const void *w,
                                  int w_is_half, const float *bias_ptr, int bias_index, ScanEmit emit, float *scores,
                                  uint32_t *hist1, uint32_t *chunk_ctr, SelState *st, const SelState *tau,
                                  SampleSlot *slots, unsigned long long *cand, Gate gate, hipStream_t s);

// Multi-classifier fp16 scan on the matrix cores (Q = 32 or 64 classifiers per call).
//   kEmitScores  scores[q][i] for every row (row stride ld_scores); behind a gate (see Gate) the kernel
//                returns at once unless the gate is open
//   kEmitSample  the same for the strided sample only (compact row numbering)
//   kEmitFilter  nothing is stored but the rows with key >= tau[q].tau_key, appended to cand[q]; with
//                a gate the kernel returns at once if gate.st->fallback is ALREADY raised
// tile_ctr: a zeroed word in global memory (the kernel hands out its tiles dynamically).
hipError_t launch_dense_mfma(const void *X, int64_t N, int D, int64_t ldx, const void *W, int Q, const float *bias,
                             ScanEmit emit, float *scores, int64_t ld_scores, const SelState *tau, SelState *st,
                             unsigned long long *cand, Gate gate, uint32_t *tile_ctr, hipStream_t s);

// Byte-indexed table scans (product-quantised codes, binary codes).
hipError_t launch_pq_build_lut(const float *codebooks, int M, int K, int dsub, const float *w, float *lut, hipStream_t s);
// Table images in scan layout; also zero both selection states.
hipError_t launch_pq_prepare(const float *lut, int M, float *image, const SelectWs &sw, const SelectWs &sample_sw,
                             hipStream_t s);
// The PQ images straight from the vocabularies and the model (no table in between).
hipError_t launch_pq_prepare_model(const float *codebooks, const float *w, int M, int dsub, float *image,
                                   const SelectWs &sw, const SelectWs &sample_sw, hipStream_t s);
hipError_t launch_binary_prepare(const float *w, int D, float *image, const SelectWs &sw, const SelectWs &sample_sw,
                                 hipStream_t s);
// row_bytes = stored bytes per row (a multiple of 16, at most 1024; rows longer than 128 bytes are walked
// through several table images).  kind: byte groups; the 2048-bit binary layout (7+7+7+7+4 bits per
// word); or no table at all: `image` is a query code of row_bytes bytes and the score is minus the
// Hamming distance to it.
enum TableKind { kTableBytes = 0, kTableSeven = 1, kTableHamming = 2 };
//   kEmitScores  scores + pass-1 histogram into (st, hist1); `gate` as above
//   kEmitSample  N = rows of the strided sample (compact numbering): every wave leaves the largest key it
//                met in its slot of `slots`; st = the sample's state, which receives the number of slots
//   kEmitFilter  append rows at or above the threshold to cand (cursor in st); every block resolves the
//                threshold from `slots` (their number in tau->ncand)
hipError_t launch_table_scan(const uint8_t *codes, int64_t N, int row_bytes, TableKind kind, const float *image,
                             float bias, ScanEmit emit, float *scores, SelState *st, uint32_t *hist1,
                             const SelState *tau, SampleSlot *slots, unsigned long long *cand, Gate gate,
                             hipStream_t s);

// Sparse-row store of 128-D features (mask + packed non-zero values per row, word offsets in start).
hipError_t launch_sparse_scan(const uint32_t *rows, const int64_t *start, int64_t N, int64_t store_rows, const float *w,
                              float bias, ScanEmit emit, float *scores, SelState *st, uint32_t *hist1,
                              const SelState *tau, SampleSlot *slots, unsigned long long *cand, Gate gate,
                              hipStream_t s);

hipError_t launch_sgd_step(float *w, float *b, int D, const float *Xpos, int64_t ld_pos, const int32_t *idx_pos,
                           int n_pos, const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int n_neg,
                           float lambda, int64_t t, int update_bias, float *coef, hipStream_t s);

// A run of consecutive steps in one launch (D <= 2048); ws holds sgd_pass_ws_bytes(D) bytes, its first word
// the status (0 complete, 1 a bounded wait expired).
bool sgd_pass_fits(int D);
size_t sgd_pass_ws_bytes(int D);
hipError_t launch_sgd_pass(float *w, float *b, int D, const float *Xpos, int64_t ld_pos, const int32_t *idx_pos,
                           int n_pos, const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int n_neg,
                           float lambda, int64_t t_first, int n_steps, int update_bias, void *ws, uint32_t spin_limit,
                           hipStream_t s);
hipError_t launch_sgd_pass_clear_status(void *ws, hipStream_t s);
hipError_t launch_check_indices(const int32_t *idx, int64_t n, int64_t rows, int32_t *bad, hipStream_t s);

// Binarisation encoder: the frame from the random matrix (scratch: n*m doubles), and the codes.
hipError_t launch_tight_frame(const float *G, int n, int m, double *scratch, float *U, hipStream_t s);
hipError_t launch_binarize(const float *phi, int64_t N, int m, int64_t ld, const float *U, int n, uint32_t *bits,
                           hipStream_t s);

// PQ encoder and one Lloyd iteration (K = 256; dsub 4, 8 or 16; M a multiple of 4).
size_t pq_train_ws_bytes(int M, int dsub);
hipError_t launch_pq_encode(const float *X, int64_t N, int64_t ldx, const float *codebooks, int M, int dsub,
                            uint8_t *codes, void *ws, hipStream_t s);
hipError_t launch_pq_lloyd_assign(const float *X, int64_t N, int64_t ldx, const float *codebooks, int M, int dsub,
                                  uint8_t *codes, void *ws, hipStream_t s);
hipError_t launch_pq_lloyd_sums(const float *X, int64_t N, int64_t ldx, const uint8_t *codes, int M, int dsub, void *ws,
                                hipStream_t s);
hipError_t launch_pq_lloyd_move(int64_t N, float *codebooks, int M, int dsub, double *distortion_out, void *ws,
                                hipStream_t s);

int device_cu_count();

// Diagnostic switch `key` (an otf_debug_key, set through otf_debug_set), else `fallback`.
int tune_int(int key, int fallback);

}  // namespace otf
