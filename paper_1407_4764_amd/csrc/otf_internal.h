// Host-side declarations shared by the translation units of libotf.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "otf_device.h"

namespace otf {

// Where the selection state of the Q classifiers lives inside the workspace.
struct SelectWs {
    SelState *st;              // [Q]
    uint32_t *hist1;           // [Q][kBins1]
    uint32_t *hist2;           // [Q][kBins2]
    uint32_t *blockhist3;      // [Q][kSelBlocks][kBins3]
    uint32_t *eqoff;           // [Q][kSelBlocks]
    unsigned long long *cand;  // [Q][kCandCap]   (key << 32 | ~index)
};

struct WsLayout {
    size_t st, hist1, hist2, blockhist3, eqoff, cand, lut_image, scores, total;
};
// Byte offsets of the workspace regions for N rows and Q classifiers (every offset 256-aligned).
WsLayout ws_layout(int64_t N, int32_t Q);
SelectWs select_ws(void *ws, const WsLayout &L);

constexpr int kDenseMaxD = 16384;  // widest dense row any kernel takes (elements)
constexpr size_t kLutImageBytes = 8u * 128u * 1024u;  // up to 8 splits of a 256 x 128 fp32 table

// Zeroes the selection state and the pass-1/2 histograms of Q classifiers.
hipError_t launch_select_init(const SelectWs &sw, int Q, hipStream_t s);
// Radix pass 1 over ready-made scores (rows of length N, stride ld).
hipError_t launch_hist1(const float *scores, int64_t N, int64_t ld, int Q, int k, const SelectWs &sw, hipStream_t s);
// Passes 2 and 3 (skipped on the device when pass 1 was decisive), gather and final sort.
hipError_t launch_select_tail(const float *scores, int64_t N, int64_t ld, int Q, int k, const SelectWs &sw,
                              float *out_scores, int32_t *out_idx, hipStream_t s);

// Dense single-classifier scan: writes N scores (bias included) and builds the pass-1 histogram.
hipError_t launch_dense_scan(const void *X, int x_is_half, int64_t N, int D, int64_t ldx,
                             const void *w, int w_is_half, const float *bias_ptr, int bias_index,
                             float *scores, SelState *st, uint32_t *hist1, int k, hipStream_t s);

// Multi-classifier fp16 scan on the matrix cores: scores[q][i], row stride lds_.  No histogram.
hipError_t launch_dense_mfma(const void *X, int64_t N, int D, int64_t ldx, const void *W, int Q,
                             const float *bias, float *scores, int64_t ld_scores, hipStream_t s);

// Byte-indexed table scans (product-quantised codes, binary codes).
hipError_t launch_pq_build_lut(const float *codebooks, int M, int K, int dsub, const float *w, float *lut, hipStream_t s);
hipError_t launch_pq_prepare(const float *lut, int M, float *image, const SelectWs &sw, hipStream_t s);
hipError_t launch_binary_prepare(const float *w, int D, float *image, const SelectWs &sw, hipStream_t s);
hipError_t launch_table_scan(const uint8_t *codes, int64_t N, int M, const float *image, float bias,
                             float *scores, SelState *st, uint32_t *hist1, int k, hipStream_t s);

hipError_t launch_sgd_step(float *w, float *b, int D, const float *Xpos, int64_t ld_pos, const int32_t *idx_pos,
                           int n_pos, const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int n_neg,
                           float lambda, int64_t t, int update_bias, float *coef, hipStream_t s);

int device_cu_count();

// Launch-shape knobs for tuning runs: integer environment variable `name`, else `fallback`.
int tune_int(const char *name, int fallback);

}  // namespace otf
