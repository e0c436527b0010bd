// Dense scan with many classifiers at once: S = W X^T, fp16 inputs, fp32 accumulation, on the
// matrix cores.  (Paper Sec. 2.1: one linear SVM per class ranks all images; with several
// classifiers live at once the scoring of Sec. 4 "Ranking" becomes a matrix product.)
// 64 flop per streamed byte keeps it HBM-bound, so the aim is again to stream X once.
//
// Workgroup = 4 waves, tile = 128 dataset rows x QT*32 classifiers, K consumed 128 at a time.
// X and W tiles go global -> registers -> shared memory (rows padded by 16 bytes so that the
// 16-byte fragment reads of 8 consecutive lanes cover all 32 banks); the next tile's global
// loads are issued before the matrix instructions of the current one.  Each wave owns 32 rows:
// fragment A = 8 halves of a dataset row, fragment B = 8 halves of a classifier row, both from
// the same K slots, fed to v_mfma_f32_32x32x16_f16.
#include <hip/hip_fp16.h>

#include <algorithm>

#include "otf_internal.h"

namespace otf {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 128;                 // dataset rows per tile
constexpr int kBK = 128;                 // K elements (halves) per step
constexpr int kRowStride = kBK * 2 + 16; // bytes per tile row in shared memory

// EMIT (ScanEmit): all scores; the scores of the strided sample (compact row numbering, N = number
// of sample rows); or only the rows at or above each classifier's threshold, appended to its list.
template <int QT, int EMIT>
__global__ __launch_bounds__(256) void dense_mfma_kernel(const uint8_t *__restrict__ X, long long N, int D,
                                                         long long row_bytes, const uint8_t *__restrict__ W,
                                                         const float *__restrict__ bias, float *__restrict__ scores,
                                                         long long ld_scores, int vec_store,
                                                         const SelState *__restrict__ tau_state, SelState *st,
                                                         unsigned long long *__restrict__ cand, const SelState *gate) {
    constexpr int QN = QT * 32;
    if (gate && gate->fallback == 0u) return;     // uniform: only the fallback of a filtered scan
    __shared__ __attribute__((aligned(16))) uint8_t xs[kBM * kRowStride];
    __shared__ __attribute__((aligned(16))) uint8_t ws[QN * kRowStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const long long ntiles = (N + kBM - 1) / kBM;
    const int ksteps = D / kBK;
    const size_t w_row_bytes = (size_t)D * 2;

    float bq[QT];
    uint32_t tau[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        bq[qt] = bias ? bias[qt * 32 + n] : 0.f;
        tau[qt] = EMIT == kEmitFilter ? tau_state[qt * 32 + n].tau_key : 0u;
    }

    for (long long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const long long row0 = tile * kBM;
        float16v acc[QT];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[qt][v] = 0.f;

        // global -> register staging: X 8 chunks, W QT*2 chunks of 16 bytes per thread
        u32x4 xr[8], wr[QT * 2];
        const uint8_t *xsrc[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int id = tid + 256 * u;
            long long row = row0 + (id >> 4);
            if (row >= N) row = N - 1;               // clamp: rows past the end are computed, never stored
            if (EMIT == kEmitSample)                 // compact sample row -> store row
                row = (row >> 10) * ((long long)kSampleGroup * kSampleStride) + (row & 1023);
            xsrc[u] = X + (size_t)row * row_bytes + (size_t)(id & 15) * 16;
        }
        auto load_step = [&](int ks) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
                xr[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(xsrc[u] + (size_t)ks * (kBK * 2)));
#pragma unroll
            for (int u = 0; u < QT * 2; ++u) {
                const int id = tid + 256 * u;
                wr[u] = *reinterpret_cast<const u32x4 *>(W + (size_t)(id >> 4) * w_row_bytes + (size_t)ks * (kBK * 2) +
                                                         (size_t)(id & 15) * 16);
            }
        };
        load_step(0);
        for (int ks = 0; ks < ksteps; ++ks) {
            __syncthreads();                          // everyone has finished reading the previous tiles
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int id = tid + 256 * u;
                *reinterpret_cast<u32x4 *>(xs + (id >> 4) * kRowStride + (id & 15) * 16) = xr[u];
            }
#pragma unroll
            for (int u = 0; u < QT * 2; ++u) {
                const int id = tid + 256 * u;
                *reinterpret_cast<u32x4 *>(ws + (id >> 4) * kRowStride + (id & 15) * 16) = wr[u];
            }
            __syncthreads();
            if (ks + 1 < ksteps) load_step(ks + 1);   // in flight while the matrix cores work
            const uint8_t *arow = xs + (wave * 32 + n) * kRowStride + h * 16;
#pragma unroll
            for (int s = 0; s < kBK / 16; ++s) {
                const half8 a = *reinterpret_cast<const half8 *>(arow + s * 32);
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    const half8 b = *reinterpret_cast<const half8 *>(ws + (qt * 32 + n) * kRowStride + h * 16 + s * 32);
                    acc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[qt], 0, 0, 0);
                }
            }
        }
        // accumulator element v of lane (n, h): dataset row 8*(v/4) + 4*h + v%4 of the wave's 32,
        // classifier n of the tile's 32
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            float *dst = scores + (size_t)(qt * 32 + n) * ld_scores;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const long long row = row0 + wave * 32 + 8 * g + 4 * h;
                float o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) o[j] = acc[qt][4 * g + j] + bq[qt];
                if (EMIT == kEmitFilter) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t key = float_to_key(o[j]);
                        if (key >= tau[qt] && row + j < N) {
                            const int q = qt * 32 + n;
                            const uint32_t pos = atomicAdd(&st[q].cursor, 1u);
                            if (pos < (uint32_t)kCandCap)
                                cand[(size_t)q * kCandCap + pos] = ((unsigned long long)key << 32) |
                                                                   (unsigned long long)(0xFFFFFFFFu - (uint32_t)(row + j));
                        }
                    }
                } else if (vec_store && row + 3 < N) {
                    *reinterpret_cast<float4 *>(dst + row) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (row + j < N) dst[row + j] = o[j];
                }
            }
        }
    }
}

template <int QT>
static hipError_t launch_mfma_qt(const uint8_t *X, int64_t N, int D, int64_t ldx, const uint8_t *W, const float *bias,
                                 ScanEmit emit, float *scores, int64_t ld_scores, const SelState *tau, SelState *st,
                                 unsigned long long *cand, const SelState *gate, hipStream_t s) {
    const int64_t ntiles = (N + kBM - 1) / kBM;
    const int grid = (int)std::min<int64_t>(ntiles, (int64_t)device_cu_count() * tune_int("OTF_MFMA_BLOCKS_PER_CU", 2));
    const int vec_store = scores && (ld_scores % 4 == 0) && ((reinterpret_cast<uintptr_t>(scores) & 15) == 0);
#define OTF_MFMA_ARGS X, (long long)N, D, (long long)ldx * 2, W, bias, scores, (long long)ld_scores, vec_store, tau, st, cand, gate
    if (emit == kEmitScores) dense_mfma_kernel<QT, kEmitScores><<<grid, 256, 0, s>>>(OTF_MFMA_ARGS);
    else if (emit == kEmitSample) dense_mfma_kernel<QT, kEmitSample><<<grid, 256, 0, s>>>(OTF_MFMA_ARGS);
    else dense_mfma_kernel<QT, kEmitFilter><<<grid, 256, 0, s>>>(OTF_MFMA_ARGS);
#undef OTF_MFMA_ARGS
    return hipGetLastError();
}

// Q must be 32 or 64, D a multiple of 128, N >= 1 (for kEmitSample: N = sample rows, a multiple of 1024).
// tau, st and cand point at the first of the Q classifiers of this call.
hipError_t launch_dense_mfma(const void *X, int64_t N, int D, int64_t ldx, const void *W, int Q, const float *bias,
                             ScanEmit emit, float *scores, int64_t ld_scores, const SelState *tau, SelState *st,
                             unsigned long long *cand, const SelState *gate, hipStream_t s) {
    const uint8_t *Xb = reinterpret_cast<const uint8_t *>(X);
    const uint8_t *Wb = reinterpret_cast<const uint8_t *>(W);
    if (Q == 32) return launch_mfma_qt<1>(Xb, N, D, ldx, Wb, bias, emit, scores, ld_scores, tau, st, cand, gate, s);
    if (Q == 64) return launch_mfma_qt<2>(Xb, N, D, ldx, Wb, bias, emit, scores, ld_scores, tau, st, cand, gate, s);
    return hipErrorInvalidValue;
}

}  // namespace otf
