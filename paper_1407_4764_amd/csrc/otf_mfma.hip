// Dense scan with many classifiers at once: S = W X^T, fp16 inputs, fp32 accumulation, on the
// matrix cores.  (Paper Sec. 2.1: one linear SVM per class ranks all images; with several
// classifiers live at once the scoring of Sec. 4 "Ranking" becomes a matrix product.)
// 64 flop per streamed byte keeps it HBM-bound, so the aim is again to stream X once.
//
// Workgroup = 4 waves, tile = 128 dataset rows x QT*32 classifiers, K consumed 128 at a time.
// X and W tiles go global -> registers -> shared memory (rows padded by 16 bytes so that the
// 16-byte fragment reads of 8 consecutive lanes cover all 32 banks); global loads run two K
// steps ahead of the matrix instructions through two register stages.  Each wave owns 32 rows:
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
__global__ __launch_bounds__(256, 2) void dense_mfma_kernel(const uint8_t *__restrict__ X, long long N, int D,
                                                         long long row_bytes, const uint8_t *__restrict__ W,
                                                         const float *__restrict__ bias, float *__restrict__ scores,
                                                         long long ld_scores, int vec_store,
                                                         const SelState *__restrict__ tau_state, SelState *st,
                                                         unsigned long long *__restrict__ cand, Gate gate,
                                                         uint32_t *tile_ctr) {
    constexpr int QN = QT * 32;
    // uniform: a gated full scan is only the fallback of a filtered one; a gated filtered scan was called off
    if (gate.st && (EMIT == kEmitFilter ? gate.st->fallback != 0u : !gate_open(gate))) return;
    __shared__ __attribute__((aligned(16))) uint8_t xs[kBM * kRowStride];
    __shared__ __attribute__((aligned(16))) uint8_t ws[QN * kRowStride];
    __shared__ uint32_t s_tile[8];                // ring: number of the block's j-th tile at slot j % 8
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

    // The (tile, K step) pairs of this block form one flat sequence.  Global loads run two steps
    // ahead of the matrix instructions through two register stages, across tile boundaries too,
    // so there is no cold start per tile (unconditional loads keep the in-order wait counters
    // exact; loads past the block's last tile re-read the store's last tile).
    //
    // Tiles are handed out dynamically, one atomic on a global counter per tile (a static split
    // leaves a tail: the chip's dies stream at different rates).  The number of the block's j-th
    // tile is ordered when the loads of its tile j - 3 begin, by thread 0, and the returned value is
    // written to the ring two steps later, right after the wait for the loads that were issued
    // behind the atomic, so that nobody ever waits for the atomic itself.
    // (A short scan -- fewer than 8 tiles per workgroup, e.g. the sample -- deals the tiles round-robin
    // instead: claiming three at a time would leave most workgroups without any.)
    const bool dynamic = ntiles >= 8LL * gridDim.x;
    if (tid == 0) {
        const uint32_t c = dynamic ? atomicAdd(tile_ctr, 3u) : 0u;
        s_tile[0] = dynamic ? c : blockIdx.x;
        s_tile[1] = dynamic ? c + 1u : blockIdx.x + gridDim.x;
        s_tile[2] = dynamic ? c + 2u : blockIdx.x + 2u * gridDim.x;
    }
    __syncthreads();
    if ((long long)s_tile[0] >= ntiles) return;   // uniform

    // load side
    uint32_t lj = 0u;                             // ordinal of the tile being loaded
    long long ltile = s_tile[0];
    // tiles start at different K steps (tile number mod steps: the order of the sum is a property
    // of the tile, whoever computes it), so that workgroups running in step do not ask the same
    // memory channels for the same slice of W and of their rows at the same time
    int lks = (int)(ltile % ksteps), lcount = 0;
    // addresses = uniform base of the tile (scalar registers) + 32-bit per-lane offsets
    const uint8_t *xbase;
    uint32_t xoff[8], woff[QT * 2];
#pragma unroll
    for (int u = 0; u < QT * 2; ++u)
        woff[u] = (uint32_t)((tid >> 4) + 16 * u) * (uint32_t)w_row_bytes + (uint32_t)(tid & 15) * 16u;
    auto point_at_tile = [&](long long tile) {
        long long row0 = tile * kBM;
        const long long last = N - 1 - row0;          // rows past the end are computed (clamped), never stored
        if (EMIT == kEmitSample)                      // compact sample row -> store row (tiles never straddle a group)
            row0 = (row0 >> 10) * ((long long)kSampleGroup * kSampleStride) + (row0 & 1023);
        xbase = X + (size_t)row0 * row_bytes;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            long long r = (tid >> 4) + 16 * u;
            if (r > last) r = last;
            xoff[u] = (uint32_t)r * (uint32_t)row_bytes + (uint32_t)(tid & 15) * 16u;
        }
    };
    point_at_tile(ltile);
    // piece p of 8: one X load, and one W load on the odd (QT = 2) or every fourth (QT = 1) piece
    auto issue_piece = [&](u32x4 *xr, u32x4 *wr, int p) {
        const uint8_t *xb = xbase + (size_t)lks * (kBK * 2);
        const uint8_t *wb = W + (size_t)lks * (kBK * 2);
        xr[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(xb + (size_t)xoff[p]));
        constexpr int every = 8 / (QT * 2);
        if (p % every == every - 1) wr[p / every] = *reinterpret_cast<const u32x4 *>(wb + (size_t)woff[p / every]);
    };
    // before the first load of a step: when the step starts the block's tile lj, order tile lj + 3
    auto begin_step = [&](uint32_t &pend, bool &has_pend, uint32_t &pend_slot) {
        if (lcount == 0) {                           // uniform
            if (tid == 0) pend = dynamic ? atomicAdd(tile_ctr, 1u) : blockIdx.x + (lj + 3u) * gridDim.x;
            has_pend = true;
            pend_slot = (lj + 3u) & 7u;
        }
    };
    auto advance_load = [&]() {
        if (++lks == ksteps) lks = 0;
        if (++lcount == ksteps) {                    // uniform
            lcount = 0;
            ++lj;
            ltile = s_tile[lj & 7u];
            if (ltile > ntiles - 1) ltile = ntiles - 1;   // nothing left: harmless re-read
            lks = (int)(ltile % ksteps);
            point_at_tile(ltile);
        }
    };
    auto issue_load = [&](u32x4 *xr, u32x4 *wr, uint32_t &pend, bool &has_pend, uint32_t &pend_slot) {
        begin_step(pend, has_pend, pend_slot);
#pragma unroll
        for (int p = 0; p < 8; ++p) issue_piece(xr, wr, p);
        advance_load();
    };

    // compute side
    uint32_t cj = 0u;
    long long ctile = s_tile[0];
    int cks = 0;
    float16v acc[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[qt][v] = 0.f;

    // Filtered scan: a wave stops appending to a classifier's list once it has seen that list full
    // (per lane: lane (n, h) only ever appends to classifiers n and n + 32).
    bool list_full[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) list_full[qt] = false;
    auto epilogue = [&](long long row0) {
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
                        if (key >= tau[qt] && row + j < N && !list_full[qt]) {
                            const int q = qt * 32 + n;
                            const uint32_t pos = atomicAdd(&st[q].cursor, 1u);
                            if (pos < (uint32_t)kCandCap)
                                cand[(size_t)q * kCandCap + pos] = ((unsigned long long)key << 32) |
                                                                   (unsigned long long)(0xFFFFFFFFu - (uint32_t)(row + j));
                            else
                                list_full[qt] = true;
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
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[qt][v] = 0.f;
        }
    };

    // one step (after the block's last tile a step works on re-read rows and stores nothing)
    auto body = [&](u32x4 *xr, u32x4 *wr, uint32_t &pend, bool &has_pend, uint32_t &pend_slot) {
        __syncthreads();                              // everyone has finished reading the previous tiles
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
        if (has_pend) {                               // uniform; the atomic is older than the loads just waited for
            if (tid == 0) s_tile[pend_slot] = pend;
            has_pend = false;
        }
        __syncthreads();
        begin_step(pend, has_pend, pend_slot);
        const uint8_t *arow = xs + (wave * 32 + n) * kRowStride + h * 16;
        const uint8_t *brow = ws + n * kRowStride + h * 16;
        {
            // global loads spread between the matrix instructions, fragments read one slot ahead
            half8 a = *reinterpret_cast<const half8 *>(arow), b[QT];
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) b[qt] = *reinterpret_cast<const half8 *>(brow + qt * 32 * kRowStride);
#pragma unroll
            for (int s = 0; s < kBK / 16; ++s) {
                half8 an = a, bn[QT];
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) bn[qt] = b[qt];
                if (s + 1 < kBK / 16) {
                    an = *reinterpret_cast<const half8 *>(arow + (s + 1) * 32);
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt)
                        bn[qt] = *reinterpret_cast<const half8 *>(brow + qt * 32 * kRowStride + (s + 1) * 32);
                }
                issue_piece(xr, wr, s);
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) acc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b[qt], acc[qt], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                a = an;
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) b[qt] = bn[qt];
            }
            advance_load();
        }
        if (++cks == ksteps) {                        // uniform: the tile is complete
            if (ctile < ntiles) {
                epilogue(ctile * kBM);
                ++cj;
                ctile = s_tile[cj & 7u];
            }
            cks = 0;
        }
    };

    u32x4 xr0[8], wr0[QT * 2], xr1[8], wr1[QT * 2];
    uint32_t pend0 = 0u, pend1 = 0u, slot0 = 0u, slot1 = 0u;
    bool has0 = false, has1 = false;
    issue_load(xr0, wr0, pend0, has0, slot0);
    issue_load(xr1, wr1, pend1, has1, slot1);
    // One exit, after the pair: a way out (or back to the loop header) from the middle would make
    // the header see either stage as the younger one and wait for both.  When the last tile ends
    // on the first step of a pair, the second one runs idle.
    do {
        body(xr0, wr0, pend0, has0, slot0);
        body(xr1, wr1, pend1, has1, slot1);
    } while (ctile < ntiles);
}

template <int QT>
static hipError_t launch_mfma_qt(const uint8_t *X, int64_t N, int D, int64_t ldx, const uint8_t *W, const float *bias,
                                 ScanEmit emit, float *scores, int64_t ld_scores, const SelState *tau, SelState *st,
                                 unsigned long long *cand, Gate gate, uint32_t *tile_ctr, hipStream_t s) {
    const int64_t ntiles = (N + kBM - 1) / kBM;
    const int grid = (int)std::min<int64_t>(ntiles, (int64_t)device_cu_count() * tune_int(OTF_DEBUG_MFMA_BLOCKS_PER_CU, 2));
    const int vec_store = scores && (ld_scores % 4 == 0) && ((reinterpret_cast<uintptr_t>(scores) & 15) == 0);
#define OTF_MFMA_ARGS X, (long long)N, D, (long long)ldx * 2, W, bias, scores, (long long)ld_scores, vec_store, tau, st, cand, gate, tile_ctr
    if (emit == kEmitScores) dense_mfma_kernel<QT, kEmitScores><<<grid, 256, 0, s>>>(OTF_MFMA_ARGS);
    else if (emit == kEmitSample) dense_mfma_kernel<QT, kEmitSample><<<grid, 256, 0, s>>>(OTF_MFMA_ARGS);
    else dense_mfma_kernel<QT, kEmitFilter><<<grid, 256, 0, s>>>(OTF_MFMA_ARGS);
#undef OTF_MFMA_ARGS
    return hipGetLastError();
}

// Q must be 32 or 64, D a multiple of 128, N >= 1 (for kEmitSample: N = sample rows, a multiple of 1024).
// tau, st and cand point at the first of the Q classifiers of this call; tile_ctr at a zeroed word.
hipError_t launch_dense_mfma(const void *X, int64_t N, int D, int64_t ldx, const void *W, int Q, const float *bias,
                             ScanEmit emit, float *scores, int64_t ld_scores, const SelState *tau, SelState *st,
                             unsigned long long *cand, Gate gate, uint32_t *tile_ctr, hipStream_t s) {
    const uint8_t *Xb = reinterpret_cast<const uint8_t *>(X);
    const uint8_t *Wb = reinterpret_cast<const uint8_t *>(W);
    if (Q == 32) return launch_mfma_qt<1>(Xb, N, D, ldx, Wb, bias, emit, scores, ld_scores, tau, st, cand, gate, tile_ctr, s);
    if (Q == 64) return launch_mfma_qt<2>(Xb, N, D, ldx, Wb, bias, emit, scores, ld_scores, tau, st, cand, gate, tile_ctr, s);
    return hipErrorInvalidValue;
}

}  // namespace otf
