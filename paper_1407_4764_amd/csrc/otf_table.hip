// Byte-indexed table scans: product-quantised codes and binary codes.
//
// PQ (paper Sec. 3, "Product quantization (PQ)"; Table 2: one byte per sub-block): the score of
// a coded row is sum_m lut[m][code_m] with lut[m][k] = <w_m, centre_k of sub-block m>.
// Binary (paper Sec. 3, "Binarization", Eq. (1)): the score is sum_d w_d (2 bit_d - 1).  Eight
// consecutive dimensions form one byte g of the row, so with the table
//     T[g][v] = sum_{j<8} (bit j of v ? +w[8g+j] : -w[8g+j])
// the score is sum_g T[g][byte_g]: the same scan as PQ with M = D/8 "sub-blocks".  One table
// lookup replaces eight signed adds, which keeps the scan below the vector-ALU ceiling.
//
// Both scans are one shared-memory gather per stored byte.  To keep the gathers free of bank
// conflicts whatever the data, the table is stored value-major, image[v][column], so that the
// bank of an access depends only on WHICH byte of the row is looked up, never on its value,
// and lanes that execute the same instruction always look up different columns:
//   * a row segment of 128 bytes is read by 8 lanes x 16 bytes (one 16-byte load per lane);
//   * byte (dword tq, byte b) of lane-chunk c lives in column 32*tq + 4*c + b;
//   * the four 128-byte segments handled by lanes 0..31 (and 32..63) read their dwords with
//     four different byte rotations (b = tb ^ (segment & 3)), so at every step the 32 lanes
//     touch columns 4*c + b with all 32 (c, b) pairs distinct: 32 lanes, 32 banks.
// Rows shorter than 128 bytes are packed several to a segment (the table columns repeat);
// rows longer than 128 bytes are processed in `nsplit` phases of 128 columns, the workgroup
// reloading the table image between phases and carrying partial sums in the score array.
#include "otf_internal.h"

namespace otf {

constexpr int kSegBytes = 128;                       // row bytes handled per phase
constexpr int kImageFloats = 256 * kSegBytes;        // one table image: 256 values x 128 columns
constexpr int kImageBytes = kImageFloats * 4;        // 128 KiB
constexpr int kScanMaxThreads = 1024;
constexpr int kScanThreads = 512;

__device__ __forceinline__ int image_column(int pos) {   // pos = byte position inside a 128-byte segment
    const int c = pos >> 4, tq = (pos >> 2) & 3, b = pos & 3;
    return 32 * tq + 4 * c + b;
}

// lut[m][k] = sum_j w[m*dsub + j] * codebooks[m][k][j]
__global__ __launch_bounds__(256) void pq_build_lut_kernel(const float *__restrict__ codebooks, int M, int K, int dsub,
                                                           const float *__restrict__ w, float *__restrict__ lut) {
    const long long total = (long long)M * K;
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (long long)gridDim.x * blockDim.x) {
        const int m = (int)(t / K);
        const float *c = codebooks + t * dsub;
        const float *wm = w + (long long)m * dsub;
        float acc = 0.f;
        for (int j = 0; j < dsub; ++j) acc = fmaf(wm[j], c[j], acc);
        lut[t] = acc;
    }
}

// Table images for PQ: image[sp][v][column(pos)] = lut[m][v],  m = sp*128 + pos (M >= 128) or
// pos mod M (M < 128).  Also zeroes the selection state (one launch instead of two).
__global__ __launch_bounds__(256) void pq_prepare_kernel(const float *__restrict__ lut, int M, int nsplit,
                                                         float *__restrict__ image, SelState *st, uint32_t *hist1,
                                                         uint32_t *hist2) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, step = gridDim.x * blockDim.x;
    for (int t = tid; t < nsplit * kImageFloats; t += step) {
        const int v = t & 255, pos = (t >> 8) & (kSegBytes - 1), sp = t >> 15;
        const int m = (M >= kSegBytes) ? sp * kSegBytes + pos : pos % M;
        image[(size_t)sp * kImageFloats + v * kSegBytes + image_column(pos)] = lut[(size_t)m * 256 + v];
    }
    uint32_t *stw = reinterpret_cast<uint32_t *>(st);
    for (int i = tid; i < (int)(sizeof(SelState) / 4); i += step) stw[i] = 0u;
    for (int i = tid; i < kBins1; i += step) hist1[i] = 0u;
    for (int i = tid; i < kBins2; i += step) hist2[i] = 0u;
}

// Table images for binary codes: byte g of a row covers dimensions 8g..8g+7, bit j = dim 8g+j.
__global__ __launch_bounds__(256) void binary_prepare_kernel(const float *__restrict__ w, int row_bytes, int nsplit,
                                                             float *__restrict__ image, SelState *st, uint32_t *hist1,
                                                             uint32_t *hist2) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, step = gridDim.x * blockDim.x;
    for (int t = tid; t < nsplit * kImageFloats; t += step) {
        const int v = t & 255, pos = (t >> 8) & (kSegBytes - 1), sp = t >> 15;
        const int g = (row_bytes >= kSegBytes) ? sp * kSegBytes + pos : pos % row_bytes;
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float wd = w[g * 8 + j];
            acc += ((v >> j) & 1) ? wd : -wd;
        }
        image[(size_t)sp * kImageFloats + v * kSegBytes + image_column(pos)] = acc;
    }
    uint32_t *stw = reinterpret_cast<uint32_t *>(st);
    for (int i = tid; i < (int)(sizeof(SelState) / 4); i += step) stw[i] = 0u;
    for (int i = tid; i < kBins1; i += step) hist1[i] = 0u;
    for (int i = tid; i < kBins2; i += step) hist2[i] = 0u;
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over groups of LPR adjacent lanes (LPR = 1, 2, 4 or 8); every lane of a group receives it.
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
    if (LPR >= 2) v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
    if (LPR >= 4) v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
    if (LPR >= 8) v += dpp_move<0x141>(v);   // row_half_mirror: lane i <-> 7 - i of each 8
    return v;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Scan.  LPR = lanes per stored row within one phase = min(M, 128) / 16;  U = 16-byte loads per
// lane per tile;  SPLIT = rows longer than 128 bytes (several phases, partial sums carried in
// the score array).
//
// The main loop is branch-free and software-pipelined: the loads of the wave's next tile are
// issued before the current tile is looked up, and tiles or rows past the end are redirected
// to the block's last row rather than skipped (an unconditional load keeps the in-order wait
// counters exact).  After the lookups the U row sums of a lane group are moved into U different
// lanes so that storing, histogramming and (SPLIT) carrying happen once per tile, not per row.
template <int LPR, int U, bool SPLIT, int MODE = 0>
__global__ __launch_bounds__(kScanMaxThreads) void table_scan_kernel(const uint8_t *__restrict__ codes, long long N,
                                                                  int M, int nsplit,
                                                                  const float *__restrict__ image, float bias,
                                                                  float *__restrict__ scores, SelState *st,
                                                                  uint32_t *hist1, int k) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    float *table = reinterpret_cast<float *>(lds_raw);          // kImageFloats
    __shared__ uint32_t lhist[kBins1];
    __shared__ uint32_t s_flag;
    constexpr int RPW = 64 / LPR;                // rows per wave load
    constexpr int TILE = RPW * U;                // rows per wave iteration
    constexpr int ACTIVE = LPR < U ? LPR : U;    // lanes of a group that own an output row per round
    constexpr int ROUNDS = U / ACTIVE;           // output rounds per tile

    for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int c = lane & 7;                      // 16-byte chunk inside the 128-byte segment
    const int seg = lane >> 3;                   // segment inside the wave load
    const int sub = lane % LPR, rr = lane / LPR; // chunk inside the row, row inside the wave load
    uint32_t shift[4], colbyte[4];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        const int b = tb ^ (seg & 3);
        shift[tb] = 8u * (uint32_t)b;
        colbyte[tb] = 4u * (uint32_t)(4 * c + b);
    }

    // this block's rows: a contiguous range, a multiple of 1024 rows long (TILE divides 1024, so
    // only the last block of the grid can end in a partial tile)
    long long per = (N + gridDim.x - 1) / gridDim.x;
    per = (per + 1023) / 1024 * 1024;
    long long begin = per * blockIdx.x, end = begin + per;
    if (begin > N) begin = N;
    if (end > N) end = N;
    const long long nfull = (end - begin) / TILE;          // full tiles
    const int rem = (int)((end - begin) % TILE);           // rows of the partial tile, if any
    const size_t tile_bytes = (size_t)TILE * (size_t)M;
    const size_t u_bytes = (size_t)RPW * (size_t)M;        // distance between the U loads of a lane
    const int out_u = sub % ACTIVE;                        // which of a round's rows this lane stores

    auto lookup16 = [&](const u32x4 &d) {
        if (MODE == 1) return __uint_as_float((d[0] ^ d[1] ^ d[2] ^ d[3]) & 0x3fffffffu);
        uint32_t addr[16];
#pragma unroll
        for (int tq = 0; tq < 4; ++tq)
#pragma unroll
            for (int tb = 0; tb < 4; ++tb)
                addr[4 * tq + tb] = (__builtin_amdgcn_ubfe(d[tq], shift[tb], 8u) << 9) + colbyte[tb];
        float t[16];
#pragma unroll
        for (int tq = 0; tq < 4; ++tq)
#pragma unroll
            for (int tb = 0; tb < 4; ++tb)
                t[4 * tq + tb] = *reinterpret_cast<const float *>(lds_raw + addr[4 * tq + tb] + 128 * tq);
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] += t[i + 8];
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] += t[i + 4];
        return group_sum<LPR>((t[0] + t[1]) + (t[2] + t[3]));
    };

    for (int sp = 0; sp < nsplit; ++sp) {
        __syncthreads();                          // previous phase done with the table
        {
            const u32x4 *src = reinterpret_cast<const u32x4 *>(image + (size_t)sp * kImageFloats);
            u32x4 *dst = reinterpret_cast<u32x4 *>(table);
            for (int i = threadIdx.x; i < kImageFloats / 4; i += blockDim.x) dst[i] = src[i];
        }
        __syncthreads();
        const bool first = sp == 0, lastp = sp == nsplit - 1;
        // lane's address in tile 0 of the block: row (begin + rr), this phase's columns
        const uint8_t *lane_codes = codes + (size_t)(begin + rr) * (size_t)M + (size_t)sp * kSegBytes + (size_t)sub * 16;
        // first row this lane stores in tile 0 (round 0)
        float *lane_scores = scores + begin + (long long)out_u * RPW + rr;

        // one output round: the U row sums of a lane group go to U different lanes, which store
        auto emit = [&](const float *s, const float *carry, float *dst, int e, bool ok) {
            float mine = s[e * ACTIVE];
#pragma unroll
            for (int a = 1; a < ACTIVE; ++a) mine = out_u == a ? s[e * ACTIVE + a] : mine;
            if (sub < ACTIVE && ok) {
                if (SPLIT && !first) mine += carry[e];
                if (lastp) {
                    mine += bias;
                    atomicAdd(&lhist[float_to_key(mine) >> 20], 1u);
                }
                *dst = mine;
            }
        };

        if (wave < nfull) {                       // uniform per wave
            auto fetch = [&](u32x4 *d, float *carry, long long tile) {
                if (tile > nfull - 1) tile = nfull - 1;      // uniform: prefetch past the end re-reads the last tile
                if (MODE == 2 && tile >= 2 * nwaves) return;
                const uint8_t *p = lane_codes + (size_t)tile * tile_bytes;
#pragma unroll
                for (int u = 0; u < U; ++u)
                    d[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + (size_t)u * u_bytes));
                if (SPLIT) {
                    const float *q = lane_scores + tile * TILE;
#pragma unroll
                    for (int e = 0; e < ROUNDS; ++e) carry[e] = q[e * ACTIVE * RPW];
                }
            };
            auto consume = [&](const u32x4 *d, const float *carry, long long tile) {
                float s[U];
#pragma unroll
                for (int u = 0; u < U; ++u) s[u] = lookup16(d[u]);
                float *q = lane_scores + tile * TILE;
#pragma unroll
                for (int e = 0; e < ROUNDS; ++e) emit(s, carry, q + e * ACTIVE * RPW, e, true);
            };
            u32x4 da[U], db[U];
            float ca[ROUNDS], cb[ROUNDS];
            fetch(da, ca, wave);
            for (long long tile = wave; tile < nfull; tile += 2 * nwaves) {
                fetch(db, cb, tile + nwaves);
                consume(da, ca, tile);
                fetch(da, ca, tile + 2 * nwaves);
                if (tile + nwaves < nfull) consume(db, cb, tile + nwaves);
            }
        }
        if (rem > 0 && wave == (int)(nfull % nwaves)) {   // the partial tile: same steps, row-checked
            const long long row0 = begin + nfull * TILE;
            u32x4 d[U];
            float carry[ROUNDS], s[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long long row = row0 + (long long)u * RPW + rr;
                d[u] = (u32x4){0u, 0u, 0u, 0u};
                if (row < end)
                    d[u] = *reinterpret_cast<const u32x4 *>(codes + (size_t)row * (size_t)M + (size_t)sp * kSegBytes +
                                                            (size_t)sub * 16);
            }
#pragma unroll
            for (int e = 0; e < ROUNDS; ++e) {
                const long long row = row0 + (long long)(e * ACTIVE + out_u) * RPW + rr;
                carry[e] = (SPLIT && !first && row < end) ? scores[row] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) s[u] = lookup16(d[u]);
#pragma unroll
            for (int e = 0; e < ROUNDS; ++e) {
                const long long row = row0 + (long long)(e * ACTIVE + out_u) * RPW + rr;
                emit(s, carry, scores + row, e, row < end);
            }
        }
    }
    finish_pass1(lhist, hist1, st, (uint32_t)k, gridDim.x, &s_flag);
}

hipError_t launch_pq_build_lut(const float *codebooks, int M, int K, int dsub, const float *w, float *lut,
                               hipStream_t s) {
    long long total = (long long)M * K;
    int blocks = (int)std::min<long long>((total + 255) / 256, 4096);
    pq_build_lut_kernel<<<blocks, 256, 0, s>>>(codebooks, M, K, dsub, w, lut);
    return hipGetLastError();
}

static int splits_of(int row_bytes) { return row_bytes >= kSegBytes ? row_bytes / kSegBytes : 1; }

hipError_t launch_pq_prepare(const float *lut, int M, float *image, const SelectWs &sw, hipStream_t s) {
    const int nsplit = splits_of(M);
    pq_prepare_kernel<<<nsplit * 32, 256, 0, s>>>(lut, M, nsplit, image, sw.st, sw.hist1, sw.hist2);
    return hipGetLastError();
}

hipError_t launch_binary_prepare(const float *w, int D, float *image, const SelectWs &sw, hipStream_t s) {
    const int row_bytes = D / 8, nsplit = splits_of(row_bytes);
    binary_prepare_kernel<<<nsplit * 32, 256, 0, s>>>(w, row_bytes, nsplit, image, sw.st, sw.hist1, sw.hist2);
    return hipGetLastError();
}

template <int LPR, int U, bool SPLIT, int MODE = 0>
static hipError_t launch_scan_cfg(const uint8_t *codes, int64_t N, int M, int nsplit, const float *image, float bias,
                                  float *scores, SelState *st, uint32_t *hist1, int k, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&table_scan_kernel<LPR, U, SPLIT, MODE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kImageBytes);
    if (e != hipSuccess) return e;
    int grid = device_cu_count();
    const int64_t max_useful = (N + 1023) / 1024;
    if (grid > max_useful) grid = (int)max_useful;
    if (grid < 1) grid = 1;
    const int threads = tune_int("OTF_SCAN_THREADS", kScanThreads);
    table_scan_kernel<LPR, U, SPLIT, MODE><<<grid, threads, kImageBytes, s>>>(codes, (long long)N, M, nsplit, image, bias,
                                                                        scores, st, hist1, k);
    return hipGetLastError();
}

template <int LPR>
static hipError_t launch_scan_lpr(const uint8_t *codes, int64_t N, int M, int nsplit, const float *image, float bias,
                                  float *scores, SelState *st, uint32_t *hist1, int k, hipStream_t s) {
    const int u = tune_int("OTF_SCAN_UNROLL", 8);
    const int mode = tune_int("OTF_SCAN_MODE", 0);
    if (LPR == 8 && mode == 1) return launch_scan_cfg<LPR, 4, false, 1>(codes, N, M, 1, image, bias, scores, st, hist1, k, s);
    if (LPR == 8 && mode == 2) return launch_scan_cfg<LPR, 4, false, 2>(codes, N, M, 1, image, bias, scores, st, hist1, k, s);
    if (nsplit > 1) {
        if (u == 8) return launch_scan_cfg<LPR, 8, true>(codes, N, M, nsplit, image, bias, scores, st, hist1, k, s);
        return launch_scan_cfg<LPR, 4, true>(codes, N, M, nsplit, image, bias, scores, st, hist1, k, s);
    }
    if (u == 8) return launch_scan_cfg<LPR, 8, false>(codes, N, M, nsplit, image, bias, scores, st, hist1, k, s);
    return launch_scan_cfg<LPR, 4, false>(codes, N, M, nsplit, image, bias, scores, st, hist1, k, s);
}

// M = stored bytes per row: 16, 32, 64 or a multiple of 128.
hipError_t launch_table_scan(const uint8_t *codes, int64_t N, int M, const float *image, float bias, float *scores,
                             SelState *st, uint32_t *hist1, int k, hipStream_t s) {
    const int nsplit = splits_of(M);
    switch (M) {
        case 16: return launch_scan_lpr<1>(codes, N, M, nsplit, image, bias, scores, st, hist1, k, s);
        case 32: return launch_scan_lpr<2>(codes, N, M, nsplit, image, bias, scores, st, hist1, k, s);
        case 64: return launch_scan_lpr<4>(codes, N, M, nsplit, image, bias, scores, st, hist1, k, s);
        default: return launch_scan_lpr<8>(codes, N, M, nsplit, image, bias, scores, st, hist1, k, s);
    }
}

}  // namespace otf
