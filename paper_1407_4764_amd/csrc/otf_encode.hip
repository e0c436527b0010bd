// Binarisation encoder (paper Sec. 3, "Binarization", Eq. (1)): a zero-centred descriptor phi in
// R^m becomes the code beta = sgn(U phi) in {0,1}^n, n > m, sgn(a) = 1 iff a > 0, where the frame U
// is the first m columns of the orthogonal factor of a QR decomposition of a random n x n matrix.
//
// tight_frame_kernel     U from the random matrix (set-up, once per frame)
// binarize_bf16_kernel   the codes of N descriptors: an N x n x m matrix product on the matrix
//                        cores at fp32 accuracy (three exact bf16 pieces per value, fp32
//                        accumulation) whose epilogue keeps only the signs, packed 32 to a word,
//                        dimension d at bit d mod 32 of word d div 32
// binarize_kernel        the same product on the fp32 matrix instructions; 1.6 times slower (they do
//                        not overlap with the vector ALU on this chip), kept behind the
//                        switch OTF_DEBUG_BINARIZE_FP32 for comparison
#include <algorithm>

#include "otf_bf16x3.h"
#include "otf_internal.h"

namespace otf {


// -------------------------------------------------------------------------------------------
// U = first m columns of Q, G = QR with a positive diagonal of R.  Those columns depend on the
// first m columns of G only: they are their Gram-Schmidt orthonormalisation.  One workgroup,
// fp64, every column orthogonalised twice against its predecessors ("twice is enough": the
// result is orthonormal to rounding whatever the conditioning of the random columns).
//   G  n x n fp32 row-major.   Qd  n x m fp64 scratch, row-major.   U  n x m fp32 row-major.
constexpr int kFrameThreads = 1024;
constexpr int kFrameMaxN = 4096;     // v (fp64) lives in shared memory
constexpr int kFrameMaxM = 256;

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__global__ __launch_bounds__(kFrameThreads) void tight_frame_kernel(const float *__restrict__ G, int n, int m,
                                                                    double *__restrict__ Qd, float *__restrict__ U) {
    __shared__ double v[kFrameMaxN];
    __shared__ double coef[kFrameMaxM];
    __shared__ double part[kFrameThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = kFrameThreads / 64;
    for (int j = 0; j < m; ++j) {
        // norm of the column as given: what is left after orthogonalisation counts as zero when it is
        // rounding noise relative to this (a column in the span of its predecessors leaves ~1e-16 of
        // its length, not exactly 0)
        double s0 = 0.0;
        for (int i = tid; i < n; i += kFrameThreads) {
            const double g = (double)G[(size_t)i * n + j];
            v[i] = g;
            s0 += g * g;
        }
        s0 = wave_sum_f64(s0);
        if (lane == 0) part[wave] = s0;
        __syncthreads();
        double norm0_2 = 0.0;
        for (int w = 0; w < nwaves; ++w) norm0_2 += part[w];
        __syncthreads();
        for (int pass = 0; pass < 2; ++pass) {
            // coef[c] = <q_c, v> for c < j: one wave per column c
            for (int c = wave; c < j; c += nwaves) {
                double s = 0.0;
                for (int i = lane; i < n; i += 64) s += Qd[(size_t)i * m + c] * v[i];
                s = wave_sum_f64(s);
                if (lane == 0) coef[c] = s;
            }
            __syncthreads();
            // v -= sum_c coef[c] q_c: one thread per row
            for (int i = tid; i < n; i += kFrameThreads) {
                const double *q = Qd + (size_t)i * m;
                double s = 0.0;
                for (int c = 0; c < j; ++c) s += coef[c] * q[c];
                v[i] -= s;
            }
            __syncthreads();
        }
        double s = 0.0;
        for (int i = tid; i < n; i += kFrameThreads) s += v[i] * v[i];
        s = wave_sum_f64(s);
        if (lane == 0) part[wave] = s;
        __syncthreads();
        double norm2 = 0.0;
        for (int w = 0; w < nwaves; ++w) norm2 += part[w];
        const double tol = (double)n * 2.220446049250313e-16;
        const double inv = norm2 > tol * tol * norm0_2 ? 1.0 / sqrt(norm2) : 0.0;   // dependent columns give a zero column
        for (int i = tid; i < n; i += kFrameThreads) {
            const double q = v[i] * inv;
            Qd[(size_t)i * m + j] = q;
            U[(size_t)i * m + j] = (float)q;
        }
        __threadfence_block();
        __syncthreads();
    }
}

// -------------------------------------------------------------------------------------------
// Codes, fp32 matrix instructions.  2 m n flop per descriptor against 4 m + n/8 bytes: at m = 128,
// n = 2048 that is 680 flop per byte, so the kernel is bound by the rate of the matrix cores and is
// organised to keep them issuing: one workgroup of eight waves per compute unit, two waves per SIMD.
//
//   * A wave owns 32 descriptors for the whole of U.  Their values stay in registers for that
//     time, already in the operand layout of v_mfma_f32_32x32x2_f32 (lane (r, h) = descriptor r,
//     K slots 64 h .. 64 h + 63: operands A and B only have to agree on which K goes into which
//     slot, so each lane takes a contiguous half row instead of every other element).
//   * U is streamed from L2 in blocks of 32 frame rows (= 32 code bits) through shared memory,
//     double-buffered, one barrier per block; rows padded by 16 bytes so that the 16-byte
//     operand reads of 8 consecutive lanes cover all 32 banks.
//   * Per block the signs come out as 16 wave votes (v_cmp + the vote mask): lanes 0..31 of vote v
//     are the 32 bits of one output word, lanes 32..63 those of another.  The words are parked in
//     lane (block mod 64) of one register per descriptor, and once 64 blocks are done every
//     descriptor's 256 bytes leave in one coalesced store.
//   * A wave issues in order, so its votes, stores and barrier waits stall its own matrix
//     instructions; the second wave of the SIMD fills those gaps (74 % -> 78 % of peak against four
//     waves of 64 descriptors with the whole register file each).
constexpr int kEncRows = 256;                   // descriptors per workgroup pass
constexpr int kEncK = 128;                      // K slots (m is padded with zeros up to this)
constexpr int kEncStride = kEncK * 4 + 16;      // bytes per frame row in shared memory

// F = 32-row halves per wave (2: four waves, one per SIMD with the whole register file; 1: eight waves, two per
// SIMD, so that one wave's sign epilogue and barrier waits hide behind the other's matrix instructions)
template <int F>
__global__ __launch_bounds__(1024 / F / 2) void binarize_kernel(const float *__restrict__ phi, long long N, int m,
                                                                long long ld, const float *__restrict__ U, int n,
                                                                uint32_t *__restrict__ bits) {
    constexpr int kEncRowsPerWave = 32 * F;
    constexpr int THREADS = 1024 / F / 2;        // 256 or 512
    constexpr int UL = 1024 / THREADS;           // 16-byte pieces of a block of U per thread
    __shared__ __attribute__((aligned(16))) uint8_t us[2][32 * kEncStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int nblocks = n / 32;                  // blocks of 32 code bits
    const int words = n / 32;                    // words per code
    const long long ntiles = (N + kEncRows - 1) / kEncRows;

    // global -> registers -> shared memory for one block of U: 32 rows x 512 bytes, 4 x 16 bytes per thread
    f32x4 ustage[UL];
    auto load_u = [&](int cb) {
#pragma unroll
        for (int u = 0; u < UL; ++u) {
            const int id = tid + THREADS * u, row = id >> 5, c16 = id & 31;
            ustage[u] = (f32x4){0.f, 0.f, 0.f, 0.f};
            if (4 * c16 < m) ustage[u] = *reinterpret_cast<const f32x4 *>(U + (size_t)(32 * cb + row) * m + 4 * c16);
        }
    };
    auto store_u = [&](int buf) {
#pragma unroll
        for (int u = 0; u < UL; ++u) {
            const int id = tid + THREADS * u, row = id >> 5, c16 = id & 31;
            *reinterpret_cast<f32x4 *>(us[buf] + row * kEncStride + c16 * 16) = ustage[u];
        }
    };

    for (long long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const long long row0 = tile * kEncRows + (long long)wave * kEncRowsPerWave;
        // operand A: descriptor values of this lane's two rows, K slots 64 h + s
        float a[F][64];
#pragma unroll
        for (int f = 0; f < F; ++f) {
            long long row = row0 + 32 * f + r;
            if (row > N - 1) row = N - 1;                    // computed, never stored
            const float *p = phi + (size_t)row * ld + 64 * h;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                f32x4 t = (f32x4){0.f, 0.f, 0.f, 0.f};
                if (64 * h + 4 * q < m) t = *reinterpret_cast<const f32x4 *>(p + 4 * q);
                a[f][4 * q + 0] = t.x; a[f][4 * q + 1] = t.y; a[f][4 * q + 2] = t.z; a[f][4 * q + 3] = t.w;
            }
        }
        uint32_t outw[kEncRowsPerWave];                      // outw[row]: lane c holds word (64 * pass + c) of the row
#pragma unroll
        for (int i = 0; i < kEncRowsPerWave; ++i) outw[i] = 0u;

        __syncthreads();                                     // the previous tile is done with shared memory
        load_u(0);
        store_u(0);
        __syncthreads();
        for (int cb = 0; cb < nblocks; ++cb) {
            const int buf = cb & 1;
            if (cb + 1 < nblocks) load_u(cb + 1);            // uniform; in flight during the matrix instructions
            float16v acc[F];
#pragma unroll
            for (int f = 0; f < F; ++f)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[f][v] = 0.f;
            const uint8_t *brow = us[buf] + r * kEncStride + h * 256;
            f32x4 b = *reinterpret_cast<const f32x4 *>(brow);
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                f32x4 bn = b;
                if (q + 1 < 16) bn = *reinterpret_cast<const f32x4 *>(brow + (q + 1) * 16);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int f = 0; f < F; ++f)
                        acc[f] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[f][4 * q + j], b[j], acc[f], 0, 0, 0);
                b = bn;
            }
            // signs: accumulator element v of lane (r, h) is descriptor 8 (v / 4) + 4 h + v % 4 of the
            // half, code bit 32 cb + r
            const bool mine = lane == (cb & 63);             // the lane that keeps this block's words
#pragma unroll
            for (int f = 0; f < F; ++f)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const unsigned long long vote = __ballot(acc[f][v] > 0.f);
                    const int lo = 32 * f + 8 * (v / 4) + (v % 4);
                    outw[lo] = mine ? (uint32_t)vote : outw[lo];
                    outw[lo + 4] = mine ? (uint32_t)(vote >> 32) : outw[lo + 4];
                }
            if ((cb & 63) == 63 || cb == nblocks - 1) {      // uniform: 64 words per descriptor are complete
                const int w0 = cb & ~63;
#pragma unroll
                for (int i = 0; i < kEncRowsPerWave; ++i) {
                    const long long row = row0 + i;
                    if (row < N && w0 + lane < words) bits[(size_t)row * words + w0 + lane] = outw[i];
                    outw[i] = 0u;
                }
            }
            if (cb + 1 < nblocks) store_u(buf ^ 1);          // last read of that buffer: block cb - 1, a barrier ago
            __syncthreads();
        }
    }
}

// The same codes on the bf16 matrix instructions at fp32 accuracy (three exact pieces per value,
// see otf_bf16x3.h): 6 instructions of 32 cycles per 16 dimensions instead of 8 of 64, and the sign
// epilogue and the splitting of U run on the vector ALU beside them.
//
//   * A wave owns 32 descriptors for the whole of U; their pieces stay in registers (lane (r, h):
//     descriptor r, dimensions 16 q + 8 h .. + 7 of every chunk q of 16), 96 registers at m = 128.
//   * U is streamed in blocks of 32 frame rows; a thread takes 8 consecutive values of a row, splits
//     them and stores the three pieces as [piece][q][h][row] x 16 bytes, so the operand reads of
//     consecutive lanes are consecutive.  Double-buffered, one barrier per block.
//   * Two accumulator chains with their instructions interleaved keep the matrix pipe busy from one
//     wave; the sign is that of their sum.  Pairs of chunks at or beyond m are left out (template
//     argument).
constexpr int kBinStage = 3 * 8 * 2 * 32 * 16;   // bytes of one block of U in shared memory: 24576

template <int NQP, int WAVES>   // NQP = pairs of 16-dimension chunks in use: ceil(m / 32); WAVES per workgroup: 4 or 8
__global__ __launch_bounds__(64 * WAVES, 8 / WAVES) void binarize_bf16_kernel(const float *__restrict__ phi, long long N, int m,
                                                           long long ld, const float *__restrict__ U, int n,
                                                           uint32_t *__restrict__ bits) {
    __shared__ __attribute__((aligned(16))) uint8_t us[2][kBinStage];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int nblocks = n / 32;                  // blocks of 32 code bits
    const int words = n / 32;                    // words per code
    constexpr int ROWS = 32 * WAVES;             // descriptors per workgroup pass
    constexpr int UL = 8 / WAVES;                // 8-dimension pieces of a block of U per thread
    const long long ntiles = (N + ROWS - 1) / ROWS;

    // one block of U: thread = (row of the block, 8 consecutive dimensions), UL times
    const int urow = tid & 31, uc0 = tid >> 5;   // piece u: dimensions 8 uc .. 8 uc + 7 with uc = uc0 + 2 WAVES u (chunk uc / 2, half uc % 2)
    f32x4 ustage[UL][2];
    auto load_u = [&](int cb) {
#pragma unroll
        for (int u = 0; u < UL; ++u)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int uc8 = uc0 + 2 * WAVES * u;
                ustage[u][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
                if (8 * uc8 + 4 * j < m)
                    ustage[u][j] = *reinterpret_cast<const f32x4 *>(U + (size_t)(32 * cb + urow) * m + 8 * uc8 + 4 * j);
            }
    };
    auto store_u = [&](int buf) {
#pragma unroll
        for (int u = 0; u < UL; ++u) {
            const int uc8 = uc0 + 2 * WAVES * u;
            if (uc8 >= 4 * NQP) continue;        // a chunk nobody reads
            uint32_t pc[3][4];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                split3(ustage[u][j][0], ustage[u][j][1], pc[0][2 * j], pc[1][2 * j], pc[2][2 * j]);
                split3(ustage[u][j][2], ustage[u][j][3], pc[0][2 * j + 1], pc[1][2 * j + 1], pc[2][2 * j + 1]);
            }
#pragma unroll
            for (int p = 0; p < 3; ++p)
                *reinterpret_cast<u32x4 *>(us[buf] + (((p * 8 + (uc8 >> 1)) * 2 + (uc8 & 1)) * 32 + urow) * 16) =
                    u32x4{pc[p][0], pc[p][1], pc[p][2], pc[p][3]};
        }
    };

    for (long long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const long long row0 = tile * ROWS + (long long)wave * 32;
        // operand A: the pieces of this lane's descriptor values
        u32x4 xa[2 * NQP][3];
        {
            uint32_t xp[3][4];
            long long row = row0 + r;
            if (row > N - 1) row = N - 1;                    // computed, never stored
            const float *p = phi + (size_t)row * ld + 8 * h;
#pragma unroll
            for (int q = 0; q < 2 * NQP; ++q) {
                f32x4 t[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    t[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
                    if (16 * q + 8 * h + 4 * j < m) t[j] = *reinterpret_cast<const f32x4 *>(p + 16 * q + 4 * j);
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    split3(t[j][0], t[j][1], xp[0][2 * j], xp[1][2 * j], xp[2][2 * j]);
                    split3(t[j][2], t[j][3], xp[0][2 * j + 1], xp[1][2 * j + 1], xp[2][2 * j + 1]);
                }
#pragma unroll
                for (int p = 0; p < 3; ++p) xa[q][p] = u32x4{xp[p][0], xp[p][1], xp[p][2], xp[p][3]};
            }
        }
        uint32_t outw[32];                                   // outw[row]: lane c holds word (64 * pass + c) of the row
#pragma unroll
        for (int i = 0; i < 32; ++i) outw[i] = 0u;

        __syncthreads();                                     // the previous tile is done with shared memory
        load_u(0);
        store_u(0);
        __syncthreads();
        for (int cb = 0; cb < nblocks; ++cb) {
            const int buf = cb & 1;
            if (cb + 1 < nblocks) load_u(cb + 1);            // uniform; in flight during the matrix instructions
            float16v acc[2];
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[e][v] = 0.f;
            // chunks in pairs, one per accumulator chain, their instructions interleaved: consecutive
            // matrix instructions never wait for each other's result.  (The number of pairs is a
            // template argument: a run-time test here costs a copy of all accumulators per branch.)
#pragma unroll
            for (int q = 0; q < 2 * NQP; q += 2) {
                u32x4 cp[2][3];
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int p = 0; p < 3; ++p)
                        cp[e][p] = *reinterpret_cast<const u32x4 *>(us[buf] + (((p * 8 + q + e) * 2 + h) * 32 + r) * 16);
                // smallest terms first: (x2,c0) (x1,c1) (x0,c2) (x1,c0) (x0,c1) (x0,c0)
                constexpr int xi[6] = {2, 1, 0, 1, 0, 0}, ci[6] = {0, 1, 2, 0, 1, 0};
#pragma unroll
                for (int t = 0; t < 6; ++t) {
                    acc[0] = mfma_bf16(xa[q][xi[t]], cp[0][ci[t]], acc[0]);
                    acc[1] = mfma_bf16(xa[q + 1][xi[t]], cp[1][ci[t]], acc[1]);
                }
            }
            // signs: accumulator element v of lane (r, h) is descriptor 8 (v / 4) + 4 h + v % 4, code bit 32 cb + r
            const bool mine = lane == (cb & 63);             // the lane that keeps this block's words
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const unsigned long long vote = __ballot(acc[0][v] > -acc[1][v]);   // the sign of the sum, which is exact near zero
                const int lo = 8 * (v / 4) + (v % 4);
                outw[lo] = mine ? (uint32_t)vote : outw[lo];
                outw[lo + 4] = mine ? (uint32_t)(vote >> 32) : outw[lo + 4];
            }
            if ((cb & 63) == 63 || cb == nblocks - 1) {      // uniform: 64 words per descriptor are complete
                const int w0 = cb & ~63;
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    const long long row = row0 + i;
                    if (row < N && w0 + lane < words) bits[(size_t)row * words + w0 + lane] = outw[i];
                    outw[i] = 0u;
                }
            }
            if (cb + 1 < nblocks) store_u(buf ^ 1);          // last read of that buffer: block cb - 1, a barrier ago
            __syncthreads();
        }
    }
}

hipError_t launch_tight_frame(const float *G, int n, int m, double *scratch, float *U, hipStream_t s) {
    if (n > kFrameMaxN || m > kFrameMaxM) return hipErrorInvalidValue;
    tight_frame_kernel<<<1, kFrameThreads, 0, s>>>(G, n, m, scratch, U);
    return hipGetLastError();
}

hipError_t launch_binarize(const float *phi, int64_t N, int m, int64_t ld, const float *U, int n, uint32_t *bits,
                           hipStream_t s) {
    if (m > kEncK || m % 4 || n % 32) return hipErrorInvalidValue;
    const int64_t ntiles = (N + kEncRows - 1) / kEncRows;
    const int grid = (int)std::min<int64_t>(ntiles, device_cu_count());
    if (!tune_int(OTF_DEBUG_BINARIZE_FP32, 0)) {
        // Two workgroups of four waves per compute unit rather than one of eight: each has its own
        // barrier, so the two waves of a SIMD drift apart and one's matrix instructions run beside
        // the other's vector work.
        const bool four = tune_int(OTF_DEBUG_BINARIZE_WAVES, 4) == 4;
        const int64_t tiles = (N + (four ? 128 : 256) - 1) / (four ? 128 : 256);
        const int g = (int)std::min<int64_t>(tiles, (int64_t)device_cu_count() * (four ? 2 : 1));
#define OTF_BIN_LAUNCH(NQP)                                                                                     \
    if (four) binarize_bf16_kernel<NQP, 4><<<g, 256, 0, s>>>(phi, (long long)N, m, (long long)ld, U, n, bits); \
    else binarize_bf16_kernel<NQP, 8><<<g, 512, 0, s>>>(phi, (long long)N, m, (long long)ld, U, n, bits)
        switch ((m + 31) / 32) {
            case 1: OTF_BIN_LAUNCH(1); break;
            case 2: OTF_BIN_LAUNCH(2); break;
            case 3: OTF_BIN_LAUNCH(3); break;
            default: OTF_BIN_LAUNCH(4); break;
        }
#undef OTF_BIN_LAUNCH
    } else if (tune_int(OTF_DEBUG_BINARIZE_WAVES, 8) == 4)       // the fp32 matrix instructions, kept for comparison
        binarize_kernel<2><<<grid, 256, 0, s>>>(phi, (long long)N, m, (long long)ld, U, n, bits);
    else
        binarize_kernel<1><<<grid, 512, 0, s>>>(phi, (long long)N, m, (long long)ld, U, n, bits);
    return hipGetLastError();
}

}  // namespace otf
