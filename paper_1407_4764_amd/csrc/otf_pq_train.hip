// Product-quantisation encoder and one Lloyd iteration of its vocabulary training (paper Sec. 3,
// "Product quantization (PQ)": every sub-block of a feature is replaced by the index of the nearest
// of the K = 256 cluster centres of that sub-block's own vocabulary, the centres having been learned
// from a training set).
//
// Nearest centre of sub-vector x among c_0..c_255: argmin_k ||x||^2/2 - <x, c_k> + ||c_k||^2/2, the lowest k
// among equals.  For 32 rows and 32 centres that is one v_mfma_f32_32x32x2_f32 chain of dsub/2 + 1
// steps (the last step adds the two norms), so an encoding pass is an N x 256 x (dsub + 2) product
// per sub-block on the matrix cores, and what remains for the vector ALU is the argmin: a running
// minimum per lane over the 8 blocks of 32 centres, then one reduction over the 32 lanes that hold
// the candidates of a row.
#include <algorithm>

#include "otf_internal.h"

namespace otf {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPqK = 256;

// Minimum over each half-wave (lanes 0..31, lanes 32..63); every lane receives it.
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
    return __builtin_amdgcn_mov_dpp(v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ int half_min_i32(int v) {
    v = min(v, dpp_i32<0xB1>(v));
    v = min(v, dpp_i32<0x4E>(v));
    v = min(v, dpp_i32<0x141>(v));
    v = min(v, dpp_i32<0x140>(v));
    return min(v, __builtin_amdgcn_ds_swizzle(v, 0x401F));
}

// norms[m][k] = ||codebooks[m][k]||^2
__global__ __launch_bounds__(256) void pq_centre_norms_kernel(const float *__restrict__ codebooks, int M, int dsub,
                                                              float *__restrict__ norms) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= M * kPqK) return;
    const float *c = codebooks + (size_t)t * dsub;
    float s = 0.f;
    for (int j = 0; j < dsub; ++j) s = fmaf(c[j], c[j], s);
    norms[t] = s;
}

// Encoding.  A workgroup of four waves takes 256 rows (64 per wave, two 32-row halves) through all
// M sub-blocks; the vocabulary of the current sub-block sits in shared memory (double-buffered, one
// barrier per sub-block), rows padded by 16 bytes so that the operand reads of 8 consecutive lanes
// fall into different banks.  Operand layout: lane (r, h) holds, for row r of a half (operand A) or
// centre r of a block of 32 (operand B), the components h * dsub/2 .. (h+1) * dsub/2 - 1: A and B
// only have to agree on which component goes into which K slot.
template <int DSUB>
__global__ __launch_bounds__(256, 3) void pq_encode_kernel(const float *__restrict__ X, long long N, long long ldx,
                                                           const float *__restrict__ codebooks, const float *__restrict__ norms,
                                                           int M, int mr, uint8_t *__restrict__ codes) {
    constexpr int HALF = DSUB / 2;                         // components per lane = MFMA steps per chain
    constexpr int STRIDE = DSUB * 4 + (DSUB == 4 ? 32 : 16);   // bytes per centre in shared memory (see above)
    constexpr int VEC = DSUB * 4 / 16;                     // 16-byte pieces per centre
    __shared__ __attribute__((aligned(16))) uint8_t cs[2][kPqK * STRIDE];
    __shared__ float ns[2][kPqK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const long long ntiles = (N + 255) / 256;

    f32x4 stage[VEC];
    float nstage;
    auto load_c = [&](int m) {                             // one centre per thread
        const float *src = codebooks + ((size_t)m * kPqK + tid) * DSUB;
#pragma unroll
        for (int v = 0; v < VEC; ++v) stage[v] = *reinterpret_cast<const f32x4 *>(src + 4 * v);
        nstage = norms[(size_t)m * kPqK + tid];
    };
    auto store_c = [&](int buf) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) *reinterpret_cast<f32x4 *>(cs[buf] + tid * STRIDE + 16 * v) = stage[v];
        ns[buf][tid] = nstage;
    };

    // Work unit = (tile of 256 rows, range of `mr` sub-blocks): the codes of different sub-blocks are
    // independent, and units a fraction of a tile long let the last round of the grid end together
    // (whole tiles: 5.09 tiles per workgroup slot at 1M rows means six rounds for five rounds' work).
    const int ranges = (M + mr - 1) / mr;
    for (long long unit = blockIdx.x; unit < ntiles * ranges; unit += gridDim.x) {
        const long long tile = unit / ranges;
        const int m_begin = (int)(unit % ranges) * mr, m_end = m_begin + mr < M ? m_begin + mr : M;
        const long long row0 = tile * 256 + (long long)wave * 64;
        const float *xrow[2];
#pragma unroll
        for (int f = 0; f < 2; ++f) {
            long long row = row0 + 32 * f + r;
            if (row > N - 1) row = N - 1;                  // computed, never stored
            xrow[f] = X + (size_t)row * ldx + h * HALF;
        }
        const long long myrow = row0 + lane;               // the row whose codes this lane writes
        uint32_t packed = 0u;                              // codes of up to four consecutive sub-blocks of myrow

        float anext[2][HALF];
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int s = 0; s < HALF; ++s) anext[f][s] = xrow[f][(size_t)m_begin * DSUB + s];
        __syncthreads();                                   // the previous unit is done with shared memory
        load_c(m_begin);
        store_c(m_begin & 1);
        __syncthreads();
        for (int m = m_begin; m < m_end; ++m) {
            const int buf = m & 1;
            if (m + 1 < m_end) load_c(m + 1);              // uniform; in flight during the matrix instructions
            // Operand A carries the negated components, and one more K step carries the two norms:
            // its slot of the h = 0 lanes multiplies ||x||^2 / 2 by 1, that of the h = 1 lanes 1 by
            // ||c||^2 / 2.  The accumulators then hold half the squared distances themselves.
            float a[2][HALF], ax[2];
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                float ss = 0.f;
#pragma unroll
                for (int s = 0; s < HALF; ++s) {
                    const float t = anext[f][s];
                    a[f][s] = -t;
                    ss = fmaf(t, t, ss);
                }
                const float other = __shfl_xor(ss, 32, 64);    // the other half of the row's components
                ax[f] = h == 0 ? 0.5f * (ss + other) : 1.0f;
            }
            {                                              // the next sub-block's components (the last one re-reads)
                const int mn = m + 1 < m_end ? m + 1 : m;
#pragma unroll
                for (int f = 0; f < 2; ++f)
#pragma unroll
                    for (int s = 0; s < HALF; ++s) anext[f][s] = xrow[f][(size_t)mn * DSUB + s];
            }

            // Running minimum per lane over the 8 blocks of 32 centres, two ALU instructions per value:
            // the block number replaces the three lowest mantissa bits of the (non-negative) value and
            // the minimum is taken on the bit patterns, so the lower block wins among equal values.
            int best[2][16];
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int v = 0; v < 16; ++v) best[f][v] = 0x7FFFFFFF;
#pragma unroll 1
            for (int cb = 0; cb < kPqK / 32; ++cb) {
                float b[HALF];
                const float *bp = reinterpret_cast<const float *>(cs[buf] + (32 * cb + r) * STRIDE) + h * HALF;
#pragma unroll
                for (int s = 0; s < HALF; ++s) b[s] = bp[s];
                const float bx = h == 0 ? 1.0f : 0.5f * ns[buf][32 * cb + r];
                float16v acc[2];
#pragma unroll
                for (int f = 0; f < 2; ++f)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[f][v] = 0.f;
#pragma unroll
                for (int s = 0; s < HALF; ++s)
#pragma unroll
                    for (int f = 0; f < 2; ++f) acc[f] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[f][s], b[s], acc[f], 0, 0, 0);
#pragma unroll
                for (int f = 0; f < 2; ++f) acc[f] = __builtin_amdgcn_mfma_f32_32x32x2f32(ax[f], bx, acc[f], 0, 0, 0);
                // accumulator element v of lane (r, h): row 8 (v / 4) + 4 h + v % 4 of the half, centre 32 cb + r
#pragma unroll
                for (int f = 0; f < 2; ++f)
#pragma unroll
                    for (int v = 0; v < 16; ++v) best[f][v] = min(best[f][v], (__float_as_int(acc[f][v]) & ~7) | cb);
            }
            // The 32 lanes of a half-wave hold 32 candidates of the same row: minimum of the keys (four
            // cross-lane steps inside the vector ALU, one swizzle across the two 16-lane rows); it names
            // the block, and the lowest lane that holds it names the centre inside the block.
            int code = 0;
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int kmin = half_min_i32(best[f][v]);
                    const unsigned long long vote = __ballot(best[f][v] == kmin);
                    const int k0 = 32 * (__builtin_amdgcn_readlane(kmin, 0) & 7) + __builtin_ctz((uint32_t)vote);
                    const int k1 = 32 * (__builtin_amdgcn_readlane(kmin, 32) & 7) + __builtin_ctz((uint32_t)(vote >> 32));
                    const int rr = 8 * (v / 4) + (v % 4);      // row of lanes 0..31 (h = 0); lanes 32..63: rr + 4
                    if (lane == 32 * f + rr) code = k0;
                    if (lane == 32 * f + rr + 4) code = k1;
                }
            packed |= (uint32_t)code << (8 * (m & 3));
            if ((m & 3) == 3 || m == m_end - 1) {          // uniform (ranges begin at multiples of 4)
                if (myrow < N) {
                    uint8_t *dst = codes + (size_t)myrow * M + (m & ~3);
                    if ((m & 3) == 3) *reinterpret_cast<uint32_t *>(dst) = packed;
                    else
                        for (int j = 0; j <= (m & 3); ++j) dst[j] = (uint8_t)(packed >> (8 * j));
                }
                packed = 0u;
            }
            if (m + 1 < m_end) store_c(buf ^ 1);           // last read of that buffer: sub-block m - 1, a barrier ago
            __syncthreads();
        }
    }
}

// Lloyd iteration, second half: per-centre sums of the assigned sub-vectors, counts, and the
// distortion.  One workgroup per (sub-block, slice of rows); sums in shared memory, merged into
// global memory by atomics at the end.
template <int DSUB>
__global__ __launch_bounds__(256) void pq_accumulate_kernel(const float *__restrict__ X, long long N, long long ldx,
                                                            const float *__restrict__ codebooks,
                                                            const uint8_t *__restrict__ codes, int M, float *sums,
                                                            uint32_t *counts, double *distortion) {
    __shared__ float lsum[kPqK * DSUB];
    __shared__ uint32_t lcnt[kPqK];
    __shared__ double ldist[4];
    const int m = blockIdx.y, tid = threadIdx.x;
    for (int i = tid; i < kPqK * DSUB; i += 256) lsum[i] = 0.f;
    for (int i = tid; i < kPqK; i += 256) lcnt[i] = 0u;
    __syncthreads();
    const long long per = (N + gridDim.x - 1) / gridDim.x;
    const long long begin = per * blockIdx.x, end = begin + per < N ? begin + per : N;
    double dist = 0.0;
    for (long long i = begin + tid; i < end; i += 256) {
        const int k = codes[(size_t)i * M + m];
        const float *x = X + (size_t)i * ldx + (size_t)m * DSUB;
        const float *c = codebooks + ((size_t)m * kPqK + k) * DSUB;
        float d = 0.f;
#pragma unroll
        for (int j = 0; j < DSUB; ++j) {
            const float xv = x[j], t = xv - c[j];
            d = fmaf(t, t, d);
            atomicAdd(&lsum[k * DSUB + j], xv);
        }
        atomicAdd(&lcnt[k], 1u);
        dist += (double)d;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) dist += __shfl_xor(dist, o, 64);
    if ((tid & 63) == 0) ldist[tid >> 6] = dist;
    __syncthreads();
    for (int i = tid; i < kPqK * DSUB; i += 256)
        if (lsum[i] != 0.f) atomicAdd(&sums[(size_t)m * kPqK * DSUB + i], lsum[i]);
    for (int i = tid; i < kPqK; i += 256)
        if (lcnt[i]) atomicAdd(&counts[(size_t)m * kPqK + i], lcnt[i]);
    if (tid == 0) atomicAdd(distortion, ldist[0] + ldist[1] + ldist[2] + ldist[3]);
}

__global__ __launch_bounds__(256) void pq_zero_kernel(float *sums, uint32_t *counts, double *distortion, int M, int dsub) {
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < (size_t)M * kPqK * dsub) sums[t] = 0.f;
    if (t < (size_t)M * kPqK) counts[t] = 0u;
    if (t == 0) *distortion = 0.0;
}

// centre <- mean of its cell; a centre with an empty cell stays.  Also publishes the distortion
// (mean over rows of the summed squared distances to the assigned centres).
__global__ __launch_bounds__(256) void pq_move_centres_kernel(float *codebooks, const float *sums, const uint32_t *counts,
                                                              int M, int dsub, const double *distortion, long long N,
                                                              double *distortion_out) {
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < (size_t)M * kPqK * dsub) {
        const uint32_t n = counts[t / dsub];
        if (n) codebooks[t] = sums[t] / (float)n;
    }
    if (t == 0 && distortion_out) *distortion_out = *distortion / (double)N;
}

struct PqTrainWs {
    float *norms, *sums;
    uint32_t *counts;
    double *distortion;
};

size_t pq_train_ws_bytes(int M, int dsub) {
    return 256 + (size_t)M * kPqK * 4 + (size_t)M * kPqK * dsub * 4 + (size_t)M * kPqK * 4;
}

static PqTrainWs pq_train_ws(void *ws, int M, int dsub) {
    uint8_t *p = reinterpret_cast<uint8_t *>(ws);
    PqTrainWs w;
    w.distortion = reinterpret_cast<double *>(p);
    w.norms = reinterpret_cast<float *>(p + 256);
    w.sums = w.norms + (size_t)M * kPqK;
    w.counts = reinterpret_cast<uint32_t *>(w.sums + (size_t)M * kPqK * dsub);
    return w;
}

hipError_t launch_pq_encode(const float *X, int64_t N, int64_t ldx, const float *codebooks, int M, int dsub,
                            uint8_t *codes, void *ws, hipStream_t s) {
    PqTrainWs w = pq_train_ws(ws, M, dsub);
    pq_centre_norms_kernel<<<(M * kPqK + 255) / 256, 256, 0, s>>>(codebooks, M, dsub, w.norms);
    const int64_t ntiles = (N + 255) / 256;
    const int mr = std::min(M, std::max(4, tune_int("OTF_PQENC_RANGE", 16) & ~3));   // sub-blocks per work unit, a multiple of 4
    const int64_t units = ntiles * ((M + mr - 1) / mr);
    const int grid = (int)std::min<int64_t>(units, (int64_t)device_cu_count() * tune_int("OTF_PQENC_BLOCKS_PER_CU", 3));
    switch (dsub) {
        case 4: pq_encode_kernel<4><<<grid, 256, 0, s>>>(X, (long long)N, (long long)ldx, codebooks, w.norms, M, mr, codes); break;
        case 8: pq_encode_kernel<8><<<grid, 256, 0, s>>>(X, (long long)N, (long long)ldx, codebooks, w.norms, M, mr, codes); break;
        case 16: pq_encode_kernel<16><<<grid, 256, 0, s>>>(X, (long long)N, (long long)ldx, codebooks, w.norms, M, mr, codes); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_pq_lloyd_step(const float *X, int64_t N, int64_t ldx, float *codebooks, int M, int dsub,
                                uint8_t *codes, double *distortion_out, void *ws, hipStream_t s) {
    hipError_t e = launch_pq_encode(X, N, ldx, codebooks, M, dsub, codes, ws, s);
    if (e != hipSuccess) return e;
    PqTrainWs w = pq_train_ws(ws, M, dsub);
    const size_t cells = (size_t)M * kPqK * dsub;
    pq_zero_kernel<<<(unsigned)((cells + 255) / 256), 256, 0, s>>>(w.sums, w.counts, w.distortion, M, dsub);
    int slices = (int)std::min<int64_t>((N + 4095) / 4096, std::max(1, device_cu_count() * 8 / M));
    if (slices < 1) slices = 1;
    dim3 grid(slices, M);
    switch (dsub) {
        case 4: pq_accumulate_kernel<4><<<grid, 256, 0, s>>>(X, (long long)N, (long long)ldx, codebooks, codes, M, w.sums, w.counts, w.distortion); break;
        case 8: pq_accumulate_kernel<8><<<grid, 256, 0, s>>>(X, (long long)N, (long long)ldx, codebooks, codes, M, w.sums, w.counts, w.distortion); break;
        case 16: pq_accumulate_kernel<16><<<grid, 256, 0, s>>>(X, (long long)N, (long long)ldx, codebooks, codes, M, w.sums, w.counts, w.distortion); break;
        default: return hipErrorInvalidValue;
    }
    pq_move_centres_kernel<<<(unsigned)((cells + 255) / 256), 256, 0, s>>>(codebooks, w.sums, w.counts, M, dsub, w.distortion,
                                                                            (long long)N, distortion_out);
    return hipGetLastError();
}

}  // namespace otf
