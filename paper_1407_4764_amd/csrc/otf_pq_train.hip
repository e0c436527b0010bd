// Product-quantisation encoder and one Lloyd iteration of its vocabulary training (paper Sec. 3,
// "Product quantization (PQ)": every sub-block of a feature is replaced by the index of the nearest
// of the K = 256 cluster centres of that sub-block's own vocabulary, the centres having been learned
// from a training set).
//
// Nearest centre of sub-vector x among c_0..c_255: argmin_k ||x||^2/2 - <x, c_k> + ||c_k||^2/2, the lowest k
// among equals.  For 32 rows and 32 centres that is one chain of matrix instructions whose last
// step adds the two norms, so an encoding pass is an N x 256 x (dsub + 2) product per sub-block on
// the matrix cores, and what remains for the vector ALU is the argmin: a running minimum per lane
// over the 8 blocks of 32 centres, then one reduction over the 32 lanes that hold the candidates of
// a row.
//
// pq_encode_bf16_kernel   bf16 matrix instructions on three exact pieces per fp32 value
// pq_encode_kernel        the fp32 matrix instructions (switch OTF_DEBUG_PQENC_FP32), kept for comparison
// pq_accumulate_kernel, pq_move_centres_kernel   the second half of a Lloyd iteration
#include <algorithm>
#include <type_traits>

#include "otf_bf16x3.h"
#include "otf_internal.h"

namespace otf {

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

// End of a sub-block: `best[f][v]` of lane (r, h) is the smallest key (half the squared distance
// with the number of the block of 32 centres in its three lowest bits) seen in column r of the
// blocks for row 8 (v / 4) + 4 h + v % 4 of half f.  The 32 lanes of a half-wave hold 32 candidates
// of the same row: minimum of the keys (four cross-lane steps inside the vector ALU, one swizzle
// across the two 16-lane rows); it names the block, and the lowest lane that holds it names the
// centre inside the block.  Returns the code of row `lane` of the wave's 64 rows.
__device__ __forceinline__ int code_from_minima(const int (&best)[2][16], int lane) {
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
    return code;
}

// The same end of a sub-block for pq_encode_bf16_kernel, at half the instructions: a reduce-scatter.
// Lane r of a half-wave holds candidates of 32 rows (registers j = 16 f + v) for one centre of the
// block; five exchange steps, one per lane bit, each halve the registers a lane keeps while merging
// in the partner's candidates for them, and leave lane r with the winner of row j = r.  A candidate
// is (key, centre within the block).  Centres sit in the lanes bit-reversed (lane bit 4 = centre
// bit 0, ...), and the lane bits are taken from 4 down to 0, i.e. the centre bits from the lowest up:
// at every step the two candidates agree in all higher centre bits, so among equal keys the one
// from the side whose bit is 0 is the lower centre, whatever the bits below.
// Returns the code of row 32 (r >> 4) + 8 ((r & 15) >> 2) + 4 h + (r & 3) of the wave's 64 rows.
__device__ __forceinline__ int rs_row_of_lane(int lane) {
    const int r = lane & 31, h = lane >> 5;
    return 32 * (r >> 4) + 8 * ((r & 15) >> 2) + 4 * h + (r & 3);
}

template <int PAIRS, int BIT, typename Partner>
__device__ __forceinline__ void rs_step(int (&k)[16], int (&i)[16], int lane, Partner partner) {
    const bool up = (lane & BIT) != 0;                     // this lane keeps the upper register of a pair
    const int tie = up ? 1 : 0;                            // ... and then the partner's side has the lower centre
#pragma unroll
    for (int j = 0; j < PAIRS; ++j) {
        const int keep_k = up ? k[j + PAIRS] : k[j], give_k = up ? k[j] : k[j + PAIRS];
        const int keep_i = up ? i[j + PAIRS] : i[j], give_i = up ? i[j] : i[j + PAIRS];
        const int got_k = partner(give_k), got_i = partner(give_i);
        const bool take = got_k < keep_k + tie;
        k[j] = min(keep_k, got_k);
        i[j] = take ? got_i : keep_i;
    }
}

__device__ __forceinline__ int code_by_reduce_scatter(const int (&best)[2][16], int lane) {
    const int c = (int)(__brev((uint32_t)(lane & 31)) >> 27);   // this lane's centre within a block
    const int c_lo = c & ~1, c_hi = c | 1;
    int k[16], i[16];
    // lane bit 4 (partner lane ^ 16): v_permlane16_swap exchanges the odd 16-lane rows of its first
    // operand with the even rows of its second; afterwards the first holds, in every lane, the
    // candidate of the side with lane bit 4 = 0 and the second that of the other side, both for
    // the register this lane keeps (f = lane bit 4).
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const auto sw = __builtin_amdgcn_permlane16_swap((uint32_t)best[0][v], (uint32_t)best[1][v], false, false);
        const int d = (int)sw[0], e = (int)sw[1];
        k[v] = min(d, e);
        i[v] = e < d ? c_hi : c_lo;
    }
    rs_step<8, 8>(k, i, lane, [](int x) { return dpp_i32<0x128>(x); });                    // row_ror:8 = lane ^ 8
    rs_step<4, 4>(k, i, lane, [](int x) { return dpp_i32<0x1B>(dpp_i32<0x141>(x)); });     // half mirror, then quad reversed = lane ^ 4
    rs_step<2, 2>(k, i, lane, [](int x) { return dpp_i32<0x4E>(x); });                     // lane ^ 2
    rs_step<1, 1>(k, i, lane, [](int x) { return dpp_i32<0xB1>(x); });                     // lane ^ 1
    return 32 * (k[0] & 7) + i[0];
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
            const int code = code_from_minima(best, lane);
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

// The encoder on the bf16 matrix instructions, at fp32 accuracy (three exact pieces per value, see
// otf_bf16x3.h).  For dsub = 16 a block of 32 rows x 32 centres takes 6 + 1 instructions of 32 cycles
// instead of 9 of 64 (dsub = 8: 4 instead of 5, dsub = 4: 2 instead of 3), and the argmin on the
// vector ALU proceeds meanwhile.
//
// Shared memory per sub-block: the image described below, 26 KB, double-buffered, three workgroups
// per CU; lane (r, h) reads the operand of centre slot 32 cb + r, consecutive lanes consecutive
// 16 bytes.
//
// Which piece products go into which matrix instruction.  One instruction has 16 K slots = 16 / DSUB
// "places" of DSUB dimensions; lane (r, h) supplies K slots 8 h .. 8 h + 7.
//   DSUB = 16: one place.  Six instructions, one product each: operand A = piece kA[t] of x,
//              operand B = piece kB[t] of c (three B entries per centre in the image); a seventh adds
//              the norms: A = [nx0 nx1 nx2 1 1 1 0 0 | 0 ..], B = [1 1 1 nc0 nc1 nc2 0 0 | ..] with
//              nx = ||x||^2 / 2, nc = ||c||^2 / 2 in three pieces each.
//   DSUB = 8:  two places, the lanes h = 0 and h = 1.  Three instructions, two products each, plus
//              the norm instruction.
//   DSUB = 4:  four places, two per lane.  Two instructions: four products, then two products and
//              the norm operand in the h = 1 lanes.
// Smallest products first.  The image holds per centre slot the B operand of every instruction (for
// DSUB = 16 the three pieces), as [entry][h][slot] x 16 bytes, then (DSUB = 16, 8) two dwords of the
// norm operand per slot; the centres negated, so that the products sum to -<x, c>.  Built once per
// call, so the encoder only copies it.
template <int DSUB>
struct Bf16Plan;
template <>
struct Bf16Plan<16> {
    static constexpr int kEntries = 3, kProducts = 6;
    static constexpr bool kNormInstr = true;
    static constexpr int kA[6] = {2, 1, 0, 1, 0, 0}, kB[6] = {0, 1, 2, 0, 1, 0};
};
template <>
struct Bf16Plan<8> {
    static constexpr int kEntries = 3, kProducts = 3;
    static constexpr bool kNormInstr = true;
    static constexpr int kA[3] = {0, 1, 2}, kB[3] = {0, 1, 2};
    // pieces (x, c) of instruction t in the lanes h = 0, 1
    static constexpr int kX[3][2] = {{2, 1}, {0, 1}, {0, 0}}, kC[3][2] = {{0, 1}, {2, 0}, {1, 0}};
};
template <>
struct Bf16Plan<4> {
    static constexpr int kEntries = 2, kProducts = 2;
    static constexpr bool kNormInstr = false;
    static constexpr int kA[2] = {0, 1}, kB[2] = {0, 1};
    // pieces (x, c) of instruction t in place 2 h + j; -1 = the norm operand (both places of the lane)
    static constexpr int kX[2][2][2] = {{{2, 1}, {0, 1}}, {{0, 0}, {-1, -1}}};
    static constexpr int kC[2][2][2] = {{{0, 1}, {2, 0}}, {{1, 0}, {-1, -1}}};
};
constexpr int kImgPieces = 3 * 2 * kPqK * 16;              // 24576 bytes (DSUB = 4 uses the first 16384)
constexpr int kImgBytes = kImgPieces + kPqK * 8;           // 26624 bytes per sub-block, whatever DSUB
constexpr uint32_t kBf16One = 0x3F80u;

// the norm operands from n = (half) a squared norm: [n0 n1 n2 1 1 1 0 0] and [1 1 1 n0 n1 n2 0 0]
__device__ __forceinline__ u32x4 norm_operand_a(float n) {
    uint32_t n0, n1, n2;
    split3(n, 0.f, n0, n1, n2);                            // low halves: the pieces
    return u32x4{(n0 & 0xFFFFu) | (n1 << 16), (n2 & 0xFFFFu) | (kBf16One << 16), kBf16One | (kBf16One << 16), 0u};
}
__device__ __forceinline__ u32x4 norm_operand_b(float n) {
    uint32_t n0, n1, n2;
    split3(n, 0.f, n0, n1, n2);
    return u32x4{kBf16One | (kBf16One << 16), kBf16One | (n0 << 16), (n1 & 0xFFFFu) | (n2 << 16), 0u};
}

template <int DSUB>
__global__ __launch_bounds__(256) void pq_centre_image_kernel(const float *__restrict__ codebooks, int M,
                                                              uint8_t *__restrict__ image, uint32_t *bound) {
    using P = Bf16Plan<DSUB>;
    const int m = blockIdx.x, k = threadIdx.x;
    if (m >= M) return;
    if (m == 0 && k == 0) *bound = 0u;                     // the encoder behind this kernel takes a maximum into it
    const float *c = codebooks + ((size_t)m * kPqK + k) * DSUB;
    uint8_t *img = image + (size_t)m * kImgBytes;
    const int slot = (k & ~31) | (int)(__brev((uint32_t)(k & 31)) >> 27);   // lane r of the encoder holds the centre with r's bits reversed
    uint32_t p[3][DSUB / 2];                               // [piece][pair of components]
    float nn = 0.f;
#pragma unroll
    for (int d = 0; d < DSUB / 2; ++d) {
        const float c0 = c[2 * d], c1 = c[2 * d + 1];
        nn = fmaf(c0, c0, fmaf(c1, c1, nn));
        split3(-c0, -c1, p[0][d], p[1][d], p[2][d]);       // negated: the products then sum to -<x, c>
    }
    const u32x4 nb = norm_operand_b(0.5f * nn);
#pragma unroll
    for (int t = 0; t < P::kEntries; ++t)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            u32x4 q;
            if constexpr (DSUB == 16) {
                q = u32x4{p[t][4 * hh], p[t][4 * hh + 1], p[t][4 * hh + 2], p[t][4 * hh + 3]};
            } else if constexpr (DSUB == 8) {
                const int pc = P::kC[t][hh];
                q = u32x4{p[pc][0], p[pc][1], p[pc][2], p[pc][3]};
            } else {
                const int pa = P::kC[t][hh][0], pb = P::kC[t][hh][1];
                q = pa < 0 ? nb : u32x4{p[pa][0], p[pa][1], p[pb][0], p[pb][1]};
            }
            *reinterpret_cast<u32x4 *>(img + ((t * 2 + hh) * kPqK + slot) * 16) = q;
        }
    if (P::kNormInstr) *reinterpret_cast<uint2 *>(img + kImgPieces + slot * 8) = make_uint2(nb[1], nb[2]);
}

template <int DSUB>
__global__ __launch_bounds__(256, 2) void pq_encode_bf16_kernel(const float *__restrict__ X, long long N, long long ldx,
                                                                const uint8_t *__restrict__ image, int M, int mr,
                                                                uint8_t *__restrict__ codes, uint32_t *bound) {
    using P = Bf16Plan<DSUB>;
    constexpr int NV = DSUB == 4 ? 1 : 2;                  // 16-byte loads of a row's components per lane and sub-block
    __shared__ __attribute__((aligned(16))) uint8_t img[2][kImgBytes];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const long long ntiles = (N + 255) / 256;
    float largest = 0.f;                                   // of the squared sub-vector norms this lane meets

    // The image of sub-block m goes from global memory straight into shared memory, 1 KB (64 lanes x
    // 16 bytes) per instruction, without passing through registers; it is complete once the wave's
    // outstanding loads have been waited for and the workgroup has met at a barrier.
    auto copy_image = [&](int m, int buf) {
        const uint8_t *src = image + (size_t)m * kImgBytes;
        for (int j = wave; j < kImgBytes / 1024; j += 4)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + j * 1024 + lane * 16),
                                             (__attribute__((address_space(3))) void *)(img[buf] + j * 1024), 16, 0, 0);
    };

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
            xrow[f] = X + (size_t)row * ldx + (DSUB == 16 ? h * 8 : 0);   // dsub 8, 4: both halves of the wave hold the whole sub-vector
        }
        const long long myrow = row0 + rs_row_of_lane(lane);   // the row whose codes this lane ends up with and writes
        uint32_t packed = 0u;                              // codes of up to four consecutive sub-blocks of myrow

        f32x4 anext[2][NV];
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int v = 0; v < NV; ++v) anext[f][v] = *reinterpret_cast<const f32x4 *>(xrow[f] + (size_t)m_begin * DSUB + 4 * v);
        __syncthreads();                                   // the previous unit is done with shared memory
        copy_image(m_begin, m_begin & 1);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        for (int m = m_begin; m < m_end; ++m) {
            const int buf = m & 1;
            if (m + 1 < m_end) copy_image(m + 1, buf ^ 1);  // uniform; that buffer was last read a barrier ago
            // operand A of every instruction (the image holds the negated centres), and the norm operand
            u32x4 xa[2][P::kEntries], xn[2];
#pragma unroll
            for (int f = 0; f < 2; ++f) {
                float ss = 0.f;
                uint32_t xp[3][2 * NV];                    // [piece][pair of components]
#pragma unroll
                for (int d = 0; d < 2 * NV; ++d) {
                    const float t0 = anext[f][d / 2][2 * (d % 2)], t1 = anext[f][d / 2][2 * (d % 2) + 1];
                    ss = fmaf(t0, t0, fmaf(t1, t1, ss));
                    split3(t0, t1, xp[0][d], xp[1][d], xp[2][d]);
                }
                if (DSUB == 16) ss += __shfl_xor(ss, 32, 64);  // the other half of the row's components
                largest = fmaxf(largest, ss);
                const u32x4 na = norm_operand_a(0.5f * ss), zero = {0u, 0u, 0u, 0u};
                xn[f] = h == 0 ? na : zero;
#pragma unroll
                for (int t = 0; t < P::kEntries; ++t) {
                    if constexpr (DSUB == 16) {
                        xa[f][t] = u32x4{xp[t][0], xp[t][1], xp[t][2], xp[t][3]};
                    } else if constexpr (DSUB == 8) {
                        const int p0 = P::kX[t][0], p1 = P::kX[t][1];
                        const u32x4 q0 = {xp[p0][0], xp[p0][1], xp[p0][2], xp[p0][3]}, q1 = {xp[p1][0], xp[p1][1], xp[p1][2], xp[p1][3]};
                        xa[f][t] = h == 0 ? q0 : q1;
                    } else {
                        const int a0 = P::kX[t][0][0], b0 = P::kX[t][0][1], a1 = P::kX[t][1][0], b1 = P::kX[t][1][1];
                        const u32x4 q0 = {xp[a0][0], xp[a0][1], xp[b0][0], xp[b0][1]};
                        const u32x4 q1 = a1 < 0 ? na : u32x4{xp[a1][0], xp[a1][1], xp[b1][0], xp[b1][1]};
                        xa[f][t] = h == 0 ? q0 : q1;
                    }
                }
            }
            // Running minimum per lane over the 8 blocks of 32 centres, taken two blocks at a time: the
            // block number replaces the three lowest mantissa bits of the (non-negative) value and the
            // minimum is taken on the bit patterns, so the lower block wins among equal values; one
            // three-way minimum folds two tagged values into the running one (1.5 ALU instructions
            // per value).
            //
            // Eight stages per sub-block, stage = (pair of centre blocks, half f of the rows): 2 x
            // (products + norm) matrix instructions into one accumulator pair.  Matrix instructions
            // and vector work overlap inside a wave's own instruction stream, hardly between waves,
            // so the loop is software-pipelined by hand: the instructions of stage s are interleaved
            // with the folding of stage s - 1 (scheduling hints: one matrix instruction, then a few
            // ALU ones), on two accumulator pairs in turn.  Fully unrolled, so the block numbers are
            // instruction constants.
            int best[2][16];
            u32x4 cp[2][P::kEntries], cnorm[2];
            float16v accs[2][2];                           // [stage parity][block of the pair]
            constexpr int kStages = 2 * (kPqK / 64);
            constexpr int kInstr = 2 * (P::kProducts + (P::kNormInstr ? 1 : 0));   // matrix instructions per stage
#pragma unroll
            for (int st = 0; st <= kStages; ++st) {
                if (st < kStages) {
                    const int cb0 = 2 * (st >> 1), f = st & 1;
                    if (f == 0) {
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
#pragma unroll
                            for (int t = 0; t < P::kEntries; ++t)
                                cp[e][t] = *reinterpret_cast<const u32x4 *>(img[buf] + ((t * 2 + h) * kPqK + 32 * (cb0 + e) + r) * 16);
                            if (P::kNormInstr) {
                                const uint2 nn = *reinterpret_cast<const uint2 *>(img[buf] + kImgPieces + (32 * (cb0 + e) + r) * 8);
                                cnorm[e] = u32x4{kBf16One | (kBf16One << 16), nn.x, nn.y, 0u};
                            }
                        }
                    }
                    float16v(&acc)[2] = accs[st & 1];
#pragma unroll
                    for (int e = 0; e < 2; ++e)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[e][v] = 0.f;
#pragma unroll
                    for (int t = 0; t < P::kProducts; ++t)
#pragma unroll
                        for (int e = 0; e < 2; ++e) acc[e] = mfma_bf16(xa[f][P::kA[t]], cp[e][P::kB[t]], acc[e]);
                    if (P::kNormInstr) {
#pragma unroll
                        for (int e = 0; e < 2; ++e) acc[e] = mfma_bf16(xn[f], cnorm[e], acc[e]);
                    }
                }
                if (st > 0) {
                    // fold the stage before: accumulator element v of lane (r, h) is row 8 (v / 4) + 4 h + v % 4
                    // of the half, centre slot 32 cb + r
                    const int pst = st - 1, cb0 = 2 * (pst >> 1), f = pst & 1;
                    const float16v(&acc)[2] = accs[pst & 1];
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int ka = (__float_as_int(acc[0][v]) & ~7) | cb0, kb = (__float_as_int(acc[1][v]) & ~7) | (cb0 + 1);
                        best[f][v] = cb0 == 0 ? min(ka, kb) : min(min(ka, kb), best[f][v]);
                    }
                }
                if (st > 0 && st < kStages) {
#pragma unroll
                    for (int g = 0; g < kInstr; ++g) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                    // one matrix instruction
                        __builtin_amdgcn_sched_group_barrier(0x002, (48 + kInstr - 1) / kInstr, 0);   // its share of the 48 folding instructions
                    }
                }
                __builtin_amdgcn_sched_barrier(0);         // a stage and the fold beside it are one scheduling region
            }
            {                                              // the next sub-block's components (the last one re-reads)
                const int mn = m + 1 < m_end ? m + 1 : m;
#pragma unroll
                for (int f = 0; f < 2; ++f)
#pragma unroll
                    for (int v = 0; v < NV; ++v) anext[f][v] = *reinterpret_cast<const f32x4 *>(xrow[f] + (size_t)mn * DSUB + 4 * v);
            }
            const int code = code_by_reduce_scatter(best, lane);
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
            __builtin_amdgcn_s_waitcnt(0);                 // this wave's part of the next image has landed
            __syncthreads();
        }
    }
    // A bound on every |x| the call has seen, for the fixed-point sums of the Lloyd iteration: the
    // bit patterns of non-negative floats order like the floats.
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) largest = fmaxf(largest, __shfl_xor(largest, o, 64));
    if (lane == 0) atomicMax(bound, __float_as_uint(largest));
}

// Lloyd iteration, second half: per-centre sums of the assigned sub-vectors, counts, and the
// distortion.
//
// A floating-point add into shared memory by atomic is executed lane by lane on this chip (about
// 130 cycles per wave instruction), a 64-bit integer add at about 7.  So the sums are kept in fixed
// point: a value x becomes the integer round(x * 2^F), with F chosen from a bound on |x| (the
// largest squared sub-vector norm, which the encoder notes on its way) and from N so that neither a
// value nor the sum of all N can leave 63 bits; for a million rows that leaves 2^-41 of the bound as
// the resolution, far below the fp32 spacing of the values themselves.  Integer sums do not depend
// on the order of the adds: the new centres are the same bits from run to run.
//
// The conversion costs two instructions: in double precision x * 2^F + 1.5 * 2^52 has round(x * 2^F)
// in its low mantissa bits, so the bit pattern of that sum is the integer plus the pattern of the
// constant, and what is added to the cell is the pattern as it is.  A cell with n entries then holds
// the fixed-point sum plus n times the constant's pattern (mod 2^64); n is the centre's count, and
// pq_move_centres_kernel takes the multiple off again.
//
// A workgroup of eight waves owns 64 dimensions (256 bytes of every row, 64/DSUB whole sub-blocks)
// and a slice of the rows; runs x slices workgroups, one per compute unit.
// Sixteen lanes read a row's 256 bytes, four dimensions each, and add them to the cells of the
// row's code: 128 KB of cells per workgroup, [sub-block][code][slot], where the four dimensions a
// lane holds sit DSUB/4 cells apart and slot s of a code is stored at s ^ (bits of the code), so
// that one instruction's 64 adds spread over the banks whatever the codes.  At the end the
// workgroup adds its non-empty cells to the global ones.
//
// Reading a column of a row-major matrix is the slow part: 128-byte pieces come in at 5.4 TB/s,
// 256-byte pieces at 6 TB/s, and only with about 32 KB in flight per compute unit (eight waves,
// four loads each); more waves or deeper unrolling make the memory system slower, not faster.
//
// The distortion is not summed row by row: sum_i ||x_i - c_k(i)||^2 = sum_i ||x_i||^2 +
// sum_k (n_k ||c_k||^2 - 2 <c_k, S_k>) with S_k the sum of the rows of cell k, so this kernel only
// adds up ||x||^2 (in double precision: every square is exact) and the second sum falls out of the
// move.  Partial sums go to a slot per workgroup and are added in a fixed order.
constexpr unsigned long long kFixMagicBits = 0x4338000000000000ull;   // the double 1.5 * 2^52
constexpr int kAccThreads = 512, kAccDims = 64;                        // dimensions per workgroup
constexpr int kAccCells = kPqK * kAccDims;                            // its cells: 128 KB
constexpr int kAccLanesPerRow = kAccDims / 4, kAccRowsPerInstr = 64 / kAccLanesPerRow;

// F of the fixed-point format from the encoder's bound (bit pattern of the largest squared
// sub-vector norm, a float >= 0) and the number of rows.
__device__ __forceinline__ int fixed_point_shift(uint32_t bound_bits, long long N) {
    const float b2 = __uint_as_float(bound_bits);
    int e = 0;
    if (b2 > 0.f && b2 < INFINITY) frexpf(b2, &e);         // b2 = f 2^e, f in [0.5, 1): |x| <= 2^ceil(e / 2)
    const int eb = ((e + 1) >> 1) + 1;                     // one more for the rounding of the norm itself
    const int lgn = N > 1 ? 64 - __clzll(N - 1) : 0;       // N <= 2^lgn
    const int fmax = 62 - lgn < 51 ? 62 - lgn : 51;        // |round(x 2^F)| < 2^fmax: sums below 2^62, values below 2^51
    return fmax - 1 - eb;
}

template <int DSUB>
struct AccLayout {
    static constexpr int G = kAccDims / DSUB;              // sub-blocks per workgroup
    static constexpr int Q = DSUB / 4;                     // lanes per row and sub-block = cells between a lane's dimensions
    static constexpr int kRotShift = DSUB == 16 ? 1 : DSUB == 8 ? 2 : 3;   // codes per 256 bytes of cells: 2, 4, 8
    __device__ static uint32_t rot(uint32_t code) { return (code >> kRotShift) & 3u; }
};

template <int DSUB, int U>
__global__ __launch_bounds__(kAccThreads) void pq_accumulate_kernel(const float *__restrict__ X, long long N, long long ldx,
                                                                     const uint8_t *__restrict__ codes, int M,
                                                                     const uint32_t *__restrict__ bound,
                                                                     unsigned long long *sums, uint32_t *counts,
                                                                     double *__restrict__ xsq, int slices) {
    using L = AccLayout<DSUB>;
    constexpr int G = L::G, Q = L::Q;
    extern __shared__ __align__(16) unsigned char acc_lds[];
    unsigned long long *cells = reinterpret_cast<unsigned long long *>(acc_lds);         // [G][256][DSUB]
    uint32_t *cnt = reinterpret_cast<uint32_t *>(acc_lds + kAccCells * 8);                // [G][256]
    double *red = reinterpret_cast<double *>(acc_lds + kAccCells * 8 + G * kPqK * 4);     // one per wave
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroups go to the chip's eight dies in turn.  Consecutive numbers are the slices of one run of
    // dimensions, so (with eight slices) a die holds all the column runs of ONE slice of rows, and the
    // line of codes of a row, which every run needs two to sixteen bytes of, is fetched into one
    // die's cache instead of eight.
    const int run = blockIdx.x / slices, slice = blockIdx.x % slices;
    for (int i = tid; i < kAccCells; i += kAccThreads) cells[i] = 0ull;
    for (int i = tid; i < G * kPqK; i += kAccThreads) cnt[i] = 0u;
    const int rr = lane / kAccLanesPerRow, cc = lane % kAccLanesPerRow;   // row of the instruction's four, run of four dimensions
    const int g = (4 * cc) / DSUB, cq = cc % Q;
    const int col = run * kAccDims + 4 * cc;
    // M * DSUB is a multiple of 16: a lane's four dimensions exist all or not at all
    const bool col_live = col < M * DSUB;
    const int m = col_live ? run * G + g : 0;
    const long long per = (N + slices - 1) / slices;
    const long long begin = per * slice, end = begin + per < N ? begin + per : N;
    const int rows = end > begin ? (int)(end - begin) : 0;
    const double scale = ldexp(1.0, fixed_point_shift(*bound, N));
    const double magic = __longlong_as_double((long long)kFixMagicBits);
    const uint32_t lane_base = (uint32_t)(g * kPqK * DSUB * 8 + cq * 8);
    const float *xlane = X + begin * ldx + (col_live ? col : 0);
    const uint8_t *klane = codes + begin * M + m;
    double sq = 0.0;
    __syncthreads();

    float4 xa[U], xb[U];                                   // two rounds of rows, by name: no indexed registers
    uint32_t ka[U], kb[U];
    // Rows past the end of the slice are read as its last row (in bounds) and left out of the adds.
    auto load = [&](int base, float4 (&xs)[U], uint32_t (&ks)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int r = base + (u * (kAccThreads / 64) + wave) * kAccRowsPerInstr + rr;
            r = r < rows ? r : rows - 1;
            xs[u] = *reinterpret_cast<const float4 *>(xlane + (long long)r * ldx);
            ks[u] = klane[(long long)r * M];
        }
    };
    auto add = [&](int base, const float4 (&xs)[U], const uint32_t (&ks)[U], auto full) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = base + (u * (kAccThreads / 64) + wave) * kAccRowsPerInstr + rr;
            if (!col_live || !(full.value || r < rows)) continue;
            const uint32_t code = ks[u];
            const uint32_t a0 = (lane_base + code * (DSUB * 8)) | (L::rot(code) * (Q * 8));
            const float v[4] = {xs[u].x, xs[u].y, xs[u].z, xs[u].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const double d = (double)v[i];
                sq = fma(d, d, sq);
                const unsigned long long fixed = (unsigned long long)__double_as_longlong(fma(d, scale, magic));
                atomicAdd(reinterpret_cast<unsigned long long *>(acc_lds + (a0 ^ (uint32_t)(i * Q * 8))), fixed);
            }
            if (cq == 0) atomicAdd(cnt + g * kPqK + code, 1u);
        }
    };
    // the loads of one round of rows are in flight while the round before is added
    constexpr int ROUND = kAccRowsPerInstr * (kAccThreads / 64) * U;
    auto add_round = [&](int base, const float4 (&xs)[U], const uint32_t (&ks)[U]) {
        if (base + ROUND <= rows) add(base, xs, ks, std::true_type{});
        else add(base, xs, ks, std::false_type{});
    };
    if (rows > 0) load(0, xa, ka);
    for (int base = 0; base < rows; base += 2 * ROUND) {
        const bool second = base + ROUND < rows;
        if (second) load(base + ROUND, xb, kb);
        add_round(base, xa, ka);
        if (second) {
            if (base + 2 * ROUND < rows) load(base + 2 * ROUND, xa, ka);
            add_round(base + ROUND, xb, kb);
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
    if (lane == 0) red[wave] = sq;
    __syncthreads();
    if (tid == 0) {
        double t = 0.0;
        for (int w = 0; w < kAccThreads / 64; ++w) t += red[w];
        xsq[blockIdx.x] = t;
    }
    // cell index -> (sub-block, code, dimension): slot s = position / Q holds dimension 4 q + (s ^ rot)
    for (int i = tid; i < kAccCells; i += kAccThreads) {
        const unsigned long long v = cells[i];
        if (v == 0ull) continue;                           // never touched: a touched cell holds at least the constant's pattern
        const int gg = i / (kPqK * DSUB), code = (i / DSUB) % kPqK, pos = i % DSUB;
        const int j = 4 * (pos % Q) + ((pos / Q) ^ (int)L::rot((uint32_t)code));
        const int mm = run * G + gg;
        atomicAdd(&sums[((size_t)mm * kPqK + code) * DSUB + j], v);
    }
    for (int i = tid; i < G * kPqK; i += kAccThreads)
        if (cnt[i]) atomicAdd(&counts[(size_t)run * G * kPqK + i], cnt[i]);
}

// the largest square of any element: the bound for the fixed-point sums when the encoder that notes
// it on its way is not the one that ran (comparison route)
__global__ __launch_bounds__(256) void pq_bound_kernel(const float *__restrict__ X, long long N, long long ldx, int D,
                                                       uint32_t *bound) {
    float mx = 0.f;
    const long long total = N * (long long)(D / 4);
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x) {
        const float4 v = *reinterpret_cast<const float4 *>(X + (t / (D / 4)) * ldx + 4 * (t % (D / 4)));
        mx = fmaxf(fmaxf(fmaxf(mx, v.x * v.x), fmaxf(v.y * v.y, v.z * v.z)), v.w * v.w);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(bound, __float_as_uint(mx));
}

__global__ __launch_bounds__(256) void pq_zero_kernel(unsigned long long *sums, uint32_t *counts, uint32_t *ticket, int M,
                                                      int dsub) {
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < (size_t)M * kPqK * dsub) sums[t] = 0ull;
    if (t < (size_t)M * kPqK) counts[t] = 0u;
    if (t == 0) *ticket = 0u;
}

// centre <- mean of its cell; a centre with an empty cell stays.  Also the distortion (mean over
// rows of the squared distance to the assigned centre, the centres being those the rows were
// assigned with): every thread contributes n c^2 - 2 c S of its cell, a workgroup's total goes to
// its slot, and the workgroup that finishes last adds the slots and those of the accumulation in a
// fixed order.
__global__ __launch_bounds__(256) void pq_move_centres_kernel(float *codebooks, const unsigned long long *sums,
                                                              const uint32_t *counts, int M, int dsub,
                                                              const uint32_t *bound, long long N, const double *xsq,
                                                              int n_xsq, double *cross, uint32_t *ticket,
                                                              double *distortion_out) {
    __shared__ double red[256];
    __shared__ bool last;
    double term = 0.0;
    const size_t cells = (size_t)M * kPqK * dsub;
    const double unit = ldexp(1.0, -fixed_point_shift(*bound, N));
    for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < cells; t += (size_t)gridDim.x * blockDim.x) {
        const uint32_t n = counts[t / dsub];
        if (n) {
            const double s = (double)(long long)(sums[t] - (unsigned long long)n * kFixMagicBits) * unit;
            const double c = (double)codebooks[t];
            term += c * ((double)n * c - 2.0 * s);
            codebooks[t] = (float)(s / (double)n);
        }
    }
    if (!distortion_out) return;
    auto block_sum = [&](double v) -> double {             // fixed tree: the same bits every run
        red[threadIdx.x] = v;
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) {
            if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
            __syncthreads();
        }
        const double r = red[0];
        __syncthreads();
        return r;
    };
    const double total = block_sum(term);
    if (threadIdx.x == 0) {
        cross[blockIdx.x] = total;
        __threadfence();                                   // the slot before the ticket
        last = atomicAdd(ticket, 1u) == gridDim.x - 1;
    }
    __syncthreads();
    if (!last) return;
    __threadfence();                                       // every workgroup's slot
    double a = 0.0;
    for (int i = threadIdx.x; i < (int)gridDim.x; i += 256) a += cross[i];
    for (int i = threadIdx.x; i < n_xsq; i += 256) a += xsq[i];
    const double sum = block_sum(a);
    if (threadIdx.x == 0) *distortion_out = sum > 0.0 ? sum / (double)N : 0.0;
}

struct PqTrainWs {
    uint32_t *bound, *ticket;
    float *norms;
    unsigned long long *sums;
    uint32_t *counts;
    double *xsq, *cross;
    uint8_t *image;                                        // the vocabulary as the bf16 encoder reads it
};

constexpr int kAccMaxGrid = 2048;                          // workgroups of the accumulation: slots for their ||x||^2

static size_t pq_train_ws_tables(int M, int dsub) {
    const size_t cells = (size_t)M * kPqK * dsub;
    const size_t b = 256 + (size_t)M * kPqK * 4 /* norms */ + cells * 8 /* sums */ + (size_t)M * kPqK * 4 /* counts */ +
                     (size_t)kAccMaxGrid * 8 + ((cells + 255) / 256) * 8;
    return (b + 255) & ~(size_t)255;
}

size_t pq_train_ws_bytes(int M, int dsub) {
    return pq_train_ws_tables(M, dsub) + (size_t)M * kImgBytes;
}

static PqTrainWs pq_train_ws(void *ws, int M, int dsub) {
    uint8_t *p = reinterpret_cast<uint8_t *>(ws);
    const size_t cells = (size_t)M * kPqK * dsub;
    PqTrainWs w;
    w.bound = reinterpret_cast<uint32_t *>(p);
    w.ticket = w.bound + 1;
    w.sums = reinterpret_cast<unsigned long long *>(p + 256);
    w.xsq = reinterpret_cast<double *>(w.sums + cells);
    w.cross = w.xsq + kAccMaxGrid;
    w.norms = reinterpret_cast<float *>(w.cross + (cells + 255) / 256);
    w.counts = reinterpret_cast<uint32_t *>(w.norms + (size_t)M * kPqK);
    w.image = p + pq_train_ws_tables(M, dsub);
    return w;
}

hipError_t launch_pq_encode(const float *X, int64_t N, int64_t ldx, const float *codebooks, int M, int dsub,
                            uint8_t *codes, void *ws, hipStream_t s) {
    PqTrainWs w = pq_train_ws(ws, M, dsub);
    const int64_t ntiles = (N + 255) / 256;
    const int mr = std::min(M, std::max(4, tune_int(OTF_DEBUG_PQENC_RANGE, 16) & ~3));   // sub-blocks per work unit, a multiple of 4
    const int64_t units = ntiles * ((M + mr - 1) / mr);
    const int grid = (int)std::min<int64_t>(units, (int64_t)device_cu_count() * tune_int(OTF_DEBUG_PQENC_BLOCKS_PER_CU, 3));
    const bool fp32 = tune_int(OTF_DEBUG_PQENC_FP32, 0) != 0;   // the fp32 matrix instructions, kept for comparison
#define OTF_PQENC_LAUNCH(D)                                                                                                   \
    if (fp32) {                                                                                                               \
        pq_centre_norms_kernel<<<(M * kPqK + 255) / 256, 256, 0, s>>>(codebooks, M, dsub, w.norms);                          \
        pq_encode_kernel<D><<<grid, 256, 0, s>>>(X, (long long)N, (long long)ldx, codebooks, w.norms, M, mr, codes);          \
    } else {                                                                                                                  \
        pq_centre_image_kernel<D><<<M, 256, 0, s>>>(codebooks, M, w.image, w.bound);                                         \
        pq_encode_bf16_kernel<D><<<grid, 256, 0, s>>>(X, (long long)N, (long long)ldx, w.image, M, mr, codes, w.bound);      \
    }
    switch (dsub) {
        case 4: OTF_PQENC_LAUNCH(4) break;
        case 8: OTF_PQENC_LAUNCH(8) break;
        case 16: OTF_PQENC_LAUNCH(16) break;
        default: return hipErrorInvalidValue;
    }
#undef OTF_PQENC_LAUNCH
    return hipGetLastError();
}

template <int DSUB>
static hipError_t launch_accumulate(const float *X, int64_t N, int64_t ldx, const uint8_t *codes, int M, const PqTrainWs &w,
                                    int groups, int slices, hipStream_t s) {
    constexpr int U = 4;
    const int lds = kAccCells * 8 + (kAccDims / DSUB) * kPqK * 4 + (kAccThreads / 64) * 8;
    static bool raised = false;                            // more shared memory than a kernel gets unasked
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pq_accumulate_kernel<DSUB, U>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    pq_accumulate_kernel<DSUB, U><<<groups * slices, kAccThreads, lds, s>>>(X, (long long)N, (long long)ldx, codes, M, w.bound,
                                                                             w.sums, w.counts, w.xsq, slices);
    return hipGetLastError();
}

// A Lloyd iteration in three parts, so that the caller can bracket the middle one with events:
// assignment (encode; a bound on |x| if the encoder left none; zeroed sums), the per-centre sums,
// the move.
hipError_t launch_pq_lloyd_assign(const float *X, int64_t N, int64_t ldx, const float *codebooks, int M, int dsub,
                                  uint8_t *codes, void *ws, hipStream_t s) {
    hipError_t e = launch_pq_encode(X, N, ldx, codebooks, M, dsub, codes, ws, s);
    if (e != hipSuccess) return e;
    PqTrainWs w = pq_train_ws(ws, M, dsub);
    if (tune_int(OTF_DEBUG_PQENC_FP32, 0) != 0) {          // that encoder leaves no bound behind
        pq_zero_kernel<<<1, 256, 0, s>>>(w.sums, w.counts, w.bound, 0, 0);
        pq_bound_kernel<<<device_cu_count() * 4, 256, 0, s>>>(X, (long long)N, (long long)ldx, M * dsub, w.bound);
    }
    const size_t cells = (size_t)M * kPqK * dsub;
    pq_zero_kernel<<<(unsigned)((cells + 255) / 256), 256, 0, s>>>(w.sums, w.counts, w.ticket, M, dsub);
    return hipGetLastError();
}

// runs of 64 dimensions x slices of rows: one workgroup per compute unit (its cells fill most of the
// shared memory), one full round of them
static void lloyd_grid(int64_t N, int M, int dsub, int *groups, int *slices) {
    *groups = (M * dsub + kAccDims - 1) / kAccDims;
    int sl = (int)std::min<int64_t>((N + 1023) / 1024, std::max(1, device_cu_count() / *groups));
    *slices = std::max(1, std::min(sl, kAccMaxGrid / *groups));
}

hipError_t launch_pq_lloyd_sums(const float *X, int64_t N, int64_t ldx, const uint8_t *codes, int M, int dsub, void *ws,
                                hipStream_t s) {
    PqTrainWs w = pq_train_ws(ws, M, dsub);
    int groups, slices;
    lloyd_grid(N, M, dsub, &groups, &slices);
    switch (dsub) {
        case 4: return launch_accumulate<4>(X, N, ldx, codes, M, w, groups, slices, s);
        case 8: return launch_accumulate<8>(X, N, ldx, codes, M, w, groups, slices, s);
        case 16: return launch_accumulate<16>(X, N, ldx, codes, M, w, groups, slices, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_pq_lloyd_move(int64_t N, float *codebooks, int M, int dsub, double *distortion_out, void *ws,
                                hipStream_t s) {
    PqTrainWs w = pq_train_ws(ws, M, dsub);
    int groups, slices;
    lloyd_grid(N, M, dsub, &groups, &slices);
    const size_t cells = (size_t)M * kPqK * dsub;
    const unsigned cell_blocks = (unsigned)((cells + 255) / 256);
    // a workgroup per compute unit: each one ends with a device-wide fence, and those cost more than the cells
    const unsigned move_blocks = std::min<unsigned>(cell_blocks, (unsigned)device_cu_count());
    pq_move_centres_kernel<<<move_blocks, 256, 0, s>>>(codebooks, w.sums, w.counts, M, dsub, w.bound, (long long)N, w.xsq,
                                                       groups * slices, w.cross, w.ticket, distortion_out);
    return hipGetLastError();
}

}  // namespace otf
