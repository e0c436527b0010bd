// Dense scan, one classifier: s_i = b + <w, x_i> for every stored row (paper Sec. 4, "Ranking":
// every pre-computed dataset feature is scored with the current linear model; Sec. 3.2: the
// predictor is <w, phi(I)>).  0.5 flop per byte: the kernel is a pure HBM stream.
//
// Layout: a row is read by `LPR` adjacent lanes, 16 bytes per lane per load, so every wave
// load covers whole 1 KiB-contiguous pieces of the store; w sits in registers (each lane keeps
// the columns it reads).  Waves draw their rows from a work queue and keep the next tile's loads
// in flight while they reduce the current one.  Each finished score is written once and counted
// into the block's pass-1 histogram of the top-k selection, so ranking needs no further pass
// over the store; rows of at most 512 bytes can instead be filtered against a threshold taken
// from a sample, in which case the scan writes only the few rows that pass.
#include <hip/hip_fp16.h>

#include <algorithm>

#include "otf_internal.h"

namespace otf {

struct alignas(16) Chunk16 {
    uint32_t u[4];
};

__device__ __forceinline__ Chunk16 load_stream16(const void *p) {
    Chunk16 c;
    const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
    // streaming data is read exactly once: non-temporal so that it does not evict the tables
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    u4 v = __builtin_nontemporal_load(reinterpret_cast<const u4 *>(q));
    c.u[0] = v.x; c.u[1] = v.y; c.u[2] = v.z; c.u[3] = v.w;
    return c;
}

template <bool HALF>
struct Elem;
template <>
struct Elem<false> {
    static constexpr int kPer16 = 4;
    __device__ static __forceinline__ void unpack(const Chunk16 &c, float *f) {
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = __uint_as_float(c.u[j]);
    }
};
template <>
struct Elem<true> {
    static constexpr int kPer16 = 8;
    __device__ static __forceinline__ void unpack(const Chunk16 &c, float *f) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            __half2 h = *reinterpret_cast<const __half2 *>(&c.u[j]);
            float2 t = __half22float2(h);
            f[2 * j] = t.x;
            f[2 * j + 1] = t.y;
        }
    }
};

__device__ __forceinline__ float load_w(const void *w, int w_is_half, int d) {
    return w_is_half ? __half2float(reinterpret_cast<const __half *>(w)[d]) : reinterpret_cast<const float *>(w)[d];
}

// ---------------------------------------------------------------------------------------------
// Wide rows: one wave per row, V 16-byte chunks per lane (D <= 64 * V * elems-per-chunk).
//
// FULL (D == 64 * V * elems-per-chunk exactly, e.g. 2048 fp32 with V = 8): branch-free and
// software-pipelined.  The loads of the wave's next row are issued before the current row is
// reduced, so 2*V 16-byte loads per lane stay in flight; with few, long-lived waves this is what
// saturates HBM (many waves with shallow queues do not).  A prefetch with no row left re-reads
// the current row instead of being skipped: an unconditional load keeps the in-order wait
// counters exact, a conditional one would force a full drain every iteration.  Rows are handed
// out dynamically (TileQueue: one row per ticket, chunks of 256 KiB of rows).
// Otherwise each block owns one contiguous range of rows, its waves taking its rows in turn.
// Three waves per compute unit, two rows (16 KiB at V = 8) in flight each: measured on 1M x 2048
// fp32, the kernel takes 2.54 ms with one wave, 1.45 with two, 1.145 with three, 1.162 with four,
// 1.19 with six or eight, and more with the same waves spread over several workgroups; a third
// row in flight per wave loses 2 % as well.  ~48 KiB in flight per compute unit is what the memory
// system takes best for whole rows of 8 KiB.
constexpr int kWideThreads = 192;
template <bool XHALF, int V, bool FULL>
__global__ __launch_bounds__(256) void dense_wide_kernel(const uint8_t *__restrict__ X, long long N, int D,
                                                         long long row_bytes, const void *__restrict__ w,
                                                         int w_is_half, const float *__restrict__ bias_ptr,
                                                         int bias_index, float *__restrict__ scores, uint32_t *hist1,
                                                         uint32_t *chunk_ctr) {
    constexpr int E = Elem<XHALF>::kPer16;
    __shared__ uint32_t lhist[kBins1];
    __shared__ TileQueue s_queue;
    if (FULL && threadIdx.x == 0) tile_queue_init(&s_queue, chunk_ctr);
    for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();

    const float bias = bias_ptr ? bias_ptr[bias_index] : 0.f;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    float wr[V][E];
    bool live[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const int col = (j * 64 + lane) * E;
        live[j] = FULL || col < D;
        if (w_is_half) {
#pragma unroll
            for (int e = 0; e < E; ++e)
                wr[j][e] = live[j] ? __half2float(reinterpret_cast<const __half *>(w)[col + e]) : 0.f;
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) wr[j][e] = live[j] ? reinterpret_cast<const float *>(w)[col + e] : 0.f;
        }
    }
    const long long per = (N + gridDim.x - 1) / gridDim.x;
    const long long begin = per * blockIdx.x;
    long long end = begin + per;
    if (end > N) end = N;

    auto dot = [&](const Chunk16 *c) {
        float a0 = 0.f, a1 = 0.f;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            float f[E];
            Elem<XHALF>::unpack(c[j], f);
#pragma unroll
            for (int e = 0; e < E; e += 2) {
                a0 = fmaf(f[e], wr[j][e], a0);
                a1 = fmaf(f[e + 1], wr[j][e + 1], a1);
            }
        }
        return wave_sum_to_lane0(a0 + a1) + bias;
    };
    auto emit = [&](long long r, float sc) {
        if (lane == 0) {
            scores[r] = sc;
            atomicAdd(&lhist[float_to_key(sc) >> 20], 1u);
        }
    };

    if (FULL) {
        const uint32_t CHUNK_ROWS = tile_queue_chunk_tiles(N, 256u / (uint32_t)V);   // x V KiB per row = 256 KiB
        const uint8_t *base = X + (size_t)lane * 16;
        auto fetch = [&](Chunk16 *c, long long r) {
            const uint8_t *p = base + (size_t)r * (size_t)row_bytes;
#pragma unroll
            for (int j = 0; j < V; ++j) c[j] = load_stream16(p + (size_t)j * 1024);
        };
        long long cur = tile_queue_draw(&s_queue, chunk_ctr, CHUNK_ROWS, N);
        if (cur >= 0) {                                     // uniform per wave
            Chunk16 a[V], b[V];
            fetch(a, cur);
            for (;;) {
                long long nxt = tile_queue_draw(&s_queue, chunk_ctr, CHUNK_ROWS, N);
                fetch(b, nxt >= 0 ? nxt : cur);
                emit(cur, dot(a));
                if (nxt < 0) break;
                cur = nxt;
                nxt = tile_queue_draw(&s_queue, chunk_ctr, CHUNK_ROWS, N);
                fetch(a, nxt >= 0 ? nxt : cur);
                emit(cur, dot(b));
                if (nxt < 0) break;
                cur = nxt;
            }
        }
    } else {
        for (long long r = begin + wave; r < end; r += nwaves) {
            const uint8_t *p = X + (size_t)r * (size_t)row_bytes + (size_t)lane * 16;
            Chunk16 c[V];
#pragma unroll
            for (int j = 0; j < V; ++j) {
                c[j] = Chunk16{{0u, 0u, 0u, 0u}};
                if (live[j]) c[j] = load_stream16(p + (size_t)j * 1024);
            }
            emit(r, dot(c));
        }
    }
    merge_hist1(lhist, hist1);
}

// ---------------------------------------------------------------------------------------------
// Cross-lane pieces of the narrow kernel's row sums (vector ALU only: DPP and v_permlane16_swap;
// a shuffle through the LDS crossbar per step and value was the kernel's bottleneck).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}
// the value of lane ^ BIT, BIT = 1, 2, 4, 8
template <int BIT>
__device__ __forceinline__ float lane_xor(float v) {
    if (BIT == 1) return dpp_f32<0xB1>(v);                       // quad_perm [1,0,3,2]
    if (BIT == 2) return dpp_f32<0x4E>(v);                       // quad_perm [2,3,0,1]
    if (BIT == 4) return dpp_f32<0x1B>(dpp_f32<0x141>(v));       // half mirror, then quad reversed
    return dpp_f32<0x128>(v);                                    // row_ror:8
}
// One reduce-scatter step over lane bit BIT on the first NV values: afterwards v[0 .. NV/2) hold
// the pairwise sums of entries 0 .. NV/2-1 in the lanes whose bit is 0 and of entries NV/2 .. NV-1
// in the lanes whose bit is 1.
template <int BIT, int NV>
__device__ __forceinline__ void rs_add(float *v, int lane) {
    if (BIT == 16) {
#pragma unroll
        for (int j = 0; j < NV / 2; ++j) {
            const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(v[j]), __float_as_uint(v[j + NV / 2]), false, false);
            v[j] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
        }
    } else {
        const bool up = (lane & BIT) != 0;
#pragma unroll
        for (int j = 0; j < NV / 2; ++j) {
            const float keep = up ? v[j + NV / 2] : v[j], give = up ? v[j] : v[j + NV / 2];
            v[j] = keep + lane_xor<BIT>(give);
        }
    }
}
// Sums over the LPR lanes of a row for the 8 loads of a tile: v[u] = this lane's partial sum of
// load u.  Up to three scatter steps over the top bits of the lane's position in its row, then
// plain exchanges over the remaining bits.  Afterwards value k < 8 >> steps of a lane is the full
// sum of load ((position >> remaining bits) * (8 >> steps) + k).
template <int LPR>
__device__ __forceinline__ void tile_row_sums(float *v, int lane) {
    if constexpr (LPR >= 2) rs_add<LPR / 2, 8>(v, lane);
    if constexpr (LPR >= 4) rs_add<LPR / 4, 4>(v, lane);
    if constexpr (LPR >= 8) rs_add<LPR / 8, 2>(v, lane);
    if constexpr (LPR >= 16) v[0] += lane_xor<LPR / 16>(v[0]);
    if constexpr (LPR >= 32) v[0] += lane_xor<1>(v[0]);
}

// Narrow rows: LPR = 1..32 lanes per row (a power of two), one 16-byte chunk per lane, so one
// wave load covers 64/LPR consecutive rows; a tile is U such loads.  Same scheme as the wide
// kernel: tiles are handed out dynamically (TileQueue, chunks of 256 KiB of rows), the loads of a
// wave's next tile are issued before the current one is reduced, and a prefetch with nothing left
// re-reads the current tile.  The rows after the last full tile go to one wave, row-checked.
//
// EMIT (ScanEmit) as in the table scans: every score plus the pass-1 histogram; the same for the
// strided sample of the store (N = rows of the sample, numbered compactly); or, given the state
// that passes 1 and 2 over the sample left, only the rows at or above the threshold, appended to
// the candidate list.  With rows this short one score per row is a store every few hundred bytes
// of the stream, and leaving it out is worth 7-11 % of the scan.
template <bool XHALF, int LPR, int EMIT>
__global__ __launch_bounds__(256) void dense_narrow_kernel(const uint8_t *__restrict__ X, long long N, int D,
                                                           long long row_bytes, const void *__restrict__ w,
                                                           int w_is_half, const float *__restrict__ bias_ptr, int bias_index,
                                                           float *__restrict__ scores, uint32_t *hist1,
                                                           uint32_t *chunk_ctr, SelState *st,
                                                           const SelState *tau_state, SampleSlot *sample_slots,
                                                           unsigned long long *__restrict__ cand,
                                                           Gate gate) {
    constexpr int E = Elem<XHALF>::kPer16;
    constexpr int RPW = 64 / LPR;   // rows per wave load
    constexpr int U = 8;
    constexpr int TILE = RPW * U;   // rows per wave iteration (U KiB of a dense store)
    static_assert(kSampleGroup % TILE == 0, "a tile of the sample scan must not straddle a sample group");
    static_assert(kBins2 <= kBins1, "the histogram area doubles as the buffer that resolves the threshold");
    __shared__ uint32_t lhist[kBins1];
    __shared__ uint32_t s_out[3];
    __shared__ TileQueue s_queue;
    if (!gate_open(gate)) return;                 // uniform: this launch is only the fallback of a filtered scan
    if (threadIdx.x == 0) tile_queue_init(&s_queue, chunk_ctr);   // visible after the barriers below
    uint32_t tau = 0u;
    if (EMIT == kEmitFilter) {
        // the threshold from the wave maxima the sample scan left, resolved by every workgroup for itself
        const TauChoice tc = resolve_tau_slots(sample_slots, tau_state, N, lhist, s_out);
        if (tc.hopeless) return;                  // uniform
        tau = tc.tau;
    } else {
        for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
        __syncthreads();
    }
    uint32_t smx = 0u, scnt = 0u;                 // sample scan: this lane's largest key and its multiplicity

    const float bias = bias_ptr ? bias_ptr[bias_index] : 0.f;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % LPR, rr = lane / LPR;
    const int col = sub * E;
    const bool live = col < D;      // D need not fill the LPR chunks: those lanes load nothing
    float wr[E];
#pragma unroll
    for (int e = 0; e < E; ++e) wr[e] = live ? load_w(w, w_is_half, col + e) : 0.f;

    const long long ntiles = N / TILE;
    const uint32_t chunk_tiles = tile_queue_chunk_tiles(ntiles, 256u / (uint32_t)U);
    const size_t lane_off = (size_t)rr * (size_t)row_bytes + (size_t)sub * 16;
    // sample row v is store row (v / group) * group * stride + v % group
    auto store_row = [&](long long v) {
        return EMIT == kEmitSample
                   ? (v / kSampleGroup) * ((long long)kSampleGroup * kSampleStride) + (v % kSampleGroup)
                   : v;
    };
    auto fetch = [&](Chunk16 *c, long long tile) {
        const uint8_t *p = X + (size_t)store_row(tile * TILE) * (size_t)row_bytes + lane_off;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (live) c[u] = load_stream16(p + (size_t)u * RPW * (size_t)row_bytes);
    };
    constexpr int LOG_LPR = LPR == 1 ? 0 : LPR == 2 ? 1 : LPR == 4 ? 2 : LPR == 8 ? 3 : LPR == 16 ? 4 : 5;
    constexpr int STEPS = LOG_LPR < 3 ? LOG_LPR : 3;        // scatter steps of tile_row_sums
    constexpr int NVF = 8 >> STEPS;                         // sums a lane ends up with
    const bool owner = (sub & ((1 << (LOG_LPR - STEPS)) - 1)) == 0;
    const int u0 = (sub >> (LOG_LPR - STEPS)) * NVF;        // ... those of loads u0 .. u0 + NVF - 1
    auto partial = [&](const Chunk16 &c) {
        float acc = 0.f;
        if (live) {
            float f[E];
            Elem<XHALF>::unpack(c, f);
#pragma unroll
            for (int e = 0; e < E; ++e) acc = fmaf(f[e], wr[e], acc);
        }
        return acc;
    };
    // the owners' stores of one value index cover 64 / LPR * (8 / NVF) consecutive rows.
    // Filtered scan: a wave that has seen the candidate list full stops appending (the list is
    // useless by then, and the appends are adds to one address, one after the other).
    bool list_full = false;
    auto consume = [&](const Chunk16 *c, long long tile, long long nrows) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = partial(c[u]);
        tile_row_sums<LPR>(v, lane);
#pragma unroll
        for (int k = 0; k < NVF; ++k) {
            const long long row = tile * TILE + (long long)(u0 + k) * RPW + rr;
            const bool ok = owner && row < nrows;
            const float sc = v[k] + bias;
            const uint32_t key = float_to_key(sc);
            if (EMIT == kEmitSample) {
                if (ok) sample_note(smx, scnt, key);
            } else if (EMIT == kEmitFilter) {
                if (ok && key >= tau && !list_full) {
                    const uint32_t pos = atomicAdd(&st->cursor, 1u);
                    if (pos < (uint32_t)kCandCap)
                        cand[pos] = ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)row);
                    else
                        list_full = true;
                }
            } else {
                if (ok) scores[row] = sc;
                hist_add_wave(lhist, key >> 20, ok);   // many rows per instruction, few bins: aggregate
            }
        }
        if (EMIT == kEmitFilter) list_full = __ballot(list_full) != 0ull;
    };
    long long cur = tile_queue_draw(&s_queue, chunk_ctr, chunk_tiles, ntiles);
    if (cur >= 0) {
        Chunk16 b0[U], b1[U];
        fetch(b0, cur);
        for (;;) {
            long long nxt = tile_queue_draw(&s_queue, chunk_ctr, chunk_tiles, ntiles);
            fetch(b1, nxt >= 0 ? nxt : cur);
            consume(b0, cur, N);
            if (nxt < 0) break;
            cur = nxt;
            nxt = tile_queue_draw(&s_queue, chunk_ctr, chunk_tiles, ntiles);
            fetch(b0, nxt >= 0 ? nxt : cur);
            consume(b1, cur, N);
            if (nxt < 0) break;
            cur = nxt;
        }
    }
    if (ntiles * TILE < N && blockIdx.x == 0 && wave == 0) {
        Chunk16 c[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long row = ntiles * TILE + (long long)u * RPW + rr;
            c[u] = Chunk16{};
            if (live && row < N) c[u] = load_stream16(X + (size_t)store_row(row) * (size_t)row_bytes + (size_t)sub * 16);
        }
        consume(c, ntiles, N);
    }
    if (EMIT == kEmitScores) merge_hist1(lhist, hist1);
    if (EMIT == kEmitSample) sample_store(sample_slots, st, smx, scnt);
}

// ---------------------------------------------------------------------------------------------
// Very wide rows (D beyond what fits the register copy of w): w in shared memory as fp32,
// one wave per row, 64 * E columns per step.
template <bool XHALF>
__global__ __launch_bounds__(256) void dense_huge_kernel(const uint8_t *__restrict__ X, long long N, int D,
                                                         long long row_bytes, const void *__restrict__ w,
                                                         int w_is_half, const float *__restrict__ bias_ptr, int bias_index,
        float *__restrict__ scores, uint32_t *hist1) {
    constexpr int E = Elem<XHALF>::kPer16;
    extern __shared__ float w_lds[];   // D floats
    __shared__ uint32_t lhist[kBins1];
    for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
    for (int d = threadIdx.x; d < D; d += blockDim.x) w_lds[d] = load_w(w, w_is_half, d);
    __syncthreads();
    const float bias = bias_ptr ? bias_ptr[bias_index] : 0.f;
    const int lane = threadIdx.x & 63;
    const long long waves_total = (long long)gridDim.x * (blockDim.x >> 6);
    const long long wave_id = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int steps = (D + 64 * E - 1) / (64 * E);
    for (long long r = wave_id; r < N; r += waves_total) {
        const uint8_t *p = X + (size_t)r * row_bytes + (size_t)lane * 16;
        float acc = 0.f;
        for (int j0 = 0; j0 < steps; j0 += 4) {
            Chunk16 c[4];
            bool ok[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int col = ((j0 + u) * 64 + lane) * E;
                ok[u] = (j0 + u) < steps && col < D;
                if (ok[u]) c[u] = load_stream16(p + (size_t)(j0 + u) * 1024);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (ok[u]) {
                    const int col = ((j0 + u) * 64 + lane) * E;
                    float f[E];
                    Elem<XHALF>::unpack(c[u], f);
#pragma unroll
                    for (int e = 0; e < E; ++e) acc = fmaf(f[e], w_lds[col + e], acc);
                }
            }
        }
        acc = wave_sum(acc) + bias;
        if (lane == 0) {
            scores[r] = acc;
            atomicAdd(&lhist[float_to_key(acc) >> 20], 1u);
        }
    }
    merge_hist1(lhist, hist1);
}

// What the narrow kernel may be asked for beyond plain scores.
struct NarrowExtra {
    ScanEmit emit;
    SelState *st;
    const SelState *tau;
    SampleSlot *slots;
    unsigned long long *cand;
    Gate gate;
};

template <bool XHALF>
static hipError_t launch_dense_typed(const uint8_t *X, int64_t N, int D, int64_t row_bytes, const void *w,
                                     int w_is_half, const float *bias_ptr, int bias_index, float *scores,
                                     uint32_t *hist1, uint32_t *chunk_ctr, const NarrowExtra &x, hipStream_t s) {
    constexpr int E = Elem<XHALF>::kPer16;
    const int chunks = (D + E - 1) / E;              // 16-byte chunks per row
    const int cus = device_cu_count();
    int grid;
#define OTF_ARGS X, (long long)N, D, (long long)row_bytes, w, w_is_half, bias_ptr, bias_index, scores, hist1
#define OTF_WIDE_ARGS OTF_ARGS, chunk_ctr
    if (chunks <= 32) {
        int lpr = 1;
        while (lpr < chunks) lpr <<= 1;
        const int64_t rows_per_wave_iter = (64 / lpr) * 8;
        int64_t waves = (N + rows_per_wave_iter - 1) / rows_per_wave_iter;
        grid = (int)std::min<int64_t>((waves + 3) / 4, (int64_t)cus * tune_int(OTF_DEBUG_NARROW_BLOCKS_PER_CU, 2));
        if (grid < 1) grid = 1;
        if (x.emit == kEmitSample) grid = std::min(grid, cus);       // (one slot per wave: at most 4 x 256 slots)
#define OTF_NARROW(L)                                                                                              \
    do {                                                                                                           \
        if (x.emit == kEmitScores)                                                                                 \
            dense_narrow_kernel<XHALF, L, kEmitScores><<<grid, 256, 0, s>>>(OTF_WIDE_ARGS, x.st, x.tau, x.slots,     \
                                                                             x.cand, x.gate);                                     \
        else if (x.emit == kEmitSample)                                                                            \
            dense_narrow_kernel<XHALF, L, kEmitSample><<<grid, 256, 0, s>>>(OTF_WIDE_ARGS, x.st, x.tau, x.slots,     \
                                                                             x.cand, x.gate);                                     \
        else                                                                                                       \
            dense_narrow_kernel<XHALF, L, kEmitFilter><<<grid, 256, 0, s>>>(OTF_WIDE_ARGS, x.st, x.tau, x.slots,     \
                                                                             x.cand, x.gate);                                     \
    } while (0)
        switch (lpr) {
            case 1: OTF_NARROW(1); break;
            case 2: OTF_NARROW(2); break;
            case 4: OTF_NARROW(4); break;
            case 8: OTF_NARROW(8); break;
            case 16: OTF_NARROW(16); break;
            default: OTF_NARROW(32); break;
        }
#undef OTF_NARROW
    } else {
        if (x.emit != kEmitScores || x.gate.st) return hipErrorInvalidValue;   // only the narrow kernel filters
        grid = (int)std::min<int64_t>((N + 3) / 4, (int64_t)cus * tune_int(OTF_DEBUG_DENSE_BLOCKS_PER_CU, 1));
        if (grid < 1) grid = 1;
        const int V = (chunks + 63) / 64;
        const bool full = chunks == V * 64;
#define OTF_WIDE(VV)                                                                        \
    do {                                                                                    \
        if (full) dense_wide_kernel<XHALF, VV, true><<<grid, kWideThreads, 0, s>>>(OTF_WIDE_ARGS);   \
        else dense_wide_kernel<XHALF, VV, false><<<grid, 256, 0, s>>>(OTF_WIDE_ARGS);                \
    } while (0)
        if (V <= 1) OTF_WIDE(1);
        else if (V <= 2) OTF_WIDE(2);
        else if (V <= 4) OTF_WIDE(4);
        else if (V <= 8) OTF_WIDE(8);
#undef OTF_WIDE
        else {
            if (D > kDenseMaxD) return hipErrorInvalidValue;
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&dense_huge_kernel<XHALF>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, kDenseMaxD * 4);
            if (e != hipSuccess) return e;
            dense_huge_kernel<XHALF><<<grid, 256, (size_t)D * 4, s>>>(OTF_ARGS);
        }
    }
#undef OTF_WIDE_ARGS
#undef OTF_ARGS
    return hipGetLastError();
}

bool dense_scan_filters(int x_is_half, int D) {
    const int per16 = x_is_half ? 8 : 4;
    return (D + per16 - 1) / per16 <= 32;
}

hipError_t launch_dense_scan(const void *X, int x_is_half, int64_t N, int D, int64_t ldx, const void *w,
                             int w_is_half, const float *bias_ptr, int bias_index, float *scores, uint32_t *hist1,
                             uint32_t *chunk_ctr, hipStream_t s) {
    return launch_dense_scan_emit(X, x_is_half, N, D, ldx, w, w_is_half, bias_ptr, bias_index, kEmitScores, scores,
                                  hist1, chunk_ctr, nullptr, nullptr, nullptr, nullptr, kNoGate, s);
}

hipError_t launch_dense_scan_emit(const void *X, int x_is_half, int64_t N, int D, int64_t ldx, const void *w,
                                  int w_is_half, const float *bias_ptr, int bias_index, ScanEmit emit, float *scores,
                                  uint32_t *hist1, uint32_t *chunk_ctr, SelState *st, const SelState *tau,
                                  SampleSlot *slots, unsigned long long *cand, Gate gate, hipStream_t s) {
    const uint8_t *Xb = reinterpret_cast<const uint8_t *>(X);
    const NarrowExtra x{emit, st, tau, slots, cand, gate};
    if (emit == kEmitFilter && (!st || !tau || !slots || !cand)) return hipErrorInvalidValue;
    if (emit == kEmitSample && (!st || !slots)) return hipErrorInvalidValue;
    if (x_is_half)
        return launch_dense_typed<true>(Xb, N, D, ldx * 2, w, w_is_half, bias_ptr, bias_index, scores, hist1, chunk_ctr, x, s);
    return launch_dense_typed<false>(Xb, N, D, ldx * 4, w, w_is_half, bias_ptr, bias_index, scores, hist1, chunk_ctr, x, s);
}

}  // namespace otf
