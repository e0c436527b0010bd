// Dense scoring of a sparse-row store of 128-D features.
//
// Paper Sec. 3.1 (discussion after Table 2): the ConvNet features are very sparse, the 128-D ones
// typically more than three fifths zeros, and a compression built around that sparsity is named
// as a way to shrink the store further.  This store keeps, per row, a presence mask of 128 bits
// and the non-zero fp32 values in ascending order of dimension, rows back to back:
//
//     row i = words [start[i], start[i+1]) of `rows`: 4 mask words (dimension d = bit d mod 32,
//             least significant first, of word d div 32), then one word per set bit
//
// (~225 bytes per row at 60 % zeros against 512 dense).  The score is the dense one,
// s_i = b + sum_d w_d x_{i,d}: the zeros simply never reach the chip.
//
// The stream has no fixed row length, so a wave reads it in fixed WINDOWS instead: 8 KiB (eight
// 16-byte loads per lane) from the 16-byte boundary at or below the first row it has not scored;
// the rows that lie completely inside the window (at most 64 of them, found from the offsets of
// the next 64 rows with one vote) are scored, the next window starts at the first row that did
// not fit.  A row that straddles a window's end is read twice, ~1.4 % of the stream.  A window
// arrives in registers, moves to shared memory, and the same registers take the loads of the next
// window before the current one is scored: 8 KiB per wave stay in flight, and twelve waves per
// compute unit hide the bubble at the start of a tile.  (Two sets of registers, one per window in
// flight, cost 36 more registers and 4 % of the time.)
//
// Scoring a window: its bytes go from registers to a buffer in shared memory that only this wave
// uses.  Eight rows are scored at a time, 8 lanes per row, lane l owning dimensions 16 l .. 16 l + 15:
// it takes its 16 bits of the mask, learns from a prefix sum over the row's lanes (three
// data-parallel moves) how many values precede its own, and reads one value per dimension (a
// cleared bit re-reads the next value and masks it out).  All sums are fp32.
//
// The row offsets a wave needs (64 rows ahead of its position) live in its registers: three
// registers hold start[] for 192 consecutive rows, lane by lane; a window's offsets come out of
// them with lane shuffles, and the third register is refilled from memory a window or more before
// its contents are needed, so no load of an offset ever stands between two windows.
//
// Work distribution: tiles of 1024 rows (256 in the sample scan) from a TileQueue, four tiles per chunk.
#include <algorithm>

#include "otf_internal.h"

namespace otf {

constexpr int kSparseD = 128;
constexpr int kSparseMaskWords = kSparseD / 32;
constexpr int kWinWords = 2048;                       // window: 8 loads x 64 lanes x 4 words
constexpr int kWinBufWords = kWinWords + 8;           // + slack: a lane may read one word past its row's last value
// rows per tile: a tile ends with a window that is only partly its own (the rest is read again by the
// wave that owns the next tile), so long scans take large tiles; the sample's short pieces small ones
template <int EMIT>
constexpr int kSparseTileRows = EMIT == kEmitSample ? 256 : 1024;
constexpr int kSparseThreads = 256;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_shr_u32(uint32_t v) {      // row_shr within 16 lanes, zero shifted in
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}

// What a scan emits, as in the table scans (ScanEmit): all scores + pass-1 histogram; the scores of
// the strided sample (N = number of sample rows, numbered compactly); or only the rows at or above
// the threshold, appended to the candidate list.
template <int EMIT>
__global__ __launch_bounds__(kSparseThreads) void sparse_scan_kernel(
    const uint32_t *__restrict__ rows, const long long *__restrict__ start, long long N, long long store_rows,
    const float *__restrict__ w, float bias, float *__restrict__ scores, SelState *st, uint32_t *hist1,
    const SelState *tau_state, SampleSlot *sample_slots, unsigned long long *__restrict__ cand,
    Gate gate) {
    __shared__ __attribute__((aligned(16))) uint32_t win[kSparseThreads / 64][kWinBufWords];
    // the pass-1 histogram of the scores; a scan that keeps no scores only needs the room once, before
    // its first window, to resolve the threshold: it borrows the windows' buffers
    __shared__ uint32_t lhist_own[EMIT == kEmitScores ? kBins1 : 1];
    static_assert(sizeof(win) >= kBins1 * 4, "the threshold resolution fits the window buffers");
    uint32_t *lhist = EMIT == kEmitScores ? lhist_own : &win[0][0];
    __shared__ uint32_t s_out[3];
    __shared__ TileQueue s_queue;
    if (!gate_open(gate)) return;                 // uniform: this launch is only the fallback of a filtered scan
    uint32_t *chunk_ctr = &st->chunk_ctr[EMIT == kEmitScores ? 1 : 0];
    if (threadIdx.x == 0) tile_queue_init(&s_queue, chunk_ctr);
    const long long total_tiles = (N + kSparseTileRows<EMIT> - 1) / kSparseTileRows<EMIT>;
    const uint32_t chunk_tiles = tile_queue_chunk_tiles(total_tiles, 4u);
    uint32_t tau = 0u;
    if (EMIT == kEmitFilter) {
        const TauChoice tc = resolve_tau_slots(sample_slots, tau_state, store_rows, lhist, s_out);
        if (tc.hopeless) return;                  // uniform
        tau = tc.tau;
    } else {
        for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
    }
    uint32_t smx = 0u, scnt = 0u;                 // sample scan: this lane's largest key and its multiplicity
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l = lane & 7, rq = lane >> 3;       // dimensions 16 l .. 16 l + 15 of row rq of the eight scored together
    uint32_t *buf = win[wave];
    float wl[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) wl[j] = w[16 * l + j];
    // last 16-byte piece of the stream that may be read (the array is padded to whole pieces)
    const long long last_piece = ((start[store_rows] + 3) / 4 - 1) * 4;

    // 8 KiB of the stream from word a0 (a multiple of 4) into registers; pieces past the end re-read the last one
    auto fetch = [&](u32x4 *d, long long a0) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            long long wa = a0 + (long long)u * 256 + (long long)lane * 4;
            wa = wa < last_piece ? wa : last_piece;
            wa = wa < 0 ? 0 : wa;                                   // (offsets that are not what the header asks for: stay inside the array)
            d[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(rows + wa));
        }
    };
    bool list_full = false;
    // scores the nrows rows of a window that is in `d`; rel = first word of this lane's row inside the window
    // (lane r holds it for row r); v0 = number of the window's first row in the output
    auto store_window = [&](const u32x4 *d) {
#pragma unroll
        for (int u = 0; u < 8; ++u) *reinterpret_cast<u32x4 *>(buf + u * 256 + lane * 4) = d[u];
    };
    auto score_window = [&](uint32_t rel, int nrows, long long v0) {
        for (int r0 = 0; r0 < nrows; r0 += 8) {                     // uniform trip count
            const int rl = r0 + rq;
            const bool valid = rl < nrows;
            uint32_t off = (uint32_t)__shfl((int)rel, rl & 63, 64);
            off = valid ? off : 0u;
            const uint32_t mw = buf[off + (uint32_t)(l >> 1)];
            const uint32_t bits16 = (mw >> (16 * (l & 1))) & 0xFFFFu;
            const uint32_t cnt = (uint32_t)__builtin_popcount(bits16);
            uint32_t incl = cnt;                                    // values up to and including this lane's, in the row
            uint32_t t = dpp_shr_u32<0x111>(incl);                  // row_shr:1 (a row of 16 lanes holds two rows of 8:
            incl += l >= 1 ? t : 0u;                                //  what comes from the other one is dropped)
            t = dpp_shr_u32<0x112>(incl);                           // row_shr:2
            incl += l >= 2 ? t : 0u;
            t = dpp_shr_u32<0x114>(incl);                           // row_shr:4
            incl += l >= 4 ? t : 0u;
            uint32_t at = off + (uint32_t)kSparseMaskWords + incl - cnt;
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int m = __builtin_amdgcn_sbfe((int)bits16, j, 1);   // 0, or -1 when dimension 16 l + j is stored
                const float x = __uint_as_float(buf[at] & (uint32_t)m);
                if (j & 1) acc1 = fmaf(wl[j], x, acc1);
                else acc0 = fmaf(wl[j], x, acc0);
                at -= (uint32_t)m;
            }
            float acc = acc0 + acc1;
            acc += dpp_f32<0xB1>(acc);    // quad_perm [1,0,3,2]
            acc += dpp_f32<0x4E>(acc);    // quad_perm [2,3,0,1]
            acc += dpp_f32<0x141>(acc);   // row_half_mirror: every lane of the 8 holds the row's sum
            if (valid && l == 0) {
                const float sc = acc + bias;
                const long long v = v0 + rl;
                if (EMIT == kEmitSample) {
                    sample_note(smx, scnt, float_to_key(sc));
                } else if (EMIT == kEmitFilter) {
                    const uint32_t key = float_to_key(sc);
                    if (key >= tau && !list_full) {
                        const uint32_t pos = atomicAdd(&st->cursor, 1u);
                        if (pos < (uint32_t)kCandCap)
                            cand[pos] = ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)v);
                        else
                            list_full = true;
                    }
                } else {
                    atomicAdd(&lhist[float_to_key(sc) >> 20], 1u);
                    scores[v] = sc;
                }
            }
        }
        if (EMIT == kEmitFilter) list_full = __ballot(list_full) != 0ull;
    };

    for (;;) {
        const long long tile = tile_queue_draw(&s_queue, chunk_ctr, chunk_tiles, total_tiles);
        if (tile < 0) break;                                        // uniform per wave
        // output rows [v, ve) of this tile are store rows [r, r + ve - v) (the sample: a piece of one group)
        long long v = tile * kSparseTileRows<EMIT>;
        const long long ve = v + kSparseTileRows<EMIT> < N ? v + kSparseTileRows<EMIT> : N;
        long long r = EMIT == kEmitSample ? ((v >> 10) * ((long long)kSampleGroup * kSampleStride) + (v & 1023)) : v;
        const long long re = r + (ve - v);
        // start[] of rows rb + lane, rb + 64 + lane, rb + 128 + lane (capped at the tile's end, whose
        // offset closes its last row)
        long long rb = r;
        auto load_starts = [&](long long first) {
            const long long i = first + lane < re ? first + lane : re;
            return start[i];
        };
        long long S0 = load_starts(rb), S1 = load_starts(rb + 64), S2 = load_starts(rb + 128);
        // start[row + i] for lane i (i = 0..63) and one row further, rb <= row < rb + 64
        auto offsets_from = [&](long long row, long long *s0, long long *s1) {
            const int i0 = (int)(row - rb) + lane, i1 = i0 + 1;
            const long long a = __shfl(S0, i0 & 63, 64), b = __shfl(S1, i0 & 63, 64);
            const long long c = __shfl(S0, i1 & 63, 64), d2 = __shfl(S1, i1 & 63, 64);
            *s0 = i0 < 64 ? a : b;
            *s1 = i1 < 64 ? c : d2;
        };
        // a window: which rows fit, where each begins inside it, and where the window after it begins
        struct Win {
            long long a0;        // first word of the window (a multiple of 4)
            uint32_t rel;        // lane i: first word of row (window's first row + i) inside the window
            int nrows;           // rows that lie completely inside it (>= 1)
            long long next_a0;   // the window of the first row that did not fit
        };
        auto plan = [&](long long row, long long a0) {
            if (row - rb >= 64) {                                   // uniform: the registers move on by 64 rows
                rb += 64;
                S0 = S1;
                S1 = S2;
                S2 = load_starts(rb + 128);                         // needed a window from now at the earliest
            }
            long long s0, s1;
            offsets_from(row, &s0, &s1);
            Win p;
            p.a0 = a0;
            const bool fits = (row + lane < re) && (s1 - a0 <= (long long)kWinWords);
            p.nrows = __builtin_popcountll(__ballot(fits));         // rows are consecutive: the fitting ones come first
            // A row of 128 dimensions always fits a window.  Offsets that claim otherwise (not ascending, or
            // rows longer than the format allows) must not stall the scan: it moves on by one row, and that
            // row's score is whatever the window holds.
            p.nrows = p.nrows < 1 ? 1 : p.nrows;
            p.rel = (uint32_t)(s0 - a0);
            const long long nxt = __shfl(s1, (p.nrows - 1) & 63, 64);   // = start[row + nrows]
            p.next_a0 = nxt & ~3LL;
            return p;
        };
        // One set of registers holds a window on its way in.  Once it has arrived it moves to the wave's
        // buffer in shared memory, the registers take the loads of the NEXT window, and the current one
        // is scored from shared memory while those are in flight.
        u32x4 b[8];
        const long long first_a0 = __shfl(S0, 0, 64) & ~3LL;
        Win cur = plan(r, first_a0);
        fetch(b, cur.a0);
        for (;;) {
            const bool more = r + cur.nrows < re;
            Win nxt = cur;
            if (more) nxt = plan(r + cur.nrows, cur.next_a0);       // uniform
            store_window(b);
            fetch(b, more ? nxt.a0 : cur.a0);
            score_window(cur.rel, cur.nrows, v);
            if (!more) break;
            v += cur.nrows;
            r += cur.nrows;
            cur = nxt;
        }
    }
    if (EMIT == kEmitScores) merge_hist1(lhist, hist1);
    if (EMIT == kEmitSample) sample_store(sample_slots, st, smx, scnt);
}

template <int EMIT>
static hipError_t launch_sparse_cfg(const uint32_t *rows, const int64_t *start, int64_t N, int64_t store_rows,
                                    const float *w, float bias, float *scores, SelState *st, uint32_t *hist1,
                                    const SelState *tau, SampleSlot *slots, unsigned long long *cand,
                                    Gate gate, hipStream_t s) {
    const int64_t tiles = (N + kSparseTileRows<EMIT> - 1) / kSparseTileRows<EMIT>;
    // three workgroups per compute unit: with one or two the kernel takes 2.2x and 1.3x as long, and a
    // fourth (the registers would allow it) makes it 3 % slower: the shared-memory unit is the limit
    const int grid = (int)std::min<int64_t>((tiles + 3) / 4, (int64_t)device_cu_count() * 3);
    sparse_scan_kernel<EMIT><<<grid < 1 ? 1 : grid, kSparseThreads, 0, s>>>(
        rows, reinterpret_cast<const long long *>(start), (long long)N, (long long)store_rows, w, bias, scores, st, hist1,
        tau, slots, cand, gate);
    return hipGetLastError();
}

// N = rows to score (kEmitSample: the sample rows, compact numbering); store_rows = rows of the store.
hipError_t launch_sparse_scan(const uint32_t *rows, const int64_t *start, int64_t N, int64_t store_rows, const float *w,
                              float bias, ScanEmit emit, float *scores, SelState *st, uint32_t *hist1,
                              const SelState *tau, SampleSlot *slots, unsigned long long *cand, Gate gate,
                              hipStream_t s) {
    switch (emit) {
        case kEmitScores:
            return launch_sparse_cfg<kEmitScores>(rows, start, N, store_rows, w, bias, scores, st, hist1, tau, slots, cand, gate, s);
        case kEmitSample:
            return launch_sparse_cfg<kEmitSample>(rows, start, N, store_rows, w, bias, scores, st, hist1, tau, slots, cand, gate, s);
        default:
            return launch_sparse_cfg<kEmitFilter>(rows, start, N, store_rows, w, bias, scores, st, hist1, tau, slots, cand, gate, s);
    }
}

}  // namespace otf
