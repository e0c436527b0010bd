// Byte-indexed table scans: product-quantised codes and binary codes.
//
// PQ (paper Sec. 3, "Product quantization (PQ)"; Table 2: one byte per sub-block): the score of
// a coded row is sum_m lut[m][code_m] with lut[m][k] = <w_m, centre_k of sub-block m>.
// Binary (paper Sec. 3, "Binarization", Eq. (1)): the score is sum_d w_d (2 bit_d - 1).  A group
// of g consecutive dimensions forms an index v into the table
//     T[group][v] = sum_{j<g} (bit j of v ? +w[first + j] : -w[first + j])
// so the score is a sum of table entries: the same scan as PQ.  One lookup replaces g signed
// adds, which keeps the scan below the vector-ALU ceiling.  Rows of up to 1024 bits use byte
// groups (256-entry tables, 128 columns: 128 KiB of shared memory).  Rows of 2048 bits would need
// 256 KiB that way, so each 32-bit word is cut into four 7-bit groups and one 4-bit group
// instead: 256 columns of 128 entries plus 64 columns of 16 entries, 132 KiB, one pass per row.
//
// Both scans are one shared-memory gather per group.  To keep the gathers free of bank conflicts
// whatever the data, the table is stored value-major, image[v][column], so that the bank of an
// access depends only on WHICH group of the row is looked up, never on its value, and lanes that
// execute the same instruction always look up different columns:
//   * every lane loads 16 consecutive bytes of a row (4 words); 8 adjacent lanes cover 128 bytes;
//   * group j of word tq of lane-chunk c lives in column (groups per word-column block)*tq + 4*c + j;
//   * the four lane octets that execute together (lanes 0..31, and 32..63) read their words with
//     four different group rotations (j = step ^ octet), so at every step the 32 lanes touch
//     columns 4*c + j with all 32 (c, j) pairs distinct: 32 lanes, 32 banks.
// Rows shorter than 128 bytes are packed several to a 128-byte segment (the table columns
// repeat; a row length that is not a power of two leaves the last lanes of its group idle, their
// table columns zero).  Byte-group rows longer than 128 bytes (PQ with more than 128 sub-blocks:
// the paper's own 4 or 8 dimensions per sub-block on 2048-D features; binary codes beyond 2048
// bits) do not fit one table image: table_walk_kernel takes a block of rows through `nphase` column
// phases of 128 bytes, reloading the image between phases and keeping the partial sums in registers.
//
// What a scan emits is a template parameter (ScanEmit): all scores plus the pass-1 histogram of
// the selection; the scores of a strided sample of the rows; or, given a threshold, only the
// rows at or above it, appended to a candidate list.  The last mode writes almost nothing, which
// matters: interleaving even 3 % of score stores with the row stream costs ~20 % of HBM rate.
#include "otf_internal.h"

namespace otf {

constexpr int kSegBytes = 128;                       // row bytes handled per phase (byte groups)
constexpr int kImageFloats = 256 * kSegBytes;        // one table image: 256 values x 128 columns
constexpr int kImageBytes = kImageFloats * 4;        // 128 KiB
constexpr int kSideFloats = 16 * 128;                // 4-bit groups of a 2048-bit row: 16 values x 64 words, twice
constexpr int kImage7Bytes = kImageBytes + kSideFloats * 4;   // 7-bit groups: 128 values x 256 columns, + side
constexpr int kScanMaxThreads = 1024;
constexpr int kScanThreads = 1024;    // 16 waves per CU overlap the gathers with the row stream best

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

// Zeroes both selection states (full selection and sample thresholding) of one classifier.
__device__ __forceinline__ void zero_states(int tid, int step, SelState *st, uint32_t *hist1, uint32_t *hist2,
                                            uint32_t *hist3, SelState *sst) {
    uint32_t *stw = reinterpret_cast<uint32_t *>(st), *sstw = reinterpret_cast<uint32_t *>(sst);
    for (int i = tid; i < (int)(sizeof(SelState) / 4); i += step) {
        stw[i] = 0u;
        sstw[i] = 0u;
    }
    for (int i = tid; i < kHist1Words; i += step) hist1[i] = 0u;
    for (int i = tid; i < kBins2; i += step) hist2[i] = 0u;
    for (int i = tid; i < kBins3; i += step) hist3[i] = 0u;
}

// Which byte of a row sits at position pos of the 128-byte segment of phase sp, or -1 for none.
// Rows of 128 bytes or more: byte 128 sp + pos while it exists (the last phase of a row length that
// is not a multiple of 128 is partly empty).  Shorter rows: a row occupies `span` = 16, 32, 64 or
// 128 bytes of the segment (the next power of two), several rows side by side, and the bytes of the
// span beyond the row are empty.  Empty positions get zero table columns.
__device__ __forceinline__ int row_byte_at(int row_bytes, int span, int sp, int pos) {
    const int g = row_bytes >= kSegBytes ? sp * kSegBytes + pos : pos % span;
    return g < row_bytes ? g : -1;
}

// Table images for PQ: image[sp][v][column(pos)] = lut[m][v] with m = row_byte_at(...).  Also zeroes
// the selection states (one launch instead of two).
__global__ __launch_bounds__(256) void pq_prepare_kernel(const float *__restrict__ lut, int M, int span, int nsplit,
                                                         float *__restrict__ image, SelState *st, uint32_t *hist1,
                                                         uint32_t *hist2, uint32_t *hist3, SelState *sst) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, step = gridDim.x * blockDim.x;
    for (int t = tid; t < nsplit * kImageFloats; t += step) {
        const int v = t & 255, pos = (t >> 8) & (kSegBytes - 1), sp = t >> 15;
        const int m = row_byte_at(M, span, sp, pos);
        image[(size_t)sp * kImageFloats + v * kSegBytes + image_column(pos)] = m >= 0 ? lut[(size_t)m * 256 + v] : 0.f;
    }
    zero_states(tid, step, st, hist1, hist2, hist3, sst);
}

// The same straight from the vocabularies and the model, for a caller that ranks under a new model
// every time and has no use for the table itself: image entry = sum_j w[m dsub + j] C[m][v][j], summed
// in the order of pq_build_lut_kernel (the two routes give identical bits).
__global__ __launch_bounds__(256) void pq_prepare_model_kernel(const float *__restrict__ codebooks,
                                                               const float *__restrict__ w, int M, int dsub, int span,
                                                               int nsplit, float *__restrict__ image, SelState *st,
                                                               uint32_t *hist1, uint32_t *hist2, uint32_t *hist3,
                                                               SelState *sst) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, step = gridDim.x * blockDim.x;
    for (int t = tid; t < nsplit * kImageFloats; t += step) {
        const int v = t & 255, pos = (t >> 8) & (kSegBytes - 1), sp = t >> 15;
        const int m = row_byte_at(M, span, sp, pos);
        float acc = 0.f;
        if (m >= 0) {
            const float *c = codebooks + ((size_t)m * 256 + v) * dsub;
            const float *wm = w + (size_t)m * dsub;
            for (int j = 0; j < dsub; ++j) acc = fmaf(wm[j], c[j], acc);
        }
        image[(size_t)sp * kImageFloats + v * kSegBytes + image_column(pos)] = acc;
    }
    zero_states(tid, step, st, hist1, hist2, hist3, sst);
}

// Table images for binary codes with byte groups: byte g of a row covers dimensions 8g..8g+7.
__global__ __launch_bounds__(256) void binary_prepare_kernel(const float *__restrict__ w, int row_bytes, int span,
                                                             int nsplit, float *__restrict__ image, SelState *st,
                                                             uint32_t *hist1,
                                                             uint32_t *hist2, uint32_t *hist3, SelState *sst) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, step = gridDim.x * blockDim.x;
    for (int t = tid; t < nsplit * kImageFloats; t += step) {
        const int v = t & 255, pos = (t >> 8) & (kSegBytes - 1), sp = t >> 15;
        const int g = row_byte_at(row_bytes, span, sp, pos);
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float wd = g >= 0 ? w[g * 8 + j] : 0.f;
            acc += ((v >> j) & 1) ? wd : -wd;
        }
        image[(size_t)sp * kImageFloats + v * kSegBytes + image_column(pos)] = acc;
    }
    zero_states(tid, step, st, hist1, hist2, hist3, sst);
}

// Table image for 2048-bit rows: word q (0..63) of a row = lane-chunk q/4, word tq = q%4 of the chunk.
//   main[v][64*tq + 4*chunk + j]  (v < 128)  group j of the word: dimensions 32q + 7j .. 32q + 7j + 6
//   side[v][32*tq + 8*o + c]      (v < 16)   the top four bits:   dimensions 32q + 28 .. 32q + 31 of word
//        q = 4*chunk + tq, chunk = c + 8*(o & 1).  o is the lane octet (0..3) that reads the entry:
//        octets 0 and 2 hold the same chunks, as do 1 and 3, so every word is stored twice and the
//        32 lanes that execute together (4 octets x 8 chunks) read 32 different banks.  (A plain
//        side[v][q] makes every side read a 4-way bank conflict: 37 % of the kernel's LDS cycles.)
__global__ __launch_bounds__(256) void binary7_prepare_kernel(const float *__restrict__ w, float *__restrict__ image,
                                                              SelState *st, uint32_t *hist1, uint32_t *hist2,
                                                              uint32_t *hist3, SelState *sst) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, step = gridDim.x * blockDim.x;
    for (int t = tid; t < 128 * 256; t += step) {
        const int v = t & 127, col = t >> 7;              // col = 4*q + j
        const int q = col >> 2, j = col & 3;
        float acc = 0.f;
#pragma unroll
        for (int b = 0; b < 7; ++b) {
            const float wd = w[32 * q + 7 * j + b];
            acc += ((v >> b) & 1) ? wd : -wd;
        }
        const int chunk = q >> 2, tq = q & 3;
        image[v * 256 + 64 * tq + 4 * chunk + j] = acc;
    }
    for (int t = tid; t < kSideFloats; t += step) {
        const int c = t & 7, o = (t >> 3) & 3, tq = (t >> 5) & 3, v = t >> 7;
        const int q = 4 * (c + 8 * (o & 1)) + tq;
        float acc = 0.f;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const float wd = w[32 * q + 28 + b];
            acc += ((v >> b) & 1) ? wd : -wd;
        }
        image[kImageFloats + t] = acc;
    }
    zero_states(tid, step, st, hist1, hist2, hist3, sst);
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over groups of LPR adjacent lanes (a power of two up to 64); every lane of a group receives it.
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
    if (LPR >= 2) v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
    if (LPR >= 4) v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
    if (LPR >= 8) v += dpp_move<0x141>(v);   // row_half_mirror: lane i <-> 7 - i of each 8
    if (LPR >= 16) v += dpp_move<0x140>(v);  // row_mirror: lane i <-> 15 - i of each 16
    if (LPR >= 32) v += __shfl_xor(v, 16, 64);
    if (LPR >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The 16 lookups of one 16-byte load (4 words x 4 groups; GB == 7: plus the 4 side lookups of the
// words' top bits), summed over the lane group of LPR lanes that shares a row.
//   shift[t], colbyte[t]  bit offset and table column (as a byte offset) of the group this lane
//                         looks up at step t of a word: the four lane octets that execute together
//                         rotate the order, so that 32 lanes always hit 32 banks
template <int LPR, int GB>
__device__ __forceinline__ float lookup16(const uint8_t *lds, const uint32_t (&d)[4], const uint32_t (&shift)[4],
                                          const uint32_t (&colbyte)[4], uint32_t sidecol) {
    constexpr int VSHIFT = GB == 8 ? 9 : 10;       // log2 of the byte stride between table values
    constexpr int TQ_BYTES = GB == 8 ? 128 : 256;  // byte distance between the column blocks of the 4 words
    uint32_t addr[16];
#pragma unroll
    for (int tq = 0; tq < 4; ++tq)
#pragma unroll
        for (int t = 0; t < 4; ++t)
            addr[4 * tq + t] = (__builtin_amdgcn_ubfe(d[tq], shift[t], (uint32_t)GB) << VSHIFT) + colbyte[t];
    float v[16];
#pragma unroll
    for (int tq = 0; tq < 4; ++tq)
#pragma unroll
        for (int t = 0; t < 4; ++t)
            v[4 * tq + t] = *reinterpret_cast<const float *>(lds + addr[4 * tq + t] + TQ_BYTES * tq);
    if (GB == 7) {
#pragma unroll
        for (int tq = 0; tq < 4; ++tq)
            v[4 * tq] += *reinterpret_cast<const float *>(lds + ((d[tq] >> 28) << 9) + sidecol + 128 * tq);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] += v[i + 8];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] += v[i + 4];
    return group_sum<LPR>((v[0] + v[1]) + (v[2] + v[3]));
}

// Hamming ranking (paper Sec. 3.1, discussion after Table 2: binary codes can be ranked by
// hardware-accelerated Hamming distance): the contribution of one 16-byte load is minus the number
// of bits in which it differs from the query's bytes at the same position (XOR, population count),
// summed over the lane group that shares a row.  Small integers: every sum is exact in fp32.
template <int LPR>
__device__ __forceinline__ float hamming16(const uint32_t (&d)[4], const uint32_t (&q)[4], bool live) {
    int c = __builtin_popcount(d[0] ^ q[0]) + __builtin_popcount(d[1] ^ q[1]) + __builtin_popcount(d[2] ^ q[2]) +
            __builtin_popcount(d[3] ^ q[3]);
    return group_sum<LPR>(live ? -(float)c : 0.f);
}

// One row that a scan has finished: append it to the candidate list when it is at or above the
// threshold (filtered scan), else store its score and count it in the pass-1 histogram.
// Filtered scan: a wave that has seen the list full stops appending (the list is already
// useless, and the appends are adds to one address, ~18 ns each one after the other: a
// threshold that lets a million rows pass would otherwise cost tens of milliseconds).
// Sample scan: the row only competes for the wave's largest key (sample_note).
template <int EMIT>
__device__ __forceinline__ void emit_row(float score, long long v, uint32_t tau, bool &list_full, SelState *st,
                                         unsigned long long *__restrict__ cand, float *__restrict__ scores,
                                         uint32_t *lhist, uint32_t &smx, uint32_t &scnt) {
    if (EMIT == kEmitSample) {
        sample_note(smx, scnt, float_to_key(score));
    } else if (EMIT == kEmitFilter) {
        const uint32_t key = float_to_key(score);
        if (key >= tau && !list_full) {
            const uint32_t pos = atomicAdd(&st->cursor, 1u);
            if (pos < (uint32_t)kCandCap)
                cand[pos] = ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)v);
            else
                list_full = true;
        }
    } else {
        atomicAdd(&lhist[float_to_key(score) >> 20], 1u);
        scores[v] = score;
    }
}

// For the sample scan the rows are numbered compactly: sample row v is store row
// (v / 1024) * 1024 * stride + v % 1024 (a tile never straddles a group: its rows divide 1024).
template <int EMIT>
__device__ __forceinline__ long long store_row(long long v) {
    return EMIT == kEmitSample ? ((v >> 10) * ((long long)kSampleGroup * kSampleStride) + (v & 1023)) : v;
}

// Scan of rows that fit one table image.
//   GB     bits per group: 8 (bytes; LPR = 1, 2, 4 or 8 lanes per row: the row occupies a span of
//          16 LPR bytes of which the first M are stored), 7 (2048-bit rows, LPR = 16, each
//          word = 4 x 7 bits + 4 bits), or 0: no table at all, the score is minus the Hamming
//          distance to the query code that `image` then points at (LPR up to 64: rows up to 8192 bits)
//   U      16-byte loads per lane per tile
//   EMIT   what is produced (ScanEmit)
//
// A tile is what one wave looks up per iteration: U loads of 64 lanes x 16 bytes.  The main loop
// is software-pipelined: the loads of the wave's next tile are issued before the current tile is
// looked up, and a prefetch with nothing left to fetch re-reads the current tile rather than
// being skipped (an unconditional load keeps the in-order wait counters exact).  After the
// lookups the U row sums of a lane group are moved into U different lanes so that the output
// step happens once per tile, not per row.
//
// Work distribution: dynamic, by a TileQueue with chunks of 256 KiB of rows.
template <int LPR, int U, int GB, int EMIT>
__global__ __launch_bounds__(kScanMaxThreads) void table_scan_kernel(
    const uint8_t *__restrict__ codes, long long N, int M, const float *__restrict__ image, float bias,
    float *__restrict__ scores, SelState *st, uint32_t *hist1, const SelState *tau_state,
    SampleSlot *sample_slots, unsigned long long *__restrict__ cand, Gate gate) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    __shared__ uint32_t lhist[EMIT == kEmitScores ? kBins1 : 1];
    __shared__ uint32_t s_out[3];
    __shared__ TileQueue s_queue;
    if (!gate_open(gate)) return;                 // uniform: this launch is only the fallback of a filtered scan
    constexpr int RPW = 64 / LPR;                // rows per wave load
    constexpr int TILE = RPW * U;                // rows per wave iteration
    constexpr int ACTIVE = LPR < U ? LPR : U;    // lanes of a group that own an output row per round
    constexpr int ROUNDS = U / ACTIVE;           // output rounds per tile
    constexpr int TABLE_VEC = (GB == 8 ? kImageBytes : GB == 7 ? kImage7Bytes : 0) / 16;
    constexpr uint32_t CHUNK_TILES = 256u / (uint32_t)U;          // x U KiB per tile = 256 KiB of rows

    // the two scans that can follow each other on one state (filtered, then the gated full scan)
    // count in different words; both were zeroed with the state
    uint32_t *chunk_ctr = &st->chunk_ctr[EMIT == kEmitScores ? 1 : 0];
    if (threadIdx.x == 0) tile_queue_init(&s_queue, chunk_ctr);   // visible after the barriers below
    const uint32_t chunk_tiles = tile_queue_chunk_tiles(N / TILE, CHUNK_TILES);

    if (EMIT == kEmitScores)
        for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
    // Filtered scan: every block resolves the threshold from the wave maxima the sample scan left
    // (the table area of shared memory is still free at this point).
    uint32_t tau = 0u;
    if (EMIT == kEmitFilter) {
        const TauChoice tc = resolve_tau_slots(sample_slots, tau_state, N, reinterpret_cast<uint32_t *>(lds_raw), s_out);
        if (tc.hopeless) return;                  // uniform
        tau = tc.tau;
    }
    uint32_t smx = 0u, scnt = 0u;                 // sample scan: this lane's largest key and its multiplicity

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = GB == 8 ? (lane & 7) : (lane & 15);   // 16-byte chunk inside the table's row span
    const int octet = (lane >> 3) & 3;                       // which of the 4 lane octets that execute together
    const int sub = lane % LPR, rr = lane / LPR;             // chunk inside the row, row inside the wave load
    uint32_t shift[4], colbyte[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int j = t ^ octet;
        shift[t] = (uint32_t)(GB * j);
        colbyte[t] = 4u * (uint32_t)(4 * chunk + j);
    }
    const uint32_t sidecol = (uint32_t)(kImageBytes + 4 * (8 * octet + (chunk & 7)));   // GB == 7 only
    // GB == 0: the query's 16 bytes at this lane's position in the row (none: the lane is idle)
    const bool q_live = (uint32_t)sub * 16u < (uint32_t)M;
    uint32_t q4[4] = {0u, 0u, 0u, 0u};
    if (GB == 0 && q_live) {
#pragma unroll
        for (int t = 0; t < 4; ++t) q4[t] = reinterpret_cast<const uint32_t *>(image)[4 * sub + t];
    }

    const size_t u_bytes = (size_t)RPW * (size_t)M;        // distance between the U loads of a lane
    const int out_u = sub % ACTIVE;                        // which of a round's rows this lane emits

    // looks up the U loads of a tile; the U row sums of a lane group (every lane of the group
    // holds each sum) are kept by U different lanes: lane out_u keeps row e*ACTIVE + out_u
    auto tile_sums = [&](const u32x4 *d, float *mine) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t w4[4] = {d[u][0], d[u][1], d[u][2], d[u][3]};
            const float su = GB == 0 ? hamming16<LPR>(w4, q4, q_live) : lookup16<LPR, GB == 0 ? 8 : GB>(lds_raw, w4, shift, colbyte, sidecol);
            if (u % ACTIVE == 0) mine[u / ACTIVE] = su;
            else mine[u / ACTIVE] = out_u == (u % ACTIVE) ? su : mine[u / ACTIVE];
        }
    };
    // compact row that lane `sub` of its group emits in round e of the tile starting at row v0
    auto out_row = [&](long long v0, int e) { return v0 + (long long)(e * ACTIVE + out_u) * RPW + rr; };

    {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(image);
        u32x4 *dst = reinterpret_cast<u32x4 *>(lds_raw);
        for (int i = threadIdx.x; i < TABLE_VEC; i += blockDim.x) dst[i] = src[i];
    }
    __syncthreads();

    // one output round: lane `sub` of each group holds in `mine` the sum of the row it owns
    bool list_full = false;
    auto emit = [&](float mine, long long v, bool ok) {
        if (sub < ACTIVE && ok) emit_row<EMIT>(mine + bias, v, tau, list_full, st, cand, scores, lhist, smx, scnt);
    };

    // first row of the next tile of this wave, or -1 when the scan has no full tile left
    // (the rows after the last full tile are handled at the end)
    auto draw = [&]() -> long long {
        const long long t = tile_queue_draw(&s_queue, chunk_ctr, chunk_tiles, N / TILE);
        return t < 0 ? t : t * TILE;
    };
    // uniform base of the tile (scalar registers) + one 32-bit lane offset.  A row shorter than
    // the span of its lane group leaves the group's last lanes without bytes of their own: they
    // re-read the row's first bytes (their table columns are zero).
    const uint32_t lane_off = (uint32_t)rr * (uint32_t)M + ((uint32_t)sub * 16u < (uint32_t)M ? (uint32_t)sub * 16u : 0u);
    auto fetch = [&](u32x4 *d, long long v0) {
        const unsigned long long a = (unsigned long long)store_row<EMIT>(v0) * (unsigned long long)M;
        // (the builtin returns int: go through uint32_t, or offsets past 2 GiB are sign-extended)
        const uint32_t a_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
        const uint32_t a_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
        const uint8_t *p = codes + (((unsigned long long)a_hi << 32) | (unsigned long long)a_lo);
#pragma unroll
        for (int u = 0; u < U; ++u)
            d[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + (size_t)u * u_bytes + (size_t)lane_off));
    };
    auto consume = [&](const u32x4 *d, long long v0) {
        float mine[ROUNDS];
        tile_sums(d, mine);
#pragma unroll
        for (int e = 0; e < ROUNDS; ++e) emit(mine[e], out_row(v0, e), true);
        if (EMIT == kEmitFilter) list_full = __ballot(list_full) != 0ull;   // one lane's news serves the wave
    };
    long long cur = draw();
    if (cur >= 0) {
        u32x4 b0[U], b1[U];
        fetch(b0, cur);
        for (;;) {
            long long nxt = draw();
            fetch(b1, nxt >= 0 ? nxt : cur);
            consume(b0, cur);
            if (nxt < 0) break;
            cur = nxt;
            nxt = draw();
            fetch(b0, nxt >= 0 ? nxt : cur);
            consume(b1, cur);
            if (nxt < 0) break;
            cur = nxt;
        }
    }
    // the rows after the last full tile (fewer than a tile): one wave, row-checked
    const long long v0 = N / TILE * TILE;
    if (v0 < N && blockIdx.x == 0 && wave == 0) {
        u32x4 d[U];
        float mine[ROUNDS];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long v = v0 + (long long)u * RPW + rr;
            d[u] = (u32x4){0u, 0u, 0u, 0u};
            if (v < N)
                d[u] = *reinterpret_cast<const u32x4 *>(codes + (size_t)store_row<EMIT>(v - rr) * (size_t)M + (size_t)lane_off);
        }
        tile_sums(d, mine);
#pragma unroll
        for (int e = 0; e < ROUNDS; ++e) {
            const long long v = out_row(v0, e);
            emit(mine[e], v, v < N);
        }
    }
    if (EMIT == kEmitScores) merge_hist1(lhist, hist1);
    if (EMIT == kEmitSample) sample_store(sample_slots, st, smx, scnt);
}

// Scan of byte-group rows longer than 128 bytes: nphase = ceil(row_bytes / 128) column phases, each
// with a table image of its own, and room in shared memory for one image.
//
// A workgroup draws blocks of R = waves x 64 x TPW consecutive rows from a counter in global
// memory and walks each block through all phases.  In phase p every wave reads bytes
// 128 p .. 128 p + 127 of its TPW tiles of 64 rows (8 lanes per row, 8 loads per lane, as in the
// one-image scan) and adds the 128 lookups per row to partial sums that stay in registers: lane
// (row slot rr, chunk c) of a wave owns row 8 c + rr of each of its tiles.  Nothing but the final
// scores (or candidates) ever leaves the chip: one launch, no partial sums in memory, so these
// rows take the sampled, filtered route like the short ones.
//
// Between two phases the image is replaced: barrier (everybody is done with the old one), 128
// KiB from L2 straight into shared memory (global_load_lds, no registers), wait, barrier.  The
// row stream must not stop meanwhile.  The loads of a wave return in order, so the loads of the
// tile after next are issued behind the image loads and the wait is for "all but the youngest
// 8": the image and the tile about to be looked up have landed, the next tile stays in flight
// across both barriers.  (Scheduling barriers pin that order in the instruction stream.)
//
// The number of the next block is ordered one block ahead by thread 0 and handed round through
// shared memory at the phase-1 barrier; every wave of a workgroup walks the same sequence of
// blocks and phases, so all of them meet at every barrier.  A tile at or behind the end of the
// store reads the store's last 64 rows and emits only what is its own (N >= 64: the caller copies
// a shorter store into a 64-row buffer).  A last phase narrower than 128 bytes leaves the
// lanes beyond it without bytes of their own: they re-read the phase's first bytes, and the table
// columns they look up are zero.
template <int EMIT, int TPW>
__global__ __launch_bounds__(kScanMaxThreads) void table_walk_kernel(
    const uint8_t *__restrict__ codes, long long N, int row_bytes, int nphase, const float *__restrict__ image,
    float bias, float *__restrict__ scores, SelState *st, uint32_t *hist1, const SelState *tau_state,
    SampleSlot *sample_slots, unsigned long long *__restrict__ cand, Gate gate) {
    static_assert(TPW % 2 == 0, "tiles alternate between two register buffers");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    __shared__ uint32_t lhist[EMIT == kEmitScores ? kBins1 : 1];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_blk[4];                 // ring: number of the workgroup's j-th block at slot j % 4
    if (!gate_open(gate)) return;                 // uniform: this launch is only the fallback of a filtered scan
    constexpr int U = 8, RPW = 8, TILE = 64;
    const int tid = threadIdx.x, lane = tid & 63, nwaves = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: tile addresses are uniform
    const long long R = (long long)nwaves * TILE * TPW;
    const long long nblocks = (N + R - 1) / R;
    uint32_t *blk_ctr = &st->chunk_ctr[EMIT == kEmitScores ? 1 : 0];
    if (tid == 0) s_blk[0] = atomicAdd(blk_ctr, 1u);

    if (EMIT == kEmitScores)
        for (int b = tid; b < kBins1; b += blockDim.x) lhist[b] = 0u;
    uint32_t tau = 0u;
    if (EMIT == kEmitFilter) {                    // as in table_scan_kernel (the image area is still free)
        const TauChoice tc = resolve_tau_slots(sample_slots, tau_state, N, reinterpret_cast<uint32_t *>(lds_raw), s_out);
        if (tc.hopeless) return;                  // uniform
        tau = tc.tau;
    }
    uint32_t smx = 0u, scnt = 0u;                 // sample scan: this lane's largest key and its multiplicity
    __syncthreads();

    const int sub = lane & 7, rr = lane >> 3, octet = (lane >> 3) & 3;
    uint32_t shift[4], colbyte[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int j = t ^ octet;
        shift[t] = (uint32_t)(8 * j);
        colbyte[t] = 4u * (uint32_t)(4 * sub + j);
    }
    // byte offset of this lane's chunk inside a phase; in a narrower last phase the lanes beyond it
    // read its first chunk instead
    const uint32_t last_width = (uint32_t)(row_bytes - (nphase - 1) * kSegBytes);
    const uint32_t sub_off = (uint32_t)sub * 16u, sub_off_last = sub_off < last_width ? sub_off : 0u;
    const size_t u_bytes = (size_t)RPW * (size_t)row_bytes;
    // Barrier between the waves of the workgroup that orders shared-memory traffic only: this wave's
    // shared-memory operations have completed, global loads stay in flight across it
    // (__syncthreads() would wait for them all).
    auto lds_barrier = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    // first row of tile t of block b for this wave: the waves of a workgroup read 1024 consecutive rows
    auto tile_row0 = [&](long long b, int t) { return b * R + ((long long)t * nwaves + wave) * TILE; };
    // A tile that holds the end of the store, or lies behind it, reads the store's last 64 rows
    // instead (the caller guarantees 64 readable rows): the window moves, the loads stay whole and
    // their base uniform; rows in front of the tile's own first row are not emitted again.
    auto window = [&](long long v0) { return v0 < N - TILE ? v0 : N - TILE; };
    const uint32_t lane_off = (uint32_t)rr * (uint32_t)row_bytes + sub_off;
    const uint32_t lane_off_last = (uint32_t)rr * (uint32_t)row_bytes + sub_off_last;
    auto fetch = [&](u32x4 *d, long long v0, int p) {
        const unsigned long long a = (unsigned long long)store_row<EMIT>(window(v0)) * (unsigned long long)row_bytes +
                                     (unsigned long long)p * kSegBytes;
        // (the builtin returns int: go through uint32_t, or offsets past 2 GiB are sign-extended)
        const uint32_t a_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
        const uint32_t a_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
        const uint8_t *base = codes + (((unsigned long long)a_hi << 32) | (unsigned long long)a_lo);
        const uint32_t lo = p == nphase - 1 ? lane_off_last : lane_off;
#pragma unroll
        for (int u = 0; u < U; ++u)
            d[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base + (size_t)u * u_bytes + (size_t)lo));
    };
    // the sum over this phase's 128 columns of the row this lane owns in the tile (row 8 sub + rr)
    auto tile_sum = [&](const u32x4 *d) {
        float mine = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t w4[4] = {d[u][0], d[u][1], d[u][2], d[u][3]};
            const float su = lookup16<8, 8>(lds_raw, w4, shift, colbyte, 0u);
            mine = (u == 0 || sub == u) ? su : mine;
        }
        return mine;
    };
    // image of phase p: 128 KiB, 1 KiB per wave instruction, the waves taking the KiB in turn
    auto copy_image = [&](int p) {
        const uint8_t *src = reinterpret_cast<const uint8_t *>(image) + (size_t)p * kImageBytes;
        for (int j = wave; j < kImageBytes / 1024; j += nwaves)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src + j * 1024 + lane * 16),
                                             (__attribute__((address_space(3))) void *)(lds_raw + j * 1024), 16, 0, 0);
    };

    // part[i] <- part[i + 2], the first two to the end
    auto turn_ring = [&](float *part) {
        const float x0 = part[0], x1 = part[1];
#pragma unroll
        for (int i = 0; i + 2 < TPW; ++i) part[i] = part[i + 2];
        part[TPW - 2] = x0;
        part[TPW - 1] = x1;
    };

    long long blk = s_blk[0];
    if (blk >= nblocks) {                          // uniform: nothing for this workgroup
        if (EMIT == kEmitScores) merge_hist1(lhist, hist1);
        if (EMIT == kEmitSample) sample_store(sample_slots, st, smx, scnt);
        return;
    }
    bool list_full = false;
    uint32_t j = 0u, pend = 0u;
    u32x4 b0[U], b1[U];
    fetch(b0, tile_row0(blk, 0), 0);
    for (;;) {
        float part[TPW];
        long long next_blk = nblocks;              // known from phase 1 on
        for (int p = 0; p < nphase; ++p) {
            if (p == 1 && tid == 0) s_blk[(j + 1u) & 3u] = pend;
            lds_barrier();                         // everybody is done with the previous image
            if (p == 1) next_blk = (long long)s_blk[(j + 1u) & 3u];
            // (the tile about to be looked up was ordered a tile ago; waiting for it here, where the
            //  compiler can see it, spares a wait for everything behind the image loads, whose
            //  number it cannot count)
            __builtin_amdgcn_s_waitcnt(0x0F70);    // vmcnt(0)
            copy_image(p);
            __builtin_amdgcn_sched_barrier(0);     // the image loads are older than the tile loads that follow
            fetch(b1, tile_row0(blk, 1), p);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_waitcnt(0x0F78);    // vmcnt(8): all but the 8 loads just issued have landed
            lds_barrier();                         // the image is complete
            if (p == 0 && tid == 0) pend = atomicAdd(blk_ctr, 1u);   // the block after this one
            // The tiles of the phase go in pairs: even ones arrive in b0, odd ones in b1.  The partial sums
            // sit in a ring of registers that turns by two after every pair, so the pair at hand is
            // always elements 0 and 1 and the loop stays rolled (unrolled, four tiles per wave spilled
            // a hundred registers).
#pragma unroll 1
            for (int t = 0; t < TPW; t += 2) {
                if (t > 0) fetch(b1, tile_row0(blk, t + 1), p);      // (the phase's first odd tile went out with the image)
                const float s0 = tile_sum(b0);
                part[0] = p == 0 ? s0 : part[0] + s0;
                // the even tile after this pair: the next of the phase, the first of the next phase, the
                // first of the next block, or (nothing left) this block's first tile once more
                long long v0;
                int pp = p;
                if (t + 2 < TPW) v0 = tile_row0(blk, t + 2);
                else if (p + 1 < nphase) v0 = tile_row0(blk, 0), pp = p + 1;
                else if (next_blk < nblocks) v0 = tile_row0(next_blk, 0), pp = 0;
                else v0 = tile_row0(blk, 0), pp = 0;
                fetch(b0, v0, pp);
                const float s1 = tile_sum(b1);
                part[1] = p == 0 ? s1 : part[1] + s1;
                turn_ring(part);
            }
        }
#pragma unroll 1
        for (int t = 0; t < TPW; t += 2) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const long long v0 = tile_row0(blk, t + h), v = window(v0) + (long long)sub * RPW + rr;
                if (v >= v0 && v < N) emit_row<EMIT>(part[h] + bias, v, tau, list_full, st, cand, scores, lhist, smx, scnt);
            }
            turn_ring(part);
        }
        if (EMIT == kEmitFilter) list_full = __ballot(list_full) != 0ull;   // one lane's news serves the wave
        if (next_blk >= nblocks) break;            // uniform
        blk = next_blk;
        ++j;
    }
    if (EMIT == kEmitScores) merge_hist1(lhist, hist1);
    if (EMIT == kEmitSample) sample_store(sample_slots, st, smx, scnt);
}

hipError_t launch_pq_build_lut(const float *codebooks, int M, int K, int dsub, const float *w, float *lut,
                               hipStream_t s) {
    long long total = (long long)M * K;
    int blocks = (int)std::min<long long>((total + 255) / 256, 4096);
    pq_build_lut_kernel<<<blocks, 256, 0, s>>>(codebooks, M, K, dsub, w, lut);
    return hipGetLastError();
}

static int phases_of(int row_bytes) { return (row_bytes + kSegBytes - 1) / kSegBytes; }

// Lanes per row of a row that fits one image, as a span in bytes: 16, 32, 64 or 128.
static int span_of(int row_bytes) { return row_bytes <= 16 ? 16 : row_bytes <= 32 ? 32 : row_bytes <= 64 ? 64 : 128; }

hipError_t launch_pq_prepare(const float *lut, int M, float *image, const SelectWs &sw, const SelectWs &ssw,
                             hipStream_t s) {
    const int nphase = phases_of(M);
    pq_prepare_kernel<<<nphase * 32, 256, 0, s>>>(lut, M, span_of(M), nphase, image, sw.st, sw.hist1, sw.hist2, sw.hist3,
                                                  ssw.st);
    return hipGetLastError();
}

hipError_t launch_pq_prepare_model(const float *codebooks, const float *w, int M, int dsub, float *image,
                                   const SelectWs &sw, const SelectWs &ssw, hipStream_t s) {
    const int nphase = phases_of(M);
    pq_prepare_model_kernel<<<nphase * 64, 256, 0, s>>>(codebooks, w, M, dsub, span_of(M), nphase, image, sw.st, sw.hist1,
                                                        sw.hist2, sw.hist3, ssw.st);
    return hipGetLastError();
}

// D == 2048 builds the 7-bit image, every other supported D the byte images.
hipError_t launch_binary_prepare(const float *w, int D, float *image, const SelectWs &sw, const SelectWs &ssw,
                                 hipStream_t s) {
    if (D == 2048) {
        binary7_prepare_kernel<<<64, 256, 0, s>>>(w, image, sw.st, sw.hist1, sw.hist2, sw.hist3, ssw.st);
        return hipGetLastError();
    }
    const int row_bytes = D / 8, nphase = phases_of(row_bytes);
    binary_prepare_kernel<<<nphase * 32, 256, 0, s>>>(w, row_bytes, span_of(row_bytes), nphase, image, sw.st, sw.hist1,
                                                      sw.hist2, sw.hist3, ssw.st);
    return hipGetLastError();
}

struct ScanArgs {
    const uint8_t *codes;
    int64_t N;
    int M;
    const float *image;
    float bias;
    float *scores;
    SelState *st;
    uint32_t *hist1;
    const SelState *tau;         // filtered scan: the sample's state (number of slots)
    SampleSlot *slots;           // sample scan: written; filtered scan: read
    unsigned long long *cand;
    Gate gate;
};

template <int LPR, int U, int GB, int EMIT>
static hipError_t launch_scan_cfg(const ScanArgs &a, hipStream_t s) {
    // (without a table the dynamic area only serves the threshold resolution of the filtered scan)
    constexpr int lds = GB == 8 ? kImageBytes : GB == 7 ? kImage7Bytes : kBins2 * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&table_scan_kernel<LPR, U, GB, EMIT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    int grid = device_cu_count();
    const int64_t max_useful = (a.N + 1023) / 1024;
    if (grid > max_useful) grid = (int)max_useful;
    if (grid < 1) grid = 1;
    // (the Hamming scan has no gathers to hide: 12 waves stream 50M x 256 B in 1.829 ms, 16 in 1.844, 8 in 1.842)
    const int threads = tune_int(OTF_DEBUG_SCAN_THREADS, GB == 0 ? 768 : kScanThreads);
    table_scan_kernel<LPR, U, GB, EMIT><<<grid, threads, lds, s>>>(a.codes, (long long)a.N, a.M, a.image, a.bias,
                                                                    a.scores, a.st, a.hist1, a.tau, a.slots, a.cand,
                                                                    a.gate);
    return hipGetLastError();
}

template <int LPR, int GB>
static hipError_t launch_scan_emit(const ScanArgs &a, ScanEmit emit, hipStream_t s) {
    constexpr int U = LPR <= 2 ? 4 : 8;    // narrow rows own many outputs per lane: fewer loads per tile
    if (LPR >= 8 && emit == kEmitFilter && tune_int(OTF_DEBUG_SCAN_UNROLL, 8) == 4)
        return launch_scan_cfg<LPR, 4, GB, kEmitFilter>(a, s);
    switch (emit) {
        case kEmitScores: return launch_scan_cfg<LPR, U, GB, kEmitScores>(a, s);
        case kEmitSample: return launch_scan_cfg<LPR, U, GB, kEmitSample>(a, s);
        default: return launch_scan_cfg<LPR, U, GB, kEmitFilter>(a, s);
    }
}

template <int EMIT, int TPW>
static hipError_t launch_walk_cfg(const ScanArgs &a, hipStream_t s) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&table_walk_kernel<EMIT, TPW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kImageBytes);
    if (e != hipSuccess) return e;
    // Long scans: the full workgroup of 16 waves, 2048 rows per block.  Short ones (the sample, small
    // stores) spread over the chip in workgroups of 4 waves, 512 rows per block.
    int threads = tune_int(OTF_DEBUG_SCAN_THREADS, kScanThreads);
    const int cus = device_cu_count();
    if (a.N < (int64_t)cus * 64 * TPW * (kScanThreads / 64)) threads = 256;
    const int64_t R = (int64_t)(threads / 64) * 64 * TPW;
    const int64_t nblocks = (a.N + R - 1) / R;
    const int grid = (int)std::min<int64_t>(nblocks, cus);
    table_walk_kernel<EMIT, TPW><<<grid, threads, kImageBytes, s>>>(a.codes, (long long)a.N, a.M, phases_of(a.M), a.image,
                                                                    a.bias, a.scores, a.st, a.hist1, a.tau, a.slots,
                                                                    a.cand, a.gate);
    return hipGetLastError();
}

template <int TPW>
static hipError_t launch_walk_emit(const ScanArgs &a, ScanEmit emit, hipStream_t s) {
    switch (emit) {
        case kEmitScores: return launch_walk_cfg<kEmitScores, TPW>(a, s);
        case kEmitSample: return launch_walk_cfg<kEmitSample, TPW>(a, s);
        default: return launch_walk_cfg<kEmitFilter, TPW>(a, s);
    }
}

// row_bytes = stored bytes per row, a multiple of 16 up to 1024; kTableSeven only with 256.
hipError_t launch_table_scan(const uint8_t *codes, int64_t N, int row_bytes, TableKind kind, const float *image,
                             float bias, ScanEmit emit, float *scores, SelState *st, uint32_t *hist1,
                             const SelState *tau, SampleSlot *slots, unsigned long long *cand, Gate gate,
                             hipStream_t s) {
    ScanArgs a{codes, N, row_bytes, image, bias, scores, st, hist1, tau, slots, cand, gate};
    if (kind == kTableSeven) return launch_scan_emit<16, 7>(a, emit, s);
    if (kind == kTableHamming) {                  // `image` is the query code; lanes per row = next power of two
        if (row_bytes <= 16) return launch_scan_emit<1, 0>(a, emit, s);
        if (row_bytes <= 32) return launch_scan_emit<2, 0>(a, emit, s);
        if (row_bytes <= 64) return launch_scan_emit<4, 0>(a, emit, s);
        if (row_bytes <= 128) return launch_scan_emit<8, 0>(a, emit, s);
        if (row_bytes <= 256) return launch_scan_emit<16, 0>(a, emit, s);
        if (row_bytes <= 512) return launch_scan_emit<32, 0>(a, emit, s);
        return launch_scan_emit<64, 0>(a, emit, s);
    }
    if (row_bytes > kSegBytes)
        // four tiles per wave and block for the long scans (half as many image changes as with two:
        // 0.410 -> 0.399 ms on 5M x 512 B; eight leave too few blocks to balance), two for short ones
        switch (tune_int(OTF_DEBUG_WALK_TILES, N >= ((int64_t)1 << 20) ? 4 : 2)) {
            case 4: return launch_walk_emit<4>(a, emit, s);
            case 8: return launch_walk_emit<8>(a, emit, s);
            default: return launch_walk_emit<2>(a, emit, s);
        }
    switch (span_of(row_bytes)) {
        case 16: return launch_scan_emit<1, 8>(a, emit, s);
        case 32: return launch_scan_emit<2, 8>(a, emit, s);
        case 64: return launch_scan_emit<4, 8>(a, emit, s);
        default: return launch_scan_emit<8, 8>(a, emit, s);
    }
}

}  // namespace otf
