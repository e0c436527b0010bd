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
// repeat); byte-group rows longer than 128 bytes are processed in `nsplit` phases of 128 columns,
// the workgroup reloading the table image between phases and carrying partial sums in the score
// array.
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
                                            uint32_t *hist3, SelState *sst, uint32_t *shist1, uint32_t *shist2) {
    uint32_t *stw = reinterpret_cast<uint32_t *>(st), *sstw = reinterpret_cast<uint32_t *>(sst);
    for (int i = tid; i < (int)(sizeof(SelState) / 4); i += step) {
        stw[i] = 0u;
        sstw[i] = 0u;
    }
    for (int i = tid; i < kHist1Words; i += step) {
        hist1[i] = 0u;
        shist1[i] = 0u;
    }
    for (int i = tid; i < kBins2; i += step) {
        hist2[i] = 0u;
        shist2[i] = 0u;
    }
    for (int i = tid; i < kBins3; i += step) hist3[i] = 0u;
}

// Table images for PQ: image[sp][v][column(pos)] = lut[m][v],  m = sp*128 + pos (M >= 128) or
// pos mod M (M < 128).  Also zeroes the selection states (one launch instead of two).
__global__ __launch_bounds__(256) void pq_prepare_kernel(const float *__restrict__ lut, int M, int nsplit,
                                                         float *__restrict__ image, SelState *st, uint32_t *hist1,
                                                         uint32_t *hist2, uint32_t *hist3, SelState *sst,
                                                         uint32_t *shist1, uint32_t *shist2) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, step = gridDim.x * blockDim.x;
    for (int t = tid; t < nsplit * kImageFloats; t += step) {
        const int v = t & 255, pos = (t >> 8) & (kSegBytes - 1), sp = t >> 15;
        const int m = (M >= kSegBytes) ? sp * kSegBytes + pos : pos % M;
        image[(size_t)sp * kImageFloats + v * kSegBytes + image_column(pos)] = lut[(size_t)m * 256 + v];
    }
    zero_states(tid, step, st, hist1, hist2, hist3, sst, shist1, shist2);
}

// Table images for binary codes with byte groups: byte g of a row covers dimensions 8g..8g+7.
__global__ __launch_bounds__(256) void binary_prepare_kernel(const float *__restrict__ w, int row_bytes, int nsplit,
                                                             float *__restrict__ image, SelState *st, uint32_t *hist1,
                                                             uint32_t *hist2, uint32_t *hist3, SelState *sst,
                                                             uint32_t *shist1, uint32_t *shist2) {
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
    zero_states(tid, step, st, hist1, hist2, hist3, sst, shist1, shist2);
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
                                                              uint32_t *hist3, SelState *sst, uint32_t *shist1,
                                                              uint32_t *shist2) {
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
    zero_states(tid, step, st, hist1, hist2, hist3, sst, shist1, shist2);
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over groups of LPR adjacent lanes (LPR = 1, 2, 4, 8 or 16); every lane of a group receives it.
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
    if (LPR >= 2) v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
    if (LPR >= 4) v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
    if (LPR >= 8) v += dpp_move<0x141>(v);   // row_half_mirror: lane i <-> 7 - i of each 8
    if (LPR >= 16) v += dpp_move<0x140>(v);  // row_mirror: lane i <-> 15 - i of each 16
    return v;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Scan.
//   GB     bits per group: 8 (bytes; LPR = min(row bytes, 128) / 16 lanes per row per phase) or 7
//          (2048-bit rows, LPR = 16, each word = 4 x 7 bits + 4 bits)
//   U      16-byte loads per lane per tile
//   EMIT   what is produced (ScanEmit)
//   SPLIT  byte-group rows longer than 128 bytes: several phases of 128 columns, one launch each,
//          partial sums carried in the score array (EMIT = kEmitScores only)
//
// A tile is what one wave looks up per iteration: U loads of 64 lanes x 16 bytes.  The main loop
// is software-pipelined: the loads of the wave's next tile are issued before the current tile is
// looked up, and a prefetch with nothing left to fetch re-reads the current tile rather than
// being skipped (an unconditional load keeps the in-order wait counters exact).  After the
// lookups the U row sums of a lane group are moved into U different lanes so that the output
// step happens once per tile, not per row.
//
// Work distribution: dynamic, by a TileQueue with chunks of 256 KiB of rows.
template <int LPR, int U, int GB, int EMIT, bool SPLIT>
__global__ __launch_bounds__(kScanMaxThreads) void table_scan_kernel(
    const uint8_t *__restrict__ codes, long long N, int M, int nsplit, const float *__restrict__ image, float bias,
    float *__restrict__ scores, SelState *st, uint32_t *hist1, int sample_rank, const SelState *tau_state,
    const uint32_t *tau_hist2, unsigned long long *__restrict__ cand, const SelState *gate, int sp0,
    uint32_t *phase_ctr) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    __shared__ uint32_t lhist[EMIT == kEmitFilter ? 1 : kBins1];
    __shared__ uint32_t s_out[3];
    __shared__ TileQueue s_queue;
    if (gate && gate->fallback == 0u) return;     // uniform: this launch is only the fallback of a filtered scan
    constexpr int RPW = 64 / LPR;                // rows per wave load
    constexpr int TILE = RPW * U;                // rows per wave iteration
    constexpr int ACTIVE = LPR < U ? LPR : U;    // lanes of a group that own an output row per round
    constexpr int ROUNDS = U / ACTIVE;           // output rounds per tile
    constexpr int VSHIFT = GB == 8 ? 9 : 10;     // log2 of the byte stride between table values
    constexpr int TQ_BYTES = GB == 8 ? 128 : 256;  // byte distance between the column blocks of the 4 words
    constexpr int TABLE_VEC = (GB == 8 ? kImageBytes : kImage7Bytes) / 16;
    constexpr uint32_t CHUNK_TILES = 256u / (uint32_t)U;          // x U KiB per tile = 256 KiB of rows

    // the two scans that can follow each other on one state (filtered, then the gated full scan)
    // count in different words; both were zeroed with the state.  A phase of a multi-phase scan
    // (one launch per phase) counts in a word of its own.
    uint32_t *chunk_ctr = SPLIT ? phase_ctr + sp0 : &st->chunk_ctr[EMIT == kEmitScores ? 1 : 0];
    if (threadIdx.x == 0) tile_queue_init(&s_queue, chunk_ctr);   // visible after the barriers below
    const uint32_t chunk_tiles = tile_queue_chunk_tiles(N / TILE, CHUNK_TILES);

    if (EMIT != kEmitFilter)
        for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
    // Filtered scan: the threshold is the top 24 bits of the k-th largest sample key (k = the
    // sample rank here); passes 1 and 2 over the sample left their state, every block resolves it
    // (the table area of shared memory is still free at this point).
    uint32_t tau = 0u;
    if (EMIT == kEmitFilter) {
        const BinChoice r2 = block_find_bin(tau_hist2, kBins2, tau_state->need1,
                                            reinterpret_cast<uint32_t *>(lds_raw), s_out);
        tau = ((tau_state->b1 << 12) | r2.bin) << 8;
        if (filter_hopeless((uint32_t)sample_rank, tau_state->need1, r2)) return;   // uniform
    }

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

    const size_t u_bytes = (size_t)RPW * (size_t)M;        // distance between the U loads of a lane
    const int out_u = sub % ACTIVE;                        // which of a round's rows this lane emits
    // For the sample scan the rows are numbered compactly: sample row v is store row
    // (v / 1024) * 1024 * stride + v % 1024 (a tile never straddles a group: TILE divides 1024).
    auto store_row = [&](long long v) {
        return EMIT == kEmitSample ? ((v >> 10) * ((long long)kSampleGroup * kSampleStride) + (v & 1023)) : v;
    };

    auto lookup16 = [&](const u32x4 &d) {
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
                v[4 * tq + t] = *reinterpret_cast<const float *>(lds_raw + addr[4 * tq + t] + TQ_BYTES * tq);
        if (GB == 7) {
#pragma unroll
            for (int tq = 0; tq < 4; ++tq)
                v[4 * tq] += *reinterpret_cast<const float *>(lds_raw + ((d[tq] >> 28) << 9) + sidecol + 128 * tq);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] += v[i + 8];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] += v[i + 4];
        return group_sum<LPR>((v[0] + v[1]) + (v[2] + v[3]));
    };
    // looks up the U loads of a tile; the U row sums of a lane group (every lane of the group
    // holds each sum) are kept by U different lanes: lane out_u keeps row e*ACTIVE + out_u
    auto tile_sums = [&](const u32x4 *d, float *mine) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float su = lookup16(d[u]);
            if (u % ACTIVE == 0) mine[u / ACTIVE] = su;
            else mine[u / ACTIVE] = out_u == (u % ACTIVE) ? su : mine[u / ACTIVE];
        }
    };
    // compact row that lane `sub` of its group emits in round e of the tile starting at row v0
    auto out_row = [&](long long v0, int e) { return v0 + (long long)(e * ACTIVE + out_u) * RPW + rr; };

    {
        const int sp = SPLIT ? sp0 : 0;           // this launch's phase (columns 128 sp .. 128 sp + 127 of every row)
        {
            const u32x4 *src = reinterpret_cast<const u32x4 *>(image + (size_t)sp * kImageFloats);
            u32x4 *dst = reinterpret_cast<u32x4 *>(lds_raw);
            for (int i = threadIdx.x; i < TABLE_VEC; i += blockDim.x) dst[i] = src[i];
        }
        __syncthreads();
        const bool first = sp == 0, lastp = sp == nsplit - 1;

        // one output round: lane `sub` of each group holds in `mine` the sum of the row it owns.
        // Filtered scan: a wave that has seen the list full stops appending (the list is already
        // useless, and the appends are adds to one address, ~18 ns each one after the other: a
        // threshold that lets a million rows pass would otherwise cost tens of milliseconds).
        bool list_full = false;
        auto emit = [&](float mine, const float *carry, long long v, int e, bool ok) {
            if (sub < ACTIVE && ok) {
                if (SPLIT && !first) mine += carry[e];
                if (lastp) mine += bias;
                if (EMIT == kEmitFilter) {
                    const uint32_t key = float_to_key(mine);
                    if (key >= tau && !list_full) {
                        const uint32_t pos = atomicAdd(&st->cursor, 1u);
                        if (pos < (uint32_t)kCandCap)
                            cand[pos] = ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)v);
                        else
                            list_full = true;
                    }
                } else {
                    if (lastp) atomicAdd(&lhist[float_to_key(mine) >> 20], 1u);
                    scores[v] = mine;
                }
            }
        };

        {
            // first row of the next tile of this wave, or -1 when the scan has no full tile left
            // (the rows after the last full tile are handled at the end)
            auto draw = [&]() -> long long {
                const long long t = tile_queue_draw(&s_queue, chunk_ctr, chunk_tiles, N / TILE);
                return t < 0 ? t : t * TILE;
            };
            // uniform base of the tile (scalar registers) + one 32-bit lane offset; a phase reads its
            // 128 columns of every row and meets the partial sums of the phases before in the score
            // array (`carry`)
            const uint32_t lane_off = (uint32_t)rr * (uint32_t)M + (SPLIT ? (uint32_t)sp * (uint32_t)kSegBytes : 0u) + (uint32_t)sub * 16u;
            auto fetch = [&](u32x4 *d, float *carry, long long v0) {
                const unsigned long long a = (unsigned long long)store_row(v0) * (unsigned long long)M;
                // (the builtin returns int: go through uint32_t, or offsets past 2 GiB are sign-extended)
                const uint32_t a_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
                const uint32_t a_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
                const uint8_t *p = codes + (((unsigned long long)a_hi << 32) | (unsigned long long)a_lo);
#pragma unroll
                for (int u = 0; u < U; ++u)
                    d[u] = __builtin_nontemporal_load(
                        reinterpret_cast<const u32x4 *>(p + (size_t)u * u_bytes + (size_t)lane_off));
                if (SPLIT && !first) {
#pragma unroll
                    for (int e = 0; e < ROUNDS; ++e) carry[e] = scores[out_row(v0, e)];
                }
            };
            auto consume = [&](const u32x4 *d, const float *carry, long long v0) {
                float mine[ROUNDS];
                tile_sums(d, mine);
#pragma unroll
                for (int e = 0; e < ROUNDS; ++e) {
                    const long long v = out_row(v0, e);
                    emit(mine[e], carry, v, e, true);
                }
                if (EMIT == kEmitFilter) list_full = __ballot(list_full) != 0ull;   // one lane's news serves the wave
            };
            long long cur = draw();
            if (cur >= 0) {
                u32x4 b0[U], b1[U];
                float c0[ROUNDS], c1[ROUNDS];
                fetch(b0, c0, cur);
                for (;;) {
                    long long nxt = draw();
                    fetch(b1, c1, nxt >= 0 ? nxt : cur);
                    consume(b0, c0, cur);
                    if (nxt < 0) break;
                    cur = nxt;
                    nxt = draw();
                    fetch(b0, c0, nxt >= 0 ? nxt : cur);
                    consume(b1, c1, cur);
                    if (nxt < 0) break;
                    cur = nxt;
                }
            }
            // the rows after the last full tile (fewer than a tile): one wave, row-checked
            const long long v0 = N / TILE * TILE;
            if (v0 < N && blockIdx.x == 0 && wave == 0) {
                u32x4 d[U];
                float carry[ROUNDS], mine[ROUNDS];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const long long v = v0 + (long long)u * RPW + rr;
                    d[u] = (u32x4){0u, 0u, 0u, 0u};
                    if (v < N)
                        d[u] = *reinterpret_cast<const u32x4 *>(codes + (size_t)store_row(v - rr) * (size_t)M + (size_t)lane_off);
                }
#pragma unroll
                for (int e = 0; e < ROUNDS; ++e) {
                    const long long v = out_row(v0, e);
                    carry[e] = (SPLIT && !first && v < N) ? scores[v] : 0.f;
                }
                tile_sums(d, mine);
#pragma unroll
                for (int e = 0; e < ROUNDS; ++e) {
                    const long long v = out_row(v0, e);
                    emit(mine[e], carry, v, e, v < N);
                }
            }
        }
    }
    if (EMIT != kEmitFilter) merge_hist1(lhist, hist1);
}

hipError_t launch_pq_build_lut(const float *codebooks, int M, int K, int dsub, const float *w, float *lut,
                               hipStream_t s) {
    long long total = (long long)M * K;
    int blocks = (int)std::min<long long>((total + 255) / 256, 4096);
    pq_build_lut_kernel<<<blocks, 256, 0, s>>>(codebooks, M, K, dsub, w, lut);
    return hipGetLastError();
}

static int splits_of(int row_bytes) { return row_bytes >= kSegBytes ? row_bytes / kSegBytes : 1; }

hipError_t launch_pq_prepare(const float *lut, int M, float *image, const SelectWs &sw, const SelectWs &ssw,
                             hipStream_t s) {
    const int nsplit = splits_of(M);
    pq_prepare_kernel<<<nsplit * 32, 256, 0, s>>>(lut, M, nsplit, image, sw.st, sw.hist1, sw.hist2, sw.hist3, ssw.st,
                                                  ssw.hist1, ssw.hist2);
    return hipGetLastError();
}

// D == 2048 builds the 7-bit image, every other supported D the byte images.
hipError_t launch_binary_prepare(const float *w, int D, float *image, const SelectWs &sw, const SelectWs &ssw,
                                 hipStream_t s) {
    if (D == 2048) {
        binary7_prepare_kernel<<<64, 256, 0, s>>>(w, image, sw.st, sw.hist1, sw.hist2, sw.hist3, ssw.st, ssw.hist1,
                                                  ssw.hist2);
        return hipGetLastError();
    }
    const int row_bytes = D / 8, nsplit = splits_of(row_bytes);
    binary_prepare_kernel<<<nsplit * 32, 256, 0, s>>>(w, row_bytes, nsplit, image, sw.st, sw.hist1, sw.hist2, sw.hist3,
                                                      ssw.st, ssw.hist1, ssw.hist2);
    return hipGetLastError();
}

struct ScanArgs {
    const uint8_t *codes;
    int64_t N;
    int M, nsplit;
    const float *image;
    float bias;
    float *scores;
    SelState *st;
    uint32_t *hist1;
    int k;
    const SelState *tau;
    const uint32_t *tau_hist2;
    unsigned long long *cand;
    const SelState *gate;
    uint32_t *phase_ctr;   // nsplit > 1: one zeroed word per phase
};

template <int LPR, int U, int GB, int EMIT, bool SPLIT>
static hipError_t launch_scan_cfg(const ScanArgs &a, hipStream_t s) {
    constexpr int lds = GB == 8 ? kImageBytes : kImage7Bytes;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&table_scan_kernel<LPR, U, GB, EMIT, SPLIT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    int grid = device_cu_count();
    const int64_t max_useful = (a.N + 1023) / 1024;
    if (grid > max_useful) grid = (int)max_useful;
    if (grid < 1) grid = 1;
    const int threads = tune_int(OTF_DEBUG_SCAN_THREADS, kScanThreads);
    // a multi-phase scan is one launch per phase: each phase meets the partial sums of the one
    // before in the score array, and the launch boundary is what orders them
    for (int sp = 0; sp < (SPLIT ? a.nsplit : 1); ++sp)
        table_scan_kernel<LPR, U, GB, EMIT, SPLIT><<<grid, threads, lds, s>>>(
            a.codes, (long long)a.N, a.M, a.nsplit, a.image, a.bias, a.scores, a.st, a.hist1, a.k, a.tau, a.tau_hist2,
            a.cand, a.gate, sp, a.phase_ctr);
    return hipGetLastError();
}

template <int LPR, int GB>
static hipError_t launch_scan_emit(const ScanArgs &a, ScanEmit emit, hipStream_t s) {
    constexpr int U = LPR <= 2 ? 4 : 8;    // narrow rows own many outputs per lane: fewer loads per tile
    if (LPR >= 8 && a.nsplit == 1 && emit == kEmitFilter) {
        if (tune_int(OTF_DEBUG_SCAN_UNROLL, 8) == 4) return launch_scan_cfg<LPR, 4, GB, kEmitFilter, false>(a, s);

    }
    if (a.nsplit > 1) {
        if (GB != 8 || emit != kEmitScores || !a.phase_ctr) return hipErrorInvalidValue;
        return launch_scan_cfg<LPR, U, 8, kEmitScores, true>(a, s);
    }
    switch (emit) {
        case kEmitScores: return launch_scan_cfg<LPR, U, GB, kEmitScores, false>(a, s);
        case kEmitSample: return launch_scan_cfg<LPR, U, GB, kEmitSample, false>(a, s);
        default: return launch_scan_cfg<LPR, U, GB, kEmitFilter, false>(a, s);
    }
}

// row_bytes = stored bytes per row: 16, 32, 64 or a multiple of 128; seven_bit only with 256.
hipError_t launch_table_scan(const uint8_t *codes, int64_t N, int row_bytes, int seven_bit, const float *image,
                             float bias, ScanEmit emit, float *scores, SelState *st, uint32_t *hist1, int k,
                             const SelState *tau, const uint32_t *tau_hist2, unsigned long long *cand,
                             const SelState *gate, uint32_t *phase_ctr, hipStream_t s) {
    ScanArgs a{codes, N,  row_bytes, seven_bit ? 1 : splits_of(row_bytes), image, bias, scores, st, hist1, k, tau,
               tau_hist2, cand, gate, phase_ctr};
    if (seven_bit) return launch_scan_emit<16, 7>(a, emit, s);
    switch (row_bytes) {
        case 16: return launch_scan_emit<1, 8>(a, emit, s);
        case 32: return launch_scan_emit<2, 8>(a, emit, s);
        case 64: return launch_scan_emit<4, 8>(a, emit, s);
        default: return launch_scan_emit<8, 8>(a, emit, s);
    }
}

}  // namespace otf
