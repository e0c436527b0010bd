// Device-side helpers shared by the libotf kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace otf {

constexpr int kWave = 64;
constexpr int kBins1 = 4096;   // radix pass 1: key bits 31..20
constexpr int kBins2 = 4096;   // radix pass 2: key bits 19..8
constexpr int kBins3 = 256;    // radix pass 3: key bits 7..0
// The pass-1 histogram of a classifier is kept in kHistShards copies, a workgroup adding to copy
// (its number mod kHistShards): scores crowd into a hundred-odd of the bins, the workgroups of a
// scan finish together, and adds to one address take ~18 ns each one after the other, so a single
// copy ends a 256-workgroup scan with a queue of ~4.6 us on every hot bin.
constexpr int kHistShards = 4;
constexpr int kHist1Words = kHistShards * kBins1;   // pass-1 words per classifier
constexpr int kCandCap = 8192; // capacity of the candidate list that the final sort takes
constexpr int kSelBlocks = 256; // blocks per classifier in the selection passes over scores
// Filtered scans: a strided sample of the store (every kSampleStride-th group of kSampleGroup rows)
// is scored first; the threshold is set so that about kFilterExpect rows of the full store pass it.
constexpr int kSampleGroup = 1024;
constexpr int kSampleStride = 128;
constexpr int kFilterExpect = 4096;
constexpr int kFilterMaxK = 1024;

// Order-preserving map float -> uint32 (larger float <=> larger key); -0.0 maps onto +0.0
// so that the two compare equal, as they do as numbers.
__device__ __forceinline__ uint32_t float_to_key(float f) {
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0u;
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
    return __uint_as_float(u);
}

// Selection state of one classifier (one row of scores).  Lives in the workspace.
struct SelState {
    uint32_t mode;     // 0: resolved after pass 1, 1: after pass 2, 2: after pass 3 (ties split by index)
    uint32_t b1;       // pass-1 bin of the k-th largest key
    uint32_t need1;    // how many of the k lie inside bin b1
    uint32_t p24;      // top 24 bits of the k-th largest key (mode >= 1)
    uint32_t need2;    // how many of the k lie inside prefix p24
    uint32_t T;        // the k-th largest key (mode 2)
    uint32_t r;        // how many rows with key == T belong to the list (mode 2), lowest indices first
    uint32_t ncand;    // entries the gather pass writes to the candidate list
    long long tex;     // gather every key with (long long)key > tex
    uint32_t cursor;   // append cursor of a filtered scan: rows it put on the candidate list, or some number
                       // beyond the list's capacity when more passed than it holds
    uint32_t chunk_ctr[2];  // next chunk of a dynamically scheduled scan (two scans may share a state)
    uint32_t spare;    // ticket of the one-launch selection: the workgroup that finishes last sorts
    uint32_t tau_key;  // filter threshold: rows with key >= tau_key are candidates (filtered scans)
    uint32_t fallback; // set by the filtered path when its candidate list cannot serve: redo by full selection
    // meeting points of the workgroups of the one-launch selection (select_fused_gated_kernel)
    uint32_t met[2];   // arrivals at meeting point 0, 1
    uint32_t verdict[2];   // 0: open, 1: all arrived, go on together, 2: somebody stopped waiting, the last arrival goes on alone
    uint32_t gcursor;  // append cursor of the gather pass of the full selection
    uint32_t pad[11];
};
static_assert(sizeof(SelState) == 128, "SelState layout");

// What stands behind a filtered scan (the re-scan that materialises the scores, the full selection)
// is enqueued with the scan, whether it will be needed or not, and looks at the scan's state when
// it starts.  The gate is OPEN -- the launch has work to do -- when the fallback flag of that
// state is raised, or, with k > 0, when the scan's candidate list cannot serve a list of k rows:
// fewer than k rows on it, or more passed than it holds.  (k = 0: the flag alone decides; whoever
// judges the lists raises it.)  No state: no gate, always open.  Uniform over the grid.
struct Gate {
    const SelState *st;
    int k;
};
constexpr Gate kNoGate{nullptr, 0};
__device__ __forceinline__ bool gate_open(const Gate &g) {
    if (!g.st) return true;
    if (g.st->fallback != 0u) return true;
    if (g.k <= 0) return false;
    const uint32_t n = g.st->cursor;
    return n < (uint32_t)g.k || n > (uint32_t)kCandCap;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

template <int CTRL>
__device__ __forceinline__ float dpp_mov_f32(float v) {
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over the 64 lanes using cross-lane data-parallel moves (no shared-memory traffic); the
// total is returned in every lane (the last step goes through scalar registers).
__device__ __forceinline__ float wave_sum_to_lane0(float v) {
    v += dpp_mov_f32<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_mov_f32<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_mov_f32<0x141>(v);   // row_half_mirror
    v += dpp_mov_f32<0x140>(v);   // row_mirror: every lane now holds the sum of its row of 16
    const int iv = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(iv, 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(iv, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(iv, 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(iv, 48));
    return (r0 + r1) + (r2 + r3);
}

// Inclusive suffix sum over the 64 lanes of a wave: lane l receives sum of lanes l..63.
__device__ __forceinline__ uint32_t wave_suffix_sum(uint32_t v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t t = __shfl_down(v, o, 64);
        if (lane + o < 64) v += t;
    }
    return v;
}

// Called by ONE full wave (64 lanes) on a histogram in shared memory with 64*per_lane bins
// (per_lane <= 64).  Finds the bin b with  count(bins > b) < need <= count(bins >= b)  and
// returns it; *above receives count(bins > b) and *inbin the population of b.
// Requires total count >= need >= 1.
__device__ __forceinline__ uint32_t wave_find_bin(const uint32_t *hist, int per_lane, uint32_t need,
                                                  uint32_t *above, uint32_t *inbin) {
    const int lane = threadIdx.x & 63;
    uint32_t mine = 0;
    for (int j = 0; j < per_lane; ++j) mine += hist[lane * per_lane + j];
    uint32_t suf = wave_suffix_sum(mine);                  // bins of lanes >= lane
    // the owning lane is the highest lane whose suffix still reaches `need`
    unsigned long long reach = __ballot(suf >= need);
    int owner = 63 - __builtin_clzll(reach | 1ull);
    uint32_t above_owner = __shfl(suf - mine, owner, 64);  // count in lanes > owner
    // second level: the per_lane bins of the owner, one per lane (lanes >= per_lane hold 0)
    uint32_t binv = (lane < per_lane) ? hist[owner * per_lane + lane] : 0u;
    uint32_t suf2 = wave_suffix_sum(binv) + above_owner;   // count in bins >= this bin
    unsigned long long reach2 = __ballot(lane < per_lane && suf2 >= need);
    int lb = 63 - __builtin_clzll(reach2 | 1ull);
    *inbin = __shfl(binv, lb, 64);
    *above = __shfl(suf2 - binv, lb, 64);
    return (uint32_t)(owner * per_lane + lb);
}

// Histogram increment for a whole wave.  Measured: an integer atomic into shared memory costs about
// 5 cycles per wave instruction when the lanes spread over 35 addresses, 16 when 8 lanes share each
// address, 129 when all 64 hit one (two cycles per lane on an address).  So lanes simply add, except
// where one vote shows heavy sharing (a quarter of the wave or more in the bin of the first active
// lane: constant scores, scores that take few values or arrive sorted): that bin is then added once
// with its count, the same is done once more for the first lane left over, and whoever is still
// left adds for itself.  The common case pays one vote and one uniform branch; the passes are bound
// by the latency of these votes, and a variant without any branch (two votes always) was slower on
// ordinary scores (35 -> 53 us per pass over 50M).  All 64 lanes must call.
__device__ __forceinline__ void hist_add_wave(uint32_t *lhist, uint32_t bin, bool active) {
    const unsigned long long act = __ballot(active);
    const int lane = threadIdx.x & 63;
    const int leader = act ? __builtin_ctzll(act) : 0;
    const uint32_t lb = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
    const unsigned long long same = __ballot(active && bin == lb);
    if (__popcll(same) < 16) {                                     // uniform: the usual case (also: no active lane)
        if (active) atomicAdd(&lhist[bin], 1u);
        return;
    }
    if (lane == leader) atomicAdd(&lhist[lb], (uint32_t)__popcll(same));
    const unsigned long long rest = act & ~same;
    if (rest == 0ull) return;                                      // uniform
    const int leader2 = __builtin_ctzll(rest);
    const uint32_t lb2 = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader2);
    const unsigned long long same2 = __ballot(active && bin == lb2);
    if (lane == leader2) atomicAdd(&lhist[lb2], (uint32_t)__popcll(same2));
    if (active && bin != lb && bin != lb2) atomicAdd(&lhist[bin], 1u);
}

// Adds a block's shared-memory histogram into the global one (device-wide atomics).  Blocks of
// one kernel never read each other's results: a histogram is consumed by the NEXT kernel on the
// stream, each of whose blocks resolves it for itself (block_find_bin).  A device-wide fence per
// block, as a "last block resolves" scheme needs, costs ~0.1 us and serialises across the chip.
__device__ __forceinline__ void merge_hist(const uint32_t *lhist, int nbins, uint32_t *ghist) {
    __syncthreads();
    for (int b = threadIdx.x; b < nbins; b += blockDim.x) {
        uint32_t c = lhist[b];
        if (c) atomicAdd(ghist + b, c);
    }
}
// The same for a pass-1 histogram (ghist1: the kHist1Words words of one classifier).
__device__ __forceinline__ void merge_hist1(const uint32_t *lhist, uint32_t *ghist1) {
    merge_hist(lhist, kBins1, ghist1 + (blockIdx.x % (unsigned)kHistShards) * (unsigned)kBins1);
}

struct BinChoice {
    uint32_t bin, above, inbin;
};

// Whole block: loads a histogram that an EARLIER kernel completed into shared memory `lds`
// (nbins words, nbins a multiple of 64 and at most 4096) and finds the bin of the need-th largest
// entry.  `s_out` points at 3 words of shared memory.  Ends with a barrier; lds may be reused.
// shards: the histogram is the sum of that many copies, nbins words apart.
__device__ __forceinline__ BinChoice block_find_bin(const uint32_t *ghist, int nbins, uint32_t need, uint32_t *lds,
                                                    uint32_t *s_out, int shards = 1) {
    __syncthreads();
    for (int b = threadIdx.x; b < nbins; b += blockDim.x) {
        uint32_t c = ghist[b];
        for (int h = 1; h < shards; ++h) c += ghist[(size_t)h * nbins + b];
        lds[b] = c;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        uint32_t above, inbin;
        uint32_t bin = wave_find_bin(lds, nbins / 64, need, &above, &inbin);
        if (threadIdx.x == 0) {
            s_out[0] = bin;
            s_out[1] = above;
            s_out[2] = inbin;
        }
    }
    __syncthreads();
    BinChoice r{s_out[0], s_out[1], s_out[2]};
    __syncthreads();
    return r;
}

// Filtered scans.  Passes 1 and 2 over the sample resolved its m-th largest key to 24 bits: need1 of
// the m lie in pass-1 bin b1, and r2 is the pass-2 choice inside it.  So (m - need1) + r2.above +
// r2.inbin sample rows lie at or above the threshold, and about kSampleStride times as many rows
// of the store will.  When that is far beyond the candidate list's capacity (ties: a zero model,
// scores that take few values) the scan is pointless: it returns at once, the list stays empty,
// and an empty list opens the gate of the full selection behind it.  Same answer in every workgroup.
__device__ __forceinline__ bool filter_hopeless(uint32_t m, uint32_t need1, const BinChoice &r2) {
    const uint32_t at_or_above = (m - need1) + r2.above + r2.inbin;
    return at_or_above > 2u * (uint32_t)kCandCap / (uint32_t)kSampleStride;
}

// Threshold of a filtered scan from the sample, second form (all single-classifier scans).  The scan
// of the strided sample keeps no scores and no histogram: every wave only remembers the largest
// key it met and how many of its rows had exactly that key, and leaves the pair in a slot of its
// own (S slots = waves of the launch; block 0 records S in the sample state).  The j-th largest of
// the S wave maxima estimates the threshold: with Nv sample rows spread over S waves, a wave's
// maximum exceeds the level that a fraction p of all rows exceed with probability
// 1 - (1 - p)^(Nv / S), so the level that kFilterExpect rows of the N-row store exceed is met by about
// j = S (1 - exp(-kFilterExpect Nv / (N S))) of the maxima (about kFilterExpect Nv / N = 32 when the
// waves' shares are small).  The consumer resolves that order statistic to 24 bits by two radix
// passes over the S keys in shared memory; rows at or above it (~kFilterExpect, give or take a
// fifth) are the candidates.  Ties show in the counts: when the maxima at or above the threshold
// stand for far more sample rows than the candidate list has room for at the sampling rate, the
// filtered scan is pointless (scores that are constant or take few values) and is called off.
constexpr int kMaxSampleSlots = 4096;   // 256 workgroups of 16 waves
struct SampleSlot {
    uint32_t key;     // largest key among the wave's sample rows (0: it had none)
    uint32_t count;   // how many of its rows had that key
};

__device__ __forceinline__ void sample_note(uint32_t &mx, uint32_t &cnt, uint32_t key) {
    cnt = key > mx ? 1u : (key == mx ? cnt + 1u : cnt);
    mx = key > mx ? key : mx;
}

// Whole wave, once, at the end of a sample scan: reduces the lanes' (mx, cnt) and stores the wave's slot;
// thread 0 of block 0 records the number of slots in the sample state.
__device__ __forceinline__ void sample_store(SampleSlot *slots, SelState *sample_st, uint32_t mx, uint32_t cnt) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t m2 = (uint32_t)__shfl_xor((int)mx, o, 64), c2 = (uint32_t)__shfl_xor((int)cnt, o, 64);
        cnt = m2 > mx ? c2 : (m2 == mx ? cnt + c2 : cnt);
        mx = m2 > mx ? m2 : mx;
    }
    const uint32_t nwaves = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) slots[blockIdx.x * nwaves + (threadIdx.x >> 6)] = SampleSlot{mx, cnt};
    if (blockIdx.x == 0 && threadIdx.x == 0) sample_st->ncand = gridDim.x * nwaves;
}

struct TauChoice {
    uint32_t tau;      // rows with key >= tau are candidates
    bool hopeless;     // ties: call the filtered scan off (same answer in every workgroup)
};

// Whole block, before its scan: the threshold from the slots a sample scan left (see above).
// N = rows of the store.  `lds` = kBins1 words of shared memory, `s_out` = 3 words.  Ends with a barrier.
__device__ __forceinline__ TauChoice resolve_tau_slots(const SampleSlot *slots, const SelState *sample_st, long long N,
                                                       uint32_t *lds, uint32_t *s_out) {
    const uint32_t S = sample_st->ncand;
    const float Nv = (float)(N / ((long long)kSampleGroup * kSampleStride) * kSampleGroup);
    float jf = (float)S * (1.f - __expf(-(float)kFilterExpect * Nv / ((float)N * (float)S)));
    uint32_t j = (uint32_t)(jf + 0.5f);
    j = j < 1u ? 1u : (j > S ? S : j);
    uint32_t b1 = 0u, need = j;
#pragma unroll 1
    for (int pass = 0; pass < 2; ++pass) {
        __syncthreads();
        for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lds[b] = 0u;
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < S; i += blockDim.x) {
            const uint32_t k = slots[i].key;
            if (pass == 0) atomicAdd(&lds[k >> 20], 1u);
            else if ((k >> 20) == b1) atomicAdd(&lds[(k >> 8) & 0xFFFu], 1u);
        }
        __syncthreads();
        if (threadIdx.x < 64) {
            uint32_t above, inbin;
            const uint32_t bin = wave_find_bin(lds, kBins1 / 64, need, &above, &inbin);
            if (threadIdx.x == 0) {
                s_out[0] = bin;
                s_out[1] = above;
                s_out[2] = 0u;
            }
        }
        __syncthreads();
        if (pass == 0) {
            b1 = s_out[0];
            need -= s_out[1];
        }
    }
    TauChoice c;
    c.tau = ((b1 << 12) | s_out[0]) << 8;
    __syncthreads();
    uint32_t mine = 0u;
    for (uint32_t i = threadIdx.x; i < S; i += blockDim.x) mine += slots[i].key >= c.tau ? slots[i].count : 0u;
    if (mine) atomicAdd(&s_out[2], mine);
    __syncthreads();
    c.hopeless = s_out[2] > 2u * (uint32_t)kCandCap / (uint32_t)kSampleStride;
    __syncthreads();
    return c;
}

// Dynamic work distribution for the streaming scans.  The chip's eight dies stream at visibly
// different rates and the waves of a workgroup drift apart, so a static split of the rows leaves
// a tail of 5-10 % in which most of the chip idles.  Instead the work is cut into tiles (what one
// wave handles per iteration) and chunks of `chunk_tiles` consecutive tiles (about 256 KiB of
// rows).  A workgroup draws chunk numbers from a counter in global memory (zero before the
// launch; one atomic per chunk, ordered one chunk ahead so its latency hides behind a chunk of
// work) and its waves draw the tiles of the current chunk from a ticket word in shared memory.
struct TileQueue {
    unsigned long long cur;   // (chunk number << 32) | next tile ticket of that chunk
    uint32_t next;            // number of the chunk after it; kNoChunk while it is being ordered
};
constexpr uint32_t kNoChunk = 0xFFFFFFFFu;

// Tiles per chunk: `full` (about 256 KiB of rows) for long scans.  A short scan is cut into two
// chunks per workgroup, which are exactly the two that tile_queue_init hands out, so that every
// workgroup finds work and no further chunk is ever ordered.  Same value in every workgroup.
__device__ __forceinline__ uint32_t tile_queue_chunk_tiles(long long total_tiles, uint32_t full) {
    const long long parts = 2LL * gridDim.x;
    const long long fair = (total_tiles + parts - 1) / parts;
    return fair >= (long long)full ? full : (fair < 1 ? 1u : (uint32_t)fair);
}

// One thread per workgroup, before a barrier that precedes the first tile_queue_draw.
__device__ __forceinline__ void tile_queue_init(TileQueue *q, uint32_t *chunk_ctr) {
    const uint32_t c = atomicAdd(chunk_ctr, 2u);
    q->cur = (unsigned long long)c << 32;
    q->next = c + 1u;
}

// Whole wave (all lanes active): the next tile of this wave, or -1 when none is left.  The result
// is the same in every lane.  Tiles are numbered chunk * chunk_tiles + ticket; only tiles below
// total_tiles exist.
__device__ __forceinline__ long long tile_queue_draw(TileQueue *q, uint32_t *chunk_ctr, uint32_t chunk_tiles,
                                                     long long total_tiles) {
    const uint32_t total_chunks = (uint32_t)((total_tiles + chunk_tiles - 1) / chunk_tiles);
    uint32_t gid = 0u, off = 0u;
    if ((threadIdx.x & 63) == 0) {
        for (;;) {
            const unsigned long long old =
                __hip_atomic_fetch_add(&q->cur, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            gid = (uint32_t)(old >> 32);
            off = (uint32_t)old;
            if (gid >= total_chunks) break;                                   // nothing left
            if (off < chunk_tiles) {
                if ((long long)gid * chunk_tiles + off < total_tiles) break;  // a tile
                continue;                                                     // past the last tile of the last chunk
            }
            if (off == chunk_tiles) {
                // first ticket past the chunk: this wave installs the next chunk and orders the
                // chunk after it (the others retry until the new chunk appears)
                uint32_t g;
                while ((g = __hip_atomic_exchange(&q->next, kNoChunk, __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_WORKGROUP)) == kNoChunk)
                    __builtin_amdgcn_s_sleep(2);
                __hip_atomic_store(&q->cur, (unsigned long long)g << 32, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
                // (with at most two chunks per workgroup every chunk was handed out at the start)
                const uint32_t after = (g < total_chunks && total_chunks > 2u * gridDim.x) ? atomicAdd(chunk_ctr, 1u) : total_chunks;
                __hip_atomic_store(&q->next, after, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                continue;                                                     // and draws again like everyone else
            }
            __builtin_amdgcn_s_sleep(2);                                      // another wave is installing
        }
    }
    // (the builtin works on int; the values are unsigned)
    gid = (uint32_t)__builtin_amdgcn_readfirstlane((int)gid);
    off = (uint32_t)__builtin_amdgcn_readfirstlane((int)off);
    return gid >= total_chunks ? -1LL : (long long)gid * chunk_tiles + off;
}

// Rows [begin, end) of the chunk that selection block b of nblocks owns; chunks are
// contiguous, ascending in b, and a multiple of 1024 rows long (except the last).
__device__ __forceinline__ void sel_chunk(long long N, int b, int nblocks, long long *begin, long long *end) {
    long long per = (N + nblocks - 1) / nblocks;
    per = (per + 1023) / 1024 * 1024;
    long long s = per * b;
    long long e = s + per;
    *begin = s < N ? s : N;
    *end = e < N ? e : N;
}

}  // namespace otf
