// Exact top-k of fp32 scores by radix selection on an order-preserving 32-bit key, followed by
// a bitonic sort of the survivors.  (Paper Sec. 4, "Ranking": the scores are sorted on the GPU
// and the head of the list goes to the front-end; only the k best are needed, so the full sort
// is replaced by select-then-sort, whose result equals the first k entries of the full sort.)
//
// Passes over the scores of one classifier (all passes use kSelBlocks blocks per classifier):
//   pass 1  histogram of key bits 31..20   (fused into the scoring kernels; stand-alone here)
//   pass 2  histogram of bits 19..8 among keys in the pass-1 bin of the k-th key   [mode >= 1]
//   pass 3  per-block histograms of bits 7..0 among keys sharing its top 24 bits    [mode == 2]
//   gather  every key above the resolved threshold is appended to a candidate list; in mode 2
//           the rows whose key EQUALS the k-th key are taken in ascending row order
//   sort    one block sorts the candidates by (key, ~index) descending and emits the first k
// A pass only accumulates its histogram (device-wide atomics).  The kernel of the NEXT pass
// resolves it: every block finds the bin for itself from the finished histogram (a few
// microseconds, no cross-block synchronisation inside a kernel) and block 0 records the result
// for the kernels after it.  A pass returns at once when the previous one was decisive, i.e. the
// candidates already fit the list (mode 0 / 1).
//
// Filtered scans end here as well.  Their threshold comes from the largest keys the waves of a
// sample scan met (resolve_tau_slots in otf_device.h; for many classifiers at once from passes 1
// and 2 over the sample's scores, `tau_key`); the full scan appends only rows at or above it.
// Two launches stand behind it, both gated on the state the scan left (Gate in otf_device.h): a
// re-scan that materialises the scores, and select_fused_gated_kernel.  If the list serves (at
// least k rows on it, none lost) the re-scan returns at once and one workgroup of the second
// launch sorts the list; otherwise the re-scan runs and the second launch does passes 2 and 3,
// the gather and the sort of the full selection.  (Many classifiers at once: filter_sort_kernel
// sorts every list and raises one flag for all if any cannot serve.)
#include <algorithm>

#include "otf_internal.h"

namespace otf {

__global__ __launch_bounds__(256) void select_init_kernel(SelState *st, uint32_t *hist1, uint32_t *hist2,
                                                          uint32_t *hist3, SelState *sample_st, int Q) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    uint32_t *stw = reinterpret_cast<uint32_t *>(st);
    for (size_t i = tid; i < (size_t)Q * (sizeof(SelState) / 4); i += step) stw[i] = 0u;
    for (size_t i = tid; i < (size_t)Q * kHist1Words; i += step) hist1[i] = 0u;
    for (size_t i = tid; i < (size_t)Q * kBins2; i += step) hist2[i] = 0u;
    if (hist3)
        for (size_t i = tid; i < (size_t)Q * kBins3; i += step) hist3[i] = 0u;
    if (sample_st) {                                  // the state that thresholds a sample, in the same launch
        uint32_t *sw = reinterpret_cast<uint32_t *>(sample_st);
        for (size_t i = tid; i < (size_t)Q * (sizeof(SelState) / 4); i += step) sw[i] = 0u;
    }
}

// Four consecutive scores of this thread for the tile starting at t0 (tile = 4 * blockDim rows);
// valid[j] tells which exist.  Uses one 16-byte load when the row of scores allows it.
__device__ __forceinline__ void load4(const float *s, long long i, long long end, bool vec_ok, float *v, bool *valid) {
    if (vec_ok && i + 3 < end) {
        const float4 t = *reinterpret_cast<const float4 *>(s + i);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        valid[0] = valid[1] = valid[2] = valid[3] = true;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            valid[j] = i + j < end;
            v[j] = valid[j] ? s[i + j] : 0.f;
        }
    }
}

__device__ __forceinline__ bool row_vec_ok(const float *s) { return (reinterpret_cast<uintptr_t>(s) & 15u) == 0; }

// Calls f(score, valid, row) for every score of [begin, end) that this thread owns (threads take groups
// of 4 consecutive scores, the block 4 * blockDim.x per step), every thread of the block the same
// number of times.  While whole steps remain and the row allows 16-byte loads, four unconditional
// loads are in flight per thread: with one checked load per step a pass over 50M scores ran at
// 0.7 TB/s.
template <typename F>
__device__ __forceinline__ void for_each_score(const float *s, long long begin, long long end, bool vec_ok, F f) {
    const long long span = 4LL * blockDim.x;
    long long t0 = begin;
    if (vec_ok) {
        for (; t0 + 4 * span <= end; t0 += 4 * span) {
            float4 t[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) t[h] = *reinterpret_cast<const float4 *>(s + t0 + h * span + 4 * threadIdx.x);
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const long long i0 = t0 + h * span + 4 * threadIdx.x;
                f(t[h].x, true, i0);
                f(t[h].y, true, i0 + 1);
                f(t[h].z, true, i0 + 2);
                f(t[h].w, true, i0 + 3);
            }
        }
    }
    for (; t0 < end; t0 += span) {
        float v[4];
        bool ok[4];
        const long long i0 = t0 + 4 * threadIdx.x;
        load4(s, i0, end, vec_ok, v, ok);
#pragma unroll
        for (int j = 0; j < 4; ++j) f(v[j], ok[j], i0 + j);
    }
}

__global__ __launch_bounds__(1024) void hist1_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                    SelState *st_all, uint32_t *hist1_all, Gate gate) {
    __shared__ uint32_t lhist[kBins1];
    if (!gate_open(gate)) return;                          // uniform over the grid
    const int q = blockIdx.y;
    const float *s = scores + (long long)q * ld;
    const bool vec_ok = row_vec_ok(s);
    for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, gridDim.x, &begin, &end);
    for_each_score(s, begin, end, vec_ok, [&](float v, bool ok, long long) { hist_add_wave(lhist, float_to_key(v) >> 20, ok); });
    merge_hist1(lhist, hist1_all + (size_t)q * kHist1Words);
}

// Pass 2.  Resolves pass 1 first (rank k in hist1); returns at once when pass 1 was decisive.
__global__ __launch_bounds__(1024) void hist2_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                    int k, SelState *st_all, const uint32_t *hist1_all,
                                                    uint32_t *hist2_all) {
    __shared__ uint32_t lhist[kBins2];
    __shared__ uint32_t s_out[3];
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    const BinChoice r1 = block_find_bin(hist1_all + (size_t)q * kHist1Words, kBins1, (uint32_t)k, lhist, s_out, kHistShards);
    const uint32_t b1 = r1.bin, need1 = (uint32_t)k - r1.above, c1 = r1.above + r1.inbin;
    const bool decisive = c1 <= (uint32_t)kCandCap;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st->b1 = b1;
        st->need1 = need1;
        st->mode = decisive ? 0u : 1u;
        if (decisive) {
            st->ncand = c1;
            st->tex = ((long long)b1 << 20) - 1;
        }
    }
    if (decisive) return;
    const float *s = scores + (long long)q * ld;
    const bool vec_ok = row_vec_ok(s);
    for (int b = threadIdx.x; b < kBins2; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, gridDim.x, &begin, &end);
    for_each_score(s, begin, end, vec_ok, [&](float v, bool ok, long long) {
        const uint32_t key = float_to_key(v);
        hist_add_wave(lhist, (key >> 8) & 0xFFFu, ok && (key >> 20) == b1);
    });
    merge_hist(lhist, kBins2, hist2_all + (size_t)q * kBins2);
}

// Resolution of pass 2 from the state pass 2's kernel left and its histogram.  Whole block.
struct Pass2 {
    uint32_t p24, need2, c2;
};
__device__ __forceinline__ Pass2 resolve_pass2(const SelState *st, const uint32_t *hist2, int k, uint32_t *lds,
                                               uint32_t *s_out) {
    const uint32_t b1 = st->b1, need1 = st->need1;
    const BinChoice r2 = block_find_bin(hist2, kBins2, need1, lds, s_out);
    Pass2 p;
    p.p24 = (b1 << 12) | r2.bin;
    p.need2 = need1 - r2.above;
    p.c2 = ((uint32_t)k - need1) + r2.above + r2.inbin;     // keys >= p24 << 8
    return p;
}

// One workgroup per classifier: the threshold of its filtered scan from the Nv scores of the strided
// sample (many classifiers at once; a single classifier's scans use wave maxima instead, see
// resolve_tau_slots).  Two radix passes in shared memory resolve the m-th largest sample key to 24
// bits: tau_key; about m * N / Nv rows of the store lie at or above it.  c2 sample rows do.  When
// that predicts far more rows of the store than the candidate list holds (ties: a zero model, scores
// that take few values) the filtered scan is called off for the whole call: the fallback flag of the
// full selection's state is raised here already, and the scan, which is given that state as its
// gate, returns at once.  (As three launches -- pass 1, pass 2, resolution, each over all
// classifiers -- this took 27 us of a 64-classifier call; a sample is a few tens of thousands of
// scores per classifier.)  Requires 1 <= m <= Nv.
__global__ __launch_bounds__(1024) void sample_threshold_kernel(const float *__restrict__ sample, long long Nv,
                                                                long long ld, int m, SelState *sample_st_all,
                                                                SelState *main_st_all) {
    __shared__ uint32_t lhist[kBins1];
    __shared__ uint32_t s_out[3];
    static_assert(kBins2 <= kBins1, "both passes use the same shared histogram");
    const int q = blockIdx.x;
    const float *s = sample + (long long)q * ld;
    const bool vec_ok = row_vec_ok(s);
    uint32_t b1 = 0u, need = (uint32_t)m, above1 = 0u;
#pragma unroll 1
    for (int pass = 0; pass < 2; ++pass) {
        for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
        __syncthreads();
        for_each_score(s, 0, Nv, vec_ok, [&](float v, bool ok, long long) {
            const uint32_t key = float_to_key(v);
            if (pass == 0) hist_add_wave(lhist, key >> 20, ok);
            else hist_add_wave(lhist, (key >> 8) & 0xFFFu, ok && (key >> 20) == b1);
        });
        __syncthreads();
        if (threadIdx.x < 64) {
            uint32_t above, inbin;
            const uint32_t bin = wave_find_bin(lhist, kBins1 / 64, need, &above, &inbin);
            if (threadIdx.x == 0) {
                s_out[0] = bin;
                s_out[1] = above;
                s_out[2] = inbin;
            }
        }
        __syncthreads();
        if (pass == 0) {
            b1 = s_out[0];
            above1 = s_out[1];
            need -= above1;
        }
    }
    if (threadIdx.x == 0) {
        sample_st_all[q].tau_key = ((b1 << 12) | s_out[0]) << 8;
        const uint32_t c2 = above1 + s_out[1] + s_out[2];           // sample keys at or above the threshold
        if (c2 > 2u * (uint32_t)kCandCap / (uint32_t)kSampleStride) atomicOr(&main_st_all[0].fallback, 1u);
    }
}

// Pass 3 (only when thousands of keys share the top 24 bits of the k-th: ties or near-ties).
__global__ __launch_bounds__(1024) void hist3_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                    int k, SelState *st_all, const uint32_t *hist2_all,
                                                    uint32_t *hist3_all, uint32_t *blockhist3_all) {
    __shared__ uint32_t lhist[kBins2];
    __shared__ uint32_t s_out[3];
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    if (st->mode == 0u) return;                         // pass 1 was decisive
    const Pass2 p = resolve_pass2(st, hist2_all + (size_t)q * kBins2, k, lhist, s_out);
    const bool decisive = p.c2 <= (uint32_t)kCandCap;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st->p24 = p.p24;
        st->need2 = p.need2;
        st->mode = decisive ? 1u : 2u;
        if (decisive) {
            st->ncand = p.c2;
            st->tex = ((long long)p.p24 << 8) - 1;
        }
    }
    if (decisive) return;
    const float *s = scores + (long long)q * ld;
    const bool vec_ok = row_vec_ok(s);
    for (int b = threadIdx.x; b < kBins3; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, gridDim.x, &begin, &end);
    for_each_score(s, begin, end, vec_ok, [&](float v, bool ok, long long) {
        const uint32_t key = float_to_key(v);
        hist_add_wave(lhist, key & 0xFFu, ok && (key >> 8) == p.p24);
    });
    __syncthreads();
    // per-block counts (for the row-ordered split of ties) and the total histogram
    uint32_t *bh = blockhist3_all + ((size_t)q * kSelBlocks + blockIdx.x) * kBins3;
    for (int b = threadIdx.x; b < kBins3; b += blockDim.x) bh[b] = lhist[b];
    merge_hist(lhist, kBins3, hist3_all + (size_t)q * kBins3);
}

__device__ __forceinline__ unsigned long long pack_cand(uint32_t key, long long row) {
    return ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)row);
}

// Gather pass over rows [begin, end) of one classifier's scores by one workgroup: every key above
// `tex` goes to the candidate list (collected per workgroup and appended with ONE device-wide atomic:
// thousands of atomics on the single cursor would serialise, ~18 ns each).  With `ordered`, the
// rows whose key EQUALS T are placed in row order at list positions k - r + rank, rank counting
// such rows from `eqbase` (those in the workgroups before this one) up to r.
constexpr uint32_t kGatherLocalCap = 2048;
__device__ __forceinline__ void gather_rows(const float *__restrict__ s, long long begin, long long end, bool vec_ok,
                                            long long tex, bool ordered, uint32_t T, uint32_t r, uint32_t eqbase, int k,
                                            SelState *st, unsigned long long *cand) {
    __shared__ uint32_t wave_cnt[64];                       // [step of a round][wave]
    __shared__ unsigned long long local[kGatherLocalCap];
    __shared__ uint32_t s_local_n, s_base;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    if (threadIdx.x == 0) s_local_n = 0u;
    __syncthreads();                                       // s_local_n is initialised
    auto take = [&](uint32_t key, long long row) {         // a row above the threshold
        const uint32_t lp = atomicAdd(&s_local_n, 1u);
        if (lp < kGatherLocalCap) {
            local[lp] = pack_cand(key, row);
        } else {                                           // block buffer full: straight to the list
            uint32_t pos = atomicAdd(&st->gcursor, 1u);
            if (pos < (uint32_t)kCandCap) cand[pos] = pack_cand(key, row);
        }
    };
    // Rows equal to the k-th key are placed in row order, a step of the block at a time, until the
    // block has met all r of them (eqbase counts those before the current step); the rows after
    // that, and all rows of a block with no ties to place, only need the keys above the threshold.
    long long t0 = begin;
    constexpr int OS = 4;                                  // steps of 4 * blockDim rows per round of barriers
    const long long span = 4LL * blockDim.x;
    for (; ordered && eqbase < r && t0 < end; t0 += OS * span) {
        float v[OS][4];
        bool ok[OS][4];
        uint32_t key[OS][4], neq[OS], incl[OS];
#pragma unroll
        for (int u = 0; u < OS; ++u) load4(s, t0 + u * span + 4 * threadIdx.x, end, vec_ok, v[u], ok[u]);
#pragma unroll
        for (int u = 0; u < OS; ++u) {
            const long long i0 = t0 + u * span + 4 * threadIdx.x;
            neq[u] = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                key[u][j] = float_to_key(v[u][j]);
                if (ok[u][j] && (long long)key[u][j] > tex) take(key[u][j], i0 + j);
                neq[u] += (ok[u][j] && key[u][j] == T) ? 1u : 0u;
            }
            // rank of each row equal to T in row order: threads hold 4 consecutive rows of a step
            incl[u] = neq[u];                              // inclusive prefix over the lanes of the wave
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t t = __shfl_up(incl[u], o, 64);
                if (lane >= o) incl[u] += t;
            }
            if (lane == 63) wave_cnt[u * 16 + wave] = incl[u];
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < OS; ++u) {
            const long long i0 = t0 + u * span + 4 * threadIdx.x;
            uint32_t before = 0, total = 0;
            for (int w = 0; w < nwaves; ++w) {
                const uint32_t c = wave_cnt[u * 16 + w];
                if (w < wave) before += c;
                total += c;
            }
            uint32_t rank = eqbase + before + incl[u] - neq[u];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (ok[u][j] && key[u][j] == T) {
                    if (rank < r) {
                        const uint32_t pos = (uint32_t)k - r + rank;
                        if (pos < (uint32_t)kCandCap) cand[pos] = pack_cand(key[u][j], i0 + j);
                    }
                    ++rank;
                }
            }
            eqbase += total;
        }
        __syncthreads();
    }
    for_each_score(s, t0, end, vec_ok, [&](float v, bool ok, long long row) {
        const uint32_t key = float_to_key(v);
        if (ok && (long long)key > tex) take(key, row);
    });
    __syncthreads();
    const uint32_t nloc = s_local_n < kGatherLocalCap ? s_local_n : kGatherLocalCap;
    if (threadIdx.x == 0 && nloc) s_base = atomicAdd(&st->gcursor, nloc);
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < nloc; i += blockDim.x) {
        const uint32_t pos = s_base + i;
        if (pos < (uint32_t)kCandCap) cand[pos] = local[i];
    }
}

__global__ __launch_bounds__(512) void gather_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                     int k, SelState *st_all, const uint32_t *hist3_all,
                                                     const uint32_t *blockhist3_all, unsigned long long *cand_all) {
    __shared__ uint32_t lhist[kBins3];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t wave_sum_s[16];
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    const uint32_t mode = st->mode;
    long long tex = st->tex;
    uint32_t T = 0, r = 0, eqbase = 0;
    if (mode == 2u) {
        // resolve pass 3: the k-th key itself, how many rows equal to it belong to the list, and
        // how many such rows lie in the blocks before this one (ties go to the lowest rows)
        const uint32_t need2 = st->need2;
        const BinChoice r3 = block_find_bin(hist3_all + (size_t)q * kBins3, kBins3, need2, lhist, s_out);
        T = (st->p24 << 8) | r3.bin;
        r = need2 - r3.above;
        tex = (long long)T;
        const uint32_t *bh = blockhist3_all + (size_t)q * kSelBlocks * kBins3 + r3.bin;
        uint32_t mine = 0;
        for (int b = threadIdx.x; b < (int)blockIdx.x; b += blockDim.x) mine += bh[(size_t)b * kBins3];
        uint32_t acc = mine;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
        if ((threadIdx.x & 63) == 0) wave_sum_s[threadIdx.x >> 6] = acc;
        __syncthreads();
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) eqbase += wave_sum_s[w];
        __syncthreads();
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            st->T = T;
            st->r = r;
            st->ncand = (uint32_t)k;
        }
    }
    const float *s = scores + (long long)q * ld;
    long long begin, end;
    sel_chunk(N, blockIdx.x, gridDim.x, &begin, &end);
    gather_rows(s, begin, end, row_vec_ok(s), tex, (mode == 2u) && (eqbase < r), T, r, eqbase, k, st,
                cand_all + (size_t)q * kCandCap);
}

// ---------------------------------------------------------------------------------------------
// Final step, one block of 1024 threads per classifier: from n <= kCandCap packed candidates
// (key << 32 | ~row, all distinct) emit the k largest in descending order.
//
//   1. pre-selection: a 4096-bin histogram over the candidates' own key range finds the bin of
//      the k-th largest; candidates below that bin are dropped (usually n ~ 4k shrinks to ~k);
//   2. bitonic sort of the survivors, padded to a power of two P: every thread keeps P/1024
//      elements in registers; compare-exchange partners less than 64 apart are reached with
//      wave shuffles, partners in another wave through shared memory, partners 1024 or more
//      apart are the thread's own registers -- 10 shared-memory exchanges instead of ~90.
constexpr int kSortThreads = 1024;
constexpr int kSortLdsBytes = kBins1 * 4 + kCandCap * 8;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xF, 0xF, true);
}
// The 32-bit value of lane ^ BIT, through the vector ALU's own lane exchanges (data-parallel moves
// within a row of 16 lanes, v_permlane16_swap / v_permlane32_swap across rows and halves) instead
// of a shuffle through shared memory, whose latency a chain of dependent sorting steps pays in full.
template <int BIT>
__device__ __forceinline__ uint32_t lane_xor_u32(uint32_t v) {
    if constexpr (BIT == 1) return dpp_u32<0xB1>(v);                       // quad_perm [1,0,3,2]
    else if constexpr (BIT == 2) return dpp_u32<0x4E>(v);                  // quad_perm [2,3,0,1]
    else if constexpr (BIT == 4) return dpp_u32<0x1B>(dpp_u32<0x141>(v));  // half mirror, then quad reversed
    else if constexpr (BIT == 8) return dpp_u32<0x128>(v);                 // row_ror:8
    else {
        // swap(v, v): [0] = the value of the lane with bit BIT clear, [1] = of the one with it set
        const bool up = (threadIdx.x & BIT) != 0;
        if constexpr (BIT == 16) {
            const auto sw = __builtin_amdgcn_permlane16_swap(v, v, false, false);
            return up ? sw[0] : sw[1];
        } else {
            static_assert(BIT == 32, "lane bit");
            const auto sw = __builtin_amdgcn_permlane32_swap(v, v, false, false);
            return up ? sw[0] : sw[1];
        }
    }
}
template <int BIT>
__device__ __forceinline__ unsigned long long lane_xor_u64(unsigned long long v) {
    const uint32_t lo = lane_xor_u32<BIT>((uint32_t)v), hi = lane_xor_u32<BIT>((uint32_t)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}
// One compare-exchange step of the bitonic network between lanes BIT apart.
template <int E, int BIT>
__device__ __forceinline__ void wave_exchange(unsigned long long *r, uint32_t size, uint32_t tid) {
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const uint32_t e = (uint32_t)j * kSortThreads + tid;
        const unsigned long long y = lane_xor_u64<BIT>(r[j]);
        const bool keep_larger = ((e & (uint32_t)BIT) == 0u) == ((e & size) == 0u);
        r[j] = keep_larger ? (r[j] > y ? r[j] : y) : (r[j] < y ? r[j] : y);
    }
}

// Sorts a[0..P) descending.  P is a power of two, 64 <= P <= 1024 * E, and E = max(1, P / 1024).
template <int E>
__device__ __forceinline__ void bitonic_desc(unsigned long long *a, uint32_t P) {
    const uint32_t tid = threadIdx.x;
    const bool live = tid < P;                       // whole waves (P >= 64)
    unsigned long long r[E];
#pragma unroll
    for (int j = 0; j < E; ++j) r[j] = live ? a[j * kSortThreads + tid] : 0ull;
    for (uint32_t size = 2; size <= P; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            if (stride >= (uint32_t)kSortThreads) {              // partner is another register of this thread
                const int dj = (int)(stride / kSortThreads);
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    if ((j & dj) == 0 && (j | dj) < E) {
                        const uint32_t e = (uint32_t)j * kSortThreads + tid;
                        const bool desc = (e & size) == 0u;
                        unsigned long long x = r[j], y = r[j | dj];
                        if (desc ? (x < y) : (x > y)) {
                            r[j] = y;
                            r[j | dj] = x;
                        }
                    }
                }
            } else if (stride >= 64u) {                           // partner in another wave: through shared memory
                __syncthreads();
                if (live) {
#pragma unroll
                    for (int j = 0; j < E; ++j) a[j * kSortThreads + tid] = r[j];
                }
                __syncthreads();
                if (live) {
#pragma unroll
                    for (int j = 0; j < E; ++j) {
                        const uint32_t e = (uint32_t)j * kSortThreads + tid;
                        const unsigned long long y = a[e ^ stride];
                        const bool keep_larger = ((e & stride) == 0u) == ((e & size) == 0u);
                        r[j] = keep_larger ? (r[j] > y ? r[j] : y) : (r[j] < y ? r[j] : y);
                    }
                }
            } else {                                              // this and all smaller strides: partners in this wave
                switch (stride) {
                    case 32: wave_exchange<E, 32>(r, size, tid); [[fallthrough]];
                    case 16: wave_exchange<E, 16>(r, size, tid); [[fallthrough]];
                    case 8: wave_exchange<E, 8>(r, size, tid); [[fallthrough]];
                    case 4: wave_exchange<E, 4>(r, size, tid); [[fallthrough]];
                    case 2: wave_exchange<E, 2>(r, size, tid); [[fallthrough]];
                    default: wave_exchange<E, 1>(r, size, tid);
                }
                break;
            }
        }
    }
    __syncthreads();
    if (live) {
#pragma unroll
        for (int j = 0; j < E; ++j) a[j * kSortThreads + tid] = r[j];
    }
    __syncthreads();
}

// lds: kSortLdsBytes of shared memory.  Every thread of the 1024 calls.
__device__ __forceinline__ void select_sort_emit(uint8_t *lds, const unsigned long long *cand, uint32_t n, int k,
                                                 float *out_scores, int32_t *out_idx) {
    uint32_t *hist = reinterpret_cast<uint32_t *>(lds);
    unsigned long long *a = reinterpret_cast<unsigned long long *>(lds + kBins1 * 4);
    __shared__ uint32_t s_lo, s_hi, s_cnt, s_bin;
    const uint32_t tid = threadIdx.x;
    constexpr int EMAX = kCandCap / kSortThreads;
    unsigned long long r[EMAX];
    uint32_t lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
    for (int j = 0; j < EMAX; ++j) {
        const uint32_t i = (uint32_t)j * kSortThreads + tid;
        r[j] = i < n ? cand[i] : 0ull;
        if (i < n) {
            const uint32_t key = (uint32_t)(r[j] >> 32);
            lo = key < lo ? key : lo;
            hi = key > hi ? key : hi;
        }
    }
    if (tid == 0) {
        s_lo = 0xFFFFFFFFu;
        s_hi = 0u;
        s_cnt = 0u;
    }
    for (uint32_t b = tid; b < (uint32_t)kBins1; b += kSortThreads) hist[b] = 0u;
    __syncthreads();
    // block-wide range of the keys: one shared-memory atomic per wave
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t olo = (uint32_t)__shfl_xor((int)lo, o, 64), ohi = (uint32_t)__shfl_xor((int)hi, o, 64);
        lo = olo < lo ? olo : lo;
        hi = ohi > hi ? ohi : hi;
    }
    if ((tid & 63u) == 0u && lo <= hi) {
        atomicMin(&s_lo, lo);
        atomicMax(&s_hi, hi);
    }
    __syncthreads();
    lo = s_lo;
    hi = s_hi;
    uint32_t n2 = n;
    if (n > (uint32_t)k) {
        // bins over [lo, hi]: (key - lo) >> sh < 4096
        const uint32_t range = hi - lo;
        const int sh = range < (uint32_t)kBins1 ? 0 : (32 - __builtin_clz(range)) - 12;
#pragma unroll
        for (int j = 0; j < EMAX; ++j) {
            const uint32_t i = (uint32_t)j * kSortThreads + tid;
            if (i < n) atomicAdd(&hist[((uint32_t)(r[j] >> 32) - lo) >> sh], 1u);
        }
        __syncthreads();
        if (tid < 64) {
            uint32_t above, inbin;
            const uint32_t bin = wave_find_bin(hist, kBins1 / 64, (uint32_t)k, &above, &inbin);
            if (tid == 0) s_bin = bin;
        }
        __syncthreads();
        const uint32_t bin = s_bin;
        // survivors are compacted into a[]; slots are handed out per wave (one atomic per wave and step)
        const uint32_t lane = tid & 63u;
#pragma unroll
        for (int j = 0; j < EMAX; ++j) {
            const uint32_t i = (uint32_t)j * kSortThreads + tid;
            const bool keep = i < n && (((uint32_t)(r[j] >> 32) - lo) >> sh) >= bin;
            const unsigned long long m = __ballot(keep);
            if (m) {                                                   // uniform per wave
                uint32_t base = 0;
                if (lane == 0) base = atomicAdd(&s_cnt, (uint32_t)__popcll(m));
                base = (uint32_t)__shfl((int)base, 0, 64);
                if (keep) a[base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull))] = r[j];
            }
        }
        __syncthreads();
        n2 = s_cnt;
    } else {
#pragma unroll
        for (int j = 0; j < EMAX; ++j) {
            const uint32_t i = (uint32_t)j * kSortThreads + tid;
            if (i < n) a[i] = r[j];
        }
    }
    uint32_t P = 64;
    while (P < n2) P <<= 1;
    for (uint32_t i = n2 + tid; i < P; i += kSortThreads) a[i] = 0ull;     // padding sorts last
    __syncthreads();
    if (P <= 1024u) bitonic_desc<1>(a, P);
    else if (P == 2048u) bitonic_desc<2>(a, P);
    else if (P == 4096u) bitonic_desc<4>(a, P);
    else bitonic_desc<8>(a, P);
    for (uint32_t j = tid; j < (uint32_t)k; j += kSortThreads) {
        const unsigned long long e = a[j];
        out_scores[j] = key_to_float((uint32_t)(e >> 32));
        out_idx[j] = (int32_t)(0xFFFFFFFFu - (uint32_t)(e & 0xFFFFFFFFull));
    }
}

// One block per classifier: sorts the candidate list of the full selection.
__global__ __launch_bounds__(kSortThreads) void sort_emit_kernel(const SelState *st_all,
                                                                 const unsigned long long *cand_all, int k,
                                                                 float *out_scores, int32_t *out_idx) {
    extern __shared__ __attribute__((aligned(16))) uint8_t sort_lds[];
    const int q = blockIdx.x;
    uint32_t n = st_all[q].ncand;
    if (n > (uint32_t)kCandCap) n = kCandCap;
    select_sort_emit(sort_lds, cand_all + (size_t)q * kCandCap, n, k, out_scores + (size_t)q * k,
                     out_idx + (size_t)q * k);
}

// One block per classifier: end of the filtered scans of many classifiers.  `cursor` counts the rows
// a scan appended, or is some number above the capacity when more passed than the list holds (a
// wave stops counting once it has seen the list full).  With k <= cursor <= capacity the list holds
// every row of the top k, so sorting it gives the exact answer; otherwise the fallback is raised
// for all classifiers.  (One classifier: the last launch of the call judges and sorts, see
// select_fused_gated_kernel.)
__global__ __launch_bounds__(kSortThreads) void filter_sort_kernel(SelState *st_all,
                                                                   const unsigned long long *cand_all, int k,
                                                                   float *out_scores, int32_t *out_idx) {
    extern __shared__ __attribute__((aligned(16))) uint8_t sort_lds[];
    const int q = blockIdx.x;
    SelState *st = st_all + q;
    const uint32_t n = st->cursor;
    if (n < (uint32_t)k || n > (uint32_t)kCandCap) {
        if (threadIdx.x == 0) atomicOr(&st_all[0].fallback, 1u);
        return;
    }
    select_sort_emit(sort_lds, cand_all + (size_t)q * kCandCap, n, k, out_scores + (size_t)q * k,
                     out_idx + (size_t)q * k);
}

// The last launch of a filtered ranking: the sort of the scan's list, or, behind a gate, the full
// selection in ONE launch.  A ranking call enqueues its fallback behind the filtered scan whether
// it will be needed or not, and a kernel that returns at once still costs ~4 us on the stream:
// four such launches (passes 2 and 3, gather, sort) and a launch of its own for the sort of the
// list were a fifteenth of a ranking call.  With the gate open this kernel does the work of the
// four:
//   every workgroup   resolves pass 1 (the gated scan accumulated its histogram).  Decisive (the
//                     usual case): gathers the candidates of its share of the rows, takes a ticket,
//                     and the workgroup that draws the last one sorts the list.
//   not decisive      (scores that crowd into one 12-bit bin or tie by the thousand: integer scores
//                     of short binary codes, duplicated rows) the passes that follow each need
//                     the sum of what all workgroups found in the pass before.  The workgroups
//                     MEET between passes: each announces its arrival (a counter in global memory,
//                     device-wide fences on both sides) and waits for the verdict of the last one
//                     to arrive.  The wait is bounded.  If nobody has given up, the last arrival's
//                     verdict is "together" and every workgroup takes its share of the next pass
//                     (pass 2's histogram, then either the gather, or pass 3 with per-workgroup tie
//                     counts and a gather that hands the ties out in row order).  If a wait ran out
//                     first (the workgroups were not all resident: another kernel held the compute
//                     units), the verdict is "alone": the waiting workgroups leave, and the last
//                     arrival -- which exists, never waits, and finds the work of all the others
//                     complete -- finishes the remaining passes over all rows by itself, slowly
//                     but exactly.  `meet` = 0 (the grid may exceed what is resident at once: many
//                     classifiers) goes that way from the start.
// Stand-alone selection (otf_topk, scans that materialise their scores) keeps the chain of four
// launches: there every pass runs, and when pass 1 does not decide -- the headline store: 1M scores
// whose k-th shares its 12-bit bin with more rows than the list holds -- this kernel takes 34 us
// against the chain's 31 (a meeting costs what a launch costs).
//
// Fences: a meeting or a ticket is ONE thread's release or acquire, passed on to its workgroup by
// the barriers around it.  Device-wide fences executed by every wave of every workgroup
// (__threadfence() before the ticket, an acquire after each meeting) cost 40-55 us apiece on 256
// workgroups of 16 waves: the worst case of the filtered ranking went from 1.10 to 0.97 ms.
enum MeetRole : uint32_t { kTogether = 1u, kAlone = 2u, kLeave = 3u };
constexpr uint32_t kMeetSpinLimit = 1u << 14;               // polls of ~1-2 us: ten times a pass over any store
                                                            // (diagnostic switch OTF_DEBUG_MEET_SPIN_LIMIT: 1 makes every wait give up)

// Whole workgroup.  Everything this workgroup wrote before the call is visible to whoever goes on.
__device__ __forceinline__ MeetRole meet(uint32_t *met, uint32_t *verdict, uint32_t groups, uint32_t spin_limit,
                                         uint32_t *s_role) {
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t role;
        const uint32_t before = __hip_atomic_fetch_add(met, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        if (before == groups - 1u) {                        // the last to arrive gives the verdict
            role = atomicCAS(verdict, 0u, 1u) == 0u ? kTogether : kAlone;
        } else {
            uint32_t v = 0u;
            for (uint32_t it = 0; it < spin_limit; ++it) {
                v = __hip_atomic_load(verdict, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (v != 0u) break;
                __builtin_amdgcn_s_sleep(8);
            }
            if (v == 0u) {                                  // gave up; unless the verdict came in this very moment
                v = atomicCAS(verdict, 0u, 2u);
                if (v == 0u) v = 2u;
            }
            role = v == 1u ? kTogether : kLeave;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // the others' histograms, not stale cache lines (one
        *s_role = role;                                     // thread: the barrier passes it on to the workgroup)
    }
    __syncthreads();
    return (MeetRole)*s_role;
}

__global__ __launch_bounds__(kSortThreads) void select_fused_gated_kernel(const float *__restrict__ scores,
                                                                           long long N, long long ld, int k,
                                                                           SelState *st_all, const uint32_t *hist1_all,
                                                                           uint32_t *hist2_all, uint32_t *hist3_all,
                                                                           uint32_t *blockhist3_all,
                                                                           unsigned long long *cand_all,
                                                                           float *out_scores, int32_t *out_idx, int meet_ok,
                                                                           uint32_t spin_limit, Gate gate, int sorts_list) {
    extern __shared__ __attribute__((aligned(16))) uint8_t sort_lds[];
    __shared__ uint32_t lhist[kBins2];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_last, s_role;
    __shared__ uint32_t wave_sum_s[16];
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    // A gate on the flag alone: the lists of many classifiers have been judged (filter_sort_kernel).
    // sorts_list (one classifier, gate on the scan's own cursor): this launch is also the end of the
    // filtered scan; when the list serves, one workgroup sorts it and that is all.
    if (!gate_open(gate)) {                                // uniform over the grid
        if (sorts_list && blockIdx.x == 0)
            select_sort_emit(sort_lds, cand_all + (size_t)q * kCandCap, st->cursor, k, out_scores + (size_t)q * k,
                             out_idx + (size_t)q * k);
        return;
    }
    if (sorts_list && blockIdx.x == 0 && threadIdx.x == 0) st_all[0].fallback = 1u;   // (for whoever asks afterwards)
    const float *s = scores + (long long)q * ld;
    const bool vec_ok = row_vec_ok(s);
    unsigned long long *cand = cand_all + (size_t)q * kCandCap;
    uint32_t *hist2 = hist2_all + (size_t)q * kBins2, *hist3 = hist3_all + (size_t)q * kBins3;
    const BinChoice r1 = block_find_bin(hist1_all + (size_t)q * kHist1Words, kBins1, (uint32_t)k, lhist, s_out, kHistShards);
    const uint32_t b1 = r1.bin, need1 = (uint32_t)k - r1.above, c1 = r1.above + r1.inbin;
    const bool decisive1 = c1 <= (uint32_t)kCandCap;
    long long begin, end;
    sel_chunk(N, blockIdx.x, gridDim.x, &begin, &end);
    uint32_t n = c1;
    bool alone = false;                                    // this workgroup finishes over all rows by itself
    if (decisive1) {
        gather_rows(s, begin, end, vec_ok, ((long long)b1 << 20) - 1, false, 0u, 0u, 0u, k, st, cand);
    } else {
        for (int b = threadIdx.x; b < kBins2; b += blockDim.x) lhist[b] = 0u;
        __syncthreads();
        for_each_score(s, begin, end, vec_ok, [&](float v, bool ok, long long) {
            const uint32_t key = float_to_key(v);
            hist_add_wave(lhist, (key >> 8) & 0xFFFu, ok && (key >> 20) == b1);
        });
        merge_hist(lhist, kBins2, hist2);
        if (meet_ok) {
            const MeetRole role = meet(&st->met[0], &st->verdict[0], gridDim.x, spin_limit, &s_role);
            if (role == kLeave) return;                    // uniform over the workgroup
            alone = role == kAlone;
        }
    }
    if (!decisive1 && meet_ok && !alone) {
        // together: pass 2 is complete in global memory
        const BinChoice r2 = block_find_bin(hist2, kBins2, need1, lhist, s_out);
        const uint32_t p24 = (b1 << 12) | r2.bin, need2 = need1 - r2.above;
        const uint32_t c2 = ((uint32_t)k - need1) + r2.above + r2.inbin;     // keys >= p24 << 8
        if (c2 <= (uint32_t)kCandCap) {
            gather_rows(s, begin, end, vec_ok, ((long long)p24 << 8) - 1, false, 0u, 0u, 0u, k, st, cand);
            n = c2;
        } else {
            // pass 3, every workgroup its share; its own counts stay behind for the split of the ties
            __syncthreads();
            for (int b = threadIdx.x; b < kBins3; b += blockDim.x) lhist[b] = 0u;
            __syncthreads();
            for_each_score(s, begin, end, vec_ok, [&](float v, bool ok, long long) {
                const uint32_t key = float_to_key(v);
                hist_add_wave(lhist, key & 0xFFu, ok && (key >> 8) == p24);
            });
            __syncthreads();
            uint32_t *bh = blockhist3_all + ((size_t)q * kSelBlocks + blockIdx.x) * kBins3;
            for (int b = threadIdx.x; b < kBins3; b += blockDim.x) bh[b] = lhist[b];
            merge_hist(lhist, kBins3, hist3);
            const MeetRole role = meet(&st->met[1], &st->verdict[1], gridDim.x, spin_limit, &s_role);
            if (role == kLeave) return;
            const BinChoice r3 = block_find_bin(hist3, kBins3, need2, lhist, s_out);
            const uint32_t T = (p24 << 8) | r3.bin, r = need2 - r3.above;
            if (role == kAlone) {
                gather_rows(s, 0, N, vec_ok, (long long)T, true, T, r, 0u, k, st, cand);
                __threadfence();
                __syncthreads();
                select_sort_emit(sort_lds, cand, (uint32_t)k, k, out_scores + (size_t)q * k, out_idx + (size_t)q * k);
                return;
            }
            // ties of the workgroups before this one (their rows are lower): they are served first
            const uint32_t *col = blockhist3_all + (size_t)q * kSelBlocks * kBins3 + r3.bin;
            uint32_t mine = 0u, eqbase = 0u;
            for (int b = threadIdx.x; b < (int)blockIdx.x; b += blockDim.x) mine += col[(size_t)b * kBins3];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
            if ((threadIdx.x & 63) == 0) wave_sum_s[threadIdx.x >> 6] = mine;
            __syncthreads();
            for (int w = 0; w < (int)(blockDim.x >> 6); ++w) eqbase += wave_sum_s[w];
            __syncthreads();
            gather_rows(s, begin, end, vec_ok, (long long)T, eqbase < r, T, r, eqbase, k, st, cand);
            n = (uint32_t)k;
        }
    }
    // ticket: the workgroup that draws the last one continues alone (and a workgroup that already
    // is alone has no one to wait for)
    if (!alone) {
        // one thread releases what the whole workgroup wrote (the barrier orders the others' stores
        // before it): a device-wide fence by every wave of every workgroup costs ~55 us here
        __syncthreads();
        if (threadIdx.x == 0)
            s_last = __hip_atomic_fetch_add(&st->spare, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1u ? 1u : 0u;
        __syncthreads();
        if (s_last == 0u) return;                          // uniform over the workgroup
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // the others' parts of the list, not stale cache lines
    }
    if (!decisive1 && (alone || !meet_ok)) {
        // passes 2 (resolve), 3 and the gather over all rows by this workgroup
        const BinChoice r2 = block_find_bin(hist2, kBins2, need1, lhist, s_out);
        const uint32_t p24 = (b1 << 12) | r2.bin, need2 = need1 - r2.above;
        const uint32_t c2 = ((uint32_t)k - need1) + r2.above + r2.inbin;     // keys >= p24 << 8
        if (c2 <= (uint32_t)kCandCap) {
            gather_rows(s, 0, N, vec_ok, ((long long)p24 << 8) - 1, false, 0u, 0u, 0u, k, st, cand);
            n = c2;
        } else {
            for (int b = threadIdx.x; b < kBins3; b += blockDim.x) lhist[b] = 0u;
            __syncthreads();
            for_each_score(s, 0, N, vec_ok, [&](float v, bool ok, long long) {
                const uint32_t key = float_to_key(v);
                hist_add_wave(lhist, key & 0xFFu, ok && (key >> 8) == p24);
            });
            __syncthreads();
            uint32_t above = 0u, inbin = 0u, bin3 = 0u;
            if (threadIdx.x < 64) bin3 = wave_find_bin(lhist, kBins3 / 64, need2, &above, &inbin);
            if (threadIdx.x == 0) {
                s_out[0] = bin3;
                s_out[1] = above;
            }
            __syncthreads();
            const uint32_t T = (p24 << 8) | s_out[0], r = need2 - s_out[1];
            __syncthreads();
            gather_rows(s, 0, N, vec_ok, (long long)T, true, T, r, 0u, k, st, cand);
            n = (uint32_t)k;
        }
    }
    __threadfence();                                       // the list this workgroup wrote itself
    __syncthreads();
    select_sort_emit(sort_lds, cand, n > (uint32_t)kCandCap ? (uint32_t)kCandCap : n, k, out_scores + (size_t)q * k,
                     out_idx + (size_t)q * k);
}

// Ranking of ready-made scores in one read (one classifier, a million scores or more): the scheme of
// the filtered scans applied to otf_topk.  topk_sample_kernel zeroes the selection state and
// leaves the largest key each of its waves met in a strided sample of the scores (every
// kSampleStride-th group of kSampleGroup); topk_filter_kernel takes the threshold from those (see
// resolve_tau_slots) and reads the scores once, keeping the ones at or above it; pass 1 and
// select_fused_gated_kernel stand behind it as the re-scan and the selection stand behind every
// filtered scan.
__global__ __launch_bounds__(256) void topk_sample_kernel(const float *__restrict__ scores, long long Nv, SelState *st,
                                                          uint32_t *hist1, uint32_t *hist2, uint32_t *hist3,
                                                          SelState *sample_st, SampleSlot *slots) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = tid; i < (size_t)kHist1Words; i += step) hist1[i] = 0u;
    for (size_t i = tid; i < (size_t)kBins2; i += step) hist2[i] = 0u;
    for (size_t i = tid; i < (size_t)kBins3; i += step) hist3[i] = 0u;
    if (blockIdx.x == 0) {                                  // (the block that records the number of slots below)
        uint32_t *a = reinterpret_cast<uint32_t *>(st), *b = reinterpret_cast<uint32_t *>(sample_st);
        for (int i = threadIdx.x; i < (int)(sizeof(SelState) / 4); i += blockDim.x) {
            a[i] = 0u;
            b[i] = 0u;
        }
        __syncthreads();
    }
    const long long waves = (long long)gridDim.x * (blockDim.x >> 6);
    const long long wave = (long long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    uint32_t mx = 0u, cnt = 0u;
    for (long long v = wave * 64 + (threadIdx.x & 63); v < Nv; v += waves * 64) {
        const long long row = (v >> 10) * ((long long)kSampleGroup * kSampleStride) + (v & 1023);
        sample_note(mx, cnt, float_to_key(scores[row]));
    }
    sample_store(slots, sample_st, mx, cnt);
}

__global__ __launch_bounds__(512) void topk_filter_kernel(const float *__restrict__ scores, long long N, SelState *st,
                                                          const SelState *sample_st, const SampleSlot *slots,
                                                          unsigned long long *__restrict__ cand) {
    constexpr uint32_t kLocal = 1024;                       // per workgroup; ~16 are expected
    __shared__ uint32_t lds[kBins1];
    __shared__ uint32_t s_out[3];
    __shared__ unsigned long long local[kLocal];
    __shared__ uint32_t s_n, s_base;
    const TauChoice tc = resolve_tau_slots(slots, sample_st, N, lds, s_out);
    if (tc.hopeless) return;                                // uniform: the list stays empty, which opens the gate of the exact passes
    if (threadIdx.x == 0) s_n = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, gridDim.x, &begin, &end);
    for_each_score(scores, begin, end, row_vec_ok(scores), [&](float v, bool ok, long long row) {
        const uint32_t key = float_to_key(v);
        if (ok && key >= tc.tau) {
            const uint32_t lp = atomicAdd(&s_n, 1u);
            if (lp < kLocal) local[lp] = pack_cand(key, row);
        }
    });
    __syncthreads();
    const uint32_t n = s_n;
    // a workgroup with more candidates than its buffer holds means the threshold is far too low:
    // the count it reports then overflows the list on purpose, and the exact passes take over
    if (threadIdx.x == 0 && n) s_base = atomicAdd(&st->cursor, n <= kLocal ? n : (uint32_t)kCandCap + 1u);
    __syncthreads();
    if (n > kLocal) return;
    for (uint32_t i = threadIdx.x; i < n; i += blockDim.x) {
        const uint32_t pos = s_base + i;
        if (pos < (uint32_t)kCandCap) cand[pos] = local[i];
    }
}

static hipError_t allow_sort_lds() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&sort_emit_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kSortLdsBytes);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&select_fused_gated_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kSortLdsBytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&filter_sort_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kSortLdsBytes);
}

// Blocks per classifier of a selection pass: every block should have a few thousand rows, and
// a few thousand blocks in total fill the chip (at most kSelBlocks: the pass-3 tables are that long).
static int sel_blocks(int64_t N, int Q) {
    int64_t by_rows = (N + 4095) / 4096;
    int64_t by_chip = (4096 + Q - 1) / Q;
    int64_t b = by_rows < by_chip ? by_rows : by_chip;
    if (b > kSelBlocks) b = kSelBlocks;
    if (b < 1) b = 1;
    return (int)b;
}

hipError_t launch_select_init(const SelectWs &sw, int Q, hipStream_t s) {
    int blocks = (int)(((size_t)Q * kHist1Words + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    select_init_kernel<<<blocks, 256, 0, s>>>(sw.st, sw.hist1, sw.hist2, sw.hist3, nullptr, Q);
    return hipGetLastError();
}

hipError_t launch_select_init_both(const SelectWs &sw, const SelectWs &sample_sw, int Q, hipStream_t s) {
    int blocks = (int)(((size_t)Q * kHist1Words + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    select_init_kernel<<<blocks, 256, 0, s>>>(sw.st, sw.hist1, sw.hist2, sw.hist3, sample_sw.st, Q);
    return hipGetLastError();
}

hipError_t launch_hist1(const float *scores, int64_t N, int64_t ld, int Q, const SelectWs &sw, Gate gate,
                        hipStream_t s) {
    // A plain histogram, free of the per-block tables of the later passes.  Every workgroup ends by
    // adding its bins to the global histogram, and the scores crowd into a hundred-odd bins, so the
    // adds to one bin queue up (~18 ns each) when the workgroups finish together: few, large
    // workgroups (one of 1024 threads per compute unit: 35 us for 50M scores; four of 512: 42 us).
    int64_t blocks = std::min<int64_t>((N + 8191) / 8192, std::max<int64_t>(1, (int64_t)device_cu_count() / Q));
    blocks = std::max<int64_t>(blocks, sel_blocks(N, Q));
    hist1_kernel<<<dim3((unsigned)blocks, Q), 1024, 0, s>>>(scores, N, ld, sw.st, sw.hist1, gate);
    return hipGetLastError();
}

hipError_t launch_select_tail(const float *scores, int64_t N, int64_t ld, int Q, int k, const SelectWs &sw,
                              float *out_scores, int32_t *out_idx, SelectTail tail, hipStream_t s) {
    dim3 grid(sel_blocks(N, Q), Q);
    if (tail == kTailBehindScan && Q != 1) return hipErrorInvalidValue;
    if (tail != kTailPlain) {                      // behind filtered scans: one launch behind one gate
        hipError_t e = allow_sort_lds();
        if (e != hipSuccess) return e;
        // the workgroups may wait for each other only if all of them are resident at once: one per compute unit
        const int meet_ok = (int64_t)grid.x * grid.y <= device_cu_count() && sw.hist3 && sw.blockhist3 ? 1 : 0;
        select_fused_gated_kernel<<<grid, kSortThreads, kSortLdsBytes, s>>>(scores, N, ld, k, sw.st, sw.hist1, sw.hist2,
                                                                            sw.hist3, sw.blockhist3, sw.cand, out_scores,
                                                                            out_idx, meet_ok,
                                                                            (uint32_t)tune_int(OTF_DEBUG_MEET_SPIN_LIMIT, (int)kMeetSpinLimit),
                                                                            Gate{sw.st, tail == kTailBehindScan ? k : 0},
                                                                            tail == kTailBehindScan ? 1 : 0);
        return hipGetLastError();
    }
    // (1024 threads: the histogram passes hide the latency of their votes and shared-memory adds behind more waves)
    hist2_kernel<<<grid, 1024, 0, s>>>(scores, N, ld, k, sw.st, sw.hist1, sw.hist2);
    hist3_kernel<<<grid, 1024, 0, s>>>(scores, N, ld, k, sw.st, sw.hist2, sw.hist3, sw.blockhist3);
    gather_kernel<<<grid, 512, 0, s>>>(scores, N, ld, k, sw.st, sw.hist3, sw.blockhist3, sw.cand);
    hipError_t e = allow_sort_lds();
    if (e != hipSuccess) return e;
    sort_emit_kernel<<<Q, kSortThreads, kSortLdsBytes, s>>>(sw.st, sw.cand, k, out_scores, out_idx);
    return hipGetLastError();
}

// Thresholds of the filtered scans of Q classifiers from their sample scores (rank m of Nv each).
hipError_t launch_sample_threshold(const float *sample_scores, int64_t Nv, int64_t ld, int Q, int m,
                                   const SelectWs &sample_sw, SelState *main_st, hipStream_t s) {
    if (m < 1 || m > Nv || !main_st) return hipErrorInvalidValue;
    sample_threshold_kernel<<<Q, 1024, 0, s>>>(sample_scores, Nv, ld, m, sample_sw.st, main_st);
    return hipGetLastError();
}

hipError_t launch_topk_filtered(const float *scores, int64_t N, int k, const SelectWs &sw, const SelectWs &sample_sw,
                                SampleSlot *slots, float *out_scores, int32_t *out_idx, hipStream_t s) {
    const int64_t Nv = N / ((int64_t)kSampleGroup * kSampleStride) * kSampleGroup;
    const int sample_grid = (int)std::min<int64_t>(std::max<int64_t>(1, Nv / 1024), device_cu_count());
    topk_sample_kernel<<<sample_grid, 256, 0, s>>>(scores, Nv, sw.st, sw.hist1, sw.hist2, sw.hist3, sample_sw.st, slots);
    topk_filter_kernel<<<kSelBlocks, 512, 0, s>>>(scores, N, sw.st, sample_sw.st, slots, sw.cand);
    hipError_t e = launch_hist1(scores, N, N, 1, sw, Gate{sw.st, k}, s);
    if (e == hipSuccess) e = launch_select_tail(scores, N, N, 1, k, sw, out_scores, out_idx, kTailBehindScan, s);
    return e;
}

hipError_t launch_filter_sort(const SelectWs &sw, int Q, int k, float *out_scores, int32_t *out_idx, hipStream_t s) {
    hipError_t e = allow_sort_lds();
    if (e != hipSuccess) return e;
    filter_sort_kernel<<<Q, kSortThreads, kSortLdsBytes, s>>>(sw.st, sw.cand, k, out_scores, out_idx);
    return hipGetLastError();
}

}  // namespace otf
