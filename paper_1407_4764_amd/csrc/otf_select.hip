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
// A pass ends in the block that finishes last (ticket counter), which resolves the bin; the
// next pass is skipped on the device as soon as the candidates fit the list (mode 0 / 1).
//
// The same passes serve the filtered scans: passes 1 and 2 over the scores of a small sample of
// the store give a 24-bit threshold (`tau_key`); the full scan then appends only rows at or above
// it, and filter_sort_kernel sorts that list.  If the list cannot serve (fewer than k rows or
// more than it can hold) it raises `fallback`, and the kernels of the full selection, launched
// behind it with `gated` set, run; otherwise they return at once.
#include "otf_internal.h"

namespace otf {

__global__ __launch_bounds__(256) void select_init_kernel(SelState *st, uint32_t *hist1, uint32_t *hist2, int Q) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    uint32_t *stw = reinterpret_cast<uint32_t *>(st);
    for (size_t i = tid; i < (size_t)Q * (sizeof(SelState) / 4); i += step) stw[i] = 0u;
    for (size_t i = tid; i < (size_t)Q * kBins1; i += step) hist1[i] = 0u;
    for (size_t i = tid; i < (size_t)Q * kBins2; i += step) hist2[i] = 0u;
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

__global__ __launch_bounds__(512) void hist1_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                    int k, SelState *st_all, uint32_t *hist1_all, int gated) {
    __shared__ uint32_t lhist[kBins1];
    __shared__ uint32_t s_flag;
    if (gated && st_all[0].fallback == 0u) return;
    const int q = blockIdx.y;
    const float *s = scores + (long long)q * ld;
    const bool vec_ok = row_vec_ok(s);
    for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, &begin, &end);
    for (long long t0 = begin; t0 < end; t0 += 4 * blockDim.x) {
        float v[4];
        bool ok[4];
        load4(s, t0 + 4 * threadIdx.x, end, vec_ok, v, ok);
#pragma unroll
        for (int j = 0; j < 4; ++j) hist_add_wave(lhist, float_to_key(v[j]) >> 20, ok[j]);
    }
    finish_pass1(lhist, hist1_all + (size_t)q * kBins1, st_all + q, (uint32_t)k, gridDim.x, &s_flag);
}

// force_tau: always run (threshold estimation on a sample) and publish tau_key = top 24 bits of
// the `need1`-th largest key, low bits zero.
__global__ __launch_bounds__(512) void hist2_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                    int k, SelState *st_all, uint32_t *hist2_all, int gated,
                                                    int force_tau, const SelState *gate_state) {
    __shared__ uint32_t lhist[kBins2];
    __shared__ uint32_t s_flag;
    if (gated && gate_state[0].fallback == 0u) return;
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    if (!force_tau && st->mode == 0u) return;         // pass 1 was decisive (uniform per block)
    const uint32_t b1 = st->b1;
    const float *s = scores + (long long)q * ld;
    const bool vec_ok = row_vec_ok(s);
    uint32_t *ghist = hist2_all + (size_t)q * kBins2;
    for (int b = threadIdx.x; b < kBins2; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, &begin, &end);
    for (long long t0 = begin; t0 < end; t0 += 4 * blockDim.x) {
        float v[4];
        bool ok[4];
        load4(s, t0 + 4 * threadIdx.x, end, vec_ok, v, ok);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t key = float_to_key(v[j]);
            hist_add_wave(lhist, (key >> 8) & 0xFFFu, ok[j] && (key >> 20) == b1);
        }
    }
    __syncthreads();
    bool last = merge_hist_and_ticket(lhist, kBins2, ghist, &st->done2, gridDim.x, &s_flag);
    if (!last) return;
    block_load_hist(lhist, ghist, kBins2);
    if (threadIdx.x < 64) {
        const uint32_t need1 = st->need1;
        uint32_t above, inbin;
        uint32_t b2 = wave_find_bin(lhist, kBins2 / 64, need1, &above, &inbin);
        if (threadIdx.x == 0) {
            uint32_t p24 = (b1 << 12) | b2;
            st->p24 = p24;
            st->need2 = need1 - above;
            st->tau_key = p24 << 8;
            uint32_t c2 = ((uint32_t)k - need1) + above + inbin;   // keys >= p24 << 8
            if (c2 <= (uint32_t)kCandCap) {
                st->mode = 1u;
                st->ncand = c2;
                st->tex = ((long long)p24 << 8) - 1;
            } else {
                st->mode = 2u;
            }
        }
    }
}

__global__ __launch_bounds__(512) void hist3_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                    int k, SelState *st_all, uint32_t *blockhist3_all,
                                                    uint32_t *eqoff_all, int gated) {
    __shared__ uint32_t lhist[kBins3];
    __shared__ uint32_t lscan[kSelBlocks];
    __shared__ uint32_t s_flag, s_b3;
    if (gated && st_all[0].fallback == 0u) return;
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    if (st->mode != 2u) return;
    const uint32_t p24 = st->p24;
    const float *s = scores + (long long)q * ld;
    const bool vec_ok = row_vec_ok(s);
    uint32_t *bh = blockhist3_all + (size_t)q * kSelBlocks * kBins3;
    for (int b = threadIdx.x; b < kBins3; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, &begin, &end);
    for (long long t0 = begin; t0 < end; t0 += 4 * blockDim.x) {
        float v[4];
        bool ok[4];
        load4(s, t0 + 4 * threadIdx.x, end, vec_ok, v, ok);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t key = float_to_key(v[j]);
            hist_add_wave(lhist, key & 0xFFu, ok[j] && (key >> 8) == p24);
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins3; b += blockDim.x) bh[(size_t)blockIdx.x * kBins3 + b] = lhist[b];
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t t = atomicAdd(&st->done3, 1u);
        s_flag = (t == gridDim.x - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_flag) return;
    __threadfence();
    // the last block: total histogram over the blocks, then the bin of the k-th key
    if (threadIdx.x < kBins3) {
        uint32_t acc = 0;
        for (int b = 0; b < kSelBlocks; ++b) acc += ld_coherent(bh + (size_t)b * kBins3 + threadIdx.x);
        lhist[threadIdx.x] = acc;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        const uint32_t need2 = st->need2;
        uint32_t above, inbin;
        uint32_t b3 = wave_find_bin(lhist, kBins3 / 64, need2, &above, &inbin);
        if (threadIdx.x == 0) {
            uint32_t T = (p24 << 8) | b3;
            st->T = T;
            st->r = need2 - above;
            st->ncand = (uint32_t)k;
            st->tex = (long long)T;
            s_b3 = b3;
        }
    }
    __syncthreads();
    // rows equal to the k-th key are taken in ascending row order: exclusive prefix of their
    // per-block counts gives each block the rank of its first such row
    const uint32_t b3 = s_b3;
    for (int b = threadIdx.x; b < kSelBlocks; b += blockDim.x) lscan[b] = ld_coherent(bh + (size_t)b * kBins3 + b3);
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        uint32_t *eo = eqoff_all + (size_t)q * kSelBlocks;
        for (int b = 0; b < kSelBlocks; ++b) {
            eo[b] = run;
            run += lscan[b];
        }
    }
}

__device__ __forceinline__ unsigned long long pack_cand(uint32_t key, long long row) {
    return ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)row);
}

__global__ __launch_bounds__(512) void gather_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                     int k, SelState *st_all, const uint32_t *eqoff_all,
                                                     unsigned long long *cand_all, int gated) {
    __shared__ uint32_t wave_cnt[8];
    if (gated && st_all[0].fallback == 0u) return;
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    const uint32_t mode = st->mode;
    const long long tex = st->tex;
    const uint32_t T = st->T, r = st->r;
    const float *s = scores + (long long)q * ld;
    const bool vec_ok = row_vec_ok(s);
    unsigned long long *cand = cand_all + (size_t)q * kCandCap;
    long long begin, end;
    sel_chunk(N, blockIdx.x, &begin, &end);
    uint32_t eqbase = (mode == 2u) ? eqoff_all[(size_t)q * kSelBlocks + blockIdx.x] : 0u;
    const bool ordered = (mode == 2u) && (eqbase < r);    // uniform over the block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    for (long long t0 = begin; t0 < end; t0 += 4 * blockDim.x) {
        const long long i0 = t0 + 4 * threadIdx.x;
        float v[4];
        bool ok[4];
        load4(s, i0, end, vec_ok, v, ok);
        uint32_t key[4];
        uint32_t neq = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            key[j] = float_to_key(v[j]);
            if (ok[j] && (long long)key[j] > tex) {
                uint32_t pos = atomicAdd(&st->cursor, 1u);
                if (pos < (uint32_t)kCandCap) cand[pos] = pack_cand(key[j], i0 + j);
            }
            neq += (ok[j] && key[j] == T) ? 1u : 0u;
        }
        if (ordered) {
            // rank of each row equal to T in row order: threads hold 4 consecutive rows
            uint32_t incl = neq;                       // inclusive prefix over the lanes of the wave
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                uint32_t t = __shfl_up(incl, o, 64);
                if (lane >= o) incl += t;
            }
            if (lane == 63) wave_cnt[wave] = incl;
            __syncthreads();
            uint32_t before = 0, total = 0;
            for (int w = 0; w < nwaves; ++w) {
                uint32_t c = wave_cnt[w];
                if (w < wave) before += c;
                total += c;
            }
            uint32_t rank = eqbase + before + incl - neq;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (ok[j] && key[j] == T) {
                    if (rank < r) {
                        uint32_t pos = (uint32_t)k - r + rank;
                        if (pos < (uint32_t)kCandCap) cand[pos] = pack_cand(key[j], i0 + j);
                    }
                    ++rank;
                }
            }
            eqbase += total;
            __syncthreads();
        }
    }
}

// Bitonic sort (descending) of P = 2^p >= n packed candidates in shared memory `a`, then the
// first k are emitted.  All threads of the block call.
__device__ __forceinline__ void sort_and_emit(unsigned long long *a, const unsigned long long *cand, uint32_t n, int k,
                                              float *out_scores, int32_t *out_idx) {
    uint32_t P = 2;
    while (P < n) P <<= 1;
    for (uint32_t i = threadIdx.x; i < P; i += blockDim.x) a[i] = (i < n) ? cand[i] : 0ull;
    for (uint32_t size = 2; size <= P; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (uint32_t i = threadIdx.x; i < (P >> 1); i += blockDim.x) {
                uint32_t lo = 2u * i - (i & (stride - 1u));
                uint32_t hi = lo + stride;
                unsigned long long x = a[lo], y = a[hi];
                bool desc = (lo & size) == 0u;
                if (desc ? (x < y) : (x > y)) {
                    a[lo] = y;
                    a[hi] = x;
                }
            }
        }
    }
    __syncthreads();
    for (uint32_t j = threadIdx.x; j < (uint32_t)k; j += blockDim.x) {
        unsigned long long e = a[j];
        out_scores[j] = key_to_float((uint32_t)(e >> 32));
        out_idx[j] = (int32_t)(0xFFFFFFFFu - (uint32_t)(e & 0xFFFFFFFFull));
    }
}

// One block per classifier: sorts the candidate list of the full selection.
__global__ __launch_bounds__(1024) void sort_emit_kernel(const SelState *st_all, const unsigned long long *cand_all,
                                                         int k, float *out_scores, int32_t *out_idx, int gated) {
    __shared__ unsigned long long a[kCandCap];
    if (gated && st_all[0].fallback == 0u) return;
    const int q = blockIdx.x;
    uint32_t n = st_all[q].ncand;
    if (n > (uint32_t)kCandCap) n = kCandCap;
    sort_and_emit(a, cand_all + (size_t)q * kCandCap, n, k, out_scores + (size_t)q * k, out_idx + (size_t)q * k);
}

// One block per classifier: end of a filtered scan.  The scan appended `cursor` rows (it stops
// writing at the capacity but keeps counting).  With k <= cursor <= capacity the list holds
// every row of the top k, so sorting it gives the exact answer; otherwise the fallback is raised
// for all classifiers and the append cursor is cleared for the full selection that follows.
__global__ __launch_bounds__(1024) void filter_sort_kernel(SelState *st_all, const unsigned long long *cand_all, int k,
                                                           float *out_scores, int32_t *out_idx) {
    __shared__ unsigned long long a[kCandCap];
    const int q = blockIdx.x;
    SelState *st = st_all + q;
    const uint32_t n = st->cursor;
    __syncthreads();
    if (threadIdx.x == 0) st->cursor = 0u;
    if (n < (uint32_t)k || n > (uint32_t)kCandCap) {
        if (threadIdx.x == 0) atomicOr(&st_all[0].fallback, 1u);
        return;
    }
    sort_and_emit(a, cand_all + (size_t)q * kCandCap, n, k, out_scores + (size_t)q * k, out_idx + (size_t)q * k);
}

hipError_t launch_select_init(const SelectWs &sw, int Q, hipStream_t s) {
    int blocks = (int)(((size_t)Q * kBins1 + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    select_init_kernel<<<blocks, 256, 0, s>>>(sw.st, sw.hist1, sw.hist2, Q);
    return hipGetLastError();
}

hipError_t launch_hist1(const float *scores, int64_t N, int64_t ld, int Q, int k, const SelectWs &sw, int gated,
                        hipStream_t s) {
    hist1_kernel<<<dim3(kSelBlocks, Q), 512, 0, s>>>(scores, N, ld, k, sw.st, sw.hist1, gated);
    return hipGetLastError();
}

hipError_t launch_select_tail(const float *scores, int64_t N, int64_t ld, int Q, int k, const SelectWs &sw,
                              float *out_scores, int32_t *out_idx, int gated, hipStream_t s) {
    dim3 grid(kSelBlocks, Q);
    hist2_kernel<<<grid, 512, 0, s>>>(scores, N, ld, k, sw.st, sw.hist2, gated, 0, sw.st);
    hist3_kernel<<<grid, 512, 0, s>>>(scores, N, ld, k, sw.st, sw.blockhist3, sw.eqoff, gated);
    gather_kernel<<<grid, 512, 0, s>>>(scores, N, ld, k, sw.st, sw.eqoff, sw.cand, gated);
    sort_emit_kernel<<<Q, 1024, 0, s>>>(sw.st, sw.cand, k, out_scores, out_idx, gated);
    return hipGetLastError();
}

// Threshold from a sample: pass 2 over the sample scores (pass 1 was fused into the sample scan
// or done by launch_hist1 on the sample state), publishing tau_key in the sample state.
hipError_t launch_sample_threshold(const float *sample_scores, int64_t Nv, int64_t ld, int Q, int m,
                                   const SelectWs &sample_sw, hipStream_t s) {
    hist2_kernel<<<dim3(kSelBlocks, Q), 512, 0, s>>>(sample_scores, Nv, ld, m, sample_sw.st, sample_sw.hist2, 0, 1,
                                                    sample_sw.st);
    return hipGetLastError();
}

hipError_t launch_filter_sort(const SelectWs &sw, int Q, int k, float *out_scores, int32_t *out_idx, hipStream_t s) {
    filter_sort_kernel<<<Q, 1024, 0, s>>>(sw.st, sw.cand, k, out_scores, out_idx);
    return hipGetLastError();
}

}  // namespace otf
