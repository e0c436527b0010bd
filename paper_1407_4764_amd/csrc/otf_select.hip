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

__global__ __launch_bounds__(512) void hist1_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                    int k, SelState *st_all, uint32_t *hist1_all) {
    __shared__ uint32_t lhist[kBins1];
    __shared__ uint32_t s_flag;
    const int q = blockIdx.y;
    const float *s = scores + (long long)q * ld;
    for (int b = threadIdx.x; b < kBins1; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, &begin, &end);
    for (long long i = begin + threadIdx.x; i < end; i += blockDim.x)
        atomicAdd(&lhist[float_to_key(s[i]) >> 20], 1u);
    finish_pass1(lhist, hist1_all + (size_t)q * kBins1, st_all + q, (uint32_t)k, gridDim.x, &s_flag);
}

__global__ __launch_bounds__(512) void hist2_kernel(const float *__restrict__ scores, long long N, long long ld,
                                                    int k, SelState *st_all, uint32_t *hist2_all) {
    __shared__ uint32_t lhist[kBins2];
    __shared__ uint32_t s_flag;
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    if (st->mode == 0u) return;                       // pass 1 was decisive (uniform per block)
    const uint32_t b1 = st->b1;
    const float *s = scores + (long long)q * ld;
    uint32_t *ghist = hist2_all + (size_t)q * kBins2;
    for (int b = threadIdx.x; b < kBins2; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, &begin, &end);
    for (long long i = begin + threadIdx.x; i < end; i += blockDim.x) {
        uint32_t key = float_to_key(s[i]);
        if ((key >> 20) == b1) atomicAdd(&lhist[(key >> 8) & 0xFFFu], 1u);
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
                                                    uint32_t *eqoff_all) {
    __shared__ uint32_t lhist[kBins3];
    __shared__ uint32_t lscan[kSelBlocks];
    __shared__ uint32_t s_flag, s_b3;
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    if (st->mode != 2u) return;
    const uint32_t p24 = st->p24;
    const float *s = scores + (long long)q * ld;
    uint32_t *bh = blockhist3_all + (size_t)q * kSelBlocks * kBins3;
    for (int b = threadIdx.x; b < kBins3; b += blockDim.x) lhist[b] = 0u;
    __syncthreads();
    long long begin, end;
    sel_chunk(N, blockIdx.x, &begin, &end);
    for (long long i = begin + threadIdx.x; i < end; i += blockDim.x) {
        uint32_t key = float_to_key(s[i]);
        if ((key >> 8) == p24) atomicAdd(&lhist[key & 0xFFu], 1u);
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
                                                     unsigned long long *cand_all) {
    __shared__ uint32_t wave_cnt[8];
    const int q = blockIdx.y;
    SelState *st = st_all + q;
    const uint32_t mode = st->mode;
    const long long tex = st->tex;
    const uint32_t T = st->T, r = st->r;
    const float *s = scores + (long long)q * ld;
    unsigned long long *cand = cand_all + (size_t)q * kCandCap;
    long long begin, end;
    sel_chunk(N, blockIdx.x, &begin, &end);
    uint32_t eqbase = (mode == 2u) ? eqoff_all[(size_t)q * kSelBlocks + blockIdx.x] : 0u;
    const bool ordered = (mode == 2u) && (eqbase < r);    // uniform over the block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    for (long long t0 = begin; t0 < end; t0 += blockDim.x) {
        const long long i = t0 + threadIdx.x;
        const bool valid = i < end;
        const uint32_t key = valid ? float_to_key(s[i]) : 0u;
        if (valid && (long long)key > tex) {
            uint32_t pos = atomicAdd(&st->cursor, 1u);
            if (pos < (uint32_t)kCandCap) cand[pos] = pack_cand(key, i);
        }
        if (ordered) {
            const bool eq = valid && key == T;
            const unsigned long long m = __ballot(eq);
            if (lane == 0) wave_cnt[wave] = (uint32_t)__popcll(m);
            __syncthreads();
            uint32_t before = 0, total = 0;
            for (int w = 0; w < nwaves; ++w) {
                uint32_t c = wave_cnt[w];
                if (w < wave) before += c;
                total += c;
            }
            if (eq) {
                uint32_t rank = eqbase + before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
                if (rank < r) {
                    uint32_t pos = (uint32_t)k - r + rank;
                    if (pos < (uint32_t)kCandCap) cand[pos] = pack_cand(key, i);
                }
            }
            eqbase += total;
            __syncthreads();
        }
    }
}

// One block per classifier: bitonic sort (descending) of the candidate list in shared memory.
__global__ __launch_bounds__(1024) void sort_emit_kernel(const SelState *st_all, const unsigned long long *cand_all,
                                                         int k, float *out_scores, int32_t *out_idx) {
    __shared__ unsigned long long a[kCandCap];
    const int q = blockIdx.x;
    const SelState *st = st_all + q;
    uint32_t n = st->ncand;
    if (n > (uint32_t)kCandCap) n = kCandCap;
    uint32_t P = 2;
    while (P < n) P <<= 1;
    const unsigned long long *cand = cand_all + (size_t)q * kCandCap;
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
        out_scores[(size_t)q * k + j] = key_to_float((uint32_t)(e >> 32));
        out_idx[(size_t)q * k + j] = (int32_t)(0xFFFFFFFFu - (uint32_t)(e & 0xFFFFFFFFull));
    }
}

hipError_t launch_select_init(const SelectWs &sw, int Q, hipStream_t s) {
    int blocks = (int)(((size_t)Q * kBins1 + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    select_init_kernel<<<blocks, 256, 0, s>>>(sw.st, sw.hist1, sw.hist2, Q);
    return hipGetLastError();
}

hipError_t launch_hist1(const float *scores, int64_t N, int64_t ld, int Q, int k, const SelectWs &sw, hipStream_t s) {
    hist1_kernel<<<dim3(kSelBlocks, Q), 512, 0, s>>>(scores, N, ld, k, sw.st, sw.hist1);
    return hipGetLastError();
}

hipError_t launch_select_tail(const float *scores, int64_t N, int64_t ld, int Q, int k, const SelectWs &sw,
                              float *out_scores, int32_t *out_idx, hipStream_t s) {
    dim3 grid(kSelBlocks, Q);
    hist2_kernel<<<grid, 512, 0, s>>>(scores, N, ld, k, sw.st, sw.hist2);
    hist3_kernel<<<grid, 512, 0, s>>>(scores, N, ld, k, sw.st, sw.blockhist3, sw.eqoff);
    gather_kernel<<<grid, 512, 0, s>>>(scores, N, ld, k, sw.st, sw.eqoff, sw.cand);
    sort_emit_kernel<<<Q, 1024, 0, s>>>(sw.st, sw.cand, k, out_scores, out_idx);
    return hipGetLastError();
}

}  // namespace otf
