// C ABI of libotf: argument validation, workspace layout and the launch sequences.
// All validation happens on the host before the first HIP call, so a rejected call has
// enqueued nothing and written nothing.
#include "otf.h"

#include <algorithm>
#include <atomic>
#include <vector>

#include "otf_internal.h"

namespace otf {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static int64_t padded_rows(int64_t N) { return (N + 63) / 64 * 64; }

WsLayout ws_layout(int64_t N, int32_t Q) {
    WsLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    L.st = take((size_t)Q * sizeof(SelState));
    L.hist1 = take((size_t)Q * kHist1Words * 4);
    L.hist2 = take((size_t)Q * kBins2 * 4);
    L.hist3 = take((size_t)Q * kBins3 * 4);
    L.blockhist3 = take((size_t)Q * kSelBlocks * kBins3 * 4);
    L.eqoff = take((size_t)Q * kSelBlocks * 4);
    L.cand = take((size_t)Q * kCandCap * 8);
    L.sample_st = take((size_t)Q * sizeof(SelState));
    L.sample_ld = padded_rows(sample_rows(N) + kSampleGroup);
    // (the single-classifier scans keep one 8-byte slot per wave of the sample scan here instead: at most 4096)
    L.sample_scores = take(std::max<size_t>((size_t)Q * (size_t)L.sample_ld * 4, (size_t)kMaxSampleSlots * sizeof(SampleSlot)));
    L.lut_image = take(kLutImageBytes);
    L.short_store = take(kShortStoreBytes);
    L.scores = take((size_t)Q * (size_t)padded_rows(N) * 4);
    L.total = off;
    return L;
}

SelectWs select_ws(void *ws, const WsLayout &L) {
    uint8_t *p = reinterpret_cast<uint8_t *>(ws);
    SelectWs sw;
    sw.st = reinterpret_cast<SelState *>(p + L.st);
    sw.hist1 = reinterpret_cast<uint32_t *>(p + L.hist1);
    sw.hist2 = reinterpret_cast<uint32_t *>(p + L.hist2);
    sw.hist3 = reinterpret_cast<uint32_t *>(p + L.hist3);
    sw.blockhist3 = reinterpret_cast<uint32_t *>(p + L.blockhist3);
    sw.eqoff = reinterpret_cast<uint32_t *>(p + L.eqoff);
    sw.cand = reinterpret_cast<unsigned long long *>(p + L.cand);
    return sw;
}

// The sample side of a filtered ranking keeps states only (work counters, slot counts, thresholds).
SelectWs sample_select_ws(void *ws, const WsLayout &L) {
    uint8_t *p = reinterpret_cast<uint8_t *>(ws);
    SelectWs sw;
    sw.st = reinterpret_cast<SelState *>(p + L.sample_st);
    sw.hist1 = nullptr;
    sw.hist2 = nullptr;
    sw.hist3 = nullptr;
    sw.blockhist3 = nullptr;
    sw.eqoff = nullptr;
    sw.cand = nullptr;
    return sw;
}

// Filtered scan or full selection?  The filtered scan needs a sample large enough to place the
// threshold (>= 8 groups) and a list that holds ~4x the requested rows.
static bool filter_eligible(int64_t N, int32_t k, const float *all_scores) {
    if (all_scores || k > kFilterMaxK) return false;
    if (sample_rows(N) < 8 * kSampleGroup) return false;
    return tune_int(OTF_DEBUG_RANK_PATH, 0) != 1;      // 1 forces the full selection (testing, comparison)
}

// Rank of the sample key that becomes the threshold: the sample holds Nv of N rows, so the m-th
// largest sample key leaves about m * N / Nv = kFilterExpect rows of the store at or above it.
static int sample_rank(int64_t N, int64_t Nv) {
    int64_t m = ((int64_t)kFilterExpect * Nv + N / 2) / N;
    return (int)(m < 32 ? 32 : m);
}

int device_cu_count() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int v = cached[dev].load(std::memory_order_relaxed);
    if (v > 0) return v;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    cached[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

// Diagnostic switches (otf_debug_set): 0 = not set, the built-in choice applies.
static std::atomic<int> g_debug[OTF_DEBUG_KEYS];

int tune_int(int key, int fallback) {
    const int v = g_debug[key].load(std::memory_order_relaxed);
    return v > 0 ? v : fallback;
}

// Which values a switch accepts (besides 0, which clears it).
static bool debug_value_ok(int key, int v) {
    switch (key) {
        case OTF_DEBUG_RANK_PATH:
        case OTF_DEBUG_BINARIZE_FP32:
        case OTF_DEBUG_PQENC_FP32: return v == 1;
        case OTF_DEBUG_SCAN_THREADS: return v >= 64 && v <= 1024 && v % 64 == 0;   // whole waves, the kernels' launch bound
        case OTF_DEBUG_SCAN_UNROLL:
        case OTF_DEBUG_BINARIZE_WAVES: return v == 4 || v == 8;
        case OTF_DEBUG_WALK_TILES: return v == 2 || v == 4 || v == 8;
        case OTF_DEBUG_SGD_PASS_PATH: return v == 1;
        case OTF_DEBUG_SGD_SPIN_LIMIT:
        case OTF_DEBUG_MEET_SPIN_LIMIT: return v >= 1 && v <= (1 << 30);
        case OTF_DEBUG_PQENC_RANGE: return v >= 4 && v <= 64 && v % 4 == 0;
        case OTF_DEBUG_DENSE_BLOCKS_PER_CU:
        case OTF_DEBUG_NARROW_BLOCKS_PER_CU:
        case OTF_DEBUG_MFMA_BLOCKS_PER_CU:
        case OTF_DEBUG_PQENC_BLOCKS_PER_CU: return v >= 1 && v <= 8;
        default: return false;
    }
}

// No store spans more bytes than this: offsets into one stay far inside 64 bits.
constexpr int64_t kMaxStoreBytes = (int64_t)1 << 48;

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int hip_status(hipError_t e) {
    if (e == hipSuccess) return OTF_OK;
    (void)hipGetLastError();   // clear the sticky error so that it is not reported twice
    return OTF_ERR_HIP;
}

// Checks shared by all ranking calls.  Returns OTF_OK or the status to hand back.
static int check_rank_common(int64_t N, int32_t k, int32_t Q, const float *out_scores, const int32_t *out_idx,
                             const void *ws, size_t ws_bytes, WsLayout *L) {
    if (N < 1 || Q < 1 || k < 1 || !out_scores || !out_idx) return OTF_ERR_INVALID_ARG;
    if (N >= ((int64_t)1 << 31)) return OTF_ERR_UNSUPPORTED;
    if (k > N) return OTF_ERR_INVALID_ARG;
    if (k > OTF_MAX_K || Q > 65535) return OTF_ERR_UNSUPPORTED;     // limits of this build, not of the operation
    *L = ws_layout(N, Q);
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || ws_bytes < L->total) return OTF_ERR_WORKSPACE;
    return OTF_OK;
}

// Optional event pairs around the scoring kernels (see otf_profile_begin in otf.h).
struct ProfileState {
    std::vector<hipEvent_t> start, stop;
    int used = 0;
    bool on = false;
};
static ProfileState g_prof;

struct ScanTimer {
    int slot = -1;
    hipStream_t s;
    explicit ScanTimer(hipStream_t stream) : s(stream) {
        if (g_prof.on && g_prof.used < (int)g_prof.start.size()) {
            slot = g_prof.used++;
            (void)hipEventRecord(g_prof.start[slot], s);
        }
    }
    void stop() {
        if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], s);
    }
};

// Scratch of the no-allocation entry point: one array per GPU, living in the code object's own
// device memory from the moment the library is loaded on that GPU until the process ends.  In
// host code the array's name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[OTF_NOALLOC_SCRATCH_BYTES];
static std::atomic<void *> g_scratch_ptr[64];   // per device: where that GPU's copy of the array lives

// Address of the current device's scratch array (resolved once per device, then remembered).
static int scratch_of_current_device(void **out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hip_status(hipErrorInvalidDevice);
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_status(e == hipSuccess ? hipErrorInvalidSymbol : e);
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return OTF_OK;
}

}  // namespace otf

using namespace otf;

extern "C" {

const char *otf_status_string(int status) {
    switch (status) {
        case OTF_OK: return "OTF_OK";
        case OTF_ERR_INVALID_ARG: return "OTF_ERR_INVALID_ARG";
        case OTF_ERR_UNSUPPORTED: return "OTF_ERR_UNSUPPORTED";
        case OTF_ERR_WORKSPACE: return "OTF_ERR_WORKSPACE";
        case OTF_ERR_HIP: return "OTF_ERR_HIP";
        case OTF_ERR_SCRATCH: return "OTF_ERR_SCRATCH";
        default: return "OTF_ERR_UNKNOWN";
    }
}

size_t otf_workspace_bytes(int64_t N, int32_t k, int32_t Q) {
    if (N < 1 || k < 1 || Q < 1 || Q > 65535 || N >= ((int64_t)1 << 31)) return 0;
    return ws_layout(N, Q).total;
}

int otf_topk(const float *scores, int64_t N, int64_t ld, int32_t Q, int32_t k, float *out_scores, int32_t *out_idx,
             void *ws, size_t ws_bytes, void *stream) {
    WsLayout L;
    if (!scores) return OTF_ERR_INVALID_ARG;
    int rc = check_rank_common(N, k, Q, out_scores, out_idx, ws, ws_bytes, &L);
    if (rc != OTF_OK) return rc;
    if (ld < N || ld > kMaxStoreBytes / 4 / Q) return OTF_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    SelectWs sw = select_ws(ws, L);
    if (Q == 1 && filter_eligible(N, k, nullptr))
        return hip_status(launch_topk_filtered(
            scores, N, k, sw, sample_select_ws(ws, L),
            reinterpret_cast<SampleSlot *>(reinterpret_cast<uint8_t *>(ws) + L.sample_scores), out_scores, out_idx, s));
    hipError_t e = launch_select_init(sw, Q, s);
    if (e == hipSuccess) e = launch_hist1(scores, N, ld, Q, sw, kNoGate, s);
    if (e == hipSuccess) e = launch_select_tail(scores, N, ld, Q, k, sw, out_scores, out_idx, kTailPlain, s);
    return hip_status(e);
}

// The argument checks of otf_rank_dense (host only: nothing is dereferenced or enqueued).
static int otf_rank_dense_check(const void *X, otf_dtype xdt, int64_t N, int32_t D, int64_t ldx, const void *W,
                                otf_dtype wdt, int32_t Q, int32_t k, const float *out_scores, const int32_t *out_idx,
                                const void *ws, size_t ws_bytes) {
    WsLayout L;
    if (!X || !W || D < 1) return OTF_ERR_INVALID_ARG;
    if ((xdt != OTF_F32 && xdt != OTF_F16) || (wdt != OTF_F32 && wdt != OTF_F16)) return OTF_ERR_INVALID_ARG;
    int rc = check_rank_common(N, k, Q, out_scores, out_idx, ws, ws_bytes, &L);
    if (rc != OTF_OK) return rc;
    if (ldx < D || ldx > kMaxStoreBytes / 4 / N) return OTF_ERR_INVALID_ARG;   // rows that overlap; a store beyond any address
    const int xsize = xdt == OTF_F16 ? 2 : 4;
    if (!aligned16(X) || ((size_t)ldx * xsize) % 16 != 0) return OTF_ERR_INVALID_ARG;
    if (xdt == OTF_F32 && wdt != OTF_F32) return OTF_ERR_UNSUPPORTED;
    if (D % (16 / xsize) != 0 || D > kDenseMaxD) return OTF_ERR_UNSUPPORTED;
    return OTF_OK;
}

int otf_rank_dense(const void *X, otf_dtype xdt, int64_t N, int32_t D, int64_t ldx, const void *W, otf_dtype wdt,
                   int32_t Q, const float *bias, int32_t k, float *out_scores, int32_t *out_idx, float *all_scores,
                   void *ws, size_t ws_bytes, void *stream) {
    const int rc = otf_rank_dense_check(X, xdt, N, D, ldx, W, wdt, Q, k, out_scores, out_idx, ws, ws_bytes);
    if (rc != OTF_OK) return rc;
    const WsLayout L = ws_layout(N, Q);

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    SelectWs sw = select_ws(ws, L);
    float *S = all_scores ? all_scores : reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + L.scores);
    const int64_t ldS = all_scores ? N : (int64_t)((N + 63) / 64 * 64);
    const int x_half = xdt == OTF_F16, w_half = wdt == OTF_F16;
    const size_t wsize = w_half ? 2 : 4;

    // (the matrix-core kernel addresses the 128 rows of a tile with 32-bit byte offsets from the tile's
    //  base: a row stride that overflows them goes to the per-classifier scan instead)
    const bool mfma = Q > 1 && x_half && w_half && Q % 32 == 0 && D % 128 == 0 && aligned16(W) &&
                      (uint64_t)ldx * 2u * 127u + 256u < ((uint64_t)1 << 32);
    const uint8_t *Wb = reinterpret_cast<const uint8_t *>(W);

    if (Q == 1 && dense_scan_filters(x_half, D) && filter_eligible(N, k, all_scores)) {
        // Short rows, one classifier: sample -> threshold -> filtered scan -> sort, with the full
        // selection behind a gate, as for the table scans.
        SelectWs ssw = sample_select_ws(ws, L);
        SampleSlot *slots = reinterpret_cast<SampleSlot *>(reinterpret_cast<uint8_t *>(ws) + L.sample_scores);
        const int64_t Nv = sample_rows(N);
        hipError_t e = launch_select_init_both(sw, ssw, 1, s);
        if (e == hipSuccess)
            e = launch_dense_scan_emit(X, x_half, Nv, D, ldx, W, w_half, bias, 0, kEmitSample, nullptr, nullptr,
                                       &ssw.st[0].chunk_ctr[0], ssw.st, nullptr, slots, nullptr, kNoGate, s);
        ScanTimer timer(s);
        if (e == hipSuccess)
            e = launch_dense_scan_emit(X, x_half, N, D, ldx, W, w_half, bias, 0, kEmitFilter, nullptr, nullptr,
                                       &sw.st[0].chunk_ctr[0], sw.st, ssw.st, slots, sw.cand, kNoGate, s);
        timer.stop();
        if (e == hipSuccess)
            e = launch_dense_scan_emit(X, x_half, N, D, ldx, W, w_half, bias, 0, kEmitScores, S, sw.hist1,
                                       &sw.st[0].chunk_ctr[1], sw.st, nullptr, nullptr, nullptr, Gate{sw.st, k}, s);
        if (e == hipSuccess) e = launch_select_tail(S, N, ldS, 1, k, sw, out_scores, out_idx, kTailBehindScan, s);
        return hip_status(e);
    }
    // (the filtered multi-classifier route also needs the states that threshold the sample: same launch)
    const bool mfma_filtered = mfma && filter_eligible(N, k, all_scores);
    hipError_t e = mfma_filtered ? launch_select_init_both(sw, sample_select_ws(ws, L), Q, s) : launch_select_init(sw, Q, s);

    // One matrix-core launch per group of 64 (or a last 32) classifiers.
    // (ctr_states[q0].chunk_ctr[ctr_word]: the zeroed work counter of each launch)
    auto mfma_scan = [&](int64_t rows, ScanEmit emit, float *dst, int64_t ld, const SelState *tau, SelState *st,
                         unsigned long long *cand, Gate gate, SelState *ctr_states, int ctr_word) {
        hipError_t err = hipSuccess;
        for (int q0 = 0; q0 < Q && err == hipSuccess;) {
            const int qn = (Q - q0 >= 64) ? 64 : 32;
            err = launch_dense_mfma(X, rows, D, ldx, Wb + (size_t)q0 * D * wsize, qn, bias ? bias + q0 : nullptr, emit,
                                    dst ? dst + (size_t)q0 * ld : nullptr, ld, tau ? tau + q0 : nullptr,
                                    st ? st + q0 : nullptr, cand ? cand + (size_t)q0 * kCandCap : nullptr, gate,
                                    &ctr_states[q0].chunk_ctr[ctr_word], s);
            q0 += qn;
        }
        return err;
    };

    if (mfma_filtered) {
        // sample -> per-classifier thresholds -> filtered scan -> sort; full selection behind a gate
        SelectWs ssw = sample_select_ws(ws, L);
        float *sample = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + L.sample_scores);
        const int64_t Nv = sample_rows(N);
        const int m = sample_rank(N, Nv);
        if (e == hipSuccess) e = mfma_scan(Nv, kEmitSample, sample, L.sample_ld, nullptr, nullptr, nullptr, kNoGate, ssw.st, 0);
        if (e == hipSuccess) e = launch_sample_threshold(sample, Nv, L.sample_ld, Q, m, ssw, sw.st, s);
        ScanTimer timer(s);
        if (e == hipSuccess) e = mfma_scan(N, kEmitFilter, nullptr, 0, ssw.st, sw.st, sw.cand, Gate{sw.st, 0}, sw.st, 0);
        timer.stop();
        if (e == hipSuccess) e = launch_filter_sort(sw, Q, k, out_scores, out_idx, s);
        if (e == hipSuccess) e = mfma_scan(N, kEmitScores, S, ldS, nullptr, nullptr, nullptr, Gate{sw.st, 0}, sw.st, 1);
        if (e == hipSuccess) e = launch_hist1(S, N, ldS, Q, sw, Gate{sw.st, 0}, s);
        if (e == hipSuccess) e = launch_select_tail(S, N, ldS, Q, k, sw, out_scores, out_idx, kTailBehindFlag, s);
        return hip_status(e);
    }
    ScanTimer timer(s);
    if (e == hipSuccess && mfma) {
        e = mfma_scan(N, kEmitScores, S, ldS, nullptr, nullptr, nullptr, kNoGate, sw.st, 1);
        timer.stop();
        if (e == hipSuccess) e = launch_hist1(S, N, ldS, Q, sw, kNoGate, s);
    } else if (e == hipSuccess) {
        for (int q = 0; q < Q && e == hipSuccess; ++q)
            e = launch_dense_scan(X, x_half, N, D, ldx, Wb + (size_t)q * D * wsize, w_half, bias, q,
                                  S + (size_t)q * ldS, sw.hist1 + (size_t)q * kHist1Words, &sw.st[q].chunk_ctr[1], s);
        timer.stop();
    }
    if (e == hipSuccess) e = launch_select_tail(S, N, ldS, Q, k, sw, out_scores, out_idx, kTailPlain, s);
    return hip_status(e);
}

int otf_rank_dense_noalloc(const void *X, otf_dtype xdt, int64_t N, int32_t D, int64_t ldx, const void *W,
                           otf_dtype wdt, int32_t Q, const float *bias, int32_t k, float *out_scores, int32_t *out_idx,
                           float *all_scores, void *stream) {
    // argument errors are reported as otf_rank_dense reports them (the stand-in workspace is never
    // dereferenced); then the size against what the static array holds
    void *ws = reinterpret_cast<void *>(256);
    const int rc = otf_rank_dense_check(X, xdt, N, D, ldx, W, wdt, Q, k, out_scores, out_idx, ws, ~(size_t)0);
    if (rc != OTF_OK) return rc;
    if (ws_layout(N, Q).total > (size_t)OTF_NOALLOC_SCRATCH_BYTES) return OTF_ERR_SCRATCH;
    const int rs = scratch_of_current_device(&ws);
    if (rs != OTF_OK) return rs;
    return otf_rank_dense(X, xdt, N, D, ldx, W, wdt, Q, bias, k, out_scores, out_idx, all_scores, ws,
                          OTF_NOALLOC_SCRATCH_BYTES, stream);
}

int otf_pq_build_lut(const float *codebooks, int32_t M, int32_t K, int32_t dsub, const float *w, float *lut,
                     void *stream) {
    if (!codebooks || !w || !lut || M < 1 || K < 1 || dsub < 1) return OTF_ERR_INVALID_ARG;
    if ((int64_t)M * K * dsub >= ((int64_t)1 << 40)) return OTF_ERR_UNSUPPORTED;
    return hip_status(launch_pq_build_lut(codebooks, M, K, dsub, w, lut, reinterpret_cast<hipStream_t>(stream)));
}

// Stored bytes per row the table scans take: whole 16-byte chunks, at most 8 table images.
static bool table_row_bytes_ok(int32_t rb) { return rb >= 16 && rb % 16 == 0 && rb <= 1024; }

// Shared tail of otf_rank_pq / otf_rank_binary once the table image is in place.
static hipError_t rank_table(const uint8_t *codes, int64_t N, int row_bytes, TableKind kind, const float *image,
                             float bias, int32_t k, float *out_scores, int32_t *out_idx, float *all_scores, void *ws,
                             const WsLayout &L, hipStream_t s) {
    SelectWs sw = select_ws(ws, L);
    uint8_t *wsb = reinterpret_cast<uint8_t *>(ws);
    float *S = all_scores ? all_scores : reinterpret_cast<float *>(wsb + L.scores);
    hipError_t e = hipSuccess;
    if (kind == kTableBytes && row_bytes > 128 && N < kShortStoreRows) {
        // the scan of rows longer than one table image reads whole tiles of 64 rows: a shorter store
        // is copied into a buffer of that many rows (the rows behind it are looked up, never emitted)
        e = hipMemcpyAsync(wsb + L.short_store, codes, (size_t)N * row_bytes, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return e;
        codes = wsb + L.short_store;
    }
    if (filter_eligible(N, k, all_scores)) {
        SelectWs ssw = sample_select_ws(ws, L);
        SampleSlot *slots = reinterpret_cast<SampleSlot *>(wsb + L.sample_scores);
        e = launch_table_scan(codes, sample_rows(N), row_bytes, kind, image, bias, kEmitSample, nullptr, ssw.st, nullptr,
                              nullptr, slots, nullptr, kNoGate, s);
        ScanTimer timer(s);
        if (e == hipSuccess)
            e = launch_table_scan(codes, N, row_bytes, kind, image, bias, kEmitFilter, nullptr, sw.st, nullptr, ssw.st,
                                  slots, sw.cand, kNoGate, s);
        timer.stop();
        if (e == hipSuccess)
            e = launch_table_scan(codes, N, row_bytes, kind, image, bias, kEmitScores, S, sw.st, sw.hist1, nullptr,
                                  nullptr, nullptr, Gate{sw.st, k}, s);
        if (e == hipSuccess) e = launch_select_tail(S, N, N, 1, k, sw, out_scores, out_idx, kTailBehindScan, s);
        return e;
    }
    ScanTimer timer(s);
    e = launch_table_scan(codes, N, row_bytes, kind, image, bias, kEmitScores, S, sw.st, sw.hist1, nullptr, nullptr,
                          nullptr, kNoGate, s);
    timer.stop();
    if (e == hipSuccess) e = launch_select_tail(S, N, N, 1, k, sw, out_scores, out_idx, kTailPlain, s);
    return e;
}

int otf_rank_pq(const uint8_t *codes, int64_t N, int32_t M, int32_t K, const float *lut, float bias, int32_t k,
                float *out_scores, int32_t *out_idx, float *all_scores, void *ws, size_t ws_bytes, void *stream) {
    WsLayout L;
    if (!codes || !lut || M < 1 || K < 1) return OTF_ERR_INVALID_ARG;
    int rc = check_rank_common(N, k, 1, out_scores, out_idx, ws, ws_bytes, &L);
    if (rc != OTF_OK) return rc;
    if (K != 256 || !table_row_bytes_ok(M)) return OTF_ERR_UNSUPPORTED;
    if (!aligned16(codes)) return OTF_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    float *image = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + L.lut_image);
    hipError_t e = launch_pq_prepare(lut, M, image, select_ws(ws, L), sample_select_ws(ws, L), s);
    if (e == hipSuccess) e = rank_table(codes, N, M, kTableBytes, image, bias, k, out_scores, out_idx, all_scores, ws, L, s);
    return hip_status(e);
}

int otf_rank_pq_model(const uint8_t *codes, int64_t N, int32_t M, int32_t K, int32_t dsub, const float *codebooks,
                      const float *w, float bias, int32_t k, float *out_scores, int32_t *out_idx, float *all_scores,
                      void *ws, size_t ws_bytes, void *stream) {
    WsLayout L;
    if (!codes || !codebooks || !w || M < 1 || K < 1 || dsub < 1) return OTF_ERR_INVALID_ARG;
    int rc = check_rank_common(N, k, 1, out_scores, out_idx, ws, ws_bytes, &L);
    if (rc != OTF_OK) return rc;
    if (K != 256 || !table_row_bytes_ok(M) || dsub > 4096) return OTF_ERR_UNSUPPORTED;
    if (!aligned16(codes)) return OTF_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    float *image = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + L.lut_image);
    hipError_t e = launch_pq_prepare_model(codebooks, w, M, dsub, image, select_ws(ws, L), sample_select_ws(ws, L), s);
    if (e == hipSuccess) e = rank_table(codes, N, M, kTableBytes, image, bias, k, out_scores, out_idx, all_scores, ws, L, s);
    return hip_status(e);
}

int otf_rank_binary(const uint32_t *bits, int64_t N, int32_t D, const float *w, float bias, int32_t k,
                    float *out_scores, int32_t *out_idx, float *all_scores, void *ws, size_t ws_bytes, void *stream) {
    WsLayout L;
    if (!bits || !w || D < 1) return OTF_ERR_INVALID_ARG;
    int rc = check_rank_common(N, k, 1, out_scores, out_idx, ws, ws_bytes, &L);
    if (rc != OTF_OK) return rc;
    if (D % 128 != 0 || !table_row_bytes_ok(D / 8)) return OTF_ERR_UNSUPPORTED;
    if (!aligned16(bits)) return OTF_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    float *image = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + L.lut_image);
    hipError_t e = launch_binary_prepare(w, D, image, select_ws(ws, L), sample_select_ws(ws, L), s);
    if (e == hipSuccess)
        e = rank_table(reinterpret_cast<const uint8_t *>(bits), N, D / 8, D == 2048 ? kTableSeven : kTableBytes, image,
                       bias, k, out_scores, out_idx, all_scores, ws, L, s);
    return hip_status(e);
}

int otf_rank_hamming(const uint32_t *bits, int64_t N, int32_t D, const uint32_t *query, int32_t k, float *out_scores,
                     int32_t *out_idx, float *all_scores, void *ws, size_t ws_bytes, void *stream) {
    WsLayout L;
    if (!bits || !query || D < 1) return OTF_ERR_INVALID_ARG;
    int rc = check_rank_common(N, k, 1, out_scores, out_idx, ws, ws_bytes, &L);
    if (rc != OTF_OK) return rc;
    if (D % 128 != 0 || !table_row_bytes_ok(D / 8)) return OTF_ERR_UNSUPPORTED;
    if (!aligned16(bits) || !aligned16(query)) return OTF_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipError_t e = launch_select_init_both(select_ws(ws, L), sample_select_ws(ws, L), 1, s);
    if (e == hipSuccess)
        e = rank_table(reinterpret_cast<const uint8_t *>(bits), N, D / 8, kTableHamming,
                       reinterpret_cast<const float *>(query), 0.f, k, out_scores, out_idx, all_scores, ws, L, s);
    return hip_status(e);
}

int otf_rank_sparse(const uint32_t *rows, const int64_t *start, int64_t N, int32_t D, const float *w, float bias,
                    int32_t k, float *out_scores, int32_t *out_idx, float *all_scores, void *ws, size_t ws_bytes,
                    void *stream) {
    WsLayout L;
    if (!rows || !start || !w || D < 1) return OTF_ERR_INVALID_ARG;
    int rc = check_rank_common(N, k, 1, out_scores, out_idx, ws, ws_bytes, &L);
    if (rc != OTF_OK) return rc;
    if (D != 128) return OTF_ERR_UNSUPPORTED;
    if (!aligned16(rows) || (reinterpret_cast<uintptr_t>(start) & 7u)) return OTF_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    SelectWs sw = select_ws(ws, L), ssw = sample_select_ws(ws, L);
    uint8_t *wsb = reinterpret_cast<uint8_t *>(ws);
    float *S = all_scores ? all_scores : reinterpret_cast<float *>(wsb + L.scores);
    hipError_t e = launch_select_init_both(sw, ssw, 1, s);
    if (e == hipSuccess && filter_eligible(N, k, all_scores)) {
        SampleSlot *slots = reinterpret_cast<SampleSlot *>(wsb + L.sample_scores);
        e = launch_sparse_scan(rows, start, sample_rows(N), N, w, bias, kEmitSample, nullptr, ssw.st, nullptr, nullptr,
                               slots, nullptr, kNoGate, s);
        ScanTimer timer(s);
        if (e == hipSuccess)
            e = launch_sparse_scan(rows, start, N, N, w, bias, kEmitFilter, nullptr, sw.st, nullptr, ssw.st, slots,
                                   sw.cand, kNoGate, s);
        timer.stop();
        if (e == hipSuccess)
            e = launch_sparse_scan(rows, start, N, N, w, bias, kEmitScores, S, sw.st, sw.hist1, nullptr, nullptr, nullptr,
                                   Gate{sw.st, k}, s);
        if (e == hipSuccess) e = launch_select_tail(S, N, N, 1, k, sw, out_scores, out_idx, kTailBehindScan, s);
        return hip_status(e);
    }
    ScanTimer timer(s);
    if (e == hipSuccess)
        e = launch_sparse_scan(rows, start, N, N, w, bias, kEmitScores, S, sw.st, sw.hist1, nullptr, nullptr, nullptr,
                               kNoGate, s);
    timer.stop();
    if (e == hipSuccess) e = launch_select_tail(S, N, N, 1, k, sw, out_scores, out_idx, kTailPlain, s);
    return hip_status(e);
}

size_t otf_sgd_workspace_bytes(int32_t B) {
    if (B < 1 || B > 4096) return 0;
    // the coefficients of one step, or the control block and partial vectors of a one-launch run
    return std::max<size_t>((size_t)4096 * sizeof(float), sgd_pass_ws_bytes(2048));
}

// The argument checks of a training step (host only).
static int sgd_step_check(const float *w, int32_t D, const float *Xpos, int64_t ld_pos, const int32_t *idx_pos,
                          int32_t n_pos, const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int32_t n_neg,
                          float lambda, int64_t t, const void *ws, size_t ws_bytes) {
    const int64_t batch = (int64_t)n_pos + n_neg;         // the two may each be the largest int32
    if (!w || D < 1 || n_pos < 0 || n_neg < 0 || batch < 1 || t < 1 || !(lambda > 0.f)) return OTF_ERR_INVALID_ARG;
    if (n_pos > 0 && (!Xpos || !idx_pos || ld_pos < D)) return OTF_ERR_INVALID_ARG;
    if (n_neg > 0 && (!Xneg || !idx_neg || ld_neg < D)) return OTF_ERR_INVALID_ARG;
    if (D % 4 != 0 || batch > 4096) return OTF_ERR_UNSUPPORTED;
    if (!aligned16(w) || (n_pos > 0 && (!aligned16(Xpos) || ld_pos % 4 != 0)) ||
        (n_neg > 0 && (!aligned16(Xneg) || ld_neg % 4 != 0)))
        return OTF_ERR_INVALID_ARG;
    if (!ws || ws_bytes < otf_sgd_workspace_bytes((int32_t)batch) || (reinterpret_cast<uintptr_t>(ws) & 15u))
        return OTF_ERR_WORKSPACE;
    return OTF_OK;
}

int otf_svm_sgd_step(float *w, float *b, int32_t D, const float *Xpos, int64_t ld_pos, const int32_t *idx_pos,
                     int32_t n_pos, const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int32_t n_neg,
                     float lambda, int64_t t, int32_t update_bias, void *ws, size_t ws_bytes, void *stream) {
    const int rc = sgd_step_check(w, D, Xpos, ld_pos, idx_pos, n_pos, Xneg, ld_neg, idx_neg, n_neg, lambda, t, ws,
                                  ws_bytes);
    if (rc != OTF_OK) return rc;
    return hip_status(launch_sgd_step(w, b, D, Xpos, ld_pos, idx_pos, n_pos, Xneg, ld_neg, idx_neg, n_neg, lambda, t,
                                      update_bias, reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + 256),
                                      reinterpret_cast<hipStream_t>(stream)));
}

int otf_svm_sgd_pass(float *w, float *b, int32_t D, const float *Xpos, int64_t ld_pos, const int32_t *idx_pos,
                     int32_t n_pos, const float *Xneg, int64_t ld_neg, const int32_t *idx_neg, int32_t n_neg,
                     float lambda, int64_t t_first, int32_t n_steps, int32_t update_bias, void *ws, size_t ws_bytes,
                     void *stream) {
    if (n_steps < 1) return OTF_ERR_INVALID_ARG;
    // the argument checks of a single step, without enqueuing anything
    const int rc = sgd_step_check(w, D, Xpos, ld_pos, idx_pos, n_pos, Xneg, ld_neg, idx_neg, n_neg, lambda, t_first, ws,
                                  ws_bytes);
    if (rc != OTF_OK) return rc;
    // One launch for the whole run exists (D <= 2048) but is not the default: its step is a chain of
    // round trips between workgroups on different dies (~15 us), slower than two launches per step (~10 us).
    if (sgd_pass_fits(D) && tune_int(OTF_DEBUG_SGD_PASS_PATH, 0) == 1) {
        const uint32_t limit = (uint32_t)tune_int(OTF_DEBUG_SGD_SPIN_LIMIT, 1 << 20);
        return hip_status(launch_sgd_pass(w, b, D, Xpos, ld_pos, idx_pos, n_pos, Xneg, ld_neg, idx_neg, n_neg, lambda,
                                          t_first, n_steps, update_bias, ws, limit,
                                          reinterpret_cast<hipStream_t>(stream)));
    }
    // two launches per step, enqueued back to back; the status word of the workspace reads 0 afterwards
    hipError_t e = hipSuccess;
    for (int32_t s = 0; s < n_steps && e == hipSuccess; ++s)
        e = launch_sgd_step(w, b, D, Xpos, ld_pos, idx_pos ? idx_pos + (size_t)s * n_pos : nullptr, n_pos, Xneg, ld_neg,
                            idx_neg ? idx_neg + (size_t)s * n_neg : nullptr, n_neg, lambda, t_first + s, update_bias,
                            reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + 256),
                            reinterpret_cast<hipStream_t>(stream));
    if (e == hipSuccess) e = launch_sgd_pass_clear_status(ws, reinterpret_cast<hipStream_t>(stream));
    return hip_status(e);
}

int otf_check_indices(const int32_t *idx, int64_t n, int64_t rows, int32_t *bad, void *stream) {
    if (!idx || !bad || n < 1 || rows < 1) return OTF_ERR_INVALID_ARG;
    return hip_status(launch_check_indices(idx, n, rows, bad, reinterpret_cast<hipStream_t>(stream)));
}

size_t otf_tight_frame_workspace_bytes(int32_t n, int32_t m) {
    if (n < 1 || m < 1 || m > n) return 0;
    return (size_t)n * (size_t)m * sizeof(double);
}

int otf_tight_frame(const float *G, int32_t n, int32_t m, float *U, void *ws, size_t ws_bytes, void *stream) {
    if (!G || !U || n < 1 || m < 1 || m > n) return OTF_ERR_INVALID_ARG;
    if (n > 4096 || m > 256) return OTF_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < otf_tight_frame_workspace_bytes(n, m) || (reinterpret_cast<uintptr_t>(ws) & 15u))
        return OTF_ERR_WORKSPACE;
    return hip_status(launch_tight_frame(G, n, m, reinterpret_cast<double *>(ws), U,
                                         reinterpret_cast<hipStream_t>(stream)));
}

int otf_binarize(const float *phi, int64_t N, int32_t m, int64_t ld_phi, const float *U, int32_t n, uint32_t *bits,
                 void *stream) {
    if (!phi || !U || !bits || N < 1 || m < 1 || n < 1 || ld_phi < m || ld_phi > kMaxStoreBytes / 4 / N)
        return OTF_ERR_INVALID_ARG;
    if (!aligned16(phi) || !aligned16(U) || ld_phi % 4 != 0) return OTF_ERR_INVALID_ARG;
    if (N >= ((int64_t)1 << 31)) return OTF_ERR_UNSUPPORTED;
    if (m % 4 != 0 || m > 128 || n % 32 != 0 || n > 65536) return OTF_ERR_UNSUPPORTED;
    return hip_status(launch_binarize(phi, N, m, ld_phi, U, n, bits, reinterpret_cast<hipStream_t>(stream)));
}

size_t otf_pq_train_workspace_bytes(int32_t M, int32_t dsub) {
    if (M < 1 || dsub < 1) return 0;
    return pq_train_ws_bytes(M, dsub);
}

static int pq_train_args(const float *X, int64_t N, int64_t ldx, const float *codebooks, int32_t M, int32_t K,
                         int32_t dsub, const uint8_t *codes, const void *ws, size_t ws_bytes) {
    if (!X || !codebooks || !codes || N < 1 || M < 1 || K < 1 || dsub < 1 || ldx < (int64_t)M * dsub ||
        ldx > kMaxStoreBytes / 4 / N)
        return OTF_ERR_INVALID_ARG;
    if (!aligned16(X) || !aligned16(codebooks) || ldx % 4 != 0 || (reinterpret_cast<uintptr_t>(codes) & 3u))
        return OTF_ERR_INVALID_ARG;
    if (N >= ((int64_t)1 << 31)) return OTF_ERR_UNSUPPORTED;
    if (K != 256 || (dsub != 4 && dsub != 8 && dsub != 16) || M % 4 != 0 || M > 4096) return OTF_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < otf_pq_train_workspace_bytes(M, dsub) || (reinterpret_cast<uintptr_t>(ws) & 255u))
        return OTF_ERR_WORKSPACE;
    return OTF_OK;
}

int otf_pq_encode(const float *X, int64_t N, int64_t ldx, const float *codebooks, int32_t M, int32_t K, int32_t dsub,
                  uint8_t *codes, void *ws, size_t ws_bytes, void *stream) {
    const int rc = pq_train_args(X, N, ldx, codebooks, M, K, dsub, codes, ws, ws_bytes);
    if (rc != OTF_OK) return rc;
    return hip_status(launch_pq_encode(X, N, ldx, codebooks, M, dsub, codes, ws, reinterpret_cast<hipStream_t>(stream)));
}

int otf_pq_lloyd_step(const float *X, int64_t N, int64_t ldx, float *codebooks, int32_t M, int32_t K, int32_t dsub,
                      uint8_t *codes, double *distortion, void *ws, size_t ws_bytes, void *stream) {
    const int rc = pq_train_args(X, N, ldx, codebooks, M, K, dsub, codes, ws, ws_bytes);
    if (rc != OTF_OK) return rc;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipError_t e = launch_pq_lloyd_assign(X, N, ldx, codebooks, M, dsub, codes, ws, s);
    if (e != hipSuccess) return hip_status(e);
    ScanTimer timer(s);                                    // the kernel of the per-centre sums, for otf_profile_*
    e = launch_pq_lloyd_sums(X, N, ldx, codes, M, dsub, ws, s);
    timer.stop();
    if (e != hipSuccess) return hip_status(e);
    return hip_status(launch_pq_lloyd_move(N, codebooks, M, dsub, distortion, ws, s));
}

int otf_debug_set(int key, int value) {
    if (key < 0 || key >= OTF_DEBUG_KEYS) return OTF_ERR_INVALID_ARG;
    if (value != 0 && !debug_value_ok(key, value)) return OTF_ERR_INVALID_ARG;
    g_debug[key].store(value, std::memory_order_relaxed);
    return OTF_OK;
}

int otf_profile_begin(int32_t max_records) {
    if (g_prof.on || max_records < 1 || max_records > 65536) return OTF_ERR_INVALID_ARG;
    g_prof.start.assign(max_records, nullptr);
    g_prof.stop.assign(max_records, nullptr);
    for (int i = 0; i < max_records; ++i) {
        if (hipEventCreate(&g_prof.start[i]) != hipSuccess || hipEventCreate(&g_prof.stop[i]) != hipSuccess) {
            for (int j = 0; j <= i; ++j) {
                if (g_prof.start[j]) (void)hipEventDestroy(g_prof.start[j]);
                if (g_prof.stop[j]) (void)hipEventDestroy(g_prof.stop[j]);
            }
            g_prof.start.clear();
            g_prof.stop.clear();
            return hip_status(hipErrorOutOfMemory);
        }
    }
    g_prof.used = 0;
    g_prof.on = true;
    return OTF_OK;
}

int otf_profile_end(double *scan_ms_total, int32_t *n_records) {
    if (!g_prof.on || !scan_ms_total || !n_records) return OTF_ERR_INVALID_ARG;
    double total = 0.0;
    int rc = OTF_OK;
    for (int i = 0; i < g_prof.used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess)
            rc = OTF_ERR_HIP;
        total += ms;
    }
    for (size_t i = 0; i < g_prof.start.size(); ++i) {
        (void)hipEventDestroy(g_prof.start[i]);
        (void)hipEventDestroy(g_prof.stop[i]);
    }
    *scan_ms_total = total;
    *n_records = g_prof.used;
    g_prof.start.clear();
    g_prof.stop.clear();
    g_prof.used = 0;
    g_prof.on = false;
    if (rc != OTF_OK) (void)hipGetLastError();
    return rc;
}

}  // extern "C"
