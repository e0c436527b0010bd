// Calls every entry point of the C ABI the way a careless caller would: null and misaligned
// pointers, sizes of zero, one too many, the largest a type holds, workspaces a byte short, switch
// keys out of range.  Every call must come back with the status the header promises before
// anything is enqueued and before any pointer is followed (the non-null "pointers" here are not
// memory).  Linked by tests/test_sanitizers.py against the library's argument-validation code
// built with -fsanitize=address,undefined: an overflow in a size computation, a table indexed out
// of range or a read of a caller's buffer ends the program with a report.  No call reaches a GPU.
// TEST INFRASTRUCTURE ONLY.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "otf.h"

static int failures = 0;
#define EXPECT(call, want)                                                                      \
    do {                                                                                        \
        const long long got_ = (long long)(call);                                               \
        if (got_ != (long long)(want)) {                                                        \
            std::printf("line %d: %s returned %lld, expected %lld\n", __LINE__, #call, got_, (long long)(want)); \
            ++failures;                                                                         \
        }                                                                                       \
    } while (0)

template <typename T>
static T *fake(uintptr_t off = 0) {
    return reinterpret_cast<T *>((uintptr_t)0x10000 + off);      // aligned to 256 bytes when off = 0; never followed
}
static const size_t BIG = (size_t)1 << 40;

int main() {
    float *F = fake<float>();
    int32_t *I = fake<int32_t>();
    uint8_t *B = fake<uint8_t>();
    uint32_t *U = fake<uint32_t>();
    int64_t *L = fake<int64_t>();
    void *WS = fake<void>();

    // workspace queries over the whole range of their arguments: no overflow on the way to the answer
    for (int64_t N : {(int64_t)INT64_MIN, (int64_t)-1, (int64_t)0, (int64_t)1, (int64_t)63, (int64_t)64, (int64_t)1000, (int64_t)1 << 20,
                      ((int64_t)1 << 31) - 1, (int64_t)1 << 31, (int64_t)1 << 40, (int64_t)INT64_MAX})
        for (int32_t k : {INT32_MIN, -1, 0, 1, 1000, (int32_t)OTF_MAX_K, (int32_t)OTF_MAX_K + 1, INT32_MAX})
            for (int32_t Q : {INT32_MIN, 0, 1, 64, 65, 4096, INT32_MAX}) {
                const size_t b = otf_workspace_bytes(N, k, Q);
                const bool valid = N >= 1 && N < ((int64_t)1 << 31) && k >= 1 && Q >= 1;
                if (!valid) EXPECT(b, 0);
                if (b % 256 != 0) { std::printf("workspace_bytes(%lld, %d, %d) = %zu is not a multiple of 256\n", (long long)N, k, Q, b); ++failures; }
            }
    for (int32_t v : {INT32_MIN, -1, 0, 1, 8, 2048, 2049, INT32_MAX}) {
        (void)otf_sgd_workspace_bytes(v);
        for (int32_t u : {INT32_MIN, -1, 0, 1, 4, 16, 128, 4096, INT32_MAX}) {
            (void)otf_pq_train_workspace_bytes(v, u);
            (void)otf_tight_frame_workspace_bytes(v, u);
        }
    }
    EXPECT(otf_tight_frame_workspace_bytes(2048, 128), (size_t)2048 * 128 * 8);
    EXPECT(otf_tight_frame_workspace_bytes(16, 32), 0);
    for (int s = -10; s <= 5; ++s) (void)otf_status_string(s);

    // otf_topk
    EXPECT(otf_topk(nullptr, 100, 100, 1, 10, F, I, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_topk(F, 0, 100, 1, 10, F, I, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_topk(F, 100, 100, 1, 0, F, I, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_topk(F, 100, 100, 1, 101, F, I, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_topk(F, 100, 99, 1, 10, F, I, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_topk(F, 100, 100, 0, 10, F, I, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_topk(F, 100000, 100000, 1, OTF_MAX_K + 1, F, I, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_topk(F, (int64_t)1 << 31, (int64_t)1 << 31, 1, 10, F, I, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_topk(F, INT64_MAX, INT64_MAX, INT32_MAX, 10, F, I, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_topk(F, 100, 100, 1, 10, F, I, nullptr, BIG, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_topk(F, 100, 100, 1, 10, F, I, fake<void>(8), BIG, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_topk(F, 100, 100, 1, 10, F, I, WS, otf_workspace_bytes(100, 10, 1) - 1, nullptr), OTF_ERR_WORKSPACE);

    // otf_rank_dense and its variant without a workspace
    EXPECT(otf_rank_dense(nullptr, OTF_F32, 1000, 128, 128, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense(F, OTF_F32, 1000, 128, 128, nullptr, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense(F, OTF_F32, 1000, 0, 128, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense(F, OTF_F32, 1000, 128, 64, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense(fake<float>(4), OTF_F32, 1000, 128, 128, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense(F, OTF_F32, 1000, 126, 126, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense(F, OTF_F32, 1000, 6, 8, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_dense(F, 7, 1000, 128, 128, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense(F, OTF_F32, 1000, 128, 128, F, OTF_F16, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_dense(F, OTF_F32, 1000, 32768, 32768, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_dense(F, OTF_F32, 1000, 128, 128, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, WS, 1024, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_rank_dense(F, OTF_F32, 1000, 128, 128, F, OTF_F32, 1, nullptr, 2000, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense(F, OTF_F16, 1000, 128, INT64_MAX - 7, F, OTF_F16, 64, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_topk(F, 100, INT64_MAX, 64, 10, F, I, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense_noalloc(nullptr, OTF_F32, 1000, 128, 128, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense_noalloc(F, OTF_F32, 1000, 128, 128, F, OTF_F32, 1, nullptr, 10, nullptr, I, nullptr, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_dense_noalloc(F, OTF_F32, 1000, 6, 8, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_dense_noalloc(F, OTF_F32, (int64_t)1 << 31, 128, 128, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_dense_noalloc(F, OTF_F32, 100000000, 128, 128, F, OTF_F32, 1, nullptr, 10, F, I, nullptr, nullptr), OTF_ERR_SCRATCH);
    EXPECT(otf_rank_dense_noalloc(F, OTF_F32, 1000000, 128, 128, F, OTF_F32, 64, nullptr, 10, F, I, nullptr, nullptr), OTF_ERR_SCRATCH);

    // code stores
    EXPECT(otf_rank_pq(nullptr, 1000, 128, 256, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_pq(B, 1000, 128, 128, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    for (int32_t M : {8, 40, 1040, 2048, INT32_MAX})
        EXPECT(otf_rank_pq(B, 1000, M, 256, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_pq(B, 1000, 128, 256, F, 0.f, 10, F, I, nullptr, WS, 0, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_rank_pq(fake<uint8_t>(1), 1000, 128, 256, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_pq_model(B, 1000, 128, 256, 16, nullptr, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_pq_model(B, 1000, 128, 256, 16, F, nullptr, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_pq_model(B, 1000, 128, 256, 0, F, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_pq_model(B, 1000, 128, 16, 16, F, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_pq_model(B, 1000, 40, 256, 16, F, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_pq_model(B, 1000, 128, 256, 16, F, F, 0.f, 10, F, I, nullptr, WS, 0, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_rank_binary(nullptr, 1000, 2048, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    for (int32_t D : {96, 100, 8320, INT32_MAX - 127})
        EXPECT(otf_rank_binary(U, 1000, D, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_binary(U, 1000, 2048, F, 0.f, 0, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_hamming(nullptr, 1000, 2048, U, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_hamming(U, 1000, 2048, nullptr, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_hamming(U, 1000, 2048, fake<uint32_t>(4), 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_hamming(U, 1000, 96, U, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_hamming(U, 1000, 16384, U, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_hamming(U, 1000, 2048, U, 1001, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_hamming(U, 1000, 2048, U, 10, F, I, nullptr, WS, 0, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_rank_sparse(nullptr, L, 1000, 128, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_sparse(U, nullptr, 1000, 128, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_sparse(fake<uint32_t>(4), L, 1000, 128, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_sparse(U, L, 1000, 2048, F, 0.f, 10, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_rank_sparse(U, L, 1000, 128, F, 0.f, 0, F, I, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_rank_sparse(U, L, 1000, 128, F, 0.f, 10, F, I, nullptr, WS, 0, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_pq_build_lut(nullptr, 1, 1, 1, F, F, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_pq_build_lut(F, 0, 1, 1, F, F, nullptr), OTF_ERR_INVALID_ARG);

    // training
    EXPECT(otf_svm_sgd_step(nullptr, nullptr, 128, F, 128, I, 4, F, 128, I, 4, 1.f, 1, 0, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_svm_sgd_step(F, nullptr, 128, F, 128, I, 4, F, 128, I, 4, 1.f, 0, 0, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_svm_sgd_step(F, nullptr, 128, F, 128, I, 4, F, 128, I, 4, 0.f, 1, 0, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_svm_sgd_step(F, nullptr, 128, F, 128, I, 0, F, 128, I, 0, 1.f, 1, 0, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_svm_sgd_step(F, nullptr, 128, nullptr, 128, I, 4, F, 128, I, 4, 1.f, 1, 0, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_svm_sgd_step(F, nullptr, 128, F, 64, I, 4, F, 128, I, 4, 1.f, 1, 0, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_svm_sgd_step(F, nullptr, 126, F, 128, I, 4, F, 128, I, 4, 1.f, 1, 0, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_svm_sgd_step(F, nullptr, 128, F, 128, I, 4000, F, 128, I, 4000, 1.f, 1, 0, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_svm_sgd_step(F, nullptr, 128, F, 128, I, INT32_MAX, F, 128, I, INT32_MAX, 1.f, 1, 0, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_svm_sgd_step(F, nullptr, 128, F, 128, I, 4, F, 128, I, 4, 1.f, 1, 0, nullptr, BIG, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_svm_sgd_step(F, nullptr, 128, F, 128, I, 4, F, 128, I, 4, 1.f, 1, 0, WS, otf_sgd_workspace_bytes(8) - 1, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_svm_sgd_pass(F, nullptr, 128, F, 128, I, 16, F, 128, I, 16, 1.f, 1, 0, 0, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_svm_sgd_pass(nullptr, nullptr, 128, F, 128, I, 16, F, 128, I, 16, 1.f, 1, 4, 0, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_svm_sgd_pass(F, nullptr, 128, F, 128, I, 16, F, 128, I, 16, 1.f, 0, 4, 0, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_svm_sgd_pass(F, nullptr, 126, F, 126, I, 16, F, 126, I, 16, 1.f, 1, 4, 0, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_svm_sgd_pass(F, nullptr, 128, F, 128, I, 16, F, 128, I, 16, 1.f, 1, 4, 0, WS, 16, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_svm_sgd_pass(F, nullptr, 128, F, 128, I, 16, F, 128, I, 16, 1.f, INT64_MAX, INT32_MAX, 0, WS, 16, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_check_indices(nullptr, 10, 10, I, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_check_indices(I, 10, 10, nullptr, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_check_indices(I, 0, 10, I, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_check_indices(I, 10, 0, I, nullptr), OTF_ERR_INVALID_ARG);

    // encoders
    EXPECT(otf_tight_frame(nullptr, 256, 32, F, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_tight_frame(F, 256, 300, F, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_tight_frame(F, 16384, 128, F, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_tight_frame(F, 256, 32, F, WS, 1024, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_binarize(F, 1000, 128, 128, F, 2048, nullptr, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_binarize(F, 1000, 128, 64, F, 2048, U, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_binarize(fake<float>(4), 1000, 128, 128, F, 2048, U, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_binarize(F, 1000, 256, 256, F, 2048, U, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_binarize(F, 1000, 126, 128, F, 2048, U, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_binarize(F, 1000, 128, 128, F, 2040, U, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_pq_encode(nullptr, 1000, 2048, F, 128, 256, 16, B, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_pq_encode(F, 1000, 1024, F, 128, 256, 16, B, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_pq_encode(F, 1000, 2048, F, 128, 256, 16, fake<uint8_t>(2), WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_pq_encode(F, 1000, 2048, F, 128, 128, 16, B, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_pq_encode(F, 1000, 4096, F, 128, 256, 12, B, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_pq_encode(F, 1000, 2048, F, 126, 256, 16, B, WS, BIG, nullptr), OTF_ERR_UNSUPPORTED);
    EXPECT(otf_pq_encode(F, 1000, 2048, F, 128, 256, 16, B, WS, 4096, nullptr), OTF_ERR_WORKSPACE);
    EXPECT(otf_pq_encode(F, 1000, INT64_MAX - 3, F, INT32_MAX - 3, 256, 16, B, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_binarize(F, INT64_MAX, 128, INT64_MAX - 3, F, 2048, U, nullptr), OTF_ERR_INVALID_ARG);
    EXPECT(otf_pq_lloyd_step(F, 1000, 2048, nullptr, 128, 256, 16, B, nullptr, WS, BIG, nullptr), OTF_ERR_INVALID_ARG);

    // switches and the profiling bracket
    EXPECT(otf_debug_set(-1, 1), OTF_ERR_INVALID_ARG);
    EXPECT(otf_debug_set(INT32_MIN, 1), OTF_ERR_INVALID_ARG);
    EXPECT(otf_debug_set(OTF_DEBUG_KEYS, 1), OTF_ERR_INVALID_ARG);
    EXPECT(otf_debug_set(INT32_MAX, 1), OTF_ERR_INVALID_ARG);
    for (int key = 0; key < OTF_DEBUG_KEYS; ++key) {
        for (int v : {INT32_MIN, -1, 3, 5, 100, 2048, 65537, INT32_MAX}) {
            const int rc = otf_debug_set(key, v);
            if (rc == OTF_OK) EXPECT(otf_debug_set(key, 0), OTF_OK);   // a value the key takes: clear it again
            else EXPECT(rc, OTF_ERR_INVALID_ARG);
        }
        EXPECT(otf_debug_set(key, 0), OTF_OK);
    }
    EXPECT(otf_debug_set(OTF_DEBUG_SCAN_THREADS, 100), OTF_ERR_INVALID_ARG);
    EXPECT(otf_debug_set(OTF_DEBUG_SCAN_THREADS, 512), OTF_OK);
    EXPECT(otf_debug_set(OTF_DEBUG_SCAN_THREADS, 0), OTF_OK);
    double ms = 0.0;
    int32_t n = 0;
    EXPECT(otf_profile_begin(0), OTF_ERR_INVALID_ARG);
    EXPECT(otf_profile_begin(1 << 20), OTF_ERR_INVALID_ARG);
    EXPECT(otf_profile_end(&ms, &n), OTF_ERR_INVALID_ARG);         // nothing was begun

    if (failures) {
        std::printf("%d unexpected results\n", failures);
        return 1;
    }
    std::printf("boundary driver: every call was rejected as documented\n");
    return 0;
}
