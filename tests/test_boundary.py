"""Host-side checks of the C ABI: the library loads, exports every function the header
declares, and rejects bad arguments before anything is enqueued (so these run without a GPU:
a rejected call makes no HIP call and dereferences no pointer)."""
import ctypes
import os
import re

import pytest

from paper_1407_4764_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # a 256-aligned non-NULL address that must never be dereferenced
BIG = 1 << 40


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_1407_4764_amd import build
        build.build_library()
    return binding.lib()


def test_header_functions_are_exported(L):
    header = open(os.path.join(ROOT, "include", "otf.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(otf_[a-z_0-9]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings(L):
    assert binding.status_string(0) == "OTF_OK"
    assert binding.status_string(-1) == "OTF_ERR_INVALID_ARG"
    assert binding.status_string(-3) == "OTF_ERR_WORKSPACE"
    assert binding.status_string(-5) == "OTF_ERR_SCRATCH"
    assert binding.status_string(-99) == "OTF_ERR_UNKNOWN"


def test_workspace_query(L):
    assert binding.workspace_bytes(0, 1, 1) == 0
    assert binding.workspace_bytes(10, 0, 1) == 0
    assert binding.workspace_bytes(1 << 31, 1, 1) == 0
    a = binding.workspace_bytes(1000, 10, 1)
    b = binding.workspace_bytes(1000000, 10, 1)
    c = binding.workspace_bytes(1000000, 10, 4)
    assert 0 < a < b < c and a % 256 == 0
    assert b - a >= (1000000 - 1000) * 4 - 4096      # room for one score per row
    assert L.otf_sgd_workspace_bytes(0) == 0 and L.otf_sgd_workspace_bytes(256) > 0


def _topk(L, scores=FAKE, N=100, ld=100, Q=1, k=10, os_=FAKE, oi=FAKE, ws=FAKE, wsb=BIG):
    return L.otf_topk(scores, N, ld, Q, k, os_, oi, ws, wsb, None)


def test_topk_argument_errors(L):
    assert _topk(L, scores=None) == binding.OTF_ERR_INVALID_ARG
    assert _topk(L, N=0) == binding.OTF_ERR_INVALID_ARG
    assert _topk(L, k=0) == binding.OTF_ERR_INVALID_ARG
    assert _topk(L, k=101) == binding.OTF_ERR_INVALID_ARG
    assert _topk(L, N=100000, ld=100000, k=binding.OTF_MAX_K + 1) == binding.OTF_ERR_UNSUPPORTED   # a limit of the build
    assert _topk(L, N=100, ld=100, k=binding.OTF_MAX_K + 1) == binding.OTF_ERR_INVALID_ARG         # k > N comes first
    assert _topk(L, ld=99) == binding.OTF_ERR_INVALID_ARG
    assert _topk(L, os_=None) == binding.OTF_ERR_INVALID_ARG
    assert _topk(L, N=1 << 31, ld=1 << 31) == binding.OTF_ERR_UNSUPPORTED
    assert _topk(L, ws=None) == binding.OTF_ERR_WORKSPACE
    assert _topk(L, ws=FAKE + 8) == binding.OTF_ERR_WORKSPACE
    assert _topk(L, wsb=binding.workspace_bytes(100, 10, 1) - 1) == binding.OTF_ERR_WORKSPACE


def _dense(L, X=FAKE, xdt=0, N=1000, D=128, ldx=128, W=FAKE, wdt=0, Q=1, k=10, ws=FAKE, wsb=BIG):
    return L.otf_rank_dense(X, xdt, N, D, ldx, W, wdt, Q, None, k, FAKE, FAKE, None, ws, wsb, None)


def test_rank_dense_argument_errors(L):
    assert _dense(L, X=None) == binding.OTF_ERR_INVALID_ARG
    assert _dense(L, W=None) == binding.OTF_ERR_INVALID_ARG
    assert _dense(L, D=0) == binding.OTF_ERR_INVALID_ARG
    assert _dense(L, ldx=64) == binding.OTF_ERR_INVALID_ARG
    assert _dense(L, X=FAKE + 4) == binding.OTF_ERR_INVALID_ARG            # misaligned base
    assert _dense(L, D=126, ldx=126) == binding.OTF_ERR_INVALID_ARG        # row stride not 16-byte
    assert _dense(L, D=6, ldx=8) == binding.OTF_ERR_UNSUPPORTED            # D not a multiple of 4
    assert _dense(L, xdt=7) == binding.OTF_ERR_INVALID_ARG
    assert _dense(L, xdt=0, wdt=1) == binding.OTF_ERR_UNSUPPORTED          # fp32 store, fp16 model
    assert _dense(L, D=32768, ldx=32768) == binding.OTF_ERR_UNSUPPORTED
    assert _dense(L, wsb=1024) == binding.OTF_ERR_WORKSPACE
    assert _dense(L, k=2000) == binding.OTF_ERR_INVALID_ARG                # k > N
    assert _dense(L, ldx=1 << 60) == binding.OTF_ERR_INVALID_ARG           # a store of more than 2^48 bytes
    assert _dense(L, xdt=-3) == binding.OTF_ERR_INVALID_ARG


def test_pq_and_binary_argument_errors(L):
    def pq(codes=FAKE, N=1000, M=128, K=256, lut=FAKE, k=10, wsb=BIG):
        return L.otf_rank_pq(codes, N, M, K, lut, 0.0, k, FAKE, FAKE, None, FAKE, wsb, None)
    assert pq(codes=None) == binding.OTF_ERR_INVALID_ARG
    assert pq(K=128) == binding.OTF_ERR_UNSUPPORTED
    assert pq(M=40) == binding.OTF_ERR_UNSUPPORTED              # rows are read in 16-byte chunks
    assert pq(M=8) == binding.OTF_ERR_UNSUPPORTED
    assert pq(M=1040) == binding.OTF_ERR_UNSUPPORTED            # more than 8 table images
    assert pq(M=2048) == binding.OTF_ERR_UNSUPPORTED
    assert pq(wsb=0) == binding.OTF_ERR_WORKSPACE
    assert pq(codes=FAKE + 1) == binding.OTF_ERR_INVALID_ARG

    def pqm(codes=FAKE, M=128, K=256, dsub=16, cb=FAKE, w=FAKE, wsb=BIG):
        return L.otf_rank_pq_model(codes, 1000, M, K, dsub, cb, w, 0.0, 10, FAKE, FAKE, None, FAKE, wsb, None)
    assert pqm(cb=None) == binding.OTF_ERR_INVALID_ARG
    assert pqm(w=None) == binding.OTF_ERR_INVALID_ARG
    assert pqm(dsub=0) == binding.OTF_ERR_INVALID_ARG
    assert pqm(K=16) == binding.OTF_ERR_UNSUPPORTED
    assert pqm(M=40) == binding.OTF_ERR_UNSUPPORTED
    assert pqm(wsb=0) == binding.OTF_ERR_WORKSPACE

    def binr(bits=FAKE, N=1000, D=2048, w=FAKE, k=10, wsb=BIG):
        return L.otf_rank_binary(bits, N, D, w, 0.0, k, FAKE, FAKE, None, FAKE, wsb, None)
    assert binr(bits=None) == binding.OTF_ERR_INVALID_ARG
    assert binr(D=100) == binding.OTF_ERR_UNSUPPORTED
    assert binr(D=96) == binding.OTF_ERR_UNSUPPORTED            # a multiple of 32 bits but not of 128
    assert binr(D=8320) == binding.OTF_ERR_UNSUPPORTED          # beyond 8192 bits
    assert binr(k=0) == binding.OTF_ERR_INVALID_ARG

    def ham(bits=FAKE, N=1000, D=2048, q=FAKE, k=10, wsb=BIG):
        return L.otf_rank_hamming(bits, N, D, q, k, FAKE, FAKE, None, FAKE, wsb, None)
    assert ham(bits=None) == binding.OTF_ERR_INVALID_ARG
    assert ham(q=None) == binding.OTF_ERR_INVALID_ARG
    assert ham(q=FAKE + 4) == binding.OTF_ERR_INVALID_ARG
    assert ham(D=96) == binding.OTF_ERR_UNSUPPORTED
    assert ham(D=16384) == binding.OTF_ERR_UNSUPPORTED
    assert ham(k=1001) == binding.OTF_ERR_INVALID_ARG
    assert ham(wsb=0) == binding.OTF_ERR_WORKSPACE

    def sparse(rows=FAKE, start=FAKE, N=1000, D=128, w=FAKE, k=10, wsb=BIG):
        return L.otf_rank_sparse(rows, start, N, D, w, 0.0, k, FAKE, FAKE, None, FAKE, wsb, None)
    assert sparse(rows=None) == binding.OTF_ERR_INVALID_ARG
    assert sparse(start=None) == binding.OTF_ERR_INVALID_ARG
    assert sparse(rows=FAKE + 4) == binding.OTF_ERR_INVALID_ARG
    assert sparse(D=2048) == binding.OTF_ERR_UNSUPPORTED
    assert sparse(k=0) == binding.OTF_ERR_INVALID_ARG
    assert sparse(wsb=0) == binding.OTF_ERR_WORKSPACE
    assert L.otf_pq_build_lut(None, 1, 1, 1, FAKE, FAKE, None) == binding.OTF_ERR_INVALID_ARG
    assert L.otf_pq_build_lut(FAKE, 0, 1, 1, FAKE, FAKE, None) == binding.OTF_ERR_INVALID_ARG


def test_sgd_argument_errors(L):
    def sgd(w=FAKE, D=128, Xp=FAKE, ldp=128, ip=FAKE, npos=4, Xn=FAKE, ldn=128, ineg=FAKE, nneg=4, lam=1.0, t=1,
            ws=FAKE, wsb=BIG):
        return L.otf_svm_sgd_step(w, None, D, Xp, ldp, ip, npos, Xn, ldn, ineg, nneg, lam, t, 0, ws, wsb, None)
    assert sgd(w=None) == binding.OTF_ERR_INVALID_ARG
    assert sgd(t=0) == binding.OTF_ERR_INVALID_ARG
    assert sgd(lam=0.0) == binding.OTF_ERR_INVALID_ARG
    assert sgd(npos=0, nneg=0) == binding.OTF_ERR_INVALID_ARG
    assert sgd(Xp=None) == binding.OTF_ERR_INVALID_ARG
    assert sgd(ldp=64) == binding.OTF_ERR_INVALID_ARG
    assert sgd(D=126, ldp=128, ldn=128) == binding.OTF_ERR_UNSUPPORTED
    assert sgd(npos=4000, nneg=4000) == binding.OTF_ERR_UNSUPPORTED
    assert sgd(npos=2 ** 31 - 1, nneg=2 ** 31 - 1) == binding.OTF_ERR_UNSUPPORTED    # the sum does not wrap
    assert sgd(ws=None) == binding.OTF_ERR_WORKSPACE
    assert sgd(wsb=16) == binding.OTF_ERR_WORKSPACE
    assert sgd(wsb=L.otf_sgd_workspace_bytes(8) - 1) == binding.OTF_ERR_WORKSPACE


def test_encoder_argument_errors(L):
    def frame(G=FAKE, n=256, m=32, U=FAKE, ws=FAKE, wsb=BIG):
        return L.otf_tight_frame(G, n, m, U, ws, wsb, None)

    def binz(phi=FAKE, N=1000, m=128, ld=128, U=FAKE, n=2048, bits=FAKE):
        return L.otf_binarize(phi, N, m, ld, U, n, bits, None)

    assert L.otf_tight_frame_workspace_bytes(2048, 128) == 2048 * 128 * 8
    assert L.otf_tight_frame_workspace_bytes(16, 32) == 0                  # m > n
    assert frame(G=None) == binding.OTF_ERR_INVALID_ARG
    assert frame(m=300, n=256) == binding.OTF_ERR_INVALID_ARG              # more columns than the matrix has
    assert frame(n=16384, m=128) == binding.OTF_ERR_UNSUPPORTED
    assert frame(wsb=1024) == binding.OTF_ERR_WORKSPACE
    assert binz(bits=None) == binding.OTF_ERR_INVALID_ARG
    assert binz(ld=64) == binding.OTF_ERR_INVALID_ARG                      # rows shorter than m
    assert binz(phi=FAKE + 4) == binding.OTF_ERR_INVALID_ARG               # misaligned
    assert binz(m=256, ld=256) == binding.OTF_ERR_UNSUPPORTED
    assert binz(m=126, ld=128) == binding.OTF_ERR_UNSUPPORTED
    assert binz(n=2040) == binding.OTF_ERR_UNSUPPORTED


def test_sgd_pass_argument_errors(L):
    def sgd(n_steps=4, w=FAKE, D=128, n=16, lam=1.0, t=1, wsb=BIG):
        return L.otf_svm_sgd_pass(w, None, D, FAKE, D, FAKE, n, FAKE, D, FAKE, n, ctypes.c_float(lam), t, n_steps, 0,
                                  FAKE, wsb, None)

    assert sgd(n_steps=0) == binding.OTF_ERR_INVALID_ARG
    assert sgd(w=None) == binding.OTF_ERR_INVALID_ARG
    assert sgd(t=0) == binding.OTF_ERR_INVALID_ARG
    assert sgd(D=126) == binding.OTF_ERR_UNSUPPORTED
    assert sgd(wsb=16) == binding.OTF_ERR_WORKSPACE


def test_check_indices_argument_errors(L):
    assert L.otf_check_indices(None, 10, 10, FAKE, None) == binding.OTF_ERR_INVALID_ARG
    assert L.otf_check_indices(FAKE, 10, 10, None, None) == binding.OTF_ERR_INVALID_ARG
    assert L.otf_check_indices(FAKE, 0, 10, FAKE, None) == binding.OTF_ERR_INVALID_ARG
    assert L.otf_check_indices(FAKE, 10, 0, FAKE, None) == binding.OTF_ERR_INVALID_ARG


def test_pq_train_argument_errors(L):
    def enc(X=FAKE, N=1000, ldx=2048, cb=FAKE, M=128, K=256, dsub=16, codes=FAKE, ws=FAKE, wsb=BIG):
        return L.otf_pq_encode(X, N, ldx, cb, M, K, dsub, codes, ws, wsb, None)

    assert L.otf_pq_train_workspace_bytes(128, 16) >= 128 * 256 * (4 + 64 + 4)
    assert L.otf_pq_train_workspace_bytes(0, 16) == 0
    assert enc(X=None) == binding.OTF_ERR_INVALID_ARG
    assert enc(ldx=1024) == binding.OTF_ERR_INVALID_ARG                   # rows shorter than M * dsub
    assert enc(codes=FAKE + 2) == binding.OTF_ERR_INVALID_ARG
    assert enc(K=128) == binding.OTF_ERR_UNSUPPORTED
    assert enc(dsub=12, ldx=4096) == binding.OTF_ERR_UNSUPPORTED
    assert enc(M=126) == binding.OTF_ERR_UNSUPPORTED
    assert enc(wsb=4096) == binding.OTF_ERR_WORKSPACE
    assert L.otf_pq_lloyd_step(FAKE, 1000, 2048, None, 128, 256, 16, FAKE, None, FAKE, BIG, None) == binding.OTF_ERR_INVALID_ARG


def test_debug_switches_accept_only_their_own_values(L):
    assert L.otf_debug_set(-1, 1) == binding.OTF_ERR_INVALID_ARG
    assert L.otf_debug_set(binding.DEBUG_KEYS, 1) == binding.OTF_ERR_INVALID_ARG
    assert L.otf_debug_set(binding.DEBUG_RANK_PATH, 2) == binding.OTF_ERR_INVALID_ARG
    assert L.otf_debug_set(binding.DEBUG_SCAN_THREADS, 100) == binding.OTF_ERR_INVALID_ARG      # not whole waves
    assert L.otf_debug_set(binding.DEBUG_SCAN_THREADS, 2048) == binding.OTF_ERR_INVALID_ARG     # above the launch bound
    assert L.otf_debug_set(binding.DEBUG_SCAN_UNROLL, 5) == binding.OTF_ERR_INVALID_ARG
    assert L.otf_debug_set(binding.DEBUG_PQENC_RANGE, 6) == binding.OTF_ERR_INVALID_ARG
    assert L.otf_debug_set(binding.DEBUG_MFMA_BLOCKS_PER_CU, 9) == binding.OTF_ERR_INVALID_ARG
    for key, value in ((binding.DEBUG_RANK_PATH, 1), (binding.DEBUG_SCAN_THREADS, 512), (binding.DEBUG_SCAN_UNROLL, 4),
                       (binding.DEBUG_PQENC_RANGE, 8), (binding.DEBUG_DENSE_BLOCKS_PER_CU, 2)):
        assert L.otf_debug_set(key, value) == binding.OTF_OK
        assert L.otf_debug_set(key, 0) == binding.OTF_OK                                        # cleared again


def test_the_library_reads_no_environment_variables():
    """Path and launch-shape switches go through otf_debug_set, never through the environment."""
    csrc = os.path.join(ROOT, "paper_1407_4764_amd", "csrc")
    for name in os.listdir(csrc):
        assert "getenv" not in open(os.path.join(csrc, name)).read(), name


def test_noalloc_entry_point_argument_errors(L):
    def call(X=FAKE, N=1000, D=128, ldx=128, W=FAKE, Q=1, k=10, os_=FAKE):
        return L.otf_rank_dense_noalloc(X, 0, N, D, ldx, W, 0, Q, None, k, os_, FAKE, None, None)
    assert call(X=None) == binding.OTF_ERR_INVALID_ARG
    assert call(os_=None) == binding.OTF_ERR_INVALID_ARG
    assert call(k=2000) == binding.OTF_ERR_INVALID_ARG
    assert call(D=6, ldx=8) == binding.OTF_ERR_UNSUPPORTED
    assert call(N=1 << 31) == binding.OTF_ERR_UNSUPPORTED
    # sizes whose workspace exceeds the static scratch are refused before anything is touched
    assert binding.workspace_bytes(100_000_000, 10, 1) > binding.OTF_NOALLOC_SCRATCH_BYTES
    assert call(N=100_000_000) == binding.OTF_ERR_SCRATCH
    assert call(N=1_000_000, Q=64, k=10) == binding.OTF_ERR_SCRATCH
    assert binding.workspace_bytes(1_000_000, 1000, 1) <= binding.OTF_NOALLOC_SCRATCH_BYTES   # the headline store fits
