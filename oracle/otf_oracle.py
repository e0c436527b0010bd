"""ctypes front for oracle/otf_oracle.c -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module.  It marshals numpy arrays into the plain-C oracle and holds no arithmetic of
the method itself (the one exception, ``topk_parity_ok``, is the comparison rule the
tests use, not part of the method).  It never imports the HIP package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "otf_oracle.c")
_LIB = os.path.join(_HERE, "libotf_oracle.so")
_lib = None


def build(force=False):
    """Compile otf_oracle.c with gcc (-O2 -fopenmp); returns the path of the library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_half_to_double.restype = ctypes.c_double
        _lib.orc_half_to_double.argtypes = [ctypes.c_uint16]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(rc, what):
    if rc != 0:
        raise RuntimeError("%s failed with oracle status %d" % (what, rc))


def num_threads():
    return int(_load().orc_num_threads())


def half_to_double(h):
    return float(_load().orc_half_to_double(int(h)))


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def dense_scores(X, W, bias=None):
    """X: (N,D) float32 or float16; W: (Q,D) or (D,) float32 or float16 -> (Q,N) float64."""
    W2 = np.atleast_2d(W)
    Q, D = W2.shape
    N = X.shape[0]
    assert X.shape[1] == D
    out = np.empty((Q, N), dtype=np.float64)
    b = None if bias is None else _c(np.atleast_1d(bias), np.float32)
    lib = _load()
    I64, I32 = ctypes.c_int64, ctypes.c_int32
    if X.dtype == np.float32 and W2.dtype == np.float32:
        Xc, Wc = _c(X, np.float32), _c(W2, np.float32)
        rc = lib.orc_dense_f32(_p(Xc), I64(N), I32(D), I64(D), _p(Wc), I32(Q), _p(b), _p(out))
    elif X.dtype == np.float16 and W2.dtype == np.float16:
        Xc, Wc = _c(X, np.float16).view(np.uint16), _c(W2, np.float16).view(np.uint16)
        rc = lib.orc_dense_f16(_p(Xc), I64(N), I32(D), I64(D), _p(Wc), I32(Q), _p(b), _p(out))
    elif X.dtype == np.float16 and W2.dtype == np.float32:
        Xc, Wc = _c(X, np.float16).view(np.uint16), _c(W2, np.float32)
        rc = lib.orc_dense_f16x_f32w(_p(Xc), I64(N), I32(D), I64(D), _p(Wc), I32(Q), _p(b), _p(out))
    else:
        raise TypeError("unsupported dtype pair %s / %s" % (X.dtype, W2.dtype))
    _chk(rc, "orc_dense")
    return out


def pq_scores_reconstruct(codes, codebooks, w, bias=0.0):
    """codes (N,M) uint8; codebooks (M,K,dsub) float32; w (M*dsub,) float32 -> (N,) float64."""
    codes = _c(codes, np.uint8)
    cb = _c(codebooks, np.float32)
    w = _c(w, np.float32)
    N, M = codes.shape
    _, K, dsub = cb.shape
    assert cb.shape[0] == M and w.shape == (M * dsub,)
    out = np.empty(N, dtype=np.float64)
    rc = _load().orc_pq_scores_reconstruct(_p(codes), ctypes.c_int64(N), ctypes.c_int32(M),
                                           ctypes.c_int32(K), ctypes.c_int32(dsub), _p(cb), _p(w),
                                           ctypes.c_double(bias), _p(out))
    _chk(rc, "orc_pq_scores_reconstruct")
    return out


def pq_lut(codebooks, w):
    cb = _c(codebooks, np.float32)
    w = _c(w, np.float32)
    M, K, dsub = cb.shape
    lut = np.empty((M, K), dtype=np.float64)
    rc = _load().orc_pq_lut(_p(cb), ctypes.c_int32(M), ctypes.c_int32(K), ctypes.c_int32(dsub),
                            _p(w), _p(lut))
    _chk(rc, "orc_pq_lut")
    return lut


def pq_scores_lut(codes, lut, bias=0.0):
    codes = _c(codes, np.uint8)
    lut = _c(lut, np.float64)
    N, M = codes.shape
    K = lut.shape[1]
    assert lut.shape[0] == M
    out = np.empty(N, dtype=np.float64)
    rc = _load().orc_pq_scores_lut(_p(codes), ctypes.c_int64(N), ctypes.c_int32(M),
                                   ctypes.c_int32(K), _p(lut), ctypes.c_double(bias), _p(out))
    _chk(rc, "orc_pq_scores_lut")
    return out


def binary_scores(bits, D, w, bias=0.0):
    """bits (N, words) uint32, dimension d = bit d%32 (LSB first) of word d//32."""
    bits = _c(bits, np.uint32)
    w = _c(w, np.float32)
    N, words = bits.shape
    assert w.shape == (D,)
    out = np.empty(N, dtype=np.float64)
    rc = _load().orc_binary_scores(_p(bits), ctypes.c_int64(N), ctypes.c_int32(D),
                                   ctypes.c_int64(words), _p(w), ctypes.c_double(bias), _p(out))
    _chk(rc, "orc_binary_scores")
    return out


def hamming_scores(bits, D, query):
    """bits (N, words) uint32, query (words,) uint32 -> minus the Hamming distance of every row to the query."""
    bits = _c(bits, np.uint32)
    query = _c(query, np.uint32)
    N, words = bits.shape
    assert query.shape == (words,) and words * 32 >= D
    out = np.empty(N, dtype=np.float64)
    rc = _load().orc_hamming_scores(_p(bits), ctypes.c_int64(N), ctypes.c_int32(D), ctypes.c_int64(words),
                                    _p(query), _p(out))
    _chk(rc, "orc_hamming_scores")
    return out


def sparse_expand(mask, values, start, D):
    """mask (N, words) uint32, values (nnz,) float32, start (N+1,) int64 -> dense (N, D) float32."""
    mask = _c(mask, np.uint32)
    values = _c(values, np.float32)
    start = _c(start, np.int64)
    N, words = mask.shape
    assert start.shape == (N + 1,)
    X = np.empty((N, D), dtype=np.float32)
    rc = _load().orc_sparse_expand(_p(mask), ctypes.c_int64(words), _p(values), _p(start), ctypes.c_int64(N),
                                   ctypes.c_int32(D), _p(X))
    _chk(rc, "orc_sparse_expand")
    return X


def topk(scores, k):
    """Full sort, score descending then index ascending; returns (idx int64[k], scores f64[k])."""
    s = _c(scores, np.float64)
    N = s.shape[0]
    idx = np.empty(k, dtype=np.int64)
    val = np.empty(k, dtype=np.float64)
    rc = _load().orc_topk(_p(s), ctypes.c_int64(N), ctypes.c_int64(k), _p(idx), _p(val))
    _chk(rc, "orc_topk")
    return idx, val


def sgd_step(w, b, Xpos, idx_pos, Xneg, idx_neg, lam, t, update_bias=False):
    """One Pegasos mini-batch step; returns (w_next f64[D], b_next float, margins f64[B])."""
    w = _c(w, np.float32)
    D = w.shape[0]
    Xpos = _c(Xpos, np.float32)
    Xneg = _c(Xneg, np.float32)
    ip = _c(idx_pos, np.int32)
    ineg = _c(idx_neg, np.int32)
    w_out = np.empty(D, dtype=np.float64)
    b_out = ctypes.c_double(0.0)
    margins = np.empty(ip.shape[0] + ineg.shape[0], dtype=np.float64)
    rc = _load().orc_sgd_step(_p(w), ctypes.c_double(b), ctypes.c_int32(D),
                              _p(Xpos), ctypes.c_int64(Xpos.shape[1] if Xpos.ndim == 2 else D),
                              _p(ip), ctypes.c_int32(ip.shape[0]),
                              _p(Xneg), ctypes.c_int64(Xneg.shape[1] if Xneg.ndim == 2 else D),
                              _p(ineg), ctypes.c_int32(ineg.shape[0]),
                              ctypes.c_double(lam), ctypes.c_int64(t), ctypes.c_int32(int(update_bias)),
                              _p(w_out), ctypes.byref(b_out), _p(margins))
    _chk(rc, "orc_sgd_step")
    return w_out, float(b_out.value), margins


def svm_objective(w, b, Xpos, Xneg, lam):
    w = _c(w, np.float64)
    Xpos = _c(Xpos, np.float32)
    Xneg = _c(Xneg, np.float32)
    D = w.shape[0]
    out = ctypes.c_double(0.0)
    rc = _load().orc_svm_objective(_p(w), ctypes.c_double(b), ctypes.c_int32(D),
                                   _p(Xpos), ctypes.c_int64(D), ctypes.c_int64(Xpos.shape[0]),
                                   _p(Xneg), ctypes.c_int64(D), ctypes.c_int64(Xneg.shape[0]),
                                   ctypes.c_double(lam), ctypes.byref(out))
    _chk(rc, "orc_svm_objective")
    return float(out.value)


# ---------------------------------------------------------------------------------------
# Comparison rule used by the parity tests (not part of the method).
def score_tolerance(oracle_scores, rtol):
    """Per-element bound rtol * max(|s|, sigma) with sigma the spread of the oracle scores:
    a purely relative bound is meaningless where the sum cancels to ~0."""
    s = np.asarray(oracle_scores, dtype=np.float64)
    sigma = float(np.std(s)) if s.size > 1 else 0.0
    return rtol * np.maximum(np.abs(s), sigma)


def topk_parity_ok(oracle_all_scores, k, got_idx, got_scores, rtol):
    """Check a returned top-k list against the oracle's full score vector.

    Rules: k distinct in-range indices; returned scores non-increasing; each returned score
    within tolerance of the oracle score of that row; every oracle row clearly above the
    k-th oracle score (by more than the tolerance) is present; no returned row lies clearly
    below it.  Returns (ok, message).
    """
    s = np.asarray(oracle_all_scores, dtype=np.float64)
    got_idx = np.asarray(got_idx, dtype=np.int64)
    got_scores = np.asarray(got_scores, dtype=np.float64)
    N = s.shape[0]
    if got_idx.shape != (k,) or got_scores.shape != (k,):
        return False, "wrong output shape"
    if got_idx.min() < 0 or got_idx.max() >= N:
        return False, "index out of range"
    if np.unique(got_idx).size != k:
        return False, "duplicate indices"
    if np.any(np.diff(got_scores) > 0):
        return False, "scores not non-increasing"
    sigma = float(np.std(s)) if N > 1 else 0.0
    tol_el = rtol * np.maximum(np.abs(s[got_idx]), sigma)
    err = np.abs(got_scores - s[got_idx])
    if np.any(err > tol_el):
        j = int(np.argmax(err - tol_el))
        return False, "score mismatch at rank %d: got %r oracle %r" % (j, got_scores[j], s[got_idx[j]])
    oidx, oval = topk(s, k)
    theta = oval[-1]
    eps = rtol * max(abs(theta), sigma)
    must = np.nonzero(s > theta + eps)[0]
    missing = np.setdiff1d(must, got_idx)
    if missing.size:
        return False, "%d rows clearly above the k-th score are missing (e.g. %d)" % (missing.size, missing[0])
    if np.any(s[got_idx] < theta - eps):
        return False, "a returned row lies clearly below the k-th oracle score"
    return True, "ok"
