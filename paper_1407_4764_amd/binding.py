"""Thin ctypes binding of libotf (include/otf.h).  Argument marshalling only: every step of
the ranking path runs in the HIP kernels of the library.  torch tensors supply device memory
and the current stream; nothing here computes on them.

The library is loaded on first use.  If it is missing the call raises: there is no fallback.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libotf.so")

OTF_OK = 0
OTF_ERR_INVALID_ARG = -1
OTF_ERR_UNSUPPORTED = -2
OTF_ERR_WORKSPACE = -3
OTF_ERR_HIP = -4
OTF_F32 = 0
OTF_F16 = 1
OTF_MAX_K = 8192

EXPORTS = ["otf_status_string", "otf_workspace_bytes", "otf_rank_dense", "otf_pq_build_lut", "otf_rank_pq",
           "otf_rank_binary", "otf_topk", "otf_sgd_workspace_bytes", "otf_svm_sgd_step", "otf_svm_sgd_pass",
           "otf_tight_frame_workspace_bytes",
           "otf_tight_frame", "otf_binarize", "otf_pq_train_workspace_bytes", "otf_pq_encode", "otf_pq_lloyd_step",
           "otf_profile_begin", "otf_profile_end"]

_lib = None


class OtfError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (what, status_string(status), status))


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_1407_4764_amd.build` "
                "(the ranking path has no fallback implementation)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        L.otf_status_string.restype = ctypes.c_char_p
        L.otf_status_string.argtypes = [ctypes.c_int]
        L.otf_workspace_bytes.restype = sz
        L.otf_workspace_bytes.argtypes = [i64, i32, i32]
        L.otf_sgd_workspace_bytes.restype = sz
        L.otf_sgd_workspace_bytes.argtypes = [i32]
        L.otf_rank_dense.restype = ctypes.c_int
        L.otf_rank_dense.argtypes = [vp, ctypes.c_int, i64, i32, i64, vp, ctypes.c_int, i32, vp, i32, vp, vp, vp,
                                     vp, sz, vp]
        L.otf_pq_build_lut.restype = ctypes.c_int
        L.otf_pq_build_lut.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        L.otf_rank_pq.restype = ctypes.c_int
        L.otf_rank_pq.argtypes = [vp, i64, i32, i32, vp, f32, i32, vp, vp, vp, vp, sz, vp]
        L.otf_rank_binary.restype = ctypes.c_int
        L.otf_rank_binary.argtypes = [vp, i64, i32, vp, f32, i32, vp, vp, vp, vp, sz, vp]
        L.otf_topk.restype = ctypes.c_int
        L.otf_topk.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, sz, vp]
        L.otf_svm_sgd_step.restype = ctypes.c_int
        L.otf_svm_sgd_step.argtypes = [vp, vp, i32, vp, i64, vp, i32, vp, i64, vp, i32, f32, i64, i32, vp, sz, vp]
        L.otf_svm_sgd_pass.restype = ctypes.c_int
        L.otf_svm_sgd_pass.argtypes = [vp, vp, i32, vp, i64, vp, i32, vp, i64, vp, i32, f32, i64, i32, i32, vp, sz, vp]
        L.otf_tight_frame_workspace_bytes.restype = sz
        L.otf_tight_frame_workspace_bytes.argtypes = [i32, i32]
        L.otf_tight_frame.restype = ctypes.c_int
        L.otf_tight_frame.argtypes = [vp, i32, i32, vp, vp, sz, vp]
        L.otf_binarize.restype = ctypes.c_int
        L.otf_binarize.argtypes = [vp, i64, i32, i64, vp, i32, vp, vp]
        L.otf_pq_train_workspace_bytes.restype = sz
        L.otf_pq_train_workspace_bytes.argtypes = [i32, i32]
        L.otf_pq_encode.restype = ctypes.c_int
        L.otf_pq_encode.argtypes = [vp, i64, i64, vp, i32, i32, i32, vp, vp, sz, vp]
        L.otf_pq_lloyd_step.restype = ctypes.c_int
        L.otf_pq_lloyd_step.argtypes = [vp, i64, i64, vp, i32, i32, i32, vp, vp, vp, sz, vp]
        L.otf_profile_begin.restype = ctypes.c_int
        L.otf_profile_begin.argtypes = [i32]
        L.otf_profile_end.restype = ctypes.c_int
        L.otf_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
        _lib = L
    return _lib


def status_string(status):
    return lib().otf_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(device):
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return OTF_F32
    if t.dtype == torch.float16:
        return OTF_F16
    raise TypeError("unsupported dtype %s" % t.dtype)


def workspace_bytes(N, k, Q=1):
    return int(lib().otf_workspace_bytes(int(N), int(k), int(Q)))


def make_workspace(N, k, Q=1, device="cuda"):
    n = workspace_bytes(N, k, Q)
    if n == 0:
        raise OtfError(OTF_ERR_INVALID_ARG, "otf_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _outputs(Q, k, device):
    return (torch.empty((Q, k), dtype=torch.float32, device=device),
            torch.empty((Q, k), dtype=torch.int32, device=device))


def rank_dense(X, W, bias, k, ws, all_scores=None, out=None):
    """X (N,D) fp32/fp16 with row stride X.stride(0); W (Q,D) or (D,); bias (Q,) fp32 tensor or
    None.  Returns (scores (Q,k) fp32, idx (Q,k) int32) on X's device, valid after a stream sync."""
    W2 = W if W.dim() == 2 else W.unsqueeze(0)
    assert X.dim() == 2 and X.stride(1) == 1 and W2.is_contiguous()
    N, D = X.shape
    Q = W2.shape[0]
    out_s, out_i = out if out is not None else _outputs(Q, k, X.device)
    rc = lib().otf_rank_dense(_ptr(X), _dtype_code(X), N, D, X.stride(0), _ptr(W2), _dtype_code(W2), Q, _ptr(bias),
                              k, _ptr(out_s), _ptr(out_i), _ptr(all_scores), _ptr(ws), ws.numel(), _stream(X.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_dense")
    return out_s, out_i


def pq_build_lut(codebooks, w, lut=None):
    assert codebooks.is_contiguous() and w.is_contiguous()
    M, K, dsub = codebooks.shape
    if lut is None:
        lut = torch.empty((M, K), dtype=torch.float32, device=codebooks.device)
    rc = lib().otf_pq_build_lut(_ptr(codebooks), M, K, dsub, _ptr(w), _ptr(lut), _stream(codebooks.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_pq_build_lut")
    return lut


def rank_pq(codes, lut, bias, k, ws, all_scores=None, out=None):
    assert codes.is_contiguous() and lut.is_contiguous()
    N, M = codes.shape
    K = lut.shape[1]
    out_s, out_i = out if out is not None else _outputs(1, k, codes.device)
    rc = lib().otf_rank_pq(_ptr(codes), N, M, K, _ptr(lut), float(bias), k, _ptr(out_s), _ptr(out_i),
                           _ptr(all_scores), _ptr(ws), ws.numel(), _stream(codes.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_pq")
    return out_s, out_i


def rank_binary(bits, D, w, bias, k, ws, all_scores=None, out=None):
    """bits (N, D/32) int32 tensor holding the packed words."""
    assert bits.is_contiguous() and w.is_contiguous()
    N = bits.shape[0]
    out_s, out_i = out if out is not None else _outputs(1, k, bits.device)
    rc = lib().otf_rank_binary(_ptr(bits), N, D, _ptr(w), float(bias), k, _ptr(out_s), _ptr(out_i),
                               _ptr(all_scores), _ptr(ws), ws.numel(), _stream(bits.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_binary")
    return out_s, out_i


def topk(scores, k, ws, out=None):
    S = scores if scores.dim() == 2 else scores.unsqueeze(0)
    assert S.stride(1) == 1
    Q, N = S.shape
    out_s, out_i = out if out is not None else _outputs(Q, k, S.device)
    rc = lib().otf_topk(_ptr(S), N, S.stride(0) if Q > 1 else N, Q, k, _ptr(out_s), _ptr(out_i), _ptr(ws),
                        ws.numel(), _stream(S.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_topk")
    return out_s, out_i


def sgd_workspace(B, device="cuda"):
    n = int(lib().otf_sgd_workspace_bytes(int(B)))
    if n == 0:
        raise OtfError(OTF_ERR_INVALID_ARG, "otf_sgd_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def svm_sgd_step(w, b, Xpos, idx_pos, Xneg, idx_neg, lam, t, update_bias, ws):
    """Updates w (D,) fp32 and b (1,) fp32 (or None) in place on the current stream."""
    D = w.shape[0]
    n_pos = 0 if idx_pos is None else idx_pos.numel()
    n_neg = 0 if idx_neg is None else idx_neg.numel()
    rc = lib().otf_svm_sgd_step(_ptr(w), _ptr(b), D, _ptr(Xpos), 0 if Xpos is None else Xpos.stride(0),
                                _ptr(idx_pos), n_pos, _ptr(Xneg), 0 if Xneg is None else Xneg.stride(0),
                                _ptr(idx_neg), n_neg, float(lam), int(t), int(bool(update_bias)), _ptr(ws),
                                ws.numel(), _stream(w.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_svm_sgd_step")


def svm_sgd_pass(w, b, Xpos, idx_pos, Xneg, idx_neg, lam, t_first, update_bias, ws):
    """idx_pos, idx_neg: contiguous int32 (steps, half) tensors; runs the steps t_first, t_first + 1, ..."""
    assert idx_pos.is_contiguous() and idx_neg.is_contiguous() and idx_pos.shape[0] == idx_neg.shape[0]
    rc = lib().otf_svm_sgd_pass(_ptr(w), _ptr(b), w.shape[0], _ptr(Xpos), Xpos.stride(0), _ptr(idx_pos),
                                idx_pos.shape[1], _ptr(Xneg), Xneg.stride(0), _ptr(idx_neg), idx_neg.shape[1],
                                float(lam), int(t_first), idx_pos.shape[0], int(bool(update_bias)), _ptr(ws),
                                ws.numel(), _stream(w.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_svm_sgd_pass")


def tight_frame(G, m, U=None):
    """U (n, m) fp32: the frame of the binarisation encoder from the random matrix G (n, n) fp32."""
    assert G.is_contiguous() and G.dtype == torch.float32 and G.shape[0] == G.shape[1]
    n = G.shape[0]
    if U is None:
        U = torch.empty((n, m), dtype=torch.float32, device=G.device)
    nbytes = int(lib().otf_tight_frame_workspace_bytes(n, int(m)))
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=G.device)
    rc = lib().otf_tight_frame(_ptr(G), n, int(m), _ptr(U), _ptr(ws), ws.numel(), _stream(G.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_tight_frame")
    torch.cuda.current_stream(G.device).synchronize()      # ws is released on return
    return U


def binarize(phi, U, bits=None):
    """bits (N, n/32) int32 (the uint32 words of the codes): sign of U phi, packed LSB first."""
    assert phi.dtype == torch.float32 and U.dtype == torch.float32 and U.is_contiguous() and phi.stride(1) == 1
    N, m = phi.shape
    n = U.shape[0]
    assert U.shape[1] == m
    if bits is None:
        bits = torch.empty((N, n // 32), dtype=torch.int32, device=phi.device)
    rc = lib().otf_binarize(_ptr(phi), N, m, phi.stride(0), _ptr(U), n, _ptr(bits), _stream(phi.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_binarize")
    return bits


def pq_train_workspace(M, dsub, device="cuda"):
    n = int(lib().otf_pq_train_workspace_bytes(int(M), int(dsub)))
    if n == 0:
        raise OtfError(OTF_ERR_INVALID_ARG, "otf_pq_train_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def pq_encode(X, codebooks, ws, codes=None):
    """codes (N, M) uint8: nearest centre of every sub-block.  X (N, M*dsub) fp32, codebooks (M, 256, dsub)."""
    assert X.dtype == torch.float32 and X.stride(1) == 1 and codebooks.is_contiguous()
    M, K, dsub = codebooks.shape
    N = X.shape[0]
    if codes is None:
        codes = torch.empty((N, M), dtype=torch.uint8, device=X.device)
    rc = lib().otf_pq_encode(_ptr(X), N, X.stride(0), _ptr(codebooks), M, K, dsub, _ptr(codes), _ptr(ws), ws.numel(),
                             _stream(X.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_pq_encode")
    return codes


def pq_lloyd_step(X, codebooks, ws, codes=None, distortion=None):
    """One k-means iteration; codebooks is updated in place.  Returns (codes, distortion (1,) float64 tensor)."""
    assert X.dtype == torch.float32 and X.stride(1) == 1 and codebooks.is_contiguous()
    M, K, dsub = codebooks.shape
    N = X.shape[0]
    if codes is None:
        codes = torch.empty((N, M), dtype=torch.uint8, device=X.device)
    if distortion is None:
        distortion = torch.zeros(1, dtype=torch.float64, device=X.device)
    rc = lib().otf_pq_lloyd_step(_ptr(X), N, X.stride(0), _ptr(codebooks), M, K, dsub, _ptr(codes), _ptr(distortion),
                                 _ptr(ws), ws.numel(), _stream(X.device))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_pq_lloyd_step")
    return codes, distortion


def debug_fallback_taken(ws):
    """True if the last ranking call on this workspace abandoned its filtered scan and redid the
    ranking by full selection (reads the flag the kernels leave in the workspace; test use only)."""
    torch.cuda.synchronize()
    return int(ws[60:64].view(torch.int32).item()) != 0


def profile_begin(max_records):
    rc = lib().otf_profile_begin(int(max_records))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_profile_begin")


def profile_end():
    """Returns (summed scoring-kernel milliseconds, number of ranking calls recorded)."""
    total = ctypes.c_double(0.0)
    n = ctypes.c_int32(0)
    rc = lib().otf_profile_end(ctypes.byref(total), ctypes.byref(n))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_profile_end")
    return float(total.value), int(n.value)
