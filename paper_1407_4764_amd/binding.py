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
OTF_ERR_SCRATCH = -5
OTF_NOALLOC_SCRATCH_BYTES = 16 << 20
OTF_F32 = 0
OTF_F16 = 1
OTF_MAX_K = 8192

EXPORTS = ["otf_status_string", "otf_workspace_bytes", "otf_rank_dense", "otf_pq_build_lut", "otf_rank_pq",
           "otf_rank_binary", "otf_topk", "otf_sgd_workspace_bytes", "otf_svm_sgd_step", "otf_svm_sgd_pass",
           "otf_tight_frame_workspace_bytes",
           "otf_tight_frame", "otf_binarize", "otf_pq_train_workspace_bytes", "otf_pq_encode", "otf_pq_lloyd_step",
           "otf_profile_begin", "otf_profile_end", "otf_debug_set", "otf_rank_dense_noalloc", "otf_rank_pq_model", "otf_rank_hamming", "otf_rank_sparse", "otf_check_indices"]

# otf_debug_key
(DEBUG_RANK_PATH, DEBUG_BINARIZE_FP32, DEBUG_PQENC_FP32, DEBUG_SCAN_THREADS, DEBUG_SCAN_UNROLL, DEBUG_BINARIZE_WAVES,
 DEBUG_PQENC_RANGE, DEBUG_DENSE_BLOCKS_PER_CU, DEBUG_NARROW_BLOCKS_PER_CU, DEBUG_MFMA_BLOCKS_PER_CU,
 DEBUG_PQENC_BLOCKS_PER_CU, DEBUG_WALK_TILES, DEBUG_SGD_PASS_PATH, DEBUG_SGD_SPIN_LIMIT, DEBUG_MEET_SPIN_LIMIT,
 DEBUG_KEYS) = range(16)

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
        L.otf_rank_dense_noalloc.restype = ctypes.c_int
        L.otf_rank_dense_noalloc.argtypes = [vp, ctypes.c_int, i64, i32, i64, vp, ctypes.c_int, i32, vp, i32, vp, vp, vp,
                                             vp]
        L.otf_pq_build_lut.restype = ctypes.c_int
        L.otf_pq_build_lut.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        L.otf_rank_pq.restype = ctypes.c_int
        L.otf_rank_pq.argtypes = [vp, i64, i32, i32, vp, f32, i32, vp, vp, vp, vp, sz, vp]
        L.otf_rank_pq_model.restype = ctypes.c_int
        L.otf_rank_pq_model.argtypes = [vp, i64, i32, i32, i32, vp, vp, f32, i32, vp, vp, vp, vp, sz, vp]
        L.otf_rank_binary.restype = ctypes.c_int
        L.otf_rank_binary.argtypes = [vp, i64, i32, vp, f32, i32, vp, vp, vp, vp, sz, vp]
        L.otf_rank_sparse.restype = ctypes.c_int
        L.otf_rank_sparse.argtypes = [vp, vp, i64, i32, vp, f32, i32, vp, vp, vp, vp, sz, vp]
        L.otf_rank_hamming.restype = ctypes.c_int
        L.otf_rank_hamming.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp, sz, vp]
        L.otf_topk.restype = ctypes.c_int
        L.otf_topk.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, sz, vp]
        L.otf_svm_sgd_step.restype = ctypes.c_int
        L.otf_svm_sgd_step.argtypes = [vp, vp, i32, vp, i64, vp, i32, vp, i64, vp, i32, f32, i64, i32, vp, sz, vp]
        L.otf_svm_sgd_pass.restype = ctypes.c_int
        L.otf_svm_sgd_pass.argtypes = [vp, vp, i32, vp, i64, vp, i32, vp, i64, vp, i32, f32, i64, i32, i32, vp, sz, vp]
        L.otf_check_indices.restype = ctypes.c_int
        L.otf_check_indices.argtypes = [vp, i64, i64, vp, vp]
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
        L.otf_debug_set.restype = ctypes.c_int
        L.otf_debug_set.argtypes = [ctypes.c_int, ctypes.c_int]
        _lib = L
    return _lib


def status_string(status):
    return lib().otf_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


class _Args:
    """The C ABI sees addresses only; this layer sees the tensors, so dtype, size, layout and
    device of every tensor of a call are checked here, before the call: a wrong dtype would be
    read as garbage and a short buffer overrun on the device.  Type, shape and size errors are
    raised as they are met; done() then requires every tensor to live on one GPU."""

    def __init__(self):
        self.seen = []

    def check(self, t, name, dtypes, numel=None, shape=None, contiguous=True, optional=False):
        if t is None:
            if optional:
                return
            raise TypeError("%s is required" % name)
        if not isinstance(t, torch.Tensor):
            raise TypeError("%s must be a torch tensor" % name)
        dtypes = dtypes if isinstance(dtypes, (tuple, list)) else (dtypes,)
        if t.dtype not in dtypes:
            raise TypeError("%s must have dtype %s, not %s" % (name, " or ".join(str(d) for d in dtypes), t.dtype))
        if shape is not None and tuple(t.shape) != tuple(shape):
            raise ValueError("%s must have shape %s, not %s" % (name, tuple(shape), tuple(t.shape)))
        if numel is not None and t.numel() < numel:
            raise ValueError("%s holds %d elements, the call needs %d" % (name, t.numel(), numel))
        if contiguous and not t.is_contiguous():
            raise ValueError("%s must be contiguous" % name)
        self.seen.append((name, t))

    def rows(self, t, name, dtypes):
        """A 2-D row-major matrix whose rows may be padded (stride(1) == 1, stride(0) >= columns)."""
        self.check(t, name, dtypes, contiguous=False)
        if t.dim() != 2 or t.stride(1) != 1 or t.stride(0) < t.shape[1]:
            raise ValueError("%s must be a 2-D tensor with unit column stride" % name)

    def rank_buffers(self, Q, N, k, ws, all_scores, out):
        if int(k) < 1:
            raise ValueError("k must be at least 1")
        if ws is not _NO_WS:
            self.check(ws, "ws", torch.uint8, numel=workspace_bytes(N, k, Q))
        self.check(all_scores, "all_scores", torch.float32, numel=Q * N, optional=True)
        if all_scores is not None and all_scores.numel() != Q * N:
            raise ValueError("all_scores must hold exactly Q * N = %d floats" % (Q * N))
        if out is not None:
            self.check(out[0], "out scores", torch.float32, numel=Q * k)
            self.check(out[1], "out indices", torch.int32, numel=Q * k)

    def done(self):
        dev = None
        for name, t in self.seen:
            if not t.is_cuda:
                raise ValueError("%s must live in GPU memory" % name)
            if dev is None:
                dev = t.device
            elif t.device != dev:
                raise ValueError("%s is on %s, the call runs on %s" % (name, t.device, dev))
        return dev


_NO_WS = object()


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


def _dense_args(X, W, bias, k, ws, all_scores, out):
    a = _Args()
    a.rows(X, "X", (torch.float32, torch.float16))
    a.check(W, "W", (torch.float32, torch.float16))
    W2 = W if W.dim() == 2 else W.unsqueeze(0)
    N, D = X.shape
    if W2.dim() != 2 or W2.shape[1] != D:
        raise ValueError("W must be (Q, %d) or (%d,)" % (D, D))
    Q = W2.shape[0]
    a.check(bias, "bias", torch.float32, numel=Q, optional=True)
    a.rank_buffers(Q, N, k, ws, all_scores, out)
    return a.done(), W2, N, D, Q


def rank_dense(X, W, bias, k, ws, all_scores=None, out=None):
    """X (N,D) fp32/fp16 with row stride X.stride(0); W (Q,D) or (D,); bias (Q,) fp32 tensor or
    None.  Returns (scores (Q,k) fp32, idx (Q,k) int32) on X's device, valid after a stream sync."""
    dev, W2, N, D, Q = _dense_args(X, W, bias, k, ws, all_scores, out)
    out_s, out_i = out if out is not None else _outputs(Q, k, dev)
    rc = lib().otf_rank_dense(_ptr(X), _dtype_code(X), N, D, X.stride(0), _ptr(W2), _dtype_code(W2), Q, _ptr(bias),
                              k, _ptr(out_s), _ptr(out_i), _ptr(all_scores), _ptr(ws), ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_dense")
    return out_s, out_i


def rank_dense_noalloc(X, W, bias, k, out, all_scores=None):
    """rank_dense on the library's own scratch: no workspace, and nothing is allocated here either,
    so the caller supplies the outputs out = (scores (Q,k) fp32, idx (Q,k) int32)."""
    dev, W2, N, D, Q = _dense_args(X, W, bias, k, _NO_WS, all_scores, out)
    rc = lib().otf_rank_dense_noalloc(_ptr(X), _dtype_code(X), N, D, X.stride(0), _ptr(W2), _dtype_code(W2), Q,
                                      _ptr(bias), k, _ptr(out[0]), _ptr(out[1]), _ptr(all_scores), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_dense_noalloc")
    return out


def pq_build_lut(codebooks, w, lut=None):
    a = _Args()
    a.check(codebooks, "codebooks", torch.float32)
    if codebooks.dim() != 3:
        raise ValueError("codebooks must be (M, K, dsub)")
    M, K, dsub = codebooks.shape
    a.check(w, "w", torch.float32, numel=M * dsub)
    a.check(lut, "lut", torch.float32, numel=M * K, optional=True)
    dev = a.done()
    if lut is None:
        lut = torch.empty((M, K), dtype=torch.float32, device=dev)
    rc = lib().otf_pq_build_lut(_ptr(codebooks), M, K, dsub, _ptr(w), _ptr(lut), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_pq_build_lut")
    return lut


def rank_pq(codes, lut, bias, k, ws, all_scores=None, out=None):
    a = _Args()
    a.check(codes, "codes", torch.uint8)
    if codes.dim() != 2:
        raise ValueError("codes must be (N, M)")
    N, M = codes.shape
    a.check(lut, "lut", torch.float32)
    if lut.dim() != 2 or lut.shape[0] != M:
        raise ValueError("lut must be (%d, K)" % M)
    K = lut.shape[1]
    a.rank_buffers(1, N, k, ws, all_scores, out)
    dev = a.done()
    out_s, out_i = out if out is not None else _outputs(1, k, dev)
    rc = lib().otf_rank_pq(_ptr(codes), N, M, K, _ptr(lut), float(bias), k, _ptr(out_s), _ptr(out_i),
                           _ptr(all_scores), _ptr(ws), ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_pq")
    return out_s, out_i


def rank_pq_model(codes, codebooks, w, bias, k, ws, all_scores=None, out=None):
    """Table build and ranking in one call: codes (N, M) uint8, codebooks (M, 256, dsub) fp32, w (M*dsub,) fp32."""
    a = _Args()
    a.check(codes, "codes", torch.uint8)
    a.check(codebooks, "codebooks", torch.float32)
    if codes.dim() != 2 or codebooks.dim() != 3 or codebooks.shape[0] != codes.shape[1]:
        raise ValueError("codes must be (N, M) and codebooks (M, K, dsub)")
    N, M = codes.shape
    _, K, dsub = codebooks.shape
    a.check(w, "w", torch.float32, numel=M * dsub)
    a.rank_buffers(1, N, k, ws, all_scores, out)
    dev = a.done()
    out_s, out_i = out if out is not None else _outputs(1, k, dev)
    rc = lib().otf_rank_pq_model(_ptr(codes), N, M, K, dsub, _ptr(codebooks), _ptr(w), float(bias), k, _ptr(out_s),
                                 _ptr(out_i), _ptr(all_scores), _ptr(ws), ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_pq_model")
    return out_s, out_i


def rank_binary(bits, D, w, bias, k, ws, all_scores=None, out=None):
    """bits (N, D/32) int32 tensor holding the packed words."""
    a = _Args()
    a.check(bits, "bits", torch.int32)
    if bits.dim() != 2 or bits.shape[1] * 32 != int(D):
        raise ValueError("bits must be (N, D/32)")
    N = bits.shape[0]
    a.check(w, "w", torch.float32, numel=int(D))
    a.rank_buffers(1, N, k, ws, all_scores, out)
    dev = a.done()
    out_s, out_i = out if out is not None else _outputs(1, k, dev)
    rc = lib().otf_rank_binary(_ptr(bits), N, D, _ptr(w), float(bias), k, _ptr(out_s), _ptr(out_i),
                               _ptr(all_scores), _ptr(ws), ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_binary")
    return out_s, out_i


def rank_sparse(rows, start, D, w, bias, k, ws, all_scores=None, out=None):
    """rows: int32 words of the sparse-row store (padded to a multiple of 4), start (N+1,) int64 word offsets."""
    a = _Args()
    a.check(rows, "rows", torch.int32)
    a.check(start, "start", torch.int64)
    if start.dim() != 1 or start.numel() < 2 or rows.numel() % 4:
        raise ValueError("start must be (N+1,) and rows a multiple of 4 words long")
    N = start.numel() - 1
    a.check(w, "w", torch.float32, numel=int(D))
    a.rank_buffers(1, N, k, ws, all_scores, out)
    dev = a.done()
    out_s, out_i = out if out is not None else _outputs(1, k, dev)
    rc = lib().otf_rank_sparse(_ptr(rows), _ptr(start), N, int(D), _ptr(w), float(bias), k, _ptr(out_s), _ptr(out_i),
                               _ptr(all_scores), _ptr(ws), ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_sparse")
    return out_s, out_i


def rank_hamming(bits, D, query, k, ws, all_scores=None, out=None):
    """bits (N, D/32) int32 words, query (D/32,) int32 words; scores are minus the Hamming distances."""
    a = _Args()
    a.check(bits, "bits", torch.int32)
    if bits.dim() != 2 or bits.shape[1] * 32 != int(D):
        raise ValueError("bits must be (N, D/32)")
    N = bits.shape[0]
    a.check(query, "query", torch.int32, shape=(int(D) // 32,))
    a.rank_buffers(1, N, k, ws, all_scores, out)
    dev = a.done()
    out_s, out_i = out if out is not None else _outputs(1, k, dev)
    rc = lib().otf_rank_hamming(_ptr(bits), N, D, _ptr(query), k, _ptr(out_s), _ptr(out_i), _ptr(all_scores),
                                _ptr(ws), ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_rank_hamming")
    return out_s, out_i


def topk(scores, k, ws, out=None):
    a = _Args()
    a.check(scores, "scores", torch.float32, contiguous=False)
    S = scores if scores.dim() == 2 else scores.unsqueeze(0)
    if S.dim() != 2 or S.stride(1) != 1 or (S.shape[0] > 1 and S.stride(0) < S.shape[1]):
        raise ValueError("scores must be (N,) or (Q, N) with unit column stride")
    Q, N = S.shape
    a.rank_buffers(Q, N, k, ws, None, out)
    dev = a.done()
    out_s, out_i = out if out is not None else _outputs(Q, k, dev)
    rc = lib().otf_topk(_ptr(S), N, S.stride(0) if Q > 1 else N, Q, k, _ptr(out_s), _ptr(out_i), _ptr(ws),
                        ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_topk")
    return out_s, out_i


def sgd_workspace(B, device="cuda"):
    n = int(lib().otf_sgd_workspace_bytes(int(B)))
    if n == 0:
        raise OtfError(OTF_ERR_INVALID_ARG, "otf_sgd_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _sgd_args(w, b, Xpos, idx_pos, Xneg, idx_neg, B, ws):
    a = _Args()
    a.check(w, "w", torch.float32)
    if w.dim() != 1:
        raise ValueError("w must be (D,)")
    a.check(b, "b", torch.float32, numel=1, optional=True)
    for X, idx, name in ((Xpos, idx_pos, "pos"), (Xneg, idx_neg, "neg")):
        if idx is None:
            continue
        # row numbers are read as int32 on the device: an int64 tensor would be read as pairs
        a.check(idx, "idx_" + name, torch.int32)
        a.rows(X, "X" + name, torch.float32)
        if X.shape[1] != w.shape[0]:
            raise ValueError("X%s has %d columns, w has %d" % (name, X.shape[1], w.shape[0]))
    if B >= 1:
        a.check(ws, "ws", torch.uint8, numel=int(lib().otf_sgd_workspace_bytes(int(B))))
    return a.done()


def svm_sgd_step(w, b, Xpos, idx_pos, Xneg, idx_neg, lam, t, update_bias, ws):
    """Updates w (D,) fp32 and b (1,) fp32 (or None) in place on the current stream."""
    n_pos = 0 if idx_pos is None else idx_pos.numel()
    n_neg = 0 if idx_neg is None else idx_neg.numel()
    dev = _sgd_args(w, b, Xpos, idx_pos, Xneg, idx_neg, n_pos + n_neg, ws)
    rc = lib().otf_svm_sgd_step(_ptr(w), _ptr(b), w.shape[0], _ptr(Xpos), 0 if Xpos is None else Xpos.stride(0),
                                _ptr(idx_pos), n_pos, _ptr(Xneg), 0 if Xneg is None else Xneg.stride(0),
                                _ptr(idx_neg), n_neg, float(lam), int(t), int(bool(update_bias)), _ptr(ws),
                                ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_svm_sgd_step")


def svm_sgd_pass(w, b, Xpos, idx_pos, Xneg, idx_neg, lam, t_first, update_bias, ws):
    """idx_pos, idx_neg: contiguous int32 (steps, half) tensors; runs the steps t_first, t_first + 1, ..."""
    for idx, name in ((idx_pos, "idx_pos"), (idx_neg, "idx_neg")):
        if not isinstance(idx, torch.Tensor) or idx.dtype != torch.int32:
            raise TypeError("%s must be an int32 tensor" % name)
    if idx_pos.dim() != 2 or idx_neg.dim() != 2 or idx_pos.shape[0] != idx_neg.shape[0]:
        raise ValueError("idx_pos and idx_neg must be (steps, n_pos) and (steps, n_neg)")
    dev = _sgd_args(w, b, Xpos, idx_pos, Xneg, idx_neg, idx_pos.shape[1] + idx_neg.shape[1], ws)
    rc = lib().otf_svm_sgd_pass(_ptr(w), _ptr(b), w.shape[0], _ptr(Xpos), Xpos.stride(0), _ptr(idx_pos),
                                idx_pos.shape[1], _ptr(Xneg), Xneg.stride(0), _ptr(idx_neg), idx_neg.shape[1],
                                float(lam), int(t_first), idx_pos.shape[0], int(bool(update_bias)), _ptr(ws),
                                ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_svm_sgd_pass")


def sgd_pass_status(ws):
    """0 after a complete svm_sgd_pass on this workspace, 1 if one of its bounded waits expired (synchronises)."""
    torch.cuda.synchronize()
    return int(ws[0:4].view(torch.int32).item())


def check_indices(idx, rows):
    """Raises IndexError if any entry of the int32 device tensor idx is not a row number of a pool of
    `rows` rows (synchronises: for use where the batches are built, not in the loop)."""
    a = _Args()
    a.check(idx, "idx", torch.int32)
    dev = a.done()
    bad = torch.zeros(1, dtype=torch.int32, device=dev)
    rc = lib().otf_check_indices(_ptr(idx), idx.numel(), int(rows), _ptr(bad), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_check_indices")
    n = int(bad.item())
    if n:
        raise IndexError("%d of %d row numbers lie outside the pool of %d rows" % (n, idx.numel(), rows))


def tight_frame(G, m, U=None):
    """U (n, m) fp32: the frame of the binarisation encoder from the random matrix G (n, n) fp32."""
    a = _Args()
    a.check(G, "G", torch.float32)
    if G.dim() != 2 or G.shape[0] != G.shape[1]:
        raise ValueError("G must be square")
    n = G.shape[0]
    a.check(U, "U", torch.float32, shape=(n, int(m)), optional=True)
    dev = a.done()
    if U is None:
        U = torch.empty((n, m), dtype=torch.float32, device=dev)
    nbytes = int(lib().otf_tight_frame_workspace_bytes(n, int(m)))
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=dev)
    rc = lib().otf_tight_frame(_ptr(G), n, int(m), _ptr(U), _ptr(ws), ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_tight_frame")
    torch.cuda.current_stream(dev).synchronize()      # ws is released on return
    return U


def binarize(phi, U, bits=None):
    """bits (N, n/32) int32 (the uint32 words of the codes): sign of U phi, packed LSB first."""
    a = _Args()
    a.rows(phi, "phi", torch.float32)
    N, m = phi.shape
    a.check(U, "U", torch.float32)
    if U.dim() != 2 or U.shape[1] != m or U.shape[0] % 32:
        raise ValueError("U must be (n, %d) with n a multiple of 32" % m)
    n = U.shape[0]
    a.check(bits, "bits", torch.int32, shape=(N, n // 32), optional=True)
    dev = a.done()
    if bits is None:
        bits = torch.empty((N, n // 32), dtype=torch.int32, device=dev)
    rc = lib().otf_binarize(_ptr(phi), N, m, phi.stride(0), _ptr(U), n, _ptr(bits), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_binarize")
    return bits


def pq_train_workspace(M, dsub, device="cuda"):
    n = int(lib().otf_pq_train_workspace_bytes(int(M), int(dsub)))
    if n == 0:
        raise OtfError(OTF_ERR_INVALID_ARG, "otf_pq_train_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _pq_train_args(X, codebooks, ws, codes, distortion=None):
    a = _Args()
    a.rows(X, "X", torch.float32)
    a.check(codebooks, "codebooks", torch.float32)
    if codebooks.dim() != 3 or codebooks.shape[0] * codebooks.shape[2] != X.shape[1]:
        raise ValueError("codebooks must be (M, K, dsub) with M * dsub = %d" % X.shape[1])
    M, K, dsub = codebooks.shape
    a.check(ws, "ws", torch.uint8, numel=int(lib().otf_pq_train_workspace_bytes(int(M), int(dsub))))
    a.check(codes, "codes", torch.uint8, shape=(X.shape[0], M), optional=True)
    a.check(distortion, "distortion", torch.float64, numel=1, optional=True)
    return a.done(), M, K, dsub, X.shape[0]


def pq_encode(X, codebooks, ws, codes=None):
    """codes (N, M) uint8: nearest centre of every sub-block.  X (N, M*dsub) fp32, codebooks (M, 256, dsub)."""
    dev, M, K, dsub, N = _pq_train_args(X, codebooks, ws, codes)
    if codes is None:
        codes = torch.empty((N, M), dtype=torch.uint8, device=dev)
    rc = lib().otf_pq_encode(_ptr(X), N, X.stride(0), _ptr(codebooks), M, K, dsub, _ptr(codes), _ptr(ws), ws.numel(),
                             _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_pq_encode")
    return codes


def pq_lloyd_step(X, codebooks, ws, codes=None, distortion=None):
    """One k-means iteration; codebooks is updated in place.  Returns (codes, distortion (1,) float64 tensor)."""
    dev, M, K, dsub, N = _pq_train_args(X, codebooks, ws, codes, distortion)
    if codes is None:
        codes = torch.empty((N, M), dtype=torch.uint8, device=dev)
    if distortion is None:
        distortion = torch.zeros(1, dtype=torch.float64, device=dev)
    rc = lib().otf_pq_lloyd_step(_ptr(X), N, X.stride(0), _ptr(codebooks), M, K, dsub, _ptr(codes), _ptr(distortion),
                                 _ptr(ws), ws.numel(), _stream(dev))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_pq_lloyd_step")
    return codes, distortion


def debug_fallback_taken(ws):
    """True if the last ranking call on this workspace abandoned its filtered scan and redid the
    ranking by full selection (reads the flag the kernels leave in the workspace; test use only)."""
    torch.cuda.synchronize()
    return int(ws[60:64].view(torch.int32).item()) != 0


def debug_set(key, value):
    """Sets one of the library's diagnostic switches (DEBUG_*); 0 clears it."""
    rc = lib().otf_debug_set(int(key), int(value))
    if rc != OTF_OK:
        raise OtfError(rc, "otf_debug_set")


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
