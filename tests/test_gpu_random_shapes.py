"""GPU parity on randomly drawn valid configurations of every ranking call: store kind, rows (one to
1.3 million, so that both the full selection and the filtered route are taken), row length, list
length, padding between rows, bias, score output on or off.  Seeded, so every run draws the same
configurations; each is compared with the oracle under the parity rule of its store (Hamming
distances and otf_topk exactly)."""
import numpy as np
import pytest
import torch

from oracle import otf_oracle as orc
from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _rows(rng):
    u = rng.random()
    if u < 0.7:
        return int(rng.integers(1, 5000))
    if u < 0.95:
        return int(rng.integers(5000, 300000))
    return int(rng.integers(1 << 20, (1 << 20) + 300000))            # the filtered route


def _list_length(rng, N):
    u = rng.random()
    if u < 0.2:
        return 1
    if u < 0.3:
        return min(N, 8192)
    if u < 0.4:
        return min(N, 1024)
    return int(rng.integers(1, min(N, 2000) + 1))


def _check(ref, val, idx, k, rtol, what, exact=False):
    val, idx = val.cpu().numpy(), idx.cpu().numpy()
    if exact:
        i, v = orc.topk(ref, k)
        assert np.array_equal(idx, i) and np.array_equal(val.astype(np.float64), v), what
    else:
        ok, msg = orc.topk_parity_ok(ref, k, idx, val, rtol)
        assert ok, what + ": " + msg


def _dense(rng, N, k, seed, want_all, half):
    D = int(rng.choice([8, 16, 24, 64, 128, 136, 256, 512, 520, 1024, 2048, 2056, 4096] if N < 300000 else [8, 64, 128, 256]))
    if half:
        D = (D + 7) // 8 * 8
    N = min(N, int(6e8 // D))
    k = min(k, N)
    pad = int(rng.choice([0, 8, 64]))
    what = "dense half=%s N=%d D=%d k=%d pad=%d scores=%s seed=%d" % (half, N, D, k, pad, want_all, seed)
    rtol = 2e-3 if half else 1e-4
    X = synth.dense_features(N, D, seed, dtype=torch.float16 if half else torch.float32)
    wide = torch.zeros((N, D + pad), dtype=X.dtype)
    wide[:, :D] = X
    w = synth.normal_vector(D, 1.0, seed + 1)
    b = synth.normal_vector(1, 1.0, seed + 2)
    scores = torch.empty(N, device=DEV) if want_all else None
    val, idx = binding.rank_dense(wide.to(DEV)[:, :D], w.to(DEV), b.to(DEV), k, binding.make_workspace(N, k), all_scores=scores)
    torch.cuda.synchronize()
    ref = orc.dense_scores(X.numpy(), w.numpy(), b.numpy())[0]
    _check(ref, val[0], idx[0], k, rtol, what)
    if want_all:
        assert np.all(np.abs(scores.cpu().numpy() - ref) <= orc.score_tolerance(ref, rtol)), what


def _dense_many(rng, N, k, seed):
    N = min(N, 60000)
    Q = int(rng.choice([2, 3, 32, 64]))
    D = int(rng.choice([128, 256, 384, 2048]))
    half = bool(rng.random() < 0.6)
    N = min(N, int(1e8 // D))
    k = min(k, N)
    what = "dense N=%d D=%d Q=%d k=%d half=%s seed=%d" % (N, D, Q, k, half, seed)
    dt = torch.float16 if half else torch.float32
    X = synth.dense_features(N, D, seed, dtype=dt)
    W = synth.normal_matrix(Q, D, 0.05, seed + 1, dtype=dt)
    val, idx = binding.rank_dense(X.to(DEV), W.to(DEV), None, k, binding.make_workspace(N, k, Q))
    torch.cuda.synchronize()
    ref = orc.dense_scores(X.numpy(), W.numpy())
    for q in range(Q):
        _check(ref[q], val[q], idx[q], k, 2e-3 if half else 1e-4, what + " q=%d" % q)


def _pq(rng, N, k, seed, want_all):
    M = int(rng.choice([16, 32, 48, 64, 128, 144, 256, 512, 1024]))
    dsub = int(rng.choice([1, 4, 8, 16]))
    N = min(N, int(4e8 // M))
    k = min(k, N)
    what = "pq N=%d M=%d dsub=%d k=%d scores=%s seed=%d" % (N, M, dsub, k, want_all, seed)
    cb = synth.pq_codebooks(M, 256, dsub, seed)
    codes = synth.pq_codes(N, M, 256, seed + 1)
    w = synth.normal_vector(M * dsub, 1.0, seed + 2)
    ws = binding.make_workspace(N, k)
    scores = torch.empty(N, device=DEV) if want_all else None
    if rng.random() < 0.5:
        val, idx = binding.rank_pq_model(codes.to(DEV), cb.to(DEV), w.to(DEV), 0.5, k, ws, all_scores=scores)
    else:
        lut = binding.pq_build_lut(cb.to(DEV), w.to(DEV))
        val, idx = binding.rank_pq(codes.to(DEV), lut, 0.5, k, ws, all_scores=scores)
    torch.cuda.synchronize()
    ref = orc.pq_scores_reconstruct(codes.numpy(), cb.numpy(), w.numpy(), 0.5)
    _check(ref, val[0], idx[0], k, 1e-4, what)


def _bits(rng, N, k, seed, want_all, hamming):
    D = int(rng.choice([128, 256, 384, 1024, 2048, 2176, 4096, 8192]))
    N = min(N, int(3e9 // D))
    k = min(k, N)
    what = "%s N=%d D=%d k=%d scores=%s seed=%d" % ("hamming" if hamming else "binary", N, D, k, want_all, seed)
    bits = synth.binary_bits_random(N, D // 32, seed)
    ws = binding.make_workspace(N, k)
    scores = torch.empty(N, device=DEV) if want_all else None
    if hamming:
        query = synth.binary_bits_random(1, D // 32, seed + 1)[0].contiguous()
        val, idx = binding.rank_hamming(bits.to(DEV), D, query.to(DEV), k, ws, all_scores=scores)
        torch.cuda.synchronize()
        ref = orc.hamming_scores(synth.as_uint32(bits.numpy()), D, synth.as_uint32(query.numpy()))
        _check(ref, val[0], idx[0], k, 0.0, what, exact=True)
    else:
        w = synth.normal_vector(D, 1.0, seed + 1)
        val, idx = binding.rank_binary(bits.to(DEV), D, w.to(DEV), -0.25, k, ws, all_scores=scores)
        torch.cuda.synchronize()
        ref = orc.binary_scores(synth.as_uint32(bits.numpy()), D, w.numpy(), -0.25)
        _check(ref, val[0], idx[0], k, 1e-4, what)


def _sparse(rng, N, k, seed, want_all):
    zeros = float(rng.choice([0.0, 0.3, 0.6, 0.95, 1.0]))
    what = "sparse N=%d k=%d zeros=%.2f scores=%s seed=%d" % (N, k, zeros, want_all, seed)
    X = synth.sparse_features(N, 128, seed, zero_fraction=zeros)
    rows, start = synth.sparse_rows_from_dense(X)
    w = synth.normal_vector(128, 1.0, seed + 1)
    scores = torch.empty(N, device=DEV) if want_all else None
    val, idx = binding.rank_sparse(rows.to(DEV), start.to(DEV), 128, w.to(DEV), 0.125, k, binding.make_workspace(N, k),
                                   all_scores=scores)
    torch.cuda.synchronize()
    ref = orc.dense_scores(X.numpy(), w.numpy(), np.array([0.125], np.float32))[0]
    _check(ref, val[0], idx[0], k, 1e-4, what)


def _topk(rng, N, k, seed):
    Q = int(rng.choice([1, 1, 2, 5]))
    if Q > 1:
        N = min(N, 200000)
        k = min(k, N)
    kind = str(rng.choice(["normal", "integers", "constant", "sorted"]))
    what = "topk N=%d Q=%d k=%d scores %s seed=%d" % (N, Q, k, kind, seed)
    g = torch.Generator().manual_seed(seed)
    S = torch.randn((Q, N), generator=g)
    if kind == "integers":
        S = torch.randint(-20, 21, (Q, N), generator=g).float()
    elif kind == "constant":
        S = torch.full((Q, N), 1.5)
    elif kind == "sorted":
        S = torch.sort(S, dim=1).values
    val, idx = binding.topk(S.to(DEV), k, binding.make_workspace(N, k, Q))
    torch.cuda.synchronize()
    for q in range(Q):
        _check(S[q].numpy().astype(np.float64), val[q], idx[q], k, 0.0, what, exact=True)


def _one_configuration(rng):
    kind = str(rng.choice(["dense32", "dense16", "dense many", "pq", "binary", "hamming", "sparse", "topk"]))
    N = _rows(rng)
    k = _list_length(rng, N)
    seed = int(rng.integers(1, 1 << 30))
    want_all = bool(rng.random() < 0.4)
    if kind in ("dense32", "dense16"):
        _dense(rng, N, k, seed, want_all, kind == "dense16")
    elif kind == "dense many":
        _dense_many(rng, N, k, seed)
    elif kind == "pq":
        _pq(rng, N, k, seed, want_all)
    elif kind in ("binary", "hamming"):
        _bits(rng, N, k, seed, want_all, kind == "hamming")
    elif kind == "sparse":
        _sparse(rng, N, k, seed, want_all)
    else:
        _topk(rng, N, k, seed)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_valid_configurations_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    for _ in range(120):
        _one_configuration(rng)
