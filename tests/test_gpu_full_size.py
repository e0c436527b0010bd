"""Parity at the full benchmark sizes, in the launch configuration bench.py times (same store
generators, same calls, default path).  The oracle cannot score 10^7..10^8 rows in test time, so:
  * the returned top-k scores are compared with the oracle on exactly those rows;
  * a random sample of rows is compared with the oracle through the all_scores output;
  * completeness is checked as a property on the GPU's own fp32 scores: no row outside the
    returned list scores above the list's last entry, and the list equals the first k of a full
    sort of those scores (ties by row index).
"""
import numpy as np
import pytest
import torch

import bench
from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SAMPLE = 20000


def _check_list_against_own_scores(all_scores, idx, val, k):
    """Exactness of the selection on the scores the GPU itself produced (index work is bit-exact)."""
    kth = val[-1]
    above = torch.nonzero(all_scores > kth).flatten()
    assert above.numel() <= k
    assert set(above.cpu().tolist()) <= set(idx.cpu().tolist()), "a row above the k-th score is missing"
    np.testing.assert_array_equal(all_scores[idx.long()].cpu().numpy(), val.cpu().numpy())
    # full ordering: score descending, row ascending
    s = val.cpu().numpy().astype(np.float64)
    i = idx.cpu().numpy().astype(np.int64)
    assert np.all((s[:-1] > s[1:]) | ((s[:-1] == s[1:]) & (i[:-1] < i[1:])))
    ties = torch.nonzero(all_scores == kth).flatten().cpu().numpy()
    need = k - int((all_scores > kth).sum().item())
    assert set(ties[:need].tolist()) <= set(i.tolist()), "ties at the k-th score must go to the lowest rows"


def _sample_rows(N, seed):
    return np.sort(np.random.default_rng(seed).choice(N, SAMPLE, replace=False))


def test_dense_full_size(oracle):
    step, cfg = bench.make_workload("dense", 1.0, torch, binding, synth)
    X, w = cfg["_keep"]
    N, k = cfg["N"], cfg["k"]
    val, idx = step()
    torch.cuda.synchronize()
    ws = binding.make_workspace(N, k)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    val2, idx2 = binding.rank_dense(X, w, None, k, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(val, val2)
    _check_list_against_own_scores(all_scores, idx[0], val[0], k)
    rows = np.union1d(_sample_rows(N, 1), idx[0].cpu().numpy())
    ref = oracle.dense_scores(X[torch.from_numpy(rows).to(DEV)].cpu().numpy(), w.cpu().numpy())[0]
    got = all_scores[torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.float64)
    sigma = float(all_scores.std().item())
    assert np.all(np.abs(got - ref) <= 1e-4 * np.maximum(np.abs(ref), sigma))


def test_dense_128d_full_size(oracle):
    """The paper's own feature size, 10M rows: the default path here is the filtered scan, the
    all_scores call the materialising one; both must give the same list."""
    step, cfg = bench.make_workload("dense128", 1.0, torch, binding, synth)
    X, w = cfg["_keep"]
    N, k = cfg["N"], cfg["k"]
    val, idx = step()
    torch.cuda.synchronize()
    ws = binding.make_workspace(N, k)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    val2, idx2 = binding.rank_dense(X, w, None, k, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(val, val2)
    _check_list_against_own_scores(all_scores, idx[0], val[0], k)
    rows = np.union1d(_sample_rows(N, 6), idx[0].cpu().numpy())
    ref = oracle.dense_scores(X[torch.from_numpy(rows).to(DEV)].cpu().numpy(), w.cpu().numpy())[0]
    got = all_scores[torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.float64)
    sigma = float(all_scores.std().item())
    assert np.all(np.abs(got - ref) <= 1e-4 * np.maximum(np.abs(ref), sigma))


def test_pq_full_size(oracle):
    step, cfg = bench.make_workload("pq", 1.0, torch, binding, synth)
    codes, cb, w = cfg["_keep"]
    N, k = cfg["N"], cfg["k"]
    val, idx = step()
    torch.cuda.synchronize()
    ws = binding.make_workspace(N, k)
    lut = binding.pq_build_lut(cb, w)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    val2, idx2 = binding.rank_pq(codes, lut, 0.0, k, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(val, val2)
    _check_list_against_own_scores(all_scores, idx[0], val[0], k)
    rows = np.union1d(_sample_rows(N, 2), idx[0].cpu().numpy())
    ref = oracle.pq_scores_reconstruct(codes[torch.from_numpy(rows).to(DEV)].cpu().numpy(), cb.cpu().numpy(),
                                       w.cpu().numpy(), 0.0)
    got = all_scores[torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.float64)
    sigma = float(all_scores.std().item())
    assert np.all(np.abs(got - ref) <= 1e-4 * np.maximum(np.abs(ref), sigma))


def test_binary_full_size(oracle):
    step, cfg = bench.make_workload("binary", 1.0, torch, binding, synth)
    bits, w = cfg["_keep"]
    N, k, D = cfg["N"], cfg["k"], cfg["D"]
    val, idx = step()
    torch.cuda.synchronize()
    ws = binding.make_workspace(N, k)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    val2, idx2 = binding.rank_binary(bits, D, w, 0.0, k, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(val, val2)
    _check_list_against_own_scores(all_scores, idx[0], val[0], k)
    rows = np.union1d(_sample_rows(N, 3), idx[0].cpu().numpy())
    ref = oracle.binary_scores(synth.as_uint32(bits[torch.from_numpy(rows).to(DEV)].cpu().numpy()), D,
                               w.cpu().numpy(), 0.0)
    got = all_scores[torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.float64)
    sigma = float(all_scores.std().item())
    assert np.all(np.abs(got - ref) <= 1e-4 * np.maximum(np.abs(ref), sigma))


def test_multi_classifier_full_size(oracle):
    step, cfg = bench.make_workload("multiquery", 1.0, torch, binding, synth)
    X, W = cfg["_keep"]
    N, k, Q = cfg["N"], cfg["k"], cfg["Q"]
    val, idx = step()
    torch.cuda.synchronize()
    ws = binding.make_workspace(N, k, Q)
    all_scores = torch.empty((Q, N), dtype=torch.float32, device=DEV)
    val2, idx2 = binding.rank_dense(X, W, None, k, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(val, val2)
    for q in (0, 17, 63):
        _check_list_against_own_scores(all_scores[q], idx[q], val[q], k)
    rows = _sample_rows(N, 4)[:4000]
    ref = oracle.dense_scores(X[torch.from_numpy(rows).to(DEV)].cpu().numpy(), W.cpu().numpy())
    got = all_scores[:, torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.float64)
    sigma = all_scores.std(dim=1).cpu().numpy().astype(np.float64)[:, None]
    assert np.all(np.abs(got - ref) <= 2e-3 * np.maximum(np.abs(ref), sigma))
    # the returned rows of a few classifiers, against the oracle
    for q in (0, 31):
        r = idx[q].cpu().numpy()
        refq = oracle.dense_scores(X[idx[q].long()].cpu().numpy(), W[q:q + 1].cpu().numpy())[0]
        assert np.all(np.abs(val[q].cpu().numpy() - refq) <= 2e-3 * np.maximum(np.abs(refq), sigma[q]))
