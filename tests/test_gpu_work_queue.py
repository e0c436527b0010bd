"""GPU parity at the sizes that exercise the dynamic work distribution of the scans: stores long
enough that workgroups draw chunks beyond the two they start with (more than 2 x 256 chunks), with
a ragged last chunk, a ragged last tile and a last chunk that holds no full tile at all; and, for
the multi-classifier scan, one to three K steps per tile (the look-ahead of its tile ring is counted
in steps).  Integer-valued tables and weights make every fp32 sum exact, so a row that is scored
twice, skipped, or scored from the wrong tile shows as a non-zero difference."""
import numpy as np
import pytest
import torch

from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = synth.BASE_SEED + 5000


@pytest.mark.parametrize("N", [2048 * 530 + 1, 2048 * 530 + 63, 2048 * 530 + 64, 2048 * 530 + 2047, 2048 * 600])
def test_pq_every_row_scored_once(oracle, N):
    """M = 128: tiles of 64 rows, chunks of 2048 rows."""
    M, K = 128, 256
    codes = synth.pq_codes(N, M, K, SEED + 1)
    g = torch.Generator().manual_seed(SEED + 2)
    lut = torch.randint(-1000, 1000, (M, K), generator=g).to(torch.float32)
    ref = oracle.pq_scores_lut(codes.numpy(), lut.numpy().astype(np.float64), 3.0)
    ws = binding.make_workspace(N, 100)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    cd, ld = codes.to(DEV), lut.to(DEV)
    val, idx = binding.rank_pq(cd, ld, 3.0, 100, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(all_scores.cpu().numpy().astype(np.float64), ref)
    # the filtered scan (no score output) must return the same list
    val2, idx2 = binding.rank_pq(cd, ld, 3.0, 100, ws)
    torch.cuda.synchronize()
    i, v = oracle.topk(ref, 100)
    np.testing.assert_array_equal(idx[0].cpu().numpy(), i)
    np.testing.assert_array_equal(idx2[0].cpu().numpy(), i)
    np.testing.assert_array_equal(val2[0].cpu().numpy().astype(np.float64), v)


@pytest.mark.parametrize("N", [1024 * 600 + 5, 1024 * 600 + 31, 1024 * 513])
def test_binary_every_row_scored_once(oracle, N):
    """D = 2048: tiles of 32 rows, chunks of 1024 rows."""
    D = 2048
    bits = synth.binary_bits_random(N, D // 32, SEED + 3)
    g = torch.Generator().manual_seed(SEED + 4)
    w = torch.randint(-512, 512, (D,), generator=g).to(torch.float32)
    ref = oracle.binary_scores(synth.as_uint32(bits.numpy()), D, w.numpy(), 1.0)
    ws = binding.make_workspace(N, 50)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    bd, wd = bits.to(DEV), w.to(DEV)
    binding.rank_binary(bd, D, wd, 1.0, 50, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(all_scores.cpu().numpy().astype(np.float64), ref)
    val2, idx2 = binding.rank_binary(bd, D, wd, 1.0, 50, ws)
    torch.cuda.synchronize()
    i, v = oracle.topk(ref, 50)
    np.testing.assert_array_equal(idx2[0].cpu().numpy(), i)


@pytest.mark.parametrize("N,D,dtype", [(100003, 4, torch.float32), (100003, 8, torch.float32), (70001, 16, torch.float32),
                                       (50021, 32, torch.float32), (40009, 64, torch.float32),
                                       (30011, 128, torch.float32), (33333, 24, torch.float16),
                                       (20001, 256, torch.float16), (129, 128, torch.float32)])
def test_narrow_dense_rows_every_row_scored_once(oracle, N, D, dtype):
    """Rows of at most 512 bytes: 1 to 32 lanes per row, several rows per wave load, the row sums
    formed by exchanges between lanes; small integers make every sum exact."""
    g = torch.Generator().manual_seed(SEED + 9)
    X = torch.randint(-4, 5, (N, D), generator=g).to(dtype)
    w = torch.randint(-8, 9, (D,), generator=g).to(torch.float32)
    ref = oracle.dense_scores(X.numpy(), w.numpy())[0]
    ws = binding.make_workspace(N, 64)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    val, idx = binding.rank_dense(X.to(DEV), w.to(DEV), None, 64, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(all_scores.cpu().numpy().astype(np.float64), ref)
    i, v = oracle.topk(ref, 64)
    np.testing.assert_array_equal(np.sort(val[0].cpu().numpy().astype(np.float64))[::-1], v)
    assert np.all(ref[idx[0].cpu().numpy()] == val[0].cpu().numpy())


@pytest.mark.parametrize("N,D", [(64 * 600 + 1, 2048), (128 * 530 + 77, 1024)])
def test_dense_every_row_scored_once(oracle, N, D):
    """fp16 rows that fill the lanes exactly take the pipelined, dynamically scheduled kernel."""
    g = torch.Generator().manual_seed(SEED + 5)
    X = torch.randint(-4, 5, (N, D), generator=g).to(torch.float16)
    w = torch.randint(-8, 9, (D,), generator=g).to(torch.float32)
    ref = oracle.dense_scores(X.numpy(), w.numpy())[0]
    ws = binding.make_workspace(N, 64)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    val, idx = binding.rank_dense(X.to(DEV), w.to(DEV), None, 64, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(all_scores.cpu().numpy().astype(np.float64), ref)
    i, v = oracle.topk(ref, 64)
    np.testing.assert_array_equal(idx[0].cpu().numpy(), i)


@pytest.mark.parametrize("D,N", [(128, 128 * 4100 + 7), (256, 128 * 4100), (384, 128 * 4097 + 127)])
def test_multi_classifier_every_row_scored_once(oracle, D, N):
    """One, two and three K steps per tile, more than 8 tiles per workgroup (dynamic hand-out)."""
    Q = 64
    g = torch.Generator().manual_seed(SEED + 6)
    X = torch.randint(-2, 3, (N, D), generator=g).to(torch.float16)
    W = torch.randint(-3, 4, (Q, D), generator=g).to(torch.float16)
    ws = binding.make_workspace(N, 10, Q)
    all_scores = torch.empty((Q, N), dtype=torch.float32, device=DEV)
    Xd, Wd = X.to(DEV), W.to(DEV)
    val, idx = binding.rank_dense(Xd, Wd, None, 10, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    want = (Xd.float() @ Wd.float().T).T.contiguous()            # exact: small integers (device memory plumbing only)
    assert torch.equal(all_scores, want)
    rows = np.concatenate([np.arange(0, N, 997), np.arange(N - 300, N)])
    ref = oracle.dense_scores(X.numpy()[rows], W.numpy())
    np.testing.assert_array_equal(all_scores[:, torch.from_numpy(rows).to(DEV)].cpu().numpy().astype(np.float64), ref)
    val2, idx2 = binding.rank_dense(Xd, Wd, None, 10, ws)          # filtered path, same lists
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(val, val2)
