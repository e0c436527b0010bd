"""GPU parity of the PQ encoder and the Lloyd iteration (paper Sec. 3, "Product quantization (PQ)")
with the CPU oracle.

A code is an integer decided by a floating-point comparison.  The kernel compares fp32 values of
||c||^2 - 2 <x, c>; their rounding error is bounded by a small multiple of dsub * 2^-24 times
(||x|| + ||c||)^2, so the kernel's centre may differ from the fp64 oracle's only when it is that
close to being the nearest.  With integer data every value is exact in fp32 and the codes, ties
included, must be identical."""
import numpy as np
import pytest
import torch

from oracle import otf_pq_train as pq
from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = synth.BASE_SEED + 4000


def _data(N, M, dsub, seed):
    """Training/store rows and a vocabulary picked from other rows of the same distribution."""
    X = synth.dense_features(N, M * dsub, seed)
    picks = synth.dense_features(256, M * dsub, seed + 1)
    C = picks.reshape(256, M, dsub).permute(1, 0, 2).contiguous()
    return X, C


def _check_codes(X, C, codes):
    d = pq.distances(X, C)                                          # N x M x K, fp64
    ref = np.argmin(d, axis=2)
    got = codes.astype(np.int64)
    chosen = np.take_along_axis(d, got[:, :, None], axis=2)[:, :, 0]
    dsub = C.shape[2]
    xs = X.astype(np.float64).reshape(X.shape[0], C.shape[0], dsub)
    scale = (np.linalg.norm(xs, axis=2) + np.linalg.norm(C.astype(np.float64), axis=2).max(axis=1)[None, :]) ** 2
    band = 8.0 * dsub * 2.0 ** -24 * scale
    assert np.all(chosen <= d.min(axis=2) + band), "a code is not a nearest centre"
    assert (got != ref).mean() < 1e-3
    return ref


@pytest.mark.parametrize("N,M,dsub", [(3001, 128, 16), (1, 128, 16), (2000, 32, 4), (1500, 16, 8), (700, 4, 16),
                                      (513, 512, 4)])
def test_codes_are_nearest_centres(N, M, dsub):
    X, C = _data(N, M, dsub, SEED + M + dsub)
    ws = binding.pq_train_workspace(M, dsub)
    codes = binding.pq_encode(X.to(DEV), C.to(DEV), ws)
    torch.cuda.synchronize()
    _check_codes(X.numpy(), C.numpy(), codes.cpu().numpy())


@pytest.mark.parametrize("N,M,dsub", [(1500, 128, 16), (900, 16, 8), (1100, 32, 4)])
def test_kernel_on_fp32_matrix_instructions_meets_the_same_bar(N, M, dsub, debug_switches):
    """The comparison kernel (diagnostic switch OTF_DEBUG_PQENC_FP32) stays correct."""
    debug_switches({binding.DEBUG_PQENC_FP32: 1})
    X, C = _data(N, M, dsub, SEED + 40 + dsub)
    ws = binding.pq_train_workspace(M, dsub)
    codes = binding.pq_encode(X.to(DEV), C.to(DEV), ws)
    torch.cuda.synchronize()
    _check_codes(X.numpy(), C.numpy(), codes.cpu().numpy())


def test_exact_data_gives_identical_codes_with_ties_to_the_lower_index():
    N, M, dsub = 3000, 8, 8
    g = torch.Generator().manual_seed(SEED + 1)
    X = torch.randint(-4, 5, (N, M * dsub), generator=g).to(torch.float32)
    C = torch.randint(-4, 5, (M, 256, dsub), generator=g).to(torch.float32)
    C[:, 200:] = C[:, :56]                                          # duplicate centres: exact ties
    X[:56, :dsub] = C[0, 200:]                                      # rows sitting on a duplicated centre
    ws = binding.pq_train_workspace(M, dsub)
    codes = binding.pq_encode(X.to(DEV), C.to(DEV), ws).cpu().numpy()
    ref = pq.encode(X.numpy(), C.numpy())
    np.testing.assert_array_equal(codes, ref)
    assert np.all(codes[:56, 0] < 200)


def test_strided_rows_and_padding_columns():
    N, M, dsub = 900, 16, 8
    X, C = _data(N, M, dsub, SEED + 2)
    wide = torch.zeros((N, M * dsub + 12))
    wide[:, :M * dsub] = X
    ws = binding.pq_train_workspace(M, dsub)
    a = binding.pq_encode(wide.to(DEV)[:, :M * dsub], C.to(DEV), ws)
    b = binding.pq_encode(X.to(DEV), C.to(DEV), ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("N,M,dsub", [(20000, 16, 8), (6000, 128, 16)])
def test_lloyd_step_matches_the_oracle(N, M, dsub):
    X, C = _data(N, M, dsub, SEED + 3)
    C[0, 255] = 50.0                                                # a centre nothing is assigned to
    Cd = C.to(DEV).clone()
    ws = binding.pq_train_workspace(M, dsub)
    codes, dist = binding.pq_lloyd_step(X.to(DEV), Cd, ws)
    torch.cuda.synchronize()
    codes = codes.cpu().numpy()
    _check_codes(X.numpy(), C.numpy(), codes)
    # the move, given the kernel's own assignment: means of the cells, in fp64
    Xs = X.numpy().astype(np.float64).reshape(N, M, dsub)
    want = C.numpy().astype(np.float64).copy()
    d_sum = 0.0
    for m in range(M):
        cm = codes[:, m]
        diff = Xs[:, m, :] - C.numpy().astype(np.float64)[m, cm]
        d_sum += (diff * diff).sum()
        counts = np.bincount(cm, minlength=256)
        sums = np.zeros((256, dsub))
        np.add.at(sums, cm, Xs[:, m, :])
        nz = counts > 0
        want[m, nz] = sums[nz] / counts[nz, None]
    got = Cd.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - want)) <= 1e-5 * np.abs(want).max()
    np.testing.assert_array_equal(got[0, 255], np.full(dsub, 50.0))
    np.testing.assert_allclose(float(dist.cpu()[0]), d_sum / N, rtol=1e-5)
    # and against the oracle's own iteration (its assignment differs from the kernel's on near-ties only)
    C_ref, _, dist_ref = pq.lloyd_step(X.numpy(), C.numpy())
    np.testing.assert_allclose(float(dist.cpu()[0]), dist_ref, rtol=1e-5)
    assert np.max(np.abs(got - C_ref)) <= 2e-3 * np.abs(C_ref).max()


@pytest.mark.parametrize("N,M,dsub", [(5003, 8, 4), (4999, 16, 8), (5001, 4, 16), (64, 4, 16), (130, 12, 4)])
def test_lloyd_step_when_many_rows_share_a_code(N, M, dsub):
    """Rows drawn from three distinct vectors only: nearly every group of rows the kernel adds in
    one instruction holds the same code several times (the degenerate case of its update step)."""
    g = torch.Generator().manual_seed(SEED + 6)
    base, C = _data(3, M, dsub, SEED + 7)
    pick = torch.randint(0, 3, (N,), generator=g)
    pick[: min(N, 40)] = 0                                          # and a run of identical rows
    X = base[pick].contiguous()
    Cd = C.to(DEV).clone()
    ws = binding.pq_train_workspace(M, dsub)
    codes, dist = binding.pq_lloyd_step(X.to(DEV), Cd, ws)
    torch.cuda.synchronize()
    codes = codes.cpu().numpy()
    C_ref, codes_ref, dist_ref = pq.lloyd_step(X.numpy(), C.numpy())
    np.testing.assert_array_equal(codes, codes_ref)                 # three well-separated candidates: no near-ties
    got = Cd.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - C_ref)) <= 1e-5 * np.abs(C_ref).max()
    np.testing.assert_allclose(float(dist.cpu()[0]), dist_ref, rtol=1e-5)


@pytest.mark.parametrize("N,M,dsub", [(257, 1024, 16), (300, 4096, 4), (1, 4, 16), (70, 20, 8)])
def test_lloyd_step_at_the_ends_of_the_shape_range(N, M, dsub):
    """The widest vocabularies the entry point takes (16384 dimensions: 256 column runs of the sums
    kernel, one slice), a single row, and a width that leaves the last column run partly empty."""
    X, C = _data(N, M, dsub, SEED + 14)
    Cd = C.to(DEV).clone()
    ws = binding.pq_train_workspace(M, dsub)
    codes, dist = binding.pq_lloyd_step(X.to(DEV), Cd, ws)
    torch.cuda.synchronize()
    codes = codes.cpu().numpy().astype(np.int64)
    Xs = X.numpy().astype(np.float64).reshape(N, M, dsub)
    C64 = C.numpy().astype(np.float64)
    chosen = C64[np.arange(M)[None, :], codes]                       # N x M x dsub: the centres the kernel assigned
    d_sum = ((Xs - chosen) ** 2).sum()
    want = C64.copy()
    for m in range(M):
        counts = np.bincount(codes[:, m], minlength=256)
        sums = np.zeros((256, dsub))
        np.add.at(sums, codes[:, m], Xs[:, m, :])
        nz = counts > 0
        want[m, nz] = sums[nz] / counts[nz, None]
    got = Cd.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - want)) <= 2.0 ** -23 * np.abs(Xs).max()
    np.testing.assert_allclose(float(dist.cpu()[0]), d_sum / N, rtol=1e-9)
    d = ((Xs[:, :, None, :] - C64[None, :, :, :]) ** 2).sum(axis=3) if N * M <= 80000 else None
    if d is not None:                                                # small enough for the full distance table
        picked = np.take_along_axis(d, codes[:, :, None], axis=2)[:, :, 0]
        assert np.all(picked <= d.min(axis=2) + 8.0 * dsub * 2.0 ** -24 * (np.sqrt(picked) + 1.0) ** 2)


def test_lloyd_step_gives_the_same_bits_every_run():
    """Fixed-point sums do not depend on the order of the adds: centres and distortion repeat bit for bit."""
    N, M, dsub = 40000, 32, 16
    X, C = _data(N, M, dsub, SEED + 8)
    Xd = X.to(DEV)
    ws = binding.pq_train_workspace(M, dsub)
    runs = []
    for _ in range(3):
        Cd = C.to(DEV).clone()
        _, dist = binding.pq_lloyd_step(Xd, Cd, ws)
        torch.cuda.synchronize()
        runs.append((Cd.cpu().numpy().copy(), dist.cpu().numpy().copy()))
    for c, d in runs[1:]:
        np.testing.assert_array_equal(c.view(np.uint32), runs[0][0].view(np.uint32))
        np.testing.assert_array_equal(d.view(np.uint64), runs[0][1].view(np.uint64))


@pytest.mark.parametrize("scale", [2.0 ** -40, 3.0e-5, 1.0, 7.0e5, 2.0 ** 50])
@pytest.mark.parametrize("N,M,dsub", [(9000, 16, 8), (5000, 8, 16), (7000, 16, 4)])
def test_lloyd_step_at_any_magnitude_of_the_data(N, M, dsub, scale):
    """The fixed-point format follows the largest sub-vector norm of the data: the means keep their
    relative accuracy when every value is tiny or huge, and with mixed signs."""
    X, C = _data(N, M, dsub, SEED + 9)
    g = torch.Generator().manual_seed(SEED + 10)
    sign = torch.where(torch.rand(X.shape, generator=g) < 0.5, -1.0, 1.0)
    X = (X * sign * scale).contiguous()
    C = (C * scale).contiguous()
    C[:, 128:] *= -1.0                                              # centres among the negative values too
    Cd = C.to(DEV).clone()
    ws = binding.pq_train_workspace(M, dsub)
    codes, dist = binding.pq_lloyd_step(X.to(DEV), Cd, ws)
    torch.cuda.synchronize()
    codes = codes.cpu().numpy().astype(np.int64)
    Xs = X.numpy().astype(np.float64).reshape(N, M, dsub)
    C64 = C.numpy().astype(np.float64)
    want = C64.copy()
    d_sum = 0.0
    for m in range(M):
        cm = codes[:, m]
        diff = Xs[:, m, :] - C64[m, cm]
        d_sum += (diff * diff).sum()
        counts = np.bincount(cm, minlength=256)
        sums = np.zeros((256, dsub))
        np.add.at(sums, cm, Xs[:, m, :])
        nz = counts > 0
        want[m, nz] = sums[nz] / counts[nz, None]
    got = Cd.cpu().numpy().astype(np.float64)
    # the mean of n values of size <= B, each rounded to 2^-41 B or better, then rounded to fp32
    assert np.max(np.abs(got - want)) <= 2.0 ** -23 * np.abs(Xs).max()
    np.testing.assert_allclose(float(dist.cpu()[0]), d_sum / N, rtol=1e-9)


def test_distortion_of_rows_that_sit_on_their_centres_is_zero():
    """The distortion is a difference of large sums; in double precision with exact fixed-point
    sums it cancels to (almost) nothing when every row coincides with its centre."""
    N, M, dsub = 6000, 16, 8
    _, C = _data(8, M, dsub, SEED + 11)
    g = torch.Generator().manual_seed(SEED + 12)
    pick = torch.randint(0, 256, (N, M), generator=g)
    X = torch.stack([C[m, pick[:, m]] for m in range(M)], dim=1).reshape(N, M * dsub).contiguous()
    Cd = C.to(DEV).clone()
    ws = binding.pq_train_workspace(M, dsub)
    codes, dist = binding.pq_lloyd_step(X.to(DEV), Cd, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(codes.cpu().numpy(), pick.numpy().astype(np.uint8))
    per_row_energy = float((X.double() ** 2).sum()) / N
    assert 0.0 <= float(dist.cpu()[0]) <= 1e-13 * per_row_energy
    np.testing.assert_array_equal(Cd.cpu().numpy(), C.numpy())       # the mean of equal values is that value


def test_lloyd_step_behind_the_comparison_encoder(debug_switches):
    """With the fp32 comparison encoder the bound for the fixed-point sums comes from a pass of its own."""
    debug_switches({binding.DEBUG_PQENC_FP32: 1})
    N, M, dsub = 6000, 16, 8
    X, C = _data(N, M, dsub, SEED + 13)
    Cd = C.to(DEV).clone()
    ws = binding.pq_train_workspace(M, dsub)
    ws.zero_()
    _, dist = binding.pq_lloyd_step((X * 300.0).to(DEV), (Cd * 300.0).contiguous(), ws)
    torch.cuda.synchronize()
    C_ref, _, dist_ref = pq.lloyd_step((X * 300.0).numpy(), (C * 300.0).numpy())
    np.testing.assert_allclose(float(dist.cpu()[0]), dist_ref, rtol=1e-5)


def test_iterations_decrease_the_distortion_and_codes_feed_the_scan(oracle):
    N, M, dsub, k = 30000, 16, 8, 50
    X, C = _data(N, M, dsub, SEED + 4)
    Xd, Cd = X.to(DEV), C.to(DEV).clone()
    ws = binding.pq_train_workspace(M, dsub)
    dists = []
    for _ in range(5):
        _, dist = binding.pq_lloyd_step(Xd, Cd, ws)
        dists.append(float(dist.cpu()[0]))
    assert all(b <= a * (1 + 1e-6) for a, b in zip(dists, dists[1:])) and dists[-1] < 0.9 * dists[0]
    C_ref = C.numpy().astype(np.float64)
    for _ in range(5):
        C_ref, _, dist_ref = pq.lloyd_step(X.numpy(), C_ref.astype(np.float32))
    np.testing.assert_allclose(dists[-1], dist_ref, rtol=2e-3)
    # encode with the trained vocabulary and rank: scores are those of the reconstruction
    codes = binding.pq_encode(Xd, Cd, ws)
    w = synth.normal_vector(M * dsub, 1.0, SEED + 5)
    lut = binding.pq_build_lut(Cd, w.to(DEV))
    rws = binding.make_workspace(N, k)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    val, idx = binding.rank_pq(codes, lut, 0.0, k, rws, all_scores=all_scores)
    torch.cuda.synchronize()
    ref = oracle.pq_scores_reconstruct(codes.cpu().numpy(), Cd.cpu().numpy(), w.numpy(), 0.0)
    ok, msg = oracle.topk_parity_ok(ref, k, idx[0].cpu().numpy(), val[0].cpu().numpy(), 1e-4)
    assert ok, msg
