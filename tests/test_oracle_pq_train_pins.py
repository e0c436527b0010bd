"""Pins for the PQ encoder / k-means oracle (paper Sec. 3, "Product quantization (PQ)"): brute-force
python loops, closed-form toy problems, Lloyd's monotonicity, and the link to the PQ scoring
oracle.  CPU only."""
import numpy as np

from oracle import otf_pq_train as pq

RNG = np.random.default_rng(140747)


def test_codes_equal_brute_force_loops():
    N, M, K, dsub = 9, 3, 5, 4
    X = RNG.standard_normal((N, M * dsub)).astype(np.float32)
    C = RNG.standard_normal((M, K, dsub)).astype(np.float32)
    got = pq.encode(X, C)
    assert got.shape == (N, M) and got.dtype == np.uint8
    for i in range(N):
        for m in range(M):
            best, arg = None, -1
            for k in range(K):
                d = 0.0
                for j in range(dsub):
                    t = float(X[i, m * dsub + j]) - float(C[m, k, j])
                    d += t * t
                if best is None or d < best:             # strict: the first of equal distances wins
                    best, arg = d, k
            assert got[i, m] == arg, (i, m)


def test_a_centre_codes_as_itself_and_ties_go_to_the_lower_index():
    M, K, dsub = 2, 6, 3
    C = RNG.standard_normal((M, K, dsub))
    X = np.concatenate([C[0, 4], C[1, 2]])[None, :]
    np.testing.assert_array_equal(pq.encode(X, C), [[4, 2]])
    C2 = np.zeros((1, 4, 1))
    C2[0, :, 0] = [-1.0, 1.0, 1.0, 3.0]
    np.testing.assert_array_equal(pq.encode(np.array([[0.0], [1.0], [2.0]]), C2)[:, 0], [0, 1, 1])


def test_sub_blocks_use_their_own_vocabulary():
    """Swapping two sub-blocks of the data and of the vocabularies swaps the code columns."""
    N, M, K, dsub = 20, 2, 7, 5
    X = RNG.standard_normal((N, M * dsub))
    C = RNG.standard_normal((M, K, dsub))
    a = pq.encode(X, C)
    Xs = np.concatenate([X[:, dsub:], X[:, :dsub]], axis=1)
    b = pq.encode(Xs, C[::-1])
    np.testing.assert_array_equal(a[:, ::-1], b)


def test_lloyd_step_on_a_line():
    """Points 0, 1, 2, 10, 11 with centres 0 and 4.  The point 2 is equally far from both: a tie,
    which goes to the lower index, so the cells are {0, 1, 2} and {10, 11}.  New centres: the means
    1 and 10.5; distortion before the move (0 + 1 + 4 + 36 + 49) / 5."""
    X = np.array([[0.0], [1.0], [2.0], [10.0], [11.0]])
    C = np.array([[[0.0], [4.0]]])
    C1, codes, dist = pq.lloyd_step(X, C)
    np.testing.assert_array_equal(codes[:, 0], [0, 0, 0, 1, 1])
    np.testing.assert_allclose(C1[0, :, 0], [1.0, 10.5])
    np.testing.assert_allclose(dist, 90.0 / 5)


def test_lloyd_never_increases_distortion_and_keeps_empty_centres():
    N, M, K, dsub = 400, 2, 8, 3
    X = RNG.standard_normal((N, M * dsub))
    C = RNG.standard_normal((M, K, dsub))
    C[0, 7] = 100.0                                        # nothing will be assigned to this centre
    prev = None
    for _ in range(6):
        C_new, codes, dist = pq.lloyd_step(X, C)
        assert prev is None or dist <= prev + 1e-12
        np.testing.assert_array_equal(C_new[0, 7], C[0, 7])
        assert not (codes[:, 0] == 7).any()
        prev, C = dist, C_new
    # at the end the centres are the means of their cells
    C_fix, codes, _ = pq.lloyd_step(X, C)
    Xs = X.reshape(N, M, dsub)
    for m in range(M):
        for k in range(K):
            rows = codes[:, m] == k
            if rows.any():
                np.testing.assert_allclose(C_fix[m, k], Xs[rows, m].mean(axis=0), rtol=1e-12)


def test_codes_and_scores_agree_with_the_scan_oracle(oracle):
    """Scoring the codes through the scan oracle's reconstruction gives w . (nearest centres)."""
    N, M, K, dsub = 30, 4, 256, 2
    X = RNG.standard_normal((N, M * dsub)).astype(np.float32)
    C = RNG.standard_normal((M, K, dsub)).astype(np.float32)
    w = RNG.standard_normal(M * dsub).astype(np.float32)
    codes = pq.encode(X, C)
    s = oracle.pq_scores_reconstruct(codes, C, w, 0.0)
    recon = np.concatenate([C[m, codes[:, m]] for m in range(M)], axis=1).astype(np.float64)
    np.testing.assert_allclose(s, recon @ w.astype(np.float64), rtol=1e-12, atol=1e-12)
    # and the reconstruction is at least as close to X as any other choice of centres
    d = pq.distances(X, C)
    assert np.all(np.take_along_axis(d, codes[:, :, None].astype(np.int64), axis=2)[:, :, 0] <= d.min(axis=2) + 1e-15)
