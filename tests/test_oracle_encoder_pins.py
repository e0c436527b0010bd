"""Pins for the binarisation-encoder oracle (paper Sec. 3, "Binarization", Eq. (1)): checked against
what the mathematics fixes -- orthonormal columns, norm preservation, a Gram-Schmidt written out
by hand, per-bit python loops -- and against the binary scan oracle, whose bit convention the codes
must share.  CPU only."""
import numpy as np
import pytest

from oracle import otf_encoders as enc

RNG = np.random.default_rng(14074764)


def _gram_schmidt(G, m):
    """Classical Gram-Schmidt on the first m columns, python loops."""
    n = G.shape[0]
    Q = np.zeros((n, m))
    for j in range(m):
        v = G[:, j].astype(np.float64).copy()
        for i in range(j):
            v -= np.dot(Q[:, i], G[:, j]) * Q[:, i]
        Q[:, j] = v / np.linalg.norm(v)
    return Q


def test_frame_has_orthonormal_columns_and_preserves_norms():
    n, m = 96, 24
    U = enc.tight_frame(RNG.standard_normal((n, n)), m)
    assert U.shape == (n, m)                                   # n x m, not m x n
    np.testing.assert_allclose(U.T @ U, np.eye(m), atol=1e-12)
    phi = RNG.standard_normal((50, m))
    proj, _ = enc.projections(phi, U)
    np.testing.assert_allclose(np.linalg.norm(proj, axis=1), np.linalg.norm(phi, axis=1), rtol=1e-12)
    P = U @ U.T                                                # projector onto the column span
    np.testing.assert_allclose(P @ P, P, atol=1e-12)


def test_frame_equals_gram_schmidt_of_the_first_columns():
    """The first m columns of Q depend on the first m columns of the matrix only, and with a
    positive diagonal of R they are what Gram-Schmidt gives (a sign slip or a row/column mix-up
    in the oracle fails here)."""
    n, m = 12, 5
    G = RNG.standard_normal((n, n))
    U = enc.tight_frame(G, m)
    np.testing.assert_allclose(U, _gram_schmidt(G, m), atol=1e-12)
    G2 = G.copy()
    G2[:, m:] = RNG.standard_normal((n, n - m))                # later columns do not matter
    np.testing.assert_allclose(enc.tight_frame(G2, m), U, atol=1e-12)
    assert np.all(np.einsum("ij,ij->j", U, G[:, :m]) > 0)      # diag(R) > 0


def _dependent_matrix(n, rng):
    """Random n x n matrix whose columns 3, 5 and 7 lie in the span of earlier ones (a repeat, a
    combination of two, a zero column)."""
    G = rng.standard_normal((n, n))
    G[:, 3] = G[:, 1]
    G[:, 5] = 2.0 * G[:, 0] - 0.5 * G[:, 2]
    G[:, 7] = 0.0
    return G


def test_dependent_leading_columns_give_zero_columns():
    """A column in the span of its predecessors has no Gram-Schmidt direction: the frame has a zero
    column there and the other columns are what the matrix without those columns gives (a
    Householder factorisation alone would put an arbitrary unit vector there and let it leak
    into the columns after it)."""
    n, m = 40, 10
    G = _dependent_matrix(n, np.random.default_rng(7))
    U = enc.tight_frame(G, m)
    dep, indep = [3, 5, 7], [0, 1, 2, 4, 6, 8, 9]
    assert np.all(U[:, dep] == 0.0)
    H = np.concatenate([G[:, indep], np.random.default_rng(8).standard_normal((n, n - len(indep)))], axis=1)
    np.testing.assert_allclose(U[:, indep], _gram_schmidt(H, len(indep)), atol=1e-12)
    np.testing.assert_allclose(U[:, indep].T @ U[:, indep], np.eye(len(indep)), atol=1e-12)
    # a column that is merely nearly dependent (1e-6 away) keeps a direction
    G[:, 3] += 1e-6 * np.random.default_rng(9).standard_normal(n)
    U2 = enc.tight_frame(G, m)
    assert abs(np.linalg.norm(U2[:, 3]) - 1.0) < 1e-9 and np.all(U2[:, [5, 7]] == 0.0)


def test_binarize_equals_per_bit_loops():
    N, m, n = 7, 6, 64
    U = enc.tight_frame(RNG.standard_normal((n, n)), m)
    phi = RNG.standard_normal((N, m)).astype(np.float32)
    got = enc.binarize(phi, U)
    assert got.shape == (N, n // 32) and got.dtype == np.uint32
    for i in range(N):
        for d in range(n):
            a = 0.0
            for j in range(m):
                a += float(U[d, j]) * float(phi[i, j])
            bit = 1 if a > 0 else 0
            assert (int(got[i, d // 32]) >> (d % 32)) & 1 == bit, (i, d)


def test_single_dimension_sets_a_single_bit():
    """With the identity as frame and a unit descriptor only bit d is set: dimension d is bit
    d mod 32 of word d div 32."""
    n = 96
    for d in (0, 1, 31, 32, 33, 63, 95):
        phi = np.zeros((1, n))
        phi[0, d] = 2.5
        got = enc.binarize(phi, np.eye(n))
        want = np.zeros(n // 32, dtype=np.uint32)
        want[d // 32] = np.uint32(1) << np.uint32(d % 32)
        np.testing.assert_array_equal(got[0], want)


def test_sign_of_zero_is_zero_and_negation_complements():
    n, m = 64, 8
    U = enc.tight_frame(RNG.standard_normal((n, n)), m)
    assert not enc.binarize(np.zeros((3, m)), U).any()          # sgn(0) = 0
    phi = RNG.standard_normal((5, m))
    a, b = enc.binarize(phi, U), enc.binarize(-phi, U)
    proj, _ = enc.projections(phi, U)
    assert np.all(proj != 0)
    np.testing.assert_array_equal(a ^ b, np.full_like(a, 0xFFFFFFFF))


def test_codes_use_the_bit_convention_of_the_scan(oracle):
    """Score of the code under the binary scan oracle with w = U phi's own sign pattern: every
    dimension then contributes +|w_d| iff encoder and scan agree on which bit is which."""
    N, m, n = 9, 16, 128
    U = enc.tight_frame(RNG.standard_normal((n, n)), m)
    phi = RNG.standard_normal((N, m))
    bits = enc.binarize(phi, U)
    proj, _ = enc.projections(phi, U)
    for i in range(N):
        w = proj[i].astype(np.float32)                          # w_d > 0 exactly where bit d is 1
        s = oracle.binary_scores(bits[i:i + 1], n, w, 0.0)[0]
        np.testing.assert_allclose(s, np.abs(w.astype(np.float64)).sum(), rtol=1e-12)


def test_margin_sums_bound_the_projection():
    n, m = 64, 10
    U = enc.tight_frame(RNG.standard_normal((n, n)), m)
    phi = RNG.standard_normal((20, m))
    proj, mag = enc.projections(phi, U)
    assert np.all(np.abs(proj) <= mag + 1e-15)
    np.testing.assert_allclose(mag, np.einsum("ij,dj->id", np.abs(phi), np.abs(U)), rtol=1e-12)
