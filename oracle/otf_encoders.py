"""Oracle for the binarisation encoder -- TEST INFRASTRUCTURE ONLY (plain numpy, float64).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.
It shares nothing with the HIP path and never imports it.

Paper Sec. 3, "Binarization", Eq. (1): a zero-centred descriptor phi in R^m becomes the code
beta = sgn(U phi) in {0,1}^n, n > m, with sgn(a) = 1 iff a > 0 (so a zero projection codes as 0),
and U the first m columns of the orthogonal factor of a QR decomposition of a random n x n matrix.
The random matrix is an input here (the caller draws it).
"""
import numpy as np


def tight_frame(G, m):
    """U (n x m, float64): first m columns of the orthogonal factor Q of G = QR, G an n x n matrix.

    QR is unique only up to the sign of each column of Q; the factorisation with a positive
    diagonal of R is taken (the one Gram-Schmidt produces), so that U is a function of G."""
    G = np.asarray(G, dtype=np.float64)
    n = G.shape[0]
    if G.shape != (n, n) or not (1 <= m <= n):
        raise ValueError("tight_frame needs an n x n matrix and 1 <= m <= n")
    Q, R = np.linalg.qr(G)                      # library step: Householder QR (LAPACK)
    # A leading column in the span of its predecessors has no direction of its own: the
    # Gram-Schmidt basis has a zero column there, while a Householder factorisation fills in an
    # arbitrary unit vector (and lets it leak into the columns after it).  |R_jj| is the distance
    # of column j from the span of the q before it; rounding leaves ~1e-16 of the column's
    # length, so anything below n * eps of it counts as zero.
    tol = n * np.finfo(np.float64).eps * np.linalg.norm(G[:, :m], axis=0)
    if np.all(np.abs(np.diag(R)[:m]) > tol):
        s = np.sign(np.diag(R))
        return (Q * s[None, :])[:, :m].copy()
    # rank-deficient leading block: column by column, each against an orthonormal basis (library
    # QR) of the independent columns found so far; the residual's own direction makes R_jj positive
    U = np.zeros((n, m))
    independent = []
    for j in range(m):
        r = G[:, j].copy()
        if independent:
            B = np.linalg.qr(G[:, independent])[0]
            r -= B @ (B.T @ r)
            r -= B @ (B.T @ r)
        if np.linalg.norm(r) > tol[j]:
            U[:, j] = r / np.linalg.norm(r)
            independent.append(j)
    return U


def projections(phi, U):
    """(U phi) for every row of phi: N x n float64, and the magnitude sums sum_j |U_dj phi_j| that
    bound the rounding error of any floating-point evaluation of the same sum."""
    phi = np.asarray(phi, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    return phi @ U.T, np.abs(phi) @ np.abs(U).T   # library step: matrix product


def pack_bits(b):
    """b: N x n array of 0/1 -> N x n/32 uint32, dimension d at bit d mod 32 of word d div 32."""
    b = np.asarray(b).astype(np.uint64)
    N, n = b.shape
    if n % 32:
        raise ValueError("n must be a multiple of 32")
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    return (b.reshape(N, n // 32, 32) * weights[None, None, :]).sum(axis=2).astype(np.uint32)


def binarize(phi, U):
    """beta = sgn(U phi), packed; sgn(a) = 1 iff a > 0."""
    proj, _ = projections(phi, U)
    return pack_bits(proj > 0.0)
