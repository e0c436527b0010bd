"""Oracle for the product-quantisation encoder and its vocabulary training -- TEST
INFRASTRUCTURE ONLY (plain numpy, float64).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.

Paper Sec. 3, "Product quantization (PQ)": the feature is split into sub-blocks and every sub-block
has a vocabulary of centres of its own, learned beforehand on training features.  Encoding
a sub-block means replacing it by the index of its nearest centre (squared Euclidean distance;
equal distances go to the lower index).  The paper does not say how the centres are learned; the
method it cites for PQ uses k-means, so the oracle performs Lloyd iterations from centres handed
in by the caller: assign every training sub-vector to its nearest centre, then move every centre
to the mean of what was assigned to it (a centre nothing was assigned to stays where it is).
"""
import numpy as np


def distances(X, codebooks):
    """Squared distances d[i, m, k] = || X[i, m*dsub:(m+1)*dsub] - codebooks[m, k] ||^2, written out."""
    X = np.asarray(X, dtype=np.float64)
    C = np.asarray(codebooks, dtype=np.float64)
    M, K, dsub = C.shape
    Xs = X.reshape(X.shape[0], M, dsub)
    diff = Xs[:, :, None, :] - C[None, :, :, :]
    return (diff * diff).sum(axis=3)


def encode(X, codebooks):
    """codes[i, m] = index of the nearest centre of sub-block m (lowest index among equals), uint8."""
    d = distances(X, codebooks)
    return np.argmin(d, axis=2).astype(np.uint8)          # numpy's argmin returns the first minimum


def lloyd_step(X, codebooks):
    """One iteration: returns (new codebooks float64, codes of the assignment step, distortion =
    mean over rows of the summed squared distance to the assigned centres, measured before the move)."""
    X = np.asarray(X, dtype=np.float64)
    C = np.asarray(codebooks, dtype=np.float64).copy()
    M, K, dsub = C.shape
    d = distances(X, C)
    codes = np.argmin(d, axis=2)
    distortion = float(np.take_along_axis(d, codes[:, :, None], axis=2).sum() / X.shape[0])
    Xs = X.reshape(X.shape[0], M, dsub)
    for m in range(M):
        for k in range(K):
            rows = codes[:, m] == k
            if rows.any():
                C[m, k] = Xs[rows, m, :].mean(axis=0)
    return C, codes.astype(np.uint8), distortion
