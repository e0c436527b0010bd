"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random inputs; it contains none of the method's arithmetic and is
the one piece of code the tests hand to both the CPU oracle and the HIP path.  The
paper's own data (PASCAL VOC 2007, MIRFLICKR-1M, downloaded web images, trained ConvNet
weights) are not available; the tensors below take their shapes and value structure:

  * dense ConvNet features: non-negative (post-ReLU), L2-normalised rows, 128 or 2048
    dimensions, fp32 (Sec. 4 "Off-line (pre-processing)", Table 2);
  * product-quantised codes: one byte per sub-block, one vocabulary per sub-block
    (Sec. 3 "Product quantization (PQ)", Table 2);
  * binary codes: sign bits of zero-centred projections, sgn(a) = 1 iff a > 0
    (Sec. 3 "Binarization", Eq. (1)), packed least-significant-bit first into 32-bit words;
  * training pools for the on-line SVM: a fixed pool of 16,000 negatives and a smaller
    pool of positives (Sec. 4 "Off-line (pre-processing)" and "On-line (GPU back-end)").

Everything is generated with torch on the requested device from an explicit seed, in
row chunks so that the multi-gigabyte stores never need a second full-size temporary.
"""
import numpy as np
import torch

BASE_SEED = 14074764


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def dense_features(N, D, seed, device="cpu", dtype=torch.float32, chunk_rows=65536):
    """|N(0,1)| entries, each row scaled to unit L2 norm (computed in fp32, then cast)."""
    g = _gen(seed, device)
    out = torch.empty((N, D), dtype=dtype, device=device)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        x = torch.randn((r1 - r0, D), generator=g, device=device, dtype=torch.float32).abs_()
        x /= x.norm(dim=1, keepdim=True).clamp_min_(1e-30)
        out[r0:r1] = x.to(dtype)
    return out


def sparse_features(N, D, seed, device="cpu", zero_fraction=0.6, chunk_rows=65536):
    """Dense features with most entries exactly zero, as the paper reports for its 128-D ConvNet
    features (Sec. 3.1: more than 60 % of their entries): |N(0,1)| entries, each zeroed with probability
    zero_fraction, then every row scaled to unit L2 norm (an all-zero row stays zero)."""
    g = _gen(seed, device)
    out = torch.empty((N, D), dtype=torch.float32, device=device)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        x = torch.randn((r1 - r0, D), generator=g, device=device, dtype=torch.float32).abs_()
        x *= (torch.rand((r1 - r0, D), generator=g, device=device) >= zero_fraction)
        x /= x.norm(dim=1, keepdim=True).clamp_min_(1e-30)
        out[r0:r1] = x
    return out


def sparse_rows_from_dense(X, chunk_rows=1 << 18):
    """The sparse-row store of a dense matrix (storage format only, no arithmetic): for row i, D/32
    presence-mask words (dimension d = bit d mod 32, least significant first, of word d div 32, set
    iff X[i][d] != 0) followed by the bit patterns of its non-zero values in ascending order of
    dimension.  Returns (rows int32 words, start int64 [N+1] word offsets); the word array is padded
    to a multiple of 4 words (16 bytes)."""
    N, D = X.shape
    assert D % 32 == 0
    wm = D // 32
    dev = X.device
    nnz = (X != 0).sum(dim=1, dtype=torch.int64)
    start = torch.zeros(N + 1, dtype=torch.int64, device=dev)
    start[1:] = torch.cumsum(nnz + wm, dim=0)
    total = int(start[-1].item())
    rows = torch.zeros((total + 3) // 4 * 4, dtype=torch.int32, device=dev)
    weights = (torch.ones(32, dtype=torch.int64, device=dev) << torch.arange(32, device=dev, dtype=torch.int64))
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        x = X[r0:r1]
        nz = x != 0
        words = (nz.reshape(r1 - r0, wm, 32).to(torch.int64) * weights).sum(dim=2)            # 0 .. 2^32 - 1
        words = torch.where(words >= 2 ** 31, words - 2 ** 32, words).to(torch.int32)       # the same 32 bits
        pos = start[r0:r1, None] + torch.arange(wm, device=dev, dtype=torch.int64)[None, :]
        rows[pos.reshape(-1)] = words.reshape(-1)
        rank = torch.cumsum(nz.to(torch.int64), dim=1) - 1                                   # rank of a non-zero in its row
        vpos = (start[r0:r1, None] + wm + rank)[nz]
        rows[vpos] = x[nz].view(torch.int32)
    return rows, start


def normal_vector(n, sigma, seed, device="cpu", dtype=torch.float32):
    g = _gen(seed, device)
    return (torch.randn(n, generator=g, device=device, dtype=torch.float32) * sigma).to(dtype)


def normal_matrix(rows, cols, sigma, seed, device="cpu", dtype=torch.float32):
    g = _gen(seed, device)
    return (torch.randn((rows, cols), generator=g, device=device, dtype=torch.float32) * sigma).to(dtype)


def pq_codebooks(M, K, dsub, seed, device="cpu", sigma=0.25):
    """M vocabularies of K centres of dsub dims, entries N(0, sigma^2) (sigma^2 = 1/16)."""
    g = _gen(seed, device)
    return torch.randn((M, K, dsub), generator=g, device=device, dtype=torch.float32) * sigma


def pq_codes(N, M, K, seed, device="cpu", chunk_rows=1 << 20):
    """Uniform codes in [0, K), one byte per sub-block."""
    g = _gen(seed, device)
    out = torch.empty((N, M), dtype=torch.uint8, device=device)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        out[r0:r1] = torch.randint(0, K, (r1 - r0, M), generator=g, device=device, dtype=torch.uint8)
    return out


def pack_sign_bits(features):
    """bit = 1 iff feature > 0; dimension d -> bit (d % 32) of word (d // 32). Returns int32
    words (the same 32 bits an unsigned word would hold)."""
    N, D = features.shape
    assert D % 32 == 0
    b = (features > 0).to(torch.int64).reshape(N, D // 32, 32)
    weights = (torch.ones(32, dtype=torch.int64, device=features.device) << torch.arange(32, device=features.device))
    words = (b * weights).sum(dim=2)                       # in [0, 2^32)
    words = torch.where(words >= 2 ** 31, words - 2 ** 32, words)
    return words.to(torch.int32)


def binary_bits_from_features(N, D, seed, device="cpu"):
    """Sign bits of N(0,1) features, packed (small sizes; draws the features explicitly)."""
    g = _gen(seed, device)
    f = torch.randn((N, D), generator=g, device=device, dtype=torch.float32)
    return pack_sign_bits(f)


def binary_bits_random(N, words, seed, device="cpu", chunk_rows=1 << 20):
    """Independent fair bits drawn directly as random 32-bit words: the same distribution as
    the signs of i.i.d. N(0,1) features, without materialising 32 floats per word."""
    g = _gen(seed, device)
    out = torch.empty((N, words), dtype=torch.int32, device=device)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        out[r0:r1] = torch.randint(-2 ** 31, 2 ** 31, (r1 - r0, words), generator=g,
                                   device=device, dtype=torch.int64).to(torch.int32)
    return out


def sgd_pools(D, n_pos, n_neg, seed, device="cpu", shift=0.5, n_shift_dims=50):
    """Negatives: the base feature distribution.  Positives: |N(0,1)| plus `shift` on one
    fixed random set of `n_shift_dims` dimensions (the class signal), then L2-normalised."""
    g = _gen(seed, device)
    neg = torch.randn((n_neg, D), generator=g, device=device, dtype=torch.float32).abs_()
    neg /= neg.norm(dim=1, keepdim=True)
    pos = torch.randn((n_pos, D), generator=g, device=device, dtype=torch.float32).abs_()
    dims = torch.randperm(D, generator=g, device=device)[:n_shift_dims]
    pos[:, dims] += shift
    pos /= pos.norm(dim=1, keepdim=True)
    return pos.contiguous(), neg.contiguous()


def sgd_batches(n_pos_pool, n_neg_pool, batch, steps, seed):
    """Index schedule of one training pass: per step batch/2 positives drawn uniformly with
    replacement and batch/2 negatives taken from one fixed permutation of the pool (each
    negative visited at most once per pass).  Returns int32 arrays (steps, batch/2) x 2."""
    rng = np.random.Generator(np.random.Philox(int(seed)))
    half = batch // 2
    pos = rng.integers(0, n_pos_pool, size=(steps, half), dtype=np.int64).astype(np.int32)
    perm = rng.permutation(n_neg_pool)
    reps = -(-steps * half // n_neg_pool)
    neg = np.concatenate([perm] * reps)[: steps * half].reshape(steps, half).astype(np.int32)
    return pos, neg


def onthefly_schedule(rounds, steps_per_round, batch, n_pos_start, pos_per_round, n_pos_total, n_neg_pool, seed):
    """Index schedule of an on-the-fly query (Sec. 4 "On-line (GPU back-end)": training starts with
    the first positives and the pool of positives keeps growing while the model is trained and the
    dataset re-ranked at intervals).  Round r trains `steps_per_round` steps on the first
    min(n_pos_total, n_pos_start + r * pos_per_round) positives of the pool, each batch half
    positives, half negatives, all drawn uniformly with replacement; a ranking follows each round.
    Returns (pool_sizes [rounds], idx_pos [rounds, steps, batch/2], idx_neg [same]) as numpy int32."""
    rng = np.random.Generator(np.random.Philox(int(seed)))
    half = batch // 2
    sizes = np.minimum(n_pos_total, n_pos_start + pos_per_round * np.arange(rounds)).astype(np.int32)
    pos = np.stack([rng.integers(0, int(p), size=(steps_per_round, half), dtype=np.int64) for p in sizes]).astype(np.int32)
    neg = rng.integers(0, n_neg_pool, size=(rounds, steps_per_round, half), dtype=np.int64).astype(np.int32)
    return sizes, pos, neg


def centred_descriptors(N, m, seed, device="cpu", chunk_rows=65536):
    """Descriptors for the binarisation encoder (Sec. 3 "Binarization": the descriptors are centred on zero first):
    the dense features above with one constant per dimension subtracted, the mean of a fixed
    seeded sample of 4096 such rows (a stand-in for the mean of a training set)."""
    centre = dense_features(4096, m, seed + 7919, device=device).mean(dim=0, keepdim=True)
    out = dense_features(N, m, seed, device=device, chunk_rows=chunk_rows)
    for r0 in range(0, N, chunk_rows):
        out[r0:r0 + chunk_rows] -= centre
    return out


def random_square(n, seed, device="cpu"):
    """The random n x n matrix whose QR decomposition gives the encoder's frame: N(0,1) entries, fp32."""
    return torch.randn((n, n), generator=_gen(seed, device), device=device, dtype=torch.float32)


def as_uint32(words_int32_numpy):
    return np.ascontiguousarray(words_int32_numpy).view(np.uint32)
