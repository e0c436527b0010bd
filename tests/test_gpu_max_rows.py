"""The largest sizes the interface admits: N = 2^31 - 1 rows (row indices are int32) of 16- and
32-byte rows, a sparse-row store whose word offsets pass 2^32, and 65535 classifiers in one call.

The oracle cannot score two thousand million rows in test time, so the expected list is PLANTED:
1200 rows, spread over the store with its first and last rows among them, are built to score above
anything a generated row can reach, and the oracle scores exactly those (plus the rows returned and a
random sample of the others, one by one).  Why no generated row can reach the list is stated per
store; where every score is written out the test also counts the scores at or above the k-th."""
import numpy as np
import pytest
import torch

from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
N = (1 << 31) - 1
K = 1000
PLANTED = 1200


def _planted_positions(n_rows, seed=4764):
    """Ascending rows of the store that receive planted content: its ends, the borders of tiles and
    chunks next to them, the middle, and random rows."""
    rng = np.random.default_rng(seed)
    fixed = sorted({0, 1, 63, 64, 511, 512, 513, (1 << 20) - 1, 1 << 20, n_rows // 2 - 1, n_rows // 2, n_rows // 2 + 1,
                    n_rows - 513, n_rows - 512, n_rows - 511, n_rows - 65, n_rows - 64, n_rows - 2, n_rows - 1})
    rest = [int(p) for p in rng.choice(n_rows, PLANTED, replace=False) if int(p) not in set(fixed)]
    pos = np.sort(np.array(fixed + rest[:PLANTED - len(fixed)], dtype=np.int64))
    assert np.unique(pos).size == PLANTED and pos[0] == 0 and pos[-1] == n_rows - 1
    return pos


def _dev_index(rows):
    return torch.from_numpy(np.asarray(rows, dtype=np.int64)).to(DEV)


def _check_planted(oracle, pos, planted_ref, val, idx, rtol, what):
    """The returned rows are planted ones, and rank among the planted rows as the oracle ranks them
    (`pos` ascends, so ties go to the lower row on both sides)."""
    got = idx[0].cpu().numpy().astype(np.int64)
    at = np.searchsorted(pos, got)
    assert np.all(at < PLANTED) and np.array_equal(pos[np.minimum(at, PLANTED - 1)], got), what + ": a row that was not planted came back"
    ok, msg = oracle.topk_parity_ok(planted_ref, K, at, val[0].cpu().numpy(), rtol)
    assert ok, what + ": " + msg


def _sample_rows(n_rows):
    return np.concatenate([np.arange(2048), np.arange(n_rows - 2048, n_rows), np.random.default_rng(5).choice(n_rows, 20000, replace=False)])


def test_hamming_and_topk_at_the_largest_row_count(oracle):
    """128-bit codes.  Planted: the query with 0 .. 11 of its bits flipped, a hundred rows per distance.
    A random 128-bit row lies 64 +- 5.7 bits from the query; that one of 2^31 comes within 11 bits has
    probability below 1e-20."""
    D = 128
    bits = synth.binary_bits_random(N, D // 32, 31, device=DEV)            # 34 GB
    query = synth.binary_bits_random(1, D // 32, 32, device=DEV)[0].contiguous()
    pos = _planted_positions(N)
    flips = np.random.default_rng(6).permutation(np.arange(PLANTED) // 100)   # 0 .. 11 bits, a hundred rows each
    rows = query.cpu().numpy()[None, :].repeat(PLANTED, axis=0).copy()
    rows[:, 0] ^= ((1 << flips) - 1).astype(np.int32)                      # the lowest `flips` bits of the first word
    bits[_dev_index(pos)] = torch.from_numpy(rows).to(DEV)
    qn = synth.as_uint32(query.cpu().numpy())

    def oracle_rows(r):
        return oracle.hamming_scores(synth.as_uint32(bits[_dev_index(r)].cpu().numpy()), D, qn)

    ref = oracle_rows(pos)
    np.testing.assert_array_equal(ref, -flips.astype(np.float64))
    want_at, want_scores = oracle.topk(ref, K)
    want_rows = pos[want_at]

    def exact(val, idx):
        np.testing.assert_array_equal(idx[0].cpu().numpy().astype(np.int64), want_rows)
        np.testing.assert_array_equal(val[0].cpu().numpy().astype(np.float64), want_scores)

    ws = binding.make_workspace(N, K)
    exact(*binding.rank_hamming(bits, D, query, K, ws))                    # sampled and filtered
    scores = torch.empty(N, dtype=torch.float32, device=DEV)
    exact(*binding.rank_hamming(bits, D, query, K, ws, all_scores=scores))  # every score, full selection
    sample = _sample_rows(N)
    np.testing.assert_array_equal(scores[_dev_index(sample)].cpu().numpy().astype(np.float64), oracle_rows(sample))
    assert int((scores >= float(want_scores[-1])).sum().item()) == int((ref >= want_scores[-1]).sum())
    exact(*binding.topk(scores.view(1, N), K, ws))                          # ready-made scores, one read


def test_pq_codes_at_the_largest_row_count(oracle):
    """16-byte PQ codes (M = 16, 4 dimensions per sub-block).  Planted: the best code of every
    sub-block, except that row i takes the code ranked 1 + i div 16 in sub-block i mod 16.  A
    generated row reaches such a score only with nearly every one of its 16 random codes among the
    best few of 256: probability below 1e-25 per row."""
    M, dsub = 16, 4
    cb = synth.pq_codebooks(M, 256, dsub, 41)
    w = synth.normal_vector(M * dsub, 1.0, 42)
    lut = np.einsum("mkd,md->mk", cb.numpy().astype(np.float64), w.numpy().astype(np.float64).reshape(M, dsub))
    by_rank = np.argsort(-lut, axis=1)                                     # by_rank[m][j] = j-th best code of sub-block m
    codes = synth.pq_codes(N, M, 256, 43, device=DEV)                      # 34 GB
    pos = _planted_positions(N)
    which = np.random.default_rng(7).permutation(PLANTED)
    rows = np.repeat(by_rank[:, 0][None, :], PLANTED, axis=0).astype(np.uint8)
    rows[np.arange(PLANTED), which % M] = by_rank[which % M, 1 + which // M].astype(np.uint8)
    codes[_dev_index(pos)] = torch.from_numpy(rows).to(DEV)

    def oracle_rows(r):
        return oracle.pq_scores_reconstruct(codes[_dev_index(r)].cpu().numpy(), cb.numpy(), w.numpy(), 0.5)

    ref = oracle_rows(pos)
    ws = binding.make_workspace(N, K)
    val, idx = binding.rank_pq_model(codes, cb.to(DEV), w.to(DEV), 0.5, K, ws)
    _check_planted(oracle, pos, ref, val, idx, 1e-4, "pq, filtered")
    scores = torch.empty(N, dtype=torch.float32, device=DEV)
    val, idx = binding.rank_pq_model(codes, cb.to(DEV), w.to(DEV), 0.5, K, ws, all_scores=scores)
    _check_planted(oracle, pos, ref, val, idx, 1e-4, "pq, every score")
    sample = _sample_rows(N)
    want = oracle_rows(sample)
    assert np.all(np.abs(scores[_dev_index(sample)].cpu().numpy() - want) <= oracle.score_tolerance(want, 1e-4))
    assert int((scores >= float(val[0, -1])).sum().item()) == K


def test_dense_rows_at_the_largest_row_count(oracle):
    """8-D fp32 rows (32 bytes, a 69 GB store).  Generated rows have unit length, so none scores above
    |w| + b (Cauchy-Schwarz); planted row i is the multiple of w that scores 10 + i / 50, and |w| + b
    is checked to lie below 10."""
    D = 8
    X = synth.dense_features(N, D, 51, device=DEV, chunk_rows=1 << 24)
    w = synth.normal_vector(D, 1.0, 52)
    b = synth.normal_vector(1, 1.0, 53)
    wn = w.numpy().astype(np.float64)
    assert np.linalg.norm(wn) + abs(float(b[0])) < 9.0
    pos = _planted_positions(N)
    target = 10.0 + np.random.default_rng(8).permutation(PLANTED) / 50.0
    rows = ((target - float(b[0])) / np.dot(wn, wn))[:, None] * wn[None, :]
    X[_dev_index(pos)] = torch.from_numpy(rows.astype(np.float32)).to(DEV)

    def oracle_rows(r):
        return oracle.dense_scores(X[_dev_index(r)].cpu().numpy(), w.numpy(), b.numpy())[0]

    ref = oracle_rows(pos)
    ws = binding.make_workspace(N, K)
    val, idx = binding.rank_dense(X, w.to(DEV), b.to(DEV), K, ws)
    _check_planted(oracle, pos, ref, val, idx, 1e-4, "dense, filtered")
    scores = torch.empty(N, dtype=torch.float32, device=DEV)
    val, idx = binding.rank_dense(X, w.to(DEV), b.to(DEV), K, ws, all_scores=scores)
    _check_planted(oracle, pos, ref, val, idx, 1e-4, "dense, every score")
    sample = _sample_rows(N)
    want = oracle_rows(sample)
    assert np.all(np.abs(scores[_dev_index(sample)].cpu().numpy() - want) <= oracle.score_tolerance(want, 1e-4))
    assert int((scores >= float(val[0, -1])).sum().item()) == K


def test_sparse_store_with_offsets_past_32_bits(oracle):
    """80 million sparse 128-D rows, three fifths zeros: 4.4e9 words, so the offsets of the last rows
    do not fit 32 bits.  Unit-length generated rows score at most |w| + b; planted row i is the
    multiple of w's positive part (its other entries stay zero) that scores 40 + i / 50."""
    D, rows_n = 128, 80_000_000
    X = synth.sparse_features(rows_n, D, 61, device=DEV, chunk_rows=1 << 20)
    w = synth.normal_vector(D, 1.0, 62)
    bias = 0.125
    wn = w.numpy().astype(np.float64)
    assert np.linalg.norm(wn) + bias < 39.0
    pos = _planted_positions(rows_n)
    target = 40.0 + np.random.default_rng(9).permutation(PLANTED) / 50.0
    wplus = np.maximum(wn, 0.0)
    planted = ((target - bias) / np.dot(wplus, wplus))[:, None] * wplus[None, :]
    X[_dev_index(pos)] = torch.from_numpy(planted.astype(np.float32)).to(DEV)
    rows, start = synth.sparse_rows_from_dense(X)
    assert int(start[pos[-10]].item()) > 1 << 32                          # planted rows lie beyond it too

    def oracle_rows(r):
        return oracle.dense_scores(X[_dev_index(r)].cpu().numpy(), w.numpy(), np.array([bias], np.float32))[0]

    ref = oracle_rows(pos)
    ws = binding.make_workspace(rows_n, K)
    val, idx = binding.rank_sparse(rows, start, D, w.to(DEV), bias, K, ws)
    _check_planted(oracle, pos, ref, val, idx, 1e-4, "sparse, filtered")
    scores = torch.empty(rows_n, dtype=torch.float32, device=DEV)
    val, idx = binding.rank_sparse(rows, start, D, w.to(DEV), bias, K, ws, all_scores=scores)
    _check_planted(oracle, pos, ref, val, idx, 1e-4, "sparse, every score")
    sample = _sample_rows(rows_n)
    want = oracle_rows(sample)
    assert np.all(np.abs(scores[_dev_index(sample)].cpu().numpy() - want) <= oracle.score_tolerance(want, 1e-4))
    assert int((scores >= float(val[0, -1])).sum().item()) == K


@pytest.mark.parametrize("half,Q,n_rows,D,k", [(False, 65535, 48, 16, 3), (True, 65504, 130, 128, 5)])
def test_largest_classifier_count(oracle, half, Q, n_rows, D, k):
    """65535 classifiers over a small store: one scan per classifier in fp32, the matrix-core scan
    (classifier counts that are multiples of 32) in fp16; then otf_topk over the Q x N scores."""
    dt = torch.float16 if half else torch.float32
    rtol = 2e-3 if half else 1e-4
    X = synth.dense_features(n_rows, D, 71, dtype=dt)
    W = synth.normal_matrix(Q, D, 0.5, 72, dtype=dt)
    ref = oracle.dense_scores(X.numpy(), W.numpy())
    ws = binding.make_workspace(n_rows, k, Q)
    scores = torch.empty((Q, n_rows), dtype=torch.float32, device=DEV)
    val, idx = binding.rank_dense(X.to(DEV), W.to(DEV), None, k, ws, all_scores=scores)
    val2, idx2 = binding.topk(scores, k, ws)
    torch.cuda.synchronize()
    assert torch.equal(val, val2) and torch.equal(idx, idx2)
    got = scores.cpu().numpy()
    val, idx = val.cpu().numpy(), idx.cpu().numpy()
    for q in range(Q):
        assert np.all(np.abs(got[q] - ref[q]) <= oracle.score_tolerance(ref[q], rtol)), "classifier %d" % q
    for q in list(range(0, Q, 997)) + [Q - 2, Q - 1]:
        ok, msg = oracle.topk_parity_ok(ref[q], k, idx[q], val[q], rtol)
        assert ok, "classifier %d: %s" % (q, msg)
    # every list is the first k of a full sort of the GPU's own scores (score descending, row ascending)
    order = np.lexsort((np.broadcast_to(np.arange(n_rows), got.shape), -got.astype(np.float64)), axis=1)[:, :k]
    np.testing.assert_array_equal(idx, order)
    np.testing.assert_array_equal(val, np.take_along_axis(got, order, axis=1))
