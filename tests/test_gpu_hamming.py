"""GPU parity of Hamming ranking (paper Sec. 3.1, discussion after Table 2) with the CPU oracle.
Distances are integers: every score must equal the oracle's bit count exactly, and the list must be
the oracle's, ties by ascending row included (distances take few values, so ties are everywhere)."""
import numpy as np
import pytest
import torch

from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = synth.BASE_SEED + 9000


def _check(oracle, bits, D, query, k, expect_filter=None):
    N = bits.shape[0]
    ref = oracle.hamming_scores(synth.as_uint32(bits.numpy()), D, synth.as_uint32(query.numpy()))
    ws = binding.make_workspace(N, k)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    bd, qd = bits.to(DEV), query.to(DEV)
    val, idx = binding.rank_hamming(bd, D, qd, k, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(all_scores.cpu().numpy().astype(np.float64), ref)
    i, v = oracle.topk(ref, k)
    np.testing.assert_array_equal(idx[0].cpu().numpy(), i)
    np.testing.assert_array_equal(val[0].cpu().numpy().astype(np.float64), v)
    val2, idx2 = binding.rank_hamming(bd, D, qd, k, ws)             # no score output: the filtered route if large
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx2[0].cpu().numpy(), i)
    np.testing.assert_array_equal(val2[0].cpu().numpy().astype(np.float64), v)
    if expect_filter is not None:
        assert binding.debug_fallback_taken(ws) != expect_filter


@pytest.mark.parametrize("N,D,k", [(5000, 2048, 100), (1, 128, 1), (777, 128, 777), (3001, 256, 50), (2000, 512, 10),
                                   (1500, 1024, 64), (900, 4096, 9), (600, 8192, 30), (1300, 768, 13), (1100, 1536, 11),
                                   (1024 * 600 + 31, 2048, 1000), (2048 * 530 + 7, 1024, 100)])
def test_hamming_ranking_is_exact(oracle, N, D, k):
    bits = synth.binary_bits_random(N, D // 32, SEED + D)
    query = synth.binary_bits_random(1, D // 32, SEED + D + 1)[0]
    _check(oracle, bits, D, query, k)


def test_near_duplicates_of_the_query_rank_first(oracle):
    """Rows planted at distances 0, 1, 2, ... from the query come back first, in that order."""
    N, D, k = 20000, 2048, 40
    bits = synth.binary_bits_random(N, D // 32, SEED + 10)
    query = synth.binary_bits_random(1, D // 32, SEED + 11)[0]
    planted = [17, 5000, 19999, 3, 12345]
    for dist, row in enumerate(planted):
        r = query.clone()
        for d in range(dist):                                   # flip `dist` different bits
            r[(97 * d) % (D // 32)] ^= (1 << (d % 31))
        bits[row] = r
    _check(oracle, bits, D, query, k)
    ws = binding.make_workspace(N, k)
    val, idx = binding.rank_hamming(bits.to(DEV), D, query.to(DEV), k, ws)
    torch.cuda.synchronize()
    assert idx[0, :5].cpu().tolist() == planted and val[0, :5].cpu().tolist() == [0.0, -1.0, -2.0, -3.0, -4.0]


def test_large_store_takes_the_filtered_route(oracle):
    N, D, k = 1300000, 2048, 1000
    bits = synth.binary_bits_random(N, D // 32, SEED + 20)
    query = synth.binary_bits_random(1, D // 32, SEED + 21)[0]
    _check(oracle, bits, D, query, k, expect_filter=True)


def test_identical_rows_tie_by_row_index(oracle):
    """Every row equal: all distances equal, the list is rows 0..k-1 (the exact fallback behind the filter)."""
    N, D, k = 1200000, 256, 100
    query = synth.binary_bits_random(1, D // 32, SEED + 30)[0]
    bits = query[None, :].repeat(N, 1).contiguous()
    bits[:, 0] ^= 5
    _check(oracle, bits, D, query, k)


@pytest.mark.parametrize("spin_limit", [0, 1])
@pytest.mark.parametrize("N,D,k,free_bits", [(3_000_000, 128, 1000, 12), (2_200_000, 256, 1, 8), (1_300_000, 128, 1024, 6),
                                             (1_300_000, 128, 8192, 10)])
def test_ties_by_the_ten_thousand_at_the_kth_distance(oracle, N, D, k, free_bits, spin_limit, debug_switches):
    """Rows that differ from the query in a few bit positions only: millions of rows share a handful
    of distances and the k-th distance is shared by more rows than any candidate list holds.  The
    filtered scan is called off, and the full selection behind it must split the tie by row number
    with all its workgroups (passes 2 and 3 and the gather, between meeting points).  spin_limit = 1
    makes every wait at a meeting point give up at once: then one workgroup finishes alone, and the
    answer must be the same."""
    if spin_limit:
        debug_switches({binding.DEBUG_MEET_SPIN_LIMIT: spin_limit})
    g = torch.Generator().manual_seed(SEED + 20 + D)
    query = synth.binary_bits_random(1, D // 32, SEED + 21 + D)[0]
    bits = query.repeat(N, 1)
    bits[:, 1] ^= torch.randint(0, 1 << free_bits, (N,), generator=g, dtype=torch.int32)
    bits = bits.contiguous()
    ref = oracle.hamming_scores(synth.as_uint32(bits.numpy()), D, synth.as_uint32(query.numpy()))
    i, v = oracle.topk(ref, k)
    assert (ref == v[-1]).sum() > 8192                             # the tie the test is about
    ws = binding.make_workspace(N, k)
    val, idx = binding.rank_hamming(bits.to(DEV), D, query.to(DEV), k, ws)
    torch.cuda.synchronize()
    assert binding.debug_fallback_taken(ws) == (k <= 1024)          # longer lists never take the filtered route
    np.testing.assert_array_equal(idx[0].cpu().numpy(), i)
    np.testing.assert_array_equal(val[0].cpu().numpy().astype(np.float64), v)
