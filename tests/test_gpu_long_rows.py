"""GPU parity of the table scans on rows that do not fit one table image (more than 128 stored bytes:
PQ with 256 or 512 sub-blocks, which is the paper's own 4 or 8 dimensions per sub-block on 2048-D
features, Table 2; binary codes beyond 2048 bits) and on row lengths that are not a power of two
or not a multiple of 128 bytes.

Integer-valued tables and weights make every fp32 sum exact, so a row scored twice, skipped, scored
with the table image of another column phase or from another tile shows as a non-zero difference.
Sizes: stores long enough that every workgroup walks several blocks of 2048 rows through all
phases (more than 2 x 256 blocks), ragged ends (a last block of 1 row, of 63, of 64, one row short
of full), stores shorter than one tile, and stores large enough for the sampled, filtered route."""
import numpy as np
import pytest
import torch

from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = synth.BASE_SEED + 8000


def _int_lut(M, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randint(-1000, 1000, (M, 256), generator=g).to(torch.float32)


def _check_pq_exact(oracle, N, M, k, seed, tiles=None, debug_switches=None):
    codes = synth.pq_codes(N, M, 256, seed)
    lut = _int_lut(M, seed + 1)
    ref = oracle.pq_scores_lut(codes.numpy(), lut.numpy().astype(np.float64), 3.0)
    ws = binding.make_workspace(N, k)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    cd, ld = codes.to(DEV), lut.to(DEV)
    val, idx = binding.rank_pq(cd, ld, 3.0, k, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(all_scores.cpu().numpy().astype(np.float64), ref)
    i, v = oracle.topk(ref, k)
    np.testing.assert_array_equal(idx[0].cpu().numpy(), i)
    np.testing.assert_array_equal(val[0].cpu().numpy().astype(np.float64), v)
    # without the score output (the filtered route when the store is large enough) the list is the same
    val2, idx2 = binding.rank_pq(cd, ld, 3.0, k, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx2[0].cpu().numpy(), i)
    np.testing.assert_array_equal(val2[0].cpu().numpy().astype(np.float64), v)
    return ws


@pytest.mark.parametrize("N,M", [(2048 * 530 + 1, 256), (2048 * 530 + 63, 512), (2048 * 530 + 64, 512),
                                 (2048 * 531 - 1, 256), (2048 * 600, 512), (2048 * 520 + 700, 1024),
                                 (2048 * 515 + 65, 384)])
def test_long_pq_rows_every_row_scored_once_and_filtered_route(oracle, N, M):
    """More than a million rows: several blocks per workgroup, and the second call takes the
    sampled, filtered route (one launch over all column phases, nothing but candidates written)."""
    ws = _check_pq_exact(oracle, N, M, 100, SEED + M)
    assert not binding.debug_fallback_taken(ws)


@pytest.mark.parametrize("N,M", [(1, 256), (63, 512), (64, 256), (65, 512), (511, 640), (513, 256), (2047, 512),
                                 (2049, 512), (40000, 144), (30011, 192), (9000, 1024), (70000, 512)])
def test_long_pq_rows_small_and_ragged_stores(oracle, N, M):
    _check_pq_exact(oracle, N, M, min(N, 37), SEED + 100 + M)


@pytest.mark.parametrize("N,M", [(1, 48), (3000, 48), (5001, 80), (777, 96), (4100, 112), (1200007, 96)])
def test_pq_rows_whose_length_is_not_a_power_of_two(oracle, N, M):
    """Rows of 48..112 bytes occupy a span of 64 or 128 bytes of lanes; the lanes beyond the row must
    contribute nothing and must not read past the end of the store."""
    _check_pq_exact(oracle, N, M, min(N, 50), SEED + 200 + M)


@pytest.mark.parametrize("tiles", [4, 8])
def test_more_tiles_per_wave_give_the_same_scores(oracle, debug_switches, tiles):
    debug_switches({binding.DEBUG_WALK_TILES: tiles})
    _check_pq_exact(oracle, 1024 * tiles * 270 + 5, 512, 64, SEED + 300)
    _check_pq_exact(oracle, 5000, 256, 10, SEED + 301)
    _check_pq_exact(oracle, 70, 384, 10, SEED + 302)


@pytest.mark.parametrize("N,D", [(3000, 4096), (1100, 8192), (5000, 1536), (2500, 768), (700, 384), (1300000, 4096),
                                 (1200000, 1536), (100, 3072)])
def test_binary_rows_of_any_multiple_of_128_bits(oracle, N, D):
    """Every D that is a multiple of 128 bits (2048 keeps its one-image layout): byte groups, one
    phase per 1024 bits, a narrower last phase for 1536 or 3072 bits."""
    k = min(N, 40)
    bits = synth.binary_bits_random(N, D // 32, SEED + 400 + D)
    g = torch.Generator().manual_seed(SEED + 401 + D)
    w = torch.randint(-512, 512, (D,), generator=g).to(torch.float32)
    ref = oracle.binary_scores(synth.as_uint32(bits.numpy()), D, w.numpy(), 1.0)
    ws = binding.make_workspace(N, k)
    all_scores = torch.empty(N, dtype=torch.float32, device=DEV)
    bd, wd = bits.to(DEV), w.to(DEV)
    binding.rank_binary(bd, D, wd, 1.0, k, ws, all_scores=all_scores)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(all_scores.cpu().numpy().astype(np.float64), ref)
    val2, idx2 = binding.rank_binary(bd, D, wd, 1.0, k, ws)
    torch.cuda.synchronize()
    i, v = oracle.topk(ref, k)
    np.testing.assert_array_equal(idx2[0].cpu().numpy(), i)
    np.testing.assert_array_equal(val2[0].cpu().numpy().astype(np.float64), v)


@pytest.mark.parametrize("N,M,dsub", [(1300001, 512, 4), (1200000, 256, 8)])
def test_paper_pq_geometries_against_the_reconstruction_oracle(oracle, N, M, dsub):
    """The paper's 2048-D features at 4 and 8 dimensions per sub-block, real-valued vocabularies:
    table build + ranking against the dot product with the reconstructed rows."""
    k = 1000
    cb = synth.pq_codebooks(M, 256, dsub, SEED + 500)
    codes = synth.pq_codes(N, M, 256, SEED + 501)
    w = synth.normal_vector(M * dsub, 1.0, SEED + 502)
    lut = binding.pq_build_lut(cb.to(DEV), w.to(DEV))
    ws = binding.make_workspace(N, k)
    val, idx = binding.rank_pq(codes.to(DEV), lut, 0.25, k, ws)
    torch.cuda.synchronize()
    assert not binding.debug_fallback_taken(ws)
    ref = oracle.pq_scores_reconstruct(codes.numpy(), cb.numpy(), w.numpy(), 0.25)
    ok, msg = oracle.topk_parity_ok(ref, k, idx[0].cpu().numpy(), val[0].cpu().numpy(), 1e-4)
    assert ok, msg


@pytest.mark.parametrize("N,M,dsub", [(30000, 128, 16), (5000, 512, 4), (1200000, 256, 8), (4000, 96, 4), (2000, 16, 8)])
def test_ranking_straight_from_the_vocabularies_equals_table_build_plus_ranking(N, M, dsub):
    """otf_rank_pq_model must give the bits of otf_pq_build_lut followed by otf_rank_pq."""
    k = min(N, 100)
    cb = synth.pq_codebooks(M, 256, dsub, SEED + 600).to(DEV)
    codes = synth.pq_codes(N, M, 256, SEED + 601).to(DEV)
    w = synth.normal_vector(M * dsub, 1.0, SEED + 602).to(DEV)
    ws = binding.make_workspace(N, k)
    a1 = torch.empty(N, dtype=torch.float32, device=DEV)
    a2 = torch.empty(N, dtype=torch.float32, device=DEV)
    v1, i1 = binding.rank_pq(codes, binding.pq_build_lut(cb, w), -0.5, k, ws, all_scores=a1)
    v1, i1 = v1.clone(), i1.clone()
    v2, i2 = binding.rank_pq_model(codes, cb, w, -0.5, k, ws, all_scores=a2)
    torch.cuda.synchronize()
    assert torch.equal(a1, a2) and torch.equal(i1, i2) and torch.equal(v1, v2)
    v3, i3 = binding.rank_pq_model(codes, cb, w, -0.5, k, ws)          # and on the filtered route
    torch.cuda.synchronize()
    assert torch.equal(i1, i3) and torch.equal(v1, v3)


@pytest.mark.parametrize("M", [512, 272])
def test_long_rows_fall_back_when_the_list_cannot_serve(oracle, M):
    """Rows of several table images behind a failed filtered scan: under a zero model every score is
    the bias (rows 0..k-1); with 10,000 maximal rows outside every sampled group the list overflows
    and the full selection splits the tie by row."""
    N, k, dsub = 1150000, 500, 4
    cb = synth.pq_codebooks(M, 256, dsub, SEED + 600)
    codes = synth.pq_codes(N, M, 256, SEED + 601)
    ws = binding.make_workspace(N, k)
    cd, cbd = codes.to(DEV), cb.to(DEV)
    val, idx = binding.rank_pq_model(cd, cbd, torch.zeros(M * dsub, device=DEV), 0.75, k, ws)
    assert binding.debug_fallback_taken(ws)
    np.testing.assert_array_equal(idx[0].cpu().numpy(), np.arange(k))
    assert torch.all(val[0] == 0.75)

    w = synth.normal_vector(M * dsub, 1.0, SEED + 602)
    lut = binding.pq_build_lut(cbd, w.to(DEV))
    codes[2048:12048] = lut.argmax(dim=1).to(torch.uint8).cpu()          # the best code of every sub-block
    cd = codes.to(DEV)
    val, idx = binding.rank_pq(cd, lut, 0.0, k, ws)
    assert binding.debug_fallback_taken(ws)
    np.testing.assert_array_equal(idx[0].cpu().numpy(), np.arange(2048, 2048 + k))
    ref = oracle.pq_scores_reconstruct(codes[2048:2049].numpy(), cb.numpy(), w.numpy(), 0.0)
    assert abs(float(val[0, 0]) - ref[0]) <= 1e-4 * abs(ref[0]) and torch.all(val[0] == val[0, 0])
