"""The no-allocation entry point (otf_rank_dense_noalloc: the library's own static scratch instead
of a caller workspace) against otf_rank_dense, through the C ABI: identical lists on two calls in a
row, the second on a smaller input, for a wide-row store (scores materialised, full selection) and
for a narrow-row store large enough for the filtered route; the size limit; and that the lists
match the oracle.  Collected last: the calls share one scratch array per GPU."""
import numpy as np
import pytest
import torch

from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = synth.BASE_SEED + 7000


def _pair(X, w, b, k):
    """(lists from otf_rank_dense on a fresh workspace, lists from the no-allocation entry point)."""
    N = X.shape[0]
    ws = binding.make_workspace(N, k)
    ref = binding.rank_dense(X, w, b, k, ws)
    out = binding._outputs(1, k, DEV)
    out[0].fill_(float("nan"))
    out[1].fill_(-1)
    got = binding.rank_dense_noalloc(X, w, b, k, out)
    torch.cuda.synchronize()
    return ref, got


@pytest.mark.parametrize("sizes,D,dtype", [(((150000, 1000), (20011, 100)), 2048, torch.float32),
                                           (((1300003, 1000), (90001, 37)), 128, torch.float32),
                                           (((2200000, 512), (1100000, 1)), 64, torch.float16)])
def test_two_calls_in_a_row_match_the_workspace_entry_point(oracle, sizes, D, dtype):
    w = synth.normal_vector(D, 0.05, SEED + 1).to(DEV)
    b = synth.normal_vector(1, 1.0, SEED + 2).to(DEV)
    for i, (N, k) in enumerate(sizes):                       # the second call is the smaller one
        X = synth.dense_features(N, D, SEED + 10 + i, device=DEV, dtype=dtype)
        (rs, ri), (gs, gi) = _pair(X, w, b, k)
        assert torch.equal(ri, gi) and torch.equal(rs, gs), "call %d (N=%d)" % (i, N)
        ref = oracle.dense_scores(X.cpu().numpy(), w.cpu().numpy(), b.cpu().numpy())[0]
        ok, msg = oracle.topk_parity_ok(ref, k, gi[0].cpu().numpy(), gs[0].cpu().numpy(),
                                        1e-4 if dtype == torch.float32 else 2e-3)
        assert ok, msg


def test_all_scores_and_several_classifiers():
    N, D, Q, k = 40000, 256, 3, 50
    X = synth.dense_features(N, D, SEED + 20, device=DEV)
    W = synth.normal_matrix(Q, D, 0.05, SEED + 21, device=DEV)
    ws = binding.make_workspace(N, k, Q)
    a_ref = torch.empty((Q, N), dtype=torch.float32, device=DEV)
    a_got = torch.empty((Q, N), dtype=torch.float32, device=DEV)
    ref = binding.rank_dense(X, W, None, k, ws, all_scores=a_ref)
    got = binding.rank_dense_noalloc(X, W, None, k, binding._outputs(Q, k, DEV), all_scores=a_got)
    torch.cuda.synchronize()
    assert torch.equal(ref[0], got[0]) and torch.equal(ref[1], got[1]) and torch.equal(a_ref, a_got)


def test_sizes_beyond_the_static_scratch_are_rejected_and_nothing_is_written():
    D, k = 16, 10
    N = 1
    while binding.workspace_bytes(N, k, 1) <= binding.OTF_NOALLOC_SCRATCH_BYTES:
        N *= 2
    X = torch.zeros((N, D), dtype=torch.float32, device=DEV)
    w = torch.zeros(D, dtype=torch.float32, device=DEV)
    out = binding._outputs(1, k, DEV)
    out[1].fill_(-7)
    with pytest.raises(binding.OtfError) as err:
        binding.rank_dense_noalloc(X, w, None, k, out)
    assert err.value.status == binding.OTF_ERR_SCRATCH
    torch.cuda.synchronize()
    assert bool((out[1] == -7).all())
    # the largest size that fits still works
    N2 = N // 2
    got = binding.rank_dense_noalloc(X[:N2], w, None, k, out)
    torch.cuda.synchronize()
    assert got[1][0].cpu().tolist() == list(range(k))        # all scores equal: lowest rows first
