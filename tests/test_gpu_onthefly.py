"""GPU parity of the on-the-fly loop (paper Sec. 4, "On-line (GPU back-end)": training continues on a
growing pool while the store is re-ranked at intervals) with the sequential CPU oracle.

What is compared: (a) every ranking against the oracle's ranking under the very model the GPU
ranked with (its fp32 snapshot), by the top-k parity rule; (b) every round of training against
the oracle started from the GPU's previous snapshot; (c) the free-running oracle's final model,
loosely (fp32 training drifts); (d) the two-stream run against the same calls on one stream:
bit-identical, i.e. the snapshots make the result independent of how the streams interleave."""
import numpy as np
import pytest
import torch

from oracle import otf_loop
from paper_1407_4764_amd import binding, onthefly, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = synth.BASE_SEED + 3000


@pytest.mark.parametrize("N,D,B,lam,rounds,steps", [(20000, 128, 32, 1.0, 6, 25), (6000, 2048, 256, 1e-4, 4, 15)])
def test_loop_matches_the_oracle(oracle, N, D, B, lam, rounds, steps):
    k = 100
    X = synth.dense_features(N, D, SEED + 1)
    pos, neg = synth.sgd_pools(D, 200, 2000, SEED + 2)
    X[:50] = pos[150:200]                                          # some store rows look like the query class
    sizes, ip, ineg = synth.onthefly_schedule(rounds, steps, B, 8, 12, 150, 2000, SEED + 3)
    args = (X.to(DEV), pos.to(DEV), neg.to(DEV), torch.from_numpy(ip).to(DEV), torch.from_numpy(ineg).to(DEV), k, lam)
    out = onthefly.run(*args, overlap=True)
    seq = onthefly.run(*args, overlap=False)
    for key in ("idx", "val", "w"):
        assert torch.equal(out[key], seq[key]), key               # (d)
    w_gpu = out["w"].cpu().numpy()
    idx, val = out["idx"].cpu().numpy(), out["val"].cpu().numpy()
    Xn, posn, negn = X.numpy(), pos.numpy(), neg.numpy()
    t = 0
    for r in range(rounds):
        # (a) the ranking of round r under the GPU's own snapshot
        ref = oracle.dense_scores(Xn, w_gpu[r])[0]
        ok, msg = oracle.topk_parity_ok(ref, k, idx[r], val[r], 1e-4)
        assert ok, "round %d: %s" % (r, msg)
        # (b) the training of round r, started from the GPU's previous snapshot
        w = np.zeros(D) if r == 0 else w_gpu[r - 1].astype(np.float64)
        for s in range(steps):
            t += 1
            w, _, _ = oracle.sgd_step(w, 0.0, posn, ip[r, s], negn, ineg[r, s], lam, t, False)
        scale = np.abs(w).max()
        assert np.max(np.abs(w_gpu[r] - w)) <= 2e-4 * scale, "round %d" % r
    # (c) free-running oracle
    w_ref, idx_ref, _, _ = otf_loop.run(Xn, posn, negn, ip, ineg, k, lam)
    assert np.max(np.abs(w_gpu[-1] - w_ref[-1])) <= 2e-3 * np.abs(w_ref[-1]).max()
    common = np.intersect1d(idx[-1], idx_ref[-1]).size
    assert common >= k - 3
    assert set(range(50)) & set(idx[-1].tolist())                  # the planted class rows reach the list
    assert all(ms > 0 for ms in out["rank_ms"])
