"""Pins for the on-the-fly loop oracle (paper Sec. 4, "On-line (GPU back-end)"): closed forms of the
Pegasos recursion that hold across rounds, and numpy's own sort for the rankings.  CPU only."""
import numpy as np

from oracle import otf_loop
from paper_1407_4764_amd import synth


def _pools(D, n_pos, n_neg, seed):
    pos, neg = synth.sgd_pools(D, n_pos, n_neg, seed)
    return pos.numpy(), neg.numpy()


def test_first_step_closed_form_and_ranking_by_numpy():
    """w_0 = 0: every row of the first batch violates the margin, so after one step
    w_1 = (sum of its positives - sum of its negatives) / (lambda B); the ranking that follows is
    numpy's descending sort of X w_1."""
    D, lam, B, k = 64, 0.5, 8, 20
    pos, neg = _pools(D, 30, 40, 1)
    X = synth.dense_features(500, D, 2).numpy()
    _, ip, ineg = synth.onthefly_schedule(1, 1, B, 30, 0, 30, 40, 3)
    w, idx, val, sc = otf_loop.run(X, pos, neg, ip, ineg, k, lam)
    w1 = (pos[ip[0, 0]].astype(np.float64).sum(0) - neg[ineg[0, 0]].astype(np.float64).sum(0)) / (lam * B)
    np.testing.assert_allclose(w[0], w1, rtol=1e-12)
    s = X.astype(np.float64) @ w1.astype(np.float32).astype(np.float64)
    order = np.lexsort((np.arange(500), -s))[:k]
    np.testing.assert_array_equal(idx[0], order)
    np.testing.assert_allclose(val[0], s[order], rtol=1e-12)


def test_step_counter_runs_through_the_rounds():
    """With a tiny lambda the first step makes w huge, no row ever violates again, and each later
    step only shrinks w by (1 - 1/t): after T steps in all w = w_1 / T, whatever the split into
    rounds -- a counter restarted per round would wipe w at every round's first step.  Scaling w
    does not change a ranking, so no list changes after the first."""
    D, lam, B, k = 32, 1e-6, 8, 15
    rng = np.random.default_rng(4)
    u = rng.standard_normal(D)
    u /= np.linalg.norm(u)
    pos = (u[None, :] + 0.05 * rng.standard_normal((20, D))).astype(np.float32)     # two tight, opposite clusters:
    neg = (-u[None, :] + 0.05 * rng.standard_normal((20, D))).astype(np.float32)    # w_1 separates them by ~1/lambda
    X = synth.dense_features(300, D, 5).numpy()
    rounds, steps = 4, 5
    _, ip, ineg = synth.onthefly_schedule(rounds, steps, B, 20, 0, 20, 20, 6)
    w, idx, val, _ = otf_loop.run(X, pos, neg, ip, ineg, k, lam)
    w1 = (pos[ip[0, 0]].astype(np.float64).sum(0) - neg[ineg[0, 0]].astype(np.float64).sum(0)) / (lam * B)
    for r in range(rounds):
        T = (r + 1) * steps
        np.testing.assert_allclose(w[r], w1 / T, rtol=1e-5)      # w is rounded to fp32 after every step
    for r in range(1, rounds):
        np.testing.assert_array_equal(idx[r], idx[0])
    np.testing.assert_array_equal(otf_loop.churn(idx), [k, 0, 0, 0])


def test_pool_grows_as_scheduled():
    sizes, ip, _ = synth.onthefly_schedule(6, 10, 32, 4, 3, 15, 100, 7)
    np.testing.assert_array_equal(sizes, [4, 7, 10, 13, 15, 15])
    for r in range(6):
        assert ip[r].max() < sizes[r] and ip[r].min() >= 0
    assert ip[5].max() > 12                                       # the late rounds do use the new rows


def test_churn_counts_new_rows():
    idx = np.array([[1, 2, 3, 4], [2, 1, 4, 9], [7, 8, 9, 2]])
    np.testing.assert_array_equal(otf_loop.churn(idx), [4, 1, 2])
