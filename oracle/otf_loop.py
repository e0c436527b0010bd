"""Oracle for the on-the-fly loop -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.

Paper Sec. 4, "On-line (GPU back-end)": the SVM is trained by Pegasos mini-batch steps (learning
rate 1/(lambda t), t counting every step since the query began) on a pool of positives that
grows while the query runs, and at intervals the whole dataset is scored with the model as it
stands and the head of the ranked list is returned.  The oracle takes the schedule (which steps
see which batch, after which step a ranking happens) as input and runs it strictly in order.
"""
import numpy as np

from . import otf_oracle as orc


def run(X, Xpos, Xneg, idx_pos, idx_neg, k, lam):
    """idx_pos, idx_neg: [rounds, steps, half] row numbers.  Returns (w after each round
    [rounds, D] float64, ranked rows [rounds, k], their scores [rounds, k], all scores [rounds, N])."""
    rounds, steps, _ = idx_pos.shape
    D = X.shape[1]
    w = np.zeros(D, dtype=np.float64)
    ws, idxs, vals, alls = [], [], [], []
    t = 0
    for r in range(rounds):
        for s in range(steps):
            t += 1
            w, _, _ = orc.sgd_step(w, 0.0, Xpos, idx_pos[r, s], Xneg, idx_neg[r, s], lam, t, False)   # w is kept in fp32
        ws.append(w.copy())
        sc = orc.dense_scores(X, w.astype(np.float32))[0]     # the model is handed over in fp32
        i, v = orc.topk(sc, k)
        idxs.append(i)
        vals.append(v)
        alls.append(sc)
    return np.stack(ws), np.stack(idxs), np.stack(vals), np.stack(alls)


def churn(idx):
    """Rows of each ranked list that were not in the previous one (first entry: k)."""
    out = [idx.shape[1]]
    for r in range(1, idx.shape[0]):
        out.append(int(np.setdiff1d(idx[r], idx[r - 1]).size))
    return np.array(out)
