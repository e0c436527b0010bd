"""The on-the-fly loop (paper Sec. 4, "On-line (GPU back-end)"): the SVM keeps training on a
growing pool of positives while, at intervals, the whole store is ranked with the model as it
stands.  Training and ranking are enqueued on two HIP streams; a ranking works on a snapshot of w
taken on the training stream, so training never waits for it and the result does not depend on
how the two streams interleave.  Every step of the work runs in the library's kernels; this
module only orders the calls (torch supplies the streams, the events and the snapshot copies).
"""
import time

import torch

from . import binding


def run(X, Xpos, Xneg, idx_pos, idx_neg, k, lam, overlap=True):
    """X: store (N, D) fp32 on the GPU.  Xpos/Xneg: training pools.  idx_pos/idx_neg: int32 device
    tensors [rounds, steps, half]: the batches of every step; a ranking follows each round.
    Returns dict(idx [rounds, k], val [rounds, k], w [rounds, D], rank_ms [rounds], total_ms,
    train_ms): rank_ms is the time of each ranking on its stream, total_ms the wall time of the
    whole query, train_ms the span of the training stream."""
    dev = X.device
    rounds, steps, half = idx_pos.shape
    N, D = X.shape
    train, rank = torch.cuda.Stream(dev), torch.cuda.Stream(dev)
    w = torch.zeros(D, dtype=torch.float32, device=dev)
    snaps = torch.zeros((rounds, D), dtype=torch.float32, device=dev)
    out_val = torch.empty((rounds, k), dtype=torch.float32, device=dev)
    out_idx = torch.empty((rounds, k), dtype=torch.int32, device=dev)
    binding.check_indices(idx_pos, Xpos.shape[0])          # the training kernels read row numbers unchecked
    binding.check_indices(idx_neg, Xneg.shape[0])
    sgd_ws = binding.sgd_workspace(2 * half, dev)
    rank_ws = binding.make_workspace(N, k, 1, dev)
    snapped = [torch.cuda.Event() for _ in range(rounds)]
    r0 = [torch.cuda.Event(enable_timing=True) for _ in range(rounds)]
    r1 = [torch.cuda.Event(enable_timing=True) for _ in range(rounds)]
    t_begin, t_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize(dev)
    wall0 = time.perf_counter()
    t = 0
    with torch.cuda.stream(train):
        t_begin.record()
    for r in range(rounds):
        with torch.cuda.stream(train):
            binding.svm_sgd_pass(w, None, Xpos, idx_pos[r], Xneg, idx_neg[r], lam, t + 1, False, sgd_ws)
            t += steps
            snaps[r].copy_(w)                      # the model this round's ranking sees
            snapped[r].record()
            if r == rounds - 1:
                t_end.record()
        target = rank if overlap else train
        with torch.cuda.stream(target):
            target.wait_event(snapped[r])
            r0[r].record()
            binding.rank_dense(X, snaps[r:r + 1], None, k, rank_ws, out=(out_val[r:r + 1], out_idx[r:r + 1]))
            r1[r].record()
    torch.cuda.synchronize(dev)
    total_ms = (time.perf_counter() - wall0) * 1e3
    return {"idx": out_idx, "val": out_val, "w": snaps, "total_ms": total_ms,
            "rank_ms": [r0[i].elapsed_time(r1[i]) for i in range(rounds)],
            "train_ms": t_begin.elapsed_time(t_end)}
