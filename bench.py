#!/usr/bin/env python3
"""Throughput of the ranking hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload dense|pq|binary|multiquery|dense128]
                    [--no-others] [--no-cpu-baseline]

A step is one ranking pass of the workload: score every stored row with the current model and
return the sorted top-k (one otf_rank_* call: scan + selection).  The store is generated on the
GPU before the clock starts.  The default workload is the full-size dense store (1,000,000 x
2048 fp32, k = 1000) on which the headline metric is quoted; the PQ, binary and multi-classifier
stores and the Pegasos training pass are measured the same way and reported inside the same JSON
line under "other_workloads".

The one JSON line also carries
  roofline      achieved HBM GB/s of the scoring kernel (algorithmic bytes = every stored row read
                once) against the 8 TB/s peak; the kernel time comes from HIP events the library
                records around that kernel on its stream during the timed steps
  cpu_baseline  the CPU oracle (oracle/, plain C, fp64, OpenMP over rows) timed on this host on
                a stated sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the scoring kernel.  NOT measured by this run: copied from
# profiles/traffic_counters.md, i.e. from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same
# command scaled by the same counters on a plain copy of known size.  The line says so
# ("traffic_source"), and a workload that is scaled down or has no counter run yet reports null.
TRAFFIC_SOURCE = "profiles/traffic_counters.md (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; not measured in this run)"
MEASURED_TRAFFIC_BYTES = {          # read + written, per launch of the scoring kernel
    "dense": 8195955717, "pq": 2590228917, "pq512": 2598162714, "pq256": 2594092640, "binary": 12825251201,
    "hamming": 12816993899, "dense128": 5131105014, "dense128h": 5131044388, "sparse128": 2450816290,
    "multiquery": 20488076562,
}
TOPK_TRAFFIC_BYTES = 200157996      # topk_filter_kernel on 50M scores
LLOYD_SUMS_TRAFFIC_BYTES = 8597935062   # pq_accumulate_kernel on 1M x 2048 (X once, the codes once per die)

WORKLOADS = {
    "dense": dict(name="dense_1Mx2048_fp32_top1000", N=1_000_000, D=2048, k=1000, row_bytes=8192, dtype="f32"),
    "pq": dict(name="pq_20Mx128B_M128_K256_top1000", N=20_000_000, M=128, K=256, dsub=16, k=1000, row_bytes=128,
               dtype="f32"),
    "binary": dict(name="binary_50Mx2048bit_top1000", N=50_000_000, D=2048, k=1000, row_bytes=256, dtype="f32"),
    "multiquery": dict(name="multiquery_5Mx2048_fp16_Q64_top1000", N=5_000_000, D=2048, Q=64, k=1000,
                       row_bytes=4096, dtype="f16"),
    # the paper's own feature size (Sec. 3, Table 2: CNN 128), ten times its ~1M images so that the
    # scan and not the launches is what is timed
    "dense128": dict(name="dense_10Mx128_fp32_top1000", N=10_000_000, D=128, k=1000, row_bytes=512, dtype="f32"),
    # the same feature size stored as fp16 (2 bytes per dimension), twice the rows in the same bytes
    "dense128h": dict(name="dense_20Mx128_fp16_top1000", N=20_000_000, D=128, k=1000, row_bytes=256, dtype="f16"),
    # the paper's own PQ geometries on its 2048-D feature (Sec. 3: 4 or 8 dimensions per sub-block;
    # Table 2 row "2048 PQ 4 dims/sq", 512 bytes per image): rows longer than one table image
    "pq512": dict(name="pq_5Mx512B_M512_K256_top1000", N=5_000_000, M=512, K=256, dsub=4, k=1000, row_bytes=512,
                  dtype="f32"),
    # the same 10M rows of 128-D features, 60 % of their entries zero (Sec. 3.1), stored as presence
    # mask + packed non-zero values; row_bytes is filled in from the store that was generated
    "sparse128": dict(name="sparse_10Mx128_fp32_60pct_zeros_top1000", N=10_000_000, D=128, k=1000, row_bytes=None,
                      dtype="f32"),
    # Hamming ranking of the binary store (Sec. 3.1, after Table 2: what the paper leaves for later)
    "hamming": dict(name="hamming_50Mx2048bit_top1000", N=50_000_000, D=2048, k=1000, row_bytes=256, dtype="u32"),
    "pq256": dict(name="pq_10Mx256B_M256_K256_top1000", N=10_000_000, M=256, K=256, dsub=8, k=1000, row_bytes=256,
                  dtype="f32"),
}


def make_workload(kind, scale, torch, binding, synth):
    """Returns (step_fn, info).  step_fn() enqueues one ranking pass on the current stream."""
    cfg = dict(WORKLOADS[kind])
    N = max(1024, int(cfg["N"] * scale))
    cfg["N"] = N
    dev = "cuda"
    seed = synth.BASE_SEED + {"dense": 2, "pq": 3, "binary": 4, "multiquery": 5, "dense128": 8, "pq512": 10,
                              "pq256": 11, "hamming": 4, "dense128h": 12, "sparse128": 13}[kind]
    k = cfg["k"]
    if kind in ("dense", "dense128", "dense128h"):
        X = synth.dense_features(N, cfg["D"], seed, device=dev,
                                 dtype=torch.float16 if kind == "dense128h" else torch.float32)
        w = synth.normal_vector(cfg["D"], 0.05, seed + 100, device=dev)
        ws = binding.make_workspace(N, k, 1, dev)
        out = binding._outputs(1, k, dev)
        step = lambda: binding.rank_dense(X, w, None, k, ws, out=out)
        keep = (X, w)
    elif kind in ("pq", "pq512", "pq256"):
        codes = synth.pq_codes(N, cfg["M"], cfg["K"], seed, device=dev)
        cb = synth.pq_codebooks(cfg["M"], cfg["K"], cfg["dsub"], seed + 100, device=dev)
        w = synth.normal_vector(cfg["M"] * cfg["dsub"], 1.0, seed + 200, device=dev)
        ws = binding.make_workspace(N, k, 1, dev)
        out = binding._outputs(1, k, dev)
        # a new model means a new table: the build is part of the pass (one call: table build + ranking)
        step = lambda: binding.rank_pq_model(codes, cb, w, 0.0, k, ws, out=out)
        keep = (codes, cb, w)
    elif kind == "binary":
        bits = synth.binary_bits_random(N, cfg["D"] // 32, seed, device=dev)
        w = synth.normal_vector(cfg["D"], 1.0, seed + 100, device=dev)
        ws = binding.make_workspace(N, k, 1, dev)
        out = binding._outputs(1, k, dev)
        step = lambda: binding.rank_binary(bits, cfg["D"], w, 0.0, k, ws, out=out)
        keep = (bits, w)
    elif kind == "sparse128":
        X = synth.sparse_features(N, cfg["D"], seed, device=dev)
        rows, start = synth.sparse_rows_from_dense(X)
        del X
        w = synth.normal_vector(cfg["D"], 0.05, seed + 100, device=dev)
        ws = binding.make_workspace(N, k, 1, dev)
        out = binding._outputs(1, k, dev)
        step = lambda: binding.rank_sparse(rows, start, cfg["D"], w, 0.0, k, ws, out=out)
        cfg["row_bytes"] = (rows.numel() * 4 + start.numel() * 8) / N      # stored bytes per row, offsets included
        keep = (rows, start, w)
    elif kind == "hamming":
        bits = synth.binary_bits_random(N, cfg["D"] // 32, seed, device=dev)
        query = synth.binary_bits_random(1, cfg["D"] // 32, seed + 100, device=dev)[0].contiguous()
        ws = binding.make_workspace(N, k, 1, dev)
        out = binding._outputs(1, k, dev)
        step = lambda: binding.rank_hamming(bits, cfg["D"], query, k, ws, out=out)
        keep = (bits, query)
    elif kind == "multiquery":
        X = synth.dense_features(N, cfg["D"], seed, device=dev, dtype=torch.float16)
        W = synth.normal_matrix(cfg["Q"], cfg["D"], 0.05, seed + 100, device=dev, dtype=torch.float16)
        ws = binding.make_workspace(N, k, cfg["Q"], dev)
        out = binding._outputs(cfg["Q"], k, dev)
        step = lambda: binding.rank_dense(X, W, None, k, ws, out=out)
        keep = (X, W)
    else:
        raise ValueError(kind)
    cfg["_keep"] = keep
    return step, cfg


RAMP_S = 0.25      # seconds of untimed calls before the warm-up steps: a GPU that has been idle (the stores are
                   # generated in short bursts) runs its first tens of milliseconds below its steady clock


def time_steps(step, steps, warmup, torch, binding):
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < RAMP_S:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    binding.profile_begin(steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    scan_ms_total, nrec = binding.profile_end()
    return (t1 - t0) / steps, (scan_ms_total / nrec if nrec else None)


def graph_replay_ms(step, steps, torch):
    """The same step captured once into a HIP graph and replayed `steps` times (no host work per
    kernel between replays); milliseconds per replay, or None if the capture is refused."""
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(5):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3
    except Exception as exc:                      # the figure is an extra: never fail the benchmark for it
        sys.stderr.write("graph replay skipped: %r\n" % (exc,))
        return None


def measure(kind, steps, warmup, scale, torch, binding, synth):
    step, cfg = make_workload(kind, scale, torch, binding, synth)
    sec_per_step, scan_ms = time_steps(step, steps, warmup, torch, binding)
    N = cfg["N"]
    alg_bytes = N * cfg["row_bytes"]
    res = {
        "workload": cfg["name"] if scale == 1.0 else cfg["name"] + "_x%g" % scale,
        "N": N,
        "k": cfg["k"],
        "value": N / sec_per_step,
        "unit": "vectors/s",
        "ms_per_step": sec_per_step * 1e3,
        "dtype": cfg["dtype"],
        "whole_path_GBps": alg_bytes / sec_per_step / 1e9,
        "whole_path_frac_of_hbm_peak": alg_bytes / sec_per_step / 1e9 / HBM_PEAK_GBS,
    }
    if scan_ms:
        achieved = alg_bytes / (scan_ms * 1e-3) / 1e9
        res["roofline"] = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": achieved / HBM_PEAK_GBS,
                           "traffic": MEASURED_TRAFFIC_BYTES.get(kind) if scale == 1.0 else None,
                           "traffic_source": TRAFFIC_SOURCE, "kernel_ms": scan_ms, "algorithmic_bytes": alg_bytes}
    res["graph_replay_ms_per_step"] = graph_replay_ms(step, steps, torch)
    return res, cfg


def measure_sgd(torch, binding, synth):
    """One training pass: 125 Pegasos steps of batch 256 over 1,000 positives / 16,000 negatives."""
    D, n_pos, n_neg, batch, steps, lam = 2048, 1000, 16000, 256, 125, 1e-4
    Xp, Xn = synth.sgd_pools(D, n_pos, n_neg, synth.BASE_SEED + 2, device="cuda")
    ip, ineg = synth.sgd_batches(n_pos, n_neg, batch, steps, synth.BASE_SEED + 2)
    ip = torch.from_numpy(ip).cuda()
    ineg = torch.from_numpy(ineg).cuda()
    ws = binding.sgd_workspace(batch, "cuda")
    w = torch.zeros(D, device="cuda")

    def one_call():                                   # otf_svm_sgd_pass: the steps enqueued back to back from C
        w.zero_()
        binding.svm_sgd_pass(w, None, Xp, ip, Xn, ineg, lam, 1, False, ws)

    def one_kernel():                                 # the same call as a single kernel (diagnostic route)
        binding.debug_set(binding.DEBUG_SGD_PASS_PATH, 1)
        try:
            one_call()
        finally:
            binding.debug_set(binding.DEBUG_SGD_PASS_PATH, 0)
    res = {}
    for name, fn in (("call", one_call), ("kernel", one_kernel)):
        fn()
        torch.cuda.synchronize()
        reps = 5
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        res[name] = (time.perf_counter() - t0) / reps
    assert binding.sgd_pass_status(ws) == 0
    return {"workload": "pegasos_pass_125steps_B256_D2048", "ms_per_pass": res["call"] * 1e3,
            "us_per_step": res["call"] / steps * 1e6, "us_per_step_as_one_kernel": res["kernel"] / steps * 1e6}


def measure_topk(torch, binding, synth):
    """otf_topk on ready-made scores: the exact sorted top 1000 of 50M fp32 scores (the size of the
    binary store), one classifier.  The scores are read once (plus a 0.8 % sample): sample ->
    threshold -> one filtering pass -> sort, the exact radix passes gated behind it."""
    N, k = 50_000_000, 1000
    S = synth.normal_vector(N, 1.0, synth.BASE_SEED + 9, device="cuda")
    ws = binding.make_workspace(N, k, 1, "cuda")
    out = binding._outputs(1, k, "cuda")
    for _ in range(3):
        binding.topk(S, k, ws, out=out)
    reps = 20
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        binding.topk(S, k, ws, out=out)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    return {"workload": "topk_50M_scores_k1000", "ms_per_call": dt * 1e3, "scores_per_s": N / dt,
            "roofline": {"bound": "hbm", "achieved": 4.0 * N / dt / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": 4.0 * N / dt / 1e9 / HBM_PEAK_GBS, "traffic": TOPK_TRAFFIC_BYTES,
                         "traffic_source": TRAFFIC_SOURCE,
                         "note": "algorithmic bytes = one read of the scores, which is what the call does; the rest of the time is four dependent launches (sample, filter, the gated pass 1 of the fallback, and the launch that sorts the list or runs the full selection)"}}


def measure_filter_fallback(steps, warmup, torch, binding, synth):
    """Worst case of the filtered ranking: the PQ store of the benchmark with 10,000 rows of the
    maximum score planted where the sample never looks, so that the candidate list overflows after
    a complete filtered scan and the call redoes the ranking by full selection (second scan, three
    selection passes, exact split of a 10,000-way tie by row number)."""
    step, cfg = make_workload("pq", 1.0, torch, binding, synth)
    codes, cb, w = cfg["_keep"]
    N, k = cfg["N"], cfg["k"]
    lut = binding.pq_build_lut(cb, w)
    best = lut.argmax(dim=1).to(torch.uint8)
    normal_ms, _ = time_steps(step, steps, warmup, torch, binding)
    codes[2048:12048] = best                               # row groups the sample scan skips
    ws = binding.make_workspace(N, k, 1, "cuda")
    out = binding._outputs(1, k, "cuda")
    planted = lambda: binding.rank_pq_model(codes, cb, w, 0.0, k, ws, out=out)
    planted()
    taken = binding.debug_fallback_taken(ws)
    first = int(out[1][0, 0].item())
    worst_ms, _ = time_steps(planted, steps, warmup, torch, binding)
    return {"workload": "pq_20Mx128B_filter_fallback_worst_case", "fallback_taken": bool(taken),
            "first_row_returned": first,
            "ms_per_step": worst_ms * 1e3, "ms_per_step_without_planted_rows": normal_ms * 1e3,
            "slowdown": worst_ms / normal_ms, "value": N / worst_ms, "unit": "vectors/s",
            "note": "filtered scan + gated rescan with histogram + passes 2 and 3 + gather + sort; rows 2048.. tie at the top"}


def measure_onthefly(torch, binding, synth, X=None):
    """The on-the-fly loop on the dense store (paper Sec. 4, "On-line (GPU back-end)"): 12 rounds of
    64 Pegasos steps (B = 256) on a pool of positives growing by 12 per round, each followed by a
    ranking of the 1M x 2048 store under a snapshot of the model.  Reports the query's wall time
    with training and ranking on two streams and on one, the latency of a ranking in both cases,
    and how many of the 1000 listed rows are new in each ranking."""
    from paper_1407_4764_amd import onthefly
    N, D, k, B, lam, rounds, steps = 1_000_000, 2048, 1000, 256, 1e-4, 12, 64
    if X is None:
        X = synth.dense_features(N, D, synth.BASE_SEED + 2, device="cuda")
    Xp, Xn = synth.sgd_pools(D, 1000, 16000, synth.BASE_SEED + 2, device="cuda")
    sizes, ip, ineg = synth.onthefly_schedule(rounds, steps, B, 12, 12, 1000, 16000, synth.BASE_SEED + 8)
    ip, ineg = torch.from_numpy(ip).cuda(), torch.from_numpy(ineg).cuda()
    res = {}
    for name, overlap in (("two_streams", True), ("one_stream", False)):
        onthefly.run(X, Xp, Xn, ip, ineg, k, lam, overlap=overlap)            # warm-up
        o = onthefly.run(X, Xp, Xn, ip, ineg, k, lam, overlap=overlap)
        rk = sorted(o["rank_ms"])
        res[name] = {"query_ms": o["total_ms"], "train_stream_ms": o["train_ms"], "rank_ms_median": rk[len(rk) // 2],
                     "rank_ms_max": rk[-1]}
        idx = o["idx"].cpu().numpy()
    import numpy as np
    churn = [int(k)] + [int(np.setdiff1d(idx[r], idx[r - 1]).size) for r in range(1, rounds)]
    return {"workload": "onthefly_loop_dense_1Mx2048_12rounds_x64steps_B256", "positives_in_pool": [int(v) for v in sizes],
            "new_rows_in_list_per_round": churn, **res}


def measure_pq_encoder(torch, binding, synth, X=None):
    """PQ encoder and one Lloyd iteration (paper Sec. 3, "Product quantization (PQ)") on 1M x 2048
    fp32 rows with the geometry of the PQ workload (M = 128 sub-blocks of 16 dimensions, K = 256)."""
    N, M, dsub = 1_000_000, 128, 16
    if X is None:
        X = synth.dense_features(N, M * dsub, synth.BASE_SEED + 2, device="cuda")
    C = X[:256].reshape(256, M, dsub).permute(1, 0, 2).contiguous()
    ws = binding.pq_train_workspace(M, dsub)
    codes = torch.empty((N, M), dtype=torch.uint8, device="cuda")
    e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
    for _ in range(2):
        binding.pq_encode(X, C, ws, codes)
    reps = 5
    torch.cuda.synchronize()
    binding.profile_begin(reps)                    # event pairs around the kernel of the per-centre sums (Lloyd calls only)
    e0.record()
    for _ in range(reps):
        binding.pq_encode(X, C, ws, codes)
    e1.record()                                    # no pause here: after an idle gap the first calls run at a lower clock
    for _ in range(reps):
        binding.pq_lloyd_step(X, C, ws, codes)
    e2.record()
    torch.cuda.synchronize()
    sums_total_ms, nrec = binding.profile_end()
    sums_ms = sums_total_ms / nrec
    enc_ms, lloyd_ms = e0.elapsed_time(e1) / reps, e1.elapsed_time(e2) / reps
    # The kernel splits every fp32 value into three exact bf16 pieces and issues, per 32 rows x 32
    # centres x 16 dimensions, six bf16 matrix instructions for the product and one for the norms:
    # 7 x the useful multiply-adds run on the bf16 matrix pipe, so that pipe's peak is the roofline.
    # `frac` counts the method's own flops, 2 N M K dsub, against the bf16 matrix peak (the pipe they run on).
    useful = 2.0 * N * M * 256 * dsub / (enc_ms * 1e-3) / 1e12
    executed = 7.0 * useful
    # the per-centre sums of a Lloyd iteration: one read of X and of the codes
    sums_gbs = (N * M * dsub * 4.0 + N * M) / (sums_ms * 1e-3) / 1e9
    return {"workload": "pq_encode_1Mx2048_M128_K256", "encode_ms": enc_ms, "rows_per_s": N / (enc_ms * 1e-3),
            "lloyd_step_ms": lloyd_ms, "lloyd_sums_kernel_ms": sums_ms,
            "lloyd_sums": {"bound": "hbm", "achieved": sums_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": sums_gbs / HBM_PEAK_GBS, "traffic": LLOYD_SUMS_TRAFFIC_BYTES,
                           "traffic_source": TRAFFIC_SOURCE,
                           "note": "pq_accumulate_kernel (64-bit fixed-point sums in shared memory) between the library's "
                                   "event pairs; algorithmic bytes = X + codes once"},
            "dtype": "bf16 x 3 pieces per fp32 value, fp32 accumulate",
            "useful_fp32_tflops": useful, "useful_frac_of_fp32_matrix_peak": useful / MFMA_FP32_PEAK_TFLOPS,
            "executed_bf16_tflops": executed, "executed_frac_of_bf16_matrix_peak": executed / MFMA_BF16_PEAK_TFLOPS,
            "roofline": {"bound": "mfma", "achieved": useful, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": useful / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                         "note": "algorithmic flops (2 N M K dsub) over the bf16 matrix peak; the kernel executes 7x as "
                                 "many bf16 multiply-adds to reach fp32 accuracy (executed_* fields)"}}


MFMA_FP32_PEAK_TFLOPS = 157.3                     # MI355X dense fp32 matrix rate
MFMA_BF16_PEAK_TFLOPS = 2500.0                    # MI355X dense bf16 matrix rate


def measure_encoder(torch, binding, synth):
    """Binarisation encoder (paper Sec. 3, Table 2 row "128 BIN 2048 dims"): 1M descriptors of 128
    dimensions to 2048-bit codes; timed with events on the stream the kernel runs on."""
    N, m, n = 1_000_000, 128, 2048
    G = synth.random_square(n, synth.BASE_SEED + 6, device="cuda")
    U = binding.tight_frame(G, m)
    phi = synth.centred_descriptors(N, m, synth.BASE_SEED + 7, device="cuda")
    bits = torch.empty((N, n // 32), dtype=torch.int32, device="cuda")
    for _ in range(3):
        binding.binarize(phi, U, bits)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 10
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        binding.binarize(phi, U, bits)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    t0 = time.perf_counter()
    binding.tight_frame(G, m)
    torch.cuda.synchronize()
    frame_ms = (time.perf_counter() - t0) * 1e3
    # six bf16 matrix instructions (products of the three exact pieces of every fp32 value) do the
    # work of eight fp32 ones: 6 x the useful multiply-adds run on the bf16 matrix pipe
    # `frac` counts the method's own flops, 2 N m n, against the bf16 matrix peak (the pipe they run on)
    useful = 2.0 * N * m * n / (ms * 1e-3) / 1e12
    executed = 6.0 * useful
    return {"workload": "binarize_1Mx128_to_2048bit", "ms_per_call": ms, "descriptors_per_s": N / (ms * 1e-3),
            "dtype": "bf16 x 3 pieces per fp32 value, fp32 accumulate", "useful_fp32_tflops": useful,
            "useful_frac_of_fp32_matrix_peak": useful / MFMA_FP32_PEAK_TFLOPS,
            "executed_bf16_tflops": executed, "executed_frac_of_bf16_matrix_peak": executed / MFMA_BF16_PEAK_TFLOPS,
            "frame_setup_ms": frame_ms,
            "roofline": {"bound": "mfma", "achieved": useful, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": useful / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                         "note": "algorithmic flops (2 N m n) over the bf16 matrix peak; the kernel executes 6x as many "
                                 "bf16 multiply-adds to reach fp32 accuracy (executed_* fields)"}}


def cpu_baseline(kind, cfg, torch, budget_s=10.0):
    """Times the CPU oracle on this host on a bounded sample of the workload's own rows (the
    headline store: all of its rows), repeated until budget_s seconds have passed."""
    from oracle import otf_oracle as orc
    import numpy as np
    cores = orc.num_threads()
    keep = cfg["_keep"]
    k = cfg["k"]
    if kind in ("dense", "dense128", "dense128h"):
        rows = min(cfg["N"], 1 << 20 if kind == "dense" else 1 << 22)
        X = keep[0][:rows].cpu().numpy()
        w = keep[1].cpu().numpy()
        run = lambda: orc.topk(orc.dense_scores(X, w)[0], min(k, rows))
        sample = ("all %d rows of the store, scored and fully sorted" if rows == cfg["N"] else
                  "first %d rows of the store, scored and fully sorted") % rows
    elif kind in ("pq", "pq512", "pq256"):
        rows = min(cfg["N"], 1 << 20)
        codes = keep[0][:rows].cpu().numpy()
        cb, w = keep[1].cpu().numpy(), keep[2].cpu().numpy()
        run = lambda: orc.topk(orc.pq_scores_reconstruct(codes, cb, w, 0.0), min(k, rows))
        sample = "first %d rows, scored by explicit reconstruction and fully sorted" % rows
    elif kind == "sparse128":
        rows = min(cfg["N"], 1 << 21)
        st = keep[1][:rows + 1].cpu().numpy()
        words = keep[0][:int(st[-1])].cpu().numpy().view(np.uint32)
        w = keep[2].cpu().numpy()
        idx = st[:-1, None] + np.arange(4)[None, :]
        mask = words[idx]
        is_value = np.ones(int(st[-1]), dtype=bool)
        is_value[idx.reshape(-1)] = False
        values = words[is_value].view(np.float32)
        vstart = np.concatenate([[0], np.cumsum(st[1:] - st[:-1] - 4)]).astype(np.int64)
        run = lambda: orc.topk(orc.dense_scores(orc.sparse_expand(mask, values, vstart, cfg["D"]), w)[0], min(k, rows))
        sample = "first %d rows, expanded to dense rows, scored and fully sorted" % rows
    elif kind == "hamming":
        rows = min(cfg["N"], 1 << 20)
        bits = keep[0][:rows].cpu().numpy().view(np.uint32)
        query = keep[1].cpu().numpy().view(np.uint32)
        run = lambda: orc.topk(orc.hamming_scores(bits, cfg["D"], query), min(k, rows))
        sample = "first %d rows, distances counted bit by bit and fully sorted" % rows
    elif kind == "binary":
        rows = min(cfg["N"], 1 << 20)
        bits = keep[0][:rows].cpu().numpy().view(np.uint32)
        w = keep[1].cpu().numpy()
        run = lambda: orc.topk(orc.binary_scores(bits, cfg["D"], w, 0.0), min(k, rows))
        sample = "first %d rows, scored bit by bit and fully sorted" % rows
    else:
        rows = min(cfg["N"], 16384)
        X = keep[0][:rows].cpu().numpy()
        W = keep[1].cpu().numpy()

        def run():
            s = orc.dense_scores(X, W)
            for q in range(s.shape[0]):
                orc.topk(s[q], min(k, rows))
        sample = "first %d rows against all %d classifiers, each fully sorted" % (rows, cfg["Q"])
    run()                                         # warm the pages
    reps, t0 = 0, time.perf_counter()
    while True:
        run()
        reps += 1
        el = time.perf_counter() - t0
        if el >= budget_s:
            break
    return {"value": rows * reps / el, "unit": "vectors/s", "cores": cores, "kind": "oracle",
            "sample": "%s; %d repetitions in %.1f s" % (sample, reps, el)}


def main():
    global RAMP_S
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="dense", choices=sorted(WORKLOADS))
    ap.add_argument("--scale", type=float, default=1.0, help="shrink N (debugging only; the result is then not the named workload)")
    ap.add_argument("--no-others", action="store_true", help="skip the other stores and the training pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--encoder-only", action="store_true", help="only time the binarisation encoder")
    ap.add_argument("--loop-only", action="store_true", help="only run the on-the-fly loop")
    ap.add_argument("--pqenc-only", action="store_true", help="only time the PQ encoder and a Lloyd iteration")
    ap.add_argument("--topk-only", action="store_true", help="only time otf_topk on ready-made scores")
    ap.add_argument("--sgd-only", action="store_true", help="only time the Pegasos training pass")
    ap.add_argument("--fallback-only", action="store_true", help="only time the worst case of the filtered ranking")
    ap.add_argument("--ramp-seconds", type=float, default=None,
                    help="untimed calls for this long before the warm-up steps (default %.2f)" % RAMP_S)
    ap.add_argument("--switch", action="append", default=[], metavar="NAME=VALUE",
                    help="set a diagnostic switch of the library first (binding.DEBUG_<NAME>), e.g. --switch PQENC_FP32=1")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 2 GiB five times (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (each GPU would rank its own "
                 "row shard and the k-entry lists would be merged). Run with --gpus 1.")
    import torch
    from paper_1407_4764_amd import binding, synth
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    binding.lib()                                  # fail loudly if the HIP library is missing
    if args.ramp_seconds is not None:
        RAMP_S = max(0.0, args.ramp_seconds)
    for item in args.switch:
        name, _, value = item.partition("=")
        binding.debug_set(getattr(binding, "DEBUG_" + name.upper()), int(value))
    if args.calibrate_copy:
        src = torch.full((1 << 29,), 1.0, dtype=torch.float32, device="cuda")     # 2 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "copies": 5}))
        return

    if args.encoder_only:
        print(json.dumps(measure_encoder(torch, binding, synth)))
        return
    if args.topk_only:
        print(json.dumps(measure_topk(torch, binding, synth)))
        return
    if args.sgd_only:
        print(json.dumps(measure_sgd(torch, binding, synth)))
        return
    if args.pqenc_only:
        print(json.dumps(measure_pq_encoder(torch, binding, synth)))
        return
    if args.fallback_only:
        print(json.dumps(measure_filter_fallback(args.steps, max(args.warmup, 100), torch, binding, synth)))
        return
    if args.loop_only:
        print(json.dumps(measure_onthefly(torch, binding, synth)))
        return

    res, cfg = measure(args.workload, args.steps, args.warmup, args.scale, torch, binding, synth)
    line = {
        "metric": "dataset vectors scored+top-k'd per sec (1 GPU)",
        "value": res["value"],
        "unit": "vectors/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": res["dtype"],
        "data": "synthetic",
        "config": {"workload": res["workload"], "N": res["N"], "k": res["k"],
                   "step": "one otf_rank_* call: scan of the whole store + exact sorted top-k"},
        "whole_path_frac_of_hbm_peak": res["whole_path_frac_of_hbm_peak"],
        "ramp_s": RAMP_S,
        "roofline": res.get("roofline"),
        "graph_replay_ms_per_step": res.get("graph_replay_ms_per_step"),
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(args.workload, cfg, torch)
    loop = pqenc = None
    if not args.no_others and args.workload == "dense" and args.scale == 1.0:
        loop = measure_onthefly(torch, binding, synth, cfg["_keep"][0])          # on the store already resident
        pqenc = measure_pq_encoder(torch, binding, synth, cfg["_keep"][0])
    del cfg
    torch.cuda.empty_cache()
    if not args.no_others:
        others = []
        for kind in sorted(WORKLOADS):
            if kind == args.workload:
                continue
            # sub-millisecond steps reach their steady rate only after ~60 calls in a fresh process
            # (0.453 -> 0.424 ms for the PQ store), so the side measurements warm up longer
            r, c = measure(kind, args.steps, max(args.warmup, 100), args.scale, torch, binding, synth)
            r["steps"], r["warmup"] = args.steps, max(args.warmup, 100)
            if not args.no_cpu_baseline:
                r["cpu_baseline"] = cpu_baseline(kind, c, torch, budget_s=2.5)
            del c
            torch.cuda.empty_cache()
            others.append(r)
        others.append(measure_sgd(torch, binding, synth))
        others.append(measure_topk(torch, binding, synth))
        others.append(measure_filter_fallback(args.steps, max(args.warmup, 100), torch, binding, synth))
        others.append(measure_encoder(torch, binding, synth))
        others.append(loop if loop is not None else measure_onthefly(torch, binding, synth))
        others.append(pqenc if pqenc is not None else measure_pq_encoder(torch, binding, synth))
        line["other_workloads"] = others
    line["paper_context"] = "paper: ~0.01 s to score + ~0.002 s to sort 1M x 128-D fp32 on a GTX Titan (Sec. 4)"
    print(json.dumps(line))


if __name__ == "__main__":
    main()
