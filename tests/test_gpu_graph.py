"""Every ranking call can be captured into a HIP graph and replayed (tight serving loops replay one
captured ranking per query).  The library records only kernels and, for stores shorter than a
tile, one device-to-device copy: no memset nodes, nothing allocated.  A replay must give the bits
of the eager call; the model changes between replays (in place, as the on-line loop does), with
eager work and synchronisations in between, and every replay is checked."""
import pytest
import torch

from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = synth.BASE_SEED + 11000


def _capture(fn):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()                                             # warm-up outside the capture (kernel attributes, lazy loads)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g


def _check_replays(call, model, out, new_model):
    """call() ranks into `out` under `model` (a tensor the call reads); replays must track changes of it."""
    g = _capture(call)
    for r in range(3):
        model.copy_(new_model(r))
        torch.cuda.synchronize()
        call()                                           # eager, under the new model
        torch.cuda.synchronize()
        want = (out[0].clone(), out[1].clone())
        out[0].zero_()
        out[1].zero_()
        _ = (torch.randn(1 << 20, device=DEV) * 2).sum().item()     # the program's own eager work in between
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out[0], want[0]) and torch.equal(out[1], want[1]), "replay %d" % r


def test_dense_rankings_replay(oracle):
    for N, D, k in ((60000, 2048, 100), (1300000, 128, 1000)):       # full selection; sampled, filtered route
        X = synth.dense_features(N, D, SEED + D, device=DEV)
        w = synth.normal_vector(D, 0.05, SEED + 1, device=DEV)
        ws = binding.make_workspace(N, k)
        out = binding._outputs(1, k, DEV)
        _check_replays(lambda: binding.rank_dense(X, w, None, k, ws, out=out), w, out,
                       lambda r: synth.normal_vector(D, 0.05, SEED + 10 + r, device=DEV))
        _check_replays(lambda: binding.rank_dense_noalloc(X, w, None, k, out), w, out,
                       lambda r: synth.normal_vector(D, 0.05, SEED + 20 + r, device=DEV))


def test_replays_take_the_fallback_when_the_model_asks_for_it():
    """One captured filtered ranking serves models whose filtered scan succeeds and a zero model, under
    which every score ties and the gated re-scan and full selection of the same graph must answer."""
    N, D, k = 1300000, 128, 200
    X = synth.dense_features(N, D, SEED + 77, device=DEV)
    w = synth.normal_vector(D, 0.05, SEED + 78, device=DEV)
    ws = binding.make_workspace(N, k)
    out = binding._outputs(1, k, DEV)
    taken = []

    def model(r):
        if r > 0:
            taken.append(binding.debug_fallback_taken(ws))          # of the replay before this one
        return torch.zeros(D, device=DEV) if r == 1 else synth.normal_vector(D, 0.05, SEED + 80 + r, device=DEV)
    _check_replays(lambda: binding.rank_dense(X, w, None, k, ws, out=out), w, out, model)
    taken.append(binding.debug_fallback_taken(ws))
    assert taken == [False, True, False]


@pytest.mark.parametrize("N,M,dsub", [(1200000, 128, 16), (1100000, 512, 4), (3000, 256, 8), (40, 512, 4)])
def test_pq_rankings_replay(N, M, dsub):
    k = min(N, 100)
    codes = synth.pq_codes(N, M, 256, SEED + 2, device=DEV)
    cb = synth.pq_codebooks(M, 256, dsub, SEED + 3, device=DEV)
    w = synth.normal_vector(M * dsub, 1.0, SEED + 4, device=DEV)
    ws = binding.make_workspace(N, k)
    out = binding._outputs(1, k, DEV)
    _check_replays(lambda: binding.rank_pq_model(codes, cb, w, 0.0, k, ws, out=out), w, out,
                   lambda r: synth.normal_vector(M * dsub, 1.0, SEED + 30 + r, device=DEV))
    lut = torch.empty((M, 256), dtype=torch.float32, device=DEV)

    def two_calls():
        binding.pq_build_lut(cb, w, lut)
        binding.rank_pq(codes, lut, 0.0, k, ws, out=out)
    _check_replays(two_calls, w, out, lambda r: synth.normal_vector(M * dsub, 1.0, SEED + 40 + r, device=DEV))


def test_binary_and_hamming_rankings_replay():
    N, D, k = 1150000, 2048, 200
    bits = synth.binary_bits_random(N, D // 32, SEED + 5, device=DEV)
    w = synth.normal_vector(D, 1.0, SEED + 6, device=DEV)
    ws = binding.make_workspace(N, k)
    out = binding._outputs(1, k, DEV)
    _check_replays(lambda: binding.rank_binary(bits, D, w, 0.0, k, ws, out=out), w, out,
                   lambda r: synth.normal_vector(D, 1.0, SEED + 50 + r, device=DEV))
    q = synth.binary_bits_random(1, D // 32, SEED + 7, device=DEV)[0].contiguous()
    _check_replays(lambda: binding.rank_hamming(bits, D, q, k, ws, out=out), q, out,
                   lambda r: synth.binary_bits_random(1, D // 32, SEED + 60 + r, device=DEV)[0])


def test_multi_classifier_topk_and_training_pass_replay():
    N, D, Q, k = 1100000, 256, 64, 50
    X = synth.dense_features(N, D, SEED + 8, device=DEV, dtype=torch.float16)
    W = synth.normal_matrix(Q, D, 0.05, SEED + 9, device=DEV, dtype=torch.float16)
    ws = binding.make_workspace(N, k, Q)
    out = binding._outputs(Q, k, DEV)
    _check_replays(lambda: binding.rank_dense(X, W, None, k, ws, out=out), W, out,
                   lambda r: synth.normal_matrix(Q, D, 0.05, SEED + 70 + r, device=DEV, dtype=torch.float16))
    S = synth.normal_vector(3000000, 1.0, SEED + 11, device=DEV)
    ws1 = binding.make_workspace(S.numel(), 1000)
    out1 = binding._outputs(1, 1000, DEV)
    _check_replays(lambda: binding.topk(S, 1000, ws1, out=out1), S, out1,
                   lambda r: synth.normal_vector(3000000, 1.0, SEED + 80 + r, device=DEV))
    # a training pass: w is input and output, so every replay starts from a fresh copy of w0
    Dw, B, steps = 512, 64, 20
    Xp, Xn = synth.sgd_pools(Dw, 200, 800, SEED + 12, device=DEV)
    ip, ineg = synth.sgd_batches(200, 800, B, steps, SEED + 13)
    ip, ineg = torch.from_numpy(ip).to(DEV), torch.from_numpy(ineg).to(DEV)
    wsg = binding.sgd_workspace(B)
    w0 = synth.normal_vector(Dw, 0.01, SEED + 14, device=DEV)
    w = torch.empty_like(w0)

    def train():
        w.copy_(w0)
        binding.svm_sgd_pass(w, None, Xp, ip, Xn, ineg, 1e-2, 1, False, wsg)
    train()
    torch.cuda.synchronize()
    want = w.clone()
    g = _capture(train)
    for r in range(3):
        w.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(w, want), "training replay %d" % r
