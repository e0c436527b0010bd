"""otf_svm_sgd_pass by both routes -- two launches per step (the default) and the whole run as one
kernel whose workgroups meet once per step (diagnostic switch) -- against the CPU oracle and against
each other; the bounded waits of the one-kernel route; the index check."""
import numpy as np
import pytest
import torch

from paper_1407_4764_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SEED = synth.BASE_SEED + 14000


def _setup(D, n_pos_pool, n_neg_pool, B, steps, seed):
    Xp, Xn = synth.sgd_pools(D, n_pos_pool, n_neg_pool, seed, n_shift_dims=min(50, D // 4))
    ip, ineg = synth.sgd_batches(n_pos_pool, n_neg_pool, B, steps, seed + 1)
    return Xp, Xn, ip, ineg


@pytest.mark.parametrize("D,B,lam,steps,update_bias", [(2048, 256, 1e-4, 40, False), (128, 32, 1.0, 60, False),
                                                       (512, 64, 1e-2, 30, True), (260, 10, 0.1, 25, True),
                                                       (1024, 2, 0.5, 20, False), (2048, 4096, 1e-3, 3, False)])
def test_run_matches_the_oracle_and_the_reference_route(oracle, D, B, lam, steps, update_bias, debug_switches):
    Xp, Xn, ip, ineg = _setup(D, 300, 1200, B, steps, SEED + D + B)
    ipd, ind = torch.from_numpy(ip).to(DEV), torch.from_numpy(ineg).to(DEV)
    Xpd, Xnd = Xp.to(DEV), Xn.to(DEV)
    ws = binding.sgd_workspace(B)
    w0 = synth.normal_vector(D, 0.01, SEED + 2)

    def run():
        w = w0.to(DEV)
        b = torch.full((1,), 0.25, device=DEV) if update_bias else None
        binding.svm_sgd_pass(w, b, Xpd, ipd, Xnd, ind, lam, 3, update_bias, ws)
        assert binding.sgd_pass_status(ws) == 0
        return w.cpu().numpy().astype(np.float64), (float(b.item()) if update_bias else 0.0)
    w_two, b_two = run()
    debug_switches({binding.DEBUG_SGD_PASS_PATH: 1})
    w_one, b_one = run()
    # the oracle, free-running in fp64 from the same start
    w, b = w0.numpy().astype(np.float64), 0.25 if update_bias else 0.0
    for s in range(steps):
        w, b, _ = oracle.sgd_step(w.astype(np.float32), b, Xp.numpy(), ip[s], Xn.numpy(), ineg[s], lam, 3 + s, update_bias)
    scale = max(np.abs(w).max(), 1e-30)
    assert np.max(np.abs(w_one - w)) <= 5e-4 * scale, "one launch vs oracle"
    assert np.max(np.abs(w_two - w)) <= 5e-4 * scale, "reference route vs oracle"
    assert np.max(np.abs(w_one - w_two)) <= 5e-4 * scale
    if update_bias:
        assert abs(b_one - b) <= 5e-4 * max(abs(b), 1.0) and abs(b_two - b) <= 5e-4 * max(abs(b), 1.0)


def test_one_step_runs_equal_single_steps_exactly_in_their_decisions(oracle, debug_switches):
    """Teacher-forced: every step started from the oracle's rounded model, one-kernel run of a single step."""
    debug_switches({binding.DEBUG_SGD_PASS_PATH: 1})
    D, B, lam = 2048, 256, 1e-4
    Xp, Xn, ip, ineg = _setup(D, 200, 900, B, 12, SEED + 5)
    Xpd, Xnd = Xp.to(DEV), Xn.to(DEV)
    ws = binding.sgd_workspace(B)
    w = np.zeros(D, dtype=np.float32)
    for s in range(12):
        wd = torch.from_numpy(w).to(DEV)
        binding.svm_sgd_pass(wd, None, Xpd, torch.from_numpy(ip[s:s + 1]).to(DEV), Xnd,
                             torch.from_numpy(ineg[s:s + 1]).to(DEV), lam, s + 1, False, ws)
        ref, _, margins = oracle.sgd_step(w, 0.0, Xp.numpy(), ip[s], Xn.numpy(), ineg[s], lam, s + 1, False)
        got = wd.cpu().numpy().astype(np.float64)
        if np.all(np.abs(1.0 - margins) > 1e-5):                  # no row sits on the kink: the violator sets agree
            assert np.max(np.abs(got - ref)) <= 1e-4 * np.abs(ref).max(), "step %d" % (s + 1)
        w = ref.astype(np.float32)


def test_a_wait_that_expires_ends_the_kernel_and_raises_the_status_word(debug_switches):
    """One poll per wait: the workgroups cannot all have arrived by then, so the first one to look gives up,
    the others follow, the kernel ends normally, the status reads 1 and the model is untouched.  Forced from
    the host through the spin limit: nothing hangs."""
    D, B, lam, steps = 2048, 256, 1e-4, 50
    Xp, Xn, ip, ineg = _setup(D, 300, 1200, B, steps, SEED + 6)
    ws = binding.sgd_workspace(B)
    w0 = synth.normal_vector(D, 0.01, SEED + 7).to(DEV)
    w = w0.clone()
    args = (Xp.to(DEV), torch.from_numpy(ip).to(DEV), Xn.to(DEV), torch.from_numpy(ineg).to(DEV), lam, 1, False, ws)
    debug_switches({binding.DEBUG_SGD_PASS_PATH: 1, binding.DEBUG_SGD_SPIN_LIMIT: 1})
    binding.svm_sgd_pass(w, None, *args)
    assert binding.sgd_pass_status(ws) == 1
    assert torch.equal(w, w0)
    binding.debug_set(binding.DEBUG_SGD_SPIN_LIMIT, 0)            # back to the default bound: the same call completes
    binding.svm_sgd_pass(w, None, *args)
    assert binding.sgd_pass_status(ws) == 0
    assert not torch.equal(w, w0)


def test_row_numbers_outside_the_pool_are_found():
    idx = torch.tensor([0, 5, 99, 100, -1, 7], dtype=torch.int32, device=DEV)
    binding.check_indices(idx[:3], 100)
    with pytest.raises(IndexError, match="2 of 6"):
        binding.check_indices(idx, 100)
