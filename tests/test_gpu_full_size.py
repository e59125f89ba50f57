"""GPU parity at the full size of the dense linear-SVM configuration (n = 1,000,000, d = 1024,
pools of 16,384), in the launch configuration bench.py times: the epoch driver with the
device-side step-size schedule.  The oracle replays the first pools in full (it needs
about 0.1 s per pool) and the last, short pool of the epoch."""
import math

import numpy as np
import pytest
import torch

from paper_1905_03381_amd import api, synth

from gpu_util import (RTOL, abs_dot_scale, assert_close_scaled, assert_logit_prob, clear_draws, dev,
                      host, scalar_dev)

pytestmark = pytest.mark.gpu

N, D, P = 1_000_000, 1024, 16384
GAMMA, LAM, LR0, LR_A, SEED = 0.1, 1e-4, 256.0, 0.1, 42   # the bench's step size


@pytest.fixture(scope="module")
def workload():
    X, y, _ = synth.dense_svm(n=N, d=D, threads=16)
    Xd = torch.from_numpy(X).cuda()
    return X, y, Xd, torch.from_numpy(y).cuda()


def test_first_pools_and_last_short_pool(ref, workload):
    from stepwise import check_epoch
    X, y, Xd, yd = workload
    perm = synth.epoch_permutation(N, seed=7, epoch=0)
    Fh = ref.Features.dense(X)
    F = api.Features.dense(Xd)
    ws = api.Workspace(P, D)
    Tt = scalar_dev(0.0)
    steps = 3
    # the first pools of the epoch at the bench's step size: every step against the oracle step
    # from the GPU's previous state (single-step tolerances), then the three steps in one call
    # (the first two compacted by the pass of the step after them, at exactly the 64 positions
    # per block that pass can carry) bit-identical to the step-wise run
    zeros = np.zeros(D, np.float32)
    counts, state = check_epoch(ref, Fh, F, y, perm, steps * P, P, zeros, zeros, 0.0, gamma=GAMMA,
                                seed=SEED, step0=0, lam=LAM, lr0=LR0, lr_a=LR_A, T=0.0, ws=ws)
    assert all(0 < m < P for m in counts)
    w, phi, b = dev(state[0]), dev(state[1]), dev(state[2])

    # one more full step from that state with every output compared element by element,
    # then the last pool of the epoch (576 rows)
    for t, lo, size in [(steps, steps * P, P), (N // P, (N // P) * P, N - (N // P) * P)]:
        idx = perm[lo:lo + size]
        w0, phi0, b0 = host(w).copy(), host(phi).copy(), float(host(b)[0])
        lr = float(np.float32(LR0 / math.sqrt(t + 1)))
        out = ref.step(Fh, y, idx, size, w0, phi0, b0, GAMMA, SEED, t, LAM, lr, 0.0, LR_A)
        clear = clear_draws(ref, out["prob"], GAMMA, SEED, t)
        cfg = api.step_config(GAMMA, LAM, lr, LR_A, 0.0, SEED, t, Tt)
        logit = torch.zeros(size, device="cuda")
        prob = torch.zeros(size, device="cuda")
        keep = torch.zeros(size, dtype=torch.uint8, device="cuda")
        pos = torch.zeros(size, dtype=torch.int32, device="cuda")
        ids = torch.zeros(size, dtype=torch.int32, device="cuda")
        loss = torch.zeros(size, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        api.fused_step(F, yd, dev(idx), size, w, phi, b, cfg, logit, prob, keep, pos, ids, loss,
                       cnt, ws)
        assert_logit_prob(host(logit), host(prob), out["logit"], out["prob"],
                          abs_dot_scale(Fh, idx, phi0), bias=b0)
        assert np.array_equal(host(keep)[clear], out["keep"][clear])
        kept = np.flatnonzero(host(keep))
        m = kept.size
        assert int(host(cnt)[0]) == m
        assert np.array_equal(host(pos)[:m], kept)                 # compaction of the GPU's own mask
        assert np.array_equal(host(ids)[:m], idx[kept])
        if clear.all():
            assert m == out["m"] and np.array_equal(kept, out["kept_pos"])
        # Boss step and Assistant update of the oracle on the rows the GPU kept
        ids_g = idx[kept].astype(np.int32)
        w_ref, loss_ref = ref.svm_sgd_step(Fh, y, ids_g, m, w0, LAM, lr)
        phi_ref, b_ref = ref.assistant_update(Fh, ids_g, m, loss_ref, 0.0, phi0, b0, LR_A)
        S = abs_dot_scale(Fh, ids_g, w0)
        assert_close_scaled(host(loss)[:m], loss_ref, S, "loss")
        Xk = np.abs(X[ids_g].astype(np.float64))
        marg = y[ids_g].astype(np.float64) * (X[ids_g].astype(np.float64) @ w0.astype(np.float64))
        near = np.abs(1.0 - marg) <= RTOL * (S + 1.0)
        w_scale = abs(1 - lr * LAM) * np.abs(w0.astype(np.float64)) + lr / m * Xk[marg < 1].sum(axis=0)
        assert_close_scaled(host(w), w_ref, w_scale, "w", atol=lr / m * Xk[near].sum(axis=0))
        phi_scale = np.abs(phi0.astype(np.float64)) + LR_A / m * Xk.sum(axis=0)
        assert_close_scaled(host(phi), phi_ref, phi_scale, "phi", atol=LR_A / m * Xk[near].sum(axis=0))
        assert abs(float(host(b)[0]) - b_ref) <= RTOL * (abs(b0) + LR_A) + LR_A / m * int(near.sum())


def test_pools_of_262144_rows(ref, workload):
    """The same whole step with pools sixteen times the configuration's (the launch bench.py
    times beside its headline figure): two steps, each against the oracle step from the GPU's
    previous state, then both in one call bit for bit.  A wave walks 128 rows here, the
    compaction runs in the update kernel's tile blocks (no carried compaction at this size)."""
    from stepwise import check_epoch
    X, y, Xd, yd = workload
    big = 262144
    perm = synth.epoch_permutation(N, seed=7, epoch=1)
    Fh = ref.Features.dense(X)
    F = api.Features.dense(Xd)
    ws = api.Workspace(big, D)
    zeros = np.zeros(D, np.float32)
    counts, _ = check_epoch(ref, Fh, F, y, perm, 2 * big, big, zeros, zeros, 0.0, gamma=GAMMA, seed=SEED,
                            step0=5, lam=LAM, lr0=LR0, lr_a=LR_A, T=0.0, ws=ws)
    assert all(0.3 * big < m < 0.8 * big for m in counts)


def test_dense_slice_five_epochs_every_step(ref):
    """A 65,536-row slice of the dense configuration (d = 1024, pools of 16,384) trained for five
    epochs at the bench's step size through aa_train_epoch: every one of the 20 steps is
    compared with the oracle step taken from the GPU's previous state, and each epoch run in one
    call is bit-identical to its step-wise run.  State, update counter and Philox step carry
    over from epoch to epoch as in the bench."""
    from stepwise import check_epoch
    n = 65_536
    X, y, _ = synth.dense_svm(n=n, d=D, threads=16)
    Fh = ref.Features.dense(X)
    F = api.Features.dense(torch.from_numpy(X).cuda())
    ws = api.Workspace(P, D)
    w, phi, b, t_upd = np.zeros(D, np.float32), np.zeros(D, np.float32), 0.0, 0
    rates = []
    for e in range(5):
        perm = synth.epoch_permutation(n, seed=7, epoch=e)
        counts, state = check_epoch(ref, Fh, F, y, perm, n, P, w, phi, b, gamma=GAMMA, seed=SEED,
                                    step0=4 * e, lam=LAM, lr0=LR0, lr_a=LR_A, T=0.0, ws=ws,
                                    t_upd0=t_upd)
        w, phi, b, t_upd = state[0], state[1], float(state[2][0]), state[3]
        rates.append(sum(counts) / n)
    assert t_upd == 20
    assert all(0.2 < r < 0.95 for r in rates)    # rows are dropped in every epoch, never all


def test_gather_full_pool_rows_bit_exact(ref, workload):
    X, y, Xd, yd = workload
    perm = synth.epoch_permutation(N, seed=7, epoch=1)
    idx = perm[:P]
    prob = np.random.default_rng(5).random(P).astype(np.float32)
    keep_ref, pos_ref = ref.shrink(prob, GAMMA, SEED, 99)
    ws = api.Workspace(P, D)
    keep = torch.zeros(P, dtype=torch.uint8, device="cuda")
    pos = torch.zeros(P, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.shrink(dev(prob), P, GAMMA, SEED, 99, keep, pos, cnt, ws)
    m = pos_ref.size
    assert int(host(cnt)[0]) == m and np.array_equal(host(pos)[:m], pos_ref)
    Xk = torch.zeros((P, D), device="cuda")
    ids = torch.zeros(P, dtype=torch.int32, device="cuda")
    api.gather(Xd, 4 * D, dev(idx), pos, cnt, P, Xk, ids)
    want_rows, want_ids = ref.gather(X, idx, pos_ref)
    assert np.array_equal(host(ids)[:m], want_ids)
    assert np.array_equal(host(Xk)[:m].view(np.uint32), want_rows.view(np.uint32))
