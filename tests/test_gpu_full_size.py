"""GPU parity at the full size of the dense linear-SVM configuration (n = 1,000,000, d = 1024,
pools of 16,384), in the launch configuration bench.py times: the epoch driver with the
device-side step-size schedule.  The oracle replays the first pools in full (it needs
about 0.1 s per pool) and the last, short pool of the epoch."""
import math

import numpy as np
import pytest
import torch

from paper_1905_03381_amd import api, synth

from gpu_util import (abs_dot_scale, assert_close_scaled, assert_logit_prob, clear_draws, dev, host,
                      scalar_dev)

pytestmark = pytest.mark.gpu

N, D, P = 1_000_000, 1024, 16384
GAMMA, LAM, LR0, LR_A, SEED = 0.1, 1e-4, 1.0, 0.1, 42


@pytest.fixture(scope="module")
def workload():
    X, y, _ = synth.dense_svm(n=N, d=D, threads=16)
    Xd = torch.from_numpy(X).cuda()
    return X, y, Xd, torch.from_numpy(y).cuda()


def test_first_pools_and_last_short_pool(ref, workload):
    X, y, Xd, yd = workload
    perm = synth.epoch_permutation(N, seed=7, epoch=0)
    Fh = ref.Features.dense(X)
    F = api.Features.dense(Xd)
    ws = api.Workspace(P, D)
    Tt = scalar_dev(0.0)
    steps = 3
    # oracle trajectory over the first pools
    w_r, phi_r, b_r = np.zeros(D, np.float32), np.zeros(D, np.float32), 0.0
    ms, batches = [], []
    for t in range(steps):
        idx = perm[t * P:(t + 1) * P]
        lr = np.float32(np.float32(LR0) / np.sqrt(np.float32(t + 1)))
        out = ref.step(Fh, y, idx, P, w_r, phi_r, b_r, GAMMA, SEED, t, LAM, lr, 0.0, LR_A)
        assert clear_draws(ref, out["prob"], GAMMA, SEED, t).all()
        assert out["m"] > 0
        w_r, phi_r, b_r = out["w"], out["phi"], out["bias"]
        ms.append(out["m"])
        batches.append((out["kept_ids"], out["loss"]))
    w, phi, b = torch.zeros(D, device="cuda"), torch.zeros(D, device="cuda"), scalar_dev(0.0)
    tu = torch.zeros(1, dtype=torch.int32, device="cuda")
    hist = torch.zeros(steps, dtype=torch.int32, device="cuda")
    cfg = api.step_config(GAMMA, LAM, LR0, LR_A, 0.0, SEED, 0, Tt)
    ids_hist = torch.full((steps, P), -1, dtype=torch.int32, device="cuda")
    loss_hist = torch.full((steps, P), -3.0, device="cuda")
    api.train_epoch(F, yd, dev(perm), steps * P, P, w, phi, b, cfg, tu, hist, ws, ids_hist, loss_hist)
    assert np.array_equal(host(hist), np.array(ms))      # kept counts: exact
    # the batch of every step (the first two compacted by the pass of the step after them,
    # at exactly the 64 positions per block that pass can carry): ids exact, losses close
    for t, (ids_ref, loss_ref) in enumerate(batches):
        assert np.array_equal(host(ids_hist)[t, :ms[t]], ids_ref), f"batch {t}"
        assert np.all(host(ids_hist)[t, ms[t]:] == -1)
        assert np.allclose(host(loss_hist)[t, :ms[t]], loss_ref, rtol=1e-4, atol=1e-5)
        assert np.all(host(loss_hist)[t, ms[t]:] == -3.0)
    assert np.allclose(host(w), w_r, rtol=1e-4, atol=1e-7)
    assert np.allclose(host(phi), phi_r, rtol=1e-4, atol=1e-7)
    assert abs(float(host(b)[0]) - b_r) < 1e-5

    # one more full step from that state with every output compared element by element,
    # then the last pool of the epoch (576 rows)
    for t, lo, size in [(steps, steps * P, P), (N // P, (N // P) * P, N - (N // P) * P)]:
        idx = perm[lo:lo + size]
        w0, phi0, b0 = host(w).copy(), host(phi).copy(), float(host(b)[0])
        lr = float(np.float32(LR0 / math.sqrt(t + 1)))
        out = ref.step(Fh, y, idx, size, w0, phi0, b0, GAMMA, SEED, t, LAM, lr, 0.0, LR_A)
        assert clear_draws(ref, out["prob"], GAMMA, SEED, t).all()
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
        m = out["m"]
        assert int(host(cnt)[0]) == m
        assert_logit_prob(host(logit), host(prob), out["logit"], out["prob"],
                          abs_dot_scale(Fh, idx, phi0), bias=b0)
        assert np.array_equal(host(keep), out["keep"])
        assert np.array_equal(host(pos)[:m], out["kept_pos"])
        assert np.array_equal(host(ids)[:m], out["kept_ids"])
        assert_close_scaled(host(loss)[:m], out["loss"], abs_dot_scale(Fh, out["kept_ids"], w0),
                            "loss")
        assert np.allclose(host(w), out["w"], rtol=1e-5, atol=1e-6)
        assert np.allclose(host(phi), out["phi"], rtol=1e-5, atol=1e-6)


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
