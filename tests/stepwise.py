"""Chained parity at the stated bar.

A chain of steps cannot be compared with an oracle chain at 1e-5 (rounding differences of one
step are the inputs of the next), so the chain is re-synchronised every step: the GPU runs the
epoch one step per call, and after each step the oracle computes the same step FROM THE GPU'S
PREVIOUS STATE.  Dense or CSR rows.  Every stage is then held to the single-step tolerances of gpu_util:

  * keep decisions: equal to the oracle's wherever the draw is farther than 1e-6 from its
    probability (the GPU's mask is rebuilt from its kept ids);
  * compaction and ids: the kept ids are exactly the pool ids at the kept positions, in
    increasing position (bit-exact, no exclusions);
  * losses, w, phi, bias: |gpu - ref| <= 1e-5 max(|ref|, S), the oracle's SVM step and
    Assistant update being taken on the rows the GPU kept; a row whose margin is within 1e-5 S
    of the hinge kink (or whose loss is that close to T) may fall on either side and widens
    the bound of w (phi) by its own term.

The caller then runs the same epoch in ONE call (compaction carried from pass to pass, device
step-size schedule) and requires bit-identical counts, batches and final state.
"""
import numpy as np
import torch

from paper_1905_03381_amd import api

from gpu_util import (DRAW_BAND, RTOL, abs_dot_scale, assert_close_scaled, col_abs_sum, dev, host, row_dots,
                      scalar_dev)


def pools_of(n_perm, P):
    return [(lo, min(P, n_perm - lo)) for lo in range(0, n_perm, P)]


def run_stepwise(ref, Fh, F, y, perm, n_perm, P, w0, phi0, b0, gamma, seed, step0, lam, lr0, lr_a, T,
                 ws, hard=False, t_upd0=0):
    """GPU epoch one step per call, oracle re-synchronised every step.  Returns the per-step
    kept counts, kept ids, losses and the final (w, phi, b, t_upd) of the GPU."""
    yd, permd = dev(y), dev(perm)
    w = dev(w0)
    phi = None if hard else dev(phi0)
    b = None if hard else scalar_dev(b0)
    Tt = scalar_dev(T)
    tu = torch.full((1,), t_upd0, dtype=torch.int32, device="cuda")
    counts, batches = [], []
    t_upd = t_upd0
    for t, (lo, Pt) in enumerate(pools_of(n_perm, P)):
        idx = perm[lo:lo + Pt]
        w_prev = host(w).copy()
        phi_prev = None if hard else host(phi).copy()
        b_prev = 0.0 if hard else float(host(b)[0])
        hist = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        ids = torch.full((1, P), -1, dtype=torch.int32, device="cuda")
        loss = torch.full((1, P), -3.0, device="cuda")
        if hard:
            api.sk_epoch(F, yd, permd[lo:], Pt, P, w, Tt, lam, lr0, tu, hist, ws, ids, loss)
        else:
            cfg = api.step_config(gamma, lam, lr0, lr_a, 0.0, seed, step0 + t, Tt)
            api.train_epoch(F, yd, permd[lo:], Pt, P, w, phi, b, cfg, tu, hist, ws, ids, loss)
        m = int(host(hist)[0])
        ids_g, loss_g = host(ids)[0].copy(), host(loss)[0].copy()
        assert np.all(ids_g[m:] == -1) and np.all(loss_g[m:] == -3.0), f"step {t}: tails touched"
        ids_g, loss_g = ids_g[:m], loss_g[:m]

        # ---- keep decisions and compaction
        where = {int(v): j for j, v in enumerate(idx)}
        pos_g = np.array([where[int(v)] for v in ids_g], dtype=np.int64)
        assert np.all(np.diff(pos_g) > 0), f"step {t}: kept ids are not in pool order"
        keep_g = np.zeros(Pt, dtype=bool)
        keep_g[pos_g] = True
        Sw_pool = abs_dot_scale(Fh, idx, w_prev)
        if hard:
            marg = (y[idx].astype(np.float64) * row_dots(Fh, idx, w_prev)).astype(np.float32)
            loss_pool = np.maximum(0.0, 1.0 - marg.astype(np.float64))
            sure = np.abs(loss_pool - T) > RTOL * (Sw_pool + 1.0)
            assert np.array_equal(keep_g[sure], (loss_pool > T)[sure]), f"step {t}: keep by loss"
        else:
            _, prob_ref = ref.assistant_score(Fh, idx, Pt, phi_prev, bias=b_prev)
            keep_ref, _ = ref.shrink(prob_ref, gamma, seed, step0 + t)
            u = ref.uniforms(seed, step0 + t, Pt).astype(np.float64)
            p = gamma + (1.0 - gamma) * prob_ref.astype(np.float64)
            sure = np.abs(u - p) > DRAW_BAND
            assert np.array_equal(keep_g[sure], keep_ref.astype(bool)[sure]), f"step {t}: keep mask"
        counts.append(m)
        batches.append((ids_g, loss_g))
        if m == 0:
            assert np.array_equal(host(w), w_prev)
            continue

        # ---- Boss step on the rows the GPU kept, from the GPU's previous state
        lr = np.float32(np.float32(lr0) / np.sqrt(np.float32(t_upd + 1)))
        t_upd += 1
        w_ref, loss_ref = ref.svm_sgd_step(Fh, y, ids_g, m, w_prev, lam, lr)
        S = abs_dot_scale(Fh, ids_g, w_prev)
        assert_close_scaled(loss_g, loss_ref, S, f"step {t}: loss")
        marg = y[ids_g].astype(np.float64) * row_dots(Fh, ids_g, w_prev)
        active = marg < 1
        near_kink = np.abs(1.0 - marg) <= RTOL * (S + 1.0)
        w_scale = (abs(1 - lr * lam) * np.abs(w_prev.astype(np.float64))
                   + float(lr) / m * col_abs_sum(Fh, ids_g[active]))
        w_atol = float(lr) / m * col_abs_sum(Fh, ids_g[near_kink]) if near_kink.any() else 0.0
        assert_close_scaled(host(w), w_ref, w_scale, f"step {t}: w", atol=w_atol)
        if hard:
            continue
        # ---- Assistant update labelled by those losses
        phi_ref, b_ref = ref.assistant_update(Fh, ids_g, m, loss_ref, T, phi_prev, b_prev, lr_a)
        near_T = np.abs(loss_ref.astype(np.float64) - T) <= RTOL * (S + 1.0)
        phi_scale = np.abs(phi_prev.astype(np.float64)) + lr_a / m * col_abs_sum(Fh, ids_g)
        phi_atol = lr_a / m * col_abs_sum(Fh, ids_g[near_T]) if near_T.any() else 0.0
        assert_close_scaled(host(phi), phi_ref, phi_scale, f"step {t}: phi", atol=phi_atol)
        b_bound = RTOL * (abs(b_prev) + lr_a) + lr_a / m * int(near_T.sum())
        assert abs(float(host(b)[0]) - b_ref) <= b_bound, f"step {t}: bias"
    state = (host(w).copy(), None if hard else host(phi).copy(), None if hard else host(b).copy(),
             int(host(tu)[0]))
    assert state[3] == t_upd
    return counts, batches, state


def run_whole(F, y, perm, n_perm, P, w0, phi0, b0, gamma, seed, step0, lam, lr0, lr_a, T, ws, hard=False,
              t_upd0=0):
    """The same epoch in one call: kept counts, batches, final state."""
    steps = len(pools_of(n_perm, P))
    w = dev(w0)
    phi = None if hard else dev(phi0)
    b = None if hard else scalar_dev(b0)
    Tt = scalar_dev(T)
    tu = torch.full((1,), t_upd0, dtype=torch.int32, device="cuda")
    hist = torch.full((steps,), -1, dtype=torch.int32, device="cuda")
    ids = torch.full((steps, P), -1, dtype=torch.int32, device="cuda")
    loss = torch.full((steps, P), -3.0, device="cuda")
    if hard:
        api.sk_epoch(F, dev(y), dev(perm), n_perm, P, w, Tt, lam, lr0, tu, hist, ws, ids, loss)
    else:
        cfg = api.step_config(gamma, lam, lr0, lr_a, 0.0, seed, step0, Tt)
        api.train_epoch(F, dev(y), dev(perm), n_perm, P, w, phi, b, cfg, tu, hist, ws, ids, loss)
    state = (host(w).copy(), None if hard else host(phi).copy(), None if hard else host(b).copy(),
             int(host(tu)[0]))
    return host(hist).tolist(), host(ids), host(loss), state


def check_epoch(ref, Fh, F, y, perm, n_perm, P, w0, phi0, b0, gamma, seed, step0, lam, lr0, lr_a, T, ws,
                hard=False, t_upd0=0):
    """Step-wise parity against the oracle, then bit-equality of the one-call epoch with the
    step-wise GPU run.  Returns (counts, final state)."""
    counts, batches, state = run_stepwise(ref, Fh, F, y, perm, n_perm, P, w0, phi0, b0, gamma, seed,
                                          step0, lam, lr0, lr_a, T, ws, hard, t_upd0)
    hist, ids, loss, state1 = run_whole(F, y, perm, n_perm, P, w0, phi0, b0, gamma, seed, step0, lam,
                                        lr0, lr_a, T, ws, hard, t_upd0)
    assert hist == counts
    for t, (ids_g, loss_g) in enumerate(batches):
        m = counts[t]
        assert np.array_equal(ids[t, :m], ids_g) and np.all(ids[t, m:] == -1), f"batch {t}: ids"
        assert np.array_equal(loss[t, :m], loss_g) and np.all(loss[t, m:] == -3.0), f"batch {t}: losses"
    assert state1[3] == state[3]
    assert np.array_equal(state1[0], state[0]), "w of the one-call epoch differs in bits"
    if not hard:
        assert np.array_equal(state1[1], state[1]) and np.array_equal(state1[2], state[2])
    return counts, state
