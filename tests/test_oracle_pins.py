"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each pin compares the oracle with
something other than itself: published known-answer vectors, closed forms,
library routines (numpy, scipy, torch autograd, scikit-learn), statistical
invariants of Bernoulli draws, or brute force on tiny inputs.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.sparse as sp
import scipy.stats as st
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------------------
# Philox and the uniform of Algorithm 1


def test_philox_known_answers(ref):
    rows = [l for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if not l.startswith("#")]
    assert len(rows) == 3
    for line in rows:
        lhs, rhs = line.split("|")
        v = [int(t, 16) for t in lhs.split()]
        want = [int(t, 16) for t in rhs.split()]
        got = ref.philox4x32_10(v[:4], v[4:6])
        assert [int(g) for g in got] == want


def test_uniform_counter_layout(ref):
    # counter = (j, 0, lo(step), hi(step)); key = (lo(seed), hi(seed)); top 24 bits of word 0
    for seed, step, j in [(42, 7, 5), (0xDEADBEEF12345678, 0x1_0000_0003, 123456), (0, 0, 0)]:
        out = ref.philox4x32_10([j, 0, step & 0xFFFFFFFF, step >> 32],
                                [seed & 0xFFFFFFFF, seed >> 32])
        assert ref.uniform(seed, step, j) == float(int(out[0]) >> 8) * 2.0 ** -24
    # value computed with an independent implementation when the counter layout was chosen
    out = ref.philox4x32_10([5, 0, 7, 0], [42, 0])
    assert int(out[0]) == 0x0D09DEB5
    assert ref.uniform(42, 7, 5) == pytest.approx(0.05093181133270264, abs=0)


def test_uniform_distribution(ref):
    u = ref.uniforms(1234, 9, 100_000).astype(np.float64)
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2 ** 24 == np.round(u * 2 ** 24))  # on the 2^-24 grid
    assert abs(u.mean() - 0.5) < 5 / math.sqrt(12 * u.size)
    assert st.kstest(u, "uniform").pvalue > 1e-3
    # different steps and seeds give different streams
    assert not np.array_equal(u[:100], ref.uniforms(1234, 10, 100))
    assert not np.array_equal(u[:100], ref.uniforms(1235, 9, 100))


# ---------------------------------------------------------------------------
# Assistant score


def test_score_selects_coordinate_and_bias(ref):
    X = rng(0).standard_normal((50, 7)).astype(np.float32)
    F = ref.Features.dense(X)
    for k in range(7):
        phi = np.zeros(7, np.float32)
        phi[k] = 1.0
        logit, prob = ref.assistant_score(F, None, 50, phi)
        assert np.array_equal(logit, X[:, k])
    logit, prob = ref.assistant_score(F, None, 50, np.zeros(7, np.float32), bias=0.75)
    assert np.all(logit == 0.75)
    assert np.allclose(prob, 1 / (1 + math.exp(-0.75)), rtol=1e-7)


def test_score_matches_torch_float64(ref):
    r = rng(1)
    X = r.standard_normal((300, 129)).astype(np.float32)
    phi = r.standard_normal(129).astype(np.float32)
    idx = r.permutation(300)[:200].astype(np.int32)
    logit, prob = ref.assistant_score(ref.Features.dense(X), idx, 200, phi, bias=-0.3)
    s = torch.from_numpy(X[idx]).double() @ torch.from_numpy(phi).double() - torch.tensor(
        np.float32(-0.3)).double().neg()
    assert np.array_equal(logit, s.float().numpy())
    assert np.allclose(prob, torch.sigmoid(s.float().double()).numpy(), rtol=1e-7, atol=0)


def test_score_padded_rows_and_csr_equal_dense(ref):
    r = rng(2)
    X = r.standard_normal((40, 12)).astype(np.float32)
    X[r.random((40, 12)) < 0.6] = 0.0
    phi = r.standard_normal(12).astype(np.float32)
    want = ref.assistant_score(ref.Features.dense(X), None, 40, phi, bias=0.1)
    Xp = np.concatenate([X, np.full((40, 4), 99.0, np.float32)], axis=1)
    got = ref.assistant_score(ref.Features.dense(Xp, d=12), None, 40, phi, bias=0.1)
    assert np.array_equal(want[0], got[0]) and np.array_equal(want[1], got[1])
    S = sp.csr_matrix(X)
    Fc = ref.Features.csr(S.indptr, S.indices, S.data, 12)
    got = ref.assistant_score(Fc, None, 40, phi, bias=0.1)
    assert np.array_equal(want[0], got[0]) and np.array_equal(want[1], got[1])
    # val == NULL means all ones
    Fo = ref.Features.csr(S.indptr, S.indices, None, 12)
    got1 = ref.assistant_score(Fo, None, 40, phi)
    ones = (X != 0).astype(np.float64) @ phi.astype(np.float64)
    assert np.array_equal(got1[0], ones.astype(np.float32))


# ---------------------------------------------------------------------------
# Keep draw and compaction (Algorithm 1)


def test_keep_certain_and_impossible(ref):
    P = 4096
    keep, pos = ref.shrink(np.ones(P, np.float32), 0.0, 3, 4)
    assert keep.all() and np.array_equal(pos, np.arange(P))
    keep, pos = ref.shrink(np.zeros(P, np.float32), 0.0, 3, 4)
    assert not keep.any() and pos.size == 0
    keep, pos = ref.shrink(rng(0).random(P).astype(np.float32), 1.0, 3, 4)  # gamma = 1
    assert keep.all() and np.array_equal(pos, np.arange(P))


def test_keep_is_strict_at_a_tie(ref):
    """c < p is strict: a candidate whose probability equals its draw is dropped, the next
    float up is kept (with gamma = 0 the probability is g itself)."""
    u = ref.uniforms(21, 6, 64)
    keep, _ = ref.shrink(u, 0.0, 21, 6)
    assert not keep.any()
    keep, _ = ref.shrink(np.nextafter(u, np.float32(2.0)), 0.0, 21, 6)
    assert keep.all()


@pytest.mark.parametrize("gamma", [0.0, 0.1, 0.5])
def test_keep_probability_is_gamma_plus_one_minus_gamma_g(ref, gamma):
    P = 50_000
    g = rng(5).random(P).astype(np.float32)
    keep, pos = ref.shrink(g, gamma, 77, 3)
    # definition, from the oracle's own uniforms only (not its compare)
    u = ref.uniforms(77, 3, P).astype(np.float64)
    p = gamma + (1 - gamma) * g.astype(np.float64)
    clear = np.abs(u - p) > 1e-6
    assert np.array_equal(keep[clear].astype(bool), (u < p)[clear])
    # kept count tracks sum p
    sigma = math.sqrt(float(np.sum(p * (1 - p))))
    assert abs(int(keep.sum()) - p.sum()) < 5 * sigma
    # compaction is numpy's flatnonzero
    assert np.array_equal(pos, np.flatnonzero(keep))


def test_kept_count_chi_square_over_steps(ref):
    P, T = 2000, 60
    g = rng(6).random(P).astype(np.float32)
    p = 0.1 + 0.9 * g.astype(np.float64)
    var = float(np.sum(p * (1 - p)))
    chi = 0.0
    for t in range(T):
        keep, _ = ref.shrink(g, 0.1, 99, t)
        chi += (keep.sum() - p.sum()) ** 2 / var
    assert st.chi2.sf(chi, T) > 1e-4 and st.chi2.cdf(chi, T) > 1e-4


@pytest.mark.parametrize("gamma", [0.0, 0.1, 0.5, 1.0])
def test_literal_two_branch_sampler_is_a_prefix_of_the_pool_compaction(ref, gamma):
    P = 3000
    g = rng(7).random(P).astype(np.float32)
    keep, pos = ref.shrink(g, gamma, 11, 2)
    u = ref.uniforms(11, 2, P).astype(np.float64)
    p = gamma + (1 - gamma) * g.astype(np.float64)
    assert np.all(np.abs(u - p) > 1e-6), "pick another seed: a draw sits in the rounding band"
    for batch_size in [0, 1, 64, pos.size, pos.size + 10]:
        B, consumed = ref.sample_batch(g, gamma, 11, 2, batch_size)
        want = pos[:batch_size]
        assert np.array_equal(B, want)
        if batch_size and batch_size <= pos.size:
            assert consumed == want[-1] + 1  # stopped right after the last kept candidate
        elif batch_size > pos.size:
            assert consumed == P


def test_threshold_shrink(ref):
    crit = rng(8).standard_normal(1000).astype(np.float32)
    crit[10] = 0.25
    keep, pos = ref.shrink_threshold(crit, 0.25)
    assert np.array_equal(keep.astype(bool), crit > np.float32(0.25)) and not keep[10]
    assert np.array_equal(pos, np.flatnonzero(crit > np.float32(0.25)))


# ---------------------------------------------------------------------------
# Gather


@pytest.mark.parametrize("row_bytes", [1, 3, 16, 4095, 4096])
def test_gather_is_fancy_indexing(ref, row_bytes):
    r = rng(9)
    src = r.integers(0, 256, (200, row_bytes), dtype=np.uint8)
    idx = r.permutation(200)[:150].astype(np.int32)
    kept_pos = np.sort(r.choice(150, 60, replace=False)).astype(np.int32)
    dst, ids = ref.gather(src, idx, kept_pos)
    assert np.array_equal(ids, idx[kept_pos])
    assert np.array_equal(dst, src[idx[kept_pos]])
    dst, ids = ref.gather(src, None, kept_pos)
    assert np.array_equal(ids, kept_pos) and np.array_equal(dst, src[kept_pos])
    _, ids = ref.gather(None, idx, kept_pos)
    assert np.array_equal(ids, idx[kept_pos])


def test_gather_csr_is_scipy_row_indexing(ref):
    r = rng(10)
    S = sp.random(300, 50, density=0.1, format="csr", random_state=3, dtype=np.float32)
    F = ref.Features.csr(S.indptr, S.indices, S.data, 50)
    idx = r.permutation(300)[:100].astype(np.int32)
    kept_pos = np.sort(r.choice(100, 37, replace=False)).astype(np.int32)
    rowptr, col, val = ref.gather_csr(F, idx, kept_pos, int(S.nnz))
    want = S[idx[kept_pos]]
    assert np.array_equal(rowptr, want.indptr)
    assert np.array_equal(col, want.indices) and np.array_equal(val, want.data)
    with pytest.raises(ValueError):
        ref.gather_csr(F, idx, kept_pos, int(want.nnz) - 1)


# ---------------------------------------------------------------------------
# SVM SGD step on kept rows


def test_hinge_step_closed_form_single_row(ref):
    x = np.array([[0.5, -2.0, 1.5]], np.float32)
    F = ref.Features.dense(x)
    for y in (1.0, -1.0):
        w, loss = ref.svm_sgd_step(F, np.array([y], np.float32), None, 1, np.zeros(3), 1e-2, 0.25)
        assert loss[0] == 1.0                       # w = 0: hinge loss is 1
        assert np.array_equal(w, (0.25 * y * x[0]).astype(np.float32))
    # margin >= 1: only the regulariser acts; loss is 0
    w0 = np.array([2.0, 0.0, 0.0], np.float32)
    w, loss = ref.svm_sgd_step(F, np.array([1.0], np.float32), None, 1, w0, 0.5, 0.1)
    assert loss[0] == 0.0 and np.allclose(w, (1 - 0.05) * w0, rtol=1e-7)
    # exactly on the kink (margin == 1): subgradient taken as 0
    w0 = np.array([2.0, 0.0, 0.0], np.float32)
    xk = np.array([[0.5, 1.0, 1.0]], np.float32)
    w, loss = ref.svm_sgd_step(ref.Features.dense(xk), np.array([1.0], np.float32), None, 1, w0,
                               0.0, 0.1)
    assert loss[0] == 0.0 and np.array_equal(w, w0)


def _torch_hinge_objective(X, y, w, lam):
    margins = y * (X @ w)
    return 0.5 * lam * (w @ w) + torch.relu(1 - margins).mean()


def test_hinge_step_matches_autograd_and_finite_differences(ref):
    r = rng(11)
    n, d, m = 80, 9, 33
    X = r.standard_normal((n, d)).astype(np.float32)
    y = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    w0 = (0.3 * r.standard_normal(d)).astype(np.float32)
    rows = r.choice(n, m, replace=False).astype(np.int32)
    lam, lr = 0.05, 0.2
    w1, loss = ref.svm_sgd_step(ref.Features.dense(X), y, rows, m, w0, lam, lr)
    Xt, yt = torch.from_numpy(X[rows]).double(), torch.from_numpy(y[rows]).double()
    wt = torch.from_numpy(w0).double().requires_grad_(True)
    obj = _torch_hinge_objective(Xt, yt, wt, lam)
    obj.backward()
    want = wt.detach() - lr * wt.grad
    assert np.allclose(w1, want.numpy(), rtol=1e-6, atol=1e-7)
    assert np.allclose(loss, torch.relu(1 - yt * (Xt @ wt.detach())).numpy(), rtol=1e-6, atol=1e-7)
    # central finite differences of the batch objective (no margin sits on the kink)
    assert np.min(np.abs(1 - (yt * (Xt @ wt.detach())).numpy())) > 1e-3
    F = ref.Features.dense(X)
    g_fd = np.zeros(d)
    for k in range(d):
        e = np.zeros(d, np.float32)
        e[k] = 1e-3
        g_fd[k] = (ref.primal_objective(F, y, rows, m, w0 + e, lam)
                   - ref.primal_objective(F, y, rows, m, w0 - e, lam)) / float(
            (w0 + e)[k].astype(np.float64) - (w0 - e)[k].astype(np.float64))
    assert np.allclose((w0 - w1) / lr, g_fd, rtol=2e-3, atol=2e-4)
    assert ref.primal_objective(F, y, rows, m, w0, lam) == pytest.approx(obj.item(), rel=1e-8)


def test_hinge_step_empty_batch_and_projection(ref):
    r = rng(12)
    X = r.standard_normal((10, 4)).astype(np.float32)
    y = np.ones(10, np.float32)
    w0 = r.standard_normal(4).astype(np.float32)
    w1, loss = ref.svm_sgd_step(ref.Features.dense(X), y, None, 0, w0, 0.1, 0.5)
    assert np.array_equal(w0, w1) and loss.size == 0
    w_free, _ = ref.svm_sgd_step(ref.Features.dense(X), y, None, 10, w0, 0.1, 0.5)
    w_proj, _ = ref.svm_sgd_step(ref.Features.dense(X), y, None, 10, w0, 0.1, 0.5, radius=0.3)
    nrm = np.linalg.norm(w_free.astype(np.float64))
    assert nrm > 0.3
    assert np.allclose(w_proj, w_free * (0.3 / nrm), rtol=1e-6)
    w_big, _ = ref.svm_sgd_step(ref.Features.dense(X), y, None, 10, w0, 0.1, 0.5, radius=1e3)
    assert np.array_equal(w_big, w_free)


def test_csr_step_equals_dense_step(ref):
    r = rng(13)
    X = r.standard_normal((60, 20)).astype(np.float32)
    X[r.random((60, 20)) < 0.7] = 0
    S = sp.csr_matrix(X)
    y = np.where(r.random(60) < 0.5, 1.0, -1.0).astype(np.float32)
    rows = r.choice(60, 25, replace=False).astype(np.int32)
    w0 = r.standard_normal(20).astype(np.float32) * 0.2
    a = ref.svm_sgd_step(ref.Features.dense(X), y, rows, 25, w0, 0.01, 0.3)
    b = ref.svm_sgd_step(ref.Features.csr(S.indptr, S.indices, S.data, 20), y, rows, 25, w0, 0.01,
                         0.3)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_keep_everything_reduces_to_vanilla_minibatch_sgd(ref):
    """gamma = 1 keeps every candidate, so the step is the plain Pegasos mini-batch step."""
    r = rng(14)
    n, d, P = 500, 16, 128
    X = r.standard_normal((n, d)).astype(np.float32)
    y = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    F = ref.Features.dense(X)
    w_a = np.zeros(d, np.float32)
    w_b = np.zeros(d, np.float32)
    phi = r.standard_normal(d).astype(np.float32)
    perm = r.permutation(n).astype(np.int32)
    for t, s in enumerate(range(0, n, P)):
        idx = perm[s:s + P]
        lr = 0.5 / math.sqrt(t + 1)
        out = ref.step(F, y, idx, idx.size, w_a, phi, 0.0, 1.0, 5, t, 1e-2, lr, 0.0, 0.0)
        assert out["m"] == idx.size and np.array_equal(out["kept_ids"], idx)
        w_a = out["w"]
        w_b = ref.vanilla_minibatch_sgd(F, y, idx, idx.size, w_b, 1e-2, lr)
        assert np.array_equal(w_a, w_b)  # bit-identical


def test_single_row_steps_match_sklearn_hinge_sgd(ref):
    """Pool of one row, everything kept: one epoch equals scikit-learn's plain SGD with
    hinge loss, L2 penalty and a constant step (its textbook per-sample update)."""
    from sklearn.linear_model import SGDClassifier
    r = rng(15)
    n, d = 150, 6
    X = r.standard_normal((n, d)).astype(np.float32)
    y = np.where(X @ r.standard_normal(d) + 0.3 * r.standard_normal(n) > 0, 1.0, -1.0).astype(
        np.float32)
    lam, lr = 0.01, 0.05
    clf = SGDClassifier(loss="hinge", penalty="l2", alpha=lam, fit_intercept=False,
                        learning_rate="constant", eta0=lr, shuffle=False, max_iter=1, tol=None,
                        average=False)
    clf.fit(X.astype(np.float64), y, coef_init=np.zeros((1, d)))
    F = ref.Features.dense(X)
    w = np.zeros(d, np.float32)
    for i in range(n):
        w, _ = ref.svm_sgd_step(F, y, np.array([i], np.int32), 1, w, lam, lr)
    assert np.allclose(w, clf.coef_[0], rtol=1e-4, atol=1e-6)


def test_objective_decreases_on_tiny_strongly_convex_instance(ref):
    r = rng(16)
    n, d = 16, 4
    X = r.standard_normal((n, d)).astype(np.float32)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    y = np.where(X @ np.array([1.0, -1.0, 0.5, 0.0]) > 0, 1.0, -1.0).astype(np.float32)
    F = ref.Features.dense(X)
    lam = 0.1
    idx = np.arange(n, dtype=np.int32)

    def run(gamma, steps, seed):
        w, phi, b = np.zeros(d, np.float32), np.zeros(d, np.float32), 0.0
        objs = [ref.primal_objective(F, y, None, n, w, lam)]
        for t in range(steps):
            out = ref.step(F, y, idx, n, w, phi, b, gamma, seed, t, lam, 0.05, 0.0, 0.1)
            w, phi, b = out["w"], out["phi"], out["bias"]
            objs.append(ref.primal_objective(F, y, None, n, w, lam))
        return np.array(objs)

    vanilla = run(1.0, 400, 1)
    # Full pool and a small constant step: the objective falls monotonically while the
    # iterate travels to the optimum (the first 200 steps here); once it chatters across
    # hinge kinks a subgradient step may rise, but never above the best value by much.
    assert np.all(np.diff(vanilla[:201]) < 0)
    assert np.all(vanilla[200:] <= vanilla[200])
    assert np.all(vanilla[200:] - np.minimum.accumulate(vanilla)[200:] < 5e-4)
    assert vanilla[-1] < 0.5 * vanilla[0]
    shrunk = run(0.1, 400, 1)
    assert shrunk[-1] < shrunk[0]
    assert abs(shrunk[-1] - vanilla[-1]) < 0.05 * vanilla[-1]   # same objective value region


# ---------------------------------------------------------------------------
# Assistant update


def test_assistant_update_matches_autograd(ref):
    r = rng(17)
    n, d, m = 70, 11, 29
    X = r.standard_normal((n, d)).astype(np.float32)
    phi0 = (0.2 * r.standard_normal(d)).astype(np.float32)
    rows = r.choice(n, m, replace=False).astype(np.int32)
    loss = r.gamma(2.0, 0.5, m).astype(np.float32)
    T, lr_a, l2_a, b0 = 0.8, 0.3, 0.02, 0.15
    phi1, b1 = ref.assistant_update(ref.Features.dense(X), rows, m, loss, T, phi0, b0, lr_a, l2_a)
    Xt = torch.from_numpy(X[rows]).double()
    pt = torch.from_numpy(phi0).double().requires_grad_(True)
    bt = torch.tensor(float(np.float32(b0)), dtype=torch.float64, requires_grad=True)
    z = torch.from_numpy((loss > np.float32(T)).astype(np.float64))
    obj = torch.nn.functional.binary_cross_entropy_with_logits(Xt @ pt + bt, z) + 0.5 * l2_a * (
        pt @ pt)
    obj.backward()
    assert np.allclose(phi1, (pt.detach() - lr_a * pt.grad).numpy(), rtol=2e-6, atol=1e-7)
    assert b1 == pytest.approx(float(bt.detach() - lr_a * bt.grad), rel=2e-6)
    # the objective function the oracle exposes is the same cross-entropy
    zz = (loss > np.float32(T)).astype(np.uint8)
    ce = ref.assistant_objective(ref.Features.dense(X), rows, m, zz, phi0, b0)
    assert ce == pytest.approx(float(obj.detach() - 0.5 * l2_a * (pt.detach() @ pt.detach())),
                               rel=1e-10)


def test_assistant_label_direction(ref):
    """T = +inf labels everything trivial (z=0): every keep probability drops;
    T = -inf labels everything informative (z=1): every keep probability rises."""
    r = rng(18)
    X = np.abs(r.standard_normal((40, 5))).astype(np.float32)   # positive features
    F = ref.Features.dense(X)
    phi0 = np.zeros(5, np.float32)
    loss = np.ones(40, np.float32)
    _, g0 = ref.assistant_score(F, None, 40, phi0, bias=0.0)
    phi_d, b_d = ref.assistant_update(F, None, 40, loss, float("inf"), phi0, 0.0, 0.5)
    phi_u, b_u = ref.assistant_update(F, None, 40, loss, float("-inf"), phi0, 0.0, 0.5)
    assert np.all(ref.assistant_score(F, None, 40, phi_d, bias=b_d)[1] < g0)
    assert np.all(ref.assistant_score(F, None, 40, phi_u, bias=b_u)[1] > g0)
    # strict '>' in the label: loss == T is trivial
    phi_e, _ = ref.assistant_update(F, None, 40, loss, 1.0, phi0, 0.0, 0.5)
    assert np.array_equal(phi_e, phi_d)


def test_single_row_assistant_steps_match_sklearn_logistic_sgd(ref):
    from sklearn.linear_model import SGDClassifier
    r = rng(19)
    n, d = 120, 5
    X = r.standard_normal((n, d)).astype(np.float32)
    loss = r.gamma(2.0, 0.5, n).astype(np.float32)
    T, lr_a = 0.9, 0.1
    z = (loss > np.float32(T)).astype(np.int64)
    clf = SGDClassifier(loss="log_loss", penalty=None, alpha=0.0, fit_intercept=True,
                        learning_rate="constant", eta0=lr_a, shuffle=False, max_iter=1, tol=None,
                        average=False)
    clf.fit(X.astype(np.float64), z, coef_init=np.zeros((1, d)), intercept_init=np.zeros(1))
    F = ref.Features.dense(X)
    phi, b = np.zeros(d, np.float32), 0.0
    for i in range(n):
        phi, b = ref.assistant_update(F, np.array([i], np.int32), 1, loss[i:i + 1], T, phi, b, lr_a)
    assert np.allclose(phi, clf.coef_[0], rtol=1e-4, atol=1e-6)
    assert b == pytest.approx(clf.intercept_[0], rel=1e-4, abs=1e-6)


# ---------------------------------------------------------------------------
# Whole step: order of operations, and brute force over every keep mask


def test_step_uses_pre_update_losses_and_composes(ref):
    r = rng(20)
    n, d, P = 64, 8, 48
    X = r.standard_normal((n, d)).astype(np.float32)
    y = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    F = ref.Features.dense(X)
    w0 = (0.4 * r.standard_normal(d)).astype(np.float32)
    phi0 = (0.4 * r.standard_normal(d)).astype(np.float32)
    idx = r.permutation(n)[:P].astype(np.int32)
    out = ref.step(F, y, idx, P, w0, phi0, 0.05, 0.2, 9, 4, 0.01, 0.3, 0.5, 0.2)
    logit, prob = ref.assistant_score(F, idx, P, phi0, bias=0.05)
    keep, pos = ref.shrink(prob, 0.2, 9, 4)
    assert np.array_equal(out["keep"], keep) and np.array_equal(out["kept_pos"], pos)
    ids = idx[pos]
    assert np.array_equal(out["kept_ids"], ids)
    # losses are the hinge losses at w0 (before the Boss update), by numpy in float64
    marg = y[ids].astype(np.float64) * (X[ids].astype(np.float64) @ w0.astype(np.float64))
    assert np.allclose(out["loss"], np.maximum(0, 1 - marg), rtol=1e-6, atol=1e-7)
    w1, loss = ref.svm_sgd_step(F, y, ids, ids.size, w0, 0.01, 0.3)
    assert np.array_equal(out["w"], w1) and np.array_equal(out["loss"], loss)
    phi1, b1 = ref.assistant_update(F, ids, ids.size, loss, 0.5, phi0, 0.05, 0.2)
    assert np.array_equal(out["phi"], phi1) and out["bias"] == b1


@pytest.mark.parametrize("n", [1, 2, 5, 10, 16])
def test_brute_force_every_keep_mask(ref, n):
    """prob in {0,1} with gamma = 0 forces any mask.  All 2^n masks (n <= 10) or 4096 of them
    (n = 16, every mask for compaction) go through keep/compact/gather/SGD and are compared
    with one-line numpy definitions in float64."""
    r = rng(100 + n)
    d = 3
    X = r.standard_normal((n, d)).astype(np.float32)
    y = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    F = ref.Features.dense(X)
    w0 = (0.5 * r.standard_normal(d)).astype(np.float32)
    idx = r.permutation(n).astype(np.int32)
    Xd, yd, wd = X.astype(np.float64), y.astype(np.float64), w0.astype(np.float64)
    lam, lr = 0.1, 0.5
    masks = np.arange(2 ** n, dtype=np.uint32)
    full_sgd = masks if n <= 10 else masks[:: 16]
    bits = ((masks[:, None] >> np.arange(n, dtype=np.uint32)[None, :]) & 1).astype(np.uint8)
    sgd_set = set(int(v) for v in full_sgd)
    for mask, b in zip(masks, bits):
        keep, pos = ref.shrink(b.astype(np.float32), 0.0, 1, 2)
        assert np.array_equal(keep, b) and np.array_equal(pos, np.flatnonzero(b))
        if int(mask) not in sgd_set:
            continue
        rows_g, ids = ref.gather(X, idx, pos)
        assert np.array_equal(ids, idx[pos]) and np.array_equal(rows_g, X[idx[pos]])
        w1, loss = ref.svm_sgd_step(F, y, ids, ids.size, w0, lam, lr)
        if ids.size == 0:
            assert np.array_equal(w1, w0)
            continue
        marg = yd[ids] * (Xd[ids] @ wd)
        G = ((marg < 1) * yd[ids]) @ Xd[ids]
        want = (1 - lr * lam) * wd + lr / ids.size * G
        assert np.allclose(w1, want, rtol=1e-6, atol=1e-7)
        assert np.allclose(loss, np.maximum(0, 1 - marg), rtol=1e-6, atol=1e-7)


# ---------------------------------------------------------------------------
# Length-bucketed batching (definition is this build's; brute force only)


def test_bucket_batches_brute_force(ref):
    r = rng(21)
    m = 500
    ls = np.clip(r.poisson(27, m), 1, 128).astype(np.int32)
    lt = np.clip(r.poisson(27, m), 1, 128).astype(np.int32)
    order, start, batch_of, nb = ref.bucket_batches(ls, lt, 8, 16, 4096)
    bucket = np.minimum(15, (np.maximum(ls, lt) - 1) // 8)
    assert np.array_equal(np.sort(order), np.arange(m))                   # a permutation
    assert np.all(np.diff(bucket[order]) >= 0)                            # grouped by bucket
    for b in range(16):
        seg = order[start[b]:start[b + 1]]
        assert np.array_equal(seg, np.flatnonzero(bucket == b))            # stable inside a bucket
        cap = max(1, 4096 // (16 * (b + 1)))
        if seg.size:
            rel = batch_of[start[b]:start[b + 1]] - batch_of[start[b]]
            assert np.array_equal(rel, np.arange(seg.size) // cap)
    assert nb == len(np.unique(batch_of)) and batch_of.max() == nb - 1
    # padded-token budget holds for every batch
    for q in range(nb):
        members = order[batch_of == q]
        width = 8 * (bucket[members[0]] + 1)
        assert members.size * 2 * width <= 4096 or members.size == 1


# ---------------------------------------------------------------------------
# Running-median threshold (estimator is this build's; the median itself is numpy's)


def test_threshold_update_is_numpy_median_with_momentum(ref):
    r = rng(22)
    T, init = 0.0, False
    want = None
    for m in [255, 256, 1, 2, 1000]:
        loss = r.gamma(2.0, 0.5, m).astype(np.float32)
        T, init = ref.threshold_update(loss, 0.9, T, init)
        med = np.float32(np.median(loss.astype(np.float64)))      # exact: mean of two floats
        if want is None:
            want = med
        else:
            want = np.float32(np.float32(np.float32(0.9) * want)
                              + np.float32(np.float32(np.float32(1.0) - np.float32(0.9)) * med))
        assert init and np.float32(T) == want
    T2, init2 = ref.threshold_update(np.zeros(0, np.float32), 0.9, 1.25, True)
    assert T2 == 1.25 and init2
    # a NaN loss has no rank: the threshold becomes NaN instead of an arbitrary value
    bad = r.gamma(2.0, 0.5, 300).astype(np.float32)
    bad[17] = np.nan
    T3, init3 = ref.threshold_update(bad, 0.9, 1.25, False)
    assert np.isnan(T3) and init3


def test_threshold_momentum_rule_by_its_closed_form(ref):
    """The momentum half of the running threshold, pinned by what the recursion
    T <- momentum T + (1 - momentum) med implies rather than by repeating it:
      * momentum = 0 returns the batch median itself, momentum = 1 never moves (both exact);
      * a threshold that already equals the median of every batch stays there;
      * for batches that all have the median `med`, T_t = med + momentum^t (T_0 - med): the
        distance to the median shrinks by the factor `momentum` (0.9, not 0.1) per batch.
    Swapping the two weights, dropping one of them or updating towards anything but the
    median breaks at least one of these."""
    r = rng(23)

    def batch_with_median(med, m):
        """m losses (odd m) whose median is exactly med, in random order."""
        half = m // 2
        lo = med - r.gamma(2.0, 0.5, half) - 1e-3
        hi = med + r.gamma(2.0, 0.5, half) + 1e-3
        x = np.concatenate([lo, [med], hi]).astype(np.float32)
        r.shuffle(x)
        assert np.float32(np.median(x.astype(np.float64))) == np.float32(med)
        return x

    # momentum 0 and 1
    loss = r.gamma(2.0, 0.5, 301).astype(np.float32)
    med = np.float32(np.median(loss.astype(np.float64)))
    T, init = ref.threshold_update(loss, 0.0, 5.0, True)
    assert init and np.float32(T) == med
    T, init = ref.threshold_update(loss, 1.0, 5.0, True)
    assert init and np.float32(T) == np.float32(5.0)
    # the first batch sets T whatever the momentum
    T, init = ref.threshold_update(loss, 1.0, 5.0, False)
    assert init and np.float32(T) == med

    # fixed point: T equal to the median of each batch does not move (one rounding per term:
    # 0.9 T + 0.1 T may differ from T by an ulp or two, never by more, and never drifts)
    med = np.float32(1.375)
    T = float(med)
    for t in range(200):
        T, _ = ref.threshold_update(batch_with_median(float(med), 101), 0.9, T, True)
        assert abs(T - float(med)) <= 4 * np.spacing(med)

    # geometric approach to a constant median from above and from below, several momenta
    for momentum in (0.9, 0.5, 0.25):
        for T0 in (4.0, 0.125):
            T = T0
            mom32 = float(np.float32(momentum))
            one_minus32 = float(np.float32(1.0) - np.float32(momentum))
            for t in range(1, 60):
                T, init = ref.threshold_update(batch_with_median(float(med), 51), momentum, T, True)
                # closed form with the fp32-rounded weights (their sum is 1 only up to an ulp)
                want = float(med) + (T0 - float(med)) * mom32 ** t
                # each step rounds three times at magnitude <= max(T0, med): <= 1.5 ulp; the
                # errors are damped by `momentum` per step, so they sum to < 1.5 ulp / (1 - momentum)
                bound = 2.0 * float(np.spacing(np.float32(max(T0, float(med))))) / (1.0 - mom32) \
                    + abs(mom32 + one_minus32 - 1.0) * t * max(T0, float(med))
                assert abs(T - want) <= bound, (momentum, T0, t, T, want, bound)
            # and the direction is towards the median: with the weights swapped the first step
            # alone would land at med + (1 - momentum)(T0 - med)
            T1, _ = ref.threshold_update(batch_with_median(float(med), 51), momentum, T0, True)
            if momentum != 0.5:
                swapped = float(med) + (1.0 - mom32) * (T0 - float(med))
                assert abs(T1 - swapped) > 0.05 * abs(T0 - float(med))


# ---------------------------------------------------------------------------
# Hard-threshold shrinking (SK) and the iteration of Theorem 1


def test_sk_step_against_its_definition(ref):
    """keep = (hinge loss at the current w) > T, written out in numpy; the update is the SVM
    step on exactly those rows; T below every loss is the plain mini-batch step bit for bit;
    T above every loss changes nothing."""
    r = rng(31)
    n, d, P = 300, 12, 200
    X = r.standard_normal((n, d)).astype(np.float32)
    y = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    w = (0.5 * r.standard_normal(d)).astype(np.float32)
    idx = r.permutation(n)[:P].astype(np.int32)
    F = ref.Features.dense(X)
    lam, lr = 1e-2, 0.3
    margins = (y[idx].astype(np.float64) * (X[idx].astype(np.float64) @ w.astype(np.float64))
               ).astype(np.float32)
    losses = np.maximum(0.0, 1.0 - margins.astype(np.float64)).astype(np.float32)
    for T in (0.0, 0.7, 1.5):
        out = ref.sk_step(F, y, idx, P, w, lam, lr, T)
        want_keep = losses > np.float32(T)
        assert 0 < want_keep.sum() < P
        assert np.array_equal(out["keep"].astype(bool), want_keep)
        assert np.array_equal(out["kept_pos"], np.flatnonzero(want_keep))
        assert np.array_equal(out["kept_ids"], idx[want_keep])
        assert np.array_equal(out["loss_pool"], losses)
        assert np.array_equal(out["loss"], losses[want_keep])
        m = int(want_keep.sum())
        # every kept row has a positive loss, hence an active hinge: G = sum of y x over them
        G = (y[idx][want_keep, None].astype(np.float64) * X[idx][want_keep].astype(np.float64)).sum(0)
        want_w = (1 - np.float64(np.float32(lr)) * np.float64(np.float32(lam))) * w.astype(np.float64) \
            + np.float64(np.float32(lr)) / m * G
        assert np.allclose(out["w"], want_w, rtol=1e-6, atol=1e-7)
    everything = ref.sk_step(F, y, idx, P, w, lam, lr, -1.0)
    assert everything["m"] == P
    assert np.array_equal(everything["w"], ref.vanilla_minibatch_sgd(F, y, idx, P, w, lam, lr))
    nothing = ref.sk_step(F, y, idx, P, w, lam, lr, 1e9)
    assert nothing["m"] == 0 and np.array_equal(nothing["w"], w)


def test_sk_step_at_T0_is_the_vanilla_direction_rescaled(ref):
    """With T = 0 the dropped rows are exactly those with zero subgradient, so the data term
    of the step is the plain mini-batch one scaled by P/m."""
    r = rng(32)
    n, d = 400, 10
    X = r.standard_normal((n, d)).astype(np.float32)
    y = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    w = r.standard_normal(d).astype(np.float32)
    F = ref.Features.dense(X)
    lam, lr = 1e-3, 0.2
    sk = ref.sk_step(F, y, None, n, w, lam, lr, 0.0)
    van = ref.vanilla_minibatch_sgd(F, y, None, n, w, lam, lr)
    shrink = 1 - np.float64(np.float32(lr)) * np.float64(np.float32(lam))
    data_sk = sk["w"].astype(np.float64) - shrink * w
    data_van = van.astype(np.float64) - shrink * w
    assert 0 < sk["m"] < n
    assert np.allclose(data_sk * sk["m"], data_van * n, rtol=1e-4, atol=1e-5)


def _svm_optimum(X, y, mu):
    """argmin (mu/2)|w|^2 + mean hinge, as a smooth program in (w, slack) solved by SLSQP."""
    import scipy.optimize as opt
    n, d = X.shape
    X64, y64 = X.astype(np.float64), y.astype(np.float64)

    def obj(v):
        return 0.5 * mu * v[:d] @ v[:d] + v[d:].mean()

    def grad(v):
        return np.concatenate([mu * v[:d], np.full(n, 1.0 / n)])

    A = np.hstack([y64[:, None] * X64, np.eye(n)])          # y x.w + xi >= 1
    cons = [{"type": "ineq", "fun": lambda v: A @ v - 1.0, "jac": lambda v: A}]
    bounds = [(None, None)] * d + [(0, None)] * n
    res = opt.minimize(obj, np.concatenate([np.zeros(d), np.ones(n)]), jac=grad, bounds=bounds,
                       constraints=cons, method="SLSQP", options={"ftol": 1e-14, "maxiter": 500})
    assert res.success
    return res.x[:d]


def _theorem_instance():
    r = rng(33)
    n, d = 16, 4
    X = r.standard_normal((n, d)).astype(np.float32)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    y = np.where(X @ np.array([1.0, -1.0, 0.5, 0.0]) + 0.3 * r.standard_normal(n) > 0, 1.0, -1.0
                 ).astype(np.float32)
    return X, y


def test_theorem_iteration_without_dropping_is_plain_sgd(ref):
    """G = 0 drops nothing: the iterates equal a numpy loop over the same index sequence,
    and that sequence is the second Philox word scaled to the row count."""
    X, y = _theorem_instance()
    n, d = X.shape
    F = ref.Features.dense(X)
    mu, K, seed = 0.5, 200, 9
    w, _, picked, dropped = ref.sk_sgd(F, y, np.zeros(d), mu, 0.0, 0.0, seed, K)
    assert dropped == 0
    want_picked = [(int(ref.philox4x32_10((k, 0, 0, 0), (seed, 0))[1]) * n) >> 32 for k in range(1, K + 1)]
    assert picked.tolist() == want_picked
    assert len(set(want_picked)) == n                        # every row is drawn
    v = np.zeros(d)
    for k, i in enumerate(want_picked, start=1):
        g = mu * v - (y[i] * X[i].astype(np.float64) if y[i] * (X[i].astype(np.float64) @ v) < 1 else 0.0)
        v = v - g / (mu * k)
    assert np.allclose(w, v, rtol=1e-12, atol=1e-14)


def test_theorem_1_bound_holds_on_average(ref):
    """Theorem 1: with step size 1/(mu k) and steps dropped when |grad f_i| <= G/k, the mean of
    |w_k - w*|^2 over many index sequences stays below max(4 D^2, G^2/mu^2 + 4 D G/mu) / k.
    The rule really drops steps here, and the iterates still reach the optimum."""
    X, y = _theorem_instance()
    n, d = X.shape
    F = ref.Features.dense(X)
    mu = 0.5
    w_star = _svm_optimum(X, y, mu)
    # the optimum found by SLSQP satisfies the subgradient optimality condition
    marg = y * (X.astype(np.float64) @ w_star)
    lo = mu * w_star - (y[:, None] * X)[marg < 1 - 1e-7].sum(0) / n
    on = (y[:, None] * X)[np.abs(marg - 1) <= 1e-7]
    resid = lo if len(on) == 0 else lo - on.T @ np.clip(np.linalg.lstsq(on.T, lo, rcond=None)[0], 0, 1.0 / n)
    assert np.linalg.norm(resid) < 1e-6
    D = 1.0 / np.sqrt(mu)                     # Pegasos: the optimum lies in this ball
    assert np.linalg.norm(w_star) <= D
    G = mu * D + 1.0                          # |mu w - y x| <= mu D + |x| on the ball, |x| = 1
    bound = max(4 * D * D, G * G / (mu * mu) + 4 * D * G / mu)
    K, seeds = 2000, 128
    dist2 = np.zeros((seeds, K + 1))
    dropped = np.zeros(seeds, dtype=int)
    for s in range(seeds):
        _, dist2[s], _, dropped[s] = ref.sk_sgd(F, y, np.zeros(d), mu, G, D, 1000 + s, K, w_star)
    mean = dist2.mean(0)
    k = np.arange(1, K + 2)
    assert np.all(mean * k <= bound)
    assert dropped.min() > 0                  # the shrinking rule takes part
    assert mean[-1] < 0.02 * mean[0]          # and the iterates close in on w*
    # without dropping (plain SGD) the same bound holds, and shrinking costs little accuracy
    plain = np.array([ref.sk_sgd(F, y, np.zeros(d), mu, 0.0, D, 1000 + s, K, w_star)[1][-1]
                      for s in range(seeds)])
    assert mean[-1] < 3 * plain.mean() + 1e-3


# ---------------------------------------------------------------------------
# Deterministic stale-Assistant schedule


def _stale_instance():
    r = rng(41)
    n, d = 1000, 16
    X = r.standard_normal((n, d)).astype(np.float32)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    y = np.where(X @ r.standard_normal(d) > 0, 1.0, -1.0).astype(np.float32)
    perm = r.permutation(n).astype(np.int32)
    return X, y, perm


def test_stale_schedule_with_zero_staleness_is_the_synchronous_step(ref):
    X, y, perm = _stale_instance()
    n, d = X.shape
    F = ref.Features.dense(X)
    P, gamma, seed, lam, lr0, T, lr_a = 128, 0.1, 3, 1e-3, 0.5, 0.0, 0.2
    got = ref.train_stale(F, y, perm, P, np.zeros(d), np.zeros(d), 0.0, gamma, seed, 10, lam, lr0,
                          T, lr_a, staleness=0)
    w, phi, b, t_upd = np.zeros(d, np.float32), np.zeros(d, np.float32), 0.0, 0
    for s in range((n + P - 1) // P):
        idx = perm[s * P:(s + 1) * P]
        lr = np.float32(np.float32(lr0) / np.sqrt(np.float32(t_upd + 1)))
        out = ref.step(F, y, idx, idx.size, w, phi, b, gamma, seed, 10 + s, lam, lr, T, lr_a)
        w, phi, b = out["w"], out["phi"], out["bias"]
        t_upd += out["m"] > 0
        assert out["m"] == got["m"][s] and np.array_equal(out["kept_ids"], got["kept_ids"][s])
    assert np.array_equal(got["w"], w) and np.array_equal(got["phi"], phi) and got["bias"] == b


def test_stale_schedule_uses_the_assistant_of_k_ticks_ago(ref):
    """Batch s is drawn with the Assistant as it stood after s - k updates: with k beyond the
    number of pools every batch comes from the initial Assistant; with k = 1 the first two
    batches do, and the third from the Assistant after exactly one update."""
    X, y, perm = _stale_instance()
    n, d = X.shape
    F = ref.Features.dense(X)
    P, gamma, seed, lam, lr0, T, lr_a = 128, 0.0, 3, 1e-3, 0.5, 0.5, 2.0
    phi0 = (0.5 * rng(42).standard_normal(d)).astype(np.float32)
    S = (n + P - 1) // P

    def batch(s, phi, b):
        idx = perm[s * P:(s + 1) * P]
        _, prob = ref.assistant_score(F, idx, idx.size, phi, b)
        _, pos = ref.shrink(prob, gamma, seed, s)
        return idx[pos]

    far = ref.train_stale(F, y, perm, P, np.zeros(d), phi0, 0.1, gamma, seed, 0, lam, lr0, T, lr_a,
                          staleness=S + 5)
    for s in range(S):
        assert np.array_equal(far["kept_ids"][s], batch(s, phi0, 0.1))
    one = ref.train_stale(F, y, perm, P, np.zeros(d), phi0, 0.1, gamma, seed, 0, lam, lr0, T, lr_a,
                          staleness=1)
    sync = ref.train_stale(F, y, perm, P, np.zeros(d), phi0, 0.1, gamma, seed, 0, lam, lr0, T, lr_a,
                           staleness=0)
    assert np.array_equal(one["kept_ids"][0], batch(0, phi0, 0.1))
    assert np.array_equal(one["kept_ids"][1], batch(1, phi0, 0.1))
    # tick 0 by hand: Boss step on batch 0, then the Assistant update at phi0
    ids0 = batch(0, phi0, 0.1)
    w1, loss0 = ref.svm_sgd_step(F, y, ids0, ids0.size, np.zeros(d, np.float32), lam, np.float32(lr0))
    phi1, b1 = ref.assistant_update(F, ids0, ids0.size, loss0, T, phi0, 0.1, lr_a)
    assert np.array_equal(one["kept_ids"][2], batch(2, phi1, b1))
    assert np.array_equal(sync["kept_ids"][1], batch(1, phi1, b1))
    # the schedules really differ on this instance
    assert not np.array_equal(one["kept_ids"][1], sync["kept_ids"][1])
