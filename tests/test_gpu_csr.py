"""GPU parity of the CSR path (sparse linear-SVM and token-list shapes) against the oracle."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch

from paper_1905_03381_amd import api, synth

from gpu_util import (RTOL, abs_dot_scale, assert_close_scaled, assert_logit_prob, clear_draws,
                      csr_features, dev, host, scalar_dev)

pytestmark = pytest.mark.gpu


def rng(seed):
    return np.random.default_rng(seed)


@pytest.fixture(scope="module")
def sparse():
    """Down-scaled sparse config: 30,000 rows, d = 2^16, about 100 entries per row."""
    rowptr, col, val, y, _ = synth.sparse_svm(n=30_000, d=1 << 16, mean_nnz=100, threads=4)
    return rowptr, col, val, y, 1 << 16


@pytest.fixture(scope="module")
def ws():
    return api.Workspace(1 << 16, 1 << 16)


def test_csr_score_and_fused_keep(ref, ws, sparse):
    rowptr, col, val, y, d = sparse
    n = rowptr.size - 1
    P = 20_000
    r = rng(1)
    phi = (3.0 * r.standard_normal(d)).astype(np.float32)
    idx = r.permutation(n)[:P].astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    ref_logit, ref_prob = ref.assistant_score(Fh, idx, P, phi, bias=0.3)
    S = abs_dot_scale(Fh, idx, phi)
    logit, prob = torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
    api.assistant_score(F, dev(idx), P, dev(phi), scalar_dev(0.3), logit, prob)
    assert_logit_prob(host(logit), host(prob), ref_logit, ref_prob, S, bias=0.3)
    gamma, seed, step = 0.1, 3, 8
    keep_ref, _ = ref.shrink(ref_prob, gamma, seed, step)
    keep = torch.zeros(P, dtype=torch.uint8, device="cuda")
    pos = torch.full((P,), -1, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.score_shrink(F, dev(idx), P, dev(phi), scalar_dev(0.3), gamma, seed, step, None, prob, keep,
                     pos, cnt, ws)
    k = host(keep)
    clear = clear_draws(ref, ref_prob, gamma, seed, step)
    assert np.array_equal(k[clear], keep_ref[clear])
    m = int(host(cnt)[0])
    assert m == int(k.sum()) and np.array_equal(host(pos)[:m], np.flatnonzero(k))


@pytest.mark.parametrize("ones", [False, True])
@pytest.mark.parametrize("indexed", [True, False])
def test_csr_score_large_pool_equals_small_pools(ref, ws, ones, indexed):
    """Pools of 16,384 rows and more over 16,385 to 79,872 columns are scored by the kernel that
    keeps the head of phi in LDS, smaller ones by the general kernel: both add a row's terms in
    the same order, so one pool of 25,001 rows and the same rows in pools of 9000 give the same
    bits -- and the oracle's values.  Rows of 0 to 260 entries: half of them exceed the 128
    entries of the first kernel's main loop and take its separate walk; a fifth of the
    columns lie past its table."""
    n, d, P = 30_000, 50_000, 25_001
    r = rng(41)
    lens = r.integers(0, 261, size=n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=rowptr[1:])
    col = r.integers(0, d, size=int(rowptr[-1])).astype(np.int32)
    val = (r.standard_normal(col.size) / 10.0).astype(np.float32)
    phi = r.standard_normal(d).astype(np.float32)
    idx = r.permutation(n)[:P].astype(np.int32) if indexed else None
    Fh = ref.Features.csr(rowptr, col, None if ones else val, d)
    F = csr_features(rowptr, col, None if ones else val, d)
    lens = lens[idx if indexed else slice(0, P)]
    assert (lens > 128).mean() > 0.3 and (lens <= 128).mean() > 0.3 and (lens == 0).sum() > 10
    bias, gamma, seed, step = scalar_dev(-0.4), 0.2, 11, 6
    logit, prob = torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
    api.assistant_score(F, None if idx is None else dev(idx), P, dev(phi), bias, logit, prob)
    ids = idx if indexed else np.arange(P, dtype=np.int32)
    ref_logit, ref_prob = ref.assistant_score(Fh, ids, P, phi, bias=-0.4)
    assert_logit_prob(host(logit), host(prob), ref_logit, ref_prob, abs_dot_scale(Fh, ids, phi), bias=-0.4)
    logit2, prob2 = torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
    for lo in range(0, P, 9000):
        m = min(9000, P - lo)
        api.assistant_score(F, dev(ids[lo:lo + m]), m, dev(phi), bias, logit2[lo:], prob2[lo:])
    assert np.array_equal(host(logit), host(logit2)) and np.array_equal(host(prob), host(prob2))
    # keep flags of the fused score + keep + compact call: same draws, same probabilities
    keep = torch.zeros(P, dtype=torch.uint8, device="cuda")
    pos = torch.full((P,), -1, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    prob3 = torch.zeros(P, device="cuda")
    api.score_shrink(F, None if idx is None else dev(idx), P, dev(phi), bias, gamma, seed, step, None,
                     prob3, keep, pos, cnt, ws)
    assert np.array_equal(host(prob3), host(prob))
    keep_ref, _ = ref.shrink(ref_prob, gamma, seed, step)
    clear = clear_draws(ref, ref_prob, gamma, seed, step)
    k = host(keep)
    assert np.array_equal(k[clear], keep_ref[clear])
    m = int(host(cnt)[0])
    assert m == int(k.sum()) and np.array_equal(host(pos)[:m], np.flatnonzero(k))


def test_csr_all_ones_values(ref, ws):
    """Token lists: val == NULL means every entry is 1; repeated tokens add."""
    rowptr, col, val, len_s, len_t, d = synth.sentence_pairs(n=5000, vocab=2000)
    r = rng(2)
    phi = (0.2 * r.standard_normal(d)).astype(np.float32)
    Fh = ref.Features.csr(rowptr, col, None, d)
    F = csr_features(rowptr, col, None, d)
    P = 5000
    ref_logit, ref_prob = ref.assistant_score(Fh, None, P, phi)
    logit, prob = torch.zeros(P, device="cuda"), torch.zeros(P, device="cuda")
    api.assistant_score(F, None, P, dev(phi), None, logit, prob)
    assert_logit_prob(host(logit), host(prob), ref_logit, ref_prob, abs_dot_scale(Fh, np.arange(P), phi))
    # with the length features as values
    Fh2 = ref.Features.csr(rowptr, col, val, d)
    F2 = csr_features(rowptr, col, val, d)
    ref_logit, ref_prob = ref.assistant_score(Fh2, None, P, phi, bias=-0.5)
    api.assistant_score(F2, None, P, dev(phi), scalar_dev(-0.5), logit, prob)
    assert_logit_prob(host(logit), host(prob), ref_logit, ref_prob,
                      abs_dot_scale(Fh2, np.arange(P), phi), bias=-0.5)


def _dots(Fh, ids, v):
    """x_r . v for the listed CSR rows, float64, by scipy."""
    S = sp.csr_matrix((Fh.val.astype(np.float64), Fh.col, Fh.rowptr), shape=(Fh.n, Fh.d))
    return S[np.asarray(ids)] @ v.astype(np.float64)


def _col_abs_sum(Fh, ids, d):
    out = np.zeros(d)
    for i in ids:
        lo, hi = Fh.rowptr[i], Fh.rowptr[i + 1]
        v = np.ones(hi - lo) if Fh.val is None else np.abs(Fh.val[lo:hi].astype(np.float64))
        np.add.at(out, Fh.col[lo:hi], v)
    return out


def test_csr_svm_step_and_assistant_update(ref, ws, sparse):
    rowptr, col, val, y, d = sparse
    n = rowptr.size - 1
    m = 3000
    r = rng(3)
    w0 = (2.0 * r.standard_normal(d)).astype(np.float32)
    phi0 = r.standard_normal(d).astype(np.float32)
    rows = r.permutation(n)[:m].astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    lam, lr, T, lr_a, b0 = 1e-3, 0.5, 0.3, 0.2, 0.1
    w_ref, loss_ref = ref.svm_sgd_step(Fh, y, rows, m, w0, lam, lr)
    S = abs_dot_scale(Fh, rows, w0)
    dots = _dots(Fh, rows, w0) * y[rows]
    assert np.all(np.abs(dots - 1) > RTOL * S)
    w = dev(w0)
    loss = torch.zeros(m, device="cuda")
    api.svm_sgd_step(F, dev(y), dev(rows), scalar_dev(m, torch.int32), m, w, lam, lr, 0.0, loss, ws)
    assert_close_scaled(host(loss), loss_ref, S, "loss")
    absx = _col_abs_sum(Fh, rows[dots < 1], d)
    assert_close_scaled(host(w), w_ref, np.abs(w0.astype(np.float64)) + lr / m * absx, "w")
    phi_ref, b_ref = ref.assistant_update(Fh, rows, m, loss_ref, T, phi0, b0, lr_a)
    phi, b = dev(phi0), scalar_dev(b0)
    api.assistant_update(F, dev(rows), scalar_dev(m, torch.int32), m, dev(loss_ref), scalar_dev(T),
                         phi, b, lr_a, 0.0, ws)
    absx = _col_abs_sum(Fh, rows, d)
    assert_close_scaled(host(phi), phi_ref, np.abs(phi0.astype(np.float64)) + lr_a / m * absx, "phi")
    assert abs(float(host(b)[0]) - b_ref) <= RTOL * (abs(b0) + lr_a)
    # m = 0 leaves everything alone
    w = dev(w0)
    api.svm_sgd_step(F, dev(y), dev(rows), scalar_dev(0, torch.int32), m, w, lam, lr, 0.0, None, ws)
    assert np.array_equal(host(w), w0)


def test_csr_fused_step(ref, ws, sparse):
    rowptr, col, val, y, d = sparse
    n = rowptr.size - 1
    P = 8000
    r = rng(4)
    w0 = (2.0 * r.standard_normal(d)).astype(np.float32)
    phi0 = (2.0 * r.standard_normal(d)).astype(np.float32)
    idx = r.permutation(n)[:P].astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    b0, gamma, step, lam, lr, T, lr_a = 0.0, 0.1, 3, 1e-3, 0.5, 0.1, 0.3
    for seed in range(1, 20):   # first Philox key with no draw inside the rounding band
        out = ref.step(Fh, y, idx, P, w0, phi0, b0, gamma, seed, step, lam, lr, T, lr_a)
        if clear_draws(ref, out["prob"], gamma, seed, step).all():
            break
    else:
        raise AssertionError("no clear seed")
    kept = out["kept_ids"]
    dots = _dots(Fh, kept, w0) * y[kept]
    # rows whose margin sits within rounding of the hinge kink may fall on either side
    on_kink = np.abs(dots - 1) <= RTOL * abs_dot_scale(Fh, kept, w0)
    assert on_kink.sum() <= 3
    w, phi, b = dev(w0), dev(phi0), scalar_dev(b0)
    Tt = scalar_dev(T)
    cfg = api.step_config(gamma, lam, lr, lr_a, 0.0, seed, step, Tt)
    prob = torch.zeros(P, device="cuda")
    keep = torch.zeros(P, dtype=torch.uint8, device="cuda")
    pos = torch.zeros(P, dtype=torch.int32, device="cuda")
    ids = torch.zeros(P, dtype=torch.int32, device="cuda")
    loss = torch.zeros(P, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.fused_step(F, dev(y), dev(idx), P, w, phi, b, cfg, None, prob, keep, pos, ids, loss, cnt, ws)
    m = out["m"]
    assert int(host(cnt)[0]) == m
    assert np.array_equal(host(keep), out["keep"])
    assert np.array_equal(host(pos)[:m], out["kept_pos"])
    assert np.array_equal(host(ids)[:m], out["kept_ids"])
    assert_close_scaled(host(loss)[:m], out["loss"], abs_dot_scale(Fh, kept, w0), "loss")
    absx_a = _col_abs_sum(Fh, kept[dots < 1], d)
    assert_close_scaled(host(w), out["w"], np.abs(w0.astype(np.float64)) + lr / m * absx_a, "w",
                        atol=lr / m * _col_abs_sum(Fh, kept[on_kink], d))
    absx = _col_abs_sum(Fh, kept, d)
    assert_close_scaled(host(phi), out["phi"], np.abs(phi0.astype(np.float64)) + lr_a / m * absx,
                        "phi")


def _bits(t):
    return host(t).view(np.uint32).copy()


def test_csr_fused_steps_repeat_bit_for_bit(ws, sparse):
    """Five chained whole steps on the sparse shape, run four times from the same state: model,
    bias and losses come out with the same bits every time.  (Entries of a column reach its
    total by three routes -- the block's table, a hashed slot, a record -- and which route an
    entry takes depends on timing; every route adds in doubles and rounds once.)"""
    rowptr, col, val, y, d = sparse
    n, P, steps = rowptr.size - 1, 6000, 5
    r = rng(31)
    w0 = r.standard_normal(d).astype(np.float32)
    phi0 = r.standard_normal(d).astype(np.float32)
    perm = dev(r.permutation(n)[:steps * P].astype(np.int32))
    F = csr_features(rowptr, col, val, d)
    yd, Tt = dev(y), scalar_dev(0.3)
    cfg = api.step_config(0.1, 1e-3, 0.5, 0.3, 0.0, 5, 0, Tt)

    def run():
        w, phi, b = dev(w0), dev(phi0), scalar_dev(0.1)
        hist = torch.zeros(steps, dtype=torch.int32, device="cuda")
        loss = torch.full((steps, P), -3.0, device="cuda")
        api.train_epoch(F, yd, perm, steps * P, P, w, phi, b, cfg, None, hist, ws, None, loss)
        return _bits(w), _bits(phi), _bits(b), _bits(loss), host(hist).tolist()

    first = run()
    assert min(first[4]) > 500 and not np.array_equal(first[0], w0.view(np.uint32))
    for _ in range(3):
        again = run()
        assert again[4] == first[4]
        for name, x0, x1 in zip(("w", "phi", "bias", "losses"), first, again):
            assert np.array_equal(x0, x1), f"{name} differs between two runs of the same steps"


def test_gather_csr(ref, ws, sparse):
    rowptr, col, val, y, d = sparse
    n = rowptr.size - 1
    P = 5000
    r = rng(5)
    idx = r.permutation(n)[:P].astype(np.int32)
    kept_pos = np.sort(r.choice(P, 2100, replace=False)).astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    cap = int(np.diff(rowptr)[idx[kept_pos]].sum())
    want_ptr, want_col, want_val = ref.gather_csr(Fh, idx, kept_pos, cap)
    out_ptr = torch.full((P + 1,), -1, dtype=torch.int64, device="cuda")
    out_col = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    out_val = torch.full((cap,), -1.0, device="cuda")
    pos_d = torch.zeros(P, dtype=torch.int32, device="cuda")
    pos_d[:2100] = dev(kept_pos)
    api.gather_csr(F, dev(idx), pos_d, scalar_dev(2100, torch.int32), P, out_ptr, out_col, out_val,
                   cap, ws)
    assert np.array_equal(host(out_ptr)[:2101], want_ptr)
    assert np.array_equal(host(out_col), want_col) and np.array_equal(host(out_val), want_val)
    # capacity too small: row pointers complete, rows past the capacity not copied
    small = cap // 2
    out_col2 = torch.full((small,), -1, dtype=torch.int32, device="cuda")
    out_val2 = torch.full((small,), -1.0, device="cuda")
    api.gather_csr(F, dev(idx), pos_d, scalar_dev(2100, torch.int32), P, out_ptr, out_col2, out_val2,
                   small, ws)
    ptr = host(out_ptr)[:2101]
    assert np.array_equal(ptr, want_ptr) and ptr[-1] > small
    fits = int(np.searchsorted(want_ptr, small, side="right") - 1)
    assert np.array_equal(host(out_col2)[:want_ptr[fits]], want_col[:want_ptr[fits]])
    assert np.all(host(out_col2)[want_ptr[fits]:] == -1)
    # one entry short: only the last kept row stays out, nothing is written past the capacity
    # (the buffers hold one guard entry behind it)
    out_col3 = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    out_val3 = torch.full((cap,), -1.0, device="cuda")
    api.gather_csr(F, dev(idx), pos_d, scalar_dev(2100, torch.int32), P, out_ptr, out_col3, out_val3,
                   cap - 1, ws)
    assert np.array_equal(host(out_ptr)[:2101], want_ptr)
    last = want_ptr[2099]
    assert np.array_equal(host(out_col3)[:last], want_col[:last])
    assert np.array_equal(host(out_val3)[:last], want_val[:last])
    assert np.all(host(out_col3)[last:] == -1) and np.all(host(out_val3)[last:] == -1.0)


def test_sparse_config_full_size_first_pools(ref):
    """The sparse linear-SVM configuration at full size (n = 2,000,000, d = 2^20, about 100
    entries per row, pools of 65,536): two chained whole steps against the oracle."""
    n, d, P = 2_000_000, 1 << 20, 65536
    rowptr, col, val, y, _ = synth.sparse_svm(n=n, d=d, threads=16)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    ws = api.Workspace(P, d)
    perm = synth.epoch_permutation(n, seed=7, epoch=0)
    gamma, seed, lam, lr_a, T = 0.1, 42, 1e-4, 0.1, 0.0
    w_r, phi_r, b_r = np.zeros(d, np.float32), np.zeros(d, np.float32), 0.0
    w, phi, b = dev(w_r), dev(phi_r), scalar_dev(0.0)
    yd, Tt = dev(y), scalar_dev(T)
    for t in range(2):
        idx = perm[t * P:(t + 1) * P]
        lr = float(np.float32(1.0 / np.sqrt(t + 1)))
        w_prev, phi_prev, b_prev = w_r, phi_r, b_r
        # the scores do not depend on the Philox key: take the first key under which no draw of
        # this pool falls into the rounding band of its keep probability
        for seed in range(42, 74):
            out = ref.step(Fh, y, idx, P, w_r, phi_r, b_r, gamma, seed, t, lam, lr, T, lr_a)
            if clear_draws(ref, out["prob"], gamma, seed, t).all():
                break
        else:
            pytest.fail("no Philox key with every draw clear of the rounding band")
        w_r, phi_r, b_r = out["w"], out["phi"], out["bias"]
        m = out["m"]
        cfg = api.step_config(gamma, lam, lr, lr_a, 0.0, seed, t, Tt)
        prob = torch.zeros(P, device="cuda")
        keep = torch.zeros(P, dtype=torch.uint8, device="cuda")
        pos = torch.zeros(P, dtype=torch.int32, device="cuda")
        ids = torch.zeros(P, dtype=torch.int32, device="cuda")
        loss = torch.zeros(P, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        api.fused_step(F, yd, dev(idx), P, w, phi, b, cfg, None, prob, keep, pos, ids, loss, cnt, ws)
        assert int(host(cnt)[0]) == m
        assert np.array_equal(host(keep), out["keep"])
        assert np.array_equal(host(ids)[:m], out["kept_ids"])
        kept = out["kept_ids"]
        S = abs_dot_scale(Fh, kept, w_prev) + 1e-3
        assert_close_scaled(host(loss)[:m], out["loss"], S, f"loss step {t}")
        dots = _dots(Fh, kept, w_prev) * y[kept]
        on_kink = np.abs(dots - 1) <= RTOL * S
        absx_a = _col_abs_sum(Fh, kept[dots < 1], d)
        assert_close_scaled(host(w), w_r, np.abs(w_prev.astype(np.float64)) + lr / m * absx_a,
                            f"w step {t}", atol=lr / m * _col_abs_sum(Fh, kept[on_kink], d))
        absx = _col_abs_sum(Fh, kept, d)
        assert_close_scaled(host(phi), phi_r, np.abs(phi_prev.astype(np.float64)) + lr_a / m * absx,
                            f"phi step {t}")
        # the same step twice more from the same state: the same bits
        got = (host(w).copy(), host(phi).copy(), host(b).copy())
        for _ in range(2):
            w, phi, b = dev(w_prev), dev(phi_prev), scalar_dev(b_prev)
            api.fused_step(F, yd, dev(idx), P, w, phi, b, cfg, None, prob, keep, pos, ids, loss, cnt, ws)
            assert np.array_equal(host(w), got[0]) and np.array_equal(host(phi), got[1])
            assert np.array_equal(host(b), got[2])
        # the GPU state goes on from the oracle's bits so that step 2 is compared on equal inputs
        w, phi, b = dev(w_r), dev(phi_r), scalar_dev(b_r)


def test_train_epoch_on_csr_rows(ref, ws, sparse):
    """aa_train_epoch over CSR rows (general kernels) with the step-size schedule on the device:
    every step against the oracle step from the GPU's previous state at the single-step
    tolerances, then the epoch in one call bit for bit (tests/stepwise.py) -- and again, twice:
    the gradient sums do not depend on the order in which waves and blocks arrive."""
    from stepwise import check_epoch, run_whole
    rowptr, col, val, y, d = sparse
    n, P = 9000, 2048
    perm = rng(21).permutation(rowptr.size - 1)[:n].astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    zeros = np.zeros(d, np.float32)
    args = dict(gamma=0.1, seed=42, step0=3, lam=1e-4, lr0=2.0, lr_a=0.3, T=0.0, ws=ws)
    counts, state = check_epoch(ref, Fh, F, y, perm, n, P, zeros, zeros, 0.0, **args)
    assert len(counts) == 5 and all(0 < m < P for m in counts) and state[3] == 5
    for _ in range(2):
        hist, _, _, again = run_whole(F, y, perm, n, P, zeros, zeros, 0.0, **args)
        assert hist == counts and again[3] == state[3]
        assert np.array_equal(again[0], state[0]) and np.array_equal(again[1], state[1])
        assert np.array_equal(again[2], state[2])
    # a constant step size (no counter) is still there
    w, phi, b = dev(zeros), dev(zeros), scalar_dev(0.0)
    Tt = scalar_dev(0.0)
    cfg = api.step_config(0.1, 1e-4, 0.5, 0.3, 0.0, 42, 3, Tt)
    hist = torch.full((5,), -1, dtype=torch.int32, device="cuda")
    api.train_epoch(F, dev(y), dev(perm), n, P, w, phi, b, cfg, None, hist, ws)
    assert host(hist).tolist()[0] == counts[0] and np.abs(host(w)).max() > 0


def _uniform_csr(r, n, d, nnz_lo, nnz_hi):
    """Rows whose columns are uniform over all of d (no hot columns), unit L2 norm."""
    lens = r.integers(nnz_lo, nnz_hi + 1, size=n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=rowptr[1:])
    col = r.integers(0, d, size=int(rowptr[-1])).astype(np.int32)
    val = r.standard_normal(col.size).astype(np.float32)
    norm = np.sqrt(np.add.reduceat(val.astype(np.float64) ** 2, rowptr[:-1]))
    val = (val / np.repeat(norm, lens)).astype(np.float32)
    return rowptr, col, val


def _col_abs_sum_sp(Fh, ids, d):
    S = sp.csr_matrix((np.abs(Fh.val.astype(np.float64)), Fh.col, Fh.rowptr), shape=(Fh.n, d))
    return np.asarray(S[np.asarray(ids)].sum(axis=0)).ravel()


@pytest.mark.parametrize("n,nnz_lo,nnz_hi", [(300_000, 8, 16), (3000, 500, 700)])
def test_csr_updates_uniform_columns(ref, n, nnz_lo, nnz_hi):
    """Columns uniform over d = 2^18: nearly every entry falls outside the per-block table.
    300,000 short rows: every block makes two rounds and empties its entry buffer many times.
    3000 rows of about 600 entries: the entries of four rows per wave overflow the buffer, and
    the bins (48 records per candidate) overflow too, so the excess goes to the accumulators."""
    r = rng(21)
    d, m = 1 << 18, n
    rowptr, col, val = _uniform_csr(r, n, d, nnz_lo, nnz_hi)
    y = np.where(r.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    w0 = (2.0 * r.standard_normal(d)).astype(np.float32)
    phi0 = r.standard_normal(d).astype(np.float32)
    rows = r.permutation(n)[:m].astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    ws = api.Workspace(m, d)
    lam, lr, T, lr_a, b0 = 1e-3, 50.0, 0.8, 40.0, 0.1
    w_ref, loss_ref = ref.svm_sgd_step(Fh, y, rows, m, w0, lam, lr)
    S = abs_dot_scale(Fh, rows, w0)
    dots = _dots(Fh, rows, w0) * y[rows]
    on_kink = np.abs(dots - 1) <= RTOL * S
    assert on_kink.sum() <= 20
    w = dev(w0)
    loss = torch.zeros(m, device="cuda")
    api.svm_sgd_step(F, dev(y), dev(rows), scalar_dev(m, torch.int32), m, w, lam, lr, 0.0, loss, ws)
    assert_close_scaled(host(loss), loss_ref, S, "loss")
    absx = _col_abs_sum_sp(Fh, rows[dots < 1], d)
    assert_close_scaled(host(w), w_ref, np.abs(w0.astype(np.float64)) + lr / m * absx, "w",
                        atol=lr / m * _col_abs_sum_sp(Fh, rows[on_kink], d))
    assert np.abs(w_ref - w0).max() > 1e-3  # the step is visible at the tolerance
    w_bits = host(w).copy()
    for _ in range(2):   # (accumulators included: the same bits on every run)
        w = dev(w0)
        api.svm_sgd_step(F, dev(y), dev(rows), scalar_dev(m, torch.int32), m, w, lam, lr, 0.0, loss, ws)
        assert np.array_equal(host(w), w_bits)
    phi_ref, b_ref = ref.assistant_update(Fh, rows, m, loss_ref, T, phi0, b0, lr_a)
    phi, b = dev(phi0), scalar_dev(b0)
    api.assistant_update(F, dev(rows), scalar_dev(m, torch.int32), m, dev(loss_ref), scalar_dev(T),
                         phi, b, lr_a, 0.0, ws)
    absx = _col_abs_sum_sp(Fh, rows, d)
    assert_close_scaled(host(phi), phi_ref, np.abs(phi0.astype(np.float64)) + lr_a / m * absx, "phi")
    assert np.abs(phi_ref - phi0).max() > 2e-4  # 20 times the tolerance
    assert abs(float(host(b)[0]) - b_ref) <= RTOL * (abs(b0) + lr_a)


def test_train_epoch_with_overflowing_bins(ref):
    """aa_train_epoch over rows of about 600 entries with columns uniform over d = 2^18: in every
    step the record buffer and the bins overflow into the accumulators.  One step per call
    (each call prepares the workspace itself) is held to the oracle step at the single-step
    tolerances; then the epoch in one call, where from the second step on no launch prepares
    the workspace -- the update kernel of the step before has cleared what it read and has
    written the model pairs -- must give the same bits: a count or an accumulator left over, or
    a stale pair, would show.  Twice."""
    from stepwise import check_epoch, run_whole
    r = rng(33)
    n, d, P = 3000, 1 << 18, 1000
    rowptr, col, val = _uniform_csr(r, n, d, 500, 700)
    y = np.where(r.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    perm = r.permutation(n).astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    ws = api.Workspace(P, d)
    w0 = (0.5 * r.standard_normal(d)).astype(np.float32)
    phi0 = (0.5 * r.standard_normal(d)).astype(np.float32)
    args = dict(gamma=0.3, seed=7, step0=0, lam=1e-3, lr0=20.0, lr_a=10.0, T=0.5, ws=ws)
    counts, state = check_epoch(ref, Fh, F, y, perm, n, P, w0, phi0, 0.1, **args)
    assert len(counts) == 3 and all(P // 4 < m <= P for m in counts)
    for _ in range(2):
        hist, _, _, again = run_whole(F, y, perm, n, P, w0, phi0, 0.1, **args)
        assert hist == counts
        assert np.array_equal(again[0], state[0]) and np.array_equal(again[1], state[1])
        assert np.array_equal(again[2], state[2])


def test_csr_fused_step_more_columns_than_the_bins_cover(ref):
    """d = 1,300,000 with both vectors updated: too many columns for the column bins, so every
    entry outside the per-block table goes to the dense accumulators."""
    r = rng(22)
    n, d, P = 6000, 1_300_000, 5000
    rowptr, col, val = _uniform_csr(r, n, d, 20, 40)
    y = np.where(r.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    w0 = (2.0 * r.standard_normal(d)).astype(np.float32)
    phi0 = (2.0 * r.standard_normal(d)).astype(np.float32)
    idx = r.permutation(n)[:P].astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    ws = api.Workspace(P, d)
    b0, gamma, step, lam, lr, T, lr_a = 0.0, 0.1, 3, 1e-3, 0.5, 0.1, 0.3
    for seed in range(1, 20):
        out = ref.step(Fh, y, idx, P, w0, phi0, b0, gamma, seed, step, lam, lr, T, lr_a)
        if clear_draws(ref, out["prob"], gamma, seed, step).all():
            break
    else:
        raise AssertionError("no clear seed")
    kept = out["kept_ids"]
    dots = _dots(Fh, kept, w0) * y[kept]
    on_kink = np.abs(dots - 1) <= RTOL * abs_dot_scale(Fh, kept, w0)
    assert on_kink.sum() <= 3
    w, phi, b = dev(w0), dev(phi0), scalar_dev(b0)
    Tt = scalar_dev(T)
    cfg = api.step_config(gamma, lam, lr, lr_a, 0.0, seed, step, Tt)
    prob = torch.zeros(P, device="cuda")
    keep = torch.zeros(P, dtype=torch.uint8, device="cuda")
    pos = torch.zeros(P, dtype=torch.int32, device="cuda")
    ids = torch.zeros(P, dtype=torch.int32, device="cuda")
    loss = torch.zeros(P, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.fused_step(F, dev(y), dev(idx), P, w, phi, b, cfg, None, prob, keep, pos, ids, loss, cnt, ws)
    m = out["m"]
    assert int(host(cnt)[0]) == m
    assert np.array_equal(host(keep), out["keep"])
    assert np.array_equal(host(ids)[:m], out["kept_ids"])
    absx_a = _col_abs_sum_sp(Fh, kept[dots < 1], d)
    assert_close_scaled(host(w), out["w"], np.abs(w0.astype(np.float64)) + lr / m * absx_a, "w",
                        atol=lr / m * _col_abs_sum_sp(Fh, kept[on_kink], d))
    absx = _col_abs_sum_sp(Fh, kept, d)
    assert_close_scaled(host(phi), out["phi"], np.abs(phi0.astype(np.float64)) + lr_a / m * absx,
                        "phi")


def _check_csr_updates(ref, r, d, n, kind, lo, hi, with_val, misalign=False):
    """Boss step, Assistant update and both in one pass on random CSR rows of `lo` to `hi`
    entries against the oracle (columns uniform, Zipf-like or hot at the end of the range).
    misalign: the model vectors start 4 bytes past a 16-byte boundary."""
    def model(a):  # device copy of a model vector
        if not misalign:
            return dev(a)
        t = dev(np.concatenate([np.zeros(1, np.float32), a]))[1:]
        assert t.data_ptr() % 16 == 4
        return t
    lens = r.integers(lo, hi + 1, size=n)
    if r.random() < 0.2 and n > 1:
        lens[r.integers(1, n, size=max(1, n // 10))] = 0  # empty rows
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lens, out=rowptr[1:])
    nnz = int(rowptr[-1])
    if kind == "uniform":
        col = r.integers(0, d, size=nnz)
    elif kind == "zipf":
        col = np.minimum(r.pareto(1.1, size=nnz).astype(np.int64), d - 1)
    else:  # a few very hot columns at the end of the range
        col = np.where(r.random(nnz) < 0.5, d - 1 - r.integers(0, min(3, d), size=nnz),
                       r.integers(0, d, size=nnz))
    col = col.astype(np.int32)
    val = r.standard_normal(nnz).astype(np.float32) if with_val else None
    y = np.where(r.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    w0 = (0.3 * r.standard_normal(d)).astype(np.float32)
    phi0 = (0.3 * r.standard_normal(d)).astype(np.float32)
    m = int(r.integers(1, n + 1))
    rows = r.permutation(n)[:m].astype(np.int32)
    tag = f"d={d} n={n} m={m} nnz={nnz} {kind}"
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    ws = api.Workspace(m, d)
    vv = np.ones(nnz) if val is None else val.astype(np.float64)
    S = sp.csr_matrix((vv, col, rowptr), shape=(n, d))
    Sa = sp.csr_matrix((np.abs(vv), col, rowptr), shape=(n, d))
    lam, lr, T, lr_a, b0 = 1e-3, 0.7, 0.4, 0.5, 0.1
    w_ref, loss_ref = ref.svm_sgd_step(Fh, y, rows, m, w0, lam, lr)
    dots = (S[rows] @ w0.astype(np.float64)) * y[rows]
    Sdot = Sa[rows] @ np.abs(w0.astype(np.float64))
    kink = np.abs(dots - 1) <= RTOL * Sdot
    w = model(w0)
    loss = torch.zeros(m, device="cuda")
    api.svm_sgd_step(F, dev(y), dev(rows), scalar_dev(m, torch.int32), m, w, lam, lr, 0.0, loss, ws)
    assert_close_scaled(host(loss), loss_ref, Sdot, "loss " + tag, atol=1e-6)
    absx_w = np.asarray(Sa[rows[dots < 1]].sum(axis=0)).ravel()
    akink = np.asarray(Sa[rows[kink]].sum(axis=0)).ravel()
    assert_close_scaled(host(w), w_ref, np.abs(w0.astype(np.float64)) + lr / m * absx_w, "w " + tag,
                        atol=lr / m * akink)
    phi_ref, b_ref = ref.assistant_update(Fh, rows, m, loss_ref, T, phi0, b0, lr_a)
    phi, b = model(phi0), scalar_dev(b0)
    api.assistant_update(F, dev(rows), scalar_dev(m, torch.int32), m, dev(loss_ref),
                         scalar_dev(T), phi, b, lr_a, 0.0, ws)
    absx = np.asarray(Sa[rows].sum(axis=0)).ravel()
    assert_close_scaled(host(phi), phi_ref, np.abs(phi0.astype(np.float64)) + lr_a / m * absx,
                        "phi " + tag)
    assert abs(float(host(b)[0]) - b_ref) <= RTOL * (abs(b0) + lr_a), tag
    # both updates in one pass over the rows (labels from the kernel's own losses: a row
    # whose loss sits within rounding of T may take either label)
    w, phi, b = model(w0), model(phi0), scalar_dev(b0)
    Tt = scalar_dev(T)
    cfg = api.step_config(0.0, lam, lr, lr_a, 0.0, 1, 0, Tt)
    api.boss_assistant_step(F, dev(y), dev(rows), scalar_dev(m, torch.int32), m, w, phi, b, cfg,
                            loss, ws)
    assert_close_scaled(host(w), w_ref, np.abs(w0.astype(np.float64)) + lr / m * absx_w,
                        "w (one pass) " + tag, atol=lr / m * akink)
    on_T = np.abs(loss_ref.astype(np.float64) - T) <= RTOL * Sdot
    a_T = np.asarray(Sa[rows[on_T]].sum(axis=0)).ravel()
    assert_close_scaled(host(phi), phi_ref, np.abs(phi0.astype(np.float64)) + lr_a / m * absx,
                        "phi (one pass) " + tag, atol=lr_a / m * a_T)
    assert abs(float(host(b)[0]) - b_ref) <= RTOL * (abs(b0) + lr_a) + lr_a / m * on_T.sum(), tag


@pytest.mark.parametrize("block", range(4))
def test_csr_updates_random_shapes(ref, block):
    """Randomised shapes for the CSR Boss step and Assistant update: d from 37 to 1,200,000
    (below, at and above the sizes of the per-block LDS table, and beyond what the column bins
    cover), 1 to 40,000 rows of 0 to 200 entries, uniform / Zipf-like / hot-at-the-end columns,
    with and without values."""
    master = rng(7000 + block)
    for case in range(6):
        r = rng(int(master.integers(1 << 30)))
        d = int(r.choice([37, 600, 3072, 4096, 5000, 8192, 8193, 20000, 70000, 300000, 1 << 20, 1_200_000]))
        n = int(r.choice([1, 7, 300, 5000, 40000]))
        kind = r.choice(["uniform", "zipf", "hot_tail"])
        lo, hi = (1, 12) if r.random() < 0.5 else (30, 200)
        n = min(n, 3_000_000 // hi)
        _check_csr_updates(ref, r, d, n, kind, lo, hi, r.random() >= 0.3)


def test_csr_updates_with_model_vectors_off_16_byte_alignment(ref):
    """The bin owners move four model columns per 128-bit access wherever the vectors start."""
    r = rng(77)
    _check_csr_updates(ref, r, 20001, 3000, "zipf", 20, 60, True, misalign=True)
    _check_csr_updates(ref, r, 300000, 3000, "hot_tail", 20, 60, False, misalign=True)


@pytest.mark.parametrize("d", [3073, 3075, 3079, 3072 + 1021, 8193, 8195, 8192 + 1022,
                               3072 + (1 << 18), 3072 + (1 << 18) + 5, 8192 + (1 << 18), 8192 + (1 << 18) + 6])
def test_csr_updates_at_the_edges_of_the_column_bins(ref, d):
    """Feature counts just past the per-block table (3072 columns when both vectors are
    updated, 8192 with one): one, three, seven columns for the bins, a count that is no
    multiple of four (the owners fold four neighbours at a time and finish the model's last
    columns singly), fewer groups than bins, and both sides of the count at which the bins
    change from groups of 4 to groups of 16 columns.  Hot columns at the end of the range."""
    r = rng(900 + d % 1000)
    _check_csr_updates(ref, r, d, 2000, "hot_tail", 20, 60, True)
    _check_csr_updates(ref, r, d, 300, "uniform", 1, 12, False)
