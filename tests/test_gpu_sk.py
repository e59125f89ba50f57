"""GPU parity of the hard-threshold shrinking step (SK) against the oracle: dense register
layouts, the general dense kernel, CSR rows, and the dense configuration at full pool size."""
import numpy as np
import pytest
import torch

from paper_1905_03381_amd import api, synth

from gpu_util import (RTOL, abs_dot_scale, assert_close_scaled, col_abs_sum, csr_features,
                      dense_features, dev, host, row_dots, scalar_dev)

pytestmark = pytest.mark.gpu


def rng(seed):
    return np.random.default_rng(seed)


@pytest.fixture(scope="module")
def ws():
    return api.Workspace(1 << 17, 1 << 16)


def _run_and_check(ref, ws, Fh, F, y, idx, P, d, T, lam=1e-3, lr=0.5, w_seed=5, w_scale=1.2):
    """One step on both sides.  A candidate whose loss lies within the rounding band of the
    threshold may be kept by one side and dropped by the other; the keep flags are compared
    outside that band, the compaction against the GPU's own flags, and the update against
    the oracle's SVM step on the rows the GPU kept.  Small pools use a start vector with no
    candidate in the band, so there every output is compared with the oracle's directly."""
    ids_all = np.arange(P, dtype=np.int32) if idx is None else idx
    for s in range(w_seed, w_seed + 20):
        w0 = (w_scale * rng(s).standard_normal(d)).astype(np.float32)
        out = ref.sk_step(Fh, y, idx, P, w0, lam, lr, T)
        S = abs_dot_scale(Fh, ids_all, w0) + 1.0
        marg = y[ids_all] * row_dots(Fh, ids_all, w0)
        # loss > T  <=>  margin < 1 - T for T >= 0; a negative T keeps every candidate
        clear = np.abs(1.0 - T - marg) > 2 * RTOL * S if T >= 0 else np.ones(P, bool)
        if clear.all() or P > 2000:
            break
    else:
        raise AssertionError("every start vector leaves a loss inside the band of the threshold")
    assert clear.mean() > 0.99
    w = dev(w0)
    loss_pool = torch.full((P,), -3.0, device="cuda")
    keep = torch.full((P,), 9, dtype=torch.uint8, device="cuda")
    pos = torch.full((P,), -1, dtype=torch.int32, device="cuda")
    ids = torch.full((P,), -1, dtype=torch.int32, device="cuda")
    loss = torch.full((P,), -3.0, device="cuda")
    cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    api.sk_step(F, dev(y), dev(idx), P, w, scalar_dev(T), lam, lr, loss_pool, keep, pos, ids, loss,
                cnt, ws)
    k = host(keep)
    assert np.array_equal(k[clear], out["keep"][clear])
    assert set(np.unique(k)) <= {0, 1}
    m = int(host(cnt)[0])
    kept_pos = np.flatnonzero(k)
    assert m == kept_pos.size
    assert np.array_equal(host(pos)[:m], kept_pos)
    assert np.array_equal(host(ids)[:m], ids_all[kept_pos])
    assert np.all(host(pos)[m:] == -1) and np.all(host(loss)[m:] == -3.0)
    if clear.all():
        assert m == out["m"] and np.array_equal(host(ids)[:m], out["kept_ids"])
    assert_close_scaled(host(loss_pool), out["loss_pool"], S, "criterion")
    assert_close_scaled(host(loss)[:m], out["loss_pool"][kept_pos], S[kept_pos], "loss of kept rows")
    out = dict(out, m_gpu=m)
    if m == 0:
        assert np.array_equal(host(w), w0)
        return out
    kept_ids = ids_all[kept_pos]
    w_ref, loss_k = ref.svm_sgd_step(Fh, y, kept_ids, m, w0, lam, lr)
    if clear.all():
        assert np.array_equal(w_ref, out["w"])      # the oracle's SK step is that very step
    active = loss_k > 0
    on_kink = np.abs(1.0 - marg[kept_pos]) <= 2 * RTOL * S[kept_pos]
    scale = abs(1 - lr * lam) * np.abs(w0.astype(np.float64)) + lr / m * col_abs_sum(Fh, kept_ids[active])
    assert_close_scaled(host(w), w_ref, scale, "w", atol=lr / m * col_abs_sum(Fh, kept_ids[on_kink]))
    return out


DENSE_SHAPES = [
    (300, 128, None, 256),
    (700, 1024, None, 613),
    (500, 512, None, 500),
    (300, 2048, None, 200),
    (400, 36, None, 333),
    (400, 200, 256, 400),       # padded rows
    (300, 130, None, 250),      # general kernel
    (200, 4100, None, 150),     # general kernel
    (64, 1024, None, 1),
    (40_000, 1024, None, 40_000),   # many rows per wave
]


@pytest.mark.parametrize("n,d,ld,P", DENSE_SHAPES)
@pytest.mark.parametrize("T", [0.0, 0.6])
def test_sk_step_dense(ref, ws, n, d, ld, P, T):
    r = rng(7)
    X = r.standard_normal((n, ld or d)).astype(np.float32)
    X /= np.linalg.norm(X[:, :d], axis=1, keepdims=True)
    y = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    idx = r.permutation(n)[:P].astype(np.int32)
    Fh = ref.Features.dense(X, d=d)
    out = _run_and_check(ref, ws, Fh, dense_features(X, d=d), y, idx, P, d, T)
    if P > 100:
        assert 0 < out["m"] < P


def test_sk_step_limits(ref, ws):
    """T below every loss keeps the whole pool (the plain mini-batch step); T above every loss
    keeps nothing and leaves w alone; an empty pool is a no-op."""
    n, d, P = 500, 256, 400
    r = rng(8)
    X = r.standard_normal((n, d)).astype(np.float32)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    y = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    Fh, F = ref.Features.dense(X), dense_features(X)
    out = _run_and_check(ref, ws, Fh, F, y, None, P, d, -1.0)
    assert out["m"] == P
    out = _run_and_check(ref, ws, Fh, F, y, None, P, d, 1e6)
    assert out["m"] == 0 and out["m_gpu"] == 0
    w0 = rng(9).standard_normal(d).astype(np.float32)
    w = dev(w0)
    cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    api.sk_step(F, dev(y), None, 0, w, scalar_dev(0.0), 1e-3, 0.5, None, None, None, None, None, cnt, ws)
    assert int(host(cnt)[0]) == 0 and np.array_equal(host(w), w0)


def test_sk_step_csr(ref, ws):
    rowptr, col, val, y, _ = synth.sparse_svm(n=30_000, d=1 << 16, mean_nnz=100, threads=4)
    d, P = 1 << 16, 20_000
    idx = rng(10).permutation(rowptr.size - 1)[:P].astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    for T in (0.0, 0.5):
        out = _run_and_check(ref, ws, Fh, F, y, idx, P, d, T, w_scale=1.0)
        assert 0 < out["m"] < P


def test_sk_step_dense_config_pool(ref, ws):
    """Pool of 16,384 rows of width 1024 (the dense configuration's step shape), two chained
    steps from the oracle's state."""
    n, d, P = 65_536, 1024, 16_384
    X, y, _ = synth.dense_svm(n=n, d=d, threads=8)
    Fh, F = ref.Features.dense(X), dense_features(X)
    perm = synth.epoch_permutation(n, seed=7, epoch=0)
    for t in range(2):
        idx = perm[t * P:(t + 1) * P]
        out = _run_and_check(ref, ws, Fh, F, y, idx, P, d, 0.0, lam=1e-4, lr=1.0, w_seed=50 + 20 * t,
                             w_scale=0.5)
        assert 0 < out["m"] < P


def test_sk_epoch_matches_chained_oracle_steps(ref, ws):
    """aa_sk_epoch (device-side lr0/sqrt(t) schedule, compaction carried by the next pass): every
    step against the oracle's step from the GPU's previous state at the single-step tolerances
    (keep decisions outside the band around loss = T), then the epoch in one call, bit-identical
    to the step-wise run."""
    from stepwise import check_epoch
    n, d, P, lam, lr0, T = 6000, 128, 500, 1e-3, 0.5, 0.4
    r = rng(20)
    X = r.standard_normal((n, d)).astype(np.float32)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    y = np.where(X @ r.standard_normal(d) > 0, 1.0, -1.0).astype(np.float32)
    perm = r.permutation(n).astype(np.int32)
    w0 = (0.8 * r.standard_normal(d)).astype(np.float32)
    Fh, F = ref.Features.dense(X), dense_features(X)
    counts, state = check_epoch(ref, Fh, F, y, perm, n, P, w0, None, 0.0, gamma=0.0, seed=0, step0=0,
                                lam=lam, lr0=lr0, lr_a=0.0, T=T, ws=ws, hard=True)
    assert len(counts) == n // P and 0 < min(counts) and max(counts) < P
    assert state[3] == n // P


def test_sk_epoch_on_csr_rows(ref):
    """aa_sk_epoch over CSR rows (general kernels, one updated vector): every step against the
    oracle's step from the GPU's previous state, then the epoch in one call -- where from the
    second step on the update kernel of the step before has left the workspace ready and no
    launch clears it -- bit-identical to the step-wise run, twice."""
    from stepwise import check_epoch, run_whole
    rowptr, col, val, y, _ = synth.sparse_svm(n=12_000, d=1 << 16, mean_nnz=60, threads=4)
    d, n, P = 1 << 16, 9000, 2048
    perm = rng(31).permutation(rowptr.size - 1)[:n].astype(np.int32)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    ws = api.Workspace(P, d)
    w0 = (0.5 * rng(32).standard_normal(d)).astype(np.float32)
    args = dict(gamma=0.0, seed=0, step0=0, lam=1e-3, lr0=2.0, lr_a=0.0, T=0.6, ws=ws, hard=True)
    counts, state = check_epoch(ref, Fh, F, y, perm, n, P, w0, None, 0.0, **args)
    assert len(counts) == 5 and all(0 < m < P for m in counts) and state[3] == 5
    for _ in range(2):
        hist, _, _, again = run_whole(F, y, perm, n, P, w0, None, 0.0, **args)
        assert hist == counts and np.array_equal(again[0], state[0])
