"""GPU parity of the two batch-generator workloads at their full shapes: the image batch
generator (65,536 candidates with 512 Assistant features, 150,528-byte images gathered into
256-image batches, labels "loss above the running median") and the translation batch generator
(1,000,000 sentence pairs as token-list CSR, kept pairs compacted into length-bucketed batches)."""
import numpy as np
import pytest
import torch

from paper_1905_03381_amd import api, synth

from gpu_util import (abs_dot_scale, assert_close_scaled, assert_logit_prob, clear_draws,
                      col_abs_sum, csr_features, dev, host, scalar_dev)

pytestmark = pytest.mark.gpu


def rng(seed):
    return np.random.default_rng(seed)


@pytest.mark.parametrize("sizes", [[255, 256, 1, 2, 1000], [16384, 16383, 7], [512, 513, 3, 4]])
def test_threshold_update_bit_exact(ref, sizes):
    r = rng(1)
    T_ref, init_ref = 0.0, False
    T = scalar_dev(123.0)
    init = torch.zeros(1, dtype=torch.int32, device="cuda")
    for m in sizes:
        loss = r.gamma(2.0, 0.5, m).astype(np.float32)
        T_ref, init_ref = ref.threshold_update(loss, 0.9, T_ref, init_ref)
        buf = torch.full((m + 3,), -7.0, device="cuda")
        buf[:m] = dev(loss)
        api.threshold_update(buf, scalar_dev(m, torch.int32), min(m + 3, 16384), 0.9, T, init)
        assert np.float32(T_ref) == host(T)[0] and int(host(init)[0]) == 1
    api.threshold_update(buf, scalar_dev(0, torch.int32), 10, 0.9, T, init)   # empty batch
    assert np.float32(T_ref) == host(T)[0]


@pytest.mark.parametrize("m", [6, 256, 511, 2000])
def test_threshold_update_with_ties(ref, m):
    """Losses drawn from three values: the middle elements are found among equal keys."""
    r = rng(2)
    T_ref, init_ref = 0.0, False
    T = scalar_dev(0.0)
    init = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(3):
        loss = r.choice(np.array([0.25, 0.5, 2.0], np.float32), m)
        T_ref, init_ref = ref.threshold_update(loss, 0.8, T_ref, init_ref)
        api.threshold_update(dev(loss), scalar_dev(m, torch.int32), m, 0.8, T, init)
        assert np.float32(T_ref) == host(T)[0]


@pytest.mark.parametrize("m", [200, 3000])
def test_threshold_update_nan_loss(ref, m):
    """A NaN among the losses (either median path): the threshold becomes NaN on both sides."""
    loss = rng(4).gamma(2.0, 0.5, m).astype(np.float32)
    loss[m // 3] = np.nan
    T_ref, init_ref = ref.threshold_update(loss, 0.9, 0.7, True)
    T = scalar_dev(0.7)
    init = torch.ones(1, dtype=torch.int32, device="cuda")
    api.threshold_update(dev(loss), scalar_dev(m, torch.int32), m, 0.9, T, init)
    assert np.isnan(T_ref) and np.isnan(host(T)[0]) and int(host(init)[0]) == 1 and init_ref


@pytest.mark.parametrize("m", [0, 1, 500, 2048, 2049, 100_003])
def test_bucket_batches_exact(ref, m):
    r = rng(m + 5)
    ls = np.clip(r.poisson(27, m), 1, 128).astype(np.int32)
    lt = np.clip(r.poisson(27, m), 1, 128).astype(np.int32)
    order_ref, start_ref, batch_ref, nb_ref = ref.bucket_batches(ls, lt, 8, 16, 4096)
    ws = api.Workspace(max(m, 1) + 10, 128)
    cap = m + 10
    order = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    batch_of = torch.full((cap,), -1, dtype=torch.int32, device="cuda")
    start = torch.full((17,), -1, dtype=torch.int32, device="cuda")
    nb = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    ls_d = torch.zeros(cap, dtype=torch.int32, device="cuda")
    lt_d = torch.zeros(cap, dtype=torch.int32, device="cuda")
    ls_d[:m], lt_d[:m] = dev(ls), dev(lt)
    api.bucket_batches(ls_d, lt_d, scalar_dev(m, torch.int32), cap, 8, 16, 4096, order, start,
                       batch_of, nb, ws)
    assert int(host(nb)[0]) == nb_ref
    assert np.array_equal(host(start), start_ref)
    assert np.array_equal(host(order)[:m], order_ref)
    assert np.array_equal(host(batch_of)[:m], batch_ref)
    assert np.all(host(order)[m:] == -1)


@pytest.mark.parametrize("m_max", [1000, 100_003])
def test_bucket_batches_32_buckets_in_the_smallest_accepted_workspace(ref, m_max):
    """The largest bucket count with a pair count that is no multiple of the tile: the call's
    own size check must cover everything its kernels index.  The workspace handed over is the
    smallest one the call accepts (found by bisection on the status code), followed in the same
    allocation by a guard region that has to stay untouched."""
    import ctypes as C
    r = rng(m_max)
    m = m_max
    ls = np.clip(r.poisson(60, m), 1, 300).astype(np.int32)
    lt = np.clip(r.poisson(60, m), 1, 300).astype(np.int32)
    order_ref, start_ref, batch_ref, nb_ref = ref.bucket_batches(ls, lt, 8, 32, 4096)
    order = torch.full((m,), -1, dtype=torch.int32, device="cuda")
    batch_of = torch.full((m,), -1, dtype=torch.int32, device="cuda")
    start = torch.full((33,), -1, dtype=torch.int32, device="cuda")
    nb = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    ls_d, lt_d, m_d = dev(ls), dev(lt), scalar_dev(m, torch.int32)
    hi = api.workspace_bytes(m_max, 128)
    guard = 1 << 16
    buf = torch.full((hi + guard + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    base = buf.data_ptr() + (-buf.data_ptr()) % 256
    L, st = api.lib(), torch.cuda.current_stream().cuda_stream

    def call(nbytes):
        return L.aa_bucket_batches(ls_d.data_ptr(), lt_d.data_ptr(), m_d.data_ptr(), m_max, 8, 32,
                                   4096, order.data_ptr(), start.data_ptr(), batch_of.data_ptr(),
                                   nb.data_ptr(), base, nbytes, st)

    lo = 0                               # refused at lo, accepted at hi
    assert call(lo) == -4 and call(hi) == 0
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if call(mid) == 0:
            hi = mid
        else:
            lo = mid
    torch.cuda.synchronize()
    buf.fill_(0xA5)
    assert call(hi) == 0
    assert int(host(nb)[0]) == nb_ref
    assert np.array_equal(host(start), start_ref)
    assert np.array_equal(host(order), order_ref) and np.array_equal(host(batch_of), batch_ref)
    off = base - buf.data_ptr()
    tail = host(buf)[off + hi: off + hi + guard]
    assert np.all(tail == 0xA5), "the call wrote past the workspace size it accepted"


def test_image_batch_generator_full_shape(ref):
    P, d, row_bytes, B = 65536, 512, 3 * 224 * 224, 256
    feats = synth.assistant_features(P, d)
    images = synth.image_store_device(P, row_bytes)
    r = rng(3)
    phi0 = (r.standard_normal(d) / np.sqrt(d)).astype(np.float32)
    idx = r.permutation(P).astype(np.int32)
    gamma, seed, step, lr_a = 0.1, 11, 0, 0.05
    Fh = ref.Features.dense(feats)
    F = api.Features.dense(dev(feats))
    ws = api.Workspace(P, d)
    # score + keep + compact
    ref_logit, ref_prob = ref.assistant_score(Fh, idx, P, phi0, bias=0.0)
    for seed in range(11, 40):
        if clear_draws(ref, ref_prob, gamma, seed, step).all():
            break
    keep_ref, pos_ref = ref.shrink(ref_prob, gamma, seed, step)
    m = pos_ref.size
    phi, b = dev(phi0), scalar_dev(0.0)
    prob = torch.zeros(P, device="cuda")
    keep = torch.zeros(P, dtype=torch.uint8, device="cuda")
    pos = torch.zeros(P, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    idx_d = dev(idx)
    api.score_shrink(F, idx_d, P, phi, b, gamma, seed, step, None, prob, keep, pos, cnt, ws)
    assert int(host(cnt)[0]) == m
    assert np.array_equal(host(keep), keep_ref) and np.array_equal(host(pos)[:m], pos_ref)
    assert_logit_prob(ref_logit, host(prob), ref_logit, ref_prob, abs_dot_scale(Fh, idx, phi0))
    # gather the kept images (one call; batches of 256 are consecutive slices) and their ids
    batches = torch.empty((P, row_bytes), dtype=torch.uint8, device="cuda")
    ids = torch.zeros(P, dtype=torch.int32, device="cuda")
    api.gather(images, row_bytes, idx_d, pos, cnt, P, batches, ids)
    kept_ids = idx[pos_ref]
    assert np.array_equal(host(ids)[:m], kept_ids)
    sample = r.choice(m, 24, replace=False)
    got = batches[torch.from_numpy(sample).cuda()].cpu().numpy()
    want = synth.image_bytes(kept_ids[sample][:, None], np.arange(row_bytes)[None, :])
    assert np.array_equal(got, want)                                     # whole images, bit-exact
    offs = r.integers(0, row_bytes, 64)
    got = batches[:m][:, torch.from_numpy(offs).cuda()].cpu().numpy()
    assert np.array_equal(got, synth.image_bytes(kept_ids[:, None], offs[None, :]))  # every row
    # the first and last 256-image batches equal a gather of just those rows
    one = torch.empty((B, row_bytes), dtype=torch.uint8, device="cuda")
    last = (m - 1) // B
    for bt in (0, last):
        size = min(B, m - bt * B)
        api.gather(images, row_bytes, idx_d, pos[bt * B:], scalar_dev(size, torch.int32), B, one,
                   None)
        assert torch.equal(one[:size], batches[bt * B:bt * B + size])
    # Assistant updates, one per batch, labelled by synthetic Boss losses against the running
    # median kept on the device
    T_r, init_r = 0.0, False
    T = scalar_dev(0.0)
    init = torch.zeros(1, dtype=torch.int32, device="cuda")
    # (a second copy of the state goes through the one-call form of the same two steps)
    phi2, b2, T2, init2 = dev(phi0), scalar_dev(0.0), scalar_dev(0.0), torch.zeros_like(init)
    n_batches = (m + B - 1) // B
    for bt in range(n_batches):
        size = min(B, m - bt * B)
        loss = synth.gamma_losses(size, 2.0, 0.5, batch=bt)
        rows = kept_ids[bt * B:bt * B + size]
        # every batch from the GPU's previous Assistant: the threshold chain is bit-exact, so the
        # labels are the oracle's; the update is held to the single-step tolerance
        phi_prev, b_prev = host(phi).copy(), float(host(b)[0])
        T_r, init_r = ref.threshold_update(loss, 0.9, T_r, init_r)
        phi_r, b_r = ref.assistant_update(Fh, rows, size, loss, T_r, phi_prev, b_prev, lr_a)
        loss_d, size_d = dev(loss), scalar_dev(size, torch.int32)
        api.threshold_update(loss_d, size_d, B, 0.9, T, init)
        api.assistant_update(F, ids[bt * B:], size_d, B, loss_d, T, phi, b, lr_a, 0.0, ws)
        assert host(T)[0] == np.float32(T_r), f"threshold after batch {bt}"
        api.threshold_assistant_update(F, ids[bt * B:], size_d, B, loss_d, 0.9, T2, init2, phi2, b2,
                                       lr_a, 0.0, ws)
        assert torch.equal(T2, T) and torch.equal(init2, init), f"one-call threshold, batch {bt}"
        assert torch.equal(phi2, phi) and torch.equal(b2, b), f"one-call update, batch {bt}"
        scale = np.abs(phi_prev.astype(np.float64)) + lr_a / size * np.abs(
            feats[rows].astype(np.float64)).sum(axis=0)
        assert_close_scaled(host(phi), phi_r, scale, f"phi after batch {bt}")
        assert abs(float(host(b)[0]) - b_r) <= 1e-5 * (abs(b_prev) + lr_a), f"bias after batch {bt}"


@pytest.mark.parametrize("d,ld", [(512, None), (128, None), (36, None), (200, 256), (1024, None), (130, None)])
@pytest.mark.parametrize("m,m_max", [(1, 1), (2, 7), (255, 256), (256, 256), (511, 512), (512, 512), (0, 64),
                                     (600, 700)])
def test_threshold_assistant_update_equals_the_two_calls(d, ld, m, m_max):
    """aa_threshold_assistant_update against aa_threshold_update + aa_assistant_update on the
    same inputs, bit for bit, over three batches in a row (first batch sets the threshold, the
    others move it): every register layout, the general kernel (d = 130) and a batch too large
    for the in-pass median (both fall back to the two calls), ties among the losses, an empty
    batch."""
    r = rng(1000 * d + m)
    n = 900
    X = r.standard_normal((n, ld or d)).astype(np.float32)
    F = api.Features.dense(dev(X), d=d)   # (ld > d: padded rows)
    ws = api.Workspace(max(m_max, 64), d)
    phi0 = (r.standard_normal(d) / 8).astype(np.float32)
    state = []
    for _ in range(2):
        state.append([dev(phi0), scalar_dev(0.25), scalar_dev(0.0), torch.zeros(1, dtype=torch.int32, device="cuda")])
    for batch in range(3):
        rows = dev(r.integers(0, n, size=max(m_max, 1)).astype(np.int32))
        loss = r.gamma(2.0, 0.5, size=max(m_max, 1)).astype(np.float32)
        loss[::3] = loss[0]                                  # ties
        loss_d, m_d = dev(loss), scalar_dev(m, torch.int32)
        phi, b, T, init = state[0]
        api.threshold_update(loss_d, m_d, m_max, 0.9, T, init)
        api.assistant_update(F, rows, m_d, m_max, loss_d, T, phi, b, 0.3, 1e-3, ws)
        phi, b, T, init = state[1]
        api.threshold_assistant_update(F, rows, m_d, m_max, loss_d, 0.9, T, init, phi, b, 0.3, 1e-3, ws)
        for name, x0, x1 in zip(("phi", "bias", "T", "initialised"), state[0], state[1]):
            assert torch.equal(x0, x1), f"{name} differs after batch {batch}"
    if m > 0:
        assert int(host(state[1][3])[0]) == 1 and not np.array_equal(host(state[1][0]), phi0)
    else:
        assert int(host(state[1][3])[0]) == 0 and np.array_equal(host(state[1][0]), phi0)


def test_threshold_assistant_update_nan_loss():
    """A NaN among the losses: the threshold becomes NaN in the one-call form as in the two calls
    (no label is 1 afterwards), and the Assistant's state equals theirs."""
    r = rng(77)
    n, d, m = 400, 512, 200
    F = api.Features.dense(dev(r.standard_normal((n, d)).astype(np.float32)))
    ws = api.Workspace(256, d)
    rows = dev(r.integers(0, n, size=m).astype(np.int32))
    loss = r.gamma(2.0, 0.5, size=m).astype(np.float32)
    loss[17] = np.nan
    phi0 = (r.standard_normal(d) / 8).astype(np.float32)
    out = []
    for one_call in (False, True):
        phi, b, T, init = dev(phi0), scalar_dev(0.0), scalar_dev(0.7), torch.ones(1, dtype=torch.int32, device="cuda")
        m_d = scalar_dev(m, torch.int32)
        if one_call:
            api.threshold_assistant_update(F, rows, m_d, m, dev(loss), 0.9, T, init, phi, b, 0.3, 0.0, ws)
        else:
            api.threshold_update(dev(loss), m_d, m, 0.9, T, init)
            api.assistant_update(F, rows, m_d, m, dev(loss), T, phi, b, 0.3, 0.0, ws)
        out.append((host(phi).copy(), host(b).copy(), host(T).copy()))
    assert np.isnan(out[0][2][0]) and np.isnan(out[1][2][0])
    assert np.array_equal(out[0][0], out[1][0]) and np.array_equal(out[0][1], out[1][1])


def test_translation_batch_generator_full_shape(ref):
    n, vocab = 1_000_000, 32_000
    rowptr, col, val, len_s, len_t, d = synth.sentence_pairs(n=n, vocab=vocab)
    Fh = ref.Features.csr(rowptr, col, val, d)
    F = csr_features(rowptr, col, val, d)
    ws = api.Workspace(n, d)
    r = rng(4)
    phi0 = (0.05 * r.standard_normal(d)).astype(np.float32)
    gamma, seed, step = 0.1, 21, 0
    # one pool of all pairs, scored in data-set order
    ref_logit, ref_prob = ref.assistant_score(Fh, None, n, phi0, bias=-0.2)
    keep_ref, pos_ref = ref.shrink(ref_prob, gamma, seed, step)
    clear = clear_draws(ref, ref_prob, gamma, seed, step)
    phi, b = dev(phi0), scalar_dev(-0.2)
    prob = torch.zeros(n, device="cuda")
    keep = torch.zeros(n, dtype=torch.uint8, device="cuda")
    pos = torch.zeros(n, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.score_shrink(F, None, n, phi, b, gamma, seed, step, None, prob, keep, pos, cnt, ws)
    k = host(keep)
    assert np.array_equal(k[clear], keep_ref[clear])
    sample = r.choice(n, 20_000, replace=False)
    S = abs_dot_scale(Fh, sample, phi0)
    assert_logit_prob(ref_logit[sample], host(prob)[sample], ref_logit[sample], ref_prob[sample], S,
                      bias=-0.2)
    m = int(host(cnt)[0])
    kept = np.flatnonzero(k)
    assert m == kept.size and np.array_equal(host(pos)[:m], kept)
    # lengths of the kept pairs, then the length-bucketed batches of 4,096 padded tokens
    ls_k = torch.zeros(n, dtype=torch.int32, device="cuda")
    lt_k = torch.zeros(n, dtype=torch.int32, device="cuda")
    api.gather(dev(len_s), 4, None, pos, cnt, n, ls_k, None)
    api.gather(dev(len_t), 4, None, pos, cnt, n, lt_k, None)
    assert np.array_equal(host(ls_k)[:m], len_s[kept]) and np.array_equal(host(lt_k)[:m], len_t[kept])
    order = torch.zeros(n, dtype=torch.int32, device="cuda")
    batch_of = torch.zeros(n, dtype=torch.int32, device="cuda")
    start = torch.zeros(17, dtype=torch.int32, device="cuda")
    nb = torch.zeros(1, dtype=torch.int32, device="cuda")
    api.bucket_batches(ls_k, lt_k, cnt, n, 8, 16, 4096, order, start, batch_of, nb, ws)
    order_ref, start_ref, batch_ref, nb_ref = ref.bucket_batches(len_s[kept], len_t[kept], 8, 16, 4096)
    assert int(host(nb)[0]) == nb_ref and np.array_equal(host(start), start_ref)
    assert np.array_equal(host(order)[:m], order_ref) and np.array_equal(host(batch_of)[:m], batch_ref)
    # compacted CSR of the kept pairs
    nnz = int(np.diff(rowptr)[kept].sum())
    out_ptr = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
    out_col = torch.zeros(nnz, dtype=torch.int32, device="cuda")
    out_val = torch.zeros(nnz, device="cuda")
    api.gather_csr(F, None, pos, cnt, n, out_ptr, out_col, out_val, nnz, ws)
    want_ptr, want_col, want_val = ref.gather_csr(Fh, None, kept.astype(np.int32), nnz)
    assert np.array_equal(host(out_ptr)[:m + 1], want_ptr)
    assert np.array_equal(host(out_col), want_col) and np.array_equal(host(out_val), want_val)
    # Assistant update over the kept pairs, labelled by synthetic Boss losses
    loss = synth.gamma_losses(m, 2.0, 1.0, batch=7)
    T, lr_a = 1.7, 0.5
    phi_ref, b_ref = ref.assistant_update(Fh, kept.astype(np.int32), m, loss, T, phi0, -0.2, lr_a)
    api.assistant_update(F, pos, cnt, n, dev(loss), scalar_dev(T), phi, b, lr_a, 0.0, ws)
    scale = np.abs(phi0.astype(np.float64)) + lr_a / m * col_abs_sum(Fh, kept)
    assert_close_scaled(host(phi), phi_ref, scale, "phi")
    assert abs(float(host(b)[0]) - b_ref) <= 1e-5 * (0.2 + lr_a)
