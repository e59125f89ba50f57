"""GPU check of aa_fused_step_static (the entry point for callers that cannot allocate): called
through the C ABI, its outputs are compared with those of aa_fused_step on the same inputs --
integers, flags and ids bit for bit, floats within the 1e-5 scaled bound -- on two calls in a
row, the second on a smaller pool, and on a CSR step that fits the static scratch.  A step
that needs more scratch than the array holds must be refused before anything is launched."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_1905_03381_amd import api, synth

from gpu_util import assert_close_scaled, dev, host

pytestmark = pytest.mark.gpu


def _outputs(P):
    return dict(logit=torch.full((P,), 3.0, device="cuda"), prob=torch.full((P,), 3.0, device="cuda"),
                keep=torch.full((P,), 7, dtype=torch.uint8, device="cuda"),
                pos=torch.full((P,), -1, dtype=torch.int32, device="cuda"),
                ids=torch.full((P,), -1, dtype=torch.int32, device="cuda"),
                loss=torch.full((P,), -1.0, device="cuda"),
                cnt=torch.full((1,), -1, dtype=torch.int32, device="cuda"))


def _step(F, y, idx, P, w0, phi0, b0, cfg, ws):
    """One fused step from (w0, phi0, b0); ws None = the static-scratch entry point (raw C ABI)."""
    L = api.lib()
    w, phi, b = w0.clone(), phi0.clone(), b0.clone()
    o = _outputs(P)
    st = torch.cuda.current_stream().cuda_stream
    args = [F.ref(), y.data_ptr(), idx.data_ptr(), P, w.data_ptr(), phi.data_ptr(), b.data_ptr(),
            C.byref(cfg), o["logit"].data_ptr(), o["prob"].data_ptr(), o["keep"].data_ptr(),
            o["pos"].data_ptr(), o["ids"].data_ptr(), o["loss"].data_ptr(), o["cnt"].data_ptr()]
    if ws is None:
        rc = L.aa_fused_step_static(*args, st)
    else:
        rc = L.aa_fused_step(*args, ws.ptr, ws.bytes, st)
    assert rc == 0, api.status_string(rc)
    torch.cuda.synchronize()
    o.update(w=w, phi=phi, b=b)
    return {k: host(v) for k, v in o.items()}


def _compare(got, want, P):
    m = int(want["cnt"][0])
    assert int(got["cnt"][0]) == m
    for k in ("keep", "pos", "ids"):
        assert np.array_equal(got[k], want[k]), k       # untouched tails included
    for k in ("logit", "prob", "loss", "w", "phi", "b"):
        scale = np.maximum(np.abs(want[k]), 1e-30)
        assert_close_scaled(got[k], want[k], scale, k)
    # same kernels, same grid, fixed summation order: the floats are in fact identical
    for k in ("logit", "prob", "loss", "w", "phi", "b"):
        assert np.array_equal(got[k], want[k]), f"{k} differs in bits"


def test_static_scratch_dense_two_calls_in_a_row():
    n, d = 6000, 1024
    r = np.random.default_rng(5)
    X = r.standard_normal((n, d)).astype(np.float32)
    X /= np.linalg.norm(X, axis=1, keepdims=True)
    yh = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    Xd, y = dev(X), dev(yh)
    F = api.Features.dense(Xd)
    w0 = dev((0.5 * r.standard_normal(d)).astype(np.float32))
    phi0 = dev((0.1 * r.standard_normal(d)).astype(np.float32))
    b0 = dev(np.array([0.05], dtype=np.float32))
    T = torch.zeros(1, device="cuda")
    perm = synth.epoch_permutation(n)
    assert api.static_scratch_bytes() == 8 << 20
    for call, P in enumerate((4099, 517)):              # the second call on a smaller pool
        idx = dev(perm[call * 4099: call * 4099 + P].astype(np.int32))
        cfg = api.step_config(0.1, 1e-4, 0.5, 0.1, 0.0, 42, 3 + call, T)
        ws = api.Workspace(P, d)
        want = _step(F, y, idx, P, w0, phi0, b0, cfg, ws)
        got = _step(F, y, idx, P, w0, phi0, b0, cfg, None)
        assert 0 < int(want["cnt"][0]) < P
        _compare(got, want, P)


def test_static_scratch_small_csr_step():
    """The general (CSR) kernels through the same entry point: their scratch is cleared by the
    call itself, so a second call on a smaller pool still matches.  Float sums of this path
    depend on the arrival order of LDS adds, so they are compared within the bound only."""
    n, d = 3000, 1500
    r = np.random.default_rng(6)
    nnz = r.integers(1, 40, size=n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(nnz, out=rowptr[1:])
    col = np.concatenate([np.sort(r.choice(d, size=k, replace=False)) for k in nnz]).astype(np.int32)
    val = r.standard_normal(col.size).astype(np.float32)
    yh = np.where(r.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    F = api.Features.csr(dev(rowptr), dev(col), dev(val), d)
    y = dev(yh)
    w0 = dev((0.5 * r.standard_normal(d)).astype(np.float32))
    phi0 = dev((0.1 * r.standard_normal(d)).astype(np.float32))
    b0 = dev(np.array([0.0], dtype=np.float32))
    T = torch.zeros(1, device="cuda")
    for call, P in enumerate((2048, 300)):
        idx = dev(r.permutation(n)[:P].astype(np.int32))
        cfg = api.step_config(0.1, 1e-4, 0.5, 0.1, 0.0, 11, call, T)
        want = _step(F, y, idx, P, w0, phi0, b0, cfg, api.Workspace(P, d))
        got = _step(F, y, idx, P, w0, phi0, b0, cfg, None)
        m = int(want["cnt"][0])
        assert int(got["cnt"][0]) == m and 0 < m < P
        for k in ("keep", "pos", "ids"):
            assert np.array_equal(got[k], want[k]), k
        for k in ("logit", "prob", "loss"):
            assert_close_scaled(got[k], want[k], np.maximum(np.abs(want[k]), 1.0), k)
        for k in ("w", "phi", "b"):
            assert_close_scaled(got[k], want[k], np.maximum(np.abs(want[k]), 1e-2), k)


def test_static_scratch_refuses_what_does_not_fit():
    """A CSR step whose bins alone exceed the array: AA_ERR_WORKSPACE, nothing launched, the
    outputs keep their fill values."""
    n, d, P = 70000, 1 << 20, 65536
    assert api.workspace_bytes(P, d) > api.static_scratch_bytes()
    rowptr = torch.arange(n + 1, dtype=torch.int64, device="cuda")
    col = torch.zeros(n, dtype=torch.int32, device="cuda")
    F = api.Features.csr(rowptr, col, None, d)
    y = torch.ones(n, device="cuda")
    idx = torch.arange(P, dtype=torch.int32, device="cuda")
    w = torch.zeros(d, device="cuda")
    phi = torch.zeros(d, device="cuda")
    b = torch.zeros(1, device="cuda")
    T = torch.zeros(1, device="cuda")
    cfg = api.step_config(0.1, 1e-4, 0.5, 0.1, 0.0, 1, 0, T)
    cnt = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    rc = api.lib().aa_fused_step_static(F.ref(), y.data_ptr(), idx.data_ptr(), P, w.data_ptr(),
                                        phi.data_ptr(), b.data_ptr(), C.byref(cfg), None, None, None,
                                        None, None, None, cnt.data_ptr(),
                                        torch.cuda.current_stream().cuda_stream)
    assert rc == -4 and "workspace" in api.status_string(rc)
    assert int(host(cnt)[0]) == -7
    with pytest.raises(api.AAError):
        api.fused_step_static(F, y, idx, P, w, phi, b, cfg, None, None, None, None, None, None, cnt)
