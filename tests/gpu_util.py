"""Helpers for the GPU parity tests: device marshalling and the tolerances.

Tolerances (fp32 path against the fp64-accumulating oracle):
  * integer / byte / index outputs: bit-exact;
  * a sum of products: |gpu - ref| <= 1e-5 * max(|ref|, S) with S the sum of the absolute
    values of its terms (a plain relative error is meaningless when the sum cancels);
  * a keep decision is compared only when the draw is farther than 1e-6 from its
    probability; decisions on `margin < 1` only when farther than 1e-5 * S from 1.
"""
import numpy as np
import torch

from paper_1905_03381_amd import api

RTOL = 1e-5
DRAW_BAND = 1e-6


def dev(a, dtype=None):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def scalar_dev(v, dtype=torch.float32):
    return torch.tensor([v], dtype=dtype, device="cuda")


def dense_features(X, d=None):
    xd = dev(X)
    return api.Features.dense(xd, d=d)


def csr_features(rowptr, col, val, d):
    return api.Features.csr(dev(rowptr.astype(np.int64)), dev(col.astype(np.int32)),
                            None if val is None else dev(val.astype(np.float32)), d)


def rows_of(F_host, ids):
    """Dense float64 copy of the given rows of an oracle Features object (dense or CSR)."""
    ids = np.asarray(ids, dtype=np.int64)
    if F_host.c.layout == 0:
        return F_host.x[ids, :F_host.d].astype(np.float64)
    out = np.zeros((ids.size, F_host.d), dtype=np.float64)
    for r, i in enumerate(ids):
        lo, hi = F_host.rowptr[i], F_host.rowptr[i + 1]
        v = np.ones(hi - lo) if F_host.val is None else F_host.val[lo:hi].astype(np.float64)
        np.add.at(out[r], F_host.col[lo:hi], v)
    return out


def abs_dot_scale(F_host, ids, v):
    """S_r = sum_k |v_k x_rk| for each listed row."""
    ids = np.asarray(ids, dtype=np.int64)
    va = np.abs(np.asarray(v, dtype=np.float64))
    if F_host.c.layout == 0:
        return np.abs(F_host.x[ids, :F_host.d].astype(np.float64)) @ va
    out = np.zeros(ids.size)
    for r, i in enumerate(ids):
        lo, hi = F_host.rowptr[i], F_host.rowptr[i + 1]
        xv = np.ones(hi - lo) if F_host.val is None else np.abs(F_host.val[lo:hi].astype(np.float64))
        out[r] = np.sum(xv * va[F_host.col[lo:hi]])
    return out


def row_dots(F_host, ids, v):
    """x_r . v in float64 for each listed row (dense or CSR)."""
    ids = np.asarray(ids, dtype=np.int64)
    v = np.asarray(v, dtype=np.float64)
    if F_host.c.layout == 0:
        return F_host.x[ids, :F_host.d].astype(np.float64) @ v
    out = np.zeros(ids.size)
    for r, i in enumerate(ids):
        lo, hi = F_host.rowptr[i], F_host.rowptr[i + 1]
        xv = np.ones(hi - lo) if F_host.val is None else F_host.val[lo:hi].astype(np.float64)
        out[r] = np.sum(xv * v[F_host.col[lo:hi]])
    return out


def col_abs_sum(F_host, ids):
    """sum over the listed rows of |x_r|, per column, float64."""
    ids = np.asarray(ids, dtype=np.int64)
    if F_host.c.layout == 0:
        return np.abs(F_host.x[ids, :F_host.d].astype(np.float64)).sum(axis=0)
    out = np.zeros(F_host.d)
    for i in ids:
        lo, hi = F_host.rowptr[i], F_host.rowptr[i + 1]
        xv = np.ones(hi - lo) if F_host.val is None else np.abs(F_host.val[lo:hi].astype(np.float64))
        np.add.at(out, F_host.col[lo:hi], xv)
    return out


def assert_close_scaled(got, ref, scale, what, rtol=RTOL, atol=0.0):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    bound = rtol * np.maximum(np.abs(ref), scale) + atol
    err = np.abs(got - ref)
    bad = err > bound
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst "
                           f"err {err[bad].max():.3e} vs bound {bound[bad][np.argmax(err[bad])]:.3e}")


def assert_logit_prob(logit, prob, ref_logit, ref_prob, S, bias=0.0):
    S = S + abs(bias)
    assert_close_scaled(logit, ref_logit, S, "logit")
    g = ref_prob.astype(np.float64)
    # d sigmoid = g (1-g) ds, plus the relative error of exp/divide
    bound = g * (1 - g) * RTOL * np.maximum(np.abs(ref_logit), S) + RTOL * g + 1e-7
    err = np.abs(prob.astype(np.float64) - g)
    assert np.all(err <= bound), f"prob: worst err {err.max():.3e}"


def clear_draws(ref, prob_ref, gamma, seed, step):
    """Mask of pool positions whose draw is farther than the band from its probability."""
    u = ref.uniforms(seed, step, prob_ref.shape[0]).astype(np.float64)
    p = gamma + (1.0 - gamma) * prob_ref.astype(np.float64)
    return np.abs(u - p) > DRAW_BAND
