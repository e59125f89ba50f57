"""numpy/ctypes front end of the CPU oracle (oracle/aa_ref.c).

TEST INFRASTRUCTURE ONLY.  Loads oracle/libaa_ref.so (plain C, gcc) and wraps
each function with host numpy arrays.  Nothing here touches the GPU library;
only tests, the smoke check and the benchmark's cpu_baseline leg import it.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


class _Features(C.Structure):
    _fields_ = [("layout", C.c_int32), ("d", C.c_int32), ("n", C.c_int64),
                ("x", C.c_void_p), ("ld", C.c_int64),
                ("rowptr", C.c_void_p), ("col", C.c_void_p), ("val", C.c_void_p)]


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.aa_ref_uniform.restype = C.c_float
        L.aa_ref_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32]
        L.aa_ref_primal_objective.restype = C.c_double
        L.aa_ref_assistant_objective.restype = C.c_double
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what} failed with status {rc}")


class Features:
    """Host feature matrix: Features.dense(x) or Features.csr(rowptr, col, val, d)."""

    def __init__(self):
        self.c = _Features()
        self._keep = []

    @classmethod
    def dense(cls, x, d=None):
        x = np.ascontiguousarray(x, dtype=np.float32)
        assert x.ndim == 2
        f = cls()
        f._keep = [x]
        f.c.layout, f.c.n, f.c.ld = 0, x.shape[0], x.shape[1]
        f.c.d = x.shape[1] if d is None else d
        f.c.x = x.ctypes.data
        f.x = x
        return f

    @classmethod
    def csr(cls, rowptr, col, val, d):
        rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
        col = np.ascontiguousarray(col, dtype=np.int32)
        val = None if val is None else np.ascontiguousarray(val, dtype=np.float32)
        f = cls()
        f._keep = [rowptr, col, val]
        f.c.layout, f.c.n, f.c.d = 1, rowptr.shape[0] - 1, d
        f.c.rowptr, f.c.col = rowptr.ctypes.data, col.ctypes.data
        f.c.val = None if val is None else val.ctypes.data
        f.rowptr, f.col, f.val = rowptr, col, val
        return f

    @property
    def d(self):
        return self.c.d

    @property
    def n(self):
        return self.c.n

    def ref(self):
        return C.byref(self.c)


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().aa_ref_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def uniform(seed, step, j):
    return float(lib().aa_ref_uniform(seed, step, j))


def uniforms(seed, step, P):
    L = lib()
    return np.array([L.aa_ref_uniform(seed, step, j) for j in range(P)], dtype=np.float32)


def assistant_score(F, idx, P, phi, bias=None):
    idx, phi = _i32(idx), _f32(phi)
    b = None if bias is None else np.array([bias], dtype=np.float32)
    logit = np.zeros(P, dtype=np.float32)
    prob = np.zeros(P, dtype=np.float32)
    _check(lib().aa_ref_assistant_score(F.ref(), _p(idx), C.c_int32(P), _p(phi), _p(b),
                                        _p(logit), _p(prob)), "assistant_score")
    return logit, prob


def shrink(prob, gamma, seed, step):
    prob = _f32(prob)
    P = prob.shape[0]
    keep = np.zeros(P, dtype=np.uint8)
    kept_pos = np.zeros(max(P, 1), dtype=np.int32)
    m = C.c_int32(0)
    _check(lib().aa_ref_shrink(_p(prob), C.c_int32(P), C.c_float(gamma), C.c_uint64(seed),
                               C.c_uint64(step), _p(keep), _p(kept_pos), C.byref(m)), "shrink")
    return keep, kept_pos[:m.value].copy()


def shrink_threshold(crit, T):
    crit = _f32(crit)
    P = crit.shape[0]
    keep = np.zeros(P, dtype=np.uint8)
    kept_pos = np.zeros(max(P, 1), dtype=np.int32)
    m = C.c_int32(0)
    _check(lib().aa_ref_shrink_threshold(_p(crit), C.c_int32(P), C.c_float(T), _p(keep),
                                         _p(kept_pos), C.byref(m)), "shrink_threshold")
    return keep, kept_pos[:m.value].copy()


def sample_batch(prob, gamma, seed, step, batch_size):
    prob = _f32(prob)
    P = prob.shape[0]
    B = np.zeros(max(batch_size, 1), dtype=np.int32)
    size, consumed = C.c_int32(0), C.c_int32(0)
    _check(lib().aa_ref_sample_batch(_p(prob), C.c_int32(P), C.c_float(gamma), C.c_uint64(seed),
                                     C.c_uint64(step), C.c_int32(batch_size), _p(B),
                                     C.byref(size), C.byref(consumed)), "sample_batch")
    return B[:size.value].copy(), consumed.value


def gather(src, idx, kept_pos):
    """src: 2-D array of any dtype (rows) or None.  Returns (dst, kept_ids)."""
    idx, kept_pos = _i32(idx), _i32(kept_pos)
    m = kept_pos.shape[0]
    ids = np.zeros(max(m, 1), dtype=np.int32)
    if src is None:
        _check(lib().aa_ref_gather(None, C.c_int64(0), _p(idx), _p(kept_pos), C.c_int32(m),
                                   None, _p(ids)), "gather")
        return None, ids[:m].copy()
    src = np.ascontiguousarray(src)
    row_bytes = src.strides[0] if src.ndim > 1 else src.itemsize
    dst = np.zeros((m,) + src.shape[1:], dtype=src.dtype)
    _check(lib().aa_ref_gather(_p(src), C.c_int64(row_bytes), _p(idx), _p(kept_pos),
                               C.c_int32(m), _p(dst), _p(ids)), "gather")
    return dst, ids[:m].copy()


def gather_csr(F, idx, kept_pos, nnz_cap):
    idx, kept_pos = _i32(idx), _i32(kept_pos)
    m = kept_pos.shape[0]
    out_rowptr = np.zeros(m + 1, dtype=np.int64)
    out_col = np.zeros(max(nnz_cap, 1), dtype=np.int32)
    out_val = None if F.val is None else np.zeros(max(nnz_cap, 1), dtype=np.float32)
    _check(lib().aa_ref_gather_csr(F.ref(), _p(idx), _p(kept_pos), C.c_int32(m), _p(out_rowptr),
                                   _p(out_col), _p(out_val), C.c_int64(nnz_cap)), "gather_csr")
    nnz = int(out_rowptr[m])
    return out_rowptr, out_col[:nnz].copy(), (None if out_val is None else out_val[:nnz].copy())


def svm_sgd_step(F, y, rows, m, w, lam, lr, radius=0.0):
    """Returns (w_new, loss[m]); w is not modified in place."""
    y, rows = _f32(y), _i32(rows)
    w = np.array(w, dtype=np.float32, copy=True)
    loss = np.zeros(max(m, 1), dtype=np.float32)
    _check(lib().aa_ref_svm_sgd_step(F.ref(), _p(y), _p(rows), C.c_int32(m), _p(w),
                                     C.c_float(lam), C.c_float(lr), C.c_float(radius),
                                     _p(loss)), "svm_sgd_step")
    return w, loss[:m].copy()


def vanilla_minibatch_sgd(F, y, idx, P, w, lam, lr):
    y, idx = _f32(y), _i32(idx)
    w = np.array(w, dtype=np.float32, copy=True)
    _check(lib().aa_ref_vanilla_minibatch_sgd(F.ref(), _p(y), _p(idx), C.c_int32(P), _p(w),
                                              C.c_float(lam), C.c_float(lr)), "vanilla_sgd")
    return w


def assistant_update(F, rows, m, loss, T, phi, bias, lr_a, l2_a=0.0):
    """Returns (phi_new, bias_new); bias None stays None."""
    rows, loss = _i32(rows), _f32(loss)
    phi = np.array(phi, dtype=np.float32, copy=True)
    b = None if bias is None else np.array([bias], dtype=np.float32)
    _check(lib().aa_ref_assistant_update(F.ref(), _p(rows), C.c_int32(m), _p(loss), C.c_float(T),
                                         _p(phi), _p(b), C.c_float(lr_a), C.c_float(l2_a)),
           "assistant_update")
    return phi, (None if b is None else float(b[0]))


def primal_objective(F, y, rows, count, w, lam):
    y, rows, w = _f32(y), _i32(rows), _f32(w)
    return float(lib().aa_ref_primal_objective(F.ref(), _p(y), _p(rows), C.c_int64(count), _p(w),
                                               C.c_float(lam)))


def assistant_objective(F, rows, m, z, phi, bias=None):
    rows, phi = _i32(rows), _f32(phi)
    z = np.ascontiguousarray(z, dtype=np.uint8)
    b = None if bias is None else np.array([bias], dtype=np.float32)
    return float(lib().aa_ref_assistant_objective(F.ref(), _p(rows), C.c_int32(m), _p(z), _p(phi),
                                                  _p(b)))


def step(F, y, idx, P, w, phi, bias, gamma, seed, step_no, lam, lr, T, lr_a, l2_a=0.0):
    """One whole step.  Returns a dict with the new state and every intermediate."""
    y, idx = _f32(y), _i32(idx)
    w = np.array(w, dtype=np.float32, copy=True)
    phi = np.array(phi, dtype=np.float32, copy=True)
    b = np.array([bias], dtype=np.float32)
    logit = np.zeros(max(P, 1), dtype=np.float32)
    prob = np.zeros(max(P, 1), dtype=np.float32)
    keep = np.zeros(max(P, 1), dtype=np.uint8)
    kept_pos = np.zeros(max(P, 1), dtype=np.int32)
    kept_ids = np.zeros(max(P, 1), dtype=np.int32)
    loss = np.zeros(max(P, 1), dtype=np.float32)
    m = C.c_int32(0)
    _check(lib().aa_ref_step(F.ref(), _p(y), _p(idx), C.c_int32(P), _p(w), _p(phi), _p(b),
                             C.c_float(gamma), C.c_uint64(seed), C.c_uint64(step_no),
                             C.c_float(lam), C.c_float(lr), C.c_float(T), C.c_float(lr_a),
                             C.c_float(l2_a), _p(logit), _p(prob), _p(keep), _p(kept_pos),
                             _p(kept_ids), _p(loss), C.byref(m)), "step")
    k = m.value
    return dict(w=w, phi=phi, bias=float(b[0]), logit=logit[:P], prob=prob[:P], keep=keep[:P],
                kept_pos=kept_pos[:k].copy(), kept_ids=kept_ids[:k].copy(),
                loss=loss[:k].copy(), m=k)


def sk_step(F, y, idx, P, w, lam, lr, T):
    """One hard-threshold shrinking step (SK).  Returns a dict like step()."""
    y, idx = _f32(y), _i32(idx)
    w = np.array(w, dtype=np.float32, copy=True)
    loss_pool = np.zeros(max(P, 1), dtype=np.float32)
    keep = np.zeros(max(P, 1), dtype=np.uint8)
    kept_pos = np.zeros(max(P, 1), dtype=np.int32)
    kept_ids = np.zeros(max(P, 1), dtype=np.int32)
    loss = np.zeros(max(P, 1), dtype=np.float32)
    m = C.c_int32(0)
    _check(lib().aa_ref_sk_step(F.ref(), _p(y), _p(idx), C.c_int32(P), _p(w), C.c_float(lam),
                                C.c_float(lr), C.c_float(T), _p(loss_pool), _p(keep),
                                _p(kept_pos), _p(kept_ids), _p(loss), C.byref(m)), "sk_step")
    k = m.value
    return dict(w=w, loss_pool=loss_pool[:P], keep=keep[:P], kept_pos=kept_pos[:k].copy(),
                kept_ids=kept_ids[:k].copy(), loss=loss[:k].copy(), m=k)


def sk_sgd(F, y, w0, mu, G, D, seed, K, w_star=None):
    """K steps of the iteration of Theorem 1.  Returns (w, dist2 or None, picked, dropped)."""
    y = _f32(y)
    w = np.array(w0, dtype=np.float64, copy=True)
    ws = None if w_star is None else np.ascontiguousarray(w_star, dtype=np.float64)
    dist2 = None if ws is None else np.zeros(K + 1, dtype=np.float64)
    picked = np.zeros(max(K, 1), dtype=np.int32)
    dropped = C.c_int32(0)
    _check(lib().aa_ref_sk_sgd(F.ref(), _p(y), _p(w), C.c_double(mu), C.c_double(G), C.c_double(D),
                               C.c_uint64(seed), C.c_int32(K), _p(ws), _p(dist2), _p(picked),
                               C.byref(dropped)), "sk_sgd")
    return w, dist2, picked[:K], dropped.value


def train_stale(F, y, perm, P, w, phi, bias, gamma, seed, step0, lam, lr0, T, lr_a, staleness,
                l2_a=0.0, schedule=True):
    """The asynchronous Boss/Assistant schedule of Section 5.3 made deterministic: the batch
    of pool s is generated (score, keep draw, compaction) with the Assistant as it stood
    after `s - staleness` updates, i.e. `staleness` batches wait in the Boss queue while the
    Assistant keeps learning from the losses the Boss sends back.  Tick s: the Boss takes
    batch s (losses at its current w, then its update, step size lr0 / sqrt(number of
    updates so far)), then the Assistant learns from (ids, losses) of that batch at its
    current parameters.  staleness = 0 is the synchronous step().  schedule=False keeps the
    Boss step size at lr0.  Returns a dict with the final state and, per tick, the kept
    count, the kept ids and the keep probabilities the batch was drawn with."""
    perm = _i32(perm)
    w = np.array(w, dtype=np.float32, copy=True)
    versions = [(np.array(phi, dtype=np.float32, copy=True), float(bias))]  # Assistant after t ticks
    ms, ids_hist, prob_hist, t_upd = [], [], [], 0
    n = perm.shape[0]
    for s in range((n + P - 1) // P):
        idx = perm[s * P:(s + 1) * P]
        phi_g, b_g = versions[max(0, s - staleness)]
        _, prob = assistant_score(F, idx, idx.shape[0], phi_g, b_g)
        _, pos = shrink(prob, gamma, seed, step0 + s)
        m = pos.shape[0]
        ids = idx[pos]
        phi_c, b_c = versions[s]
        if m > 0:
            t_upd += 1
            lr = np.float32(np.float32(lr0) / np.sqrt(np.float32(t_upd))) if schedule else np.float32(lr0)
            w, loss = svm_sgd_step(F, y, ids, m, w, lam, lr)
            phi_n, b_n = assistant_update(F, ids, m, loss, T, phi_c, b_c, lr_a, l2_a)
        else:
            phi_n, b_n = phi_c, b_c
        versions.append((phi_n, b_n))
        ms.append(m)
        ids_hist.append(ids.copy())
        prob_hist.append(prob)
    phi_f, b_f = versions[-1]
    return dict(w=w, phi=phi_f, bias=b_f, m=ms, kept_ids=ids_hist, prob=prob_hist, t_upd=t_upd)


def threshold_update(loss, momentum, T, initialised):
    """Returns (T_new, initialised_new)."""
    loss = _f32(loss)
    t = np.array([T], dtype=np.float32)
    init = C.c_int32(1 if initialised else 0)
    _check(lib().aa_ref_threshold_update(_p(loss), C.c_int32(loss.shape[0]), C.c_float(momentum),
                                         _p(t), C.byref(init)), "threshold_update")
    return float(t[0]), bool(init.value)


def bucket_batches(len_s, len_t, width, n_buckets, token_budget):
    len_s, len_t = _i32(len_s), _i32(len_t)
    m = len_s.shape[0]
    order = np.zeros(max(m, 1), dtype=np.int32)
    bucket_start = np.zeros(n_buckets + 1, dtype=np.int32)
    batch_of = np.zeros(max(m, 1), dtype=np.int32)
    nb = lib().aa_ref_bucket_batches(_p(len_s), _p(len_t), C.c_int32(m), C.c_int32(width),
                                     C.c_int32(n_buckets), C.c_int32(token_budget), _p(order),
                                     _p(bucket_start), _p(batch_of))
    if nb < 0:
        raise ValueError(f"bucket_batches failed with status {nb}")
    return order[:m].copy(), bucket_start, batch_of[:m].copy(), nb
