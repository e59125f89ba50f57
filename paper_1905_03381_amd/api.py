"""Thin ctypes binding of libautoassist.so (include/autoassist.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
Tensors are torch CUDA tensors (device memory and streams come from PyTorch);
each function takes the same arguments as the C entry point of the same name
and launches on torch's current stream.  There is no CPU fallback: if the
library is missing or fails to load, every call raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libautoassist.so")

AA_OK = 0
AA_DENSE, AA_CSR = 0, 1

SYMBOLS = [
    "aa_version", "aa_status_string", "aa_workspace_bytes", "aa_workspace_init", "aa_profile_hook",
    "aa_profile_hooks",
    "aa_assistant_score", "aa_shrink", "aa_score_shrink", "aa_shrink_threshold", "aa_gather",
    "aa_gather_csr", "aa_svm_sgd_step", "aa_assistant_update", "aa_boss_assistant_step",
    "aa_fused_step", "aa_sk_step", "aa_train_epoch", "aa_threshold_update",
    "aa_threshold_assistant_update", "aa_bucket_batches",
    "aa_pipeline_workspace_bytes", "aa_train_epoch_stale", "aa_sk_epoch",
    "aa_static_scratch_bytes", "aa_fused_step_static",
]


class AAError(RuntimeError):
    pass


class aa_features(C.Structure):
    _fields_ = [("layout", C.c_int32), ("d", C.c_int32), ("n", C.c_int64),
                ("x", C.c_void_p), ("ld", C.c_int64),
                ("rowptr", C.c_void_p), ("col", C.c_void_p), ("val", C.c_void_p)]


class aa_step_config(C.Structure):
    _fields_ = [("gamma", C.c_float), ("lambda_", C.c_float), ("lr", C.c_float),
                ("lr_a", C.c_float), ("l2_a", C.c_float), ("reserved", C.c_int32),
                ("seed", C.c_uint64), ("step", C.c_uint64), ("T", C.c_void_p)]


_lib = None


def lib():
    """Load the HIP library built in-tree (build with `python -m paper_1905_03381_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise AAError(f"{LIB_PATH} is missing: build it with paper_1905_03381_amd/build.py; "
                      "there is no CPU fallback")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_size_t
    FP, CP = C.POINTER(aa_features), C.POINTER(aa_step_config)
    sig = {
        "aa_version": (i32, []),
        "aa_status_string": (C.c_char_p, [i32]),
        "aa_workspace_bytes": (sz, [i32, i32]),
        "aa_workspace_init": (i32, [vp, sz, vp]),
        "aa_profile_hook": (i32, [vp, vp]),
        "aa_profile_hooks": (i32, [vp, vp, i32]),
        "aa_assistant_score": (i32, [FP, vp, i32, vp, vp, vp, vp, vp]),
        "aa_shrink": (i32, [vp, i32, f32, u64, u64, vp, vp, vp, vp, sz, vp]),
        "aa_score_shrink": (i32, [FP, vp, i32, vp, vp, f32, u64, u64, vp, vp, vp, vp, vp, vp, sz, vp]),
        "aa_shrink_threshold": (i32, [vp, i32, vp, vp, vp, vp, vp, sz, vp]),
        "aa_gather": (i32, [vp, i64, vp, vp, vp, i32, vp, vp, vp]),
        "aa_gather_csr": (i32, [FP, vp, vp, vp, i32, vp, vp, vp, i64, vp, sz, vp]),
        "aa_svm_sgd_step": (i32, [FP, vp, vp, vp, i32, vp, f32, f32, f32, vp, vp, sz, vp]),
        "aa_assistant_update": (i32, [FP, vp, vp, i32, vp, vp, vp, vp, f32, f32, vp, sz, vp]),
        "aa_boss_assistant_step": (i32, [FP, vp, vp, vp, i32, vp, vp, vp, CP, vp, vp, sz, vp]),
        "aa_fused_step": (i32, [FP, vp, vp, i32, vp, vp, vp, CP, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "aa_static_scratch_bytes": (sz, []),
        "aa_fused_step_static": (i32, [FP, vp, vp, i32, vp, vp, vp, CP, vp, vp, vp, vp, vp, vp, vp, vp]),
        "aa_sk_step": (i32, [FP, vp, vp, i32, vp, vp, f32, f32, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "aa_train_epoch": (i32, [FP, vp, vp, i64, i32, vp, vp, vp, CP, vp, vp, vp, vp, vp, sz, vp]),
        "aa_sk_epoch": (i32, [FP, vp, vp, i64, i32, vp, vp, f32, f32, vp, vp, vp, vp, vp, sz, vp]),
        "aa_threshold_update": (i32, [vp, vp, i32, f32, vp, vp, vp]),
        "aa_threshold_assistant_update": (i32, [FP, vp, vp, i32, vp, f32, vp, vp, vp, vp, f32, f32, vp, sz, vp]),
        "aa_pipeline_workspace_bytes": (sz, [i32, i32, i32]),
        "aa_train_epoch_stale": (i32, [FP, vp, vp, i64, i32, i32, vp, vp, vp, CP, vp, vp, vp, vp, sz, vp, vp]),
        "aa_bucket_batches": (i32, [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def status_string(rc):
    return lib().aa_status_string(rc).decode()


def _check(rc, what):
    if rc != AA_OK:
        raise AAError(f"{what}: {status_string(rc)} ({rc})")


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


class Features:
    """Device feature matrix handle: Features.dense(x[, d]) or Features.csr(rowptr, col, val, d)."""

    def __init__(self, c, keep):
        self.c, self._keep = c, keep

    @classmethod
    def dense(cls, x, d=None):
        assert x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.stride(1) == 1
        c = aa_features(AA_DENSE, x.shape[1] if d is None else d, x.shape[0], x.data_ptr(),
                        x.stride(0), None, None, None)
        return cls(c, [x])

    @classmethod
    def csr(cls, rowptr, col, val, d):
        assert rowptr.is_cuda and rowptr.dtype == torch.int64 and col.dtype == torch.int32
        assert val is None or val.dtype == torch.float32
        c = aa_features(AA_CSR, d, rowptr.shape[0] - 1, None, 0, rowptr.data_ptr(),
                        col.data_ptr(), _ptr(val))
        return cls(c, [rowptr, col, val])

    @property
    def d(self):
        return self.c.d

    def ref(self):
        return C.byref(self.c)


class Workspace:
    """Device scratch for pools up to P_max candidates and d_max features."""

    def __init__(self, P_max, d_max, device="cuda", staleness=None):
        """staleness: size the workspace for aa_train_epoch_stale with up to that staleness."""
        if staleness is None:
            self.bytes = int(lib().aa_workspace_bytes(P_max, d_max))
        else:
            self.bytes = int(lib().aa_pipeline_workspace_bytes(P_max, d_max, staleness))
        self.buf = torch.empty(self.bytes + 256, dtype=torch.uint8, device=device)
        off = (-self.buf.data_ptr()) % 256
        self.ptr = self.buf.data_ptr() + off
        _check(lib().aa_workspace_init(self.ptr, self.bytes, _stream()), "aa_workspace_init")


def step_config(gamma, lam, lr, lr_a, l2_a, seed, step, T):
    """T: 1-element float32 CUDA tensor (device scalar).  The returned structure holds a
    reference to it, so the address stays valid as long as the configuration lives."""
    cfg = aa_step_config(gamma, lam, lr, lr_a, l2_a, 0, seed, step, T.data_ptr())
    cfg._threshold = T
    return cfg


def version():
    return int(lib().aa_version())


def workspace_bytes(P_max, d_max):
    return int(lib().aa_workspace_bytes(P_max, d_max))


def profile_hook(event_before, event_after):
    """Raw hipEvent_t handles (ints) or two Nones to disarm."""
    _check(lib().aa_profile_hook(event_before, event_after), "aa_profile_hook")


def profile_hooks(events_before, events_after):
    """Lists of raw hipEvent_t handles: pair i receives the start and stop time stamps of the i-th
    row-pass launch from now on.
    Returns the two ctypes arrays, which the caller keeps alive until those launches are issued."""
    n = len(events_before)
    assert n == len(events_after)
    arr_b = (C.c_void_p * max(n, 1))(*events_before)
    arr_a = (C.c_void_p * max(n, 1))(*events_after)
    _check(lib().aa_profile_hooks(arr_b, arr_a, n), "aa_profile_hooks")
    return arr_b, arr_a


def assistant_score(F, idx, P, phi, bias, logit, prob):
    _check(lib().aa_assistant_score(F.ref(), _ptr(idx), P, _ptr(phi), _ptr(bias), _ptr(logit),
                                    _ptr(prob), _stream()), "aa_assistant_score")


def shrink(prob, P, gamma, seed, step, keep, kept_pos, kept_count, ws):
    _check(lib().aa_shrink(_ptr(prob), P, gamma, seed, step, _ptr(keep), _ptr(kept_pos),
                           _ptr(kept_count), ws.ptr, ws.bytes, _stream()), "aa_shrink")


def shrink_threshold(crit, P, T, keep, kept_pos, kept_count, ws):
    _check(lib().aa_shrink_threshold(_ptr(crit), P, _ptr(T), _ptr(keep), _ptr(kept_pos),
                                     _ptr(kept_count), ws.ptr, ws.bytes, _stream()),
           "aa_shrink_threshold")


def score_shrink(F, idx, P, phi, bias, gamma, seed, step, logit, prob, keep, kept_pos, kept_count,
                 ws):
    _check(lib().aa_score_shrink(F.ref(), _ptr(idx), P, _ptr(phi), _ptr(bias), gamma, seed, step,
                                 _ptr(logit), _ptr(prob), _ptr(keep), _ptr(kept_pos),
                                 _ptr(kept_count), ws.ptr, ws.bytes, _stream()), "aa_score_shrink")


def gather(src, row_bytes, idx, kept_pos, kept_count, max_rows, dst, kept_ids):
    _check(lib().aa_gather(_ptr(src), row_bytes, _ptr(idx), _ptr(kept_pos), _ptr(kept_count),
                           max_rows, _ptr(dst), _ptr(kept_ids), _stream()), "aa_gather")


def gather_csr(F, idx, kept_pos, kept_count, max_rows, out_rowptr, out_col, out_val, out_nnz_cap,
               ws):
    _check(lib().aa_gather_csr(F.ref(), _ptr(idx), _ptr(kept_pos), _ptr(kept_count), max_rows,
                               _ptr(out_rowptr), _ptr(out_col), _ptr(out_val), out_nnz_cap,
                               ws.ptr, ws.bytes, _stream()), "aa_gather_csr")


def svm_sgd_step(F, y, rows, m_dev, m_max, w, lam, lr, radius, loss, ws):
    _check(lib().aa_svm_sgd_step(F.ref(), _ptr(y), _ptr(rows), _ptr(m_dev), m_max, _ptr(w), lam,
                                 lr, radius, _ptr(loss), ws.ptr, ws.bytes, _stream()),
           "aa_svm_sgd_step")


def assistant_update(F, rows, m_dev, m_max, loss, T, phi, bias, lr_a, l2_a, ws):
    _check(lib().aa_assistant_update(F.ref(), _ptr(rows), _ptr(m_dev), m_max, _ptr(loss), _ptr(T),
                                     _ptr(phi), _ptr(bias), lr_a, l2_a, ws.ptr, ws.bytes,
                                     _stream()), "aa_assistant_update")


def boss_assistant_step(F, y, rows, m_dev, m_max, w, phi, bias, cfg, loss, ws):
    _check(lib().aa_boss_assistant_step(F.ref(), _ptr(y), _ptr(rows), _ptr(m_dev), m_max, _ptr(w),
                                        _ptr(phi), _ptr(bias), C.byref(cfg), _ptr(loss), ws.ptr,
                                        ws.bytes, _stream()), "aa_boss_assistant_step")


def fused_step(F, y, idx, P, w, phi, bias, cfg, logit, prob, keep, kept_pos, kept_ids, loss,
               kept_count, ws):
    _check(lib().aa_fused_step(F.ref(), _ptr(y), _ptr(idx), P, _ptr(w), _ptr(phi), _ptr(bias),
                               C.byref(cfg), _ptr(logit), _ptr(prob), _ptr(keep), _ptr(kept_pos),
                               _ptr(kept_ids), _ptr(loss), _ptr(kept_count), ws.ptr, ws.bytes,
                               _stream()), "aa_fused_step")


def static_scratch_bytes():
    return int(lib().aa_static_scratch_bytes())


def fused_step_static(F, y, idx, P, w, phi, bias, cfg, logit, prob, keep, kept_pos, kept_ids, loss,
                      kept_count):
    _check(lib().aa_fused_step_static(F.ref(), _ptr(y), _ptr(idx), P, _ptr(w), _ptr(phi),
                                      _ptr(bias), C.byref(cfg), _ptr(logit), _ptr(prob), _ptr(keep),
                                      _ptr(kept_pos), _ptr(kept_ids), _ptr(loss), _ptr(kept_count),
                                      _stream()), "aa_fused_step_static")


def sk_step(F, y, idx, P, w, T, lam, lr, loss_pool, keep, kept_pos, kept_ids, loss, kept_count, ws):
    _check(lib().aa_sk_step(F.ref(), _ptr(y), _ptr(idx), P, _ptr(w), _ptr(T), lam, lr,
                            _ptr(loss_pool), _ptr(keep), _ptr(kept_pos), _ptr(kept_ids), _ptr(loss),
                            _ptr(kept_count), ws.ptr, ws.bytes, _stream()), "aa_sk_step")


def train_epoch(F, y, perm, n_perm, P, w, phi, bias, cfg, t_upd, kept_hist, ws, kept_ids_hist=None,
                loss_hist=None):
    _check(lib().aa_train_epoch(F.ref(), _ptr(y), _ptr(perm), n_perm, P, _ptr(w), _ptr(phi),
                                _ptr(bias), C.byref(cfg), _ptr(t_upd), _ptr(kept_hist),
                                _ptr(kept_ids_hist), _ptr(loss_hist), ws.ptr, ws.bytes, _stream()),
           "aa_train_epoch")


def sk_epoch(F, y, perm, n_perm, P, w, T, lam, lr0, t_upd, kept_hist, ws, kept_ids_hist=None,
             loss_hist=None):
    _check(lib().aa_sk_epoch(F.ref(), _ptr(y), _ptr(perm), n_perm, P, _ptr(w), _ptr(T), lam, lr0,
                             _ptr(t_upd), _ptr(kept_hist), _ptr(kept_ids_hist), _ptr(loss_hist),
                             ws.ptr, ws.bytes, _stream()), "aa_sk_epoch")


def train_epoch_stale(F, y, perm, n_perm, P, staleness, w, phi, bias, cfg, t_upd, kept_hist,
                      kept_ids_hist, ws, stream_gen):
    """stream_gen: a torch.cuda.Stream other than the current one (the Boss runs on the current)."""
    _check(lib().aa_train_epoch_stale(F.ref(), _ptr(y), _ptr(perm), n_perm, P, staleness, _ptr(w),
                                      _ptr(phi), _ptr(bias), C.byref(cfg), _ptr(t_upd),
                                      _ptr(kept_hist), _ptr(kept_ids_hist), ws.ptr, ws.bytes,
                                      _stream(), stream_gen.cuda_stream), "aa_train_epoch_stale")


def threshold_update(loss, m_dev, m_max, momentum, T, initialised):
    _check(lib().aa_threshold_update(_ptr(loss), _ptr(m_dev), m_max, momentum, _ptr(T),
                                     _ptr(initialised), _stream()), "aa_threshold_update")


def threshold_assistant_update(F, rows, m_dev, m_max, loss, momentum, T, initialised, phi, bias, lr_a,
                               l2_a, ws):
    _check(lib().aa_threshold_assistant_update(F.ref(), _ptr(rows), _ptr(m_dev), m_max, _ptr(loss),
                                               momentum, _ptr(T), _ptr(initialised), _ptr(phi),
                                               _ptr(bias), lr_a, l2_a, ws.ptr, ws.bytes, _stream()),
           "aa_threshold_assistant_update")


def bucket_batches(len_s, len_t, m_dev, m_max, width, n_buckets, token_budget, order, bucket_start,
                   batch_of, n_batches, ws):
    _check(lib().aa_bucket_batches(_ptr(len_s), _ptr(len_t), _ptr(m_dev), m_max, width, n_buckets,
                                   token_budget, _ptr(order), _ptr(bucket_start), _ptr(batch_of),
                                   _ptr(n_batches), ws.ptr, ws.bytes, _stream()), "aa_bucket_batches")
