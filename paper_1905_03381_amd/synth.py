"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws inputs (features, labels, permutations, stand-in Boss
losses).  It holds none of the method's arithmetic and is the one module both
the GPU tests and the CPU reference checks may import.  Everything is host
numpy, generated in fixed-size row chunks whose seeds depend only on
(seed, chunk number), so any chunk can be regenerated on its own.

The data sets of the paper's experiments (LIBSVM text sets of Section 3.4,
image and translation corpora of Section 6) are not available; these recipes
stand in for them by shape, sparsity and value distribution only.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

CHUNK_ROWS = 65536


def _rng(*key):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


def sign_pm1(v):
    """sign with sign(0) = +1, as float32."""
    return np.where(v >= 0, 1.0, -1.0).astype(np.float32)


def planted_w(d, seed=3381):
    return _rng(seed, 0).standard_normal(d).astype(np.float32)


def epoch_permutation(n, seed=7, epoch=0):
    """Shuffled index list the pools of one epoch are cut from (int32)."""
    return _rng(seed, epoch).permutation(n).astype(np.int32)


def pools(perm, P):
    """Consecutive slices of the epoch permutation; the last one may be short."""
    return [perm[s:s + P] for s in range(0, perm.shape[0], P)]


# ---------------------------------------------------------------------------
# dense linear-SVM workloads


def tiny_svm(n=10_000, d=128, seed=1905, w_seed=3381, noise=0.1):
    """x ~ N(0,1); y = sign(x.w* + noise*N(0,1)), w* ~ N(0,I)."""
    r = _rng(seed, 0)
    X = r.standard_normal((n, d), dtype=np.float32)
    w_star = planted_w(d, w_seed)
    eps = r.standard_normal(n).astype(np.float32)
    y = sign_pm1(X.astype(np.float64) @ w_star.astype(np.float64) + noise * eps)
    return X, y, w_star


def _dense_chunk(c, rows, d, seed, w_star, flip):
    r = _rng(seed, 1, c)
    x = r.standard_normal((rows, d), dtype=np.float32)
    nrm = np.sqrt(np.einsum("ij,ij->i", x, x, dtype=np.float64)).astype(np.float32)
    x /= nrm[:, None]
    y = sign_pm1(x @ w_star)
    flips = r.random(rows) < flip
    y[flips] = -y[flips]
    return x, y


def dense_svm(n=1_000_000, d=1024, seed=1905, w_seed=3381, flip=0.05, threads=8, out_x=None):
    """Unit-L2-norm Gaussian rows, labels from a planted w* with a share of flips.

    out_x: optional preallocated float32 [n, d] array (e.g. pinned host memory).
    """
    w_star = planted_w(d, w_seed)
    X = np.empty((n, d), dtype=np.float32) if out_x is None else out_x
    y = np.empty(n, dtype=np.float32)
    n_chunks = (n + CHUNK_ROWS - 1) // CHUNK_ROWS

    def job(c):
        lo = c * CHUNK_ROWS
        rows = min(CHUNK_ROWS, n - lo)
        X[lo:lo + rows], y[lo:lo + rows] = _dense_chunk(c, rows, d, seed, w_star, flip)

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(job, range(n_chunks)))
    return X, y, w_star


def dense_svm_rows(row_ids, n=1_000_000, d=1024, seed=1905, w_seed=3381, flip=0.05):
    """Regenerate selected rows of dense_svm() without building the whole set."""
    w_star = planted_w(d, w_seed)
    row_ids = np.asarray(row_ids, dtype=np.int64)
    X = np.empty((row_ids.shape[0], d), dtype=np.float32)
    y = np.empty(row_ids.shape[0], dtype=np.float32)
    chunk_of = row_ids // CHUNK_ROWS
    for c in np.unique(chunk_of):
        lo = int(c) * CHUNK_ROWS
        cx, cy = _dense_chunk(int(c), min(CHUNK_ROWS, n - lo), d, seed, w_star, flip)
        sel = np.nonzero(chunk_of == c)[0]
        X[sel], y[sel] = cx[row_ids[sel] - lo], cy[row_ids[sel] - lo]
    return X, y


# ---------------------------------------------------------------------------
# sparse linear-SVM workload (CSR)


def zipf_cdf(n_items, exponent):
    p = 1.0 / np.arange(1, n_items + 1, dtype=np.float64) ** exponent
    cdf = np.cumsum(p)
    return cdf / cdf[-1]


def _sparse_chunk(c, rows, d, seed, cdf, mean_nnz):
    r = _rng(seed, 2, c)
    want = np.maximum(1, r.poisson(mean_nnz, rows)).astype(np.int64)
    # Draw about twice as many Zipf column ids as wanted and keep, per row, the first
    # `want` distinct ones in draw order (a heavy-headed Zipf repeats itself a lot).
    draws = 2 * want + 16
    total = int(draws.sum())
    cols = np.minimum(np.searchsorted(cdf, r.random(total), side="left"), d - 1).astype(np.int64)
    row_of = np.repeat(np.arange(rows, dtype=np.int64), draws)
    _, first = np.unique(row_of * d + cols, return_index=True)
    first.sort()
    row_f = row_of[first]
    starts = np.searchsorted(row_f, np.arange(rows, dtype=np.int64), side="left")
    rank = np.arange(first.shape[0], dtype=np.int64) - starts[row_f]
    chosen = first[rank < want[row_f]]
    key = np.sort(row_of[chosen] * d + cols[chosen])  # ascending column ids within a row
    row_of, cols = key // d, (key % d).astype(np.int32)
    counts = np.bincount(row_of, minlength=rows).astype(np.int64)
    vals = r.lognormal(0.0, 1.0, cols.shape[0])
    ss = np.bincount(row_of, weights=vals * vals, minlength=rows)
    vals = (vals / np.sqrt(ss)[row_of]).astype(np.float32)
    return counts, cols, vals


def sparse_svm(n=2_000_000, d=1 << 20, seed=1905, w_seed=3381, mean_nnz=100, zipf=1.1,
               w_density=0.01, threads=8):
    """CSR rows: Poisson(mean_nnz) entries (at least 1, duplicates removed), Zipf column
    ids, lognormal values scaled to unit row norm; labels from a sparse planted w*."""
    cdf = zipf_cdf(d, zipf)
    n_chunks = (n + CHUNK_ROWS - 1) // CHUNK_ROWS
    jobs = [(c, min(CHUNK_ROWS, n - c * CHUNK_ROWS)) for c in range(n_chunks)]
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        parts = list(ex.map(lambda j: _sparse_chunk(j[0], j[1], d, seed, cdf, mean_nnz), jobs))
    counts = np.concatenate([p[0] for p in parts])
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    col = np.concatenate([p[1] for p in parts]).astype(np.int32)
    val = np.concatenate([p[2] for p in parts]).astype(np.float32)
    rw = _rng(w_seed, 2)
    w_star = np.zeros(d, dtype=np.float32)
    support = rw.choice(d, size=max(1, int(round(w_density * d))), replace=False)
    w_star[support] = rw.standard_normal(support.shape[0]).astype(np.float32)
    contrib = val.astype(np.float64) * w_star[col].astype(np.float64)
    score = np.add.reduceat(contrib, rowptr[:-1]) if col.shape[0] else np.zeros(n)
    y = sign_pm1(score)
    return rowptr, col, val, y, w_star


# ---------------------------------------------------------------------------
# image batch generator workload


def assistant_features(P=65536, d=512, seed=1905):
    return _rng(seed, 3).standard_normal((P, d), dtype=np.float32)


def image_bytes(image_ids, offsets, seed=1905):
    """Pixel byte of image `id` at byte offset `off`: a counter hash, so any gathered
    byte can be checked without keeping a host copy of the image store."""
    i = np.asarray(image_ids, dtype=np.uint64)
    o = np.asarray(offsets, dtype=np.uint64)
    with np.errstate(over="ignore"):
        h = (i * np.uint64(0x9E3779B97F4A7C15) + o * np.uint64(0xC2B2AE3D27D4EB4F)
             + np.uint64(seed))
        h ^= h >> np.uint64(29)
        h *= np.uint64(0xBF58476D1CE4E5B9)
        h ^= h >> np.uint64(32)
    return (h & np.uint64(0xFF)).astype(np.uint8)


def image_store_device(n_images, row_bytes, seed=1905, device="cuda", chunk=512):
    """The whole image store [n_images, row_bytes] uint8 built on the device with the same
    counter hash as image_bytes() (torch integer ops; 64-bit wrap-around arithmetic)."""
    import torch

    def s64(v):  # unsigned 64-bit constant as the signed value with the same bits
        return v - (1 << 64) if v >= (1 << 63) else v

    out = torch.empty((n_images, row_bytes), dtype=torch.uint8, device=device)
    off = torch.arange(row_bytes, dtype=torch.int64, device=device) * s64(0xC2B2AE3D27D4EB4F) + seed
    for lo in range(0, n_images, chunk):
        hi = min(n_images, lo + chunk)
        ids = torch.arange(lo, hi, dtype=torch.int64, device=device) * s64(0x9E3779B97F4A7C15)
        h = ids[:, None] + off[None, :]
        h ^= (h >> 29) & ((1 << 35) - 1)          # logical shift right by 29
        h *= s64(0xBF58476D1CE4E5B9)
        h ^= (h >> 32) & ((1 << 32) - 1)          # logical shift right by 32
        out[lo:hi] = (h & 0xFF).to(torch.uint8)
    return out


def gamma_losses(count, shape=2.0, scale=0.5, seed=1905, batch=0):
    """Stand-in Boss per-instance losses for one batch."""
    return _rng(seed, 4, batch).gamma(shape, scale, count).astype(np.float32)


# ---------------------------------------------------------------------------
# translation batch generator workload


def sentence_pairs(n=1_000_000, vocab=32_000, mean_len=27, max_len=128, zipf=1.0, seed=1905):
    """Token-list CSR over [source vocab | target vocab | len_s | len_t] (d = 2*vocab+2).

    Per pair: len_s, len_t ~ clip(Poisson(mean_len), 1, max_len); tokens Zipf over the
    vocab; target ids offset by vocab; two trailing entries hold len/max_len.  Token
    entries have value 1 and may repeat (a bag of tokens).
    """
    r = _rng(seed, 5)
    len_s = np.clip(r.poisson(mean_len, n), 1, max_len).astype(np.int32)
    len_t = np.clip(r.poisson(mean_len, n), 1, max_len).astype(np.int32)
    cdf = zipf_cdf(vocab, zipf)
    per_row = len_s.astype(np.int64) + len_t.astype(np.int64) + 2
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(per_row, out=rowptr[1:])
    nnz = int(rowptr[-1])
    col = np.empty(nnz, dtype=np.int32)
    val = np.ones(nnz, dtype=np.float32)
    tok = np.minimum(np.searchsorted(cdf, r.random(nnz)), vocab - 1).astype(np.int32)
    pos_in_row = np.arange(nnz, dtype=np.int64) - np.repeat(rowptr[:-1], per_row)
    ls = np.repeat(len_s.astype(np.int64), per_row)
    lt = np.repeat(len_t.astype(np.int64), per_row)
    is_src = pos_in_row < ls
    is_tgt = (~is_src) & (pos_in_row < ls + lt)
    col[is_src] = tok[is_src]
    col[is_tgt] = tok[is_tgt] + vocab
    f_s = pos_in_row == ls + lt
    f_t = pos_in_row == ls + lt + 1
    col[f_s] = 2 * vocab
    col[f_t] = 2 * vocab + 1
    val[f_s] = (ls[f_s] / max_len).astype(np.float32)
    val[f_t] = (lt[f_t] / max_len).astype(np.float32)
    return rowptr, col, val, len_s, len_t, 2 * vocab + 2
