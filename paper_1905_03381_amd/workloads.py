"""Timing drivers for the workloads beside the dense linear-SVM benchmark.

    python -m paper_1905_03381_amd.workloads sparse        # sparse linear SVM, CSR rows
    python -m paper_1905_03381_amd.workloads images        # image batch generator
    python -m paper_1905_03381_amd.workloads translation   # translation batch generator
    python -m paper_1905_03381_amd.workloads sk            # hard-threshold shrinking, dense rows
    python -m paper_1905_03381_amd.workloads stale         # two-stream Boss / Assistant pipeline
    python -m paper_1905_03381_amd.workloads rho           # dense fused step at fixed keep rates
    python -m paper_1905_03381_amd.workloads score         # dense scoring pass at growing pool sizes

Each prints one JSON line: the stages of the workload with their time per call (HIP events
on the launch stream, median of the repeats), the bytes each stage has to move and the
resulting GB/s.  Inputs are the seeded synthetic generators of `synth`, resident in HBM
before anything is timed.  Every stage runs in the HIP library; a missing library raises.
"""
import argparse
import json
import sys
import time

import numpy as np


def _timed(torch, fn, repeats, setup=None):
    """Median time of fn() in microseconds, measured with events on the current stream."""
    times = []
    for i in range(repeats + 1):
        if setup:
            setup()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        if i:                                   # the first call loads the kernels
            times.append(e0.elapsed_time(e1) * 1e3)
    return float(np.median(times))


def _stage(name, us, nbytes=None, calls=1, note=None):
    s = {"stage": name, "us": us, "calls": calls}
    if nbytes is not None:
        s["bytes"] = int(nbytes)
        s["GBps"] = nbytes / us / 1e3
    if note:
        s["note"] = note
    return s


def sparse(a, torch, api, synth):
    """Sparse linear SVM: n rows, d = 2^20 columns, about 100 entries per row, pools of 65,536."""
    n, d, P = a.n or 2_000_000, 1 << 20, 65536
    rowptr, col, val, y, _ = synth.sparse_svm(n=n, d=d, threads=a.threads)
    F = api.Features.csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda(),
                         torch.from_numpy(val).cuda(), d)
    yd = torch.from_numpy(y).cuda()
    perm = torch.from_numpy(synth.epoch_permutation(n, seed=7, epoch=0)).cuda()
    ws = api.Workspace(P, d)
    w, phi, b = (torch.zeros(d, device="cuda"), torch.zeros(d, device="cuda"),
                 torch.zeros(1, device="cuda"))
    T = torch.zeros(1, device="cuda")
    prob = torch.zeros(P, device="cuda")
    steps = n // P
    nnz_pool = float(rowptr[-1]) / n * P
    tu = torch.zeros(1, dtype=torch.int32, device="cuda")
    hist = torch.zeros(steps, dtype=torch.int32, device="cuda")
    cfg = api.step_config(0.1, 1e-4, 1.0, 0.1, 0.0, 42, 0, T)

    def reset():
        w.zero_(), phi.zero_(), b.zero_(), tu.zero_()

    def epoch():   # one call: every step's batch in the workspace, step size 1 / sqrt(t) on the device
        api.train_epoch(F, yd, perm, steps * P, P, w, phi, b, cfg, tu, hist, ws)

    def score():
        for t in range(steps):
            api.assistant_score(F, perm[t * P:(t + 1) * P], P, phi, b, None, prob)

    us_step = _timed(torch, epoch, a.repeats, reset) / steps
    us_score = _timed(torch, score, a.repeats) / steps
    row_bytes = nnz_pool * 8 + P * (16 + 4)          # col + val per entry, row pointers, pool id
    return {"workload": f"sparse linear SVM n={n} d=2^20 nnz/row~{rowptr[-1] / n:.0f}, pool {P}, "
                        f"{steps} pools per epoch",
            "candidates_per_s": P / us_step * 1e6, "keep_rate": float(hist.sum().item()) / (steps * P),
            "stages": [_stage("fused step (score, keep, compact, SVM step, Assistant update)", us_step,
                              row_bytes, note="bound by the latency of the cold-column gathers, not by HBM"),
                       _stage("assistant score only", us_score, row_bytes)]}


def images(a, torch, api, synth):
    """Image batch generator: 65,536 candidates, 512 Assistant features, 150,528-byte images,
    batches of 256, labels "loss above the running median"."""
    P, d, row_bytes, B = a.n or 65536, 512, 3 * 224 * 224, 256
    feats = torch.from_numpy(synth.assistant_features(P, d)).cuda()
    store = synth.image_store_device(P, row_bytes)
    F = api.Features.dense(feats)
    ws = api.Workspace(P, d)
    r = np.random.default_rng(3)
    phi0 = torch.from_numpy((r.standard_normal(d) / np.sqrt(d)).astype(np.float32)).cuda()
    idx = torch.from_numpy(r.permutation(P).astype(np.int32)).cuda()
    phi, b = phi0.clone(), torch.zeros(1, device="cuda")
    prob = torch.zeros(P, device="cuda")
    keep = torch.zeros(P, dtype=torch.uint8, device="cuda")
    pos = torch.zeros(P, dtype=torch.int32, device="cuda")
    ids = torch.zeros(P, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    batches = torch.empty((P, row_bytes), dtype=torch.uint8, device="cuda")
    T, init = torch.zeros(1, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda")

    def score():
        api.score_shrink(F, idx, P, phi, b, 0.1, 11, 0, None, prob, keep, pos, cnt, ws)

    def gather():
        api.gather(store, row_bytes, idx, pos, cnt, P, batches, ids)

    us_score = _timed(torch, score, a.repeats)
    m = int(cnt.item())
    us_gather = _timed(torch, gather, a.repeats)
    nb = (m + B - 1) // B
    losses = [torch.from_numpy(synth.gamma_losses(min(B, m - i * B), 2.0, 0.5, batch=i)).cuda()
              for i in range(nb)]
    sizes = [torch.tensor([min(B, m - i * B)], dtype=torch.int32, device="cuda") for i in range(nb)]

    def updates():
        for i in range(nb):
            api.threshold_update(losses[i], sizes[i], B, 0.9, T, init)
            api.assistant_update(F, ids[i * B:], sizes[i], B, losses[i], T, phi, b, 0.05, 0.0, ws)

    def updates_one_call():   # the same two steps per batch in one call: two launches, not three
        for i in range(nb):
            api.threshold_assistant_update(F, ids[i * B:], sizes[i], B, losses[i], 0.9, T, init, phi, b,
                                           0.05, 0.0, ws)

    reset = lambda: (phi.copy_(phi0), b.zero_(), init.zero_())
    us_upd = _timed(torch, updates, a.repeats, reset)

    def as_graph(fn):   # the same sequence of launches replayed as one hipGraph
        reset()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fn()
        return _timed(torch, graph.replay, a.repeats, reset)

    us_upd_graph = as_graph(updates)
    phi_two = phi.clone()
    us_one = _timed(torch, updates_one_call, a.repeats, reset)
    us_one_graph = as_graph(updates_one_call)
    assert torch.equal(phi, phi_two), "the one-call form must reproduce the two calls bit for bit"
    total = us_score + us_gather + us_one_graph
    return {"workload": f"image batch generator P={P} d={d} image {row_bytes} B, batches of {B}",
            "kept": m, "images_per_s": m / total * 1e6, "candidates_per_s": P / total * 1e6,
            "stages": [_stage("score + keep + compact", us_score, P * (4 * d + 4 + 1 + 4) + 4 * m),
                       _stage("gather kept images", us_gather, 2 * m * row_bytes + 12 * m),
                       _stage("running median + Assistant update, per batch", us_upd / nb,
                              B * (4 * d + 4 + 4), calls=nb, note="eager launches"),
                       _stage("the same, all batches replayed as one hipGraph", us_upd_graph / nb,
                              B * (4 * d + 4 + 4), calls=nb, note="launch-latency bound"),
                       _stage("the same as one call per batch (aa_threshold_assistant_update)",
                              us_one / nb, B * (4 * d + 4 + 4), calls=nb, note="eager launches"),
                       _stage("the one-call form, all batches replayed as one hipGraph",
                              us_one_graph / nb, B * (4 * d + 4 + 4), calls=nb,
                              note="two dependent launches per batch")]}


def translation(a, torch, api, synth):
    """Translation batch generator: sentence pairs as token lists, kept pairs compacted into
    length-bucketed batches of 4,096 padded tokens."""
    n, vocab = a.n or 1_000_000, 32_000
    rowptr, col, val, len_s, len_t, d = synth.sentence_pairs(n=n, vocab=vocab)
    F = api.Features.csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda(),
                         None if val is None else torch.from_numpy(val).cuda(), d)
    ws = api.Workspace(n, d)
    r = np.random.default_rng(4)
    phi0 = torch.from_numpy((0.05 * r.standard_normal(d)).astype(np.float32)).cuda()
    phi, b = phi0.clone(), torch.full((1,), -0.2, device="cuda")
    prob = torch.zeros(n, device="cuda")
    keep = torch.zeros(n, dtype=torch.uint8, device="cuda")
    pos = torch.zeros(n, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    ls, lt = torch.from_numpy(len_s).cuda(), torch.from_numpy(len_t).cuda()
    ls_k, lt_k = torch.zeros_like(ls), torch.zeros_like(lt)
    order = torch.zeros(n, dtype=torch.int32, device="cuda")
    batch_of = torch.zeros(n, dtype=torch.int32, device="cuda")
    start = torch.zeros(17, dtype=torch.int32, device="cuda")
    nb = torch.zeros(1, dtype=torch.int32, device="cuda")
    nnz = int(rowptr[-1])
    out_ptr = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
    out_col = torch.zeros(nnz, dtype=torch.int32, device="cuda")
    out_val = None if val is None else torch.zeros(nnz, device="cuda")

    def score():
        api.score_shrink(F, None, n, phi, b, 0.1, 21, 0, None, prob, keep, pos, cnt, ws)

    def lens():
        api.gather(ls, 4, None, pos, cnt, n, ls_k, None)
        api.gather(lt, 4, None, pos, cnt, n, lt_k, None)

    def bucket():
        api.bucket_batches(ls_k, lt_k, cnt, n, 8, 16, 4096, order, start, batch_of, nb, ws)

    def gather_rows():
        api.gather_csr(F, None, pos, cnt, n, out_ptr, out_col, out_val, nnz, ws)

    us_score = _timed(torch, score, a.repeats)
    m = int(cnt.item())
    us_lens = _timed(torch, lens, a.repeats)
    us_bucket = _timed(torch, bucket, a.repeats)
    us_rows = _timed(torch, gather_rows, a.repeats)
    loss = torch.from_numpy(synth.gamma_losses(m, 2.0, 1.0, batch=7)).cuda()
    Tt = torch.full((1,), 1.7, device="cuda")

    def update():
        api.assistant_update(F, pos, cnt, n, loss, Tt, phi, b, 0.5, 0.0, ws)

    us_upd = _timed(torch, update, a.repeats, lambda: (phi.copy_(phi0), b.fill_(-0.2)))
    entry = 4 if val is None else 8
    kept_nnz = nnz * m / n
    total = us_score + us_lens + us_bucket + us_rows + us_upd
    return {"workload": f"translation batch generator {n} pairs, vocab {vocab}, d={d}, "
                        f"{nnz / n:.1f} entries per pair",
            "kept": m, "batches": int(nb.item()), "pairs_per_s": n / total * 1e6,
            "stages": [_stage("score + keep + compact", us_score, nnz * entry + n * (8 + 4 + 1) + 4 * m),
                       _stage("gather lengths of kept pairs", us_lens, m * (4 + 8) * 2),
                       _stage("length-bucketed batches", us_bucket, m * (8 + 4 + 4 + 4)),
                       _stage("compacted CSR of kept pairs", us_rows, 2 * kept_nnz * entry + m * 20),
                       _stage("Assistant update over kept pairs", us_upd, kept_nnz * entry + m * 16,
                              note="latency-bound: no unit is busy more than 40 % of the time")]}


def _dense_job(a, torch, api, synth):
    n, d, P = a.n or 1_000_000, 1024, 16384
    X, y, _ = synth.dense_svm(n=n, d=d, threads=a.threads)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    perm = torch.from_numpy(synth.epoch_permutation(n, seed=7, epoch=0)).cuda()
    return n, d, P, api.Features.dense(Xd), Xd, yd, perm


def sk(a, torch, api, synth):
    """Hard-threshold shrinking (keep a candidate when its own hinge loss exceeds T = 0) on
    the dense linear-SVM configuration: one pass per pool, no Assistant."""
    n, d, P, F, Xd, yd, perm = _dense_job(a, torch, api, synth)
    ws = api.Workspace(P, d)
    w = torch.zeros(d, device="cuda")
    T = torch.zeros(1, device="cuda")
    steps = (n + P - 1) // P
    tu = torch.zeros(1, dtype=torch.int32, device="cuda")
    kept = torch.zeros(steps, dtype=torch.int32, device="cuda")

    def epoch():
        api.sk_epoch(F, yd, perm, n, P, w, T, 1e-4, 256.0, tu, kept, ws)

    us = _timed(torch, epoch, a.repeats, lambda: (w.zero_(), tu.zero_())) / steps
    return {"workload": f"hard-threshold shrinking, dense n={n} d={d}, pool {P}",
            "candidates_per_s": n / steps / us * 1e6, "keep_rate": float(kept.sum().item()) / n,
            "stages": [_stage("SK step (losses, keep, compact, SVM step)", us, n / steps * (4 * d + 4 + 4 + 1 + 4))]}


def stale(a, torch, api, synth):
    """The two-stream Boss / Assistant pipeline against the fused synchronous epoch."""
    n, d, P, F, Xd, yd, perm = _dense_job(a, torch, api, synth)
    steps = (n + P - 1) // P
    T = torch.zeros(1, device="cuda")
    cfg = api.step_config(0.1, 1e-4, 1.0, 0.1, 0.0, 42, 0, T)
    w, phi, b = (torch.zeros(d, device="cuda"), torch.zeros(d, device="cuda"),
                 torch.zeros(1, device="cuda"))
    tu = torch.zeros(1, dtype=torch.int32, device="cuda")
    hist = torch.zeros(steps, dtype=torch.int32, device="cuda")

    def reset():
        w.zero_(), phi.zero_(), b.zero_(), tu.zero_()

    ws0 = api.Workspace(P, d)
    stages = []
    us = _timed(torch, lambda: api.train_epoch(F, yd, perm, n, P, w, phi, b, cfg, tu, hist, ws0),
                a.repeats, reset) / steps
    stages.append(_stage("fused synchronous epoch, per step", us, P * (4 * d + 9),
                         note=f"keep rate {float(hist.sum().item()) / n:.3f}"))
    gen = torch.cuda.Stream()
    for k in (0, 1, 2, 3):
        ws = api.Workspace(P, d, staleness=k)
        us = _timed(torch, lambda: api.train_epoch_stale(F, yd, perm, n, P, k, w, phi, b, cfg, tu,
                                                          hist, None, ws, gen), a.repeats, reset) / steps
        rho = float(hist.sum().item()) / n
        stages.append(_stage(f"two-stream pipeline, staleness {k}, per step", us,
                             P * (4 * d + 9) + rho * P * (4 * d + 12), note=f"keep rate {rho:.3f}"))
    return {"workload": f"dense n={n} d={d}, pool {P}: synchronous step against the stale pipeline",
            "stages": stages}


def rho(a, torch, api, synth):
    """Fixed keep rates on the dense configuration: phi = 0 and lr_a = 0 hold every keep
    probability at sigmoid(b), gamma = 0, so the keep rate is set by the bias alone and the
    step time is decoupled from the learning dynamics."""
    n, d, P, F, Xd, yd, perm = _dense_job(a, torch, api, synth)
    steps = (n + P - 1) // P
    T = torch.zeros(1, device="cuda")
    w, phi, b = (torch.zeros(d, device="cuda"), torch.zeros(d, device="cuda"),
                 torch.zeros(1, device="cuda"))
    tu = torch.zeros(1, dtype=torch.int32, device="cuda")
    hist = torch.zeros(steps, dtype=torch.int32, device="cuda")
    ws = api.Workspace(P, d)
    cfg = api.step_config(0.0, 1e-4, 1.0, 0.0, 0.0, 42, 0, T)
    stages = []
    for target in (0.1, 0.25, 0.5, 1.0):
        bias = 40.0 if target >= 1.0 else float(np.log(target / (1.0 - target)))

        def reset():
            w.zero_(), phi.zero_(), tu.zero_(), b.fill_(bias)

        reset()
        g = torch.cuda.CUDAGraph()
        api.train_epoch(F, yd, perm, n, P, w, phi, b, cfg, tu, hist, ws)    # loads the kernels
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            api.train_epoch(F, yd, perm, n, P, w, phi, b, cfg, tu, hist, ws)
        us = _timed(torch, g.replay, a.repeats, reset) / steps
        kept = float(hist.sum().item()) / n
        stages.append(_stage(f"fused step at keep probability {target}", us, P * (4 * d + 9) + 4 * kept * P,
                             note=f"measured keep rate {kept:.3f}, {P / us:.0f} M candidates/s"))
    return {"workload": f"dense n={n} d={d}, pool {P}: fused step at fixed keep rates (hipGraph replay of one epoch)",
            "stages": stages}


def score(a, torch, api, synth):
    """The scoring pass (a1) and the fused score + keep + compact (a7) on the dense configuration
    at growing pool sizes: these calls depend on no earlier step, so a caller may score many
    pools at once, and a larger launch streams closer to the HBM peak."""
    n, d, P, F, Xd, yd, perm = _dense_job(a, torch, api, synth)
    phi = torch.from_numpy((np.random.default_rng(5).standard_normal(d) / 32).astype(np.float32)).cuda()
    b = torch.zeros(1, device="cuda")
    stages = []
    for pool in (16384, 65536, 262144, 983040):
        pool = min(pool, n)
        prob = torch.zeros(pool, device="cuda")
        keep = torch.zeros(pool, dtype=torch.uint8, device="cuda")
        pos = torch.zeros(pool, dtype=torch.int32, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws = api.Workspace(pool, d)
        calls = max(1, min(n // pool, 16))

        def run_score():
            for t in range(calls):
                api.assistant_score(F, perm[t * pool:(t + 1) * pool], pool, phi, b, None, prob)

        def run_fused():
            for t in range(calls):
                api.score_shrink(F, perm[t * pool:(t + 1) * pool], pool, phi, b, 0.1, 42, t, None, prob,
                                 keep, pos, cnt, ws)

        us = _timed(torch, run_score, a.repeats) / calls
        stages.append(_stage(f"assistant score, pool of {pool}", us, pool * (4 * d + 4 + 4), calls=calls))
        us = _timed(torch, run_fused, a.repeats) / calls
        m = int(cnt.item())
        stages.append(_stage(f"score + keep + compact, pool of {pool}", us,
                             pool * (4 * d + 4 + 4 + 1) + pool + 4 * m, calls=calls))
        # the whole step with pools of this size (one aa_train_epoch call over calls * pool rows)
        w, ph, bb = (torch.zeros(d, device="cuda"), torch.zeros(d, device="cuda"),
                     torch.zeros(1, device="cuda"))
        T = torch.zeros(1, device="cuda")
        tu = torch.zeros(1, dtype=torch.int32, device="cuda")
        hist = torch.zeros(calls, dtype=torch.int32, device="cuda")
        cfg = api.step_config(0.1, 1e-4, 256.0, 0.1, 0.0, 42, 0, T)
        us = _timed(torch, lambda: api.train_epoch(F, yd, perm, calls * pool, pool, w, ph, bb, cfg, tu,
                                                   hist, ws),
                    a.repeats, lambda: (w.zero_(), ph.zero_(), bb.zero_(), tu.zero_())) / calls
        rate = float(hist.sum().item()) / (calls * pool)
        stages.append(_stage(f"whole step (aa_train_epoch), pool of {pool}", us,
                             pool * (4 * d + 9) + 4 * rate * pool, calls=calls,
                             note=f"keep rate {rate:.2f}, {pool / us:.0f} M candidates/s"))
    return {"workload": f"dense n={n} d={d}: scoring at pool sizes 16,384 to 983,040 (random rows)",
            "stages": stages}


WORKLOADS = {"rho": rho, "sparse": sparse, "images": images, "translation": translation, "sk": sk,
             "stale": stale, "score": score}


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawTextHelpFormatter)
    ap.add_argument("workload", choices=sorted(WORKLOADS))
    ap.add_argument("--n", type=int, default=0, help="rows / candidates / pairs (0: the full size)")
    ap.add_argument("--repeats", type=int, default=5)
    ap.add_argument("--threads", type=int, default=16, help="host threads of the data generator")
    a = ap.parse_args(argv)
    import torch

    from . import api, synth
    api.lib()   # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    t0 = time.time()
    out = WORKLOADS[a.workload](a, torch, api, synth)
    out["wall_s"] = time.time() - t0
    out["data"] = "synthetic"
    print(json.dumps(out))


if __name__ == "__main__":
    main(sys.argv[1:])
