"""Per-wave phase time stamps of the whole-step dense pass (measurement tool).

Loads libautoassist_trace.so (the library built with -DAA_PHASE_TRACE, see build.py), runs
one epoch slice of the dense configuration (n = 1,000,000, d = 1024, pools of 16,384) through
aa_train_epoch and prints, for the last step, when each phase was reached: mean / min / max
over all waves, in microseconds from the first wave's entry (10 ns clock).

    python -m paper_1905_03381_amd.phase_trace [--steps 40] [--lr0 256]

The rows are unit-norm Gaussian rows drawn on the GPU (same shape and distribution as the
bench workload, not the same bytes): only timing is looked at here.
"""
import argparse
import ctypes as C
import os

import numpy as np
import torch

from . import api

NAMES = ["entry", "ids, model, scalars, carried flags there", "past the start-up barrier",
         "rows requested, draws made", "first row used", "all rows consumed",
         "past the reduction barrier", "partials stored"]
STAMPS = 8


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--lr0", type=float, default=256.0)
    ap.add_argument("--waves", type=int, default=8, help="waves per block of the pass at d = 1024")
    a = ap.parse_args()
    here = os.path.dirname(os.path.abspath(__file__))
    api.LIB_PATH = os.path.join(here, "libautoassist_trace.so")
    L = api.lib()
    L.aa_phase_trace_buffer.argtypes = [C.c_void_p]
    L.aa_phase_trace_buffer.restype = C.c_int32
    torch.manual_seed(0)
    n, d, P = 1_000_000, 1024, 16384
    X = torch.randn(n, d, device="cuda")
    X /= X.norm(dim=1, keepdim=True)
    y = torch.where(X @ torch.randn(d, device="cuda") >= 0, 1.0, -1.0).float()
    perm = torch.randperm(n, device="cuda").to(torch.int32)
    F = api.Features.dense(X)
    ws = api.Workspace(P, d)
    w, phi, b = (torch.zeros(d, device="cuda"), torch.zeros(d, device="cuda"), torch.zeros(1, device="cuda"))
    T = torch.zeros(1, device="cuda")
    tu = torch.zeros(1, dtype=torch.int32, device="cuda")
    hist = torch.zeros(a.steps, dtype=torch.int32, device="cuda")
    cfg = api.step_config(0.1, 1e-4, a.lr0, 0.1, 0.0, 42, 0, T)
    nblk = torch.cuda.get_device_properties(0).multi_processor_count
    trace = torch.zeros(nblk * a.waves * STAMPS, dtype=torch.int64, device="cuda")
    L.aa_phase_trace_buffer(trace.data_ptr())
    api.train_epoch(F, y, perm, a.steps * P, P, w, phi, b, cfg, tu, hist, ws)
    torch.cuda.synchronize()
    L.aa_phase_trace_buffer(None)
    tr = trace.cpu().numpy().reshape(nblk, a.waves, STAMPS).astype(np.int64)
    assert (tr[..., 0] > 0).all(), "no stamps: is this the trace build, and --waves right?"
    rel = (tr - tr[..., 0].min()) * 0.01
    print(f"k_step_pass, step {a.steps - 1} of an eager aa_train_epoch call: {nblk} blocks x {a.waves} waves, "
          f"kept {int(hist[-1])} of {P}")
    print(f"{'phase':44s} {'mean':>7s} {'min':>7s} {'max':>7s}   (us after the first wave's entry)")
    for k, name in enumerate(NAMES):
        v = rel[..., k]
        print(f"{k} {name:42s} {v.mean():7.2f} {v.min():7.2f} {v.max():7.2f}")
    end = rel[..., STAMPS - 1].max(axis=1)
    print(f"last wave of a block done: mean {end.mean():.2f}, earliest block {end.min():.2f}, latest {end.max():.2f}")
    print("mean block end per XCD (block b runs on XCD b mod 8):",
          " ".join(f"{end[x::8].mean():.2f}" for x in range(8)))


if __name__ == "__main__":
    main()
