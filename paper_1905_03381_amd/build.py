"""Compile the HIP kernels and the C ABI into paper_1905_03381_amd/libautoassist.so (gfx950).

hipcc cross-compiles without a GPU.  Objects go to paper_1905_03381_amd/_build/.

Two measurement artefacts are built beside the library (python -m paper_1905_03381_amd.build
--measure, also built by default): libautoassist_trace.so, the same sources with
-DAA_PHASE_TRACE (the whole-step dense pass records per-wave phase time stamps; read them with
phase_trace.py), and bare_read_probe, a stand-alone program that times kernels which only read
the rows of a pool (the reference the row passes are measured against).
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libautoassist.so")
TRACE_LIB = os.path.join(HERE, "libautoassist_trace.so")
PROBE = os.path.join(HERE, "bare_read_probe")
SOURCES = ["aa_api.hip", "aa_batching.hip", "aa_dense.hip", "aa_general.hip", "aa_select.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, verbose=False, extra_flags=(), lib=LIB, tag=""):
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "autoassist.h"))
    hipcc = _hipcc()

    def compile_one(src):
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, tag + src.replace(".hip", ".o"))
        if force or _stale(o, [s] + headers):
            cmd = [hipcc] + FLAGS + list(extra_flags) + ["-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd), flush=True)
            r = subprocess.run(cmd, capture_output=True, text=True)
            msgs = [l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l and l.strip()]
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n" + "\n".join(msgs))
            if verbose and msgs:
                print("\n".join(msgs), flush=True)
        return o

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    if force or _stale(lib, objs):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    return lib


def build_measure(force=True, verbose=False):
    """The phase-trace build of the library and the bare-read reference program."""
    build(force=force, verbose=verbose, extra_flags=("-DAA_PHASE_TRACE",), lib=TRACE_LIB, tag="trace_")
    src = os.path.join(CSRC, "bare_read_probe.hip")
    if force or _stale(PROBE, [src]):
        cmd = [_hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", src, "-o", PROBE]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("bare_read_probe failed to build:\n" + r.stdout + r.stderr)
    return TRACE_LIB, PROBE


if __name__ == "__main__":
    force = "--if-stale" not in sys.argv
    print(build(force=force, verbose=True))
    if "--no-measure" not in sys.argv:
        print(*build_measure(force=force, verbose=True))
