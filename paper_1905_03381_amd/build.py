"""Compile the HIP kernels and the C ABI into paper_1905_03381_amd/libautoassist.so (gfx950).

hipcc cross-compiles without a GPU.  Objects go to paper_1905_03381_amd/_build/.

Two measurement artefacts are built beside the library (python -m paper_1905_03381_amd.build
--measure, also built by default; --resources prints the compiler's per-kernel register, scratch
and LDS figures of the last build): libautoassist_trace.so, the same sources with
-DAA_PHASE_TRACE (the whole-step dense pass records per-wave phase time stamps; read them with
phase_trace.py), and bare_read_probe, a stand-alone program that times kernels which only read
the rows of a pool (the reference the row passes are measured against).
"""
import json
import os
import re
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
         "-Wall", "-Wno-unused-function", "-Rpass-analysis=kernel-resource-usage"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _without_remarks(text):
    """Compiler output without the resource-usage remarks (each a remark line, and for the
    first of a kernel two lines of source context)."""
    keep, skip = [], 0
    for line in text.splitlines():
        if "-Rpass-analysis=kernel-resource-usage" in line:
            skip = 2 if "Function Name:" in line else 0
            continue
        if skip > 0 and re.match(r"\s*(\d+ \||\|)", line):
            skip -= 1
            continue
        skip = 0
        keep.append(line)
    return keep


def kernel_resources(tag=""):
    """Resource table of the last build of the library: {kernel symbol: {...}} over all sources."""
    out = {}
    for src in SOURCES:
        path = os.path.join(OBJ, tag + src.replace(".hip", ".o")) + ".resources.json"
        with open(path) as f:
            out.update(json.load(f))
    return out


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _resource_remarks(text):
    """{kernel symbol: {"vgprs", "scratch", "lds", "occupancy"}} from the compiler's
    kernel-resource-usage remarks (printed per kernel while it compiles)."""
    out, cur = {}, None
    keys = {"VGPRs": "vgprs", "ScratchSize [bytes/lane]": "scratch", "LDS Size [bytes/block]": "lds",
            "Occupancy [waves/SIMD]": "occupancy"}
    for line in text.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z /\[\]]+): (\d+) \[-Rpass-analysis", line)
        if m and cur is not None and m.group(1).strip() in keys:
            cur[keys[m.group(1).strip()]] = int(m.group(2))
    return out


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
            text = r.stdout + r.stderr
            if r.returncode != 0:
                msgs = [l for l in text.splitlines() if "packed-fp32-ops" not in l and l.strip()]
                raise RuntimeError(f"hipcc failed on {src}:\n" + "\n".join(msgs))
            # registers, scratch and LDS of every kernel, as the compiler reports them
            with open(o + ".resources.json", "w") as f:
                json.dump(_resource_remarks(text), f, indent=1, sort_keys=True)
            msgs = [l for l in _without_remarks(text) if "packed-fp32-ops" not in l and l.strip()]
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


def resource_table():
    """Markdown table of what the compiler reports per kernel of the last build."""
    table = kernel_resources()
    names = subprocess.run(["c++filt"] + list(table), capture_output=True, text=True).stdout.splitlines()
    if len(names) != len(table):
        names = list(table)
    rows = sorted(zip(names, table.values()), key=lambda t: (-t[1]["vgprs"], t[0]))
    out = ["| kernel | VGPRs | scratch bytes/lane | LDS bytes/block | waves/SIMD |", "|---|---|---|---|---|"]
    for name, v in rows:
        short = name.replace("aa::(anonymous namespace)::", "").replace("(anonymous namespace)::", "")
        short = re.sub(r"^void ", "", short)
        short = re.sub(r"\(.*\)$", "", short)
        out.append(f"| `{short}` | {v['vgprs']} | {v['scratch']} | {v['lds']} | {v['occupancy']} |")
    return "\n".join(out)


if __name__ == "__main__":
    if "--resources" in sys.argv:  # table of the last build (build first)
        print(resource_table())
        sys.exit(0)
    force = "--if-stale" not in sys.argv
    print(build(force=force, verbose=True))
    if "--no-measure" not in sys.argv:
        print(*build_measure(force=force, verbose=True))
