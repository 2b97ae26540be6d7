"""Build libssmv.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libssmv.so")
SOURCES = ["api.hip", "aux_kernels.hip", "verify_scalar.hip", "verify_diag.hip", "verify_mfma.hip", "prefill.hip", "prefill_bf16.hip"]
HEADERS = [os.path.join(CSRC, "ssmv_internal.h"), os.path.join(CSRC, "verify_impl.h"),
           os.path.join(ROOT, "include", "ssmv.h")]

# packed-fp32 VALU forms are switched off for every device compile of this library
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-variable",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# verify_mfma.hip: the first 14 dwords of kernel arguments (seven pointers its first scalar loads go through) are handed to
# the waves in scalar registers at their start (gfx950 kernel-argument preload; where the firmware does not do it the
# compiler's prologue loads them)
EXTRA_FLAGS = {"verify_mfma.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=14"]}


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False, trace: bool = False) -> str:
    """trace=True builds libssmv_trace.so instead: the same library with -DSSMV_TRACE (per-workgroup wall-clock stamps
    inside the matrix-core verify kernel and the hook that hands it a buffer; for trace_stamps.py, not for use)."""
    obj_dir = OBJ + ("_trace" if trace else "")
    lib = os.path.join(PKG, "libssmv_trace.so") if trace else LIB
    flags = FLAGS + (["-DSSMV_TRACE"] if trace else [])
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = _hipcc()
    jobs = []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(obj_dir, s.replace(".hip", ".o"))
        if force or _stale(obj, [src] + HEADERS):
            jobs.append([hipcc] + flags + EXTRA_FLAGS.get(s, []) + ["-c", src, "-o", obj])

    def run(cmd):
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n%s\n%s" % (" ".join(cmd), r.stdout + r.stderr))
        if verbose and r.stderr.strip():
            print(r.stderr)

    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(run, jobs))
    objs = [os.path.join(obj_dir, s.replace(".hip", ".o")) for s in SOURCES]
    if force or jobs or _stale(lib, objs):
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib + ".tmp"])
        os.replace(lib + ".tmp", lib)
    return lib


if __name__ == "__main__":
    import sys
    print(build(force="--force" in sys.argv, verbose=True, trace="--trace" in sys.argv))
