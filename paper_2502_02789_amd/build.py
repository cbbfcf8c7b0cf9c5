"""Builds libspecprefill.so (gfx950 only) in-tree with hipcc.

Every translation unit under csrc/ is compiled on its own (in parallel) into _build/, then the
objects are linked into the shared library next to this file."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
OBJ_DIR = os.path.join(PKG_DIR, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libspecprefill.so")
PROBE_SRC = os.path.join(PKG_DIR, "csrc_probe", "sp_probe.hip")
PROBE_LIB_PATH = os.path.join(PKG_DIR, "libspprobe.so")     # the benchmark's read-only probes, a library of its own

COMMON_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fvisibility=hidden",
    # packed fp32 VALU forms are kept off on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the kernel-argument struct is read through a by-value copy; without this the copy stays in
    # scratch memory once a kernel has more than 300 reads of it
    "-mllvm", "-instcombine-max-copied-from-constant-users=1000000",
    "-Wall", "-Wno-unused-function",
]
# no NaN canonicalisation around fmax in the DEVICE code of the scoring kernels only (NaN inputs
# are a documented precondition violation there).  Host code must still see NaNs (argument
# checks), and so must the selection kernels, which report NaN scores in band.
SCORE_DEVICE_FLAGS = ["-Xarch_device", "-fno-honor-nans"]


def _extra_flags(src):
    return SCORE_DEVICE_FLAGS if os.path.basename(src).startswith("sp_score") else []


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, flush=True)


def _headers_mtime():
    hdrs = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h")) + [__file__]
    return max(os.path.getmtime(h) for h in hdrs)


def build_library(verbose: bool = False, extra_flags=(), lib_path: str = LIB_PATH, incremental: bool = False) -> str:
    """incremental=True skips translation units whose object is newer than the source and every
    header (a developer convenience; the default recompiles everything)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    tag = os.path.splitext(os.path.basename(lib_path))[0]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    jobs, objs = [], []
    newest_header = _headers_mtime()
    for src in sources():
        obj = os.path.join(OBJ_DIR, f"{tag}.{os.path.splitext(os.path.basename(src))[0]}.o")
        objs.append(obj)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        jobs.append((obj, [hipcc, *COMMON_FLAGS, *_extra_flags(src), *extra_flags, *inc, "-c", src, "-o", obj]))
    with ThreadPoolExecutor(max_workers=8) as pool:
        list(pool.map(lambda j: _run(j[1], verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden", *objs, "-o", lib_path],
         verbose)
    return lib_path


def build_probe(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _run([hipcc, *COMMON_FLAGS, "-shared", "-I", os.path.join(ROOT, "include"), PROBE_SRC, "-o", PROBE_LIB_PATH], verbose)
    return PROBE_LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True, incremental="--incremental" in sys.argv[1:]))
    print(build_probe(verbose=True))
    sys.exit(0)
