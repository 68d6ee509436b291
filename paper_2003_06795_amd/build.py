"""Build libks_gemm.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2003_06795_amd.build [--force] [-j N] [--kept-only]

--kept-only builds libks_gemm_kept.so, the pruned library: only the members the deployed trees can
return (csrc/kept_set.inc) and the four bring-up tiles are compiled; everything else of the C ABI
is the same.  The full library is what the tuner and the tests use.

The kernel family is compiled as shards of one source (-DKS_SHARD=n) so that the 64 fp32 and the
bf16 instantiations build in parallel.  Objects go to _build/ (not tracked); the library lands
next to this file.
"""
import argparse
import concurrent.futures as cf
import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libks_gemm.so")
SHARDS = 16

HIPCC = os.environ.get("HIPCC", "hipcc")
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
CXX_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra"]


def _deps():
    return (glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(CSRC, "*.def"))
            + glob.glob(os.path.join(CSRC, "*.inc")) + glob.glob(os.path.join(ROOT, "include", "*.h")))


LIB_KEPT = os.path.join(PKG, "libks_gemm_kept.so")


def _jobs(kept_only=False):
    obj = os.path.join(OBJ, "kept") if kept_only else OBJ
    extra = ["-DKS_KEPT_ONLY"] if kept_only else []
    jobs = []
    for n in range(SHARDS):
        for kind in ("f32", "bf16", "bf16_dma"):
            src = os.path.join(CSRC, "instances_%s.hip" % kind)
            jobs.append((src, os.path.join(obj, "inst_%s_%02d.o" % (kind, n)),
                         [HIPCC] + HIP_FLAGS + extra + ["-DKS_SHARD=%d" % n, "-c", src]))
    for name in ("dispatch", "measure"):
        src = os.path.join(CSRC, name + ".hip")
        jobs.append((src, os.path.join(obj, name + ".o"), [HIPCC] + HIP_FLAGS + extra + ["-c", src]))
    for name in ("selector", "tune"):
        src = os.path.join(CSRC, name + ".cpp")
        jobs.append((src, os.path.join(obj, name + ".o"), ["g++"] + CXX_FLAGS + ["-c", src]))
    return jobs


def _compile(job):
    src, obj, cmd = job
    r = subprocess.run(cmd + ["-o", obj], capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    return obj, r.returncode, err


def build(force=False, jobs=None, verbose=True, kept_only=False):
    lib = LIB_KEPT if kept_only else LIB
    os.makedirs(os.path.join(OBJ, "kept") if kept_only else OBJ, exist_ok=True)
    newest_dep = max(os.path.getmtime(p) for p in _deps())
    todo, objs = [], []
    for job in _jobs(kept_only):
        src, obj, _ = job
        objs.append(obj)
        stale = (force or not os.path.exists(obj)
                 or os.path.getmtime(obj) < max(newest_dep, os.path.getmtime(src)))
        if stale:
            todo.append(job)
    jobs = jobs or min(8, os.cpu_count() or 1)
    if todo:
        if verbose:
            print("[build] compiling %d objects with %d jobs" % (len(todo), jobs), flush=True)
        with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
            for obj, rc, err in ex.map(_compile, todo):
                if err.strip() and verbose:
                    print(err, file=sys.stderr)
                if rc != 0:
                    raise RuntimeError("compile failed: %s\n%s" % (obj, err))
    if todo or not os.path.exists(lib):
        tmp = lib + ".tmp.%d" % os.getpid()
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs, check=True)
        os.replace(tmp, lib)
        if verbose:
            print("[build] linked %s (%.1f MB)" % (lib, os.path.getsize(lib) / 1e6), flush=True)
    return lib


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--force", action="store_true")
    ap.add_argument("-j", type=int, default=None)
    ap.add_argument("--kept-only", action="store_true", help="build the pruned library libks_gemm_kept.so")
    a = ap.parse_args()
    import time
    t0 = time.time()
    build(force=a.force, jobs=a.j, kept_only=a.kept_only)
    print("[build] %.0f s" % (time.time() - t0))
