"""Compiles csrc/ into libdistdl.so (gfx950) next to this file.

Every source is compiled to an object of its own (in parallel), then linked.  `build()` recompiles everything;
`build(incremental=True)` (or DISTDL_INCREMENTAL=1) skips objects newer than their source and every header, which
is what an edit-compile-test loop wants."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = sorted(f for f in os.listdir(os.path.join(HERE, "csrc")) if f.endswith((".hip", ".cpp")))
LIB = os.path.join(HERE, "libdistdl.so")
OBJ_DIR = os.path.join(HERE, "_build")


def _flags():
    return ["-fPIC", "-O3", "-std=c++17", "--offload-arch=gfx950",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-result", "-Wno-unknown-warning-option",
            "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]


def _headers_mtime():
    newest = os.path.getmtime(os.path.abspath(__file__))
    for d in (os.path.join(ROOT, "include"), os.path.join(HERE, "csrc")):
        for f in os.listdir(d):
            if f.endswith(".h"):
                newest = max(newest, os.path.getmtime(os.path.join(d, f)))
    return newest


def build(verbose=True, incremental=None):
    if incremental is None:
        incremental = os.environ.get("DISTDL_INCREMENTAL", "0") == "1"
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdr = _headers_mtime()
    jobs = []
    objs = []
    for s in SOURCES:
        src = os.path.join(HERE, "csrc", s)
        obj = os.path.join(OBJ_DIR, s + ".o")
        objs.append(obj)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), hdr):
            continue
        cmd = [hipcc, "-c"] + _flags() + (["-x", "hip"] if s.endswith(".cpp") else []) + [src, "-o", obj]
        jobs.append(cmd)

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)

    workers = max(1, min(len(jobs), int(os.environ.get("MAX_JOBS", os.cpu_count() or 4)), 16))
    with ThreadPoolExecutor(workers) as pool:
        results = list(pool.map(run, jobs))
    failed = False
    for cmd, r in zip(jobs, results):
        out = "\n".join(l for l in r.stdout.splitlines() if "is not a recognized feature for this target" not in l)
        if out.strip() and (verbose or r.returncode):
            print(out, flush=True)
        failed |= r.returncode != 0
    if failed:
        raise subprocess.CalledProcessError(1, "hipcc -c")
    link = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv)
    sys.exit(0)
