"""Build libindexcache.so (hand-written HIP for gfx950) in-tree with hipcc.

Every source is compiled to an object file of its own (in parallel) under _build/, then linked.
`build()` recompiles everything; `build(incremental=True)` skips objects that are newer than their
source and every header.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
OUT = os.path.join(HERE, "libindexcache.so")
SOURCES = ["ic_api.hip", "ic_indexer_score.hip", "ic_topk_select.hip", "ic_sparse_attn.hip",
           "ic_overlap.hip", "ic_similarity.hip", "ic_distill.hip", "ic_calibrate.hip"]
HEADERS = [os.path.join(CSRC, "ic_common.hpp"), os.path.join(ROOT, "include", "indexcache.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 feature flag and says so once per file: harmless noise
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if out.strip():
        print(out, flush=True)
    if p.returncode != 0:
        raise subprocess.CalledProcessError(p.returncode, cmd)


def compile_objects(verbose: bool = False, extra=(), incremental: bool = False, tag: str = "", jobs: int = 8):
    """Compile every source to _build/<source><tag>.o (in parallel); returns the object paths."""
    os.makedirs(OBJ, exist_ok=True)
    newest_hdr = max(os.path.getmtime(h) for h in HEADERS)
    work = []
    objs = []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJ, s + tag + ".o")
        objs.append(obj)
        fresh = os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(src), newest_hdr)
        if not (incremental and fresh):
            work.append(["hipcc"] + FLAGS + list(extra) + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(work) or 1))) as ex:
        list(ex.map(lambda c: _run(c, verbose), work))
    return objs


def build(verbose: bool = False, extra=(), incremental: bool = False, out: str = OUT, jobs: int = 8) -> str:
    objs = compile_objects(verbose, extra, incremental, "" if out == OUT else "." + os.path.basename(out), jobs)
    _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC"] + list(extra) + objs + ["-o", out], verbose)
    return out


if __name__ == "__main__":
    inc = "--incremental" in sys.argv[1:]
    print(build(verbose=True, extra=[a for a in sys.argv[1:] if a != "--incremental"], incremental=inc))
