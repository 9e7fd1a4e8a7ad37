"""Build libbed.so in-tree with hipcc for gfx950.

    python -m paper_2207_04228_amd.build [--force] [--remarks]

Each .hip translation unit is compiled to an object in parallel, then linked.
The object directory (``_build/``) is ignored by git; ``libbed.so`` lands next
to the Python binding so that it travels with the tree.
"""
from __future__ import annotations

import argparse
import concurrent.futures as cf
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbed.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # hipcc turns ordinary float code into packed-fp32 instructions on its own;
    # keep that off for this target.
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _newer(target: str, deps) -> bool:
    if not os.path.exists(target):
        return False
    t = os.path.getmtime(target)
    return all(os.path.getmtime(d) <= t for d in deps)


def source_hash() -> str:
    """sha256 over the device and host sources of libbed.so (csrc/ and include/bed.h): identifies
    the kernels a stored profile was taken from."""
    import hashlib
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.h"))
                   + glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(ROOT, "include", "*.h")))
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def build(force: bool = False, remarks: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    sources = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    headers = sorted(glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(CSRC, "*.hpp"))
                     + glob.glob(os.path.join(ROOT, "include", "*.h")))
    # a change of compiler flags rebuilds everything
    stamp = os.path.join(OBJ, "flags.txt")
    flags_now = " ".join([HIPCC] + FLAGS)
    if not os.path.exists(stamp) or open(stamp).read() != flags_now:
        force = True
    objs = []
    todo = []
    for s in sources:
        o = os.path.join(OBJ, os.path.basename(s)[:-4] + ".o")
        objs.append(o)
        if force or not _newer(o, [s] + headers):
            todo.append((s, o))

    def compile_one(so):
        s, o = so
        cmd = [HIPCC] + FLAGS + ["-c", s, "-o", o]
        if remarks:
            cmd.append("-Rpass-analysis=kernel-resource-usage")
        r = subprocess.run(cmd, capture_output=True, text=True)
        log = os.path.join(OBJ, os.path.basename(s)[:-4] + ".log")
        with open(log, "w") as f:
            f.write(r.stdout + r.stderr)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {s}:\n{r.stderr[-4000:]}")
        return o

    if todo:
        with cf.ThreadPoolExecutor(max_workers=max(1, min(jobs, len(todo)))) as ex:
            list(ex.map(compile_one, todo))
    with open(stamp, "w") as f:
        f.write(flags_now)
    if todo or force or not os.path.exists(LIB):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr[-4000:]}")
    return LIB


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--force", action="store_true")
    ap.add_argument("--remarks", action="store_true", help="write per-kernel resource usage to _build/*.log")
    ap.add_argument("-j", "--jobs", type=int, default=8)
    ap.add_argument("--source-hash", action="store_true", help="print the hash of the sources and exit")
    a = ap.parse_args(argv)
    if a.source_hash:
        print(source_hash())
        return 0
    print(build(a.force, a.remarks, a.jobs))


if __name__ == "__main__":
    sys.exit(main())
