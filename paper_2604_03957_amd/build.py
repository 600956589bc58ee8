"""Compile csrc/*.hip into csrc/libbwta.so for gfx950 with hipcc (cross-compiles without a GPU).

Each source is its own translation unit: the files are compiled side by side (up to 8 at a time)
into objects under csrc/_build/ and then linked.  Every call compiles everything again unless
`incremental=True` (a developer convenience: objects newer than their source and every header are
kept)."""
import concurrent.futures
import glob
import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(CSRC, "libbwta.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers():
    return glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))


def build_id():
    """Digest of every source and header the library is built from (and of the compiler flags)."""
    h = hashlib.sha1(" ".join(HIPCC_FLAGS).encode())
    for f in sorted(sources() + _headers(), key=os.path.basename):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:12]


def build_library(verbose=True, extra_flags=(), incremental=False, jobs=8):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    bid = build_id()
    newest_header = max(os.path.getmtime(h) for h in _headers())
    todo, objs = [], []
    for src in sources():
        obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        fresh = (incremental and not extra_flags and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header))
        if not fresh or os.path.basename(src) == "bwta_api.hip":
            todo.append((src, obj))

    def compile_one(job):
        src, obj = job
        cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-c", src, "-o", obj]
        if os.path.basename(src) == "bwta_api.hip":  # the one file that records the digest: always rebuilt
            cmd.insert(-4, '-DBWTA_BUILD_ID="%s"' % bid)
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)

    with concurrent.futures.ThreadPoolExecutor(max_workers=max(1, min(jobs, len(todo) or 1))) as pool:
        list(pool.map(compile_one, todo))
    tmp = LIB + ".tmp%d" % os.getpid()
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    flags = [a for a in sys.argv[1:] if a != "--incremental"]
    build_library(extra_flags=flags, incremental="--incremental" in sys.argv[1:])
