"""Build the HIP library in-tree: python -m paper_2302_02407_amd.build [--incremental]"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhe_mi355x.so")
SOURCES = ["ctx.hip", "ntt.hip", "ntt16.hip", "elementwise.hip", "keyswitch.hip", "conv2d.hip", "noalloc.hip", "smallring.hip"]
HEADERS = ["he_internal.h", "modarith.h", "ntt_blocks.h", os.path.join("..", "..", "include", "he_mi355x.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out:
        print(out)


def source_hash() -> str:
    """sha256 over the library's sources and headers (the build identifier compiled into the library)."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(SOURCES) + sorted(HEADERS):
        with open(os.path.join(CSRC, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def build_library(verbose: bool = True, incremental: bool = False) -> str:
    """Compile every HIP source for gfx950 (one object per source, in parallel) and link them into one
    shared library next to this file.  incremental=True skips objects newer than their source and the
    headers."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(os.path.join(CSRC, h)) for h in HEADERS)
    jobs = []
    build_id = source_hash()
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        if incremental and s != "ctx.hip" and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        extra = ['-DHE_BUILD_ID="%s"' % build_id] if s == "ctx.hip" else []
        jobs.append([hipcc] + FLAGS + extra + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=8) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + [os.path.join(OBJ, s + ".o") for s in SOURCES]
         + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    build_library(incremental="--incremental" in sys.argv[1:])
    sys.exit(0)
