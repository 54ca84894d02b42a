"""Compile the HIP sources under csrc/ into paper_2503_16163_amd/libspecache.so for gfx950."""
import hashlib
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libspecache.so")
STAMP = os.path.join(HERE, "libspecache.srchash")   # hash of the sources the library was built from
SOURCES = ["specache.hip", "quant.hip", "score.hip", "score_mfma.hip", "score_i8.hip", "select.hip", "topk.hip", "gather.hip", "attend.hip", "attend_i8.hip", "fourbit.hip", "measure.hip"]
# -ffp-contract=off: the quantiser's binary32 operation order is part of its definition and
# fused multiply-adds are written out where they are wanted.  Packed FP32 code generation is
# switched off for the device pass.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Wall",
         "-Wno-unused-result", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    r = subprocess.run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj],
                       capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    return obj, err


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        results = list(ex.map(_compile, SOURCES))
    if verbose:
        for _, err in results:
            if err.strip():
                print(err)
    objs = [o for o, _ in results]
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    with open(STAMP, "w") as f:
        f.write(source_hash())
    return LIB


def source_hash():
    """sha256 over the HIP sources, their headers and the C ABI header (names and contents)."""
    h = hashlib.sha256()
    deps = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC)) + [os.path.join(HERE, "..", "include", "specache.h")]
    for d in deps:
        h.update(os.path.basename(d).encode())
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def kernel_sources(kernel):
    """The .hip file that defines __global__ `kernel` and every header it includes, directly or not
    (base names, sorted); None if no source defines it."""
    import re
    pat = re.compile(r"__global__[^;{]*?\b" + re.escape(kernel) + r"\s*\(", re.S)
    for f in sorted(os.listdir(CSRC)):
        if not f.endswith(".hip"):
            continue
        with open(os.path.join(CSRC, f)) as fh:
            if not pat.search(fh.read()):
                continue
        seen, todo = set(), [os.path.join(CSRC, f)]
        while todo:
            path = os.path.normpath(todo.pop())
            if path in seen or not os.path.exists(path):
                continue
            seen.add(path)
            with open(path) as fh:
                for inc in re.findall(r'#include\s+"([^"]+)"', fh.read()):
                    todo.append(os.path.join(os.path.dirname(path), inc))
        return sorted(seen)
    return None


def kernel_source_hash(kernel):
    """sha256 over the sources one kernel is compiled from (kernel_sources), so that a figure measured on a
    kernel stays attributable to it while other kernels change; None for an unknown kernel."""
    files = kernel_sources(kernel)
    if files is None:
        return None
    h = hashlib.sha256()
    for path in files:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_built():
    """True when libspecache.so exists and was built from the sources as they are now (by content, so that
    a copy of the tree to another machine does not look stale)."""
    if not (os.path.exists(LIB) and os.path.exists(STAMP)):
        return False
    with open(STAMP) as f:
        return f.read().strip() == source_hash()


if __name__ == "__main__":
    print(build(verbose=True))
