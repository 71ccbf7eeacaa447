"""Build librh.so (the HIP library) in-tree with hipcc for gfx950.

Every source is compiled to an object of its own (in parallel, objects kept under _build/ and
reused while the source, the headers and the flags are unchanged), then linked."""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(HERE, "..", "include")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librh.so")
STAMP = LIB + ".sources"      # digest of the sources the library was built from
SOURCES = ["rh_api.hip", "select.hip", "plan.hip", "pack.hip", "unpack.hip", "conv_fp32.hip", "conv_mfma.hip",
           "conv_mfma_duo.hip", "conv_tail.hip", "conv_head.hip", "conv_fold.hip", "conv_mask.hip", "temporal.hip", "noalloc.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-ffp-contract=off"]


def _digest(paths, extra: str = "") -> str:
    h = hashlib.sha256(extra.encode())
    for p in paths:
        h.update(os.path.basename(p).encode())
        with open(p, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def _headers():
    return sorted(os.path.join(d, n) for d in (CSRC, INCLUDE) for n in os.listdir(d) if n.endswith(".h"))


def source_digest() -> str:
    """SHA-256 over the names and contents of every file the library is compiled from."""
    return _digest([os.path.join(CSRC, s) for s in SOURCES] + _headers(), " ".join(FLAGS))


def _compile(hipcc: str, src: str, force: bool):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    tag = _digest([os.path.join(CSRC, src)] + _headers(), " ".join(FLAGS))
    if not force and os.path.exists(obj) and os.path.exists(obj + ".tag") and open(obj + ".tag").read() == tag:
        return obj, ""
    cmd = [hipcc] + FLAGS + ["-I" + INCLUDE, "-I" + CSRC, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}{r.stderr}")
    with open(obj + ".tag", "w") as f:
        f.write(tag)
    return obj, r.stdout + r.stderr


def build(verbose: bool = False, force: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    jobs = min(8, int(os.environ.get("MAX_JOBS", "8")), len(SOURCES))
    with ThreadPoolExecutor(jobs) as ex:
        res = list(ex.map(lambda s: _compile(hipcc, s, force), SOURCES))
    if verbose:
        sys.stderr.write("".join(log for _, log in res))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [o for o, _ in res],
                       capture_output=True, text=True)
    if verbose or r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed linking librh.so")
    with open(STAMP, "w") as f:
        f.write(source_digest() + "\n")
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, force="--force" in sys.argv))
