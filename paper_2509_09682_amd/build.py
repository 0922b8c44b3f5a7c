"""Compile the HIP sources under csrc/ into paper_2509_09682_amd/libcce_neg.so for gfx950."""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import tempfile

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcce_neg.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-munsafe-fp-atomics",
    # packed fp32 VALU forms are switched off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _hipcc(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 target feature; that is harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    return err


def build(verbose: bool = False) -> str:
    """Compiles every source to an object of its own (in parallel: the matrix-core file takes most of the time) and
    links them.  Objects live in a temporary directory; only the library stays in the tree."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="cce_build_") as tmp:
        jobs = [(src, os.path.join(tmp, os.path.basename(src) + ".o")) for src in sources()]
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(len(jobs), 8)) as pool:
            notes = list(pool.map(lambda j: _hipcc([hipcc, *flags, *inc, "-c", j[0], "-o", j[1]]), jobs))
        notes.append(_hipcc([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[o for _, o in jobs], "-o", LIB]))
    if verbose:
        for n in notes:
            if n.strip():
                print(n)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
