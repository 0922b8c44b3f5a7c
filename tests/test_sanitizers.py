"""CPU-side sanitizer builds (-fsanitize=address,undefined) of the oracle and of the library's host code.

Both programs are compiled here, into a temporary directory, and run as processes of their own: the sanitizer run-time
aborts with a report on the first out-of-bounds access, misaligned or overflowing index computation, or leak.  No GPU
and no HIP runtime is involved: the library's host code is compiled for the host alone and linked against inert
stand-ins of the few runtime entry points it names (tests/sanitize/api_host_main.cpp).
"""
import glob
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
ENV.pop("LD_PRELOAD", None)   # the sanitizer run-time must come first in the program's own library list


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout}\n{res.stderr}"
    return res.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", *SAN,
          os.path.join(ROOT, "oracle", "cce_oracle.c"), os.path.join(ROOT, "tests", "sanitize", "oracle_main.c"),
          "-o", exe, "-lm"])
    out = _run([exe], env=ENV)
    assert out.startswith("ok ")


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clangxx = "/opt/rocm/llvm/bin/clang++"
    if not (os.path.exists(hipcc) and os.path.exists(clangxx) and shutil.which("nm")):
        pytest.skip("no ROCm toolchain here")
    csrc = os.path.join(ROOT, "paper_2509_09682_amd", "csrc")
    host_san = [a for s in SAN for a in ("-Xarch_host", s)]   # host code only: nothing is compiled for the GPU
    base = [hipcc, "--offload-arch=gfx950", "--offload-host-only", "-O1", "-g", "-std=c++17", *host_san,
            "-I", os.path.join(ROOT, "include"), "-I", csrc, "-c"]
    objs = []
    for src in sorted(glob.glob(os.path.join(csrc, "*.hip"))) + [os.path.join(ROOT, "tests", "sanitize", "api_host_main.cpp")]:
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        _run(base + [src, "-o", obj])
        objs.append(obj)
    # a host-only object still names the symbol of its (absent) device code; it is only passed to the registration
    # stand-in, which ignores it
    names = sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", _run(["nm", *objs]))))
    exe = str(tmp_path / "api_san")
    _run([clangxx, *SAN, *objs, *[f"-Wl,--defsym,{n}=0" for n in names], "-o", exe])
    out = _run([exe], env=ENV)
    assert out.startswith("ok ")
