"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU work).

* The oracle (plain C): every function on small ragged inputs, gcc -fsanitize=address,undefined.
* The library's host side: a copy of libasa built with the HOST pass instrumented (the device
  code is compiled as usual), driven through every argument-validation path and the Gilbert
  order, none of which reaches the GPU.
"""

import os
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-4000:]}"
    return r.stdout


def test_oracle_is_clean_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "san_oracle")
        _run(["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
              "-fno-sanitize-recover=undefined", "-fopenmp",
              os.path.join(ROOT, "tests", "sanitize_oracle_driver.c"),
              os.path.join(ROOT, "oracle", "asa_ref.c"), "-o", exe, "-lm"])
        out = _run([exe], env=ENV)
        assert out.strip().endswith("ok"), out


def test_library_host_code_is_clean_under_asan_and_ubsan():
    from paper_2508_10774_amd import build
    clangxx = "/opt/rocm/llvm/bin/clang++"
    if not os.path.exists(clangxx):
        pytest.skip("no ROCm clang++ for the driver")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    with tempfile.TemporaryDirectory() as tmp:
        lib = build.build_lib(extra=san, lib_path=os.path.join(tmp, "libasa_san.so"), objdir=tmp,
                              link_extra=["-fsanitize=address", "-fsanitize=undefined",
                                          "-fno-gpu-sanitize"])
        exe = os.path.join(tmp, "san_abi")
        _run([clangxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
              "-fno-sanitize-recover=undefined", "-I" + os.path.join(ROOT, "include"),
              os.path.join(ROOT, "tests", "sanitize_abi_driver.cpp"), lib, "-Wl,-rpath," + tmp,
              "-Wl,-rpath,/opt/rocm/lib", "-o", exe])
        # (leak checking off here: the HIP runtime that the library links keeps its own allocations)
        out = _run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))
        assert out.strip().endswith("ok"), out
