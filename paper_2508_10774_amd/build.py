"""Build libasa.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2508_10774_amd.build

The library is loaded by ``binding.load()``; nothing is compiled at import time.
"""

from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libasa.so")
SOURCES = ["asa_api.hip", "asa_fwd.hip", "asa_mask.hip", "asa_bwd.hip", "asa_reorder.hip", "asa_order.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def build_lib(verbose: bool = False, extra=(), lib_path: str = LIB, objdir: str = CSRC,
              link_extra=()) -> str:
    """Compile every translation unit and link libasa.so; returns its path.

    extra / link_extra: more hipcc flags for the compile / link lines; lib_path, objdir: where the
    library and the objects go (the host-sanitizer build of the tests uses a directory of its
    own, so that the product library is never replaced by an instrumented one)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        text = out.decode(errors="replace")
        # the host pass does not know the packed-fp32 target feature; that warning is harmless
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed = True
            print(f"--- {src} failed\n{text}", file=sys.stderr)
        elif verbose and text.strip():
            print(f"--- {src}\n{text}")
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *link_extra, *objs, "-o", lib_path]
    subprocess.run(cmd, check=True)
    return lib_path


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv))
