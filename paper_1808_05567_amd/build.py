"""Build libconv_mi355x.so (gfx950) in-tree with hipcc.

    python -m paper_1808_05567_amd.build

Cross-compiles without a GPU.  The library is the product; nothing here falls
back to another implementation when the build is missing.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libconv_mi355x.so")
SOURCES = ("api.hip", "igemm.hip", "igemm_rect.hip", "igemm_stem.hip", "upd.hip", "upd_f32.hip", "upd_f32_1x1.hip", "upd_f32_c4.hip", "upd_bf16.hip", "upd_bf16_1x1.hip", "upd_bf16_c4.hip", "direct.hip", "pack.hip", "ceilings.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions stay off for every device function
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # an unroll-by-2 hint on loops with run-time bounds is a hint: no warning where it is declined
    "-Wno-pass-failed",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_lib(verbose: bool = True) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    # every symbol must resolve (a kernel instantiation the host pass dropped would only
    # show up when the library is loaded): load it in a child process before installing it
    r = subprocess.run([sys.executable, "-c", "import ctypes, sys; ctypes.CDLL(sys.argv[1])", tmp],
                       capture_output=True, text=True)
    if r.returncode != 0:
        os.unlink(tmp)
        raise RuntimeError("the built library does not load:\n" + r.stderr)
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_lib()
