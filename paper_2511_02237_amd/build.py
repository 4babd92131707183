"""Compile the HIP library for gfx950 into paper_2511_02237_amd/liboea.so (hipcc cross-compiles
without a GPU).  Run as `python -m paper_2511_02237_amd.build`."""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "liboea.so")
SOURCES = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
HEADERS = sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + [os.path.join(ROOT, "include", "oea.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
]


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    return all(os.path.getmtime(f) <= t for f in SOURCES + HEADERS + [os.path.abspath(__file__)])


TIMELINE_LIB = os.path.join(HERE, "liboea_timeline.so")


def build(force: bool = True, extra=(), out: str = LIB) -> str:
    if not force and out == LIB and up_to_date():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + list(extra) + ["-o", out] + SOURCES
    subprocess.check_call(cmd)
    return out


def build_timeline() -> str:
    """The measurement variant: same sources with -DOEA_TIMELINE (per-workgroup phase stamps and the
    oea_timeline_read export), as liboea_timeline.so beside the product library."""
    return build(force=True, extra=("-DOEA_TIMELINE",), out=TIMELINE_LIB)


if __name__ == "__main__":
    if sys.argv[1:2] == ["--timeline"]:
        print(build_timeline())
    else:
        print(build(force=True, extra=sys.argv[1:]))
