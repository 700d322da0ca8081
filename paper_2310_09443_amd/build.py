"""Builds the HIP library for gfx950 into paper_2310_09443_amd/libg10.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = [os.path.join(HERE, "csrc", f) for f in ("g10_api.hip", "g10_mem.hip", "g10_vitality.hip", "g10_plan.hip", "g10_loop.hip", "g10_prefetch.hip", "g10_replay.hip")]
DEPS = SRC + [os.path.join(HERE, "csrc", "g10_internal.h"), os.path.join(HERE, "csrc", "g10_plan_defs.h"),
              os.path.join(ROOT, "include", "g10.h")]
LIB = os.path.join(HERE, "libg10.so")


def up_to_date() -> bool:
    return os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS)


def build(force: bool = True) -> str:
    if not force and up_to_date():
        return LIB
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           "-Wall", "-Wno-unused-function"] + SRC + ["-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
