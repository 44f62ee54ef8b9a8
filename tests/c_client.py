"""Builds tests/abi_c_client (a plain C consumer of include/tabx.h) with gcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
SOURCE = os.path.join(_HERE, "abi_c_client.c")
BINARY = os.path.join(_HERE, "abi_c_client")
_ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build() -> str:
    """Needs libtabx.so and the checker's library to be built already."""
    pkg = os.path.join(_ROOT, "paper_2602_01665_amd")
    oracle = os.path.join(_ROOT, "oracle")
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(_ROOT, "include"), "-I", oracle, "-I", os.path.join(_ROCM, "include"),
           SOURCE, "-o", BINARY,
           "-L", pkg, "-ltabx", "-L", oracle, "-ltabx_ref", "-L", os.path.join(_ROCM, "lib"),
           "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../paper_2602_01665_amd", "-Wl,-rpath,$ORIGIN/../oracle",
           "-Wl,-rpath," + os.path.join(_ROCM, "lib")]
    subprocess.run(cmd, check=True)
    return BINARY


def is_stale() -> bool:
    return (not os.path.exists(BINARY)) or os.path.getmtime(BINARY) < os.path.getmtime(SOURCE)


if __name__ == "__main__":
    print(build())
