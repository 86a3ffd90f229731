"""Builds the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libqsl.so")
SOURCES = [os.path.join(_HERE, "csrc", "qsl.hip")]
HEADERS = [os.path.join(_HERE, "csrc", h) for h in ("qsl_device.h", "qsl_layout.h", "qsl_stream.h", "qsl_select.h",
                                                    "qsl_encode.h", "qsl_decode.h")] + [os.path.join(ROOT, "include", "qsl.h")]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17",
    "-ffp-contract=off",                                        # one rounding per written fp operation
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fPIC", "-shared",
    "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(_HERE, "csrc"),
]


def build(verbose: bool = False) -> str:
    """Compile libqsl.so (always recompiles)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB_PATH] + SOURCES
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(res.stderr)
    return LIB_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True))
