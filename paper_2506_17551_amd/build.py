"""Build libgradcomp.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_PKG, "csrc")
LIB_PATH = os.path.join(_PKG, "libgradcomp.so")
SOURCES = ["gc_api.hip", "gc_compress.hip", "gc_decompress.hip", "gc_dense.hip", "gc_rows.hip"]

# -ffp-contract=off: every fp32 operation of the method rounds on its own (no fused multiply-add),
# which the bit-exact residual needs. Packed fp32 instructions are disabled for the device pass.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libgradcomp needs the ROCm toolchain")
    return exe


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source into paper_2506_17551_amd/libgradcomp.so (always rebuilds)."""
    cmd = [hipcc()] + HIPCC_FLAGS + list(extra_flags) + [os.path.join(_CSRC, s) for s in SOURCES] + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB_PATH


def stale_sources():
    """HIP sources and headers that are newer than the built library (empty if it is up to date)."""
    if not os.path.exists(LIB_PATH):
        return list(SOURCES)
    built = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(_CSRC, f) for f in os.listdir(_CSRC)] + [os.path.join(os.path.dirname(_PKG), "include", "gradcomp.h")]
    return [os.path.basename(d) for d in deps if os.path.exists(d) and os.path.getmtime(d) > built]


def ensure_library() -> str:
    """Path of the built library. Builds it only if it is missing (a GPU run loads what was built
    beforehand); if a source is newer than the library it says so, loudly, instead of silently
    testing a stale binary: run `python -m paper_2506_17551_amd.build` after editing csrc/."""
    if not os.path.exists(LIB_PATH):
        build_library()
    else:
        newer = stale_sources()
        if newer:
            import sys
            print(f"paper_2506_17551_amd: WARNING: {os.path.basename(LIB_PATH)} is older than {', '.join(sorted(newer))}; "
                  "rebuild with `python -m paper_2506_17551_amd.build`", file=sys.stderr, flush=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
