"""Build step of the HIP library: hipcc, gfx950 only, in-tree shared object."""
from __future__ import annotations

import subprocess
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libloza_ssa.so"
SOURCES = ["ssa_bf16.hip", "ssa_bwd.hip", "ssa_f32.hip", "ssa_api.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instruction selection is switched off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the score phase is one long asm statement that names M0 as clobbered; clang only warns
    "-Wno-inline-asm",
]


def build(verbose: bool = False) -> Path:
    """Compile every HIP source of the library for gfx950 into ``libloza_ssa.so`` (always rebuilds)."""
    cmd = ["hipcc", *HIPCC_FLAGS, *[str(CSRC / s) for s in SOURCES], "-o", str(LIB)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the device-only feature flag; that one warning is harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
