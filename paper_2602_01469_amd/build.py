"""Builds the HIP extension in-tree: paper_2602_01469_amd/libpeagle_attn.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpeagle_attn.so")
SOURCES = ["tilemap.cpp", "api.cpp", "attn_kernels.hip", "rope_kernels.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build(verbose: bool = False, sanitize_host_to: str = "") -> str:
    """Builds the library in-tree.  With `sanitize_host_to`, builds a second library at that path instead whose HOST
    code (tile-map builder, argument validation, launch drivers) carries AddressSanitizer and
    UndefinedBehaviorSanitizer; the device code is the same (no sanitizer runs on the GPU)."""
    out_path = sanitize_host_to or LIB
    opt = ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-shared-libsan"] if sanitize_host_to else ["-O3"]
    cmd = [
        HIPCC, "-x", "hip", "--offload-arch=gfx950", *opt, "-std=c++17", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        # Matrix instructions write ordinary vector registers in every kernel.  Kernels with one wave per SIMD (the
        # D=128 dK/dV kernel) would otherwise get all their accumulators in the accumulation registers and copy
        # every score out before the vector unit can touch it (that kernel: -7 %); the others are unaffected.
        "-mllvm", "-amdgpu-mfma-vgpr-form",
        "-fgpu-flush-denormals-to-zero", "-Wno-unused-command-line-argument",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        "-o", out_path,
    ] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out:
        print(out)
    return out_path


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
