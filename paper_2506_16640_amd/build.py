"""Builds the C-ABI library (csrc/ -> lib/libentmax_attn.so) with hipcc for gfx950."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SRC = os.path.join(_HERE, "csrc", "entmax_attn.hip")
LIB_DIR = os.path.join(_HERE, "lib")
LIB = os.path.join(LIB_DIR, "libentmax_attn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 arithmetic stays off: ordinary float code must not be fused into v_pk_* forms
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results go straight to VGPRs (no AGPR round trip before the VALU work on the scores)
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    # the kernels never produce or consume NaN (masked scores are -inf and are tested before use):
    # lets max/min chains compile to v_max3 / v_min3 without a canonicalising self-max per operand.
    # Device code only: the host-side argument checks must keep rejecting NaN parameters.
    "-Xarch_device", "-fno-honor-nans",
]


def build_library(verbose=False):
    """Compile every HIP source into lib/libentmax_attn.so (always recompiles)."""
    os.makedirs(LIB_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-o", LIB, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if "not a recognized feature" not in l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building " + LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
