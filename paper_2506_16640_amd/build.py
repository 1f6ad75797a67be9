"""Builds the C-ABI library (csrc/ -> lib/libentmax_attn.so) with hipcc for gfx950.

The kernels of each (launcher, element type, head dimension, with / without the distance-bias code)
combination are a translation unit of their own (csrc/inst.hip compiled with different -D flags), so the units compile in parallel."""
import concurrent.futures
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_DIR = os.path.join(_HERE, "lib")
OBJ_DIR = os.path.join(LIB_DIR, "obj")
LIB = os.path.join(LIB_DIR, "libentmax_attn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 arithmetic stays off: ordinary float code must not be fused into v_pk_* forms
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results go straight to VGPRs (no AGPR round trip before the VALU work on the scores)
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    # the kernels never produce or consume NaN (masked scores are -inf and are tested before use):
    # lets max/min chains compile to v_max3 / v_min3 without a canonicalising self-max per operand.
    # Device code only: the host-side argument checks must keep rejecting NaN parameters.
    "-Xarch_device", "-fno-honor-nans",
]


def translation_units():
    """(object name, source, extra flags) of every unit of the library."""
    units = [("api", "entmax_attn.hip", []), ("scale_proj", "scale_proj.hip", [])]
    for leg in ("FWD", "BWD"):
        for tname, ctype in (("bf16", "bf16_t"), ("f32", "float")):
            for d in (64, 128):
                for bias in (0, 1):
                    units.append(("%s_%s_%d%s" % (leg.lower(), tname, d, "_bias" if bias else ""), "inst.hip",
                                  ["-DENTMAX_INST_%s" % leg, "-DENTMAX_INST_T=%s" % ctype, "-DENTMAX_INST_D=%d" % d,
                                   "-DENTMAX_INST_BIAS=%d" % bias]))
    return units


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "not a recognized feature" not in l)
    return res.returncode, res.stdout, err


def build_library(verbose=False, jobs=None):
    """Compile every HIP source into lib/libentmax_attn.so (always recompiles)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    jobs = jobs or min(8, os.cpu_count() or 1)
    cmds = []
    objs = []
    for name, src, extra in translation_units():
        obj = os.path.join(OBJ_DIR, name + ".o")
        objs.append(obj)
        cmds.append([hipcc] + HIPCC_FLAGS + extra + inc + ["-c", os.path.join(CSRC, src), "-o", obj])
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(_run, cmds))
    failed = False
    for cmd, (rc, out, err) in zip(cmds, results):
        if verbose or rc != 0:
            print(" ".join(cmd[-4:]))
            print(out)
            print(err)
        failed = failed or rc != 0
    if failed:
        raise RuntimeError("hipcc failed building " + LIB)
    rc, out, err = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    if verbose or rc != 0:
        print(out)
        print(err)
    if rc != 0:
        raise RuntimeError("hipcc failed linking " + LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
