"""Build ``libigconv.so`` (HIP kernels for gfx950 + the C-ABI host code) in-tree."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libigconv.so")
SOURCES = ["igconv_api.cpp", "igconv_kernels_f32_taps9.hip", "igconv_kernels_f32_tapmajor.hip", "igconv_kernels_f32_nopad.hip",
           "igconv_kernels_f32_generic.hip", "igconv_kernels_f32_masked.hip", "igconv_kernels_f32_direct.hip", "igconv_kernels_f32_swap.hip", "igconv_kernels_bf16.hip",
           "igconv_kernels_bf16_channels.hip", "igconv_kernels_wgrad.hip", "igconv_kernels_f64.hip", "igconv_kernels_f64_masked.hip", "igconv_kernels_wgrad_bf16c.hip", "igconv_kernels_bf16_pw.hip", "igconv_kernels_f32_teams.hip", "igconv_other.hip", "igconv_probe.hip", "igconv_noalloc.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -packed-fp32-ops is switched off: hipcc must not form v_pk_*_f32 from float code.
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument"]


def _compile(src):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + COMMON
    cmd += ["-x", "hip"] + DEVICE_FLAGS if src.endswith(".hip") else ["-x", "c++"]
    cmd += ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    return obj, err


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        results = list(ex.map(_compile, SOURCES))
    objs = [o for o, _ in results]
    if verbose:
        for _, e in results:
            if e.strip():
                print(e)
    tmp = LIB + ".tmp"
    subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
