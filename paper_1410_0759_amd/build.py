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
           "igconv_kernels_bf16_channels.hip", "igconv_kernels_wgrad.hip", "igconv_kernels_f64.hip", "igconv_kernels_f64_masked.hip", "igconv_kernels_wgrad_bf16c.hip", "igconv_kernels_bf16_pw.hip", "igconv_kernels_f32_teams.hip", "igconv_other.hip", "igconv_bias_grad.hip", "igconv_probe.hip", "igconv_noalloc.hip"]
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


def build_host_check():
    """The host tier under AddressSanitizer and UndefinedBehaviorSanitizer: ``csrc/igconv_api.cpp`` and the driver
    ``csrc/host_check.cpp`` compiled with both (any report aborts), linked with the ordinary objects of the kernel
    files (their device code never runs: the driver makes no launch).  Builds those first if they are missing.
    Returns the executable's path."""
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES if s != "igconv_api.cpp"]
    if not all(os.path.exists(o) for o in objs):
        build()
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    exe = os.path.join(OBJ, "host_check_san")
    host_objs = []
    for src in ("igconv_api.cpp", "host_check.cpp"):
        obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".san.o")
        subprocess.run([HIPCC, "-std=c++17", "-Wall", "-Wno-unused-command-line-argument", "-x", "c++"] + san +
                       ["-c", os.path.join(CSRC, src), "-o", obj], check=True)
        host_objs.append(obj)
    subprocess.run([HIPCC, "--offload-arch=gfx950"] + san + ["-o", exe] + host_objs + objs, check=True)
    return exe


if __name__ == "__main__":
    import sys
    print(build_host_check() if "--host-check" in sys.argv else build(verbose=True))
