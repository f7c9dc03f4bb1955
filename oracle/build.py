"""Compile the C oracles with gcc into ``oracle/lib*_oracle.so`` (host code only)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "conv_oracle.c")
LIB = os.path.join(HERE, "libconv_oracle.so")
POINTWISE_SRC = os.path.join(HERE, "pointwise_oracle.c")
POINTWISE_LIB = os.path.join(HERE, "libpointwise_oracle.so")
POINTWISE_DEPS = (os.path.join(HERE, "pointwise_oracle_impl.inc"),)


def _compile(src, lib, force, extra, deps=()):
    newest = max(os.path.getmtime(f) for f in (src,) + tuple(deps))
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= newest:
        return lib
    cmd = ["gcc", "-O2", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra"] + extra + ["-o", lib + ".tmp", src]
    subprocess.run(cmd, check=True)
    os.replace(lib + ".tmp", lib)
    return lib


def build(force: bool = True) -> str:
    """Build both shared libraries; with ``force=False`` keep existing up-to-date ones.
    Returns the path of the convolution oracle."""
    _compile(POINTWISE_SRC, POINTWISE_LIB, force, ["-lm"], POINTWISE_DEPS)
    return _compile(SRC, LIB, force, ["-fopenmp"])


def build_sanitized() -> str:
    """Both oracles and ``sanitize_main.c`` as one executable under AddressSanitizer and
    UndefinedBehaviorSanitizer (any report aborts the run); returns its path."""
    out_dir = os.path.join(HERE, "_build")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "oracle_check_san")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-Wall", "-Wextra", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", exe,
           os.path.join(HERE, "sanitize_main.c"), SRC, POINTWISE_SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return exe


def build_pointwise(force: bool = False) -> str:
    return _compile(POINTWISE_SRC, POINTWISE_LIB, force, ["-lm"], POINTWISE_DEPS)


if __name__ == "__main__":
    print(build())
