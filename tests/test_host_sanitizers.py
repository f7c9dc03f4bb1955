"""The host tier of the library and the C oracles under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU).

Each is built as an executable of its own (sanitized code plus a driver that exercises it: see
``paper_1410_0759_amd/csrc/host_check.cpp`` and ``oracle/sanitize_main.c``) rather than loaded into this Python
process, which would need the sanitizer runtime preloaded.  Any report aborts the executable."""
import subprocess

import pytest

from oracle import build as oracle_build
from paper_1410_0759_amd import build as lib_build


def _run(exe):
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-3000:]
    assert "Sanitizer" not in out and "runtime error" not in out, out[-3000:]
    return out


def test_host_tier_is_clean_under_asan_and_ubsan():
    """Descriptors, validation, kernel choice, plans, workspace sizes and the address-reach check over 3000 random
    layers (three data types, both layouts, a varying compute-unit count), the refusal paths of every pass, and
    the multiply+shift division over 200000 pairs."""
    assert "host check ok" in _run(lib_build.build_host_check())


def test_oracles_are_clean_under_asan_and_ubsan():
    """Every oracle function on 60 random small problems in buffers of exactly the spanned size."""
    assert "oracle check ok" in _run(oracle_build.build_sanitized())
