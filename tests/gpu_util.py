"""What the GPU tests share: the launch helpers (re-exported from the package) and the
parity bars.
"""
from paper_1410_0759_amd.runner import *  # noqa: F401,F403
from paper_1410_0759_amd.runner import _desc_for, _dt, _handle, _output  # noqa: F401

# The stated acceptance bars, max|gpu - oracle| / max|oracle|: 2e-5 for float inputs, 1e-2 for
# bfloat16 inputs.  (Double precision: sums of up to ~1e5 products of magnitude <= 1, each
# rounded to 2^-53, leave errors of 1e-14 relative to the largest output; 1e-12 tells a double
# path from a float one by 5 orders.)
TOL = {"f32": 2e-5, "bf16": 1e-2, "f64": 1e-12}

# What the tests assert.  Every bfloat16 test input is rounded to bfloat16 before both the
# oracle and the library see it, and a product of two bfloat16 values (8 + 8 significant bits)
# is exact in float: only the order of the float additions differs from the oracle, exactly as
# on the float path.  So the float bar applies; the stated 1e-2 could not see one dropped
# term of a long reduction (one tap of C*R*S = 4608 moves an output by about 5e-3 of the
# largest), 2e-5 does.
BOUND = {"f32": TOL["f32"], "bf16": 2e-5, "f64": TOL["f64"]}
assert all(BOUND[k] <= TOL[k] for k in TOL)
