"""What the GELU of the HIP epilogue may differ from the exact function by, and the check of re-quantised GELU codes that
follows from it.

The kernels evaluate GELU(x) = max(x, 0) - t * 2^P(t), t = |x|, with a degree-5 polynomial P in fp32 (csrc/epilogue.h);
the oracle evaluates x * Phi(x) with erf in fp64.  `FIT_BOUND_ULP16` is the bound the library states for the difference,
in units of the last place of the exact value as an fp16 number; test_abi_host.py checks it on the CPU by running the
same fp32 operation sequence in numpy over every fp16 argument and a dense fp32 grid.  The GPU tests use the bound to
decide, element by element, whether an int8 code that differs from the oracle's is allowed to.
"""
import os
import re

import numpy as np

FIT_BOUND_ULP16 = 0.15
_EPILOGUE_H = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2305_10727_amd", "csrc", "epilogue.h")


def coefficients():
    """P0..P5 as fp32, read from the kernel source"""
    found = dict(re.findall(r"kGeluP(\d) = (-?[0-9.eE+-]+)f", open(_EPILOGUE_H).read()))
    assert sorted(found) == list("012345"), found
    return [np.float32(found[str(i)]) for i in range(6)]


def _fma32(a, b, c):
    # a * b is exact in fp64 (24 x 24 bits); the sum is rounded to fp64 and then to fp32, which differs from a fused fp32
    # operation only in double-rounding cases (2^-29 relative): far below what is measured here
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)


def gelu_fit_f32(x):
    """the kernel's operation sequence (gelu_f32) in numpy; v_exp_f32 is modelled as a correctly rounded 2^p"""
    P = coefficients()
    x = np.asarray(x, np.float32)
    t = np.abs(x)
    p = _fma32(t, np.full_like(t, P[5]), np.full_like(t, P[4]))
    for k in (3, 2, 1, 0):
        p = _fma32(p, t, np.full_like(t, P[k]))
    q = np.exp2(p.astype(np.float64)).astype(np.float32)
    return _fma32(-t, q, np.maximum(x, np.float32(0)))


def ulp16(y):
    """unit in the last place of |y| as an fp16 number (subnormal spacing below 2^-14)"""
    e = np.floor(np.log2(np.maximum(np.abs(np.asarray(y, np.float64)), 1e-300)))
    return 2.0 ** (np.maximum(e, -14.0) - 10.0)


def assert_gelu_codes_equal_up_to_near_ties(q_gpu, q_oracle, v32, gelu64, out_scale):
    """q_gpu, q_oracle: int8 codes clamp(rint(GELU(v) / out_scale)); v32: the fp32 pre-activation (identical on both
    sides); gelu64: the exact GELU of v32 in fp64 (from the oracle).  Both sides decide the code in fp32 from their own
    GELU value: the oracle's is the exact value rounded to fp32 (2^-24 relative), the kernel's is within
    FIT_BOUND_ULP16 * ulp16 of the exact value, and the quotient by the scale is rounded once more (2^-24 relative on
    either side).  So the codes can differ only by one, and only where the exact quotient lies within
        delta = (FIT_BOUND_ULP16 * ulp16(g) + 2^-23 |g|) / s + 2^-22 |g / s|
    of the half-integer between them.  Every differing element is checked against that; no rate is tolerated."""
    q_gpu = np.asarray(q_gpu).astype(np.int32)
    q_oracle = np.asarray(q_oracle).astype(np.int32)
    idx = np.nonzero(q_gpu != q_oracle)
    if idx[0].size == 0:
        return 0
    assert np.abs(q_gpu[idx] - q_oracle[idx]).max() == 1
    g = np.asarray(gelu64, np.float64)[idx]
    s = float(out_scale)
    t = g / s
    boundary = np.minimum(q_gpu[idx], q_oracle[idx]) + 0.5
    delta = (FIT_BOUND_ULP16 * ulp16(g) + 2.0 ** -23 * np.abs(g)) / s + 2.0 ** -22 * np.abs(t)
    worst = (np.abs(t - boundary) / delta).max()
    assert worst <= 1.0, "a code differs from the oracle's although GELU(v)/scale is %.3g deltas away from the boundary" % worst
    assert np.abs(np.asarray(v32)[idx]).max() < 1e30  # (finite inputs)
    return int(idx[0].size)
