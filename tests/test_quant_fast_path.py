"""Host proof of the quantiser's short route (CPU only).

The HIP row routine (`csrc/slim_common.h`) replaces the IEEE divisions of the definition
(scale = fl32(amax / 127), code = rint(fl32(x / scale)), paper section 2.2 with the rounding fixed as in the
oracle) by a multiply-and-correct scale and a reciprocal-multiply code wherever a guard says that is safe.  The C
model under `tests/host_models/` sweeps that arithmetic over every bf16 amax and every bf16 |x| <= amax, for every
value a 1-ulp reciprocal can return, against host IEEE divisions.  The GPU parity tests then compare the kernel's
bits with the oracle's.
"""
import ctypes
import os
import re
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "host_models", "quant_fast_path.c")
COMMON_H = os.path.join(ROOT, "paper_2407_07304_amd", "csrc", "slim_common.h")


@pytest.fixture(scope="module")
def model(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("quant_model") / "libquant_model.so")
    subprocess.run(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-fno-fast-math",
                    "-ffp-contract=off", "-o", so, SRC, "-lm"], check=True)
    lib = ctypes.CDLL(so)
    lib.model_scale_sweep.argtypes = [ctypes.c_float, ctypes.c_float, ctypes.c_void_p]
    lib.model_code_sweep.argtypes = [ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_int, ctypes.c_void_p]
    return lib


def kernel_constants():
    """The guard constants as the HIP header spells them (hex float literals)."""
    text = open(COMMON_H).read()
    lo = re.search(r"kQuantFastLo\s*=\s*(0x1p[-+]?\d+)f", text).group(1)
    hi = re.search(r"kQuantFastHi\s*=\s*(0x1p[-+]?\d+)f", text).group(1)
    guard = re.search(r"kQuantTieGuard\s*=\s*(0x1p[-+]?\d+)f", text).group(1)
    assert re.search(r"kQuantMagic\s*=\s*12582912\.0f", text)
    return float.fromhex(lo), float.fromhex(hi), float.fromhex(guard)


def test_fast_scale_equals_the_ieee_quotient_for_every_bf16_amax_in_range(model):
    lo, hi, _ = kernel_constants()
    out = (ctypes.c_long * 2)()
    assert model.model_scale_sweep(lo, hi, out) == 0
    n, bad = out[0], out[1]
    assert n == 120 * 128 + 1 and bad == 0, (n, bad)   # exponents 2^-60 .. 2^59 with 128 mantissas each, and 2^60


def test_fast_codes_equal_the_definition_wherever_the_guard_accepts_them(model):
    lo, hi, guard = kernel_constants()
    out = (ctypes.c_long * 4)()
    assert model.model_code_sweep(lo, hi, guard, 1, out) == 0
    cases, accepted, bad, worst = out[0], out[1], out[2], out[3]
    assert cases > 10 ** 9 and bad == 0, (cases, accepted, bad)
    # the guard is not vacuous, and the error it has to cover is what the comment in the header derives: |y - x/scale|
    # stays below 2^-15 (here in units of 2^-24; the model's reciprocals are up to 1.5 ulp off, the instruction's 1),
    # half of the guard of 2^-14
    assert accepted / cases > 0.999
    assert worst <= 2 ** (24 - 15), worst


def test_the_guard_matters(model):
    # with no guard at all the short route does disagree with the definition somewhere: the sweep can see mistakes
    lo, hi, _ = kernel_constants()
    out = (ctypes.c_long * 4)()
    assert model.model_code_sweep(lo, hi, ctypes.c_float(0.0), 8, out) == 0
    assert out[2] > 0
