"""The bf16-mode kernels form the quantizer ratio v = (a - z) / s (Section 3.1, Eq. 1) without a
division: t = n * r, v = t + (n - s t) * r with r = fl(1 / s) and fused multiply-adds.  The parity
protocol rests on that being the correctly rounded IEEE fp32 quotient, bit for bit.  This test builds
the kernels' own header for the host and compares it with numpy's fp32 division on 1.2e7 pairs,
including exact rounding ties and the extremes of the ranges that occur."""
import ctypes
import os
import subprocess
import tempfile

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    out = os.path.join(tempfile.mkdtemp(prefix="mrem_qm_"), "libqm.so")
    cmd = ["g++", "-O2", "-ffp-contract=off", "-shared", "-fPIC", os.path.join(ROOT, "tests", "host_quant_math.cpp"), "-o", out]
    subprocess.run(cmd, check=True, capture_output=True)
    l = ctypes.CDLL(out)
    for f in (l.mrem_host_ratio_fma, l.mrem_host_ratio_div):
        f.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_long]
        f.restype = None
    return l


def _run(f, a, z, s):
    out = np.empty_like(a)
    f(a.ctypes.data, z.ctypes.data, s.ctypes.data, out.ctypes.data, a.size)
    return out


def _check(lib, a, z, s):
    a, z, s = (np.ascontiguousarray(t, dtype=np.float32) for t in (a, z, s))
    want = ((a - z).astype(np.float32) / s).astype(np.float32)           # two IEEE fp32 operations
    got_div = _run(lib.mrem_host_ratio_div, a, z, s)
    got_fma = _run(lib.mrem_host_ratio_fma, a, z, s)
    assert np.array_equal(got_div.view(np.uint32), want.view(np.uint32))
    bad = np.flatnonzero(got_fma.view(np.uint32) != want.view(np.uint32))
    assert bad.size == 0, (bad[:5], a[bad[:5]], z[bad[:5]], s[bad[:5]], got_fma[bad[:5]], want[bad[:5]])


def test_fma_ratio_equals_ieee_division_on_random_pairs(lib):
    rng = np.random.default_rng(20211)
    n = 4_000_000
    # activations of a LayerNorm'd stream with outliers, steps of an 8-bit and of a 2-bit range
    for lo, hi in ((-3.0, 2.0), (-8.0, -3.0), (0.0, 3.0)):
        a = (rng.standard_normal(n) * rng.choice([1.0, 20.0, 1e-3], size=n)).astype(np.float32)
        s = np.exp(rng.uniform(lo, hi, size=n) * np.log(10.0)).astype(np.float32)
        z = np.where(rng.random(n) < 0.5, 0.0, -0.17 * rng.random(n)).astype(np.float32)
        _check(lib, a, z, s)


def test_fma_ratio_on_exact_ties_bounds_and_extremes(lib):
    rng = np.random.default_rng(7)
    # exact ties and clip bounds: a = (k + 1/2) * s and a = +-Qp * s with dyadic and non-dyadic steps
    k = np.arange(-300, 300, dtype=np.float32)
    for s0 in (2.0 ** -7, 0.0123, 0.55, 3.1e-5, 1.7):
        s = np.full(k.size, s0, dtype=np.float32)
        for a in ((k + 0.5) * s, k * s, np.nextafter((k + 0.5) * s, np.float32(np.inf)), np.nextafter((k + 0.5) * s, np.float32(-np.inf))):
            _check(lib, a.astype(np.float32), np.zeros_like(s), s)
    # extremes that stay free of overflow and of subnormal results: |a| up to 1e4, s from 1e-8 (the floor
    # that the update keeps step sizes above) to 1e4, quotients from 1e-12 to 1e12
    n = 200_000
    a = (rng.choice([-1.0, 1.0], size=n) * np.exp(rng.uniform(-4, 4, size=n) * np.log(10.0))).astype(np.float32)
    s = np.exp(rng.uniform(-8, 4, size=n) * np.log(10.0)).astype(np.float32)
    _check(lib, a, np.zeros(n, dtype=np.float32), s)
    # a = 0 and a = z
    _check(lib, np.zeros(16, dtype=np.float32), np.zeros(16, dtype=np.float32), np.full(16, 0.3, dtype=np.float32))
    zz = np.full(16, -0.169, dtype=np.float32)
    _check(lib, zz.copy(), zz, np.full(16, 0.004, dtype=np.float32))
