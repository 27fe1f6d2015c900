"""The kernels' own sigmoid / tanh / exp (csrc/q8_math.h, plain fma arithmetic that is the same on
host and device) against libm: the float results must be the correctly rounded ones, which is
what the oracle computes (double libm value, rounded once)."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    out = os.path.join(ROOT, "tests", "support", "_build")
    os.makedirs(out, exist_ok=True)
    so = os.path.join(out, "q8_math_host.so")
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
           "-I" + os.path.join(ROOT, "paper_1804_05038_amd", "csrc"), os.path.join(ROOT, "tests", "support", "q8_math_host.c"),
           "-o", so, "-lm"]
    try:
        subprocess.run(cmd[:1] + ["-mfma"] + cmd[1:], check=True, capture_output=True)
    except subprocess.CalledProcessError:
        subprocess.run(cmd, check=True, capture_output=True)
    L = ctypes.CDLL(so)
    for f in (L.q8m_tanh, L.q8m_sigmoid, L.q8m_exp):
        f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_long]
    return L


def _samples(rng, n):
    """Floats of every magnitude the model produces and beyond: dense near zero, around the
    branch points of the range reduction, large, tiny, denormal, signed zeros."""
    parts = [rng.standard_normal(n), rng.standard_normal(n) * 8, rng.uniform(-0.6, 0.6, n), rng.uniform(-45, 45, n),
             np.ldexp(rng.uniform(1, 2, n // 4), rng.integers(-140, 8, n // 4)) * rng.choice([-1, 1], n // 4),
             np.array([0.0, -0.0, 1e-45, -1e-45, 1e-38, 0.17328679, 0.34657359, 0.5198604, 9.0, 9.1, 20.0, 88.0, 89.0, 104.0,
                       -104.0, 700.0, -700.0, 1e30, -1e30, 3.4e38, -3.4e38])]
    k = np.arange(-60, 61)
    parts.append(np.concatenate([k * 0.34657359027997264 + d for d in (-1e-7, 0.0, 1e-7)]))   # half-integers of ln 2
    return np.concatenate(parts).astype(np.float32)


def _call(fn, x, dtype):
    x = np.ascontiguousarray(x, dtype=dtype)
    y = np.empty_like(x)
    fn(x.ctypes.data, y.ctypes.data, x.size)
    return y


def test_tanh_is_the_correctly_rounded_double_tanh(lib):
    x = _samples(np.random.default_rng(0), 1_000_000)
    got = _call(lib.q8m_tanh, x, np.float32)
    ref = np.tanh(x.astype(np.float64)).astype(np.float32)
    bad = got != ref
    # libm's own double tanh is good to about an ulp, so a handful of boundary cases may differ
    assert bad.sum() <= 3, (int(bad.sum()), x[bad][:5], got[bad][:5], ref[bad][:5])
    assert np.abs(got[bad].astype(np.float64) - ref[bad]).max(initial=0.0) <= np.spacing(np.abs(ref[bad])).max(initial=0.0)
    assert (np.signbit(got) == np.signbit(x)).all() and (np.abs(got) <= 1).all()
    assert got[x == 0].tolist() == x[x == 0].tolist()


def test_sigmoid_is_the_correctly_rounded_double_sigmoid(lib):
    x = _samples(np.random.default_rng(1), 1_000_000)
    got = _call(lib.q8m_sigmoid, x, np.float32)
    with np.errstate(over="ignore"):
        ref = (1.0 / (1.0 + np.exp(-x.astype(np.float64)))).astype(np.float32)
    bad = got != ref
    assert bad.sum() <= 3, (int(bad.sum()), x[bad][:5], got[bad][:5], ref[bad][:5])
    assert ((got >= 0) & (got <= 1)).all()


def test_exp_double_accuracy(lib):
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.uniform(-700, 700, 200_000), rng.uniform(-2, 2, 200_000), rng.uniform(-90, 0, 400_000),
                        np.arange(-1000, 1001) * 0.34657359027997264, [0.0, -0.0, 1e-300, -1e-300]])
    got = _call(lib.q8m_exp, x, np.float64)
    ref = np.exp(x)
    rel = np.abs(got - ref) / ref
    assert rel.max() < 4.5e-16, rel.max()                 # two ulps of double
    assert got[x == 0].tolist() == [1.0] * int((x == 0).sum())
