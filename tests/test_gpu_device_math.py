"""The device's own sigmoid / tanh / exp (csrc/q8_math.h as the kernels call it, including the
device's form of the division) evaluated on the GPU through q8_math_eval and compared value by
value with what the oracle computes: the double libm value rounded once to float."""
import numpy as np
import pytest
import torch

from test_device_math import _samples

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def q():
    import paper_1804_05038_amd as q
    return q


@pytest.fixture(scope="module")
def ctx(q):
    return q.Context()


def test_device_tanh_is_the_correctly_rounded_double_tanh(q, ctx):
    x = _samples(np.random.default_rng(0), 1_000_000)
    got = q.q8_math_eval(ctx, "tanh", torch.from_numpy(x).to(ctx.device)).cpu().numpy()
    ref = np.tanh(x.astype(np.float64)).astype(np.float32)
    bad = got != ref
    # libm's own double tanh is good to about an ulp, so a handful of boundary cases may differ
    assert bad.sum() <= 3, (int(bad.sum()), x[bad][:5], got[bad][:5], ref[bad][:5])
    assert np.abs(got[bad].astype(np.float64) - ref[bad]).max(initial=0.0) <= np.spacing(np.abs(ref[bad])).max(initial=0.0)
    assert (np.signbit(got) == np.signbit(x)).all() and (np.abs(got) <= 1).all()
    assert got[x == 0].tolist() == x[x == 0].tolist()


def test_device_sigmoid_is_the_correctly_rounded_double_sigmoid(q, ctx):
    x = _samples(np.random.default_rng(1), 1_000_000)
    got = q.q8_math_eval(ctx, "sigmoid", torch.from_numpy(x).to(ctx.device)).cpu().numpy()
    with np.errstate(over="ignore"):
        ref = (1.0 / (1.0 + np.exp(-x.astype(np.float64)))).astype(np.float32)
    bad = got != ref
    assert bad.sum() <= 3, (int(bad.sum()), x[bad][:5], got[bad][:5], ref[bad][:5])
    assert ((got >= 0) & (got <= 1)).all()


def test_device_exp_double_accuracy(q, ctx):
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.uniform(-700, 700, 200_000), rng.uniform(-2, 2, 200_000), rng.uniform(-90, 0, 400_000),
                        np.arange(-1000, 1001) * 0.34657359027997264, [0.0, -0.0, 1e-300, -1e-300]])
    got = q.q8_math_eval(ctx, "exp", torch.from_numpy(x).to(ctx.device)).cpu().numpy()
    ref = np.exp(x)
    rel = np.abs(got - ref) / ref
    assert rel.max() < 4.5e-16, rel.max()                 # two ulps of double
    assert got[x == 0].tolist() == [1.0] * int((x == 0).sum())


def test_device_and_host_forms_agree(q, ctx):
    """The host build of the same header (plain division) and the device (reciprocal, Newton steps, one
    correction of the quotient): the same floats on every sample."""
    import ctypes, os, subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = os.path.join(root, "tests", "support", "_build")
    os.makedirs(out, exist_ok=True)
    so = os.path.join(out, "q8_math_host.so")
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
           "-I" + os.path.join(root, "paper_1804_05038_amd", "csrc"), os.path.join(root, "tests", "support", "q8_math_host.c"),
           "-o", so, "-lm"]
    try:
        subprocess.run(cmd[:1] + ["-mfma"] + cmd[1:], check=True, capture_output=True)
    except subprocess.CalledProcessError:
        subprocess.run(cmd, check=True, capture_output=True)
    L = ctypes.CDLL(so)
    x = _samples(np.random.default_rng(3), 500_000)
    for name, fn in (("tanh", L.q8m_tanh), ("sigmoid", L.q8m_sigmoid)):
        fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_long]
        host = np.empty_like(x)
        fn(x.ctypes.data, host.ctypes.data, x.size)
        dev = q.q8_math_eval(ctx, name, torch.from_numpy(x).to(ctx.device)).cpu().numpy()
        assert (host == dev).all(), (name, int((host != dev).sum()))


def test_wave_sort_orders_every_group_of_64(q, ctx):
    """The wave-wide sort behind the top-k threshold (cross-lane moves only): random values, many equal
    values, infinities and already sorted input, against numpy's sort."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal(64 * 4096).astype(np.float32)
    x[: 64 * 512] = rng.integers(-3, 4, 64 * 512).astype(np.float32)          # heavy ties
    x[64 * 512: 64 * 520] = np.tile(np.arange(64, dtype=np.float32), 8)        # ascending
    x[64 * 520: 64 * 528] = np.tile(np.arange(64, dtype=np.float32)[::-1], 8)  # descending
    x[64 * 528: 64 * 536: 3] = -np.inf
    x[64 * 536] = np.inf
    y = q.q8_math_eval(ctx, "sort64", torch.from_numpy(x).to(ctx.device)).cpu().numpy()
    ref = -np.sort(-x.reshape(-1, 64), axis=1)
    assert (y.reshape(-1, 64) == ref).all()
