"""Pins for the oracle's quantize / accumulate / dequantize steps (Section 3 of the paper)."""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "quantize_hand_vectors.txt")


def _hand_vectors():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        v, q, s = [part.split() for part in line.split(";")]
        out.append((np.array(v, np.float32), np.array(q, np.int64), np.float32(s[0])))
    return out


def test_hand_derived_vectors(oracle):
    for v, q_exp, s_exp in _hand_vectors():
        q, s = oracle.quantize(v)
        assert q.tolist() == q_exp.tolist()
        assert s == s_exp


def test_half_to_even_not_half_away(oracle):
    v = np.array([127.0, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5], np.float32)
    q, _ = oracle.quantize(v)
    assert q.tolist() == [127, 0, 2, 2, 4, 0, -2, -2]


def test_invariants_random(oracle):
    rng = np.random.default_rng(7)
    for n in (1, 3, 16, 257, 2048):
        for std in (1e-3, 1.0, 50.0):
            v = (rng.standard_normal(n) * std).astype(np.float32)
            q, s = oracle.quantize(v)
            m = np.abs(v).max()
            assert s == np.float32(m) / np.float32(127.0)
            assert abs(int(q[np.argmax(np.abs(v))])) == 127          # the largest element maps to +-127
            assert q.min() >= -127 and q.max() <= 127                # -128 never produced
            qn, sn = oracle.quantize(-v)
            assert sn == s and (qn == -q).all()                      # odd symmetry
            err = np.abs(v.astype(np.float64) - float(s) * q.astype(np.float64))
            assert err.max() <= float(s) / 2 * (1 + 1e-4)            # round-trip bound scale/2
            assert (q[v == 0] == 0).all()


def test_zero_and_tiny_vectors(oracle):
    q, s = oracle.quantize(np.zeros(9, np.float32))
    assert s == 1.0 and not q.any()
    q, s = oracle.quantize(np.full(5, 2.0 ** -101, np.float32))
    assert s == 1.0 and not q.any()
    q, s = oracle.quantize(np.array([2.0 ** -99, -2.0 ** -100], np.float32))
    assert q.tolist() == [127, -64] and s == np.float32(2.0 ** -99) / np.float32(127)


def test_matrix_has_one_scale_and_zero_padding(oracle):
    rng = np.random.default_rng(3)
    W = rng.standard_normal((5, 20)).astype(np.float32)
    Wq, s = oracle.quantize_matrix(W)
    assert Wq.shape == (5, 32)
    assert not Wq[:, 20:].any()
    qf, sf = oracle.quantize(W.reshape(-1))                          # per-matrix == per flattened vector
    assert s == sf and (Wq[:, :20].reshape(-1) == qf).all()


def test_accumulate_brute_force_tiny(oracle):
    rng = np.random.default_rng(11)
    for _ in range(50):
        M, K = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        ld = K + int(rng.integers(0, 4))
        Wq = rng.integers(-127, 128, size=(M, ld)).astype(np.int8)
        xq = rng.integers(-127, 128, size=K).astype(np.int8)
        acc = oracle.accumulate(Wq, K, xq)
        for i in range(M):                                           # pure-Python integers, no overflow possible
            assert int(acc[i]) == sum(int(Wq[i, k]) * int(xq[k]) for k in range(K))


def test_accumulate_extremes_and_layout(oracle):
    K = 2048
    Wq = np.full((3, K), 127, np.int8)
    Wq[1] = -127
    Wq[2, ::2] = 0
    xq = np.full(K, -127, np.int8)
    assert oracle.accumulate(Wq, K, xq).tolist() == [-33032192, 33032192, -16516096]
    # row-major, K contiguous: a matrix that is not equal to its transpose
    Wq = np.array([[1, 2, 3], [4, 5, 6]], np.int8)
    assert oracle.accumulate(Wq, 3, np.array([1, 0, -1], np.int8)).tolist() == [-2, -2]
    assert oracle.accumulate(Wq, 3, np.array([1, 10, 100], np.int8)).tolist() == [321, 654]


def test_dequantize_exact_small_case(oracle):
    y = oracle.dequantize(np.array([3, -8, 0], np.int32), 0.5, 0.25, None)
    assert y.tolist() == [0.375, -1.0, 0.0]
    y = oracle.dequantize(np.array([3, -8, 0], np.int32), 0.5, 0.25, np.array([1, 2, 3], np.float32))
    assert y.tolist() == [1.375, 1.0, 3.0]


@pytest.mark.parametrize("M,K", [(64, 512), (33, 1000), (7, 2048)])
def test_q8_product_within_closed_form_bound_of_fp64(oracle, M, K):
    """|y_i - (W x)_i| <= (s_w/2)||x||_1 + (s_x/2)||W_i||_1 + K s_w s_x / 4 (+ float rounding)."""
    rng = np.random.default_rng(K)
    W = (rng.standard_normal((M, K)) * 0.05).astype(np.float32)
    x = rng.standard_normal(K).astype(np.float32)
    L = oracle.QLinear(W)
    y, xq, sx, acc = L.gemv(x, taps=True)
    exact = W.astype(np.float64) @ x.astype(np.float64)
    sw = float(L.scale)
    bound = sw / 2 * np.abs(x).sum() + float(sx) / 2 * np.abs(W).sum(axis=1) + K * sw * float(sx) / 4
    err = np.abs(y - exact)
    assert (err <= bound * (1 + 1e-3) + 1e-6).all()
    # and the approximation is good: rms relative error around one percent for Gaussian data
    rel = np.sqrt((err ** 2).mean()) / np.sqrt((exact ** 2).mean())
    assert 1e-4 < rel < 0.03
    # the fp32 engine's product is the exact one rounded
    np.testing.assert_allclose(L.gemv_fp32(x), exact, rtol=1e-6, atol=1e-6)


def test_scale_equivariance_power_of_two(oracle):
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((16, 48)) * 0.1).astype(np.float32)
    x = rng.standard_normal(48).astype(np.float32)
    y1 = oracle.QLinear(W).gemv(x)
    y4 = oracle.QLinear(W * 4).gemv(x)
    assert (y4 == 4 * y1).all()
    y8 = oracle.QLinear(W).gemv(x * 0.125)
    assert (y8 == 0.125 * y1).all()


def test_narrow_matrix_equals_column_by_column(oracle):
    rng = np.random.default_rng(9)
    W = (rng.standard_normal((40, 100)) * 0.05).astype(np.float32)
    b = rng.standard_normal(40).astype(np.float32)
    L = oracle.QLinear(W, b)
    X = rng.standard_normal((5, 100)).astype(np.float32) * np.array([[1], [10], [0.1], [0], [3]], np.float32)
    Y, xq, xs, acc = L.gemm_narrow(X, taps=True)
    for j in range(5):
        y, q, s, a = L.gemv(X[j], taps=True)
        assert (Y[j] == y).all() and (xq[j] == q).all() and xs[j] == s and (acc[j] == a).all()
    assert xs[3] == 1.0 and (Y[3] == b).all()                        # the zero column: scale 1, result = bias


# ---- the variant with one weight scale per row -------------------------------------------

def test_row_scales_hand_case(oracle):
    """Worked by hand: rows (1, -0.5, 0.25) and (0, 0, 0) and (-254, 127, 2): row maxima 1, 0, 254."""
    W = np.array([[1.0, -0.5, 0.25], [0, 0, 0], [-254.0, 127.0, 2.0]], np.float32)
    L = oracle.QLinearRows(W)
    assert L.row_scale.tolist() == [np.float32(1.0) / np.float32(127.0), 1.0, 2.0]
    assert L.Wq[:, :3].tolist() == [[127, -64, 32], [0, 0, 0], [-127, 64, 1]]      # 63.5 -> 64 and 31.75 -> 32
    assert (L.Wq[:, 3:] == 0).all()
    # x = (127, 0, -127)/127 quantizes to codes (127, 0, -127) with scale 1/127
    x = np.array([1.0, 0.0, -1.0], np.float32)
    y, xq, sx, acc = L.gemv(x, taps=True)
    assert xq.tolist() == [127, 0, -127] and sx == np.float32(1.0) / np.float32(127.0)
    assert acc.tolist() == [127 * 127 - 32 * 127, 0, -127 * 127 - 127]
    c0 = np.float32(L.row_scale[0]) * sx
    assert y[0] == np.float32(acc[0]) * c0 and y[1] == 0.0 and y[2] == np.float32(acc[2]) * (np.float32(2.0) * sx)


def test_row_scales_commute_with_row_scaling(oracle):
    """Scaling row i of W by a power of two scales y_i by exactly that factor and nothing else:
    true for per-row scales, false for one scale per matrix."""
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((24, 80)) * 0.1).astype(np.float32)
    d = np.float32(2.0) ** rng.integers(-6, 7, size=24).astype(np.float32)
    X = rng.standard_normal((3, 80)).astype(np.float32)
    A, B = oracle.QLinearRows(W), oracle.QLinearRows(W * d[:, None])
    assert (A.Wq == B.Wq).all() and (B.row_scale == A.row_scale * d).all()
    assert (B.gemm_narrow(X) == A.gemm_narrow(X) * d[None, :]).all()
    assert not (oracle.QLinear(W * d[:, None]).gemm_narrow(X) == oracle.QLinear(W).gemm_narrow(X) * d[None, :]).all()


def test_row_scales_equal_matrix_scale_when_row_maxima_agree(oracle):
    rng = np.random.default_rng(12)
    W = (rng.standard_normal((10, 64)) * 0.05).astype(np.float32)
    W[:, 7] = np.float32(0.75) * np.where(rng.random(10) < 0.5, -1, 1)      # every row's largest entry is +-0.75
    b = rng.standard_normal(10).astype(np.float32)
    X = rng.standard_normal((4, 64)).astype(np.float32)
    R, M = oracle.QLinearRows(W, b), oracle.QLinear(W, b)
    assert (R.row_scale == M.scale).all() and (R.Wq == M.Wq).all()
    assert (R.gemm_narrow(X) == M.gemm_narrow(X)).all()


@pytest.mark.parametrize("M,K", [(50, 512), (9, 1000)])
def test_row_scales_bound_and_gain(oracle, M, K):
    """Same closed-form bound as the per-matrix product with s_w replaced by the row's own scale;
    on rows of very different size the per-row variant is the more accurate one."""
    rng = np.random.default_rng(K + 1)
    W = (rng.standard_normal((M, K)) * 0.05).astype(np.float32) * np.logspace(-2, 0, M, dtype=np.float32)[:, None]
    x = rng.standard_normal(K).astype(np.float32)
    R = oracle.QLinearRows(W)
    y, xq, sx, acc = R.gemv(x, taps=True)
    exact = W.astype(np.float64) @ x.astype(np.float64)
    sw = R.row_scale.astype(np.float64)
    bound = sw / 2 * np.abs(x).sum() + float(sx) / 2 * np.abs(W).sum(axis=1) + K * sw * float(sx) / 4
    err = np.abs(y - exact)
    assert (err <= bound * (1 + 1e-3) + 1e-7).all()
    err_m = np.abs(oracle.QLinear(W).gemv(x) - exact)
    small = slice(0, M // 3)                                                 # the rows a matrix-wide scale crushes
    assert np.sqrt((err[small] ** 2).mean()) < 0.2 * np.sqrt((err_m[small] ** 2).mean())
    # accumulators against a brute-force integer product
    assert (acc == R.Wq[:, :K].astype(np.int64) @ xq.astype(np.int64)).all()


def test_dequantize_rows_exact_small_case(oracle):
    y = oracle.dequantize_rows(np.array([3, -8, 5], np.int32), np.array([0.5, 2.0, 0.0], np.float32), 0.25, None)
    assert y.tolist() == [0.375, -4.0, 0.0]
    y = oracle.dequantize_rows(np.array([3, -8, 5], np.int32), np.array([0.5, 2.0, 0.0], np.float32), 0.25,
                               np.array([1, 2, 3], np.float32))
    assert y.tolist() == [1.375, -2.0, 3.0]
