"""GPU parity: q8_quantize_matrix, q8_gemv, q8_gemm_narrow against the CPU oracle (Section 3)."""
import numpy as np
import pytest
import torch

from parity import assert_close, assert_same, np_

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def q():
    import paper_1804_05038_amd as q
    return q


@pytest.fixture(scope="module")
def ctx(q):
    return q.Context()


def _w(rng, rows, cols, std=0.05):
    return (rng.standard_normal((rows, cols)) * std).astype(np.float32)


@pytest.mark.parametrize("rows,cols", [(768, 256), (3072, 512), (1024, 2048), (33, 620), (7, 5), (1, 16), (2500, 1000)])
def test_quantize_matrix_bit_exact(q, ctx, oracle, rows, cols):
    rng = np.random.default_rng(rows * 7 + cols)
    W = _w(rng, rows, cols)
    W[rng.integers(rows), rng.integers(cols)] = 0.0
    m = q.q8_quantize_matrix(ctx, W)
    Wq, s = oracle.quantize_matrix(W)
    assert m.ld == Wq.shape[1] and m.scale == float(s)
    assert_same(m.data, Wq, "Wq")


def test_quantize_matrix_zero_and_halfway(q, ctx, oracle):
    m = q.q8_quantize_matrix(ctx, np.zeros((4, 20), np.float32))
    assert m.scale == 1.0 and not np_(m.data).any()
    W = np.array([[127, -63.5, 0.5, 1.5, 2.5, 0], [-127, 63.5, -0.5, -1.5, -2.5, 3.5]], np.float32)
    m = q.q8_quantize_matrix(ctx, W)
    assert np_(m.data)[:, :6].tolist() == [[127, -64, 0, 2, 2, 0], [-127, 64, 0, -2, -2, 4]]


GEMV_SHAPES = [(768, 256), (3072, 512), (3072, 1024), (1024, 2048), (1000, 620), (5, 16), (37, 3000),
               (100, 8200), (131, 48), (50000, 512)]


@pytest.mark.parametrize("rows,cols", GEMV_SHAPES)
@pytest.mark.parametrize("use_bias", [False, True])
def test_gemv(q, ctx, oracle, rows, cols, use_bias):
    rng = np.random.default_rng(rows + cols)
    W = _w(rng, rows, cols)
    b = (rng.standard_normal(rows) * 0.01).astype(np.float32) if use_bias else None
    x = rng.standard_normal(cols).astype(np.float32)
    L = oracle.QLinear(W, b)
    M = q.q8_quantize_matrix(ctx, W)
    y, taps = q.q8_gemv(ctx, M, ctx.f32(x), ctx.f32(b), taps=True)
    y_ref, xq, xs, acc = L.gemv(x, taps=True)
    assert_same(taps["xq"][0], xq, "xq")
    assert float(taps["xscale"][0]) == float(xs)
    assert_same(taps["acc"][0], acc, "acc")
    assert_same(y, y_ref, "y (one multiply and one add per element: identical bits expected)")
    # taps off gives the same result
    assert_same(q.q8_gemv(ctx, M, ctx.f32(x), ctx.f32(b)), y_ref, "y, no taps")


def test_gemv_degenerate_inputs(q, ctx, oracle):
    rng = np.random.default_rng(0)
    W = _w(rng, 64, 128)
    L, M = oracle.QLinear(W), q.q8_quantize_matrix(ctx, W)
    for x in (np.zeros(128, np.float32), np.full(128, 1e-35, np.float32),
              np.eye(128, dtype=np.float32)[5] * -3, np.full(128, 7.0, np.float32)):
        y, taps = q.q8_gemv(ctx, M, ctx.f32(x), taps=True)
        y_ref, xq, xs, acc = L.gemv(x, taps=True)
        assert_same(taps["xq"][0], xq); assert float(taps["xscale"][0]) == float(xs)
        assert_same(taps["acc"][0], acc); assert_same(y, y_ref)
    # extreme accumulators: all +127 against all -127 over 2048 columns
    Wq = torch.full((16, 2048), 127, dtype=torch.int8, device=ctx.device)
    M2 = q.Mat(Wq, 2048, 1.0)
    y, taps = q.q8_gemv(ctx, M2, ctx.f32(np.full(2048, -1.0, np.float32)), taps=True)
    assert (np_(taps["acc"]) == -33032192).all()


@pytest.mark.parametrize("rows,cols", [(3072, 512), (1024, 2048), (1000, 620), (50, 16), (50000, 512)])
@pytest.mark.parametrize("n", [2, 5, 8])
def test_gemm_narrow_streaming(q, ctx, oracle, rows, cols, n):
    rng = np.random.default_rng(rows + cols + n)
    W = _w(rng, rows, cols)
    b = (rng.standard_normal(rows) * 0.01).astype(np.float32)
    X = rng.standard_normal((n, cols)).astype(np.float32) * rng.uniform(0.1, 10, (n, 1)).astype(np.float32)
    if n > 2:
        X[1] = 0
    L, M = oracle.QLinear(W, b), q.q8_quantize_matrix(ctx, W)
    Y, taps = q.q8_gemm_narrow(ctx, M, ctx.f32(X), ctx.f32(b), taps=True)
    Y_ref, xq, xs, acc = L.gemm_narrow(X, taps=True)
    assert_same(taps["xq"], xq, "xq"); assert_same(taps["xscale"], xs, "xscale")
    assert_same(taps["acc"], acc, "acc"); assert_same(Y, Y_ref, "Y")
    # column identity: the narrow product is n matrix-vector products
    y0 = q.q8_gemv(ctx, M, ctx.f32(X[0]), ctx.f32(b))
    assert_same(y0, np_(Y)[0], "column 0 vs gemv")


@pytest.mark.parametrize("rows,cols", [(50000, 512), (9001, 1024), (8300, 1012), (40003, 252), (17000, 500)])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7, 8])
def test_gemm_narrow_one_pass_over_a_large_matrix(q, ctx, oracle, rows, cols, n):
    """One product without taps over a matrix of more than 8 MB with rows of 256, 512 or 1024 bytes runs on the
    kernel without a loop (8 KB of consecutive rows per wave, totals over 16, 32 or 64 lanes per row): identical
    to the oracle and to the looping kernel (which the taps select)."""
    rng = np.random.default_rng(rows + cols + n)
    W = _w(rng, rows, cols)
    b = (rng.standard_normal(rows) * 0.01).astype(np.float32)
    X = rng.standard_normal((n, cols)).astype(np.float32) * rng.uniform(0.1, 10, (n, 1)).astype(np.float32)
    L, M = oracle.QLinear(W, b), q.q8_quantize_matrix(ctx, W)
    assert M.data.shape[0] * M.data.shape[1] >= 8 << 20 and M.data.shape[1] in (256, 512, 1024)
    Y_ref = L.gemm_narrow(X)
    assert_same(q.q8_gemm_narrow(ctx, M, ctx.f32(X), ctx.f32(b)), Y_ref, "Y, with bias")
    Y_taps, _ = q.q8_gemm_narrow(ctx, M, ctx.f32(X), ctx.f32(b), taps=True)
    assert_same(Y_taps, Y_ref, "Y from the looping kernel")
    assert_same(q.q8_gemm_narrow(ctx, M, ctx.f32(X)), oracle.QLinear(W).gemm_narrow(X), "Y, no bias")
    if n in (1, 5, 8):
        # the variant with one weight scale per row takes the same kernel
        R, rs = q.q8_quantize_matrix_rows(ctx, W)
        assert_same(q.q8_gemm_narrow_rows(ctx, R, rs, ctx.f32(X), ctx.f32(b)), oracle.QLinearRows(W, b).gemm_narrow(X), "Y, row scales")


@pytest.mark.parametrize("rows,cols,n", [(3072, 512, 50), (1024, 2048, 30), (1000, 620, 13), (100, 48, 9),
                                         (3072, 512, 60), (77, 1000, 70), (3072, 1024, 320), (130, 272, 129),
                                         (9000, 512, 130), (50000, 512, 40), (8200, 144, 257)])
def test_gemm_narrow_matrix_cores(q, ctx, oracle, rows, cols, n):
    rng = np.random.default_rng(rows + cols + n)
    W = _w(rng, rows, cols)
    b = (rng.standard_normal(rows) * 0.01).astype(np.float32)
    X = rng.standard_normal((n, cols)).astype(np.float32) * rng.uniform(0.1, 10, (n, 1)).astype(np.float32)
    X[3] = 0
    L, M = oracle.QLinear(W, b), q.q8_quantize_matrix(ctx, W)
    Y, taps = q.q8_gemm_narrow(ctx, M, ctx.f32(X), ctx.f32(b), taps=True)
    Y_ref, xq, xs, acc = L.gemm_narrow(X, taps=True)
    assert_same(taps["xq"], xq, "xq"); assert_same(taps["xscale"], xs, "xscale")
    assert_same(taps["acc"], acc, "acc"); assert_same(Y, Y_ref, "Y")
    assert_same(q.q8_gemm_narrow(ctx, M, ctx.f32(X), ctx.f32(b)), Y_ref, "Y, no taps")
    assert_same(q.q8_gemm_narrow(ctx, M, ctx.f32(X)), oracle.QLinear(W, None).gemm_narrow(X), "Y, no taps, no bias")


def test_argument_errors_are_reported_not_launched(q, ctx):
    W = q.q8_quantize_matrix(ctx, np.ones((4, 16), np.float32))
    x = ctx.f32(np.ones(20, np.float32))
    with pytest.raises(q.Q8Error) as e:
        q.q8_gemv(ctx, W, x[1:17])            # misaligned vector
    assert e.value.code == 3
    bad = q.Mat(W.data, 16, 1.0); bad.c.ld = 8
    with pytest.raises(q.Q8Error) as e:
        q.q8_gemv(ctx, bad, x[:16])
    assert e.value.code == 2
    with pytest.raises(q.Q8Error) as e:
        q.q8_gemm_narrow(ctx, W, ctx.f32(np.ones((2000, 16), np.float32)))
    assert e.value.code == 2


# ---- the variant with one weight scale per row -------------------------------------------

def _rows_case(rng, rows, cols):
    # rows of very different size, one zero row, one tiny row: per-row scales differ by orders of magnitude
    W = _w(rng, rows, cols) * np.logspace(-3, 0, rows, dtype=np.float32)[:, None]
    W[rows // 2] = 0.0
    if rows > 4:
        W[3] = 1e-36
    return W


@pytest.mark.parametrize("rows,cols", [(768, 256), (3072, 1024), (33, 620), (7, 5), (2500, 1000), (50000, 512)])
def test_quantize_matrix_rows_bit_exact(q, ctx, oracle, rows, cols):
    rng = np.random.default_rng(rows * 3 + cols)
    W = _rows_case(rng, rows, cols)
    M, rs = q.q8_quantize_matrix_rows(ctx, W)
    R = oracle.QLinearRows(W)
    assert_same(rs, R.row_scale, "row scales")
    assert_same(M.data, R.Wq, "Wq")


@pytest.mark.parametrize("rows,cols", [(3072, 512), (1024, 2048), (1000, 620), (50, 16), (37, 3001), (50000, 512)])
@pytest.mark.parametrize("n", [1, 5, 8])
def test_gemm_narrow_rows_streaming(q, ctx, oracle, rows, cols, n):
    if cols % 4 and n > 1:
        pytest.skip("several vectors need a leading dimension that is a multiple of 4")
    rng = np.random.default_rng(rows + cols + n + 1)
    W = _rows_case(rng, rows, cols)
    b = (rng.standard_normal(rows) * 0.01).astype(np.float32)
    X = rng.standard_normal((n, cols)).astype(np.float32) * rng.uniform(0.1, 10, (n, 1)).astype(np.float32)
    R = oracle.QLinearRows(W, b)
    M, rs = q.q8_quantize_matrix_rows(ctx, W)
    Y, taps = q.q8_gemm_narrow_rows(ctx, M, rs, ctx.f32(X), ctx.f32(b), taps=True)
    Y_ref, xq, xs, acc = R.gemm_narrow(X, taps=True)
    assert_same(taps["xq"], xq, "xq"); assert_same(taps["xscale"], xs, "xscale")
    assert_same(taps["acc"], acc, "acc"); assert_same(Y, Y_ref, "Y")
    assert_same(q.q8_gemm_narrow_rows(ctx, M, rs, ctx.f32(X)), oracle.QLinearRows(W).gemm_narrow(X), "Y, no taps, no bias")


@pytest.mark.parametrize("rows,cols,n", [(3072, 512, 50), (1024, 2048, 30), (1000, 620, 13), (3072, 1024, 320),
                                         (130, 272, 129), (9000, 512, 130)])
def test_gemm_narrow_rows_matrix_cores(q, ctx, oracle, rows, cols, n):
    rng = np.random.default_rng(rows + cols + n + 2)
    W = _rows_case(rng, rows, cols)
    b = (rng.standard_normal(rows) * 0.01).astype(np.float32)
    X = rng.standard_normal((n, cols)).astype(np.float32) * rng.uniform(0.1, 10, (n, 1)).astype(np.float32)
    X[3] = 0
    R = oracle.QLinearRows(W, b)
    M, rs = q.q8_quantize_matrix_rows(ctx, W)
    Y, taps = q.q8_gemm_narrow_rows(ctx, M, rs, ctx.f32(X), ctx.f32(b), taps=True)
    Y_ref, xq, xs, acc = R.gemm_narrow(X, taps=True)
    assert_same(taps["acc"], acc, "acc"); assert_same(Y, Y_ref, "Y")
    assert_same(q.q8_gemm_narrow_rows(ctx, M, rs, ctx.f32(X), ctx.f32(b)), Y_ref, "Y, no taps")
    assert_same(q.q8_gemm_narrow_rows(ctx, M, rs, ctx.f32(X)), oracle.QLinearRows(W).gemm_narrow(X), "Y, no taps, no bias")


def test_rows_variant_argument_errors(q, ctx):
    M, rs = q.q8_quantize_matrix_rows(ctx, np.ones((4, 16), np.float32))
    with pytest.raises(q.Q8Error) as e:
        q.q8_gemm_narrow_rows(ctx, M, None, ctx.f32(np.ones((1, 16), np.float32)))
    assert e.value.code == 1
