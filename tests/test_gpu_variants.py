"""GPU parity of the quantization variants beside the default scheme: the attention block with
8-bit energy and context products against the oracle's q8o_attention_q8.  (The variant with one
weight scale per row is covered with the other products.)"""
import numpy as np
import pytest

from parity import assert_close, assert_same, np_

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def q():
    import paper_1804_05038_amd as q
    return q


@pytest.fixture(scope="module")
def ctx(q):
    return q.Context(workspace_bytes=q.q8_workspace_bytes(max_n=1024, max_l=1024, max_rows=4096, max_ld=2048) + (64 << 20))


@pytest.mark.parametrize("l,A,C,n", [(30, 1024, 2048, 5), (30, 1024, 2048, 1), (1, 64, 40, 1), (7, 128, 100, 1),
                                     (50, 1000, 300, 3), (60, 2048, 512, 8), (300, 256, 64, 8), (13, 1024, 2048, 4)])
def test_attention_q8_against_oracle(q, ctx, oracle, l, A, C, n):
    rng = np.random.default_rng(l * 1000 + A + C + n)
    P = rng.standard_normal((l, A)).astype(np.float32)
    a = rng.standard_normal((n, A)).astype(np.float32)
    v = (rng.standard_normal(A) * 0.05).astype(np.float32)
    h = rng.standard_normal((l, C)).astype(np.float32)
    vm = q.q8_quantize_matrix(ctx, v[None, :])
    hT = q.q8_attention_states_q8(ctx, ctx.f32(h))
    e, alpha, cvec = q.q8_attention_q8(ctx, vm, hT, ctx.f32(P), ctx.f32(a))
    for b in range(n):
        e_ref, alpha_ref, ctx_ref, (vq, s_v), (hTq, s_h) = oracle.attention_q8(P, h, a[b], v)
        if b == 0:
            assert_same(vm.data[:, :A], vq, "v codes"); assert vm.scale == float(s_v)
            assert_same(hT.data, hTq, "transposed state codes"); assert hT.scale == float(s_h)
        assert_same(e[b], e_ref, "energies of hypothesis %d (integer sums, one multiply each)" % b)
        assert_close(alpha[b], alpha_ref, "alpha of hypothesis %d" % b)
        assert_close(cvec[b], ctx_ref, "context of hypothesis %d" % b)


def test_attention_q8_argument_errors(q, ctx):
    v = q.q8_quantize_matrix(ctx, np.ones((2, 16), np.float32))          # two rows: not an energy vector
    hT = q.q8_attention_states_q8(ctx, ctx.f32(np.ones((5, 8), np.float32)))
    with pytest.raises(q.Q8Error) as e:
        q.q8_attention_q8(ctx, v, hT, ctx.f32(np.ones((5, 16), np.float32)), ctx.f32(np.ones((1, 16), np.float32)))
    assert e.value.code == 2
    v1 = q.q8_quantize_matrix(ctx, np.ones((1, 16), np.float32))
    with pytest.raises(q.Q8Error) as e:                                   # six positions against states of five
        q.q8_attention_q8(ctx, v1, hT, ctx.f32(np.ones((6, 16), np.float32)), ctx.f32(np.ones((1, 16), np.float32)))
    assert e.value.code == 2
