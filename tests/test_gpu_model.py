"""GPU parity: gru_step_q8, cgru_decoder_step_q8, output_logits_q8, q8_encode against the
CPU oracle (Section 2, Eq. 1-6, driven by Section 3's product).

Protocol.  Integer tensors (int8 codes, int32 sums) must be bit-identical.  To keep that
checkable through a chain of float stages, every stage is also checked "teacher-forced":
the oracle stage is fed the GPU's own upstream fp32 vector, so an ulp of difference
upstream cannot hide behind, or be blamed for, a difference downstream.  The free-running
comparison (oracle on its own intermediate values) is asserted to the same 1e-5 bound.
"""
import numpy as np
import pytest
import torch

from parity import assert_close, assert_same, np_, gpu_gru, gpu_mat
from workloads import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def q():
    import paper_1804_05038_amd as q
    return q


@pytest.fixture(scope="module")
def ctx(q):
    return q.Context()


def _check_product(oracle, L, x_gpu, tap, j, what):
    """Teacher-forced check of one product: codes, scale and sums from the GPU's own input."""
    xq, xs = oracle.quantize(x_gpu)
    assert_same(tap["xq"][j], xq, what + " xq")
    assert float(tap["xscale"][j]) == float(xs), what + " xscale"
    acc = oracle.accumulate(L.Wq, L.cols, xq)
    assert_same(tap["acc"][j], acc, what + " acc")
    return oracle.dequantize(acc, L.scale, xs, L.bias)


# -------------------------------------------------------------------- GRU cell ----

@pytest.mark.parametrize("I,H,n", [(256, 256, 1), (256, 256, 5), (512, 1024, 1), (2048, 1024, 5), (512, 1024, 8),
                                   (36, 20, 3), (620, 1000, 2), (16, 8, 1)])
def test_gru_step(q, ctx, oracle, I, H, n):
    p = synth.gru_cell(seed=0, I=I, H=H, n_batch=n)
    g = oracle.QGru(p["Wx"], p["Wh"], p["bx"], p["bh"])
    G = q.GruWeights(gpu_mat(q, ctx, p["Wx"]), gpu_mat(q, ctx, p["Wh"]), ctx.f32(p["bx"]), ctx.f32(p["bh"]))
    assert_same(G.Wx.data, g.Wx.Wq); assert_same(G.Wh.data, g.Wh.Wq)
    h, taps = q.gru_step_q8(ctx, G, ctx.f32(p["x"]), ctx.f32(p["h_prev"]), taps=True)
    for j in range(n):
        gx = _check_product(oracle, g.Wx, p["x"][j], taps[0], j, "Wx")
        gh = _check_product(oracle, g.Wh, p["h_prev"][j], taps[1], j, "Wh")
        ref = oracle.gru_gates(gx, gh, p["h_prev"][j])
        assert_close(h[j], ref, "h' (teacher-forced)")
        assert_close(h[j], g.step(p["x"][j], p["h_prev"][j]), "h' (free-running)")
    assert_same(q.gru_step_q8(ctx, G, ctx.f32(p["x"]), ctx.f32(p["h_prev"])), np_(h), "no taps")


# ---------------------------------------------------------------- decoder step ----

def _decoder(q, ctx, oracle, p):
    m = oracle.OracleModel(p)
    w = q.CgruWeights(gpu_gru(q, ctx, p, "dec_r"), gpu_mat(q, ctx, p["att.U"]), ctx.f32(p["att.v"]),
                      gpu_gru(q, ctx, p, "dec_q"))
    return m, w


@pytest.mark.parametrize("E,H,A,l,n", [(512, 1024, 1024, 30, 1), (512, 1024, 1024, 30, 5), (36, 40, 28, 7, 3),
                                       (512, 1024, 1024, 1, 2), (620, 1000, 1000, 60, 8), (64, 64, 64, 300, 1)])
def test_cgru_decoder_step(q, ctx, oracle, E, H, A, l, n):
    p = synth.cgru_step(seed=1, E=E, H=H, A=A, l=l, n_beam=n)
    m, w = _decoder(q, ctx, oracle, p)
    enc_h = p["enc_h"]
    # attention precompute P = w(h_i) + b_att through the narrow product (bit-exact against the oracle)
    attW = gpu_mat(q, ctx, p["att.W"])
    P = q.q8_gemm_narrow(ctx, attW, ctx.f32(enc_h), ctx.f32(p["att.b"]))
    P_ref = m.attention_precompute(enc_h)
    assert_same(P, P_ref, "P")
    r = q.cgru_decoder_step_q8(ctx, w, P, ctx.f32(enc_h), ctx.f32(p["y_emb"]), ctx.f32(p["s_prev"]), taps=True)
    T = r["taps"]
    s_mid, ctxv, alpha, s = (np_(r[k]) for k in ("s_mid", "ctx", "alpha", "s"))
    for j in range(n):
        # Eq. 3, teacher-forced
        gx = _check_product(oracle, m.dec_r.Wx, p["y_emb"][j], T[0], j, "r.Wx")
        gh = _check_product(oracle, m.dec_r.Wh, p["s_prev"][j], T[1], j, "r.Wh")
        assert_close(s_mid[j], oracle.gru_gates(gx, gh, p["s_prev"][j]), "s'")
        # Eq. 6 from the GPU's s'
        a = _check_product(oracle, m.att_U, s_mid[j], T[2], j, "att_U")
        e, al, cx = oracle.attention(P_ref, enc_h, a, p["att.v"])
        assert_close(alpha[j], al, "alpha"); assert_close(ctxv[j], cx, "H_t")
        assert abs(float(alpha[j].astype(np.float64).sum()) - 1) < 1e-6
        # Eq. 4 from the GPU's H_t and s'
        gxq = _check_product(oracle, m.dec_q.Wx, ctxv[j], T[3], j, "q.Wx")
        ghq = _check_product(oracle, m.dec_q.Wh, s_mid[j], T[4], j, "q.Wh")
        assert_close(s[j], oracle.gru_gates(gxq, ghq, s_mid[j]), "s")
        # free-running oracle on its own intermediates
        sm_o, al_o, cx_o, s_o = m.cgru_step(P_ref, enc_h, p["y_emb"][j], p["s_prev"][j])
        assert_close(s_mid[j], sm_o, "s' free"); assert_close(alpha[j], al_o, "alpha free")
        assert_close(ctxv[j], cx_o, "H_t free"); assert_close(s[j], s_o, "s free")
    # taps off, and a second call on the same context (the arrival counters must be back at zero)
    for _ in range(2):
        r2 = q.cgru_decoder_step_q8(ctx, w, P, ctx.f32(enc_h), ctx.f32(p["y_emb"]), ctx.f32(p["s_prev"]))
        assert_same(r2["s"], s, "repeat s"); assert_same(r2["ctx"], ctxv, "repeat ctx")


def _step_with_codes(q, ctx, w, P, enc_h, y, s_prev, n):
    codes = (q.Codes(ctx, n, w.r.Wx.ld), q.Codes(ctx, n, w.q.Wx.ld))
    codes[1].q.fill_(77)        # pad bytes past C must come out zero whatever was there
    r = q.cgru_decoder_step_q8(ctx, w, P, enc_h, y, s_prev, codes=codes)
    assert codes[1].valid
    return {k: np_(r[k]) for k in ("s", "ctx", "alpha", "s_mid")} | {"cq": np_(codes[1].q), "cs": np_(codes[1].scale)}


@pytest.mark.parametrize("E,H,A,l,n", [(512, 1024, 1024, 30, 5), (512, 1024, 1024, 30, 1), (512, 1024, 1024, 1, 2), (512, 1024, 1024, 2, 3),
                                       (512, 1024, 1024, 10, 8), (512, 1024, 1024, 64, 5), (512, 1024, 1024, 65, 3),
                                       (512, 1024, 1024, 128, 2), (36, 40, 28, 7, 3), (64, 64, 64, 100, 4),
                                       (620, 1000, 1000, 60, 8), (64, 2048, 64, 3, 2)])
def test_attention_blocks_that_exchange_equal_the_finishing_block(q, ctx, oracle, E, H, A, l, n):
    """Eq. 5-6: the attention kernel whose blocks exchange energies and finish their own slices of the
    context vector gives the bits of the kernel whose last block per hypothesis finishes alone
    (weights, context vector, its codes and scale, the new state), call after call."""
    p = synth.cgru_step(seed=11, E=E, H=H, A=A, l=l, n_beam=n)
    _, w = _decoder(q, ctx, oracle, p)
    P = q.q8_gemm_narrow(ctx, gpu_mat(q, ctx, p["att.W"]), ctx.f32(p["enc_h"]), ctx.f32(p["att.b"]))
    enc_h, y, s_prev = ctx.f32(p["enc_h"]), ctx.f32(p["y_emb"]), ctx.f32(p["s_prev"])
    try:
        q.q8_attention_options(ctx, exchange=False)
        ref = _step_with_codes(q, ctx, w, P, enc_h, y, s_prev, n)
    finally:
        q.q8_attention_options(ctx, exchange=True)
    for rep in range(3):
        got = _step_with_codes(q, ctx, w, P, enc_h, y, s_prev, n)
        for key in ref:
            assert_same(got[key], ref[key], "%s (call %d)" % (key, rep))
    q.q8_encode_check(ctx)
    assert not ref["cq"][:, 2 * H:].any()


def test_attention_wait_that_gives_up_ends_the_kernel_and_is_reported(q, ctx, oracle):
    """With a bound of one poll per wait some block gives up at once: the kernel still ends normally,
    q8_encode_check reports it once, and the next call with the default bound is good again (the
    exchange words were cleared by the abandoned run too)."""
    p = synth.cgru_step(seed=12, E=512, H=1024, A=1024, l=30, n_beam=5)
    _, w = _decoder(q, ctx, oracle, p)
    P = q.q8_gemm_narrow(ctx, gpu_mat(q, ctx, p["att.W"]), ctx.f32(p["enc_h"]), ctx.f32(p["att.b"]))
    enc_h, y, s_prev = ctx.f32(p["enc_h"]), ctx.f32(p["y_emb"]), ctx.f32(p["s_prev"])
    good = _step_with_codes(q, ctx, w, P, enc_h, y, s_prev, 5)
    q.q8_encode_check(ctx)
    try:
        q.q8_attention_options(ctx, exchange=True, spin_limit=1)
        _step_with_codes(q, ctx, w, P, enc_h, y, s_prev, 5)
        with pytest.raises(q.Q8Error):
            q.q8_encode_check(ctx)
    finally:
        q.q8_attention_options(ctx, exchange=True, spin_limit=0)
    q.q8_encode_check(ctx)
    again = _step_with_codes(q, ctx, w, P, enc_h, y, s_prev, 5)
    q.q8_encode_check(ctx)
    for key in good:
        assert_same(again[key], good[key], key + " after the abandoned run")


def test_cgru_uniform_attention_special_case(q, ctx, oracle):
    p = synth.cgru_step(seed=5, E=64, H=64, A=32, l=9, n_beam=2)
    m, w = _decoder(q, ctx, oracle, p)
    P = np.tile(p["att.b"][None, :], (9, 1)).astype(np.float32)       # identical rows -> uniform weights
    r = q.cgru_decoder_step_q8(ctx, w, ctx.f32(P), ctx.f32(p["enc_h"]), ctx.f32(p["y_emb"]), ctx.f32(p["s_prev"]))
    np.testing.assert_allclose(np_(r["alpha"]), 1 / 9, rtol=1e-6)
    np.testing.assert_allclose(np_(r["ctx"])[0], p["enc_h"].astype(np.float64).mean(0), rtol=1e-5, atol=1e-6)


# ---------------------------------------------------------------- output layer ----

@pytest.mark.parametrize("packed", [False, True])
@pytest.mark.parametrize("V,R,n,k", [(50000, 512, 5, 12), (50000, 512, 1, 12), (300, 64, 3, 12), (129, 48, 8, 16),
                                     (1000, 512, 2, 1), (12, 16, 2, 12), (777, 1024, 4, 12), (33658, 640, 6, 12),
                                     (5000, 320, 8, 16), (4097, 256, 7, 12), (17, 128, 4, 12), (2049, 448, 3, 5),
                                     (40000, 384, 6, 12), (45000, 640, 5, 12)])      # the last: 28.8 MB, streamed rather than kept in the L2
def test_output_layer_given_t(q, ctx, oracle, V, R, n, k, packed):
    p = synth.output_layer(seed=2, V=V, R=R, n_beam=n)
    L = oracle.QLinear(p["out.W"], p["out.b"])
    W = gpu_mat(q, ctx, p["out.W"])
    if packed:
        if W.ld % 64:
            with pytest.raises(q.Q8Error):
                q.q8_pack_tiles(ctx, W)
            return
        W = q.q8_pack_tiles(ctx, W)
    r = q.output_logits_q8(ctx, None, W, ctx.f32(p["out.b"]), t_in=ctx.f32(p["t"]), k=k, taps=True)
    tap = r["taps"][3]
    for j in range(n):
        logits_ref = _check_product(oracle, L, p["t"][j], tap, j, "W_out")
        assert_same(r["logits"][j], logits_ref, "logits")
        lse, lp, idx = oracle.logsoftmax_topk(logits_ref, k)
        assert_close(r["lse"][j:j + 1], np.array([lse]), "lse")
        assert_same(r["topk_idx"][j], idx, "top-k indices")
        assert_close(r["topk_logp"][j], lp, "top-k logp")
    r2 = q.output_logits_q8(ctx, None, W, ctx.f32(p["out.b"]), t_in=ctx.f32(p["t"]), k=k, want_logits=False)
    assert_same(r2["topk_idx"], np_(r["topk_idx"]), "no logits written: same top-k")
    assert_same(r2["topk_logp"], np_(r["topk_logp"]))


def test_output_layer_ties_lowest_index_first(q, ctx, oracle):
    V, R = 700, 32
    W = np.zeros((V, R), np.float32); W[:, 0] = 1.0
    b = np.zeros(V, np.float32)
    b[[5, 130, 131, 400, 699]] = 2.0          # five equal maxima spread over several blocks
    b[[7, 300]] = 1.0
    t = np.zeros((2, R), np.float32); t[:, 0] = 0.5
    Wm = gpu_mat(q, ctx, W)
    r = q.output_logits_q8(ctx, None, Wm, ctx.f32(b), t_in=ctx.f32(t), k=12)
    L = oracle.QLinear(W, b)
    for j in range(2):
        lse, lp, idx = oracle.logsoftmax_topk(L.gemv(t[j]), 12)
        assert idx[:7].tolist() == [5, 130, 131, 400, 699, 7, 300]
        assert_same(r["topk_idx"][j], idx); assert_close(r["topk_logp"][j], lp)


@pytest.mark.parametrize("n", [1, 5])
def test_output_layer_with_readout(q, ctx, oracle, n):
    p = synth.full_model(seed=4, V=3000, E=512, H=1024, A=64, R=512)
    m = oracle.OracleModel(p)
    rng = np.random.default_rng(n)
    s, y, c = (rng.standard_normal((n, d)).astype(np.float32) for d in (1024, 512, 2048))
    ro = q.ReadoutWeights(gpu_mat(q, ctx, p["ro.Ws"]), gpu_mat(q, ctx, p["ro.Wy"]), gpu_mat(q, ctx, p["ro.Wc"]),
                          ctx.f32(p["ro.b"]))
    W = q.q8_pack_tiles(ctx, gpu_mat(q, ctx, p["out.W"]))
    r = q.output_logits_q8(ctx, ro, W, ctx.f32(p["out.b"]), s=ctx.f32(s), y_emb=ctx.f32(y), ctx_vec=ctx.f32(c),
                           k=12, taps=True)
    T = r["taps"]
    Ls = oracle.QLinear(p["ro.Ws"])
    for j in range(n):
        u1 = _check_product(oracle, Ls, s[j], T[0], j, "W_s")
        u2 = _check_product(oracle, m.ro_y, y[j], T[1], j, "W_y")
        u3 = _check_product(oracle, m.ro_c, c[j], T[2], j, "W_c")
        pre = ((u1 + u2) + u3) + p["ro.b"]
        t_gpu = np_(r["t"])[j]
        assert_close(t_gpu, np.tanh(pre.astype(np.float64)).astype(np.float32), "t (teacher-forced)")
        assert_close(t_gpu, m.readout(s[j], y[j], c[j]), "t (free-running)")
        logits = _check_product(oracle, m.out, t_gpu, T[3], j, "W_out")
        lse, lp, idx = oracle.logsoftmax_topk(logits, 12)
        assert_same(r["topk_idx"][j], idx); assert_close(r["topk_logp"][j], lp)


# --------------------------------------------------------------------- encoder ----

@pytest.mark.parametrize("l,E,H", [(50, 512, 1024), (1, 512, 1024), (5, 36, 40), (11, 100, 60)])
def test_encoder(q, ctx, oracle, l, E, H):
    p = synth.encoder(seed=3, l=l, E=E, H=H)
    m = oracle.OracleModel(p)
    fwd, bwd = gpu_gru(q, ctx, p, "enc_fwd"), gpu_gru(q, ctx, p, "enc_bwd")
    enc = np_(q.q8_encode(ctx, fwd, bwd, ctx.f32(p["X"])))
    ref = m.encode(p["X"])
    # teacher-forced along the recurrence: each oracle step starts from the GPU's previous state
    z = np.zeros(H, np.float32)
    for i in range(l):
        prev = enc[i - 1, H:] if i > 0 else z
        assert_close(enc[i, H:], m.enc_fwd.step(p["X"][i], prev), "forward state %d" % i)
        prev = enc[i + 1, :H] if i < l - 1 else z
        assert_close(enc[i, :H], m.enc_bwd.step(p["X"][i], prev), "backward state %d" % i)
    assert_close(enc, ref, "encoder states (free-running)")


@pytest.mark.parametrize("l,E,H", [(50, 512, 1024), (1, 512, 1024), (2, 512, 1024), (5, 36, 40), (11, 100, 64), (60, 620, 1000),
                                   (7, 64, 1032)])
def test_encoder_in_one_launch_equals_one_launch_per_position(q, ctx, oracle, l, E, H):
    """The recurrence of Eq. 1 as one cooperative launch (blocks hand the new state to each other through
    tagged words) and as l launches: the same bits; the one-launch form reports no abandoned wait."""
    p = synth.encoder(seed=3, l=l, E=E, H=H)
    fwd, bwd = gpu_gru(q, ctx, p, "enc_fwd"), gpu_gru(q, ctx, p, "enc_bwd")
    X = ctx.f32(p["X"])
    try:
        q.q8_encoder_options(ctx, one_launch=False)
        per_position = np_(q.q8_encode(ctx, fwd, bwd, X))
        q.q8_encoder_options(ctx, one_launch=True)
        for _ in range(3):                                   # the exchange buffers are reused from call to call
            one = np_(q.q8_encode(ctx, fwd, bwd, X))
            q.q8_encode_check(ctx)
            assert_same(one, per_position, "encoder states")
    finally:
        q.q8_encoder_options(ctx, one_launch=True)
    assert_close(one, oracle.OracleModel(p).encode(p["X"]), "encoder states (free-running)")


def test_encoder_wait_that_gives_up_ends_the_kernel_and_is_reported(q, ctx):
    """With a bound of one poll per wait some block gives up at once: the kernel still ends normally,
    q8_encode_check reports it, and the next call with the default bound is good again."""
    p = synth.encoder(seed=3, l=20, E=512, H=1024)
    fwd, bwd = gpu_gru(q, ctx, p, "enc_fwd"), gpu_gru(q, ctx, p, "enc_bwd")
    X = ctx.f32(p["X"])
    good = np_(q.q8_encode(ctx, fwd, bwd, X))
    q.q8_encode_check(ctx)
    try:
        q.q8_encoder_options(ctx, one_launch=True, spin_limit=1)
        q.q8_encode(ctx, fwd, bwd, X)
        with pytest.raises(q.Q8Error):
            q.q8_encode_check(ctx)
    finally:
        q.q8_encoder_options(ctx, one_launch=True, spin_limit=0)
    again = np_(q.q8_encode(ctx, fwd, bwd, X))
    q.q8_encode_check(ctx)
    assert_same(again, good, "encoder states after the abandoned run")


def test_output_layer_all_logits_equal_takes_the_exact_fallback(q, ctx, oracle):
    """Every logit ties: the survivor list of the pruned selection overflows and the exact rounds run."""
    V, R = 5000, 32
    W = np.zeros((V, R), np.float32); W[0, 0] = 1.0     # scale needs a non-zero entry; t has a zero there
    t = np.ones((2, R), np.float32); t[:, 0] = 0.0
    Wm = gpu_mat(q, ctx, W)
    r = q.output_logits_q8(ctx, None, Wm, None, t_in=ctx.f32(t), k=12)
    assert np_(r["topk_idx"]).tolist() == [list(range(12))] * 2
    np.testing.assert_allclose(np_(r["topk_logp"]), -np.log(V), rtol=1e-6)
