"""GPU parity of the panel / batched paths (more than 8 vectors, hypotheses of several sentences
side by side; Section 6's "batching"): every product on the int8 matrix cores.

Per-vector quantization makes a panel's result for vector j the result of the single-vector
call, so each case is checked twice: against the oracle (codes and sums bit-exact through the
taps, floats to 1e-5) and against this library's own streaming kernels (bit for bit).
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
    return q.Context(workspace_bytes=q.q8_workspace_bytes(max_n=160, max_l=256, max_rows=50000, max_ld=2048) + (64 << 20))


def _check_product(oracle, L, x_gpu, tap, j, what):
    xq, xs = oracle.quantize(x_gpu)
    assert_same(tap["xq"][j], xq, what + " xq")
    assert float(tap["xscale"][j]) == float(xs), what + " xscale"
    acc = oracle.accumulate(L.Wq, L.cols, xq)
    assert_same(tap["acc"][j], acc, what + " acc")
    return oracle.dequantize(acc, L.scale, xs, L.bias)


@pytest.mark.parametrize("I,H,n,tiled", [(512, 1024, 9, False), (512, 1024, 70, False), (2048, 1024, 33, False), (36, 20, 12, False),
                                         (620, 1000, 17, False), (256, 256, 130, False), (512, 1024, 70, True), (512, 1024, 145, True),
                                         (2048, 1024, 33, True), (256, 256, 130, True), (1024, 1000, 20, True)])
def test_gru_step_panel(q, ctx, oracle, I, H, n, tiled):
    p = synth.gru_cell(seed=0, I=I, H=H, n_batch=n)
    p["x"] = p["x"] * np.random.default_rng(n).uniform(0.1, 10, (n, 1)).astype(np.float32)
    g = oracle.QGru(p["Wx"], p["Wh"], p["bx"], p["bh"])
    G = q.GruWeights(gpu_mat(q, ctx, p["Wx"], tiled), gpu_mat(q, ctx, p["Wh"], tiled), ctx.f32(p["bx"]), ctx.f32(p["bh"]))
    x, h0 = ctx.f32(p["x"]), ctx.f32(p["h_prev"])
    h, taps = q.gru_step_q8(ctx, G, x, h0, taps=True)
    for j in range(0, n, max(1, n // 7)):
        gx = _check_product(oracle, g.Wx, p["x"][j], taps[0], j, "Wx")
        gh = _check_product(oracle, g.Wh, p["h_prev"][j], taps[1], j, "Wh")
        assert_close(h[j], oracle.gru_gates(gx, gh, p["h_prev"][j]), "h' (teacher-forced)")
        assert_close(h[j], g.step(p["x"][j], p["h_prev"][j]), "h' (free-running)")
    assert_same(q.gru_step_q8(ctx, G, x, h0), np_(h), "no taps")
    # the streaming kernel on groups of at most 8 vectors gives the same bits
    for j0 in (0, n - 5):
        assert_same(q.gru_step_q8(ctx, G, x[j0:j0 + 5].contiguous(), h0[j0:j0 + 5].contiguous()), np_(h)[j0:j0 + 5],
                    "panel vs streaming kernel")


@pytest.mark.parametrize("V,R,n,k", [(50000, 512, 20, 12), (300, 64, 9, 12), (1000, 512, 130, 5), (33658, 640, 11, 12),
                                     (129, 48, 40, 16)])
def test_output_layer_panel_given_t(q, ctx, oracle, V, R, n, k):
    p = synth.output_layer(seed=2, V=V, R=R, n_beam=n)
    L = oracle.QLinear(p["out.W"], p["out.b"])
    W = gpu_mat(q, ctx, p["out.W"])
    t = ctx.f32(p["t"])
    r = q.output_logits_q8(ctx, None, W, ctx.f32(p["out.b"]), t_in=t, k=k, taps=True)
    tap = r["taps"][3]
    for j in range(0, n, max(1, n // 6)):
        logits_ref = _check_product(oracle, L, p["t"][j], tap, j, "W_out")
        assert_same(r["logits"][j], logits_ref, "logits")
        lse, lp, idx = oracle.logsoftmax_topk(logits_ref, k)
        assert_close(r["lse"][j:j + 1], np.array([lse]), "lse")
        assert_same(r["topk_idx"][j], idx, "top-k indices")
        assert_close(r["topk_logp"][j], lp, "top-k logp")
    r2 = q.output_logits_q8(ctx, None, W, ctx.f32(p["out.b"]), t_in=t, k=k, want_logits=False)
    assert_same(r2["topk_idx"], np_(r["topk_idx"]), "logits in the workspace: same top-k")
    r8 = q.output_logits_q8(ctx, None, W, ctx.f32(p["out.b"]), t_in=t[:8].contiguous(), k=k)
    assert_same(r8["logits"], np_(r["logits"])[:8], "panel vs streaming kernel: logits")
    assert_same(r8["topk_idx"], np_(r["topk_idx"])[:8], "panel vs streaming kernel: top-k")
    assert_same(r8["topk_logp"], np_(r["topk_logp"])[:8])


def test_output_layer_panel_with_readout(q, ctx, oracle):
    n = 23
    p = synth.full_model(seed=4, V=3000, E=512, H=1024, A=64, R=512)
    m = oracle.OracleModel(p)
    rng = np.random.default_rng(n)
    s, y, c = (rng.standard_normal((n, d)).astype(np.float32) for d in (1024, 512, 2048))
    ro = q.ReadoutWeights(gpu_mat(q, ctx, p["ro.Ws"]), gpu_mat(q, ctx, p["ro.Wy"]), gpu_mat(q, ctx, p["ro.Wc"]),
                          ctx.f32(p["ro.b"]))
    W = gpu_mat(q, ctx, p["out.W"])
    r = q.output_logits_q8(ctx, ro, W, ctx.f32(p["out.b"]), s=ctx.f32(s), y_emb=ctx.f32(y), ctx_vec=ctx.f32(c),
                           k=12, taps=True)
    T = r["taps"]
    Ls = oracle.QLinear(p["ro.Ws"])
    for j in range(0, n, 4):
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
    r5 = q.output_logits_q8(ctx, ro, W, ctx.f32(p["out.b"]), s=ctx.f32(s[:5]), y_emb=ctx.f32(y[:5]), ctx_vec=ctx.f32(c[:5]), k=12)
    assert_same(r5["t"], np_(r["t"])[:5], "panel vs streaming kernels: t")
    assert_same(r5["topk_idx"], np_(r["topk_idx"])[:5]); assert_same(r5["topk_logp"], np_(r["topk_logp"])[:5])


@pytest.mark.parametrize("E,H,A,lens,beam,tiled", [(512, 1024, 1024, (30, 11, 50), 5, False), (36, 40, 28, (7, 1, 3, 12), 3, False),
                                                   (64, 64, 64, (5, 300), 2, True), (512, 1024, 1024, (9,) * 26, 5, False),
                                                   (512, 1024, 1024, (9,) * 26, 5, True), (512, 1024, 1024, (30, 11, 50), 5, True),
                                                   (512, 1024, 1024, (4,) * 67, 3, True), (512, 1024, 1024, (3, 5, 2) * 20, 5, True),
                                                   (64, 64, 64, (2, 7, 1) * 30, 3, False), (64, 64, 64, (3,) * 130, 7, False)])
def test_cgru_decoder_step_batch(q, ctx, oracle, E, H, A, lens, beam, tiled):
    """tiled: the weights also carry their tile-packed copies, which the panel's matrix-core kernels read;
    the single-sentence calls it is compared with read the rows."""
    S, L, n = len(lens), sum(lens), len(lens) * beam
    p = synth.cgru_step(seed=1, E=E, H=H, A=A, l=L, n_beam=n)
    m = oracle.OracleModel(p)
    w = q.CgruWeights(gpu_gru(q, ctx, p, "dec_r", tiled), gpu_mat(q, ctx, p["att.U"], tiled), ctx.f32(p["att.v"]),
                      gpu_gru(q, ctx, p, "dec_q", tiled))
    enc_h = ctx.f32(p["enc_h"])
    P = q.q8_gemm_narrow(ctx, gpu_mat(q, ctx, p["att.W"]), enc_h, ctx.f32(p["att.b"]))
    P_ref = m.attention_precompute(p["enc_h"])
    assert_same(P, P_ref, "P")
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    y, s0 = ctx.f32(p["y_emb"]), ctx.f32(p["s_prev"])
    r = q.cgru_decoder_step_batch_q8(ctx, w, P, enc_h, torch.tensor(off, device=ctx.device), beam, max(lens), y, s0)
    for si in range(S):
        lo, hi, sl = off[si], off[si + 1], slice(si * beam, (si + 1) * beam)
        # the single-sentence entry point on this sentence's slots: the same bits
        r1 = q.cgru_decoder_step_q8(ctx, w, P[lo:hi].contiguous(), enc_h[lo:hi].contiguous(), y[sl].contiguous(), s0[sl].contiguous())
        for key in ("s_mid", "ctx", "s"):
            assert_same(r[key][sl], np_(r1[key]), "sentence %d %s vs single-sentence call" % (si, key))
        assert_same(r["alpha"][sl, :hi - lo], np_(r1["alpha"]), "alpha")
        # and the oracle, free-running, on the sentence's first and last slot
        for j in (si * beam, (si + 1) * beam - 1):
            sm_o, al_o, cx_o, s_o = m.cgru_step(P_ref[lo:hi], p["enc_h"][lo:hi], p["y_emb"][j], p["s_prev"][j])
            assert_close(r["s_mid"][j], sm_o, "s'"); assert_close(r["alpha"][j, :hi - lo], al_o, "alpha")
            assert_close(r["ctx"][j], cx_o, "H_t"); assert_close(r["s"][j], s_o, "s")
    r2 = q.cgru_decoder_step_batch_q8(ctx, w, P, enc_h, torch.tensor(off, device=ctx.device), beam, max(lens), y, s0)
    assert_same(r2["s"], np_(r["s"]), "second call: arrival counters back at zero")


def _translate_all(q, ctx, m_gpu, m_ref, sents, beam, k, max_steps):
    got = q.q8_translate_batch(ctx, m_gpu, sents, beam=beam, k=k, max_steps=max_steps)
    finished = 0
    for src, (toks, score, steps) in zip(sents, got):
        r_toks, r_score, r_steps = m_ref.translate(src, beam=beam, topk=k, max_steps=max_steps)
        assert toks.tolist() == r_toks.tolist(), (src.tolist(), toks.tolist(), r_toks.tolist())
        assert abs(float(score) - float(r_score)) <= 1e-5 * max(1.0, abs(float(r_score)))
        assert steps == r_steps               # a finished sentence stops counting while the batch runs on
        t1, s1, st1 = q.q8_translate(ctx, m_gpu, src, beam=beam, k=k, max_steps=max_steps)
        assert t1.tolist() == toks.tolist() and np.float32(s1) == np.float32(score)
        finished += len(toks) < max_steps
    return finished


@pytest.mark.parametrize("V,E,H,A,R,beam,k,S", [(13, 16, 24, 20, 12, 5, 6, 4), (50, 32, 48, 40, 24, 3, 5, 7),
                                                (200, 64, 64, 32, 48, 5, 12, 3), (40, 36, 40, 28, 20, 8, 12, 2),
                                                (13, 16, 24, 20, 12, 1, 4, 11)])
def test_translate_batch_small_models(q, ctx, oracle, V, E, H, A, R, beam, k, S):
    p = synth.full_model(seed=V + beam, V=V, E=E, H=H, A=A, R=R, w_std=0.3, b_std=0.1)
    p["out.b"][0] += 1.5                 # make the end token frequent enough to finish hypotheses
    m_ref, m_gpu = oracle.OracleModel(p), q.Model.from_params(ctx, p)
    rng = np.random.default_rng(V + S)
    sents = [rng.integers(1, V, size=int(rng.integers(1, 12))).astype(np.int32) for _ in range(S)]
    finished = _translate_all(q, ctx, m_gpu, m_ref, sents, beam, k, max_steps=15)
    assert finished > 0 or V > 100       # some searches ended early while others went on


def test_translate_batch_full_size_model(q, ctx, oracle):
    p = synth.full_model(seed=4)
    m_ref, m_gpu = oracle.OracleModel(p), q.Model.from_params(ctx, p)
    sents = synth.sentences(seed=4, n=4, V=50000, min_len=5, max_len=14)
    _translate_all(q, ctx, m_gpu, m_ref, sents, beam=5, k=12, max_steps=4)


@pytest.mark.parametrize("E,H,lens", [(512, 1024, (12, 1, 30, 7)), (36, 40, (5, 5, 9, 2, 1, 17)), (100, 60, (3,) * 12 + (40,)),
                                      (512, 1024, (20,))])
def test_encoder_batch(q, ctx, oracle, E, H, lens):
    L = sum(lens)
    p = synth.encoder(seed=3, l=L, E=E, H=H)
    fwd, bwd = gpu_gru(q, ctx, p, "enc_fwd"), gpu_gru(q, ctx, p, "enc_bwd")
    X = ctx.f32(p["X"])
    enc = q.q8_encode_batch(ctx, fwd, bwd, X, list(lens))
    gf = oracle.QGru(p["enc_fwd.Wx"], p["enc_fwd.Wh"], p["enc_fwd.bx"], p["enc_fwd.bh"])
    gb = oracle.QGru(p["enc_bwd.Wx"], p["enc_bwd.Wh"], p["enc_bwd.bx"], p["enc_bwd.bh"])
    o = 0
    for l in lens:
        one = q.q8_encode(ctx, fwd, bwd, X[o:o + l].contiguous())
        assert_same(enc[o:o + l], np_(one), "sentence at row %d vs q8_encode" % o)
        # the oracle's recurrences, free-running, on this sentence
        hf, hb = np.zeros(H, np.float32), np.zeros(H, np.float32)
        ref = np.zeros((l, 2 * H), np.float32)
        for i in range(l):
            hf = gf.step(p["X"][o + i], hf); ref[i, H:] = hf
        for i in range(l - 1, -1, -1):
            hb = gb.step(p["X"][o + i], hb); ref[i, :H] = hb
        assert_close(enc[o:o + l], ref, "sentence at row %d vs oracle" % o)
        o += l


def test_output_layer_panel_ties(q, ctx, oracle):
    """Heavily tied logits overflow the survivor list and take the exact fallback, with the logits
    in the caller's row-major buffer or tile by tile in the workspace.  Equals: lowest index first."""
    V, R, n = 2500, 32, 9
    W = np.zeros((V, R), np.float32); W[:, 0] = 1.0
    b = np.zeros(V, np.float32)
    b[[5, 130, 131, 400, 2499]] = 2.0
    t = np.zeros((n, R), np.float32); t[:, 0] = 0.5
    Wm = gpu_mat(q, ctx, W)
    L = oracle.QLinear(W, b)
    for want in (False, True):
        r = q.output_logits_q8(ctx, None, Wm, ctx.f32(b), t_in=ctx.f32(t), k=12, want_logits=want)
        for j in range(n):
            lse, lp, idx = oracle.logsoftmax_topk(L.gemv(t[j]), 12)
            assert idx[:5].tolist() == [5, 130, 131, 400, 2499] and idx[5:].tolist() == list(range(0, 5)) + [6, 7]
            assert_same(r["topk_idx"][j], idx); assert_close(r["topk_logp"][j], lp)


@pytest.mark.parametrize("V,R,n,k", [(50000, 512, 20, 12), (3001, 512, 300, 12), (2000, 620, 250, 5), (777, 512, 9, 16),
                                     (5000, 640, 1000, 12), (100, 512, 12, 12), (3001, 512, 40, 1), (16, 512, 9, 16),
                                     (4097, 640, 161, 7)])
def test_output_layer_panel_persistent_kernel(q, ctx, oracle, V, R, n, k):
    """Tile-packed vocabulary matrix and no logits requested: the panel kernel that keeps the slots'
    codes in LDS and streams weight tiles (rows of 512 or 640 bytes)."""
    p = synth.output_layer(seed=2, V=V, R=R, n_beam=n)
    L = oracle.QLinear(p["out.W"], p["out.b"])
    W = q.q8_pack_tiles(ctx, q.q8_quantize_matrix(ctx, p["out.W"], ld_out=(R + 63) // 64 * 64))
    t = ctx.f32(p["t"])
    r = q.output_logits_q8(ctx, None, W, ctx.f32(p["out.b"]), t_in=t, k=k, want_logits=False)
    full = q.output_logits_q8(ctx, None, W, ctx.f32(p["out.b"]), t_in=t, k=k)          # stored logits: block kernel
    assert_same(r["topk_idx"], np_(full["topk_idx"]), "panel kernel vs block kernel: top-k")
    assert_same(r["topk_logp"], np_(full["topk_logp"])); assert_same(r["lse"], np_(full["lse"]))
    for j in sorted(set([0, n // 3, n - 1])):
        lse, lp, idx = oracle.logsoftmax_topk(L.gemv(p["t"][j]), k)
        assert_same(r["topk_idx"][j], idx, "top-k indices"); assert_close(r["topk_logp"][j], lp, "top-k logp")
        assert_close(r["lse"][j:j + 1], np.array([lse]), "lse")


def test_output_layer_panel_persistent_kernel_ties(q, ctx, oracle):
    """The panel path keeps no logits and computes those of the qualifying tiles a second time.  With
    nearly all logits equal every tile qualifies and the survivors overflow their list: the exact
    fallback (k rounds over all tiles) has to give the raised entries first, then the lowest indices."""
    V, R, n = 4100, 512, 11
    W = np.zeros((V, R), np.float32); W[:, 0] = 1.0
    b = np.zeros(V, np.float32)
    raised = [7, 130, 131, 2047, 4099]
    b[raised] = 2.0
    t = np.zeros((n, R), np.float32); t[:, 0] = 0.5
    Wm = q.q8_pack_tiles(ctx, q.q8_quantize_matrix(ctx, W, ld_out=512))
    L = oracle.QLinear(W, b)
    r = q.output_logits_q8(ctx, None, Wm, ctx.f32(b), t_in=ctx.f32(t), k=12, want_logits=False)
    for j in range(n):
        lse, lp, idx = oracle.logsoftmax_topk(L.gemv(t[j]), 12)
        assert idx.tolist() == raised + [0, 1, 2, 3, 4, 5, 6]
        assert_same(r["topk_idx"][j], idx); assert_close(r["topk_logp"][j], lp)
        assert_close(r["lse"][j:j + 1], np.array([lse]), "lse")


@pytest.mark.parametrize("dims,S,beam,l", [(dict(), 4, 5, 7), (dict(), 30, 5, 30), (dict(), 3, 3, 5),
                                           (dict(V=33658, E=620, H=1000, A=1000, R=620), 4, 5, 9),
                                           (dict(V=50, E=32, H=48, A=40, R=24, w_std=0.3), 6, 2, 5)])
def test_codes_travel_from_the_batched_step_to_the_output_layer(q, ctx, oracle, dims, S, beam, l):
    """cgru_decoder_step_batch_codes_q8 + output_logits_codes_q8 against the plain calls (identical bits);
    the three sets of codes against the oracle's quantization of the fp32 vectors they belong to."""
    p = synth.full_model(seed=12, **dims)
    m = q.Model.from_params(ctx, p)
    E, H = m.E_tgt.shape[1], m.dec.r.H
    n = S * beam
    rng = np.random.default_rng(S + l)
    enc_h = ctx.f32(rng.standard_normal((S * l, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    off = torch.arange(0, (S + 1) * l, l, dtype=torch.int32, device=ctx.device)
    y = ctx.f32(rng.standard_normal((n, E)).astype(np.float32))
    s = ctx.f32(rng.standard_normal((n, H)).astype(np.float32))
    res = []
    for use in (False, True):
        codes = (q.Codes(ctx, n, m.dec.r.Wx.ld), q.Codes(ctx, n, m.dec.q.Wx.ld), q.Codes(ctx, n, m.ro.W_s.ld)) if use else None
        r1 = q.cgru_decoder_step_batch_q8(ctx, m.dec, P, enc_h, off, beam, l, y, s, codes=codes)
        if use:
            assert all(c.valid for c in codes)
            for c, X in ((codes[0], y), (codes[1], r1["ctx"]), (codes[2], r1["s"])):
                for j in (0, n // 2, n - 1):
                    xq, xs = oracle.quantize(np_(X)[j])
                    K = X.shape[1]
                    assert_same(c.q[j, :K], xq, "codes of slot %d" % j)
                    assert not np_(c.q[j, K:]).any() and float(c.scale[j]) == float(xs)
        r2 = q.output_logits_q8(ctx, m.ro, m.W_out, m.b_out, s=r1["s"], y_emb=y, ctx_vec=r1["ctx"], k=12, codes=codes)
        res.append((r1["s"], r1["ctx"], r2["t"], r2["logits"], r2["lse"], r2["topk_logp"], r2["topk_idx"]))
    for a, b, what in zip(res[0], res[1], ("s", "ctx", "t", "logits", "lse", "topk_logp", "topk_idx")):
        assert_same(b, np_(a), what + ": with codes against without")


@pytest.mark.parametrize("dims,S,beam,l", [(dict(), 6, 5, 9), (dict(V=500, E=64, H=128, A=64, R=64, w_std=0.2, b_std=0.1), 20, 3, 5),
                                           (dict(V=700, E=620, H=1000, A=1000, R=620, w_std=0.2, b_std=0.1), 3, 5, 6)])
def test_codes_handed_from_the_batched_search_step_to_the_next_step(q, ctx, oracle, dims, S, beam, l):
    """A batched decoding loop in which q8_beam_update_batch_loop gathers the codes of the rows it gathers and
    cgru_decoder_step_batch_loop_q8 takes them in place of its quantization launch, against the loop that
    quantizes again: every state, context vector, top-k table and gathered row bit for bit at every step; the
    handed codes against the oracle's quantization of the rows.  At 620 / 1000 the gather has no room for them."""
    T = 6
    p = synth.full_model(seed=41, **dims)
    m = q.Model.from_params(ctx, p)
    E, H = m.E_tgt.shape[1], m.dec.r.H
    n = S * beam
    rng = np.random.default_rng(S + l)
    enc_h = ctx.f32(rng.standard_normal((S * l, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    off = torch.arange(0, (S + 1) * l, l, dtype=torch.int32, device=ctx.device)

    def loop(hand_on):
        states = torch.zeros(q.q8_beam_state_bytes(T) * S, dtype=torch.uint8, device=ctx.device)
        y, s = ctx.empty(n, E), ctx.empty(n, H)
        done = torch.zeros(S, dtype=torch.int32, device=ctx.device)
        q.q8_beam_init_batch(ctx, states, S, beam, T, enc_h, off, m.E_tgt, y, s, done)
        codes = [q.Codes(ctx, n, m.dec.r.Wx.ld), q.Codes(ctx, n, m.dec.q.Wx.ld), q.Codes(ctx, n, m.ro.W_s.ld)]
        if hand_on:
            codes.append(q.Codes(ctx, n, m.dec.r.Wh.ld))
        trace, used = [], 0
        for _ in range(T):
            given = hand_on and codes[0].c.valid == 2 and codes[3].c.valid == 2
            used += bool(given)
            if given:
                trace += [np_(codes[0].q), np_(codes[0].scale), np_(codes[3].q), np_(codes[3].scale)]
            r = q.cgru_decoder_step_batch_q8(ctx, m.dec, P, enc_h, off, beam, l, y, s, codes=codes)
            o = q.output_logits_q8(ctx, m.ro, m.W_out, m.b_out, s=r["s"], y_emb=y, ctx_vec=r["ctx"], k=8, want_logits=False,
                                   codes=codes[:3])
            q.q8_beam_update_batch(ctx, states, S, beam, T, o["topk_logp"], o["topk_idx"], r["s"], m.E_tgt, y, s, done,
                                   codes=(codes[2], codes[0], codes[3]) if hand_on else None,
                                   E_codes=m.E_tgt_codes if hand_on else None)
            trace += [np_(r["s"]), np_(r["ctx"]), np_(o["topk_logp"]), np_(o["topk_idx"]), np_(y), np_(s)]
        return trace, used, q.q8_beam_result_batch(ctx, states, S, T)

    ref, _, ref_res = loop(False)
    got, used, got_res = loop(True)
    fits = E // 4 + m.dec.r.Wx.ld // 16 + m.ro.W_s.ld // 16 <= 256
    assert used == (T - 1 if fits else 0)
    gi = iter(got)
    for step in range(T):
        if fits and step > 0:
            yq, ys, sq, ss = next(gi), next(gi), next(gi), next(gi)
            y_rows, s_rows = ref[6 * (step - 1) + 4], ref[6 * (step - 1) + 5]
            for j in (0, n // 2, n - 1):
                cq, cs = oracle.quantize(y_rows[j])
                assert_same(yq[j, :E], cq, "codes of y"); assert_same(ys[j:j + 1], np.array([cs], np.float32), "scale of y")
                cq, cs = oracle.quantize(s_rows[j])
                assert_same(sq[j, :H], cq, "codes of s"); assert_same(ss[j:j + 1], np.array([cs], np.float32), "scale of s")
                assert not yq[j, E:].any() and not sq[j, H:].any()
        for i in range(6):
            assert_same(next(gi), ref[6 * step + i], "step %d, output %d" % (step, i))
    for a, b in zip(got_res, ref_res):
        assert a[0].tolist() == b[0].tolist() and a[1:] == b[1:]


def _batched_step_with_codes(q, ctx, m, P, enc_h, off, beam, l, y, s):
    n = y.shape[0]
    codes = (q.Codes(ctx, n, m.dec.r.Wx.ld), q.Codes(ctx, n, m.dec.q.Wx.ld), q.Codes(ctx, n, m.ro.W_s.ld))
    r = q.cgru_decoder_step_batch_q8(ctx, m.dec, P, enc_h, off, beam, l, y, s, codes=codes)
    return {"s_mid": np_(r["s_mid"]), "s": np_(r["s"]), "ctx": np_(r["ctx"]), "alpha": np_(r["alpha"]),
            "sq": np_(codes[2].q), "ss": np_(codes[2].scale), "cq": np_(codes[1].q), "cs": np_(codes[1].scale)}


def _panel_case(q, ctx, S, beam, l, seed=31):
    p = synth.full_model(seed=seed)
    m = q.Model.from_params(ctx, p)
    E, H = m.E_tgt.shape[1], m.dec.r.H
    n = S * beam
    rng = np.random.default_rng(S + l)
    enc_h = ctx.f32(rng.standard_normal((S * l, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    off = torch.arange(0, (S + 1) * l, l, dtype=torch.int32, device=ctx.device)
    y = ctx.f32(rng.standard_normal((n, E)).astype(np.float32))
    s = ctx.f32((rng.standard_normal((n, H)) * rng.uniform(0.05, 3.0, (n, 1))).astype(np.float32))
    return m, P, enc_h, off, y, s


@pytest.mark.parametrize("S,beam,l", [(2, 5, 6), (64, 5, 12), (67, 5, 4), (12, 8, 9), (70, 5, 3)])
def test_panel_gru_in_one_launch_equals_products_and_gates_apart(q, ctx, oracle, S, beam, l):
    """The transitions of a batched step as one kernel each, whose blocks exchange their partial maxima for the
    codes of the new states (the default where the grid fits the device: up to 336 slots), against the same
    step with that form switched off (matrix-core products, then a gates kernel): the same bits, states and
    codes.  70 sentences x 5 = 350 slots is past the limit and runs the second form either way."""
    m, P, enc_h, off, y, s = _panel_case(q, ctx, S, beam, l)
    one = _batched_step_with_codes(q, ctx, m, P, enc_h, off, beam, l, y, s)
    again = _batched_step_with_codes(q, ctx, m, P, enc_h, off, beam, l, y, s)
    try:
        q.q8_attention_options(ctx, exchange=False)
        apart = _batched_step_with_codes(q, ctx, m, P, enc_h, off, beam, l, y, s)
    finally:
        q.q8_attention_options(ctx, exchange=True)
    q.q8_encode_check(ctx)
    for key in one:
        assert_same(one[key], apart[key], key + ": one launch against products and gates apart")
        assert_same(again[key], one[key], key + ": second call (exchange words cleared by the launch between)")
    j = one["s"].shape[0] - 1
    sq, ss = oracle.quantize(one["s"][j])
    assert_same(one["sq"][j, :sq.shape[0]], sq, "codes of the last slot's new state")
    assert float(one["ss"][j]) == float(ss)


def test_panel_gru_wait_that_gives_up_is_reported_and_the_next_step_is_good(q, ctx, oracle):
    """With a bound of one poll a block of the one-launch panel GRU gives up at once: the kernel still ends,
    q8_encode_check reports it once and clears the exchange words, and the next step with the default bound
    gives the first one's bits again."""
    m, P, enc_h, off, y, s = _panel_case(q, ctx, 40, 5, 5)
    good = _batched_step_with_codes(q, ctx, m, P, enc_h, off, 5, 5, y, s)
    q.q8_encode_check(ctx)
    try:
        q.q8_attention_options(ctx, exchange=True, spin_limit=1)
        _batched_step_with_codes(q, ctx, m, P, enc_h, off, 5, 5, y, s)
        with pytest.raises(q.Q8Error):
            q.q8_encode_check(ctx)
    finally:
        q.q8_attention_options(ctx, exchange=True, spin_limit=0)
    q.q8_encode_check(ctx)
    again = _batched_step_with_codes(q, ctx, m, P, enc_h, off, 5, 5, y, s)
    q.q8_encode_check(ctx)
    for key in good:
        assert_same(again[key], good[key], key + " after the abandoned run")


def _batched_search(q, ctx, m, P, enc_h, off, S, beam, l, T, fused, hand_on, k=8):
    """T steps of a batched search from its start; fused: output_logits_beam_batch_q8, else the output layer and
    q8_beam_update_batch apart.  Returns every step's states, contexts, top-k tables and gathered rows, and the result."""
    E, H = m.E_tgt.shape[1], m.dec.r.H
    n = S * beam
    states = torch.zeros(q.q8_beam_state_bytes(T) * S, dtype=torch.uint8, device=ctx.device)
    y, s = ctx.empty(n, E), ctx.empty(n, H)
    done = torch.zeros(S, dtype=torch.int32, device=ctx.device)
    q.q8_beam_init_batch(ctx, states, S, beam, T, enc_h, off, m.E_tgt, y, s, done)
    codes = [q.Codes(ctx, n, m.dec.r.Wx.ld), q.Codes(ctx, n, m.dec.q.Wx.ld), q.Codes(ctx, n, m.ro.W_s.ld)]
    if hand_on:
        codes.append(q.Codes(ctx, n, m.dec.r.Wh.ld))
    trace, used = [], 0
    for _ in range(T):
        used += bool(hand_on and codes[0].c.valid == 2 and codes[3].c.valid == 2)
        r = q.cgru_decoder_step_batch_q8(ctx, m.dec, P, enc_h, off, beam, l, y, s, codes=codes)
        if fused:
            o = q.output_logits_beam_batch_q8(ctx, m.ro, m.W_out, m.b_out, r["s"], y, r["ctx"], states, S, beam, T, m.E_tgt, s,
                                              done, k=k, codes=(codes[2], codes[0], codes[1]),
                                              s_next_codes=codes[3] if hand_on else None,
                                              E_codes=m.E_tgt_codes if hand_on else None)
        else:
            o = q.output_logits_q8(ctx, m.ro, m.W_out, m.b_out, s=r["s"], y_emb=y, ctx_vec=r["ctx"], k=k, want_logits=False,
                                   codes=codes[:3])
            q.q8_beam_update_batch(ctx, states, S, beam, T, o["topk_logp"], o["topk_idx"], r["s"], m.E_tgt, y, s, done,
                                   codes=(codes[2], codes[0], codes[3]) if hand_on else None,
                                   E_codes=m.E_tgt_codes if hand_on else None)
        trace += [np_(r["s"]), np_(r["ctx"]), np_(o["topk_logp"]), np_(o["topk_idx"]), np_(y), np_(s), np_(done)]
    return trace, used, q.q8_beam_result_batch(ctx, states, S, T)


@pytest.mark.parametrize("dims,S,beam,l,k,hand_on", [
    (dict(), 6, 5, 9, 12, True), (dict(), 64, 5, 7, 12, True), (dict(), 200, 5, 3, 12, True), (dict(), 2, 8, 5, 16, False),
    (dict(), 40, 1, 4, 3, True), (dict(V=700, E=620, H=1000, A=1000, R=620, w_std=0.2, b_std=0.1), 3, 5, 6, 8, True),
    (dict(V=500, E=64, H=128, A=64, R=64, w_std=0.2, b_std=0.1), 20, 3, 5, 8, True), (dict(), 1, 5, 6, 12, False)])
def test_search_steps_inside_the_panel_selection(q, ctx, oracle, dims, S, beam, l, k, hand_on):
    """output_logits_beam_batch_q8 (the sentences' search steps run in the selection kernel's launch where the
    vocabulary matrix is tile-packed with rows of 512 or 640 bytes and there are more than 8 slots; the other
    shapes here take its two-call path) against output layer and q8_beam_update_batch apart: every state,
    context vector, top-k table, gathered row and done flag bit for bit at every step, the same results, and
    as many steps that took their codes from the search step."""
    T = 5
    p = synth.full_model(seed=43, **dims)
    m = q.Model.from_params(ctx, p)
    H = m.dec.r.H
    rng = np.random.default_rng(S + l)
    enc_h = ctx.f32(rng.standard_normal((S * l, 2 * H)).astype(np.float32))
    P = torch.cat([q.q8_gemm_narrow(ctx, m.att_W, enc_h[o:o + 1000].contiguous(), m.att_b) for o in range(0, S * l, 1000)])
    off = torch.arange(0, (S + 1) * l, l, dtype=torch.int32, device=ctx.device)
    ref, ref_used, ref_res = _batched_search(q, ctx, m, P, enc_h, off, S, beam, l, T, False, hand_on, k)
    for rep in range(2):                              # (the second run finds the exchange words as the first left them)
        got, used, got_res = _batched_search(q, ctx, m, P, enc_h, off, S, beam, l, T, True, hand_on, k)
        q.q8_encode_check(ctx)
        assert used == ref_used
        for i, (a, b) in enumerate(zip(got, ref)):
            assert_same(a, b, "run %d, step %d, output %d" % (rep, i // 7, i % 7))
        for a, b in zip(got_res, ref_res):
            assert a[0].tolist() == b[0].tolist() and a[1:] == b[1:]


def test_panel_search_wait_that_gives_up_is_reported_and_the_next_search_is_good(q, ctx, oracle):
    """With a bound of one poll the block that runs a sentence's search step inside the panel selection may stop
    waiting for the sentence's other slots: the kernel still ends normally, q8_encode_check reports it once and
    clears the exchange words, and the same search run again gives the first result."""
    S, beam, l, T = 12, 5, 4, 4
    m = q.Model.from_params(ctx, synth.full_model(seed=43))
    rng = np.random.default_rng(5)
    enc_h = ctx.f32(rng.standard_normal((S * l, 2 * m.dec.r.H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    off = torch.arange(0, (S + 1) * l, l, dtype=torch.int32, device=ctx.device)
    good = _batched_search(q, ctx, m, P, enc_h, off, S, beam, l, T, True, True)
    q.q8_encode_check(ctx)
    gave_up = False
    try:
        q.q8_attention_options(ctx, exchange=True, spin_limit=1)
        for _ in range(5):                            # (a single poll can succeed when the other blocks are quick)
            _batched_search(q, ctx, m, P, enc_h, off, S, beam, l, T, True, True)
            try:
                q.q8_encode_check(ctx)
            except q.Q8Error:
                gave_up = True
                break
    finally:
        q.q8_attention_options(ctx, exchange=True, spin_limit=0)
    assert gave_up
    q.q8_encode_check(ctx)
    again = _batched_search(q, ctx, m, P, enc_h, off, S, beam, l, T, True, True)
    q.q8_encode_check(ctx)
    for a, b in zip(again[0], good[0]):
        assert_same(a, b, "after the abandoned run")
    for a, b in zip(again[2], good[2]):
        assert a[0].tolist() == b[0].tolist() and a[1:] == b[1:]
