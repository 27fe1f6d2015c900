"""Pins for the oracle's model functions (Section 2 of the paper, Eq. 1-6): library
special cases, closed forms and brute force."""
import itertools

import numpy as np
import pytest
import torch

from workloads import synth


def _rng_gru(seed, I, H, std=0.3):
    rng = np.random.default_rng(seed)
    f = lambda *s: (rng.standard_normal(s) * std).astype(np.float32)
    return f(3 * H, I), f(3 * H, H), f(3 * H), f(3 * H), f(I), f(H)


# ------------------------------------------------------------------ GRU cell ----

def test_fp32_gru_equals_torch_grucell(oracle):
    for seed, (I, H) in enumerate([(5, 7), (32, 16), (64, 64)]):
        Wx, Wh, bx, bh, x, h = _rng_gru(seed, I, H)
        cell = torch.nn.GRUCell(I, H)
        with torch.no_grad():
            cell.weight_ih.copy_(torch.from_numpy(Wx)); cell.weight_hh.copy_(torch.from_numpy(Wh))
            cell.bias_ih.copy_(torch.from_numpy(bx)); cell.bias_hh.copy_(torch.from_numpy(bh))
            ref = cell(torch.from_numpy(x)[None], torch.from_numpy(h)[None])[0].numpy()
        got = oracle.QGru(Wx, Wh, bx, bh).step(x, h, use_q8=False)
        np.testing.assert_allclose(got, ref, rtol=2e-6, atol=2e-6)


def test_q8_gru_close_to_fp32_gru_but_not_equal(oracle):
    Wx, Wh, bx, bh, x, h = _rng_gru(3, 128, 96, std=0.1)
    g = oracle.QGru(Wx, Wh, bx, bh)
    a, b = g.step(x, h, True), g.step(x, h, False)
    assert 0 < np.abs(a - b).max() < 0.02


def test_gates_closed_forms(oracle):
    H = 6
    rng = np.random.default_rng(0)
    h = rng.standard_normal(H).astype(np.float32)
    # update gate saturated at 1 keeps the state
    gx = np.zeros(3 * H, np.float32); gh = np.zeros(3 * H, np.float32)
    gx[H:2 * H] = 100.0
    assert (oracle.gru_gates(gx, gh, h) == h).all()
    # update gate saturated at 0 replaces it by the candidate tanh(gx_n + r*gh_n)
    gx[H:2 * H] = -100.0
    gx[2 * H:] = 0.5; gh[2 * H:] = 0.25; gx[:H] = 100.0          # r = 1
    np.testing.assert_allclose(oracle.gru_gates(gx, gh, h), np.tanh(0.75), rtol=1e-7)
    gx[:H] = -100.0                                               # r = 0: recurrent candidate term drops out
    np.testing.assert_allclose(oracle.gru_gates(gx, gh, h), np.tanh(0.5), rtol=1e-7)
    # all-zero weights: h' = (1-s(bz)) tanh(bxn + s(br) bhn) + s(bz) h
    bx = rng.standard_normal(3 * H).astype(np.float32); bh = rng.standard_normal(3 * H).astype(np.float32)
    g = oracle.QGru(np.zeros((3 * H, 4), np.float32), np.zeros((3 * H, H), np.float32), bx, bh)
    sig = lambda t: 1 / (1 + np.exp(-t.astype(np.float64)))
    b = (bx + bh).astype(np.float64)
    exp = (1 - sig(bx[H:2*H] + bh[H:2*H])) * np.tanh(bx[2*H:] + sig(bx[:H] + bh[:H]) * bh[2*H:]) + sig(bx[H:2*H] + bh[H:2*H]) * h
    for q8 in (True, False):
        np.testing.assert_allclose(g.step(rng.standard_normal(4), h, q8), exp, rtol=1e-6, atol=1e-7)


# ------------------------------------------------------------------- encoder ----

def _small_model(oracle, seed=0, V=11, E=6, H=8, A=5, R=7, std=0.4):
    p = synth.full_model(seed=seed, V=V, E=E, H=H, A=A, R=R, w_std=std, b_std=0.1)
    return p, oracle.OracleModel(p)


def test_encoder_single_position_and_layout(oracle):
    p, m = _small_model(oracle)
    x = p["E_src"][3:4]
    enc = m.encode(x)
    z = np.zeros(m.H, np.float32)
    assert (enc[0, :m.H] == m.enc_bwd.step(x[0], z)).all()       # backward state stacked first (Eq. 1)
    assert (enc[0, m.H:] == m.enc_fwd.step(x[0], z)).all()


def test_encoder_recurrence_and_reversal_symmetry(oracle):
    p, m = _small_model(oracle)
    X = p["E_src"][[1, 5, 2, 9, 4]]
    enc = m.encode(X)
    l, H = X.shape[0], m.H
    h = np.zeros(H, np.float32)
    for i in range(l):
        h = m.enc_fwd.step(X[i], h)
        assert (enc[i, H:] == h).all()
    h = np.zeros(H, np.float32)
    for i in reversed(range(l)):
        h = m.enc_bwd.step(X[i], h)
        assert (enc[i, :H] == h).all()
    # swapping the two cells and reversing the sentence swaps the two halves
    p2 = dict(p)
    for k in ("Wx", "Wh", "bx", "bh"):
        p2["enc_fwd." + k], p2["enc_bwd." + k] = p["enc_bwd." + k], p["enc_fwd." + k]
    enc2 = oracle.OracleModel(p2).encode(X[::-1].copy())
    assert (enc2[::-1, :H] == enc[:, H:]).all() and (enc2[::-1, H:] == enc[:, :H]).all()


# ----------------------------------------------------------------- attention ----

def test_attention_special_cases(oracle):
    rng = np.random.default_rng(1)
    l, A, C = 7, 12, 10
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    enc_h, a, v = f(l, C), f(A), f(A)
    # identical rows of P -> uniform weights, context = mean of the states
    P = np.tile(f(1, A), (l, 1))
    e, alpha, ctx = oracle.attention(P, enc_h, a, v)
    np.testing.assert_allclose(alpha, 1.0 / l, rtol=1e-6)
    np.testing.assert_allclose(ctx, enc_h.astype(np.float64).mean(0), rtol=1e-5, atol=1e-6)
    # v = 0 -> the same
    e, alpha, ctx = oracle.attention(f(l, A), enc_h, a, np.zeros(A, np.float32))
    assert (e == 0).all()
    np.testing.assert_allclose(alpha, 1.0 / l, rtol=1e-6)
    # saturated tanh: e_i = sum(v) for +inf-like P, -sum(v) for -inf-like P
    P = np.full((l, A), 50.0, np.float32); P[2] = -50.0
    e, alpha, ctx = oracle.attention(P, enc_h, np.zeros(A, np.float32), v)
    np.testing.assert_allclose(e[0], v.astype(np.float64).sum(), rtol=1e-6)
    np.testing.assert_allclose(e[2], -v.astype(np.float64).sum(), rtol=1e-6)
    # one position: weight 1, context is that state exactly
    e, alpha, ctx = oracle.attention(f(1, A), enc_h[:1], a, v)
    assert alpha.tolist() == [1.0] and (ctx == enc_h[0]).all()
    # a dominating energy picks out its state; weights are a distribution
    P = f(l, A) * 0.01; P[4] = 3.0
    vpos = np.full(A, 5.0, np.float32)
    e, alpha, ctx = oracle.attention(P, enc_h, np.zeros(A, np.float32), vpos)
    assert alpha.min() >= 0 and abs(alpha.astype(np.float64).sum() - 1) < 1e-6
    assert alpha[4] > 1 - 1e-6
    np.testing.assert_allclose(ctx, enc_h[4], rtol=1e-4, atol=1e-5)


def test_attention_softmax_matches_library(oracle):
    rng = np.random.default_rng(2)
    l, A, C = 30, 64, 16
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    P, enc_h, a, v = f(l, A), f(l, C), f(A), f(A)
    e, alpha, ctx = oracle.attention(P, enc_h, a, v)
    te = torch.tanh(torch.from_numpy(P).double() + torch.from_numpy(a).double()) @ torch.from_numpy(v).double()
    np.testing.assert_allclose(e, te.numpy(), rtol=1e-5, atol=1e-6)
    ta = torch.softmax(torch.from_numpy(e).double(), 0)
    np.testing.assert_allclose(alpha, ta.numpy(), rtol=1e-6)
    np.testing.assert_allclose(ctx, (ta[:, None] * torch.from_numpy(enc_h).double()).sum(0).numpy(), rtol=1e-5, atol=1e-6)


def test_cgru_step_is_r_then_attention_then_q(oracle):
    p, m = _small_model(oracle, seed=2)
    X = p["E_src"][[1, 2, 3, 4]]
    enc = m.encode(X)
    P = m.attention_precompute(enc)
    for i in range(4):
        assert (P[i] == m.att_W.gemv(enc[i])).all()
    y, s0 = p["E_tgt"][5], enc[0, :m.H].copy()
    s_mid, alpha, ctx, s = m.cgru_step(P, enc, y, s0)
    sm = m.dec_r.step(y, s0)
    assert (s_mid == sm).all()
    e, al, cx = oracle.attention(P, enc, m.att_U.gemv(sm), p["att.v"])
    assert (alpha == al).all() and (ctx == cx).all()
    assert (s == m.dec_q.step(cx, sm)).all()


# -------------------------------------------------------------- output layer ----

def test_logsoftmax_topk_against_sort_and_library(oracle):
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(5000) * 3).astype(np.float32)
    lse, lp, idx = oracle.logsoftmax_topk(x, 12)
    ref = torch.log_softmax(torch.from_numpy(x).double(), 0).numpy()
    order = np.argsort(-x, kind="stable")[:12]
    assert idx.tolist() == order.tolist()
    np.testing.assert_allclose(lp, ref[order], rtol=1e-6, atol=1e-6)
    assert abs(np.exp((x.astype(np.float64) - float(lse))).sum() - 1) < 1e-6
    assert (lp == x[idx] - lse).all()


def test_topk_ties_lowest_index_first(oracle):
    x = np.array([1, 5, 5, 0, 5, 2, 2, -1], np.float32)
    _, lp, idx = oracle.logsoftmax_topk(x, 6)
    assert idx.tolist() == [1, 2, 4, 5, 6, 0]
    x = np.zeros(20, np.float32)
    lse, lp, idx = oracle.logsoftmax_topk(x, 5)
    assert idx.tolist() == [0, 1, 2, 3, 4]
    np.testing.assert_allclose(lp, -np.log(20), rtol=1e-6)


def test_readout_and_output_compose(oracle):
    p, m = _small_model(oracle, seed=5)
    rng = np.random.default_rng(0)
    s, y, c = (rng.standard_normal(n).astype(np.float32) for n in (m.H, m.E, m.Cdim))
    t = m.readout(s, y, c)
    # b_t is added once, after the three separately quantized products
    Ls = oracle.QLinear(p["ro.Ws"])
    pre = ((Ls.gemv(s) + m.ro_y.gemv(y)) + m.ro_c.gemv(c)) + p["ro.b"]
    np.testing.assert_allclose(t, np.tanh(pre.astype(np.float64)), rtol=1e-6)
    logits, lse, lp, idx = m.output(t, 3)
    assert (logits == m.out.gemv(t)).all()
    lse2, lp2, idx2 = oracle.logsoftmax_topk(logits, 3)
    assert lse == lse2 and (lp == lp2).all() and (idx == idx2).all()


# --------------------------------------------------------------- beam search ----

def _step_logp(m, p, P, enc, s_prev, last_tok):
    y = p["E_tgt"][last_tok]
    s_mid, alpha, ctx, s = m.cgru_step(P, enc, y, s_prev)
    t = m.readout(s, y, ctx)
    V = m.out.rows
    logits, lse, lp, idx = m.output(t, V)
    full = np.empty(V, np.float32)
    full[idx] = lp
    return full, s


def test_beam_one_is_greedy(oracle):
    p, m = _small_model(oracle, seed=6, V=13)
    src = np.array([3, 7, 1, 12, 5], np.int32)
    toks, score, steps = m.translate(src, beam=1, topk=4, max_steps=6)
    enc = m.encode(p["E_src"][src]); P = m.attention_precompute(enc)
    s, last, total, exp = enc[0, :m.H].copy(), 0, np.float32(0), []
    for _ in range(6):
        lp, s = _step_logp(m, p, P, enc, s, last)
        last = int(np.argmax(lp))                                  # first maximum = lowest index
        total = np.float32(total + lp[last])
        if last == 0:
            break
        exp.append(last)
    assert toks.tolist() == exp and score == total


def test_wide_beam_equals_exhaustive_search(oracle):
    V, T = 4, 3
    for seed in (7, 8, 9):
        p, m = _small_model(oracle, seed=seed, V=V, std=0.8)
        src = np.array([1, 3, 2], np.int32)
        toks, score, steps = m.translate(src, beam=64, topk=V, max_steps=T)
        enc = m.encode(p["E_src"][src]); P = m.attention_precompute(enc)
        best = None

        def walk(prefix, s, last, total, depth):
            nonlocal best
            if depth == T:
                return
            lp, s2 = _step_logp(m, p, P, enc, s, last)
            for tok in range(V):
                sc = np.float32(total + lp[tok])
                if tok == 0:
                    if best is None or sc > best[0]:
                        best = (sc, list(prefix))
                else:
                    walk(prefix + [tok], s2, tok, sc, depth + 1)

        walk([], enc[0, :m.H].copy(), 0, np.float32(0), 0)
        assert best is not None
        assert score == best[0] and toks.tolist() == best[1]


def test_int8_step_close_to_fp32_step(oracle):
    """Same state, same previous word: the 8-bit engine's next-word distribution is a small
    perturbation of the 32-bit engine's (the paper's Section 5 finds outputs similar, not identical)."""
    p, m = _small_model(oracle, seed=10, V=50, E=32, H=48, A=40, R=24, std=0.15)
    src = np.array([4, 9, 30, 2, 17, 11], np.int32)
    X = p["E_src"][src]
    enc8, enc32 = m.encode(X, True), m.encode(X, False)
    assert 0 < np.abs(enc8 - enc32).max() < 0.05
    P = m.attention_precompute(enc32, False)
    y, s0 = p["E_tgt"][7], enc32[0, :m.H].copy()
    out = []
    for q8 in (True, False):
        s_mid, alpha, ctx, s = m.cgru_step(P, enc32, y, s0, q8)
        t = m.readout(s, y, ctx, q8)
        logits, lse, lp, idx = m.output(t, 50, q8)
        full = np.empty(50, np.float32); full[idx] = lp
        out.append(full)
    d = np.abs(out[0] - out[1]).max()
    assert 0 < d < 0.05


# ------------------------------------------------------------------ ensemble ----

def test_ensemble_logp_is_log_of_mean_probability(oracle):
    """Section 4's ensemble averages probabilities: checked against the library's logaddexp and
    against plain probabilities; the result is again a distribution."""
    rng = np.random.default_rng(20)
    V = 500
    lps = []
    for scale in (1.0, 3.0, 0.2):
        z = (rng.standard_normal(V) * scale).astype(np.float64)
        lps.append((z - np.log(np.exp(z).sum())).astype(np.float32))
    c2 = oracle.ensemble_logp(lps[:2])
    ref2 = np.logaddexp(lps[0].astype(np.float64), lps[1].astype(np.float64)) - np.log(2.0)
    np.testing.assert_allclose(c2, ref2, rtol=1e-6, atol=1e-7)
    c3 = oracle.ensemble_logp(lps)
    p3 = sum(np.exp(l.astype(np.float64)) for l in lps) / 3.0
    np.testing.assert_allclose(np.exp(c3.astype(np.float64)), p3, rtol=1e-6)
    assert abs(np.exp(c3.astype(np.float64)).sum() - 1.0) < 1e-6
    # not the average of log-probabilities (a plausible mistake): Jensen's inequality is strict here
    assert (c2 > (lps[0] + lps[1]) / 2 + 1e-4).any()
    # one model: the identity, up to one rounding of log(exp(x))
    np.testing.assert_allclose(oracle.ensemble_logp(lps[:1]), lps[0], rtol=1e-6)


def test_ensemble_of_a_model_with_itself_is_the_model(oracle):
    p, _ = _small_model(oracle, seed=21, V=30, std=0.3)
    p["out.b"][0] += 1.0                 # make some hypotheses finish
    m = oracle.OracleModel(p)
    rng = np.random.default_rng(21)
    for _ in range(4):
        src = rng.integers(1, 30, size=int(rng.integers(1, 8))).astype(np.int32)
        one = m.translate(src, beam=3, topk=5, max_steps=8)
        two = oracle.translate_ensemble([m, m], src, beam=3, topk=5, max_steps=8)
        assert one[0].tolist() == two[0].tolist() and one[2] == two[2]
        assert abs(float(one[1]) - float(two[1])) < 1e-5


def test_ensemble_beam_one_follows_the_mean_distribution(oracle):
    """Greedy decoding with two different models, replayed step by step from the models' own
    distributions: the token taken is the arg-max of the mean probability, and each model's
    decoder state advances with its own weights."""
    pa, ma = _small_model(oracle, seed=22, V=17, std=0.4)
    pb, mb = _small_model(oracle, seed=23, V=17, std=0.4)
    src = np.array([4, 9, 2, 16], np.int32)
    toks, score, steps = oracle.translate_ensemble([ma, mb], src, beam=1, topk=3, max_steps=5)
    st = []
    for p, m in ((pa, ma), (pb, mb)):
        enc = m.encode(p["E_src"][src])
        st.append([p, m, enc, m.attention_precompute(enc), enc[0, :m.H].copy()])
    last, total, exp = 0, np.float32(0), []
    differs = False
    for _ in range(5):
        lps = []
        for e in st:
            lp, e[4] = _step_logp(e[1], e[0], e[3], e[2], e[4], last)
            lps.append(lp)
        mean = (np.exp(lps[0].astype(np.float64)) + np.exp(lps[1].astype(np.float64))) / 2
        differs |= int(np.argmax(lps[0])) != int(np.argmax(lps[1]))
        last = int(np.argmax(mean))
        total = np.float32(total + np.float32(np.log(mean[last])))
        if last == 0:
            break
        exp.append(last)
    assert toks.tolist() == exp
    assert abs(float(score) - float(total)) < 1e-5
    assert differs          # the two models disagree somewhere, so averaging mattered


# ---- attention with its two activation products in 8 bits (variant) ------------------------

def test_attention_q8_hand_case(oracle):
    """P + a = 0 everywhere: T = 0 (scale 1, codes 0), e = 0, alpha = (1/2, 1/2) with codes (127, 127)
    and scale 0.5/127; states [[1, -1], [0.5, 0.25]] transposed: maximum 1, codes [[127, 64], [-127, 32]]."""
    P = np.array([[0.3, -0.2, 0.1], [1.0, 2.0, -3.0]], np.float32)
    a = np.zeros(3, np.float32)
    h = np.array([[1.0, -1.0], [0.5, 0.25]], np.float32)
    e, alpha, ctx, (vq, s_v), (hTq, s_h) = oracle.attention_q8(P * 0, h, a, np.array([0.5, -1.0, 0.25], np.float32))
    assert vq[0].tolist() == [64, -127, 32] and s_v == np.float32(1.0) / np.float32(127.0)
    assert hTq[:, :2].tolist() == [[127, 64], [-127, 32]] and s_h == np.float32(1.0) / np.float32(127.0)
    assert e.tolist() == [0.0, 0.0] and alpha.tolist() == [0.5, 0.5]
    s_a = np.float32(0.5) / np.float32(127.0)
    c = s_h * s_a
    assert ctx.tolist() == [np.float32(127 * (127 + 64)) * c, np.float32(127 * (-127 + 32)) * c]
    np.testing.assert_allclose(ctx, [0.75, -0.375], atol=0.005)


def test_attention_q8_single_position_and_energy(oracle):
    """One source position: alpha = 1 (code 127, scale 1/127), so the context is the state's int8 image;
    the energy is the plain 8-bit product of v with tanh(P + a), recomputed here with integer numpy."""
    rng = np.random.default_rng(21)
    A, Cc = 64, 40
    P = rng.standard_normal((1, A)).astype(np.float32)
    a = rng.standard_normal(A).astype(np.float32)
    v = (rng.standard_normal(A) * 0.05).astype(np.float32)
    h = rng.standard_normal((1, Cc)).astype(np.float32)
    e, alpha, ctx, (vq, s_v), (hTq, s_h) = oracle.attention_q8(P, h, a, v)
    assert alpha.tolist() == [1.0]
    assert (ctx == (hTq[:, 0].astype(np.float32) * np.float32(127.0)) * (s_h * (np.float32(1.0) / np.float32(127.0)))).all()
    assert np.abs(ctx - h[0]).max() <= float(s_h) / 2 * (1 + 1e-3)
    T = np.tanh((P[0] + a).astype(np.float64)).astype(np.float32)
    Tq, s_T = oracle.quantize(T)
    assert e[0] == np.float32(int(vq[0].astype(np.int64) @ Tq.astype(np.int64))) * (s_v * s_T)


def test_attention_q8_within_bound_of_float_attention(oracle):
    rng = np.random.default_rng(22)
    l, A, Cc = 30, 1024, 256
    P = rng.standard_normal((l, A)).astype(np.float32)
    a = rng.standard_normal(A).astype(np.float32)
    v = (rng.standard_normal(A) * 0.05).astype(np.float32)
    h = rng.standard_normal((l, Cc)).astype(np.float32)
    e, alpha, ctx, (vq, s_v), (hTq, s_h) = oracle.attention_q8(P, h, a, v)
    e_f, alpha_f, ctx_f = oracle.attention(P, h, a, v)
    T = np.tanh((P + a[None, :]).astype(np.float64))
    s_T = np.abs(T).max(axis=1) / 127
    bound = float(s_v) / 2 * np.abs(T).sum(axis=1) + s_T / 2 * np.abs(v).sum() + A * float(s_v) * s_T / 4
    assert (np.abs(e - e_f) <= bound * (1 + 1e-3) + 1e-6).all() and np.abs(e - e_f).max() > 0
    # softmax of the variant's own energies, by the library
    w = np.exp(e.astype(np.float64) - e.max())
    np.testing.assert_allclose(alpha, w / w.sum(), rtol=1e-6)
    # the context against the exact weighted sum with the variant's own alpha
    exact = alpha.astype(np.float64) @ h.astype(np.float64)
    s_a = alpha.max() / 127
    cb = float(s_h) / 2 * np.abs(alpha).sum() + s_a / 2 * np.abs(h).sum(axis=0) + l * float(s_h) * s_a / 4
    assert (np.abs(ctx - exact) <= cb * (1 + 1e-3) + 1e-6).all()
    assert np.abs(ctx - ctx_f).max() < 0.2 and np.abs(ctx - ctx_f).max() > 0
    # scaling v by a power of two scales the energies by exactly that factor
    e4 = oracle.attention_q8(P, h, a, v * 4)[0]
    assert (e4 == 4 * e).all()
