"""GPU parity: q8_beam_* and q8_translate (encoder, attention pre-computation, decoder steps,
output layer and beam search chained on the device) against the oracle's translate."""
import numpy as np
import pytest
import torch

from parity import assert_close, assert_same, np_
from workloads import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def q():
    import paper_1804_05038_amd as q
    return q


@pytest.fixture(scope="module")
def ctx(q):
    return q.Context()


def _check_sentence(q, ctx, m_gpu, m_ref, src, beam, k, max_steps):
    toks, score, steps = q.q8_translate(ctx, m_gpu, src, beam=beam, k=k, max_steps=max_steps)
    r_toks, r_score, r_steps = m_ref.translate(src, beam=beam, topk=k, max_steps=max_steps)
    assert toks.tolist() == r_toks.tolist(), (src.tolist(), toks.tolist(), r_toks.tolist())
    assert steps == r_steps
    assert abs(float(score) - float(r_score)) <= 1e-5 * max(1.0, abs(float(r_score)))
    return len(toks), steps


@pytest.mark.parametrize("V,E,H,A,R,beam,k", [(13, 16, 24, 20, 12, 1, 4), (13, 16, 24, 20, 12, 5, 6),
                                              (50, 32, 48, 40, 24, 3, 5), (200, 64, 64, 32, 48, 5, 12),
                                              (7, 8, 8, 8, 8, 5, 7), (40, 36, 40, 28, 20, 8, 12)])
def test_translate_small_models(q, ctx, oracle, V, E, H, A, R, beam, k):
    """Small vocabularies make the end token likely: hypotheses finish, the beam shrinks, searches end early."""
    p = synth.full_model(seed=V + beam, V=V, E=E, H=H, A=A, R=R, w_std=0.3, b_std=0.1)
    p["out.b"][0] += 1.5                 # make the end token frequent enough to finish hypotheses
    m_ref = oracle.OracleModel(p)
    m_gpu = q.Model.from_params(ctx, p)
    rng = np.random.default_rng(V)
    finished = 0
    for i in range(6):
        src = rng.integers(1, V, size=int(rng.integers(1, 12))).astype(np.int32)
        n, steps = _check_sentence(q, ctx, m_gpu, m_ref, src, beam, k, max_steps=15)
        finished += n < steps            # the result is a hypothesis that ended before the last step
    assert finished > 0 or V > 100       # the finishing path was exercised


def test_translate_full_size_model(q, ctx, oracle):
    """The benchmark's model (embedding 512, hidden 1024, vocabulary 50000), beam 5, a few steps."""
    p = synth.full_model(seed=4)
    m_ref = oracle.OracleModel(p)
    m_gpu = q.Model.from_params(ctx, p)
    src = synth.sentences(seed=4, n=3, V=50000, min_len=10, max_len=14)[0]
    _check_sentence(q, ctx, m_gpu, m_ref, src, beam=5, k=12, max_steps=6)
    _check_sentence(q, ctx, m_gpu, m_ref, src[:3], beam=1, k=12, max_steps=4)


def test_translate_config5_sentences_at_full_length(q, ctx, oracle):
    """The end-to-end workload itself: the full-size model, sentences of the benchmark's set (one of
    the shortest, one of the longest), beam 5, top-12, up to 100 steps, through q8_translate and
    q8_translate_batch against the oracle's search.  With random weights the end token is
    practically never chosen, so these are 100 steps of 5 hypotheses: long back-pointer walks, a
    hundred re-quantizations of drifting states, every "search over" read-back.  The token
    sequences are expected to be identical; should one differ, the oracle's own candidates must
    nearly tie at the step where they part (both sides round differently only in the last bit of
    a log-sum-exp)."""
    from concurrent.futures import ThreadPoolExecutor
    from parity import first_divergence_gap
    p = synth.full_model(seed=4)
    m_ref = oracle.OracleModel(p)
    m_gpu = q.Model.from_params(ctx, p)
    sents = synth.sentences(seed=4, n=200)
    lens = [len(x) for x in sents]
    pick = [sents[int(np.argmin(lens))], sents[int(np.argmax(lens))]]
    assert len(pick[0]) <= 12 and len(pick[1]) >= 58
    with ThreadPoolExecutor(2) as ex:        # the oracle's calls release the interpreter lock
        refs = list(ex.map(lambda src: m_ref.translate(src, beam=5, topk=12, max_steps=100), pick))
    single = [q.q8_translate(ctx, m_gpu, src, beam=5, k=12, max_steps=100) for src in pick]
    bctx = q.Context(workspace_bytes=q.q8_workspace_bytes(max_n=16, max_l=64, max_rows=50000, max_ld=2048) + (64 << 20))
    batch = q.q8_translate_batch(bctx, m_gpu, pick, beam=5, k=12, max_steps=100)
    for src, ref, one, bat in zip(pick, refs, single, batch):
        assert ref[2] >= 50                                  # a long search, as the workload has them
        for got, what in ((one, "q8_translate"), (bat, "q8_translate_batch")):
            if got[0].tolist() != ref[0].tolist():
                t, gap = first_divergence_gap(m_ref, p, src, got[0], ref[0])
                assert gap < 1e-4, "%s parts from the oracle at step %d where the oracle's gap is %.3g" % (what, t, gap)
                continue
            assert got[2] == ref[2], what
            assert abs(float(got[1]) - float(ref[1])) <= 1e-5 * max(1.0, abs(float(ref[1]))), what


def test_source_id_outside_the_table_is_a_zero_embedding(q, ctx):
    """Ids that reach the library on the device are not seen by the host: one outside [0, V_src) must
    read nothing and count as a zero vector, the same as an in-range id whose table row is zero."""
    V = 40
    p = synth.full_model(seed=9, V=V, E=32, H=48, A=40, R=24, w_std=0.3, b_std=0.1)
    p["E_src"][7] = 0.0
    m = q.Model.from_params(ctx, p)
    inside = torch.tensor([3, 7, 11, 7], dtype=torch.int32, device=ctx.device)
    res = [q.q8_translate(ctx, m, inside, beam=3, k=5, max_steps=8)]
    for bad in (V, V + 1000, -1, 2 ** 31 - 1, -2 ** 31):
        outside = torch.tensor([3, bad, 11, 7], dtype=torch.int32, device=ctx.device)
        res.append(q.q8_translate(ctx, m, outside, beam=3, k=5, max_steps=8))
    for r in res[1:]:
        assert r[0].tolist() == res[0][0].tolist() and r[1] == res[0][1] and r[2] == res[0][2]
    got = q.q8_translate_batch(ctx, m, [inside, torch.tensor([V + 5, 3], dtype=torch.int32, device=ctx.device)], beam=3, k=5, max_steps=4)
    assert len(got) == 2
    with pytest.raises(ValueError):
        q.q8_translate(ctx, m, [3, V, 11], beam=3, k=5, max_steps=8)       # host ids are checked before any launch


def test_translate_paper_dimensions(q, ctx, oracle):
    """Embedding 620, hidden 1000 (Section 4) and the smallest vocabulary of Table 4: no dimension is a
    multiple of 64, so every row is padded; single-sentence and batched drivers against the oracle."""
    p = synth.full_model(seed=6, V=33658, E=620, H=1000, A=1000, R=620)
    m_ref = oracle.OracleModel(p)
    m_gpu = q.Model.from_params(ctx, p)
    sents = synth.sentences(seed=6, n=3, V=33658, min_len=4, max_len=9)
    for src in sents[:2]:
        _check_sentence(q, ctx, m_gpu, m_ref, src, beam=5, k=12, max_steps=3)
    bctx = q.Context(workspace_bytes=q.q8_workspace_bytes(max_n=16, max_l=64, max_rows=33658, max_ld=2048) + (64 << 20))
    got = q.q8_translate_batch(bctx, m_gpu, sents, beam=5, k=12, max_steps=3)
    for src, (toks, score, steps) in zip(sents, got):
        r_toks, r_score, r_steps = m_ref.translate(src, beam=5, topk=12, max_steps=3)
        assert toks.tolist() == r_toks.tolist() and steps == r_steps
        assert abs(float(score) - float(r_score)) <= 1e-5 * max(1.0, abs(float(r_score)))


def test_beam_update_rules(q, ctx):
    """Hand-made top-k tables: ordering by (score, parent, token), finishing on token 0, dead slots."""
    n, k, E, H, T = 4, 4, 8, 8, 6
    E_tgt = ctx.f32(np.arange(10 * E, dtype=np.float32).reshape(10, E))
    s0 = ctx.f32(np.full(H, 7.0, np.float32))
    state = torch.zeros(q.q8_beam_state_bytes(T), dtype=torch.uint8, device=ctx.device)
    y, s, s_next = ctx.empty(n, E), ctx.empty(n, H), ctx.empty(n, H)
    q.q8_beam_init(ctx, state, n, T, s0, E_tgt, y, s)
    assert (np_(y) == np_(E_tgt)[0]).all() and (np_(s) == 7.0).all()
    # step 0: one live hypothesis; candidates (logp, token): equal scores tie-break on token id
    lp = ctx.f32(np.array([[-1.0, -1.0, -2.0, -3.0]] + [[-0.1] * 4] * 3, np.float32))
    ix = torch.tensor([[5, 3, 0, 9]] + [[1, 2, 3, 4]] * 3, dtype=torch.int32, device=ctx.device)
    s_step = ctx.f32(np.arange(n * H, dtype=np.float32).reshape(n, H))
    q.q8_beam_update(ctx, state, lp, ix, s_step, E_tgt, y, s_next)
    toks, score, steps, done = q.q8_beam_result(ctx, state, T)
    # kept: token 3 (-1), token 5 (-1), token 0 (-2, finishes), token 9 (-3); dead slots ignored
    assert steps == 1 and not done
    assert toks.tolist() == [] and score == np.float32(-2.0)            # the finished hypothesis is the result
    assert np_(y)[:3].tolist() == np_(E_tgt)[[3, 5, 9]].tolist()
    assert (np_(s_next)[:3] == np_(s_step)[0]).all()                      # all survivors descend from slot 0
    # step 1: three live, beam has 3 slots left; parent order breaks ties between equal scores
    lp = ctx.f32(np.array([[-1.0, -5, -6, -7], [-1.0, -5, -6, -7], [0.5, -5, -6, -7], [9, 9, 9, 9]], np.float32))
    ix = torch.tensor([[4, 1, 2, 3], [4, 1, 2, 3], [0, 1, 2, 3], [1, 1, 1, 1]], dtype=torch.int32, device=ctx.device)
    q.q8_beam_update(ctx, state, lp, ix, s_step, E_tgt, y, s)
    toks, score, steps, done = q.q8_beam_result(ctx, state, T)
    # scores: parent0 -2, parent1 -2, parent2 -2.5 (token 0: finishes, but -2.5 < -2 keeps the old result)
    assert steps == 2 and not done and toks.tolist() == [] and score == np.float32(-2.0)
    assert np_(y)[:2].tolist() == np_(E_tgt)[[4, 4]].tolist()
    assert (np_(s)[0] == np_(s_step)[0]).all() and (np_(s)[1] == np_(s_step)[1]).all()


def _decode_loop(q, c, m, P, enc_h, n, s0, T):
    """Bound calls of a search: init, decoder step, fused output layer + beam update."""
    E, H = m.E_tgt.shape[1], m.dec.r.H
    state = torch.zeros(q.q8_beam_state_bytes(T), dtype=torch.uint8, device=c.device)
    y, s = c.empty(n, E), c.empty(n, H)
    c0 = q.q8_beam_init(c, state, n, T, s0, m.E_tgt, y, s, bind=True)
    c1 = q.cgru_decoder_step_q8(c, m.dec, P, enc_h, y, s, bind=True)
    c2 = q.output_logits_beam_q8(c, m.ro, m.W_out, m.b_out, c1.out["s"], y, c1.out["ctx"], state, m.E_tgt, s, k=6, bind=True)
    return state, c0, c1, c2


def test_non_finite_logits_keep_the_search_inside_its_tables(q, ctx):
    """A NaN bias makes every logit NaN: none qualifies for the top-k tables, whose entries then
    carry token 0 and a non-finite log-probability whatever they held before (here: ids far outside
    the vocabulary).  The fused search step must still gather only rows of E_tgt and of the
    decoder states."""
    V, E, H, A, R, n, T = 500, 64, 128, 64, 64, 4, 6
    p = synth.full_model(seed=22, V=V, E=E, H=H, A=A, R=R, w_std=0.2, b_std=0.1)
    m = q.Model.from_params(ctx, p)
    rng = np.random.default_rng(4)
    enc_h = ctx.f32(rng.standard_normal((7, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))
    m.b_out = torch.full_like(m.b_out, float("nan"))
    state, c0, c1, c2 = _decode_loop(q, ctx, m, P, enc_h, n, s0, T)
    c2.out["topk_idx"].fill_(2 ** 31 - 1)
    c2.out["topk_logp"].fill_(float("nan"))
    c0.launch()
    E_rows = np_(m.E_tgt)
    for _ in range(3):
        c1.launch(); c2.launch()
    toks, score, steps, done = q.q8_beam_result(ctx, state, T)
    assert all(0 <= int(t) < V for t in toks)
    y = np_(c2.out["keep"][4])
    assert ((y[:, None, :] == E_rows[None, :, :]).all(-1)).any(-1).all()     # every row of y is a row of E_tgt


def test_fused_tail_equals_separate_calls_and_graph_replays(q, ctx, oracle):
    """output_logits_beam_q8 against output_logits_q8 + q8_beam_update, eagerly and from a HIP
    graph replayed several times with eager work between the replays."""
    V, E, H, A, R, n, T = 500, 64, 128, 64, 64, 4, 12
    p = synth.full_model(seed=21, V=V, E=E, H=H, A=A, R=R, w_std=0.2, b_std=0.1)
    m = q.Model.from_params(ctx, p)
    rng = np.random.default_rng(3)
    enc_h = ctx.f32(rng.standard_normal((9, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))

    # reference: separate calls
    state = torch.zeros(q.q8_beam_state_bytes(T), dtype=torch.uint8, device=ctx.device)
    y, s = ctx.empty(n, E), ctx.empty(n, H)
    q.q8_beam_init(ctx, state, n, T, s0, m.E_tgt, y, s)
    for _ in range(T):
        r = q.cgru_decoder_step_q8(ctx, m.dec, P, enc_h, y, s)
        o = q.output_logits_q8(ctx, m.ro, m.W_out, m.b_out, s=r["s"], y_emb=y, ctx_vec=r["ctx"], k=6, want_logits=False)
        q.q8_beam_update(ctx, state, o["topk_logp"], o["topk_idx"], r["s"], m.E_tgt, y, s)
    ref = q.q8_beam_result(ctx, state, T)

    # fused, eager
    st2, c0, c1, c2 = _decode_loop(q, ctx, m, P, enc_h, n, s0, T)
    c0.launch()
    for _ in range(T):
        c1.launch(); c2.launch()
    got = q.q8_beam_result(ctx, st2, T)
    assert got[0].tolist() == ref[0].tolist() and got[1] == ref[1] and got[2:] == ref[2:]

    # fused, captured: one graph holds the whole search; replay it three times
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        gctx = q.Context("cuda:0", stream=side)
        st3, g0, g1, g2 = _decode_loop(q, gctx, m, P, enc_h, n, s0, T)
        g0.launch(); g1.launch(); g2.launch()
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            g0.launch()
            for _ in range(T):
                g1.launch(); g2.launch()
    torch.cuda.synchronize()
    for rep in range(3):
        g.replay()
        torch.cuda.synchronize()
        got = q.q8_beam_result(gctx, st3, T)
        assert got[0].tolist() == ref[0].tolist() and got[1] == ref[1] and got[2:] == ref[2:], rep
        q.q8_gemv(ctx, m.att_W, enc_h[0])          # unrelated eager work between replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("dims", [dict(V=50000, E=512, H=1024, A=1024, R=512), dict(V=500, E=64, H=128, A=64, R=64),
                                  dict(V=700, E=620, H=1000, A=1000, R=620), dict(V=300, E=36, H=40, A=28, R=24)])
@pytest.mark.parametrize("n", [5, 1, 8])
def test_codes_handed_from_the_search_step_to_the_next_decoder_step(q, ctx, oracle, dims, n):
    """A decoding loop in which the search step gathers the codes of the rows it gathers (embedding rows
    quantized once, the readout's codes of the surviving states) and GRU r of the next step takes them
    (Eq. 3, Section 3: a vector's codes depend on the vector alone) against the loop that quantizes
    again: every state, context vector, top-k table, gathered row and code buffer bit for bit, step by
    step.  At 620 / 1000 the gather has no room for the codes and the loop quantizes as before."""
    T = 7
    p = synth.full_model(seed=31, **dims, **(dict(w_std=0.2, b_std=0.1) if dims["V"] < 1000 else {}))
    m = q.Model.from_params(ctx, p)
    E, H = dims["E"], dims["H"]
    rng = np.random.default_rng(5)
    enc_h = ctx.f32(rng.standard_normal((11, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))

    def loop(hand_on):
        state = torch.zeros(q.q8_beam_state_bytes(T), dtype=torch.uint8, device=ctx.device)
        y, s = ctx.empty(n, E), ctx.empty(n, H)
        codes = [q.Codes(ctx, n, m.dec.r.Wx.ld), q.Codes(ctx, n, m.dec.q.Wx.ld)]
        if hand_on:
            codes.append(q.Codes(ctx, n, m.dec.r.Wh.ld))
        q.q8_beam_init(ctx, state, n, T, s0, m.E_tgt, y, s)
        trace, used = [], 0
        for _ in range(T):
            given = hand_on and codes[0].c.valid == 2 and codes[2].c.valid == 2
            used += bool(given)
            if given:          # what GRU r is about to take: the codes of y and s as they are now
                trace += [np_(codes[0].q), np_(codes[0].scale), np_(codes[2].q), np_(codes[2].scale)]
            r = q.cgru_decoder_step_q8(ctx, m.dec, P, enc_h, y, s, codes=codes)
            o = q.output_logits_beam_q8(ctx, m.ro, m.W_out, m.b_out, r["s"], y, r["ctx"], state, m.E_tgt, s, k=12,
                                        codes=codes, E_codes=m.E_tgt_codes if hand_on else None)
            trace += [np_(r[k]) for k in ("s", "ctx", "alpha", "s_mid")] + [np_(o["topk_logp"]), np_(o["topk_idx"]), np_(y), np_(s)]
        return trace, used, q.q8_beam_result(ctx, state, T)

    ref, _, ref_res = loop(False)
    got, used, got_res = loop(True)
    fits = E // 4 + m.dec.r.Wx.ld // 16 + m.dec.r.Wh.ld // 16 <= 256
    assert used == (T - 1 if fits else 0)
    # the code buffers in `got` have no counterpart in `ref`: check them against the oracle's quantization of the rows
    gi = iter(got)
    for step in range(T):
        if fits and step > 0:
            yq, ys, sq, ss = next(gi), next(gi), next(gi), next(gi)
            y_rows, s_rows = ref[8 * (step - 1) + 6], ref[8 * (step - 1) + 7]
            for j in range(n):
                cq, cs = oracle.quantize(y_rows[j])
                assert_same(yq[j, :E], cq, "codes of y"); assert_same(ys[j:j + 1], np.array([cs], np.float32), "scale of y")
                assert not yq[j, E:].any()
                cq, cs = oracle.quantize(s_rows[j])
                assert_same(sq[j, :H], cq, "codes of s"); assert_same(ss[j:j + 1], np.array([cs], np.float32), "scale of s")
                assert not sq[j, H:].any()
        for i in range(8):
            assert_same(next(gi), ref[8 * step + i], "step %d, output %d" % (step, i))
    assert got_res[0].tolist() == ref_res[0].tolist() and got_res[1:] == ref_res[1:]


def test_translate_with_and_without_the_embedding_codes(q, ctx, oracle):
    """q8_translate hands codes from the search step to the next decoder step when the model brings its
    embeddings' codes; without them it quantizes in every step.  Same tokens, score bits and step count."""
    p = synth.full_model(seed=33, V=900, E=64, H=128, A=64, R=64, w_std=0.2, b_std=0.1)
    m = q.Model.from_params(ctx, p)
    srcs = synth.sentences(seed=8, n=4, V=900, min_len=3, max_len=12)
    with_codes = [q.q8_translate(ctx, m, src, beam=5, k=8, max_steps=20) for src in srcs]
    keep = m.c.E_tgt_codes
    m.c.E_tgt_codes = type(keep)()
    try:
        without = [q.q8_translate(ctx, m, src, beam=5, k=8, max_steps=20) for src in srcs]
    finally:
        m.c.E_tgt_codes = keep
    for a, b in zip(with_codes, without):
        assert a[0].tolist() == b[0].tolist() and np.float32(a[1]).tobytes() == np.float32(b[1]).tobytes() and a[2] == b[2]


def test_search_step_wait_that_gives_up_is_reported_and_the_next_search_is_good(q, ctx, oracle):
    """With a bound of one poll the block that runs the search step inside the selection kernel may
    stop waiting for the other hypotheses' k best: the kernel still ends normally, q8_encode_check
    reports it once and clears the exchange words, and the same search run again gives the result
    of the separate calls."""
    V, E, H, A, R, n, T = 500, 64, 128, 64, 64, 4, 12
    p = synth.full_model(seed=21, V=V, E=E, H=H, A=A, R=R, w_std=0.2, b_std=0.1)
    m = q.Model.from_params(ctx, p)
    rng = np.random.default_rng(3)
    enc_h = ctx.f32(rng.standard_normal((9, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))
    st, c0, c1, c2 = _decode_loop(q, ctx, m, P, enc_h, n, s0, T)

    def search():
        c0.launch()
        for _ in range(T):
            c1.launch(); c2.launch()
        return q.q8_beam_result(ctx, st, T)

    good = search()
    q.q8_encode_check(ctx)
    gave_up = False
    try:
        q.q8_attention_options(ctx, exchange=True, spin_limit=1)
        for _ in range(5):                         # (a single poll can succeed when the other blocks are quick)
            search()
            try:
                q.q8_encode_check(ctx)
            except q.Q8Error:
                gave_up = True
                break
    finally:
        q.q8_attention_options(ctx, exchange=True, spin_limit=0)
    assert gave_up
    q.q8_encode_check(ctx)
    again = search()
    q.q8_encode_check(ctx)
    assert again[0].tolist() == good[0].tolist() and again[1:] == good[1:]


def test_two_contexts_on_two_streams(q, ctx, oracle):
    """Independent contexts (own stream, own workspace) translate concurrently and agree with the oracle."""
    p = synth.full_model(seed=33, V=60, E=32, H=48, A=40, R=24, w_std=0.3, b_std=0.1)
    p["out.b"][0] += 1.0
    m_ref = oracle.OracleModel(p)
    m = q.Model.from_params(ctx, p)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctxs = [q.Context("cuda:0", stream=st) for st in streams]
    rng = np.random.default_rng(5)
    for i in range(4):
        srcs = [rng.integers(1, 60, size=int(rng.integers(2, 10))).astype(np.int32) for _ in ctxs]
        outs = []
        for c, st, src in zip(ctxs, streams, srcs):
            with torch.cuda.stream(st):
                outs.append(q.q8_translate(c, m, src, beam=4, k=6, max_steps=10))
        for (toks, score, steps), src in zip(outs, srcs):
            r_toks, r_score, r_steps = m_ref.translate(src, beam=4, topk=6, max_steps=10)
            assert toks.tolist() == r_toks.tolist() and steps == r_steps


@pytest.mark.parametrize("V,dims_a,dims_b,beam,k", [(13, (16, 24, 20, 12), (16, 24, 20, 12), 3, 5),
                                                    (50, (32, 48, 40, 24), (16, 24, 20, 12), 5, 6),
                                                    (200, (64, 64, 32, 48), (36, 40, 28, 20), 5, 12)])
def test_translate_ensemble_of_two_models(q, ctx, oracle, V, dims_a, dims_b, beam, k):
    """Section 4's ensemble: two models (of different sizes) sharing the vocabulary, probabilities
    averaged before the top-k; the whole search against the oracle's."""
    ps = []
    for seed, (E, H, A, R) in ((V + 1, dims_a), (V + 2, dims_b)):
        p = synth.full_model(seed=seed, V=V, E=E, H=H, A=A, R=R, w_std=0.3, b_std=0.1)
        p["out.b"][0] += 1.2
        ps.append(p)
    refs = [oracle.OracleModel(p) for p in ps]
    gpus = [q.Model.from_params(ctx, p) for p in ps]
    rng = np.random.default_rng(V)
    finished = differs = 0
    for i in range(5):
        src = rng.integers(1, V, size=int(rng.integers(1, 10))).astype(np.int32)
        toks, score, steps = q.q8_translate_ensemble(ctx, gpus, src, beam=beam, k=k, max_steps=12)
        r_toks, r_score, r_steps = oracle.translate_ensemble(refs, src, beam=beam, topk=k, max_steps=12)
        assert toks.tolist() == r_toks.tolist(), (src.tolist(), toks.tolist(), r_toks.tolist())
        assert steps == r_steps
        assert abs(float(score) - float(r_score)) <= 1e-5 * max(1.0, abs(float(r_score)))
        finished += len(toks) < steps
        differs += toks.tolist() != q.q8_translate(ctx, gpus[0], src, beam=beam, k=k, max_steps=12)[0].tolist()
    assert finished > 0 and differs > 0       # searches ended early, and the second model changed results
    # one model through the ensemble entry point is the single-model search
    one = q.q8_translate_ensemble(ctx, gpus[:1], src, beam=beam, k=k, max_steps=12)
    assert one[0].tolist() == q.q8_translate(ctx, gpus[0], src, beam=beam, k=k, max_steps=12)[0].tolist()


def test_translate_ensemble_full_size(q, ctx, oracle):
    pa, pb = synth.full_model(seed=4), synth.full_model(seed=14)
    refs = [oracle.OracleModel(pa), oracle.OracleModel(pb)]
    gpus = [q.Model.from_params(ctx, pa), q.Model.from_params(ctx, pb)]
    src = synth.sentences(seed=4, n=1, V=50000, min_len=6, max_len=8)[0]
    ectx = q.Context(workspace_bytes=q.q8_workspace_bytes() + q.q8_translate_ensemble_bytes(gpus, 16) + (1 << 20))
    toks, score, steps = q.q8_translate_ensemble(ectx, gpus, src, beam=5, k=12, max_steps=3)
    r_toks, r_score, r_steps = oracle.translate_ensemble(refs, src, beam=5, topk=12, max_steps=3)
    assert toks.tolist() == r_toks.tolist() and steps == r_steps
    assert abs(float(score) - float(r_score)) <= 1e-5 * max(1.0, abs(float(r_score)))


@pytest.mark.parametrize("dims,n,l", [(dict(), 5, 30), (dict(), 1, 7), (dict(), 8, 60),
                                      (dict(V=33658, E=620, H=1000, A=1000, R=620), 5, 12),
                                      (dict(V=50, E=32, H=48, A=40, R=24, w_std=0.3), 3, 5)])
def test_codes_travel_from_the_decoder_step_to_the_output_layer(q, ctx, oracle, dims, n, l):
    """cgru_decoder_step_codes_q8 + output_logits_beam_codes_q8 against the plain calls (identical bits)
    and the codes they hand over against the oracle's quantization of the same fp32 vectors."""
    p = synth.full_model(seed=11, **dims)
    m = q.Model.from_params(ctx, p)
    E, H = m.E_tgt.shape[1], m.dec.r.H
    rng = np.random.default_rng(n + l)
    enc_h = ctx.f32(rng.standard_normal((l, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    y = ctx.f32(rng.standard_normal((n, E)).astype(np.float32))
    s = ctx.f32(rng.standard_normal((n, H)).astype(np.float32))
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))
    res = []
    for use in (False, True):
        st = torch.zeros(q.q8_beam_state_bytes(20), dtype=torch.uint8, device=ctx.device)
        yy, ss = y.clone(), s.clone()
        q.q8_beam_init(ctx, st, n, 20, s0, m.E_tgt, yy, ss)
        yy.copy_(y); ss.copy_(s)
        codes = (q.Codes(ctx, n, m.dec.r.Wx.ld), q.Codes(ctx, n, m.dec.q.Wx.ld)) if use else None
        r1 = q.cgru_decoder_step_q8(ctx, m.dec, P, enc_h, yy, ss, codes=codes)
        if use:
            assert codes[0].valid and codes[1].valid
            for c, X in ((codes[0], y), (codes[1], r1["ctx"])):
                for j in range(n):
                    xq, xs = oracle.quantize(np_(X)[j])
                    K = X.shape[1]
                    assert_same(c.q[j, :K], xq, "codes of vector %d" % j)
                    assert not np_(c.q[j, K:]).any() and float(c.scale[j]) == float(xs)
        r2 = q.output_logits_beam_q8(ctx, m.ro, m.W_out, m.b_out, r1["s"], yy, r1["ctx"], st, m.E_tgt, ss, k=12, codes=codes)
        res.append((r1["s"], r1["ctx"], r2["topk_logp"], r2["topk_idx"], yy, ss))
    for a, b, what in zip(res[0], res[1], ("s", "ctx", "topk_logp", "topk_idx", "y_emb", "s_next")):
        assert_same(b, np_(a), what + ": with codes against without")
    # codes of another pitch are ignored, not misread
    bad = (q.Codes(ctx, n, m.dec.r.Wx.ld + 16), q.Codes(ctx, n, m.dec.q.Wx.ld + 16))
    r1 = q.cgru_decoder_step_q8(ctx, m.dec, P, enc_h, y.clone(), s.clone(), codes=bad)
    assert not bad[0].valid and not bad[1].valid
    assert_same(r1["s"], np_(res[0][0]), "s with unusable code buffers")


def _ahead_search(q, c, m, P, enc_h, n, s0, T, gx, codes, k=6):
    """A search of T steps with GRU r taken off the chain (cgru_decoder_step_ahead_q8 +
    output_logits_beam_ahead_q8); returns every step's s', s, context, top-k tables and y, and the result."""
    E, H = m.E_tgt.shape[1], m.dec.r.H
    state = torch.zeros(q.q8_beam_state_bytes(T), dtype=torch.uint8, device=c.device)
    y, s = c.empty(n, E), c.empty(n, H)
    q.q8_beam_init(c, state, n, T, s0, m.E_tgt, y, s)
    s_mid = [q.gru_step_q8(c, m.dec.r, y, s), c.empty(n, H)]
    yc = q.Codes(c, n, m.dec.r.Wx.ld) if codes else None
    cc = q.Codes(c, n, m.dec.q.Wx.ld) if codes else None
    trace = []
    for t in range(T):
        r = q.cgru_decoder_step_ahead_q8(c, m.dec, P, enc_h, s_mid[t & 1], ctx_codes=cc)
        o = q.output_logits_beam_ahead_q8(c, m.ro, m.W_out, m.b_out, r["s"], y, r["ctx"], state, m.E_tgt, m.dec.r, gx,
                                          s_mid[(t + 1) & 1], k=k, y_codes=yc, ctx_codes=cc,
                                          E_codes=m.E_tgt_codes if codes else None)
        trace += [np_(s_mid[t & 1]), np_(r["s"]), np_(r["ctx"]), np_(o["topk_logp"]), np_(o["topk_idx"]), np_(y)]
    return trace, q.q8_beam_result(c, state, T)


@pytest.mark.parametrize("dims,n,l,T,codes", [
    (dict(V=500, E=64, H=128, A=64, R=64, w_std=0.2, b_std=0.1), 4, 9, 12, True),
    (dict(V=13, E=16, H=32, A=16, R=16, w_std=0.5, b_std=0.3), 3, 5, 15, False),
    (dict(V=60, E=32, H=64, A=32, R=32, w_std=0.4, b_std=0.2), 8, 7, 15, True),
    (dict(V=700, E=620, H=1000, A=1000, R=620, w_std=0.2, b_std=0.1), 5, 6, 6, True),
    (dict(), 5, 30, 8, True), (dict(), 1, 11, 5, False)])
def test_decoding_loop_with_gru_r_ahead_of_the_decision(q, ctx, oracle, dims, n, l, T, codes):
    """cgru_decoder_step_ahead_q8 + output_logits_beam_ahead_q8 (the next step's s' from a table of the input
    products over the vocabulary, the recurrent products made in the readout's launch, and gates computed by
    blocks of the selection kernel once the search step has decided) against cgru_decoder_step_q8 +
    output_logits_beam_q8: every s', state, context vector, top-k table and embedding row bit for bit at every
    step, over searches in which hypotheses end and slots die, twice in a row (exchange words left clear)."""
    p = synth.full_model(seed=27, **dims)
    m = q.Model.from_params(ctx, p)
    E, H = m.E_tgt.shape[1], m.dec.r.H
    rng = np.random.default_rng(n + l)
    enc_h = ctx.f32(rng.standard_normal((l, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))
    gx = m.gx_r
    # the table against the plain product of a few rows
    rows = [0, m.E_tgt.shape[0] // 2, m.E_tgt.shape[0] - 1]
    assert_same(gx[rows], np_(q.q8_gemm_narrow(ctx, m.dec.r.Wx, m.E_tgt[rows].contiguous(), m.dec.r.bx)), "table rows")

    state = torch.zeros(q.q8_beam_state_bytes(T), dtype=torch.uint8, device=ctx.device)
    y, s = ctx.empty(n, E), ctx.empty(n, H)
    q.q8_beam_init(ctx, state, n, T, s0, m.E_tgt, y, s)
    ref = []
    for t in range(T):
        r = q.cgru_decoder_step_q8(ctx, m.dec, P, enc_h, y, s)
        o = q.output_logits_beam_q8(ctx, m.ro, m.W_out, m.b_out, r["s"], y, r["ctx"], state, m.E_tgt, s, k=max(6, n))
        ref += [np_(r["s_mid"]), np_(r["s"]), np_(r["ctx"]), np_(o["topk_logp"]), np_(o["topk_idx"]), np_(y)]
    ref_res = q.q8_beam_result(ctx, state, T)
    for rep in range(2):
        got, res = _ahead_search(q, ctx, m, P, enc_h, n, s0, T, gx, codes, k=max(6, n))
        q.q8_encode_check(ctx)
        for i, (a, b) in enumerate(zip(got, ref)):
            assert_same(a, b, "run %d, step %d, output %d" % (rep, i // 6, i % 6))
        assert res[0].tolist() == ref_res[0].tolist() and res[1:] == ref_res[1:]


@pytest.mark.parametrize("dims,beam,k,T", [(dict(V=13, E=16, H=32, A=16, R=16, w_std=0.5, b_std=0.3), 3, 5, 15),
                                           (dict(V=500, E=64, H=128, A=64, R=64, w_std=0.2, b_std=0.1), 5, 8, 14),
                                           (dict(), 5, 12, 10)])
def test_translate_with_and_without_the_table_of_input_products(q, ctx, oracle, dims, beam, k, T):
    """q8_translate on a model that brings the table of GRU r's input products (the loop with GRU r ahead of the
    decision) and on the same model without it (the plain loop): the same tokens, score and step count, and
    both equal to the oracle's."""
    p = synth.full_model(seed=29, **dims)
    with_table = q.Model.from_params(ctx, p)
    without = q.Model.from_params(ctx, p, gx_table=False)
    assert with_table.gx_r is not None and without.gx_r is None
    m_ref = oracle.OracleModel(p)
    V = p["E_src"].shape[0]
    for seed, l in ((1, 4), (2, 9), (3, 17)):
        src = np.random.default_rng(seed).integers(1, V, size=l).astype(np.int32)
        a = q.q8_translate(ctx, with_table, src, beam=beam, k=k, max_steps=T)
        b = q.q8_translate(ctx, without, src, beam=beam, k=k, max_steps=T)
        assert a[0].tolist() == b[0].tolist() and a[1:] == b[1:]
        _check_sentence(q, ctx, with_table, m_ref, src, beam, k, T)
