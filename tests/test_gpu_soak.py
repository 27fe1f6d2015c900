"""GPU soak: the decoder step and the fused output layer + search step, repeated a few hundred times
on the same inputs, must give the same bits every time.  The kernels hand results between blocks
(the last block to arrive finishes the attention of a hypothesis and the search step), so a missing
wait or a stale read would show up here as a run that differs from the first."""
import numpy as np
import pytest
import torch

from workloads import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def setup():
    import paper_1804_05038_amd as q
    ctx = q.Context()
    return q, ctx, q.Model.from_params(ctx, synth.full_model(seed=4))


@pytest.mark.parametrize("hand_on", [False, True])
@pytest.mark.parametrize("n,l,reps", [(5, 30, 300), (8, 60, 100), (1, 7, 100)])
def test_decoder_step_and_search_step_are_bit_reproducible(setup, n, l, reps, hand_on):
    """hand_on: the search step also gathers the codes of its rows and the second decoder step's GRU r takes them."""
    q, ctx, m = setup
    E, H, T = m.E_tgt.shape[1], m.dec.r.H, 4
    rng = np.random.default_rng(100 + n)
    enc_h = ctx.f32(rng.standard_normal((l, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))
    state = torch.zeros(q.q8_beam_state_bytes(T), dtype=torch.uint8, device=ctx.device)
    y, s = ctx.empty(n, E), ctx.empty(n, H)
    codes = (q.Codes(ctx, n, m.dec.r.Wx.ld), q.Codes(ctx, n, m.dec.q.Wx.ld))
    if hand_on:
        codes = codes + (q.Codes(ctx, n, m.dec.r.Wh.ld),)
    c0 = q.q8_beam_init(ctx, state, n, T, s0, m.E_tgt, y, s, bind=True)
    c1 = q.cgru_decoder_step_q8(ctx, m.dec, P, enc_h, y, s, bind=True, codes=codes)
    c2 = q.output_logits_beam_q8(ctx, m.ro, m.W_out, m.b_out, c1.out["s"], y, c1.out["ctx"], state, m.E_tgt, s, k=12,
                                 bind=True, codes=codes, E_codes=m.E_tgt_codes if hand_on else None)

    def run():
        # two steps of a search from its start: the second step runs on gathered states and embeddings
        c0.launch()
        if hand_on:
            codes[0].invalidate(); codes[2].invalidate()
        outs = []
        for _ in range(2):
            c1.launch()
            c2.launch()
            outs += [c1.out["s"].clone(), c1.out["ctx"].clone(), c1.out["alpha"].clone(), c1.out["s_mid"].clone(),
                     codes[0].q.clone(), codes[1].q.clone(), codes[1].scale.clone(),
                     c2.out["topk_logp"].clone(), c2.out["topk_idx"].clone(), y.clone(), s.clone()]
        outs.append(state.clone())           # (after both steps: rows of later steps keep an earlier run's links until then)
        return outs

    ref = run()
    assert all(torch.isfinite(t).all() for t in ref if t.is_floating_point())
    for rep in range(reps):
        got = run()
        for i, (a, b) in enumerate(zip(got, ref)):
            assert torch.equal(a, b), "repetition %d: output %d differs from the first run" % (rep, i)


@pytest.mark.parametrize("S,l,reps", [(64, 8, 150), (13, 5, 100)])
def test_batched_step_is_bit_reproducible(setup, S, l, reps):
    """The batched decoder step with codes handed on (GRU r and GRU q as one kernel each, whose blocks exchange
    their partial maxima through two regions of words that take turns), the panel output layer and the batched
    search step: two steps of a search from its start, the same bits in every repetition."""
    q, ctx0, m = setup
    ctx = q.Context("cuda:0", workspace_bytes=q.q8_workspace_bytes(max_n=S * 5, max_l=64, max_rows=50000, max_ld=2048) + (256 << 20))
    beam, T, n = 5, 4, S * 5
    E, H = m.E_tgt.shape[1], m.dec.r.H
    rng = np.random.default_rng(7 + S)
    enc_h = ctx.f32(rng.standard_normal((S * l, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    off = torch.arange(0, (S + 1) * l, l, dtype=torch.int32, device=ctx.device)
    states = torch.zeros(q.q8_beam_state_bytes(T) * S, dtype=torch.uint8, device=ctx.device)
    y, s = ctx.empty(n, E), ctx.empty(n, H)
    done = torch.zeros(S, dtype=torch.int32, device=ctx.device)
    codes = (q.Codes(ctx, n, m.dec.r.Wx.ld), q.Codes(ctx, n, m.dec.q.Wx.ld), q.Codes(ctx, n, m.ro.W_s.ld))
    sp = q.Codes(ctx, n, m.dec.r.Wh.ld)
    c0 = q.q8_beam_init_batch(ctx, states, S, beam, T, enc_h, off, m.E_tgt, y, s, done, bind=True)
    c1 = q.cgru_decoder_step_batch_q8(ctx, m.dec, P, enc_h, off, beam, l, y, s, bind=True, codes=codes + (sp,))
    c2 = q.output_logits_q8(ctx, m.ro, m.W_out, m.b_out, s=c1.out["s"], y_emb=y, ctx_vec=c1.out["ctx"], k=12,
                            want_logits=False, bind=True, codes=codes)
    c3 = q.q8_beam_update_batch(ctx, states, S, beam, T, c2.out["topk_logp"], c2.out["topk_idx"], c1.out["s"], m.E_tgt, y, s,
                                done, bind=True, codes=(codes[2], codes[0], sp), E_codes=m.E_tgt_codes)

    def run():
        c0.launch()
        codes[0].invalidate(); sp.invalidate()
        outs = []
        for _ in range(2):
            c1.launch(); c2.launch(); c3.launch()
            outs += [c1.out["s"].clone(), c1.out["ctx"].clone(), c1.out["s_mid"].clone(), codes[1].q.clone(), codes[2].q.clone(),
                     codes[2].scale.clone(), c2.out["topk_logp"].clone(), c2.out["topk_idx"].clone(), y.clone(), s.clone(),
                     codes[0].q.clone(), sp.q.clone(), sp.scale.clone()]
        outs.append(states.clone())
        return outs

    ref = run()
    assert all(torch.isfinite(t).all() for t in ref if t.is_floating_point())
    for rep in range(reps):
        got = run()
        for i, (a, b) in enumerate(zip(got, ref)):
            assert torch.equal(a, b), "repetition %d: output %d differs from the first run" % (rep, i)
    q.q8_encode_check(ctx)


def _ahead_calls(q, ctx, m, P, enc_h, n, s0, T):
    """Bound calls of the loop with GRU r ahead: init, the first s', and the two calls for either parity of the step."""
    E, H = m.E_tgt.shape[1], m.dec.r.H
    state = torch.zeros(q.q8_beam_state_bytes(T), dtype=torch.uint8, device=ctx.device)
    y, s = ctx.empty(n, E), ctx.empty(n, H)
    s_mid = [ctx.empty(n, H), ctx.empty(n, H)]
    yc, cc = q.Codes(ctx, n, m.dec.r.Wx.ld), q.Codes(ctx, n, m.dec.q.Wx.ld)
    c0 = q.q8_beam_init(ctx, state, n, T, s0, m.E_tgt, y, s, bind=True)
    cr = q.gru_step_q8(ctx, m.dec.r, y, s, h_out=s_mid[0], bind=True)
    c1, c2, out = [], [], None
    for i in (0, 1):
        c = q.cgru_decoder_step_ahead_q8(ctx, m.dec, P, enc_h, s_mid[i], out=out, bind=True, ctx_codes=cc)
        out = c.out
        c1.append(c)
        c2.append(q.output_logits_beam_ahead_q8(ctx, m.ro, m.W_out, m.b_out, out["s"], y, out["ctx"], state, m.E_tgt, m.dec.r, m.gx_r,
                                                s_mid[1 - i], k=12, bind=True, y_codes=yc, ctx_codes=cc, E_codes=m.E_tgt_codes))

    def run(steps=3):
        c0.launch()
        yc.invalidate()
        cr.launch()
        outs = []
        for t in range(steps):
            c1[t & 1].launch()
            c2[t & 1].launch()
            outs += [s_mid[t & 1].clone(), out["s"].clone(), out["ctx"].clone(), c2[t & 1].out["topk_logp"].clone(),
                     c2[t & 1].out["topk_idx"].clone(), y.clone(), yc.q.clone(), s_mid[1 - (t & 1)].clone()]
        outs.append(state.clone())
        return outs
    return run


@pytest.mark.parametrize("n,l,reps", [(5, 30, 300), (8, 60, 100), (1, 7, 100)])
def test_loop_with_gru_r_ahead_is_bit_reproducible(setup, n, l, reps):
    """Three steps of a search with GRU r ahead of the decision (blocks of the selection kernel wait for the search
    step's decision and compute the next s'; the readout's launch carries the recurrent product), the same bits
    in every repetition."""
    q, ctx, m = setup
    H = m.dec.r.H
    rng = np.random.default_rng(200 + n)
    enc_h = ctx.f32(rng.standard_normal((l, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))
    run = _ahead_calls(q, ctx, m, P, enc_h, n, s0, 4)
    ref = run()
    assert all(torch.isfinite(t).all() for t in ref if t.is_floating_point())
    for rep in range(reps):
        got = run()
        for i, (a, b) in enumerate(zip(got, ref)):
            assert torch.equal(a, b), "repetition %d: output %d differs from the first run" % (rep, i)
    q.q8_encode_check(ctx)


def test_wait_for_the_decision_that_gives_up_is_reported_and_the_next_search_is_good(setup):
    """With a bound of one poll the blocks that wait for the search step's decision give up at once (it comes
    microseconds later): the kernel still ends normally with every index inside its table, q8_encode_check
    reports it and clears the exchange words, and the same search run again gives the first run's bits."""
    q, ctx, m = setup
    H = m.dec.r.H
    rng = np.random.default_rng(9)
    enc_h = ctx.f32(rng.standard_normal((12, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))
    run = _ahead_calls(q, ctx, m, P, enc_h, 5, s0, 4)
    good = run()
    q.q8_encode_check(ctx)
    try:
        q.q8_attention_options(ctx, exchange=True, spin_limit=1)
        run()
        with pytest.raises(q.Q8Error):
            q.q8_encode_check(ctx)
    finally:
        q.q8_attention_options(ctx, exchange=True, spin_limit=0)
    q.q8_encode_check(ctx)
    again = run()
    q.q8_encode_check(ctx)
    for i, (a, b) in enumerate(zip(again, good)):
        assert torch.equal(a, b), "output %d after the abandoned run" % i


def test_loop_with_gru_r_ahead_replayed_from_a_graph(setup):
    """The launch mode of the benchmark's headline: one HIP graph holds a whole search of the loop with GRU r ahead
    (full-size model, beam 5); it is replayed four times with eager work and synchronizations between the replays,
    and every replay's outputs and search state equal the eager run's bit for bit."""
    q, ctx, m = setup
    H, T = m.dec.r.H, 6
    rng = np.random.default_rng(31)
    enc_h = ctx.f32(rng.standard_normal((30, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, m.att_W, enc_h, m.att_b)
    s0 = ctx.f32(rng.standard_normal(H).astype(np.float32))
    ref = _ahead_calls(q, ctx, m, P, enc_h, 5, s0, T)(steps=T)
    q.q8_encode_check(ctx)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        gctx = q.Context("cuda:0", stream=side)
        run = _ahead_calls(q, gctx, m, P, enc_h, 5, s0, T)
        run(steps=T)
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            captured = run(steps=T)          # (the clones it returns are made inside the graph: they hold every step's outputs)
    torch.cuda.synchronize()
    for rep in range(4):
        g.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(captured, ref)):
            assert torch.equal(a, b), "replay %d: output %d differs from the eager run" % (rep, i)
        q.q8_gemv(ctx, m.att_W, enc_h[0])    # unrelated eager work between replays
        for t in captured:
            t.zero_()                        # (a replay must write every output again)
        torch.cuda.synchronize()
    q.q8_encode_check(gctx)
