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
