"""GPU check of the decoder step that allocates nothing: cgru_decoder_step_noalloc_q8 keeps its
kernels' scratch in the library's static device array.  Its outputs must equal those of
cgru_decoder_step_q8 bit for bit, on two calls in a row of which the second is smaller (the array
keeps the first call's contents), and sizes beyond the array must be refused before any launch."""
import numpy as np
import pytest
import torch

from workloads import synth

pytestmark = pytest.mark.gpu


def _case(q, ctx, seed, E, H, A, l, n):
    rng = np.random.default_rng(seed)
    p = synth.decoder_params(rng, E=E, H=H, A=A)
    mat = lambda k: q.q8_quantize_matrix(ctx, p[k])
    gru = lambda pre: q.GruWeights(mat(pre + ".Wx"), mat(pre + ".Wh"), ctx.f32(p[pre + ".bx"]), ctx.f32(p[pre + ".bh"]))
    w = q.CgruWeights(gru("dec_r"), mat("att.U"), ctx.f32(p["att.v"]), gru("dec_q"))
    enc_h = ctx.f32(rng.standard_normal((l, 2 * H)).astype(np.float32))
    P = q.q8_gemm_narrow(ctx, mat("att.W"), enc_h, ctx.f32(p["att.b"]))
    y = ctx.f32(rng.standard_normal((n, E)).astype(np.float32))
    s = ctx.f32(rng.standard_normal((n, H)).astype(np.float32))
    return w, P, enc_h, y, s


def test_decoder_step_without_allocation_equals_the_plain_call():
    import paper_1804_05038_amd as q
    ctx = q.Context()
    assert q.q8_noalloc_scratch_bytes() == 1 << 20
    q.q8_noalloc_setup(ctx)
    # first the benchmark's shape at beam 5, then a smaller one: fewer hypotheses, shorter sentence, narrower model
    for seed, (E, H, A, l, n) in enumerate([(512, 1024, 1024, 30, 5), (64, 128, 96, 7, 2)]):
        w, P, enc_h, y, s = _case(q, ctx, seed, E, H, A, l, n)
        ref = q.cgru_decoder_step_q8(ctx, w, P, enc_h, y, s)
        out = {"s": ctx.empty(n, H), "ctx": ctx.empty(n, 2 * H), "alpha": ctx.empty(n, l), "s_mid": ctx.empty(n, H)}
        for t in out.values():
            t.fill_(float("nan"))
        before = torch.cuda.memory_allocated()
        q.cgru_decoder_step_noalloc_q8(ctx, w, P, enc_h, y, s, out)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        for k in ("s", "ctx", "alpha", "s_mid"):
            a, b = out[k].cpu().numpy(), ref[k].cpu().numpy()
            assert np.isfinite(a).all() and (a == b).all(), (seed, k)
        # again, into the same outputs: the counters at the head of the array went back to zero
        q.cgru_decoder_step_noalloc_q8(ctx, w, P, enc_h, y, s, out)
        torch.cuda.synchronize()
        assert (out["s"].cpu().numpy() == ref["s"].cpu().numpy()).all()
    # a shape whose scratch does not fit the array (hidden size 8192: 1.3 MB): refused, nothing launched
    # (the weights are uninitialized device memory of the declared shapes; they are never read)
    H, E, A, n, l = 8192, 64, 64, 8, 30
    raw = lambda rows, cols: q.Mat(torch.empty(rows, cols, dtype=torch.int8, device=ctx.device), cols, 1.0)
    zeros = lambda k: torch.zeros(k, device=ctx.device)
    w = q.CgruWeights(q.GruWeights(raw(3 * H, E), raw(3 * H, H), zeros(3 * H), zeros(3 * H)), raw(A, H), zeros(A),
                      q.GruWeights(raw(3 * H, 2 * H), raw(3 * H, H), zeros(3 * H), zeros(3 * H)))
    out = {"s": ctx.empty(n, H), "ctx": ctx.empty(n, 2 * H)}
    with pytest.raises(q.Q8Error) as e:
        q.cgru_decoder_step_noalloc_q8(ctx, w, ctx.empty(l, A), ctx.empty(l, 2 * H), ctx.empty(n, E), ctx.empty(n, H), out)
    assert "static array" in str(e.value)
