"""Shared helpers of the GPU parity tests: the tolerance rule and oracle/GPU model builders."""
import numpy as np
import torch

REL = 1e-5   # spec tolerance on dequantized fp32 values


def assert_close(gpu, ref, what="", rel=REL):
    """|gpu - ref| <= rel * max(|ref_i|, rms(ref)) element by element.

    The rms floor covers elements that cancel to almost zero (bias against product,
    gate outputs near zero), where a purely relative test is meaningless."""
    gpu = np.asarray(gpu.detach().cpu().numpy() if isinstance(gpu, torch.Tensor) else gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    rms = np.sqrt((ref ** 2).mean()) if ref.size else 0.0
    tol = rel * np.maximum(np.abs(ref), rms)
    bad = np.abs(gpu - ref) > tol
    assert not bad.any(), "%s: %d of %d outside tolerance, worst |diff| %.3e at ref %.6g" % (
        what, bad.sum(), ref.size, np.abs(gpu - ref).max(), ref.reshape(-1)[np.argmax(np.abs(gpu - ref))])


def assert_same(gpu, ref, what=""):
    g = gpu.detach().cpu().numpy() if isinstance(gpu, torch.Tensor) else np.asarray(gpu)
    r = np.asarray(ref)
    assert g.shape == r.shape, (what, g.shape, r.shape)
    assert (g == r).all(), "%s: %d of %d differ" % (what, (g != r).sum(), r.size)


def np_(t):
    return t.detach().cpu().numpy()


def gpu_mat(q, ctx, W, tiled=False):
    """The quantized matrix; tiled: also its tile-packed copy, which the matrix-core products of
    panels read when it is there (rows of whole 64-byte k steps only)."""
    M = q.q8_quantize_matrix(ctx, W)
    return q.q8_pack_tiles(ctx, M) if tiled and M.ld % 64 == 0 else M


def gpu_gru(q, ctx, p, prefix, tiled=False):
    return q.GruWeights(gpu_mat(q, ctx, p[prefix + ".Wx"], tiled), gpu_mat(q, ctx, p[prefix + ".Wh"], tiled),
                        ctx.f32(p[prefix + ".bx"]), ctx.f32(p[prefix + ".bh"]))


def first_divergence_gap(m_ref, p, src, toks_a, toks_b):
    """Two translations of `src` that differ: the step where they part, and the oracle's gap in
    log-probability between the two tokens chosen there, after the common prefix (a sequence that
    has ended counts as token 0).  A search that followed the rules can only differ from the
    oracle's where the oracle's candidates nearly tie."""
    a, b = list(toks_a), list(toks_b)
    t = 0
    while t < len(a) and t < len(b) and a[t] == b[t]:
        t += 1
    enc = m_ref.encode(p["E_src"][src])
    P = m_ref.attention_precompute(enc)
    s, last = enc[0, :m_ref.H].copy(), 0
    for i in range(t + 1):
        y = p["E_tgt"][last]
        _, _, ctx, s = m_ref.cgru_step(P, enc, y, s)
        if i == t:
            logits, lse, _, _ = m_ref.output(m_ref.readout(s, y, ctx), 1)
            ta = a[t] if t < len(a) else 0
            tb = b[t] if t < len(b) else 0
            return t, abs(float(logits[ta]) - float(logits[tb]))
        last = a[i]
