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


def gpu_mat(q, ctx, W):
    return q.q8_quantize_matrix(ctx, W)


def gpu_gru(q, ctx, p, prefix):
    return q.GruWeights(gpu_mat(q, ctx, p[prefix + ".Wx"]), gpu_mat(q, ctx, p[prefix + ".Wh"]),
                        ctx.f32(p[prefix + ".bx"]), ctx.f32(p[prefix + ".bh"]))
