"""Seeded synthetic workloads shaped like the paper's (Sections 2 and 4).

The paper measures on trained 620/1000-dimensional models and news test sets that
are not available; these generators stand in for them with random weights of the
same structure: a bidirectional-GRU encoder, a conditional-GRU decoder with
attention, a two-layer output network over a ~50k vocabulary (vocabularies of
33.7k-63.6k in the paper's Table 4), sentence lengths of 10-60 (test-set averages of
22.5-51.8 in its Table 5) and Zipf-distributed token ids.

Only numpy random draws live here; quantization, products and nonlinearities are
the business of the two implementations under test.  All arrays are float32 and
drawn in the order listed, from numpy.random.default_rng(seed).
"""
import numpy as np


def _n(rng, shape, std):
    return (rng.standard_normal(shape, dtype=np.float64) * std).astype(np.float32)


def gru_cell(seed=0, I=256, H=256, n_batch=1, w_std=0.1, b_std=0.01):
    """Config 1: one GRU step.  Gate row blocks r, z, n."""
    rng = np.random.default_rng(seed)
    return {
        "Wx": _n(rng, (3 * H, I), w_std), "Wh": _n(rng, (3 * H, H), w_std),
        "bx": _n(rng, (3 * H,), b_std), "bh": _n(rng, (3 * H,), b_std),
        "x": _n(rng, (n_batch, I), 1.0), "h_prev": _n(rng, (n_batch, H), 1.0),
    }


def _gru_params(rng, prefix, I, H, w_std, b_std, out):
    out[prefix + ".Wx"] = _n(rng, (3 * H, I), w_std)
    out[prefix + ".Wh"] = _n(rng, (3 * H, H), w_std)
    out[prefix + ".bx"] = _n(rng, (3 * H,), b_std)
    out[prefix + ".bh"] = _n(rng, (3 * H,), b_std)


def decoder_params(rng, E=512, H=1024, A=1024, w_std=0.05, b_std=0.01):
    C = 2 * H
    p = {}
    _gru_params(rng, "dec_r", E, H, w_std, b_std, p)
    p["att.U"] = _n(rng, (A, H), w_std)
    p["att.W"] = _n(rng, (A, C), w_std)
    p["att.b"] = _n(rng, (A,), b_std)
    p["att.v"] = _n(rng, (A,), w_std)
    _gru_params(rng, "dec_q", C, H, w_std, b_std, p)
    return p


def cgru_step(seed=1, E=512, H=1024, A=1024, l=30, n_beam=1, w_std=0.05, b_std=0.01):
    """Config 2: one conditional-GRU decoder step; enc_h stands in for an encoded sentence."""
    rng = np.random.default_rng(seed)
    p = decoder_params(rng, E, H, A, w_std, b_std)
    p["enc_h"] = _n(rng, (l, 2 * H), 1.0)
    p["y_emb"] = _n(rng, (n_beam, E), 1.0)
    p["s_prev"] = _n(rng, (n_beam, H), 1.0)
    return p


def output_layer(seed=2, V=50000, R=512, n_beam=5, w_std=0.05, b_std=0.01):
    """Config 3: vocabulary output layer fed with a given hidden vector t per beam entry."""
    rng = np.random.default_rng(seed)
    return {
        "out.W": _n(rng, (V, R), w_std), "out.b": _n(rng, (V,), b_std),
        "t": _n(rng, (n_beam, R), 1.0),
    }


def encoder(seed=3, l=50, E=512, H=1024, w_std=0.05, b_std=0.01):
    """Config 4: bidirectional GRU encoder over l embedding vectors."""
    rng = np.random.default_rng(seed)
    p = {"X": _n(rng, (l, E), 1.0)}
    _gru_params(rng, "enc_fwd", E, H, w_std, b_std, p)
    _gru_params(rng, "enc_bwd", E, H, w_std, b_std, p)
    return p


def zipf_tokens(rng, n, V, exponent=1.1):
    """n token ids in 1..V-1 with p(r) proportional to r^-exponent (inverse-CDF sampling)."""
    ranks = np.arange(1, V, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-exponent))
    cdf /= cdf[-1]
    u = rng.random(n)
    return (np.searchsorted(cdf, u, side="left") + 1).astype(np.int32)


def full_model(seed=4, V=50000, E=512, H=1024, A=1024, R=512, w_std=0.05, b_std=0.01, emb_std=1.0):
    """Config 5 model: every trained tensor of Section 2's network, random."""
    rng = np.random.default_rng(seed)
    C = 2 * H
    p = {"E_src": _n(rng, (V, E), emb_std), "E_tgt": _n(rng, (V, E), emb_std)}
    _gru_params(rng, "enc_fwd", E, H, w_std, b_std, p)
    _gru_params(rng, "enc_bwd", E, H, w_std, b_std, p)
    p.update(decoder_params(rng, E, H, A, w_std, b_std))
    p["ro.Ws"] = _n(rng, (R, H), w_std)
    p["ro.Wy"] = _n(rng, (R, E), w_std)
    p["ro.Wc"] = _n(rng, (R, C), w_std)
    p["ro.b"] = _n(rng, (R,), b_std)
    p["out.W"] = _n(rng, (V, R), w_std)
    p["out.b"] = _n(rng, (V,), b_std)
    return p


def sentences(seed=4, n=200, V=50000, min_len=10, max_len=60):
    """Config 5 inputs: n source sentences, lengths uniform in [min_len, max_len], Zipf(1.1) ids."""
    rng = np.random.default_rng(seed + 1000)
    lens = rng.integers(min_len, max_len + 1, size=n)
    return [zipf_tokens(rng, int(L), V) for L in lens]
