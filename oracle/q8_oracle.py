"""ctypes front-end of the CPU oracle (q8_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this module.  It holds no arithmetic of its own: every number comes out of the C
functions, whose header says which passage of the paper each one follows.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "q8_oracle.c")
_LIB = os.path.join(_HERE, "libq8oracle.so")
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC"]


def build(force=False):
    """Compile q8_oracle.c with gcc (no intrinsics, contraction off)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "q8_oracle.h"))):
        return _LIB
    subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


def build_selftest(out=None, sanitize=False):
    """Compile q8_oracle.c with its self-test driver into an executable; sanitize: under
    AddressSanitizer and UndefinedBehaviorSanitizer (host code only), any finding is fatal."""
    out = out or os.path.join(_HERE, "q8_oracle_selftest")
    flags = ["-std=c11", "-Wall", "-Wextra", "-ffp-contract=off", "-fno-fast-math", "-g"]
    flags += ["-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"] if sanitize else ["-O2"]
    subprocess.check_call(["gcc", *flags, "-I" + _HERE, _SRC, os.path.join(_HERE, "q8_oracle_selftest.c"), "-o", out, "-lm"])
    return out


class Linear(C.Structure):
    _fields_ = [("rows", C.c_int), ("cols", C.c_int),
                ("Wf", C.c_void_p), ("ldf", C.c_int),
                ("Wq", C.c_void_p), ("ldq", C.c_int),
                ("scale", C.c_float), ("bias", C.c_void_p)]


class Gru(C.Structure):
    _fields_ = [("Wx", Linear), ("Wh", Linear)]


class Model(C.Structure):
    _fields_ = [("V_src", C.c_int), ("V_tgt", C.c_int), ("E", C.c_int), ("H", C.c_int),
                ("C", C.c_int), ("A", C.c_int), ("R", C.c_int),
                ("E_src", C.c_void_p), ("E_tgt", C.c_void_p),
                ("enc_fwd", Gru), ("enc_bwd", Gru),
                ("att_W", Linear), ("att_U", Linear), ("att_v", C.c_void_p),
                ("dec_r", Gru), ("dec_q", Gru),
                ("ro_s", Linear), ("ro_y", Linear), ("ro_c", Linear),
                ("out", Linear)]


_lib = None


class _Checked:
    """The C library with the oracle's finiteness rule applied to every call: a call that saw
    a NaN or an infinity in a vector or matrix it was given raises FloatingPointError (the
    method defines no result for such inputs)."""

    def __init__(self, cdll):
        self._c = cdll
        cdll.q8o_translate.restype = C.c_int
        cdll.q8o_translate_ensemble.restype = C.c_int
        cdll.q8o_nonfinite_count.restype = C.c_long
        cdll.q8o_nonfinite_count(C.c_int(1))

    def __getattr__(self, name):
        fn = getattr(self._c, name)

        def call(*args):
            r = fn(*args)
            bad = self._c.q8o_nonfinite_count(C.c_int(1))
            if bad:
                raise FloatingPointError("%s: %d non-finite input values" % (name, bad))
            return r

        setattr(self, name, call)
        return call


def load(path):
    """Front-end over a library built from q8_oracle.c at another path (a sanitizer or test build)."""
    return _Checked(C.CDLL(path))


def lib():
    global _lib
    if _lib is None:
        _lib = load(build())
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def pad16(n):
    return (n + 15) // 16 * 16


# ---------------------------------------------------------------- primitives ----

def quantize(v):
    v = _f32(v)
    q = np.empty(v.shape[0], np.int8)
    s = C.c_float()
    lib().q8o_quantize(_p(v), C.c_int(v.shape[0]), _p(q), C.byref(s))
    return q, np.float32(s.value)


def quantize_matrix(W, ld_out=None):
    W = _f32(W)
    rows, cols = W.shape
    ld_out = pad16(cols) if ld_out is None else ld_out
    Wq = np.full((rows, ld_out), 99, np.int8)
    s = C.c_float()
    lib().q8o_quantize_matrix(_p(W), C.c_int(rows), C.c_int(cols), C.c_int(cols), _p(Wq), C.c_int(ld_out), C.byref(s))
    return Wq, np.float32(s.value)


def accumulate(Wq, cols, xq):
    Wq = np.ascontiguousarray(Wq, np.int8)
    xq = np.ascontiguousarray(xq, np.int8)
    acc = np.empty(Wq.shape[0], np.int32)
    lib().q8o_accumulate(_p(Wq), C.c_int(Wq.shape[0]), C.c_int(cols), C.c_int(Wq.shape[1]), _p(xq), _p(acc))
    return acc


def dequantize(acc, s_w, s_x, bias=None):
    acc = np.ascontiguousarray(acc, np.int32)
    bias = None if bias is None else _f32(bias)
    y = np.empty(acc.shape[0], np.float32)
    lib().q8o_dequantize(_p(acc), C.c_int(acc.shape[0]), C.c_float(s_w), C.c_float(s_x), _p(bias), _p(y))
    return y


class QLinear:
    """A weight matrix in both stored forms (fp32 and its int8 image) plus bias."""

    def __init__(self, W, bias=None):
        self.Wf = _f32(W)
        self.rows, self.cols = self.Wf.shape
        self.Wq, self.scale = quantize_matrix(self.Wf)
        self.bias = None if bias is None else _f32(bias)
        self.c = Linear(self.rows, self.cols, _p(self.Wf).value, self.cols,
                        _p(self.Wq).value, self.Wq.shape[1], float(self.scale),
                        None if self.bias is None else _p(self.bias).value)

    def gemv(self, x, taps=False):
        x = _f32(x)
        y = np.empty(self.rows, np.float32)
        if not taps:
            lib().q8o_gemv(C.byref(self.c), _p(x), _p(y), None, None, None)
            return y
        xq = np.empty(self.cols, np.int8)
        xs = C.c_float()
        acc = np.empty(self.rows, np.int32)
        lib().q8o_gemv(C.byref(self.c), _p(x), _p(y), _p(xq), C.byref(xs), _p(acc))
        return y, xq, np.float32(xs.value), acc

    def gemm_narrow(self, X, taps=False):
        X = _f32(X)
        n = X.shape[0]
        Y = np.empty((n, self.rows), np.float32)
        if not taps:
            lib().q8o_gemm_narrow(C.byref(self.c), _p(X), C.c_int(n), C.c_int(X.shape[1]), _p(Y),
                                  C.c_int(self.rows), None, None, None)
            return Y
        xq = np.empty((n, self.cols), np.int8)
        xs = np.empty(n, np.float32)
        acc = np.empty((n, self.rows), np.int32)
        lib().q8o_gemm_narrow(C.byref(self.c), _p(X), C.c_int(n), C.c_int(X.shape[1]), _p(Y),
                              C.c_int(self.rows), _p(xq), _p(xs), _p(acc))
        return Y, xq, xs, acc

    def gemv_fp32(self, x):
        x = _f32(x)
        y = np.empty(self.rows, np.float32)
        lib().q8o_gemv_fp32(C.byref(self.c), _p(x), _p(y))
        return y


class QLinearRows:
    """A weight matrix quantized with one scale per row (the variant of Section 3's scheme)."""

    def __init__(self, W, bias=None):
        self.Wf = _f32(W)
        self.rows, self.cols = self.Wf.shape
        self.Wq = np.full((self.rows, pad16(self.cols)), 99, np.int8)
        self.row_scale = np.empty(self.rows, np.float32)
        lib().q8o_quantize_matrix_rows(_p(self.Wf), C.c_int(self.rows), C.c_int(self.cols), C.c_int(self.cols),
                                       _p(self.Wq), C.c_int(self.Wq.shape[1]), _p(self.row_scale))
        self.bias = None if bias is None else _f32(bias)

    def gemm_narrow(self, X, taps=False):
        X = _f32(X)
        n = X.shape[0]
        Y = np.empty((n, self.rows), np.float32)
        xq = np.empty((n, self.cols), np.int8)
        xs = np.empty(n, np.float32)
        acc = np.empty((n, self.rows), np.int32)
        lib().q8o_gemm_narrow_rows(_p(self.Wq), C.c_int(self.rows), C.c_int(self.cols), C.c_int(self.Wq.shape[1]),
                                   _p(self.row_scale), _p(self.bias), _p(X), C.c_int(n), C.c_int(X.shape[1]),
                                   _p(Y), C.c_int(self.rows), _p(xq), _p(xs), _p(acc))
        return (Y, xq, xs, acc) if taps else Y

    def gemv(self, x, taps=False):
        r = self.gemm_narrow(_f32(x)[None, :], taps)
        return tuple(a[0] for a in r) if taps else r[0]


def dequantize_rows(acc, row_scale, s_x, bias=None):
    acc = np.ascontiguousarray(acc, np.int32)
    row_scale = _f32(row_scale)
    bias = None if bias is None else _f32(bias)
    y = np.empty(acc.shape[0], np.float32)
    lib().q8o_dequantize_rows(_p(acc), C.c_int(acc.shape[0]), _p(row_scale), C.c_float(s_x), _p(bias), _p(y))
    return y


class QGru:
    def __init__(self, Wx, Wh, bx=None, bh=None):
        self.Wx = QLinear(Wx, bx)
        self.Wh = QLinear(Wh, bh)
        self.H = self.Wh.cols
        self.c = Gru(self.Wx.c, self.Wh.c)

    def step(self, x, h_prev, use_q8=True):
        x, h_prev = _f32(x), _f32(h_prev)
        h = np.empty(self.H, np.float32)
        lib().q8o_gru_step(C.byref(self.c), _p(x), _p(h_prev), C.c_int(int(use_q8)), _p(h))
        return h


def gru_gates(gx, gh, h_prev):
    gx, gh, h_prev = _f32(gx), _f32(gh), _f32(h_prev)
    H = h_prev.shape[0]
    h = np.empty(H, np.float32)
    lib().q8o_gru_gates(_p(gx), _p(gh), _p(h_prev), C.c_int(H), _p(h))
    return h


def attention(P, enc_h, a, v):
    P, enc_h, a, v = _f32(P), _f32(enc_h), _f32(a), _f32(v)
    l, A = P.shape
    Cc = enc_h.shape[1]
    e = np.empty(l, np.float32)
    alpha = np.empty(l, np.float32)
    ctx = np.empty(Cc, np.float32)
    lib().q8o_attention(_p(P), _p(enc_h), C.c_int(l), C.c_int(A), C.c_int(Cc), _p(a), _p(v), _p(e), _p(alpha), _p(ctx))
    return e, alpha, ctx


def attention_q8(P, enc_h, a, v):
    """The attention block with its two activation products in 8 bits (q8o_attention_q8); v and the
    transposed encoder states are quantized here by the oracle's matrix rule.  Returns
    (e, alpha, ctx, (vq, s_v), (hTq, s_h))."""
    P, enc_h, a, v = _f32(P), _f32(enc_h), _f32(a), _f32(v)
    l, A = P.shape
    Cc = enc_h.shape[1]
    vq, s_v = quantize_matrix(v[None, :], ld_out=A)
    hTq, s_h = quantize_matrix(np.ascontiguousarray(enc_h.T))
    e = np.empty(l, np.float32)
    alpha = np.empty(l, np.float32)
    ctx = np.empty(Cc, np.float32)
    lib().q8o_attention_q8(_p(P), C.c_int(l), C.c_int(A), _p(a), _p(vq), C.c_float(s_v), _p(hTq), C.c_int(Cc),
                           C.c_int(hTq.shape[1]), C.c_float(s_h), _p(e), _p(alpha), _p(ctx))
    return e, alpha, ctx, (vq, s_v), (hTq, s_h)


def logsoftmax_topk(logits, k):
    logits = _f32(logits)
    lse = C.c_float()
    lp = np.empty(k, np.float32)
    idx = np.empty(k, np.int32)
    lib().q8o_logsoftmax_topk(_p(logits), C.c_int(logits.shape[0]), C.c_int(k), C.byref(lse), _p(lp), _p(idx))
    return np.float32(lse.value), lp, idx


class OracleModel:
    """The whole translation model (Section 2) built from a dict of fp32 arrays.

    Keys: E_src, E_tgt, {enc_fwd,enc_bwd,dec_r,dec_q}.{Wx,Wh,bx,bh}, att.W, att.b,
    att.U, att.v, ro.Ws, ro.Wy, ro.Wc, ro.b, out.W, out.b.  Missing groups are
    allowed (a test of the decoder alone needs no encoder); their entries stay zero.
    """

    def __init__(self, p):
        self.p = p
        self.keep = []
        m = Model()
        g = lambda k: p.get(k)

        def gru(prefix):
            if prefix + ".Wx" not in p:
                return None
            q = QGru(p[prefix + ".Wx"], p[prefix + ".Wh"], g(prefix + ".bx"), g(prefix + ".bh"))
            self.keep.append(q)
            return q

        def lin(wk, bk=None):
            if wk not in p:
                return None
            q = QLinear(p[wk], g(bk) if bk else None)
            self.keep.append(q)
            return q

        self.enc_fwd, self.enc_bwd = gru("enc_fwd"), gru("enc_bwd")
        self.dec_r, self.dec_q = gru("dec_r"), gru("dec_q")
        self.att_W, self.att_U = lin("att.W", "att.b"), lin("att.U")
        self.ro_s, self.ro_y, self.ro_c = lin("ro.Ws", "ro.b"), lin("ro.Wy"), lin("ro.Wc")
        self.out = lin("out.W", "out.b")
        for name in ("enc_fwd", "enc_bwd", "dec_r", "dec_q", "att_W", "att_U", "ro_s", "ro_y", "ro_c", "out"):
            q = getattr(self, name)
            if q is not None:
                setattr(m, name, q.c)
        for name, key in (("E_src", "E_src"), ("E_tgt", "E_tgt"), ("att_v", "att.v")):
            if key in p:
                arr = _f32(p[key])
                self.keep.append(arr)
                setattr(self, name if name != "att_v" else "att_v_arr", arr)
                setattr(m, name, _p(arr).value)
        some_gru = self.dec_r or self.dec_q or self.enc_fwd
        m.H = some_gru.H if some_gru else 0
        m.C = 2 * m.H
        if self.dec_r:
            m.E = self.dec_r.Wx.cols
        elif self.enc_fwd:
            m.E = self.enc_fwd.Wx.cols
        if self.dec_q:
            m.C = self.dec_q.Wx.cols
        if self.att_U:
            m.A = self.att_U.rows
        if self.ro_s:
            m.R = self.ro_s.rows
        elif self.out:
            m.R = self.out.cols
        if "E_src" in p:
            m.V_src = p["E_src"].shape[0]
        if "E_tgt" in p:
            m.V_tgt = p["E_tgt"].shape[0]
        self.c = m
        self.H, self.E, self.Cdim, self.A, self.R = m.H, m.E, m.C, m.A, m.R

    # -- Eq. 1
    def encode(self, X, use_q8=True):
        X = _f32(X)
        l = X.shape[0]
        enc_h = np.empty((l, 2 * self.H), np.float32)
        lib().q8o_encode(C.byref(self.c), _p(X), C.c_int(l), C.c_int(int(use_q8)), _p(enc_h))
        return enc_h

    # -- Eq. 6, w(h_i)
    def attention_precompute(self, enc_h, use_q8=True):
        enc_h = _f32(enc_h)
        l = enc_h.shape[0]
        P = np.empty((l, self.A), np.float32)
        lib().q8o_attention_precompute(C.byref(self.c), _p(enc_h), C.c_int(l), C.c_int(int(use_q8)), _p(P))
        return P

    # -- Eq. 3-6
    def cgru_step(self, P, enc_h, y_emb, s_prev, use_q8=True):
        P, enc_h, y_emb, s_prev = _f32(P), _f32(enc_h), _f32(y_emb), _f32(s_prev)
        l = P.shape[0]
        s_mid = np.empty(self.H, np.float32)
        alpha = np.empty(l, np.float32)
        ctx = np.empty(self.Cdim, np.float32)
        s_out = np.empty(self.H, np.float32)
        lib().q8o_cgru_step(C.byref(self.c), _p(P), _p(enc_h), C.c_int(l), _p(y_emb), _p(s_prev),
                            C.c_int(int(use_q8)), _p(s_mid), _p(alpha), _p(ctx), _p(s_out))
        return s_mid, alpha, ctx, s_out

    # -- Eq. 2
    def readout(self, s, y_emb, ctx, use_q8=True):
        s, y_emb, ctx = _f32(s), _f32(y_emb), _f32(ctx)
        t = np.empty(self.R, np.float32)
        lib().q8o_readout(C.byref(self.c), _p(s), _p(y_emb), _p(ctx), C.c_int(int(use_q8)), _p(t))
        return t

    def output(self, t, k, use_q8=True):
        t = _f32(t)
        V = self.out.rows
        logits = np.empty(V, np.float32)
        lse = C.c_float()
        lp = np.empty(k, np.float32)
        idx = np.empty(k, np.int32)
        lib().q8o_output(C.byref(self.c), _p(t), C.c_int(int(use_q8)), C.c_int(k), _p(logits), C.byref(lse), _p(lp), _p(idx))
        return logits, np.float32(lse.value), lp, idx

    def translate(self, src_tokens, beam=5, topk=12, max_steps=100, use_q8=True):
        src = np.ascontiguousarray(src_tokens, np.int32)
        out = np.zeros(max_steps, np.int32)
        score = C.c_float()
        steps = C.c_int()
        n = lib().q8o_translate(C.byref(self.c), _p(src), C.c_int(src.shape[0]), C.c_int(beam), C.c_int(topk),
                                C.c_int(max_steps), C.c_int(int(use_q8)), _p(out), C.byref(score), C.byref(steps))
        return out[:n].copy(), np.float32(score.value), steps.value


def ensemble_logp(logps):
    """c[v] = log(mean_m exp(logp_m[v])) for a list of log-probability vectors (Section 4's ensemble)."""
    arrs = [_f32(a) for a in logps]
    V = arrs[0].shape[0]
    ptrs = (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])
    out = np.empty(V, np.float32)
    lib().q8o_ensemble_logp(ptrs, C.c_int(len(arrs)), C.c_int(V), _p(out))
    return out


def translate_ensemble(models, src_tokens, beam=5, topk=12, max_steps=100, use_q8=True):
    """Beam search over several OracleModel objects with averaged next-word probabilities."""
    src = np.ascontiguousarray(src_tokens, np.int32)
    out = np.zeros(max_steps, np.int32)
    score = C.c_float()
    steps = C.c_int()
    ptrs = (C.c_void_p * len(models))(*[C.addressof(m.c) for m in models])
    n = lib().q8o_translate_ensemble(ptrs, C.c_int(len(models)), _p(src), C.c_int(src.shape[0]), C.c_int(beam),
                                     C.c_int(topk), C.c_int(max_steps), C.c_int(int(use_q8)), _p(out), C.byref(score),
                                     C.byref(steps))
    return out[:n].copy(), np.float32(score.value), steps.value
