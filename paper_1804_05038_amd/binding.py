"""ctypes binding of libq8nmt.so: argument marshalling only.

Every function below has the name of the C entry point it calls (see include/q8nmt.h
for semantics, layouts and limits).  Tensors are torch CUDA tensors used as plain
device buffers; results come back in freshly allocated (or caller-supplied) tensors.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libq8nmt.so")

__all__ = ["Q8Error", "Context", "Mat", "Codes", "RowCodes", "GruWeights", "CgruWeights", "ReadoutWeights", "load_library",
           "q8_quantize_matrix", "q8_quantize_matrix_rows", "q8_pack_tiles", "q8_gemv", "q8_gemm_narrow", "q8_gemm_narrow_rows", "q8_attention_states_q8", "q8_attention_q8", "gru_step_q8", "cgru_decoder_step_q8",
           "output_logits_q8", "output_logits_beam_q8", "output_logits_beam_batch_q8", "cgru_decoder_step_ahead_q8", "output_logits_beam_ahead_q8", "gru_input_table", "q8_encode", "q8_encoder_options", "q8_encode_check", "q8_attention_options", "q8_workspace_bytes", "Model", "q8_translate", "q8_translate_bytes",
           "q8_beam_state_bytes", "q8_beam_init", "q8_beam_update", "q8_beam_result", "q8_profile_begin", "q8_profile_end", "q8_probe_read", "q8_math_eval", "MatF", "GruWeightsF32", "CgruWeightsF32", "ReadoutWeightsF32", "q8_gemv_f32",
           "cgru_decoder_step_f32", "output_logits_f32", "q8_translate_ensemble", "q8_translate_ensemble_bytes", "cgru_decoder_step_batch_q8", "q8_encode_batch", "q8_encode_batch_bytes", "q8_beam_init_batch",
           "q8_beam_update_batch", "q8_beam_result_batch", "q8_translate_batch", "q8_translate_batch_bytes",
           "KERNEL_CLASSES", "LIB_PATH", "source_ids",
           "cgru_decoder_step_noalloc_q8", "q8_noalloc_setup", "q8_noalloc_scratch_bytes"]
LIB_PATH = _LIB_PATH

STATUS = {0: "Q8_OK", 1: "Q8_ERR_NULL", 2: "Q8_ERR_SHAPE", 3: "Q8_ERR_ALIGN", 4: "Q8_ERR_WORKSPACE", 5: "Q8_ERR_DEVICE"}


class Q8Error(RuntimeError):
    def __init__(self, code, text):
        super().__init__("%s: %s" % (STATUS.get(code, code), text))
        self.code = code


class _Mat(C.Structure):
    _fields_ = [("data", C.c_void_p), ("rows", C.c_int), ("cols", C.c_int), ("ld", C.c_int), ("scale", C.c_float),
                ("tiles", C.c_void_p)]


class _RowCodes(C.Structure):
    _fields_ = [("q", C.c_void_p), ("scale", C.c_void_p), ("ld", C.c_int)]


class _Codes(C.Structure):
    _fields_ = [("q", C.c_void_p), ("scale", C.c_void_p), ("ld", C.c_int), ("valid", C.c_int)]


class _Taps(C.Structure):
    _fields_ = [("xq", C.c_void_p), ("xscale", C.c_void_p), ("acc", C.c_void_p)]


class _Gru(C.Structure):
    _fields_ = [("Wx", _Mat), ("Wh", _Mat), ("bx", C.c_void_p), ("bh", C.c_void_p)]


class _Cgru(C.Structure):
    _fields_ = [("r", _Gru), ("att_U", _Mat), ("att_v", C.c_void_p), ("q", _Gru)]


class _Readout(C.Structure):
    _fields_ = [("W_s", _Mat), ("W_y", _Mat), ("W_c", _Mat), ("b_t", C.c_void_p)]


class _Model(C.Structure):
    _fields_ = [("E_src", C.c_void_p), ("E_tgt", C.c_void_p), ("V_src", C.c_int), ("V_tgt", C.c_int), ("E", C.c_int),
                ("enc_fwd", _Gru), ("enc_bwd", _Gru), ("att_W", _Mat), ("att_b", C.c_void_p),
                ("dec", _Cgru), ("ro", _Readout), ("W_out", _Mat), ("b_out", C.c_void_p), ("E_tgt_codes", _RowCodes),
                ("gx_r", C.c_void_p)]


_lib = None


def load_library():
    """Loads the built HIP library; there is no fallback if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libq8nmt.so is not built: run `python -m paper_1804_05038_amd.build` "
                              "(or __graft_entry__.build()) first; there is no CPU fallback")
        lib = C.CDLL(_LIB_PATH)
        lib.q8_workspace_bytes.restype = C.c_size_t
        lib.q8_workspace_bytes.argtypes = [C.c_int] * 4
        lib.q8_last_error.restype = C.c_char_p
        lib.q8_last_error.argtypes = [C.c_void_p]
        lib.q8_create.argtypes = [C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p, C.c_size_t]
        lib.q8_destroy.argtypes = [C.c_void_p]
        vp, ci = C.c_void_p, C.c_int
        lib.q8_quantize_matrix.argtypes = [vp, vp, ci, ci, ci, vp, ci, C.POINTER(C.c_float)]
        lib.q8_tiles_bytes.restype = C.c_size_t
        lib.q8_tiles_bytes.argtypes = [ci, ci]
        lib.q8_pack_tiles.argtypes = [vp, C.POINTER(_Mat), vp]
        lib.q8_gemv.argtypes = [vp, C.POINTER(_Mat), vp, vp, vp, C.POINTER(_Taps)]
        lib.q8_gemm_narrow.argtypes = [vp, C.POINTER(_Mat), vp, ci, ci, vp, vp, ci, C.POINTER(_Taps)]
        lib.q8_quantize_matrix_rows.argtypes = [vp, vp, ci, ci, ci, vp, ci, vp]
        lib.q8_gemm_narrow_rows.argtypes = [vp, C.POINTER(_Mat), vp, vp, ci, ci, vp, vp, ci, C.POINTER(_Taps)]
        lib.q8_attention_states_q8.argtypes = [vp, vp, ci, ci, vp, ci, C.POINTER(C.c_float)]
        lib.q8_attention_q8.argtypes = [vp, C.POINTER(_Mat), C.POINTER(_Mat), vp, vp, ci, ci, vp, vp, vp]
        lib.gru_step_q8.argtypes = [vp, C.POINTER(_Gru), vp, vp, ci, vp, C.POINTER(_Taps)]
        lib.cgru_decoder_step_q8.argtypes = [vp, C.POINTER(_Cgru), vp, vp, ci, vp, vp, ci, vp, vp, vp, vp, C.POINTER(_Taps)]
        lib.cgru_decoder_step_codes_q8.argtypes = lib.cgru_decoder_step_q8.argtypes + [C.POINTER(_Codes), C.POINTER(_Codes)]
        lib.cgru_decoder_step_loop_q8.argtypes = lib.cgru_decoder_step_q8.argtypes + [C.POINTER(_Codes)] * 3
        lib.cgru_decoder_step_noalloc_q8.argtypes = lib.cgru_decoder_step_q8.argtypes[:-1]
        lib.q8_noalloc_setup.argtypes = [vp]
        lib.q8_noalloc_scratch_bytes.restype = C.c_size_t
        lib.q8_noalloc_scratch_bytes.argtypes = []
        lib.output_logits_q8.argtypes = [vp, C.POINTER(_Readout), C.POINTER(_Mat), vp, vp, vp, vp, vp, ci, ci,
                                         vp, vp, vp, vp, vp, C.POINTER(_Taps)]
        lib.q8_encode.argtypes = [vp, C.POINTER(_Gru), C.POINTER(_Gru), vp, ci, vp]
        lib.q8_encoder_options.argtypes = [vp, ci, ci]
        lib.q8_encode_check.argtypes = [vp]
        lib.q8_attention_options.argtypes = [vp, ci, ci]
        lib.q8_beam_state_bytes.restype = C.c_size_t
        lib.q8_beam_state_bytes.argtypes = [ci]
        lib.q8_beam_init.argtypes = [vp, vp, ci, ci, vp, vp, ci, ci, vp, vp]
        lib.q8_beam_update.argtypes = [vp, vp, vp, vp, ci, ci, vp, ci, vp, ci, vp, vp]
        ip = C.POINTER(C.c_int)
        lib.q8_beam_result.argtypes = [vp, vp, ci, vp, ip, C.POINTER(C.c_float), ip, ip]
        lib.output_logits_beam_q8.argtypes = [vp, C.POINTER(_Readout), C.POINTER(_Mat), vp, vp, vp, vp, ci, ci, vp,
                                              vp, ci, vp, vp, vp]
        lib.output_logits_beam_codes_q8.argtypes = lib.output_logits_beam_q8.argtypes + [C.POINTER(_Codes), C.POINTER(_Codes)]
        lib.output_logits_beam_loop_q8.argtypes = lib.output_logits_beam_q8.argtypes + [C.POINTER(_Codes)] * 3 + [C.POINTER(_RowCodes)]
        lib.q8_translate_bytes.restype = C.c_size_t
        lib.q8_translate_bytes.argtypes = [C.POINTER(_Model), ci, ci, ci, ci]
        lib.q8_translate.argtypes = [vp, C.POINTER(_Model), vp, ci, ci, ci, ci, vp, ip, C.POINTER(C.c_float), ip]
        lib.q8_profile_begin.argtypes = [vp, ci, ci]
        lib.q8_probe_read.argtypes = [vp, vp, C.c_size_t]
        lib.q8_math_eval.argtypes = [vp, ci, vp, vp, C.c_size_t]
        lib.cgru_decoder_step_batch_q8.argtypes = [vp, C.POINTER(_Cgru), vp, vp, vp, ci, ci, ci, vp, vp, vp, vp, vp, vp]
        lib.cgru_decoder_step_batch_codes_q8.argtypes = lib.cgru_decoder_step_batch_q8.argtypes + [C.POINTER(_Codes)] * 3
        lib.cgru_decoder_step_batch_loop_q8.argtypes = lib.cgru_decoder_step_batch_q8.argtypes + [C.POINTER(_Codes)] * 4
        lib.output_logits_codes_q8.argtypes = [vp, C.POINTER(_Readout), C.POINTER(_Mat), vp, vp, vp, vp, ci, ci,
                                               vp, vp, vp, vp, vp] + [C.POINTER(_Codes)] * 3
        lib.q8_gemv_f32.argtypes = [vp, C.POINTER(_MatF), vp, ci, ci, vp, vp, ci]
        lib.cgru_decoder_step_f32.argtypes = [vp, C.POINTER(_CgruF), vp, vp, ci, vp, vp, ci, vp, vp, vp, vp]
        lib.output_logits_f32.argtypes = [vp, C.POINTER(_ReadoutF), C.POINTER(_MatF), vp, vp, vp, vp, ci, ci, vp, vp, vp, vp, vp]
        lib.q8_translate_ensemble_bytes.restype = C.c_size_t
        lib.q8_translate_ensemble_bytes.argtypes = [vp, ci, ci, ci, ci, ci]
        lib.q8_translate_ensemble.argtypes = [vp, vp, ci, vp, ci, ci, ci, ci, vp, ip, C.POINTER(C.c_float), ip]
        lib.q8_encode_batch_bytes.restype = C.c_size_t
        lib.q8_encode_batch_bytes.argtypes = [C.POINTER(_Gru), ci, ci]
        lib.q8_encode_batch.argtypes = [vp, C.POINTER(_Gru), C.POINTER(_Gru), vp, vp, ip, ci, vp]
        lib.q8_beam_init_batch.argtypes = [vp, vp, ci, ci, ci, vp, vp, ci, vp, ci, ci, vp, vp, vp]
        lib.q8_beam_update_batch.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, vp, ci, vp, ci, vp, vp, vp]
        lib.q8_beam_update_batch_loop.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp, vp, ci, vp, ci, ci, vp, vp, vp,
                                                  C.POINTER(_RowCodes), C.POINTER(_Codes), C.POINTER(_Codes), C.POINTER(_Codes)]
        lib.cgru_decoder_step_ahead_q8.argtypes = [vp, C.POINTER(_Cgru), vp, vp, ci, vp, ci, vp, vp, vp, C.POINTER(_Codes)]
        lib.output_logits_beam_ahead_q8.argtypes = [vp, C.POINTER(_Readout), C.POINTER(_Mat), vp, vp, vp, vp, ci, ci, vp, vp, ci,
                                                    vp, vp, C.POINTER(_Codes), C.POINTER(_Codes), C.POINTER(_RowCodes),
                                                    C.POINTER(_Gru), vp, vp]
        lib.output_logits_beam_batch_q8.argtypes = [vp, C.POINTER(_Readout), C.POINTER(_Mat), vp, vp, vp, vp, ci, ci, ci, ci, vp,
                                                    vp, ci, vp, vp, vp, vp, C.POINTER(_Codes), C.POINTER(_Codes),
                                                    C.POINTER(_Codes), C.POINTER(_Codes), C.POINTER(_RowCodes)]
        lib.q8_beam_result_batch.argtypes = [vp, vp, ci, ci, vp, ip, C.POINTER(C.c_float), ip]
        lib.q8_translate_batch_bytes.restype = C.c_size_t
        lib.q8_translate_batch_bytes.argtypes = [C.POINTER(_Model), ci, ci, ci, ci, ci]
        lib.q8_translate_batch.argtypes = [vp, C.POINTER(_Model), vp, ip, ci, ci, ci, ci, vp, ip, C.POINTER(C.c_float), ip]
        lib.q8_profile_end.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_int)]
        _lib = lib
    return _lib


def q8_workspace_bytes(max_n=8, max_l=64, max_rows=65536, max_ld=2048):
    return load_library().q8_workspace_bytes(max_n, max_l, max_rows, max_ld)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dev_f32(t, device):
    if t is None:
        return None
    return torch.as_tensor(t, dtype=torch.float32).to(device).contiguous()


class Context:
    """q8_create / q8_destroy: a stream and a caller-owned workspace."""

    def __init__(self, device="cuda:0", workspace_bytes=None, stream=None):
        self.lib = load_library()
        self.device = torch.device(device)
        if workspace_bytes is None:
            workspace_bytes = q8_workspace_bytes()
        self.workspace = torch.empty(workspace_bytes, dtype=torch.uint8, device=self.device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        st = self.lib.q8_create(C.byref(h), C.c_void_p(self.stream.cuda_stream), _ptr(self.workspace),
                                C.c_size_t(workspace_bytes))
        if st != 0:
            raise Q8Error(st, "q8_create failed")
        self.handle = h

    def check(self, st):
        if st != 0:
            raise Q8Error(st, self.lib.q8_last_error(self.handle).decode())

    def close(self):
        if getattr(self, "handle", None):
            self.lib.q8_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def f32(self, a):
        return _dev_f32(a, self.device)

    def empty(self, *shape, dtype=torch.float32):
        return torch.empty(*shape, dtype=dtype, device=self.device)


class Mat:
    """q8_mat: int8 device matrix [rows x ld] plus its host-side scale."""

    def __init__(self, data, cols, scale, tiles=None):
        self.data = data
        self.rows, self.ld = data.shape
        self.cols = cols
        self.scale = float(scale)
        self.tiles = tiles
        self.c = _Mat(data.data_ptr(), self.rows, cols, self.ld, self.scale, tiles.data_ptr() if tiles is not None else None)


class _MatF(C.Structure):
    _fields_ = [("data", C.c_void_p), ("rows", C.c_int), ("cols", C.c_int), ("ld", C.c_int)]


class _GruF(C.Structure):
    _fields_ = [("Wx", _MatF), ("Wh", _MatF), ("bx", C.c_void_p), ("bh", C.c_void_p)]


class _CgruF(C.Structure):
    _fields_ = [("r", _GruF), ("att_U", _MatF), ("att_v", C.c_void_p), ("q", _GruF)]


class _ReadoutF(C.Structure):
    _fields_ = [("W_s", _MatF), ("W_y", _MatF), ("W_c", _MatF), ("b_t", C.c_void_p)]


class MatF:
    """q8_matf: fp32 device matrix [rows x ld] of the 32-bit engine (ld padded to a multiple of 4)."""

    def __init__(self, ctx, W):
        import numpy as np
        W = np.asarray(W, dtype=np.float32)
        rows, cols = W.shape
        ld = (cols + 3) // 4 * 4
        buf = np.zeros((rows, ld), np.float32)
        buf[:, :cols] = W
        self.data = ctx.f32(buf)
        self.rows, self.cols, self.ld = rows, cols, ld
        self.c = _MatF(self.data.data_ptr(), rows, cols, ld)


class GruWeightsF32:
    def __init__(self, Wx, Wh, bx, bh):
        self.Wx, self.Wh, self.bx, self.bh = Wx, Wh, bx, bh
        self.H = Wh.cols
        self.c = _GruF(Wx.c, Wh.c, bx.data_ptr(), bh.data_ptr())


class CgruWeightsF32:
    def __init__(self, r, att_U, att_v, q):
        self.r, self.att_U, self.att_v, self.q = r, att_U, att_v, q
        self.c = _CgruF(r.c, att_U.c, att_v.data_ptr(), q.c)


class ReadoutWeightsF32:
    def __init__(self, W_s, W_y, W_c, b_t):
        self.W_s, self.W_y, self.W_c, self.b_t = W_s, W_y, W_c, b_t
        self.c = _ReadoutF(W_s.c, W_y.c, W_c.c, b_t.data_ptr())


class Codes:
    """q8_codes: buffers for the int8 codes [n x ld] and scales [n] that one entry point leaves for the next."""

    def __init__(self, ctx, n, ld):
        self.q = ctx.empty(n, ld, dtype=torch.int8)
        self.scale = ctx.empty(n)
        self.c = _Codes(self.q.data_ptr(), self.scale.data_ptr(), ld, 0)

    @property
    def valid(self):
        return bool(self.c.valid)

    def invalidate(self):
        """To be called by whoever changes the vectors these codes belong to."""
        self.c.valid = 0


class RowCodes:
    """q8_row_codes: every row of a table (the target embeddings) quantized on its own maximum, at pitch ld."""

    def __init__(self, ctx, table, ld):
        mat, self.scale = q8_quantize_matrix_rows(ctx, table, ld_out=ld)
        self.q = mat.data
        self.c = _RowCodes(self.q.data_ptr(), self.scale.data_ptr(), ld)


class _Bound:
    """A call with its arguments already marshalled: launch() re-issues it on the same
    buffers (what a decode loop or a captured graph needs); results live in .out."""

    def __init__(self, ctx, fn, args, out):
        self.ctx, self.fn, self.args, self.out = ctx, fn, args, out

    def launch(self):
        st = self.fn(*self.args)
        if st != 0:
            self.ctx.check(st)


class _TapSet:
    def __init__(self, ctx, specs):
        """specs: list of (n, cols, rows) per product."""
        self.arr = (_Taps * len(specs))()
        self.t = []
        for i, (n, cols, rows) in enumerate(specs):
            xq = ctx.empty(n, cols, dtype=torch.int8)
            xs = ctx.empty(n)
            acc = ctx.empty(n, rows, dtype=torch.int32)
            self.arr[i] = _Taps(xq.data_ptr(), xs.data_ptr(), acc.data_ptr())
            self.t.append({"xq": xq, "xscale": xs, "acc": acc})


def q8_quantize_matrix(ctx, W, ld_out=None):
    W = ctx.f32(W)
    rows, cols = W.shape
    ld_out = (cols + 15) // 16 * 16 if ld_out is None else ld_out
    Wq = ctx.empty(rows, ld_out, dtype=torch.int8)
    scale = C.c_float()
    ctx.check(ctx.lib.q8_quantize_matrix(ctx.handle, _ptr(W), rows, cols, W.stride(0) if rows > 1 else cols, _ptr(Wq), ld_out,
                                         C.byref(scale)))
    return Mat(Wq, cols, scale.value)


def q8_pack_tiles(ctx, W):
    """Returns a Mat sharing W's codes plus their copy in the matrix-core streaming order."""
    nbytes = ctx.lib.q8_tiles_bytes(W.rows, W.ld)
    tiles = ctx.empty(nbytes, dtype=torch.int8)
    ctx.check(ctx.lib.q8_pack_tiles(ctx.handle, C.byref(W.c), _ptr(tiles)))
    return Mat(W.data, W.cols, W.scale, tiles)


def q8_gemv(ctx, W, x, bias=None, y=None, taps=False):
    y = ctx.empty(W.rows) if y is None else y
    ts = _TapSet(ctx, [(1, W.cols, W.rows)]) if taps else None
    ctx.check(ctx.lib.q8_gemv(ctx.handle, C.byref(W.c), _ptr(x), _ptr(bias), _ptr(y), ts.arr if ts else None))
    return (y, ts.t[0]) if taps else y


def q8_gemm_narrow(ctx, W, X, bias=None, Y=None, taps=False):
    n = X.shape[0]
    Y = ctx.empty(n, W.rows) if Y is None else Y
    ts = _TapSet(ctx, [(n, W.cols, W.rows)]) if taps else None
    ctx.check(ctx.lib.q8_gemm_narrow(ctx.handle, C.byref(W.c), _ptr(X), n, X.stride(0), _ptr(bias), _ptr(Y),
                                     Y.stride(0), ts.arr if ts else None))
    return (Y, ts.t[0]) if taps else Y


def q8_quantize_matrix_rows(ctx, W, ld_out=None):
    """One weight scale per row: returns (Mat with scale 0, device tensor of the rows' scales)."""
    W = ctx.f32(W)
    rows, cols = W.shape
    ld_out = (cols + 15) // 16 * 16 if ld_out is None else ld_out
    Wq = ctx.empty(rows, ld_out, dtype=torch.int8)
    row_scale = ctx.empty(rows)
    ctx.check(ctx.lib.q8_quantize_matrix_rows(ctx.handle, _ptr(W), rows, cols, W.stride(0) if rows > 1 else cols, _ptr(Wq),
                                              ld_out, _ptr(row_scale)))
    return Mat(Wq, cols, 0.0), row_scale


def q8_gemm_narrow_rows(ctx, W, row_scale, X, bias=None, Y=None, taps=False):
    n = X.shape[0]
    Y = ctx.empty(n, W.rows) if Y is None else Y
    ts = _TapSet(ctx, [(n, W.cols, W.rows)]) if taps else None
    ctx.check(ctx.lib.q8_gemm_narrow_rows(ctx.handle, C.byref(W.c), _ptr(row_scale), _ptr(X), n, X.stride(0), _ptr(bias),
                                          _ptr(Y), Y.stride(0), ts.arr if ts else None))
    return (Y, ts.t[0]) if taps else Y


def q8_attention_states_q8(ctx, enc_h):
    """The transposed encoder states [C x l] as an int8 matrix with one scale."""
    l, Cc = enc_h.shape
    ld = (l + 15) // 16 * 16
    hT = ctx.empty(Cc, ld, dtype=torch.int8)
    scale = C.c_float()
    ctx.check(ctx.lib.q8_attention_states_q8(ctx.handle, _ptr(enc_h), l, Cc, _ptr(hT), ld, C.byref(scale)))
    return Mat(hT, l, scale.value)


def q8_attention_q8(ctx, v, hT, P, a):
    """Returns (e [n x l], alpha [n x l], ctx [n x C])."""
    n, l = a.shape[0], P.shape[0]
    e, alpha, cvec = ctx.empty(n, l), ctx.empty(n, l), ctx.empty(n, hT.rows)
    ctx.check(ctx.lib.q8_attention_q8(ctx.handle, C.byref(v.c), C.byref(hT.c), _ptr(P), _ptr(a), n, l, _ptr(e),
                                      _ptr(alpha), _ptr(cvec)))
    return e, alpha, cvec


class GruWeights:
    def __init__(self, Wx, Wh, bx=None, bh=None):
        self.Wx, self.Wh, self.bx, self.bh = Wx, Wh, bx, bh
        self.H = Wh.cols
        self.c = _Gru(Wx.c, Wh.c, bx.data_ptr() if bx is not None else None, bh.data_ptr() if bh is not None else None)


class CgruWeights:
    def __init__(self, r, att_U, att_v, q):
        self.r, self.att_U, self.att_v, self.q = r, att_U, att_v, q
        self.c = _Cgru(r.c, att_U.c, att_v.data_ptr(), q.c)


class ReadoutWeights:
    def __init__(self, W_s, W_y, W_c, b_t=None):
        self.W_s, self.W_y, self.W_c, self.b_t = W_s, W_y, W_c, b_t
        self.c = _Readout(W_s.c, W_y.c, W_c.c, b_t.data_ptr() if b_t is not None else None)


def gru_step_q8(ctx, g, x, h_prev, h_out=None, taps=False, bind=False):
    n = x.shape[0]
    h_out = ctx.empty(n, g.H) if h_out is None else h_out
    ts = _TapSet(ctx, [(n, g.Wx.cols, g.Wx.rows), (n, g.Wh.cols, g.Wh.rows)]) if taps else None
    if bind:
        return _Bound(ctx, ctx.lib.gru_step_q8, (ctx.handle, C.byref(g.c), _ptr(x), _ptr(h_prev), n, _ptr(h_out), None),
                      {"h": h_out, "keep": (g, x, h_prev)})
    ctx.check(ctx.lib.gru_step_q8(ctx.handle, C.byref(g.c), _ptr(x), _ptr(h_prev), n, _ptr(h_out), ts.arr if ts else None))
    return (h_out, ts.t) if taps else h_out


def cgru_decoder_step_q8(ctx, w, P, enc_h, y_emb, s_prev, out=None, taps=False, bind=False, codes=None):
    """Returns dict(s, ctx, alpha, s_mid) (+ 'taps': five entries).  codes = (y, ctx) Codes objects:
    cgru_decoder_step_codes_q8, which also leaves the codes of y_emb and of the context vectors there;
    codes = (y, ctx, s_prev): cgru_decoder_step_loop_q8, which also takes the codes of y_emb and s_prev
    that output_logits_beam_q8(codes=(y, ctx, s_next), E_codes=...) left (valid == 2)."""
    n, l = y_emb.shape[0], P.shape[0]
    H, Cd = w.r.H, w.q.Wx.cols
    o = out or {}
    s_out = o.get("s", None)
    s_out = ctx.empty(n, H) if s_out is None else s_out
    c_out = o.get("ctx", None)
    c_out = ctx.empty(n, Cd) if c_out is None else c_out
    alpha = o["alpha"] if "alpha" in o else ctx.empty(n, l)
    s_mid = o["s_mid"] if "s_mid" in o else ctx.empty(n, H)
    ts = None
    if taps:
        A = w.att_U.rows
        ts = _TapSet(ctx, [(n, w.r.Wx.cols, 3 * H), (n, H, 3 * H), (n, H, A), (n, Cd, 3 * H), (n, H, 3 * H)])
    args = (ctx.handle, C.byref(w.c), _ptr(P), _ptr(enc_h), l, _ptr(y_emb), _ptr(s_prev), n,
            _ptr(s_out), _ptr(c_out), _ptr(alpha), _ptr(s_mid), ts.arr if ts else None)
    r = {"s": s_out, "ctx": c_out, "alpha": alpha, "s_mid": s_mid}
    if taps:
        r["taps"] = ts.t
    fn = ctx.lib.cgru_decoder_step_q8
    if codes is not None:
        fn = ctx.lib.cgru_decoder_step_codes_q8 if len(codes) == 2 else ctx.lib.cgru_decoder_step_loop_q8
        args = args + tuple(C.byref(c.c) for c in codes)
    if bind:
        r["keep"] = (w, P, enc_h, y_emb, s_prev, codes)
        return _Bound(ctx, fn, args, r)
    ctx.check(fn(*args))
    return r


def q8_noalloc_setup(ctx):
    ctx.check(ctx.lib.q8_noalloc_setup(ctx.handle))


def q8_noalloc_scratch_bytes():
    return load_library().q8_noalloc_scratch_bytes()


def cgru_decoder_step_noalloc_q8(ctx, w, P, enc_h, y_emb, s_prev, out):
    """cgru_decoder_step_q8 with its scratch in the library's static device array; `out` holds the
    caller's s, ctx, alpha and s_mid tensors (nothing is allocated, here or in the library)."""
    n, l = y_emb.shape[0], P.shape[0]
    ctx.check(ctx.lib.cgru_decoder_step_noalloc_q8(ctx.handle, C.byref(w.c), _ptr(P), _ptr(enc_h), l, _ptr(y_emb), _ptr(s_prev), n,
                                                   _ptr(out["s"]), _ptr(out["ctx"]), _ptr(out.get("alpha")), _ptr(out.get("s_mid"))))
    return out


def cgru_decoder_step_batch_q8(ctx, w, P, enc_h, sent_off, beam, max_l, y_emb, s_prev, out=None, bind=False, codes=None):
    """Decoder step for len(sent_off) - 1 sentences side by side; sent_off: device int32 offsets
    into P / enc_h.  Returns dict(s, ctx, alpha [n x max_l], s_mid).  codes = (y, ctx, s) Codes objects:
    cgru_decoder_step_batch_codes_q8, which leaves the three sets of codes there; codes = (y, ctx, s, s_prev):
    cgru_decoder_step_batch_loop_q8, which also takes the codes of y_emb and s_prev that
    q8_beam_update_batch(codes=..., E_codes=...) left."""
    n = y_emb.shape[0]
    S = sent_off.shape[0] - 1
    assert n == S * beam
    H, Cd = w.r.H, w.q.Wx.cols
    o = out or {}
    s_out = o["s"] if "s" in o else ctx.empty(n, H)
    c_out = o["ctx"] if "ctx" in o else ctx.empty(n, Cd)
    alpha = o["alpha"] if "alpha" in o else torch.zeros(n, max_l, dtype=torch.float32, device=ctx.device)
    s_mid = o["s_mid"] if "s_mid" in o else ctx.empty(n, H)
    args = (ctx.handle, C.byref(w.c), _ptr(P), _ptr(enc_h), _ptr(sent_off), S, beam, max_l, _ptr(y_emb), _ptr(s_prev),
            _ptr(s_out), _ptr(c_out), _ptr(alpha), _ptr(s_mid))
    r = {"s": s_out, "ctx": c_out, "alpha": alpha, "s_mid": s_mid}
    fn = ctx.lib.cgru_decoder_step_batch_q8
    if codes is not None:
        fn = ctx.lib.cgru_decoder_step_batch_codes_q8 if len(codes) == 3 else ctx.lib.cgru_decoder_step_batch_loop_q8
        args = args + tuple(C.byref(c.c) for c in codes)
    if bind:
        r["keep"] = (w, P, enc_h, sent_off, y_emb, s_prev, codes)
        return _Bound(ctx, fn, args, r)
    ctx.check(fn(*args))
    return r


def output_logits_q8(ctx, ro, W_out, b_out, s=None, y_emb=None, ctx_vec=None, t_in=None, k=12,
                     want_logits=True, taps=False, bind=False, codes=None):
    """Returns dict(logits?, lse, topk_logp, topk_idx, t?) (+ 'taps': four entries).  codes = (y, ctx, s)
    Codes objects from cgru_decoder_step_batch_q8(codes=...): output_logits_codes_q8 (needs ro, no taps)."""
    n = (t_in if ro is None else s).shape[0]
    V, R = W_out.rows, W_out.cols
    logits = ctx.empty(n, V) if want_logits else None
    lse = ctx.empty(n)
    lp = ctx.empty(n, k)
    idx = ctx.empty(n, k, dtype=torch.int32)
    t_out = ctx.empty(n, R) if ro is not None else None
    ts = None
    if taps:
        if ro is not None:
            specs = [(n, ro.W_s.cols, R), (n, ro.W_y.cols, R), (n, ro.W_c.cols, R), (n, R, V)]
        else:
            specs = [(1, 1, 1)] * 3 + [(n, R, V)]
        ts = _TapSet(ctx, specs)
    args = (ctx.handle, C.byref(ro.c) if ro is not None else None, C.byref(W_out.c), _ptr(b_out),
            _ptr(s), _ptr(y_emb), _ptr(ctx_vec), _ptr(t_in), n, k, _ptr(logits), _ptr(lse),
            _ptr(lp), _ptr(idx), _ptr(t_out), ts.arr if ts else None)
    r = {"logits": logits, "lse": lse, "topk_logp": lp, "topk_idx": idx, "t": t_out}
    if taps:
        r["taps"] = ts.t
    fn = ctx.lib.output_logits_q8
    if codes is not None:
        assert ro is not None and not taps
        fn = ctx.lib.output_logits_codes_q8
        args = (ctx.handle, C.byref(ro.c), C.byref(W_out.c), _ptr(b_out), _ptr(s), _ptr(y_emb), _ptr(ctx_vec), n, k,
                _ptr(logits), _ptr(lse), _ptr(lp), _ptr(idx), _ptr(t_out),
                C.byref(codes[2].c), C.byref(codes[0].c), C.byref(codes[1].c))
    if bind:
        r["keep"] = (ro, W_out, b_out, s, y_emb, ctx_vec, t_in, codes)
        return _Bound(ctx, fn, args, r)
    ctx.check(fn(*args))
    return r


def q8_encoder_options(ctx, one_launch=True, spin_limit=0):
    ctx.check(ctx.lib.q8_encoder_options(ctx.handle, 1 if one_launch else 0, spin_limit))


def q8_encode_check(ctx):
    ctx.check(ctx.lib.q8_encode_check(ctx.handle))


def q8_attention_options(ctx, exchange=True, spin_limit=0):
    ctx.check(ctx.lib.q8_attention_options(ctx.handle, int(exchange), spin_limit))


def q8_encode(ctx, fwd, bwd, X, enc_h=None):
    l = X.shape[0]
    enc_h = ctx.empty(l, 2 * fwd.H) if enc_h is None else enc_h
    ctx.check(ctx.lib.q8_encode(ctx.handle, C.byref(fwd.c), C.byref(bwd.c), _ptr(X), l, _ptr(enc_h)))
    return enc_h


KERNEL_CLASSES = {"vocab": 0, "select": 1, "gemv": 2, "gru": 3, "attention": 4, "readout": 5, "mfma": 6, "probe": 7}


def q8_encode_batch_bytes(fwd, total_l, n_sent):
    return load_library().q8_encode_batch_bytes(C.byref(fwd.c), total_l, n_sent)


def q8_encode_batch(ctx, fwd, bwd, X, lengths, enc_h=None):
    """Encoder for sentences of the given lengths, whose embeddings are the rows of X back to back."""
    import numpy as np
    off = np.zeros(len(lengths) + 1, dtype=np.int32)
    off[1:] = np.cumsum(lengths)
    assert off[-1] == X.shape[0]
    off_dev = torch.as_tensor(off).to(ctx.device)
    enc_h = ctx.empty(X.shape[0], 2 * fwd.H) if enc_h is None else enc_h
    ctx.check(ctx.lib.q8_encode_batch(ctx.handle, C.byref(fwd.c), C.byref(bwd.c), _ptr(X), _ptr(off_dev),
                                      off.ctypes.data_as(C.POINTER(C.c_int)), len(lengths), _ptr(enc_h)))
    return enc_h


def q8_profile_begin(ctx, kernel_class, max_samples):
    ctx.check(ctx.lib.q8_profile_begin(ctx.handle, KERNEL_CLASSES[kernel_class], max_samples))


def q8_math_eval(ctx, fn, x):
    """The device's own tanh ("tanh"), sigmoid ("sigmoid") (float32 tensors) or exp ("exp", float64) of x;
    "sort64": every 64 consecutive floats in descending order (a multiple of 256 values)."""
    code = {"tanh": 0, "sigmoid": 1, "exp": 2, "sort64": 3}[fn]
    want = torch.float64 if code == 2 else torch.float32
    if x.dtype != want or not x.is_contiguous():
        raise ValueError("q8_math_eval(%s) takes a contiguous %s tensor" % (fn, want))
    y = torch.empty_like(x)
    ctx.check(ctx.lib.q8_math_eval(ctx.handle, code, _ptr(x), _ptr(y), x.numel()))
    return y


def q8_probe_read(ctx, buf):
    ctx.check(ctx.lib.q8_probe_read(ctx.handle, _ptr(buf), buf.numel() * buf.element_size()))


def q8_profile_end(ctx):
    ms, n = C.c_float(), C.c_int()
    ctx.check(ctx.lib.q8_profile_end(ctx.handle, C.byref(ms), C.byref(n)))
    return ms.value, n.value


class Model:
    """q8_model: every tensor of the translation model, already on the device."""

    def __init__(self, E_src, E_tgt, enc_fwd, enc_bwd, att_W, att_b, dec, ro, W_out, b_out):
        self.keep = (E_src, E_tgt, enc_fwd, enc_bwd, att_W, att_b, dec, ro, W_out, b_out)
        self.E_src, self.E_tgt, self.dec, self.ro, self.W_out, self.b_out = E_src, E_tgt, dec, ro, W_out, b_out
        self.enc_fwd, self.enc_bwd, self.att_W, self.att_b = enc_fwd, enc_bwd, att_W, att_b
        self.c = _Model(E_src.data_ptr(), E_tgt.data_ptr(), E_src.shape[0], E_tgt.shape[0], E_src.shape[1],
                        enc_fwd.c, enc_bwd.c, att_W.c, att_b.data_ptr() if att_b is not None else None,
                        dec.c, ro.c, W_out.c, b_out.data_ptr() if b_out is not None else None)

    @classmethod
    def from_params(cls, ctx, p, gx_table=True):
        """Quantizes a dict of fp32 arrays (keys as in workloads.synth.full_model) on the device.  gx_table: also
        make the table of GRU r's input products over the target vocabulary (12 H bytes per token), with which
        q8_translate keeps GRU r off the chain of dependent launches."""
        def mat(k):
            # rows of whole 64-byte k steps are also kept tile-packed: the matrix-core products of panels read
            # that copy (one contiguous KiB per operand)
            W = q8_quantize_matrix(ctx, p[k])
            return q8_pack_tiles(ctx, W) if W.ld % 64 == 0 else W
        gru = lambda pre: GruWeights(mat(pre + ".Wx"), mat(pre + ".Wh"), ctx.f32(p[pre + ".bx"]), ctx.f32(p[pre + ".bh"]))
        dec = CgruWeights(gru("dec_r"), mat("att.U"), ctx.f32(p["att.v"]), gru("dec_q"))
        ro = ReadoutWeights(mat("ro.Ws"), mat("ro.Wy"), mat("ro.Wc"), ctx.f32(p["ro.b"]))
        # the streaming order of the vocabulary layer needs whole 64-byte k steps: wide rows are
        # padded (with zero codes) to the next multiple of 64, narrow test models stay unpacked
        R = p["out.W"].shape[1]
        out_W = q8_quantize_matrix(ctx, p["out.W"], ld_out=(R + 63) // 64 * 64 if R >= 256 else None)
        if out_W.ld % 64 == 0:
            out_W = q8_pack_tiles(ctx, out_W)
        m = cls(ctx.f32(p["E_src"]), ctx.f32(p["E_tgt"]), gru("enc_fwd"), gru("enc_bwd"), mat("att.W"),
                ctx.f32(p["att.b"]), dec, ro, out_W, ctx.f32(p["out.b"]))
        # the target embeddings' codes, row by row, for decoding loops that hand codes from step to step
        m.E_tgt_codes = RowCodes(ctx, m.E_tgt, dec.r.Wx.ld)
        m.c.E_tgt_codes = m.E_tgt_codes.c
        m.gx_r = gru_input_table(ctx, dec.r, m.E_tgt) if gx_table else None
        m.c.gx_r = m.gx_r.data_ptr() if gx_table else None
        return m


def gru_input_table(ctx, g, E, rows=1024):
    """W_x q(E[v]) + b_x for every row v of the embedding table E: [V x 3H] fp32 on the device (the table
    cgru_decoder_step_ahead_q8 / output_logits_beam_ahead_q8 gather GRU r's input half from), made with
    q8_gemm_narrow in panels of `rows` rows on a context of its own (a panel needs a larger workspace)."""
    tmp = Context(ctx.device, workspace_bytes=q8_workspace_bytes(max_n=rows, max_ld=max(2048, g.Wx.ld)), stream=ctx.stream)
    V = E.shape[0]
    G = torch.empty(V, g.Wx.rows, dtype=torch.float32, device=ctx.device)
    for o in range(0, V, rows):
        q8_gemm_narrow(tmp, g.Wx, E[o:o + rows], g.bx, Y=G[o:o + rows])
    torch.cuda.synchronize(ctx.device)
    tmp.close()
    return G


def cgru_decoder_step_ahead_q8(ctx, w, P, enc_h, s_mid, out=None, bind=False, ctx_codes=None):
    """The decoder step from a given s' (Eq. 4-6); returns dict(s, ctx, alpha)."""
    n, l = s_mid.shape[0], P.shape[0]
    H, Cd = w.r.H, w.q.Wx.cols
    o = out or {}
    s_out = o["s"] if "s" in o else ctx.empty(n, H)
    c_out = o["ctx"] if "ctx" in o else ctx.empty(n, Cd)
    alpha = o["alpha"] if "alpha" in o else ctx.empty(n, l)
    args = (ctx.handle, C.byref(w.c), _ptr(P), _ptr(enc_h), l, _ptr(s_mid), n, _ptr(s_out), _ptr(c_out), _ptr(alpha),
            C.byref(ctx_codes.c) if ctx_codes is not None else None)
    r = {"s": s_out, "ctx": c_out, "alpha": alpha}
    if bind:
        r["keep"] = (w, P, enc_h, s_mid, ctx_codes)
        return _Bound(ctx, ctx.lib.cgru_decoder_step_ahead_q8, args, r)
    ctx.check(ctx.lib.cgru_decoder_step_ahead_q8(*args))
    return r


def output_logits_beam_ahead_q8(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, state, E_tgt, gru_r, gx_table, s_mid_next, k=12,
                                bind=False, y_codes=None, ctx_codes=None, E_codes=None):
    """Output layer + top-k + search step + GRU r of the next step (its recurrent product in the readout's launch,
    its gates in the selection kernel's: s_mid_next); returns dict(topk_logp, topk_idx)."""
    n = s.shape[0]
    lp = ctx.empty(n, k)
    idx = ctx.empty(n, k, dtype=torch.int32)
    by = lambda c: C.byref(c.c) if c is not None else None
    args = (ctx.handle, C.byref(ro.c), C.byref(W_out.c), _ptr(b_out), _ptr(s), _ptr(y_emb), _ptr(ctx_vec), n, k,
            _ptr(state), _ptr(E_tgt), E_tgt.shape[1], _ptr(lp), _ptr(idx), by(y_codes), by(ctx_codes), by(E_codes),
            C.byref(gru_r.c), _ptr(gx_table), _ptr(s_mid_next))
    r = {"topk_logp": lp, "topk_idx": idx}
    if bind:
        r["keep"] = (ro, W_out, b_out, s, y_emb, ctx_vec, state, E_tgt, gru_r, gx_table, s_mid_next, y_codes, ctx_codes, E_codes)
        return _Bound(ctx, ctx.lib.output_logits_beam_ahead_q8, args, r)
    ctx.check(ctx.lib.output_logits_beam_ahead_q8(*args))
    return r


def source_ids(ids, V_src, device=None):
    """Source token ids as a device int32 tensor.  Ids that arrive on the host (lists, arrays, CPU
    tensors) are checked against [0, V_src) here and a violation raises ValueError; a tensor that
    is already on the device is passed through unread (the kernels look up an id outside the
    table as a zero vector)."""
    import numpy as np
    if isinstance(ids, torch.Tensor) and ids.is_cuda:
        if ids.dtype != torch.int32:
            raise ValueError("device token ids must be int32")
        return ids
    a = np.asarray(ids.numpy() if isinstance(ids, torch.Tensor) else ids)
    if a.ndim != 1 or a.size == 0 or not np.issubdtype(a.dtype, np.integer):
        raise ValueError("token ids: a non-empty one-dimensional integer sequence is required")
    if int(a.min()) < 0 or int(a.max()) >= V_src:
        raise ValueError("token id outside [0, %d)" % V_src)
    t = torch.as_tensor(a.astype(np.int32))
    return t if device is None else t.to(device)


def q8_translate_bytes(model, max_l, beam, k, max_steps):
    return load_library().q8_translate_bytes(C.byref(model.c), max_l, beam, k, max_steps)


def q8_translate(ctx, model, src_tokens, beam=5, k=12, max_steps=100):
    """Returns (tokens ndarray, score, steps)."""
    import numpy as np
    src = source_ids(src_tokens, model.E_src.shape[0], ctx.device)
    out = (C.c_int32 * max_steps)()
    n, steps, score = C.c_int(), C.c_int(), C.c_float()
    ctx.check(ctx.lib.q8_translate(ctx.handle, C.byref(model.c), _ptr(src), src.shape[0], beam, k, max_steps,
                                   out, C.byref(n), C.byref(score), C.byref(steps)))
    return np.array(out[:n.value], dtype=np.int32), np.float32(score.value), steps.value


def q8_gemv_f32(ctx, W, X, bias=None, Y=None):
    """fp32 product of the 32-bit engine for n <= 8 vectors X [n x cols] (or one vector [cols])."""
    one = X.dim() == 1
    n = 1 if one else X.shape[0]
    ldx = W.cols if one else X.stride(0)
    Y = ctx.empty(n, W.rows) if Y is None else Y
    ctx.check(ctx.lib.q8_gemv_f32(ctx.handle, C.byref(W.c), _ptr(X), n, ldx, _ptr(bias), _ptr(Y), W.rows))
    return Y[0] if one else Y


def cgru_decoder_step_f32(ctx, w, P, enc_h, y_emb, s_prev, bind=False):
    n, l = y_emb.shape[0], P.shape[0]
    H, Cd = w.r.H, w.q.Wx.cols
    r = {"s": ctx.empty(n, H), "ctx": ctx.empty(n, Cd), "alpha": ctx.empty(n, l), "s_mid": ctx.empty(n, H)}
    args = (ctx.handle, C.byref(w.c), _ptr(P), _ptr(enc_h), l, _ptr(y_emb), _ptr(s_prev), n, _ptr(r["s"]), _ptr(r["ctx"]),
            _ptr(r["alpha"]), _ptr(r["s_mid"]))
    if bind:
        r["keep"] = (w, P, enc_h, y_emb, s_prev)
        return _Bound(ctx, ctx.lib.cgru_decoder_step_f32, args, r)
    ctx.check(ctx.lib.cgru_decoder_step_f32(*args))
    return r


def output_logits_f32(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, k=12, want_logits=True, bind=False):
    n, V, R = s.shape[0], W_out.rows, W_out.cols
    r = {"lse": ctx.empty(n), "topk_logp": ctx.empty(n, k), "topk_idx": ctx.empty(n, k, dtype=torch.int32), "t": ctx.empty(n, R)}
    if want_logits:
        r["logits"] = ctx.empty(n, V)
    args = (ctx.handle, C.byref(ro.c), C.byref(W_out.c), _ptr(b_out), _ptr(s), _ptr(y_emb), _ptr(ctx_vec), n, k,
            _ptr(r.get("logits")), _ptr(r["lse"]), _ptr(r["topk_logp"]), _ptr(r["topk_idx"]), _ptr(r["t"]))
    if bind:
        r["keep"] = (ro, W_out, b_out, s, y_emb, ctx_vec)
        return _Bound(ctx, ctx.lib.output_logits_f32, args, r)
    ctx.check(ctx.lib.output_logits_f32(*args))
    return r


def _model_ptrs(models):
    return (C.c_void_p * len(models))(*[C.addressof(m.c) for m in models])


def q8_translate_ensemble_bytes(models, max_l, beam=5, k=12, max_steps=100):
    return load_library().q8_translate_ensemble_bytes(_model_ptrs(models), len(models), max_l, beam, k, max_steps)


def q8_translate_ensemble(ctx, models, src_tokens, beam=5, k=12, max_steps=100):
    """Ensemble decoding over a list of Model objects; returns (tokens ndarray, score, steps)."""
    import numpy as np
    src = source_ids(src_tokens, min(m.E_src.shape[0] for m in models), ctx.device)
    out = (C.c_int32 * max_steps)()
    n, steps, score = C.c_int(), C.c_int(), C.c_float()
    ctx.check(ctx.lib.q8_translate_ensemble(ctx.handle, _model_ptrs(models), len(models), _ptr(src), src.shape[0], beam, k,
                                            max_steps, out, C.byref(n), C.byref(score), C.byref(steps)))
    return np.array(out[:n.value], dtype=np.int32), np.float32(score.value), steps.value


def q8_translate_batch_bytes(model, total_l, n_sent, beam=5, k=12, max_steps=100):
    return load_library().q8_translate_batch_bytes(C.byref(model.c), total_l, n_sent, beam, k, max_steps)


def q8_translate_batch(ctx, model, sentences, beam=5, k=12, max_steps=100):
    """Translates the sentences together; returns a list of (tokens ndarray, score, steps)."""
    import numpy as np
    S = len(sentences)
    off = np.zeros(S + 1, dtype=np.int32)
    off[1:] = np.cumsum([len(x) for x in sentences])
    V_src = model.E_src.shape[0]
    if any(isinstance(x, torch.Tensor) and x.is_cuda for x in sentences):
        src = torch.cat([source_ids(x, V_src, ctx.device) for x in sentences])
    else:
        # ids that arrive on the host: checked here, then one transfer for all sentences (not one per sentence)
        src = torch.cat([source_ids(x, V_src) for x in sentences]).to(ctx.device)
    out = (C.c_int32 * (max_steps * S))()
    n, steps, score = (C.c_int * S)(), (C.c_int * S)(), (C.c_float * S)()
    ctx.check(ctx.lib.q8_translate_batch(ctx.handle, C.byref(model.c), _ptr(src), off.ctypes.data_as(C.POINTER(C.c_int)), S,
                                         beam, k, max_steps, out, n, score, steps))
    return [(np.array(out[i * max_steps:i * max_steps + n[i]], dtype=np.int32), np.float32(score[i]), steps[i])
            for i in range(S)]


def q8_beam_init_batch(ctx, states, n_sent, beam, max_steps, enc_h, sent_off, E_tgt, y_emb, s, done, bind=False):
    args = (ctx.handle, _ptr(states), n_sent, beam, max_steps, _ptr(enc_h), _ptr(sent_off), enc_h.shape[1], _ptr(E_tgt),
            E_tgt.shape[1], s.shape[1], _ptr(y_emb), _ptr(s), _ptr(done))
    if bind:
        return _Bound(ctx, ctx.lib.q8_beam_init_batch, args, {"keep": (states, enc_h, sent_off, E_tgt, y_emb, s, done)})
    ctx.check(ctx.lib.q8_beam_init_batch(*args))


def q8_beam_update_batch(ctx, states, n_sent, beam, max_steps, topk_logp, topk_idx, s_step, E_tgt, y_emb, s_next, done,
                         bind=False, codes=None, E_codes=None):
    """codes = (s, y_next, s_next) Codes objects with E_codes (RowCodes of E_tgt): q8_beam_update_batch_loop, which
    gathers the codes of s_step's rows (s) and of the new tokens' embeddings into s_next / y_next."""
    k = topk_logp.shape[1]
    args = (ctx.handle, _ptr(states), n_sent, beam, k, max_steps, _ptr(topk_logp), _ptr(topk_idx), _ptr(s_step),
            s_step.shape[1], _ptr(E_tgt), E_tgt.shape[1])
    fn = ctx.lib.q8_beam_update_batch
    if codes is not None:
        fn = ctx.lib.q8_beam_update_batch_loop
        args = args + (E_tgt.shape[0], _ptr(y_emb), _ptr(s_next), _ptr(done), C.byref(E_codes.c)) + tuple(C.byref(c.c) for c in codes)
    else:
        args = args + (_ptr(y_emb), _ptr(s_next), _ptr(done))
    if bind:
        return _Bound(ctx, fn, args, {"keep": (states, topk_logp, topk_idx, s_step, E_tgt, y_emb, s_next, done, codes, E_codes)})
    ctx.check(fn(*args))


def output_logits_beam_batch_q8(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, states, n_sent, beam, max_steps, E_tgt, s_next,
                                done, k=12, bind=False, codes=None, s_next_codes=None, E_codes=None):
    """Output layer of a panel of n_sent beams, top-k and every sentence's search step; returns
    dict(topk_logp, topk_idx).  codes = (s, y, ctx) Codes objects of this step (as for output_logits_q8);
    with s_next_codes and E_codes (RowCodes of E_tgt) the codes of the new y_emb (in y) and of s_next go
    to the next decoder step."""
    n = s.shape[0]
    lp = ctx.empty(n, k)
    idx = ctx.empty(n, k, dtype=torch.int32)
    by = lambda c: C.byref(c.c) if c is not None else None
    sc, yc, cc = codes if codes is not None else (None, None, None)
    args = (ctx.handle, C.byref(ro.c), C.byref(W_out.c), _ptr(b_out), _ptr(s), _ptr(y_emb), _ptr(ctx_vec), n_sent, beam, k,
            max_steps, _ptr(states), _ptr(E_tgt), E_tgt.shape[1], _ptr(s_next), _ptr(done), _ptr(lp), _ptr(idx),
            by(sc), by(yc), by(cc), by(s_next_codes), by(E_codes))
    r = {"topk_logp": lp, "topk_idx": idx}
    if bind:
        r["keep"] = (ro, W_out, b_out, s, y_emb, ctx_vec, states, E_tgt, s_next, done, codes, s_next_codes, E_codes)
        return _Bound(ctx, ctx.lib.output_logits_beam_batch_q8, args, r)
    ctx.check(ctx.lib.output_logits_beam_batch_q8(*args))
    return r


def q8_beam_result_batch(ctx, states, n_sent, max_steps):
    import numpy as np
    out = (C.c_int32 * (max_steps * n_sent))()
    n, steps, score = (C.c_int * n_sent)(), (C.c_int * n_sent)(), (C.c_float * n_sent)()
    ctx.check(ctx.lib.q8_beam_result_batch(ctx.handle, _ptr(states), n_sent, max_steps, out, n, score, steps))
    return [(np.array(out[i * max_steps:i * max_steps + n[i]], dtype=np.int32), np.float32(score[i]), steps[i])
            for i in range(n_sent)]


def q8_beam_state_bytes(max_steps):
    return load_library().q8_beam_state_bytes(max_steps)


def q8_beam_init(ctx, state, beam, max_steps, s0, E_tgt, y_emb, s, bind=False):
    args = (ctx.handle, _ptr(state), beam, max_steps, _ptr(s0), _ptr(E_tgt), E_tgt.shape[1], s.shape[1], _ptr(y_emb), _ptr(s))
    if bind:
        return _Bound(ctx, ctx.lib.q8_beam_init, args, {"keep": (state, s0, E_tgt, y_emb, s)})
    ctx.check(ctx.lib.q8_beam_init(*args))


def q8_beam_update(ctx, state, topk_logp, topk_idx, s_step, E_tgt, y_emb, s_next, bind=False):
    n, k = topk_logp.shape
    args = (ctx.handle, _ptr(state), _ptr(topk_logp), _ptr(topk_idx), n, k, _ptr(s_step), s_step.shape[1],
            _ptr(E_tgt), E_tgt.shape[1], _ptr(y_emb), _ptr(s_next))
    if bind:
        return _Bound(ctx, ctx.lib.q8_beam_update, args, {"keep": (state, topk_logp, topk_idx, s_step, E_tgt, y_emb, s_next)})
    ctx.check(ctx.lib.q8_beam_update(*args))


def q8_beam_result(ctx, state, max_steps):
    """Returns (tokens, score, steps, done)."""
    import numpy as np
    out = (C.c_int32 * max_steps)()
    n, steps, done, score = C.c_int(), C.c_int(), C.c_int(), C.c_float()
    ctx.check(ctx.lib.q8_beam_result(ctx.handle, _ptr(state), max_steps, out, C.byref(n), C.byref(score), C.byref(steps),
                                     C.byref(done)))
    return np.array(out[:n.value], dtype=np.int32), np.float32(score.value), steps.value, bool(done.value)


def output_logits_beam_q8(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, state, E_tgt, s_next, k=12, bind=False, codes=None,
                          E_codes=None):
    """Output layer + top-k + beam update; returns dict(topk_logp, topk_idx).  codes = (y, ctx) Codes
    objects filled by cgru_decoder_step_q8(codes=...): output_logits_beam_codes_q8.  codes = (y, ctx,
    s_next) with E_codes (RowCodes of E_tgt): output_logits_beam_loop_q8, which also leaves the codes
    of the new y_emb and of s_next for the next decoder step."""
    n = s.shape[0]
    lp = ctx.empty(n, k)
    idx = ctx.empty(n, k, dtype=torch.int32)
    args = (ctx.handle, C.byref(ro.c), C.byref(W_out.c), _ptr(b_out), _ptr(s), _ptr(y_emb), _ptr(ctx_vec), n, k,
            _ptr(state), _ptr(E_tgt), E_tgt.shape[1], _ptr(s_next), _ptr(lp), _ptr(idx))
    r = {"topk_logp": lp, "topk_idx": idx}
    fn = ctx.lib.output_logits_beam_q8
    if codes is not None and len(codes) == 3:
        fn = ctx.lib.output_logits_beam_loop_q8
        args = args + tuple(C.byref(c.c) for c in codes) + (C.byref(E_codes.c) if E_codes is not None else None,)
    elif codes is not None:
        fn = ctx.lib.output_logits_beam_codes_q8
        args = args + (C.byref(codes[0].c), C.byref(codes[1].c))
    if bind:
        r["keep"] = (ro, W_out, b_out, s, y_emb, ctx_vec, state, E_tgt, s_next, codes, E_codes)
        return _Bound(ctx, fn, args, r)
    ctx.check(fn(*args))
    return r
