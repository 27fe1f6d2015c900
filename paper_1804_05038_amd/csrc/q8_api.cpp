// q8_api.cpp -- the C ABI declared in q8nmt.h: argument validation, workspace carving
// and the sequence of launches that makes up each call.  All arithmetic is in the
// kernels (the .hip files beside this one).
#include "q8_internal.h"

#include <new>
#include <stdlib.h>
#include <string.h>

namespace {

const int kMaxLd = 16384, kMaxNarrow = 8, kMaxMfmaN = 1024, kMaxL = 1024, kMaxK = 16;

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

// Bump allocator over the caller's workspace (after the header).
struct Carver {
    char *base;
    size_t cap, off;
    bool ok;
    explicit Carver(q8_ctx *c) : base(c->ws), cap(c->ws_bytes - c->ws_reserved_top), off(Q8_WS_HEADER), ok(true) {}
    template <class T> T *take(size_t count)
    {
        size_t bytes = up256(count * sizeof(T));
        if (off + bytes > cap) { ok = false; return nullptr; }
        T *p = (T *)(base + off);
        off += bytes;
        return p;
    }
};

q8_status check_mat(q8_ctx *ctx, const q8_mat *W, const char *name)
{
    if (!W || !W->data) return q8_fail(ctx, Q8_ERR_NULL, "%s: NULL matrix", name);
    if (W->rows <= 0 || W->cols <= 0 || W->ld < W->cols || W->ld > kMaxLd)
        return q8_fail(ctx, Q8_ERR_SHAPE, "%s: bad shape %d x %d (ld %d)", name, W->rows, W->cols, W->ld);
    if (!aligned16(W->data) || W->ld % 16 != 0)
        return q8_fail(ctx, Q8_ERR_ALIGN, "%s: int8 matrix needs a 16-byte aligned base and ld %% 16 == 0", name);
    return Q8_OK;
}

q8_status check_vecs(q8_ctx *ctx, const float *p, int ld, int cols, const char *name)
{
    if (!p) return q8_fail(ctx, Q8_ERR_NULL, "%s: NULL", name);
    if (ld < cols) return q8_fail(ctx, Q8_ERR_SHAPE, "%s: leading dimension %d < %d", name, ld, cols);
    if (!aligned16(p) || ld % 4 != 0)
        return q8_fail(ctx, Q8_ERR_ALIGN, "%s: fp32 vectors need a 16-byte aligned base and ld %% 4 == 0", name);
    return Q8_OK;
}

q8_status check_gru(q8_ctx *ctx, const q8_gru_weights *g, const char *name)
{
    if (!g) return q8_fail(ctx, Q8_ERR_NULL, "%s: NULL", name);
    q8_status st = check_mat(ctx, &g->Wx, name);
    if (!st) st = check_mat(ctx, &g->Wh, name);
    if (st) return st;
    const int H = g->Wh.cols;
    if (g->Wh.rows != 3 * H || g->Wx.rows != 3 * H)
        return q8_fail(ctx, Q8_ERR_SHAPE, "%s: expected Wx [3H x I], Wh [3H x H]", name);
    return Q8_OK;
}

#define TRY(expr) do { q8_status st_ = (expr); if (st_) return st_; } while (0)

// ---- panels of more than 8 vectors: quantize, matrix-core products, element-wise tail ----

// One GRU transition for n vectors (Eq. 1, 3, 4): h_out = GRU(x, h_prev).  gh_pre non-NULL:
// the recurrent product (bias included) is already there and x alone is multiplied.
// codes of the new states for whoever consumes them next (see q8i_gru_gates_q)
struct PanelCodesOut {
    int8_t *q1; int ld1; float *s1;
    int8_t *q2; int ld2; float *s2;
};

// whether a caller's code buffers can hold the codes of vectors multiplied by a matrix of pitch ld
bool codes_usable(const q8_codes *c, int ld)
{
    return c && c->q && c->scale && c->ld == ld && aligned16(c->q);
}

// xq_pre / xs_pre (with gh_pre only): x arrives quantized.  out: the gates kernel also quantizes h_out.
// x_keep: x's codes are written to the caller's buffers; with h_given (no gh_pre, no taps) they are there
// already, like those of h_prev in h_given, and nothing is quantized.
q8_status gru_panel(q8_ctx *ctx, Carver &cv, const q8_gru_weights *g, const float *x, const float *h_prev, int n,
                    const float *gh_pre, float *h_out, const q8_taps *taps2, const int8_t *xq_pre = nullptr,
                    const float *xs_pre = nullptr, const PanelCodesOut *out = nullptr, const q8_codes *x_keep = nullptr,
                    const q8_codes *h_given = nullptr, int region = 0)
{
    const int I = g->Wx.cols, H = g->Wh.cols;
    // products, gates and codes in one launch where the shape allows (no pre-activations in memory)
    const bool one_launch = !taps2 && q8i_gru_panel_ok(ctx, g, gh_pre != nullptr, n, H, H, out != nullptr, out ? out->ld1 : 0, out ? out->ld2 : 0, out && out->q2);
    auto panel = [&](const int8_t *xq_, const float *xs_, const int8_t *hq_, const float *hs_) {
        return q8i_gru_panel(ctx, g, xq_, xs_, hq_, hs_, gh_pre, h_prev, H, h_out, H, n, out ? out->q1 : nullptr, out ? out->ld1 : 0,
                             out ? out->s1 : nullptr, out ? out->q2 : nullptr, out ? out->ld2 : 0, out ? out->s2 : nullptr, region);
    };
    if (h_given && x_keep && !gh_pre && !taps2) {
        if (one_launch) return panel(x_keep->q, x_keep->scale, h_given->q, h_given->scale);
        float *gx = cv.take<float>((size_t)n * 3 * H), *gh = cv.take<float>((size_t)n * 3 * H);
        if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "GRU panel: workspace too small");
        const q8i_gemm_job gj[2] = {{&g->Wx, x_keep->q, x_keep->scale, g->bx, gx, 3 * H, nullptr, nullptr, nullptr, 0},
                                    {&g->Wh, h_given->q, h_given->scale, g->bh, gh, 3 * H, nullptr, nullptr, nullptr, 0}};
        TRY(q8i_gemm_jobs(ctx, gj, 2, n));
        if (out)
            return q8i_gru_gates_q(ctx, gx, gh, h_prev, H, h_out, H, H, n, out->q1, out->ld1, out->s1, out->q2, out->ld2, out->s2);
        return q8i_gru_gates(ctx, gx, gh, h_prev, H, h_out, H, H, n);
    }
    const bool have_x = gh_pre && xq_pre && xs_pre && !taps2;
    int8_t *xq = have_x ? nullptr : cv.take<int8_t>((size_t)n * g->Wx.ld), *hq = gh_pre ? nullptr : cv.take<int8_t>((size_t)n * g->Wh.ld);
    float *xs = have_x ? nullptr : cv.take<float>(n), *hs = cv.take<float>(n);
    if (!have_x && x_keep) { xq = x_keep->q; xs = x_keep->scale; }       // x's codes stay with the caller (pitch checked there)
    float *gx = one_launch ? nullptr : cv.take<float>((size_t)n * 3 * H);
    float *gh = gh_pre || one_launch ? nullptr : cv.take<float>((size_t)n * 3 * H);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "GRU panel: workspace too small");
    if (!have_x) {
        const q8i_quant_job qj[2] = {{x, I, I, g->Wx.ld, xq, xs, taps2}, {h_prev, H, H, g->Wh.ld, hq, hs, taps2 ? taps2 + 1 : nullptr}};
        TRY(q8i_quantize_jobs(ctx, qj, gh_pre ? 1 : 2, n));
    }
    if (one_launch) return panel(have_x ? xq_pre : xq, have_x ? xs_pre : xs, hq, hs);
    const q8i_gemm_job gj[2] = {{&g->Wx, have_x ? xq_pre : xq, have_x ? xs_pre : xs, g->bx, gx, 3 * H, taps2 ? taps2[0].acc : nullptr, nullptr, nullptr, 0},
                                {&g->Wh, hq, hs, g->bh, gh, 3 * H, taps2 ? taps2[1].acc : nullptr, nullptr, nullptr, 0}};
    TRY(q8i_gemm_jobs(ctx, gj, gh_pre ? 1 : 2, n));
    if (out)
        return q8i_gru_gates_q(ctx, gx, gh_pre ? gh_pre : gh, h_prev, H, h_out, H, H, n, out->q1, out->ld1, out->s1, out->q2,
                               out->ld2, out->s2);
    return q8i_gru_gates(ctx, gx, gh_pre ? gh_pre : gh, h_prev, H, h_out, H, H, n);
}

}  // namespace

extern "C" {

size_t q8_workspace_bytes(int max_n, int max_l, int max_rows, int max_ld)
{
    if (max_n < 1) max_n = 1;
    if (max_l < 1) max_l = 1;
    if (max_rows < 1) max_rows = 1;
    if (max_ld < 16) max_ld = 16;
    const size_t nv = (size_t)(max_n > max_l ? max_n : max_l);
    size_t b = Q8_WS_HEADER;
    b += up256(nv * (size_t)max_ld) + up256(nv * 4);              // quantized vectors + scales (MFMA path)
    b += 2 * up256((size_t)max_l * max_rows * 4);                 // encoder input pre-activations, both directions
    b += 8 * up256((size_t)max_n * max_rows * 4);                 // per-hypothesis vectors of a decoder step
    b += up256((size_t)max_n * max_l * 4);                        // attention energies
    const size_t ngrp = (size_t)q8i_out_tiles(max_rows);
    b += up256(ngrp * max_n * 4) + up256(ngrp * max_n * 8);
    return b + 65536;
}

q8_status q8_create(q8_ctx **out, void *hip_stream, void *workspace, size_t workspace_bytes)
{
    if (!out) return Q8_ERR_NULL;
    *out = nullptr;
    if (!workspace) return Q8_ERR_NULL;
    if (((uintptr_t)workspace & 255) != 0) return Q8_ERR_ALIGN;
    if (workspace_bytes < Q8_WS_HEADER) return Q8_ERR_WORKSPACE;
    q8_ctx *c = new (std::nothrow) q8_ctx;
    if (!c) return Q8_ERR_DEVICE;
    c->stream = (hipStream_t)hip_stream;
    c->ws = (char *)workspace;
    c->ws_bytes = workspace_bytes;
    c->err[0] = 0;
    c->prof_ev = nullptr;
    c->prof_cap = c->prof_n = 0;
    c->prof_kind = Q8_KERNEL_VOCAB;
    c->ws_reserved_top = 0;
    c->enc_one_launch = 1;
    c->enc_spin_limit = Q8_ENC_SPIN_DEFAULT;
    c->att_split = 1;
    c->att_spin_limit = Q8_ENC_SPIN_DEFAULT;
    c->att_capacity = -1;
    c->att_words_set = 0;
    c->grup_used[0] = c->grup_used[1] = 0;
    c->gate_pause = Q8_GATE_PAUSE_DEFAULT;
    q8_status st = q8i_fill_u32(c, c->ws, Q8_WS_HEADER / 4, 0u);
    if (st) { delete c; return st; }
    *out = c;
    return Q8_OK;
}

q8_status q8_destroy(q8_ctx *ctx)
{
    if (!ctx) return Q8_ERR_NULL;
    if (ctx->prof_ev) q8_profile_end(ctx, nullptr, nullptr);
    delete ctx;
    return Q8_OK;
}

q8_status q8_profile_begin(q8_ctx *ctx, int kernel_class, int max_samples)
{
    if (!ctx) return Q8_ERR_NULL;
    if (kernel_class < 0 || kernel_class >= Q8_KERNEL_CLASSES) return q8_fail(ctx, Q8_ERR_SHAPE, "unknown kernel class %d", kernel_class);
    if (max_samples <= 0 || max_samples > 65536) return q8_fail(ctx, Q8_ERR_SHAPE, "max_samples outside [1, 65536]");
    if (ctx->prof_ev) q8_profile_end(ctx, nullptr, nullptr);
    ctx->prof_ev = (hipEvent_t *)calloc(2 * (size_t)max_samples, sizeof(hipEvent_t));
    if (!ctx->prof_ev) return q8_fail(ctx, Q8_ERR_DEVICE, "out of host memory");
    for (int i = 0; i < 2 * max_samples; ++i)
        if (hipEventCreate(&ctx->prof_ev[i]) != hipSuccess) {
            for (int t = 0; t < i; ++t) (void)hipEventDestroy(ctx->prof_ev[t]);
            free(ctx->prof_ev);
            ctx->prof_ev = nullptr;
            return q8_fail(ctx, Q8_ERR_DEVICE, "hipEventCreate failed");
        }
    ctx->prof_cap = max_samples;
    ctx->prof_n = 0;
    ctx->prof_kind = kernel_class;
    return Q8_OK;
}

q8_status q8_profile_end(q8_ctx *ctx, float *avg_ms_host, int *samples_host)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!ctx->prof_ev) return q8_fail(ctx, Q8_ERR_SHAPE, "q8_profile_end without q8_profile_begin");
    q8_status st = Q8_OK;
    double sum = 0.0;
    int n = 0;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) st = q8_fail(ctx, Q8_ERR_DEVICE, "stream synchronize failed");
    for (int i = 0; i < ctx->prof_n && st == Q8_OK; ++i) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]) == hipSuccess) {
            sum += ms;
            ++n;
        }
    }
    for (int i = 0; i < 2 * ctx->prof_cap; ++i) (void)hipEventDestroy(ctx->prof_ev[i]);
    free(ctx->prof_ev);
    ctx->prof_ev = nullptr;
    ctx->prof_cap = ctx->prof_n = 0;
    if (avg_ms_host) *avg_ms_host = n ? (float)(sum / n) : 0.0f;
    if (samples_host) *samples_host = n;
    return st;
}

const char *q8_last_error(const q8_ctx *ctx) { return ctx ? ctx->err : "NULL context"; }

q8_status q8_quantize_matrix(q8_ctx *ctx, const float *W, int rows, int cols, int ld_in, int8_t *Wq_out, int ld_out,
                             float *scale_out_host)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!W || !Wq_out || !scale_out_host) return q8_fail(ctx, Q8_ERR_NULL, "q8_quantize_matrix: NULL argument");
    if (rows <= 0 || cols <= 0 || ld_in < cols || ld_out < cols || ld_out > kMaxLd)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_quantize_matrix: bad shape %d x %d (ld_in %d, ld_out %d)", rows, cols, ld_in, ld_out);
    if (!aligned16(Wq_out) || ld_out % 16 != 0)
        return q8_fail(ctx, Q8_ERR_ALIGN, "q8_quantize_matrix: output needs a 16-byte aligned base and ld_out %% 16 == 0");
    return q8i_quantize_matrix(ctx, W, rows, cols, ld_in, Wq_out, ld_out, scale_out_host);
}

q8_status q8_probe_read(q8_ctx *ctx, const void *buf, size_t bytes)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!buf) return q8_fail(ctx, Q8_ERR_NULL, "q8_probe_read: NULL buffer");
    if (!aligned16(buf) || bytes % 16 != 0 || bytes == 0)
        return q8_fail(ctx, Q8_ERR_ALIGN, "q8_probe_read needs a 16-byte aligned buffer and a positive multiple of 16 bytes");
    if (ctx->ws_bytes < Q8_WS_HEADER + 2048 * 4) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_probe_read: workspace too small");
    return q8i_probe_read(ctx, buf, bytes);
}

q8_status q8_math_eval(q8_ctx *ctx, int fn, const void *x, void *y, size_t n)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!x || !y) return q8_fail(ctx, Q8_ERR_NULL, "q8_math_eval: NULL buffer");
    if (fn < 0 || fn > 3 || n == 0 || n > ((size_t)1 << 31)) return q8_fail(ctx, Q8_ERR_SHAPE, "q8_math_eval: fn in 0..3, 1 <= n <= 2^31");
    if (fn == 3 && n % 256) return q8_fail(ctx, Q8_ERR_SHAPE, "q8_math_eval: the sort takes a multiple of 256 values");
    return q8i_math_eval(ctx, fn, x, y, n);
}

size_t q8_tiles_bytes(int rows, int ld)
{
    if (rows <= 0 || ld <= 0) return 0;
    return q8i_tiles_bytes(rows, ld);
}

q8_status q8_pack_tiles(q8_ctx *ctx, const q8_mat *W, int8_t *tiles_out)
{
    if (!ctx) return Q8_ERR_NULL;
    TRY(check_mat(ctx, W, "W"));
    if (!tiles_out) return q8_fail(ctx, Q8_ERR_NULL, "tiles_out: NULL");
    if (W->ld % 64 != 0) return q8_fail(ctx, Q8_ERR_ALIGN, "q8_pack_tiles needs ld %% 64 == 0");
    if (!aligned16(tiles_out)) return q8_fail(ctx, Q8_ERR_ALIGN, "tiles_out needs 16-byte alignment");
    return q8i_pack_tiles(ctx, W, tiles_out);
}

static q8_status gemm_narrow_any(q8_ctx *ctx, const q8_mat *W, const float *row_scale, const float *X, int n, int ldx,
                                 const float *bias, float *Y, int ldy, const q8_taps *taps);

q8_status q8_gemm_narrow(q8_ctx *ctx, const q8_mat *W, const float *X, int n, int ldx, const float *bias, float *Y,
                         int ldy, const q8_taps *taps)
{
    if (!ctx) return Q8_ERR_NULL;
    return gemm_narrow_any(ctx, W, nullptr, X, n, ldx, bias, Y, ldy, taps);
}

q8_status q8_gemm_narrow_rows(q8_ctx *ctx, const q8_mat *W, const float *row_scale, const float *X, int n, int ldx,
                              const float *bias, float *Y, int ldy, const q8_taps *taps)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!row_scale) return q8_fail(ctx, Q8_ERR_NULL, "row_scale: NULL");
    if ((uintptr_t)row_scale % 4 != 0) return q8_fail(ctx, Q8_ERR_ALIGN, "row_scale: not aligned to 4 bytes");
    return gemm_narrow_any(ctx, W, row_scale, X, n, ldx, bias, Y, ldy, taps);
}

q8_status q8_quantize_matrix_rows(q8_ctx *ctx, const float *W, int rows, int cols, int ld_in, int8_t *Wq_out, int ld_out,
                                  float *row_scale_out)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!W || !Wq_out || !row_scale_out) return q8_fail(ctx, Q8_ERR_NULL, "q8_quantize_matrix_rows: NULL argument");
    if (rows <= 0 || cols <= 0 || ld_in < cols || ld_out < cols || ld_out > kMaxLd)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_quantize_matrix_rows: bad shape %d x %d (ld_in %d, ld_out %d)", rows, cols, ld_in, ld_out);
    if (!aligned16(Wq_out) || ld_out % 16 != 0)
        return q8_fail(ctx, Q8_ERR_ALIGN, "q8_quantize_matrix_rows: output needs a 16-byte aligned base and ld_out %% 16 == 0");
    return q8i_quantize_matrix_rows(ctx, W, rows, cols, ld_in, Wq_out, ld_out, row_scale_out);
}

static q8_status gemm_narrow_any(q8_ctx *ctx, const q8_mat *W, const float *row_scale, const float *X, int n, int ldx,
                                 const float *bias, float *Y, int ldy, const q8_taps *taps)
{
    TRY(check_mat(ctx, W, "W"));
    if (n <= 0 || n > kMaxMfmaN) return q8_fail(ctx, Q8_ERR_SHAPE, "n = %d outside [1, %d]", n, kMaxMfmaN);
    TRY(check_vecs(ctx, X, n == 1 ? W->cols + ((4 - W->cols % 4) % 4) : ldx, W->cols, "X"));
    if (!Y) return q8_fail(ctx, Q8_ERR_NULL, "Y: NULL");
    if (n > 1 && ldy < W->rows) return q8_fail(ctx, Q8_ERR_SHAPE, "ldy %d < rows %d", ldy, W->rows);
    if (n <= kMaxNarrow) {
        if ((size_t)n * W->ld > 65536) return q8_fail(ctx, Q8_ERR_SHAPE, "n * ld = %zu exceeds 65536", (size_t)n * W->ld);
        q8i_gemv_desc d = {W, X, ldx, bias, Y, ldy, taps, row_scale};
        return q8i_gemv_jobs(ctx, &d, 1, n);
    }
    Carver cv(ctx);
    int8_t *xq = cv.take<int8_t>((size_t)n * W->ld);
    float *xs = cv.take<float>(n);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_gemm_narrow: workspace too small");
    return q8i_gemm_mfma(ctx, W, X, n, ldx, bias, Y, ldy, taps, xq, xs, row_scale);
}

q8_status q8_attention_states_q8(q8_ctx *ctx, const float *enc_h, int l, int C, int8_t *hT_out, int ld_out,
                                 float *scale_out_host)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!enc_h || !hT_out || !scale_out_host) return q8_fail(ctx, Q8_ERR_NULL, "q8_attention_states_q8: NULL argument");
    if (l <= 0 || l > kMaxL || C <= 0 || ld_out < l || ld_out > kMaxLd)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_attention_states_q8: bad shape l %d, C %d, ld_out %d", l, C, ld_out);
    if (!aligned16(hT_out) || ld_out % 16 != 0)
        return q8_fail(ctx, Q8_ERR_ALIGN, "q8_attention_states_q8: output needs a 16-byte aligned base and ld_out %% 16 == 0");
    Carver cv(ctx);
    float *t = cv.take<float>((size_t)C * l);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_attention_states_q8: workspace too small");
    TRY(q8i_transpose(ctx, enc_h, l, C, t));
    return q8i_quantize_matrix(ctx, t, C, l, l, hT_out, ld_out, scale_out_host);
}

q8_status q8_attention_q8(q8_ctx *ctx, const q8_mat *v, const q8_mat *hT, const float *P, const float *a, int n, int l,
                          float *e_out, float *alpha_out, float *ctx_out)
{
    if (!ctx) return Q8_ERR_NULL;
    TRY(check_mat(ctx, v, "v"));
    TRY(check_mat(ctx, hT, "hT"));
    const int A = v->cols, C = hT->rows;
    if (v->rows != 1) return q8_fail(ctx, Q8_ERR_SHAPE, "v: expected a 1 x A matrix, got %d rows", v->rows);
    if (n <= 0 || n > kMaxNarrow) return q8_fail(ctx, Q8_ERR_SHAPE, "n = %d outside [1, %d]", n, kMaxNarrow);
    if (l <= 0 || l > kMaxL || hT->cols != l) return q8_fail(ctx, Q8_ERR_SHAPE, "l = %d outside [1, %d] or hT has %d columns", l, kMaxL, hT->cols);
    if (A % 4) return q8_fail(ctx, Q8_ERR_ALIGN, "A must be a multiple of 4");
    if (!P || !a || !ctx_out) return q8_fail(ctx, Q8_ERR_NULL, "q8_attention_q8: NULL argument");
    if (!aligned16(P) || !aligned16(a) || !aligned16(ctx_out))
        return q8_fail(ctx, Q8_ERR_ALIGN, "q8_attention_q8: fp32 buffers need 16-byte alignment");
    if ((size_t)n * hT->ld > 65536 || (size_t)kMaxNarrow * v->ld > 65536)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_attention_q8: rows too long for the streaming kernel");
    const int nl = n * l, lda = (l + 3) & ~3, chunk = nl < kMaxMfmaN ? nl : kMaxMfmaN;
    Carver cv(ctx);
    float *T = cv.take<float>((size_t)nl * A);
    float *e = cv.take<float>((size_t)nl);
    float *alpha = cv.take<float>((size_t)n * lda);
    int8_t *xq = cv.take<int8_t>((size_t)chunk * v->ld);
    float *xs = cv.take<float>((size_t)chunk);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_attention_q8: workspace too small");
    TRY(q8i_att_tanh(ctx, P, a, T, l, A, n));
    for (int v0 = 0; v0 < nl; v0 += kMaxMfmaN) {                     // the energies: one product per <= 1024 positions
        const int cnt = nl - v0 < kMaxMfmaN ? nl - v0 : kMaxMfmaN;
        if (cnt <= kMaxNarrow) {
            q8i_gemv_desc d = {v, T + (size_t)v0 * A, A, nullptr, e + v0, 1, nullptr};
            TRY(q8i_gemv_jobs(ctx, &d, 1, cnt));
        } else {
            TRY(q8i_gemm_mfma(ctx, v, T + (size_t)v0 * A, cnt, A, nullptr, e + v0, 1, nullptr, xq, xs));
        }
    }
    TRY(q8i_att_softmax(ctx, e, n, l, lda, alpha, alpha_out, e_out));
    q8i_gemv_desc d = {hT, alpha, lda, nullptr, ctx_out, C, nullptr};
    return q8i_gemv_jobs(ctx, &d, 1, n);
}

q8_status q8_gemv(q8_ctx *ctx, const q8_mat *W, const float *x, const float *bias, float *y, const q8_taps *taps)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!W) return q8_fail(ctx, Q8_ERR_NULL, "W: NULL");
    return q8_gemm_narrow(ctx, W, x, 1, (W->cols + 3) & ~3, bias, y, W->rows, taps);
}

q8_status gru_step_q8(q8_ctx *ctx, const q8_gru_weights *g, const float *x, const float *h_prev, int n, float *h_out,
                      const q8_taps *taps2)
{
    if (!ctx) return Q8_ERR_NULL;
    TRY(check_gru(ctx, g, "gru"));
    if (n <= 0 || n > kMaxMfmaN) return q8_fail(ctx, Q8_ERR_SHAPE, "n = %d outside [1, %d]", n, kMaxMfmaN);
    const int I = g->Wx.cols, H = g->Wh.cols;
    if (n > 1 && (I % 4 || H % 4)) return q8_fail(ctx, Q8_ERR_ALIGN, "batched vectors need dims %% 4 == 0");
    TRY(check_vecs(ctx, x, (I + 3) & ~3, I, "x"));
    TRY(check_vecs(ctx, h_prev, (H + 3) & ~3, H, "h_prev"));
    if (!h_out) return q8_fail(ctx, Q8_ERR_NULL, "h_out: NULL");
    if (h_out == h_prev) return q8_fail(ctx, Q8_ERR_SHAPE, "h_out must not alias h_prev");
    if (n > kMaxNarrow) {
        Carver cv(ctx);
        return gru_panel(ctx, cv, g, x, h_prev, n, nullptr, h_out, taps2);
    }
    if ((size_t)n * (g->Wx.ld + g->Wh.ld) > 65536) return q8_fail(ctx, Q8_ERR_SHAPE, "n * (ld_x + ld_h) exceeds 65536");
    q8i_gru_desc d = {g, x, I, h_prev, H, nullptr, 0, h_out, H, taps2};
    return q8i_gru(ctx, &d, 1, n, Q8I_GRU_FULL);
}

q8_status cgru_decoder_step_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h, int l,
                               const float *y_emb, const float *s_prev, int n_beam, float *s_out, float *ctx_out,
                               float *alpha_out, float *s_mid_out, const q8_taps *taps5)
{
    return cgru_decoder_step_codes_q8(ctx, w, P, enc_h, l, y_emb, s_prev, n_beam, s_out, ctx_out, alpha_out, s_mid_out,
                                      taps5, nullptr, nullptr);
}

q8_status cgru_decoder_step_codes_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h, int l,
                                     const float *y_emb, const float *s_prev, int n_beam, float *s_out, float *ctx_out,
                                     float *alpha_out, float *s_mid_out, const q8_taps *taps5, q8_codes *y_codes,
                                     q8_codes *ctx_codes)
{
    if (y_codes) y_codes->valid = 0;                           // (whatever they held is not taken as an input here)
    return cgru_decoder_step_loop_q8(ctx, w, P, enc_h, l, y_emb, s_prev, n_beam, s_out, ctx_out, alpha_out, s_mid_out, taps5,
                                     y_codes, ctx_codes, nullptr);
}

namespace {
q8_status cgru_after_r(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h, int l, const float *s_mid,
                       int n, float *s_out, float *ctx_out, float *alpha_out, const q8_taps *taps5, q8_codes *ctx_codes,
                       float *a, float *ghq, float *e, int8_t *cq, float *cqs);
}

q8_status cgru_decoder_step_loop_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h, int l,
                                    const float *y_emb, const float *s_prev, int n_beam, float *s_out, float *ctx_out,
                                    float *alpha_out, float *s_mid_out, const q8_taps *taps5, q8_codes *y_codes,
                                    q8_codes *ctx_codes, q8_codes *s_prev_codes)
{
    // codes that the search step left for this call: both inputs of GRU r or neither
    const bool y_in = y_codes && y_codes->valid == 2, s_in = s_prev_codes && s_prev_codes->valid == 2;
    if (y_codes) y_codes->valid = 0;
    if (ctx_codes) ctx_codes->valid = 0;
    if (s_prev_codes) s_prev_codes->valid = 0;
    if (!ctx) return Q8_ERR_NULL;
    if (!w) return q8_fail(ctx, Q8_ERR_NULL, "weights: NULL");
    TRY(check_gru(ctx, &w->r, "r"));
    TRY(check_gru(ctx, &w->q, "q"));
    TRY(check_mat(ctx, &w->att_U, "att_U"));
    const int n = n_beam, H = w->r.Wh.cols, E = w->r.Wx.cols, C = w->q.Wx.cols, A = w->att_U.rows;
    if (n <= 0 || n > kMaxNarrow) return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam = %d outside [1, %d]", n, kMaxNarrow);
    if (l <= 0 || l > kMaxL) return q8_fail(ctx, Q8_ERR_SHAPE, "l = %d outside [1, %d]", l, kMaxL);
    if (w->q.Wh.cols != H || w->att_U.cols != H) return q8_fail(ctx, Q8_ERR_SHAPE, "hidden sizes of r, q and att_U differ");
    if (E % 4 || H % 4 || C % 4 || A % 4) return q8_fail(ctx, Q8_ERR_ALIGN, "E, H, C, A must be multiples of 4");
    if (!w->att_v || !P || !enc_h || !y_emb || !s_prev || !s_out || !ctx_out)
        return q8_fail(ctx, Q8_ERR_NULL, "cgru_decoder_step_q8: NULL argument");
    if (!aligned16(w->att_v) || !aligned16(P) || !aligned16(enc_h) || !aligned16(y_emb) || !aligned16(s_prev) || !aligned16(s_out) || !aligned16(ctx_out))
        return q8_fail(ctx, Q8_ERR_ALIGN, "cgru_decoder_step_q8: fp32 buffers need 16-byte alignment");
    if (s_out == s_prev) return q8_fail(ctx, Q8_ERR_SHAPE, "s_out must not alias s_prev");
    if ((size_t)n * (w->r.Wx.ld + w->r.Wh.ld) > 65536 || (size_t)n * w->q.Wx.ld > 65536)
        return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam * row length exceeds 65536");

    Carver cv(ctx);
    float *s_mid = s_mid_out ? s_mid_out : cv.take<float>((size_t)n * H);
    float *a = cv.take<float>((size_t)n * A);
    float *ghq = cv.take<float>((size_t)n * 3 * H);
    float *e = cv.take<float>((size_t)n * l);
    int8_t *cq = cv.take<int8_t>((size_t)n * w->q.Wx.ld);      // codes and scales of the context vectors,
    float *cqs = cv.take<float>(n);                             // from the attention kernel to GRU q
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "cgru_decoder_step_q8: workspace too small");
    if (codes_usable(ctx_codes, w->q.Wx.ld)) { cq = ctx_codes->q; cqs = ctx_codes->scale; }    // the caller keeps them
    const bool y_out = codes_usable(y_codes, w->r.Wx.ld);
    const bool given = y_in && s_in && y_out && codes_usable(s_prev_codes, w->r.Wh.ld) && !taps5;

    // Eq. 3: s' = r(y, s_prev)
    q8i_gru_desc dr = {&w->r, y_emb, E, s_prev, H, nullptr, 0, s_mid, H, taps5, nullptr, nullptr,
                       y_out ? y_codes->q : nullptr, y_out ? y_codes->scale : nullptr};
    if (given) {
        dr.xq_pre = y_codes->q; dr.xs_pre = y_codes->scale; dr.xq_out = nullptr; dr.xs_out = nullptr;
        dr.hq_pre = s_prev_codes->q; dr.hs_pre = s_prev_codes->scale;
    }
    TRY(q8i_gru(ctx, &dr, 1, n, Q8I_GRU_FULL));
    if (y_out) y_codes->valid = 1;
    return cgru_after_r(ctx, w, P, enc_h, l, s_mid, n, s_out, ctx_out, alpha_out, taps5, ctx_codes, a, ghq, e, cq, cqs);
}

namespace {
// The decoder step from s' on (Eq. 4-6); a, ghq, e, cq, cqs: scratch of the sizes cgru_decoder_step_loop_q8 takes.
q8_status cgru_after_r(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h, int l, const float *s_mid,
                       int n, float *s_out, float *ctx_out, float *alpha_out, const q8_taps *taps5, q8_codes *ctx_codes,
                       float *a, float *ghq, float *e, int8_t *cq, float *cqs)
{
    const int H = w->r.Wh.cols, C = w->q.Wx.cols, A = w->att_U.rows;
    // everything that depends on s' alone: u(s') of Eq. 6 and the recurrent half of GRU q
    q8_mat qWh = w->q.Wh;
    q8i_gemv_desc dj[2] = {{&w->att_U, s_mid, H, nullptr, a, A, taps5 ? taps5 + 2 : nullptr},
                           {&qWh, s_mid, H, w->q.bh, ghq, 3 * H, taps5 ? taps5 + 4 : nullptr}};
    TRY(q8i_gemv_jobs(ctx, dj, 2, n));
    // Eq. 5-6: energies, weights, context
    int have_codes = 0;
    TRY(q8i_attention(ctx, P, enc_h, l, A, C, a, w->att_v, n, e, alpha_out, ctx_out, nullptr, 0, cq, cqs, w->q.Wx.ld, &have_codes));
    // Eq. 4: s = q(H_t, s')
    q8_taps tq[2];
    if (taps5) { tq[0] = taps5[3]; tq[1].xq = nullptr; tq[1].xscale = nullptr; tq[1].acc = nullptr; }
    q8i_gru_desc dq = {&w->q, ctx_out, C, s_mid, H, ghq, 3 * H, s_out, H, taps5 ? tq : nullptr,
                       have_codes ? cq : nullptr, have_codes ? cqs : nullptr};
    if (have_codes && codes_usable(ctx_codes, w->q.Wx.ld)) ctx_codes->valid = 1;
    // (the attention kernel whose blocks exchange words leaves them set: this GRU zeroes them on its way out)
    if (ctx->att_words_set) {
        dq.clear = (unsigned long long *)(ctx->ws + Q8_WS_ATT_XCHG);
        dq.clear_words = n * (Q8_WS_ATT_XCHG_PER_HYP / 8);
    }
    const q8_status st = q8i_gru(ctx, &dq, 1, n, Q8I_GRU_GH_PRE);
    if (!st && dq.clear) ctx->att_words_set = 0;
    return st;
}

}  // namespace

q8_status cgru_decoder_step_ahead_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h, int l,
                                     const float *s_mid, int n_beam, float *s_out, float *ctx_out, float *alpha_out,
                                     q8_codes *ctx_codes)
{
    if (ctx_codes) ctx_codes->valid = 0;
    if (!ctx) return Q8_ERR_NULL;
    if (!w) return q8_fail(ctx, Q8_ERR_NULL, "weights: NULL");
    TRY(check_gru(ctx, &w->r, "r"));
    TRY(check_gru(ctx, &w->q, "q"));
    TRY(check_mat(ctx, &w->att_U, "att_U"));
    const int n = n_beam, H = w->r.Wh.cols, C = w->q.Wx.cols, A = w->att_U.rows;
    if (n <= 0 || n > kMaxNarrow) return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam = %d outside [1, %d]", n, kMaxNarrow);
    if (l <= 0 || l > kMaxL) return q8_fail(ctx, Q8_ERR_SHAPE, "l = %d outside [1, %d]", l, kMaxL);
    if (w->q.Wh.cols != H || w->att_U.cols != H) return q8_fail(ctx, Q8_ERR_SHAPE, "hidden sizes of r, q and att_U differ");
    if (H % 4 || C % 4 || A % 4) return q8_fail(ctx, Q8_ERR_ALIGN, "H, C, A must be multiples of 4");
    if (!w->att_v || !P || !enc_h || !s_mid || !s_out || !ctx_out)
        return q8_fail(ctx, Q8_ERR_NULL, "cgru_decoder_step_ahead_q8: NULL argument");
    if (!aligned16(w->att_v) || !aligned16(P) || !aligned16(enc_h) || !aligned16(s_mid) || !aligned16(s_out) || !aligned16(ctx_out))
        return q8_fail(ctx, Q8_ERR_ALIGN, "cgru_decoder_step_ahead_q8: fp32 buffers need 16-byte alignment");
    if (s_out == s_mid) return q8_fail(ctx, Q8_ERR_SHAPE, "s_out must not alias s_mid");
    if ((size_t)n * w->r.Wh.ld > 65536 || (size_t)n * w->q.Wx.ld > 65536)
        return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam * row length exceeds 65536");
    Carver cv(ctx);
    float *a = cv.take<float>((size_t)n * A);
    float *ghq = cv.take<float>((size_t)n * 3 * H);
    float *e = cv.take<float>((size_t)n * l);
    int8_t *cq = cv.take<int8_t>((size_t)n * w->q.Wx.ld);
    float *cqs = cv.take<float>(n);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "cgru_decoder_step_ahead_q8: workspace too small");
    if (codes_usable(ctx_codes, w->q.Wx.ld)) { cq = ctx_codes->q; cqs = ctx_codes->scale; }
    return cgru_after_r(ctx, w, P, enc_h, l, s_mid, n, s_out, ctx_out, alpha_out, nullptr, ctx_codes, a, ghq, e, cq, cqs);
}

q8_status cgru_decoder_step_batch_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                                     const int32_t *sent_off, int n_sent, int beam, int max_l, const float *y_emb,
                                     const float *s_prev, float *s_out, float *ctx_out, float *alpha_out, float *s_mid_out)
{
    return cgru_decoder_step_batch_codes_q8(ctx, w, P, enc_h, sent_off, n_sent, beam, max_l, y_emb, s_prev, s_out, ctx_out,
                                            alpha_out, s_mid_out, nullptr, nullptr, nullptr);
}

q8_status cgru_decoder_step_batch_codes_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                                           const int32_t *sent_off, int n_sent, int beam, int max_l, const float *y_emb,
                                           const float *s_prev, float *s_out, float *ctx_out, float *alpha_out,
                                           float *s_mid_out, q8_codes *y_codes, q8_codes *ctx_codes, q8_codes *s_codes)
{
    if (y_codes) y_codes->valid = 0;                           // (whatever they held is not taken as an input here)
    return cgru_decoder_step_batch_loop_q8(ctx, w, P, enc_h, sent_off, n_sent, beam, max_l, y_emb, s_prev, s_out, ctx_out,
                                           alpha_out, s_mid_out, y_codes, ctx_codes, s_codes, nullptr);
}

q8_status cgru_decoder_step_batch_loop_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                                          const int32_t *sent_off, int n_sent, int beam, int max_l, const float *y_emb,
                                          const float *s_prev, float *s_out, float *ctx_out, float *alpha_out,
                                          float *s_mid_out, q8_codes *y_codes, q8_codes *ctx_codes, q8_codes *s_codes,
                                          q8_codes *s_prev_codes)
{
    // codes that the search step left for this call: both inputs of GRU r or neither
    const bool y_in = y_codes && y_codes->valid == 2, s_in = s_prev_codes && s_prev_codes->valid == 2;
    if (y_codes) y_codes->valid = 0;
    if (ctx_codes) ctx_codes->valid = 0;
    if (s_codes) s_codes->valid = 0;
    if (s_prev_codes) s_prev_codes->valid = 0;
    if (!ctx) return Q8_ERR_NULL;
    if (!w) return q8_fail(ctx, Q8_ERR_NULL, "weights: NULL");
    TRY(check_gru(ctx, &w->r, "r"));
    TRY(check_gru(ctx, &w->q, "q"));
    TRY(check_mat(ctx, &w->att_U, "att_U"));
    const int H = w->r.Wh.cols, E = w->r.Wx.cols, C = w->q.Wx.cols, A = w->att_U.rows;
    if (n_sent <= 0 || beam <= 0 || beam > Q8_MAX_BEAM || (long long)n_sent * beam > kMaxMfmaN)
        return q8_fail(ctx, Q8_ERR_SHAPE, "need n_sent > 0, 1 <= beam <= %d, n_sent * beam <= %d", Q8_MAX_BEAM, kMaxMfmaN);
    const int n = n_sent * beam;
    if (max_l <= 0 || max_l > kMaxL) return q8_fail(ctx, Q8_ERR_SHAPE, "max_l = %d outside [1, %d]", max_l, kMaxL);
    if (w->q.Wh.cols != H || w->att_U.cols != H) return q8_fail(ctx, Q8_ERR_SHAPE, "hidden sizes of r, q and att_U differ");
    if (E % 4 || H % 4 || C % 4 || A % 4) return q8_fail(ctx, Q8_ERR_ALIGN, "E, H, C, A must be multiples of 4");
    if (!w->att_v || !P || !enc_h || !sent_off || !y_emb || !s_prev || !s_out || !ctx_out)
        return q8_fail(ctx, Q8_ERR_NULL, "cgru_decoder_step_batch_q8: NULL argument");
    if (!aligned16(w->att_v) || !aligned16(P) || !aligned16(enc_h) || !aligned16(y_emb) || !aligned16(s_prev) || !aligned16(s_out) || !aligned16(ctx_out))
        return q8_fail(ctx, Q8_ERR_ALIGN, "cgru_decoder_step_batch_q8: fp32 buffers need 16-byte alignment");
    if (s_out == s_prev) return q8_fail(ctx, Q8_ERR_SHAPE, "s_out must not alias s_prev");

    Carver cv(ctx);
    float *s_mid = s_mid_out ? s_mid_out : cv.take<float>((size_t)n * H);
    float *a = cv.take<float>((size_t)n * A);
    float *ghq = cv.take<float>((size_t)n * 3 * H);
    float *e = cv.take<float>((size_t)n * max_l);
    int8_t *mq_u = cv.take<int8_t>((size_t)n * w->att_U.ld), *mq_h = cv.take<int8_t>((size_t)n * w->q.Wh.ld);
    float *ms_u = cv.take<float>(n), *ms_h = cv.take<float>(n);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "cgru_decoder_step_batch_q8: workspace too small");
    int8_t *cq = cv.take<int8_t>((size_t)n * w->q.Wx.ld);      // codes and scales of the context vectors,
    float *cqs = cv.take<float>(n);                             // from the attention kernel to GRU q
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "cgru_decoder_step_batch_q8: workspace too small");
    if (codes_usable(ctx_codes, w->q.Wx.ld)) { cq = ctx_codes->q; cqs = ctx_codes->scale; }    // the caller keeps them
    const bool y_keep = codes_usable(y_codes, w->r.Wx.ld);
    const bool given = y_in && s_in && y_keep && codes_usable(s_prev_codes, w->r.Wh.ld);
    // Eq. 3: s' = r(y, s_prev); the gates kernel leaves s' quantized for the two products below
    const bool fused_codes = q8i_gru_gates_q_ok(H, H, H, w->att_U.ld, w->q.Wh.ld);
    {
        Carver sub = cv;
        const PanelCodesOut out = {mq_u, w->att_U.ld, ms_u, mq_h, w->q.Wh.ld, ms_h};
        TRY(gru_panel(ctx, sub, &w->r, y_emb, s_prev, n, nullptr, s_mid, nullptr, nullptr, nullptr, fused_codes ? &out : nullptr,
                      y_keep ? y_codes : nullptr, given ? s_prev_codes : nullptr));
        if (y_keep) y_codes->valid = 1;
    }
    // everything that depends on s' alone: u(s') of Eq. 6 and the recurrent half of GRU q
    if (!fused_codes) {
        const q8i_quant_job qj[2] = {{s_mid, H, H, w->att_U.ld, mq_u, ms_u, nullptr}, {s_mid, H, H, w->q.Wh.ld, mq_h, ms_h, nullptr}};
        TRY(q8i_quantize_jobs(ctx, qj, 2, n));
    }
    const q8i_gemm_job gj[2] = {{&w->att_U, mq_u, ms_u, nullptr, a, A, nullptr, nullptr, nullptr, 0},
                                {&w->q.Wh, mq_h, ms_h, w->q.bh, ghq, 3 * H, nullptr, nullptr, nullptr, 0}};
    if (q8i_gemm_ksplit2_ok(gj, 2, n)) TRY(q8i_gemm_ksplit2(ctx, gj, 2, n));
    else TRY(q8i_gemm_jobs(ctx, gj, 2, n));
    // Eq. 5-6 per hypothesis, against the positions of its own sentence
    int have_codes = 0;
    TRY(q8i_attention(ctx, P, enc_h, max_l, A, C, a, w->att_v, n, e, alpha_out, ctx_out, sent_off, beam, cq, cqs, w->q.Wx.ld, &have_codes));
    if (have_codes && codes_usable(ctx_codes, w->q.Wx.ld)) ctx_codes->valid = 1;
    // Eq. 4: s = q(H_t, s'); the gates kernel can leave s quantized for the caller's next product
    Carver sub = cv;
    const bool s_keep = s_codes && s_codes->q && s_codes->scale && aligned16(s_codes->q) && s_codes->ld >= H &&
                        q8i_gru_gates_q_ok(H, H, H, s_codes->ld, s_codes->ld);
    const PanelCodesOut s_out_codes = {s_keep ? s_codes->q : nullptr, s_keep ? s_codes->ld : 0, s_keep ? s_codes->scale : nullptr, nullptr, 0, nullptr};
    q8_status st = gru_panel(ctx, sub, &w->q, ctx_out, s_mid, n, ghq, s_out, nullptr, have_codes ? cq : nullptr,
                             have_codes ? cqs : nullptr, s_keep ? &s_out_codes : nullptr, nullptr, nullptr, 1);
    if (!st && s_keep) s_codes->valid = 1;
    return st;
}

static q8_status output_impl(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                             const float *s, const float *y_emb, const float *ctx_vec, const float *t_in, int n_beam,
                             int k, float *logits, float *lse, float *topk_logp, int32_t *topk_idx, float *t_out,
                             const q8_taps *taps4, q8i_beam_desc *beam, const q8_codes *y_codes = nullptr,
                             const q8_codes *ctx_codes = nullptr, const q8_codes *s_codes = nullptr,
                             const BeamBatchArgs *search = nullptr, int *search_fused = nullptr)
{
    if (search_fused) *search_fused = 0;
    if (!ctx) return Q8_ERR_NULL;
    TRY(check_mat(ctx, W_out, "W_out"));
    const int n = n_beam, R = W_out->cols, V = W_out->rows;
    if (n <= 0 || n > kMaxMfmaN) return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam = %d outside [1, %d]", n, kMaxMfmaN);
    if (n > kMaxNarrow && beam) return q8_fail(ctx, Q8_ERR_SHAPE, "the fused beam update takes at most %d hypotheses", kMaxNarrow);
    if (k <= 0 || k > kMaxK || k > V) return q8_fail(ctx, Q8_ERR_SHAPE, "k = %d outside [1, min(%d, rows)]", k, kMaxK);
    if (V > q8i_out_max_rows()) return q8_fail(ctx, Q8_ERR_SHAPE, "W_out: more than %d rows", q8i_out_max_rows());
    if (W_out->ld > 4096) return q8_fail(ctx, Q8_ERR_SHAPE, "W_out: ld above 4096");
    if (R % 4) return q8_fail(ctx, Q8_ERR_ALIGN, "R must be a multiple of 4");
    if (W_out->tiles && !aligned16(W_out->tiles)) return q8_fail(ctx, Q8_ERR_ALIGN, "W_out.tiles needs 16-byte alignment");
    if (!beam && (!topk_logp || !topk_idx)) return q8_fail(ctx, Q8_ERR_NULL, "top-k outputs: NULL");
    Carver cv(ctx);
    if (!topk_logp) topk_logp = cv.take<float>((size_t)n * k);
    if (!topk_idx) topk_idx = cv.take<int32_t>((size_t)n * k);
    const float *T = t_in;
    if (ro) {
        TRY(check_mat(ctx, &ro->W_s, "W_s"));
        TRY(check_mat(ctx, &ro->W_y, "W_y"));
        TRY(check_mat(ctx, &ro->W_c, "W_c"));
        if (ro->W_s.rows != R || ro->W_y.rows != R || ro->W_c.rows != R)
            return q8_fail(ctx, Q8_ERR_SHAPE, "readout matrices must have %d rows", R);
        if (ro->W_s.cols % 4 || ro->W_y.cols % 4 || ro->W_c.cols % 4)
            return q8_fail(ctx, Q8_ERR_ALIGN, "H, E, C must be multiples of 4");
        if (!s || !y_emb || !ctx_vec) return q8_fail(ctx, Q8_ERR_NULL, "s, y_emb, ctx: NULL");
        if (!aligned16(s) || !aligned16(y_emb) || !aligned16(ctx_vec))
            return q8_fail(ctx, Q8_ERR_ALIGN, "s, y_emb, ctx need 16-byte alignment");
        if (n <= kMaxNarrow && (size_t)n * (ro->W_s.ld + ro->W_y.ld + ro->W_c.ld) > 65536)
            return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam * (H + E + C) exceeds 65536");
    } else {
        TRY(check_vecs(ctx, t_in, R, R, "t_in"));
    }
    const size_t ngrp = (size_t)q8i_out_tiles(V);
    float *pm = cv.take<float>(ngrp * n);
    double *ps = cv.take<double>(ngrp * n);
    // the selection reads the logits back; a panel's logits that stay in the workspace are kept
    // tile by tile (contiguous stores from the matrix cores' result layout)
    const int tiled = (n > kMaxNarrow && !logits) ? 1 : 0;
    // (where the panel kernel runs nothing is kept at all: the selection computes the logits it needs again)
    const bool none_kept = tiled && !(taps4 && taps4[3].acc) && q8i_output_codes_keeps_no_logits(W_out, k);
    float *lg = logits ? logits : (none_kept ? nullptr : cv.take<float>(tiled ? ngrp * 16 * n : (size_t)n * V));
    if (n > kMaxNarrow) {
        // panel path: codes of t from the combine kernel (or from t_in), then the blocked product
        int8_t *tq = cv.take<int8_t>((size_t)n * W_out->ld);
        float *tsc = cv.take<float>(n);
        if (ro) {
            const q8_mat *M[3] = {&ro->W_s, &ro->W_y, &ro->W_c};
            const float *X[3] = {s, y_emb, ctx_vec};
            float *t = t_out ? t_out : cv.take<float>((size_t)n * R);
            q8i_quant_job qj[3];
            q8i_gemm_job gj[3];
            // the three inputs' codes from their producers (all or none), else quantized here
            const q8_codes *pre[3] = {s_codes, y_codes, ctx_codes};
            bool have_pre = !taps4;
            for (int u = 0; u < 3; ++u) have_pre = have_pre && pre[u] && pre[u]->valid && codes_usable(pre[u], M[u]->ld);
            for (int u = 0; u < 3; ++u) {
                int8_t *xq = cv.take<int8_t>((size_t)n * M[u]->ld);
                float *xs = cv.take<float>(n), *part = cv.take<float>((size_t)n * R);
                if (have_pre) { xq = pre[u]->q; xs = pre[u]->scale; }
                qj[u] = {X[u], M[u]->cols, M[u]->cols, M[u]->ld, xq, xs, taps4 ? taps4 + u : nullptr};
                gj[u] = {M[u], xq, xs, nullptr, part, R, taps4 ? taps4[u].acc : nullptr, nullptr, nullptr, 0};
            }
            if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "output_logits_q8: workspace too small");
            if (!have_pre) TRY(q8i_quantize_jobs(ctx, qj, 3, n));
            if (q8i_gemm_ksplit3_ok(gj, n)) TRY(q8i_gemm_ksplit3(ctx, gj, n));
            else TRY(q8i_gemm_jobs(ctx, gj, 3, n));
            TRY(q8i_readout_combine(ctx, gj[0].Y, gj[1].Y, gj[2].Y, ro->b_t, R, n, t, W_out->ld, tq, tsc, taps4 ? taps4 + 3 : nullptr));
        } else {
            if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "output_logits_q8: workspace too small");
            const q8i_quant_job qj = {t_in, R, R, W_out->ld, tq, tsc, taps4 ? taps4 + 3 : nullptr};
            TRY(q8i_quantize_jobs(ctx, &qj, 1, n));
        }
        return q8i_output_codes(ctx, W_out, b_out, tq, tsc, n, k, lg, tiled, lse, topk_logp, topk_idx,
                                taps4 ? taps4[3].acc : nullptr, pm, ps, search, search_fused);
    }
    if (ro) {
        float *t = t_out ? t_out : cv.take<float>((size_t)n * R);
        // the search step hands the codes of the surviving states on: the readout leaves those of s for it
        int8_t *sq = nullptr;
        float *ss = nullptr;
        if (beam && beam->Eq && beam->lds > 0) {
            sq = cv.take<int8_t>((size_t)n * ro->W_s.ld);
            ss = cv.take<float>(n);
        }
        if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "output_logits_q8: workspace too small");
        int exported = 0;
        if (beam && beam->gx_table) {
            // the recurrent half of the next step's GRU r, W_h^r q(s_j) + b_h for every state of this step: in the
            // readout's launch where both run on their fast kernels, else in a launch of its own
            const q8_gru_weights *g = beam->gru_r;
            float *gh = cv.take<float>((size_t)n * g->Wh.rows);
            if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "output_logits_q8: workspace too small");
            q8_mat rWh = g->Wh;
            const q8i_gemv_desc xd = {&rWh, s, g->Wh.cols, g->bh, gh, g->Wh.rows, nullptr};
            int xdone = 0;
            TRY(q8i_readout(ctx, ro, s, y_emb, ctx_vec, n, t, taps4, y_codes, ctx_codes, sq, ss, &exported, &xd, &xdone));
            if (!xdone) TRY(q8i_gemv_jobs(ctx, &xd, 1, n));
            beam->gh_r = gh;
        } else
        TRY(q8i_readout(ctx, ro, s, y_emb, ctx_vec, n, t, taps4, y_codes, ctx_codes, sq, ss, &exported));
        if (beam && beam->Eq && beam->lds > 0) {
            if (exported) { beam->sq_in = sq; beam->ss_in = ss; }
            else beam->Eq = nullptr;                               // (this readout kernel keeps its codes to itself)
        }
        T = t;
    }
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "output_logits_q8: workspace too small");
    return q8i_output(ctx, W_out, b_out, T, R, n, k, lg, lse, topk_logp, topk_idx, taps4 ? taps4 + 3 : nullptr, pm, ps,
                      beam);
}

q8_status output_logits_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                           const float *s, const float *y_emb, const float *ctx_vec, const float *t_in, int n_beam,
                           int k, float *logits, float *lse, float *topk_logp, int32_t *topk_idx, float *t_out,
                           const q8_taps *taps4)
{
    return output_impl(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, t_in, n_beam, k, logits, lse, topk_logp, topk_idx,
                       t_out, taps4, nullptr);
}

q8_status output_logits_codes_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                 const float *s, const float *y_emb, const float *ctx_vec, int n_beam, int k, float *logits,
                                 float *lse, float *topk_logp, int32_t *topk_idx, float *t_out, const q8_codes *s_codes,
                                 const q8_codes *y_codes, const q8_codes *ctx_codes)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!ro) return q8_fail(ctx, Q8_ERR_NULL, "output_logits_codes_q8: the readout weights are required");
    return output_impl(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, nullptr, n_beam, k, logits, lse, topk_logp, topk_idx, t_out,
                       nullptr, nullptr, y_codes, ctx_codes, s_codes);
}

q8_status output_logits_beam_codes_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                      const float *s, float *y_emb, const float *ctx_vec, int n_beam, int k, void *state,
                                      const float *E_tgt, int E, float *s_next, float *topk_logp, int32_t *topk_idx,
                                      const q8_codes *y_codes, const q8_codes *ctx_codes)
{
    q8_codes y = {nullptr, nullptr, 0, 0};
    if (y_codes) y = *y_codes;
    return output_logits_beam_loop_q8(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, n_beam, k, state, E_tgt, E, s_next, topk_logp,
                                      topk_idx, y_codes ? &y : nullptr, ctx_codes, nullptr, nullptr);
}

q8_status output_logits_beam_loop_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                     const float *s, float *y_emb, const float *ctx_vec, int n_beam, int k, void *state,
                                     const float *E_tgt, int E, float *s_next, float *topk_logp, int32_t *topk_idx,
                                     q8_codes *y_codes, const q8_codes *ctx_codes, q8_codes *s_next_codes,
                                     const q8_row_codes *E_codes)
{
    // y_codes as an input: the codes of this step's y_emb for the readout (valid == 1)
    q8_codes y_in = {nullptr, nullptr, 0, 0};
    if (y_codes) { y_in = *y_codes; y_in.valid = y_codes->valid == 1; y_codes->valid = 0; }
    if (s_next_codes) s_next_codes->valid = 0;
    if (!ctx) return Q8_ERR_NULL;
    if (!ro || !state || !E_tgt || !s_next || !s || !y_emb)
        return q8_fail(ctx, Q8_ERR_NULL, "output_logits_beam_q8: NULL argument");
    if (k < n_beam) return q8_fail(ctx, Q8_ERR_SHAPE, "output_logits_beam_q8: need k >= n_beam");
    if (s_next == s) return q8_fail(ctx, Q8_ERR_SHAPE, "s_next must not alias s");
    if (!aligned16(E_tgt) || !aligned16(s_next)) return q8_fail(ctx, Q8_ERR_ALIGN, "fp32 buffers need 16-byte alignment");
    if (E != ro->W_y.cols) return q8_fail(ctx, Q8_ERR_SHAPE, "E does not match the readout's embedding width");
    q8i_beam_desc bd = {state, s, E_tgt, y_emb, s_next, E, ro->W_s.cols};
    // The codes of the rows that the search step gathers travel with them where everything fits: the table of
    // embedding codes at the pitch of the matrices that multiply y (the readout's W_y here, GRU r's Wx in the next
    // step), code buffers of the caller at those pitches, and a gather whose pass of 256 16-byte pieces has room.
    const int H = ro->W_s.cols, ldy = ro->W_y.ld, lds = ro->W_s.ld;
    const bool hand_on = E_codes && E_codes->q && E_codes->scale && E_codes->ld == ldy && aligned16(E_codes->q) &&
                         codes_usable(y_codes, ldy) && codes_usable(s_next_codes, lds) && n_beam <= kMaxNarrow &&
                         E % 4 == 0 && H % 4 == 0 && E / 4 + ldy / 16 + lds / 16 <= 256;
    if (hand_on) {
        bd.Eq = E_codes->q; bd.Es = E_codes->scale; bd.ldy = ldy; bd.lds = lds;
        bd.yq_out = y_codes->q; bd.ys_out = y_codes->scale; bd.sq_out = s_next_codes->q; bd.ss_out = s_next_codes->scale;
    }
    const q8_status st = output_impl(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, nullptr, n_beam, k, nullptr, nullptr, topk_logp,
                                     topk_idx, nullptr, nullptr, &bd, y_codes ? &y_in : nullptr, ctx_codes);
    if (!st && hand_on && bd.Eq) { y_codes->valid = 2; s_next_codes->valid = 2; }
    return st;
}

q8_status output_logits_beam_ahead_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                      const float *s, float *y_emb, const float *ctx_vec, int n_beam, int k, void *state,
                                      const float *E_tgt, int E, float *topk_logp, int32_t *topk_idx, q8_codes *y_codes,
                                      const q8_codes *ctx_codes, const q8_row_codes *E_codes, const q8_gru_weights *r,
                                      const float *gx_table, float *s_mid_next)
{
    // y_codes as an input: the codes of this step's y_emb for the readout (left by this call a step earlier, or by
    // cgru_decoder_step_codes_q8 in the search's first step)
    q8_codes y_in = {nullptr, nullptr, 0, 0};
    if (y_codes) { y_in = *y_codes; y_codes->valid = 0; }
    if (!ctx) return Q8_ERR_NULL;
    if (!ro || !W_out || !state || !E_tgt || !s || !y_emb || !r || !gx_table || !s_mid_next)
        return q8_fail(ctx, Q8_ERR_NULL, "output_logits_beam_ahead_q8: NULL argument");
    TRY(check_gru(ctx, r, "r"));
    if (r->Wh.cols != ro->W_s.cols || r->Wx.cols != E)
        return q8_fail(ctx, Q8_ERR_SHAPE, "output_logits_beam_ahead_q8: GRU r does not match the readout's H and E");
    if (k < n_beam) return q8_fail(ctx, Q8_ERR_SHAPE, "output_logits_beam_ahead_q8: need k >= n_beam");
    if (n_beam > kMaxNarrow) return q8_fail(ctx, Q8_ERR_SHAPE, "output_logits_beam_ahead_q8: at most %d hypotheses", kMaxNarrow);
    if (!aligned16(E_tgt) || !aligned16(gx_table) || !aligned16(s_mid_next))
        return q8_fail(ctx, Q8_ERR_ALIGN, "fp32 buffers need 16-byte alignment");
    if (E != ro->W_y.cols) return q8_fail(ctx, Q8_ERR_SHAPE, "E does not match the readout's embedding width");
    if (W_out->rows >= (1 << 24)) return q8_fail(ctx, Q8_ERR_SHAPE, "output_logits_beam_ahead_q8: vocabulary of 2^24 or more");
    const int H = ro->W_s.cols, ldy = ro->W_y.ld;
    q8i_beam_desc bd = {state, s, E_tgt, y_emb, nullptr, E, H};
    bd.gx_table = gx_table; bd.gru_r = r; bd.s_mid_next = s_mid_next;
    // (the codes of the new embedding rows travel with them where the gather's pass has room; no state rows move)
    const bool hand_on = E_codes && E_codes->q && E_codes->scale && E_codes->ld == ldy && aligned16(E_codes->q) &&
                         codes_usable(y_codes, ldy) && E % 4 == 0 && E / 4 + ldy / 16 <= 256;
    if (hand_on) {
        bd.Eq = E_codes->q; bd.Es = E_codes->scale; bd.ldy = ldy; bd.lds = 0;
        bd.yq_out = y_codes->q; bd.ys_out = y_codes->scale;
    }
    const q8_status st = output_impl(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, nullptr, n_beam, k, nullptr, nullptr, topk_logp,
                                     topk_idx, nullptr, nullptr, &bd, y_codes && y_in.valid ? &y_in : nullptr, ctx_codes);
    if (!st && hand_on && bd.Eq) y_codes->valid = 2;
    return st;
}

q8_status output_logits_beam_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                const float *s, float *y_emb, const float *ctx_vec, int n_beam, int k, void *state,
                                const float *E_tgt, int E, float *s_next, float *topk_logp, int32_t *topk_idx)
{
    return output_logits_beam_codes_q8(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, n_beam, k, state, E_tgt, E, s_next,
                                       topk_logp, topk_idx, nullptr, nullptr);
}

q8_status q8_encode(q8_ctx *ctx, const q8_gru_weights *fwd, const q8_gru_weights *bwd, const float *X, int l,
                    float *enc_h)
{
    if (!ctx) return Q8_ERR_NULL;
    TRY(check_gru(ctx, fwd, "fwd"));
    TRY(check_gru(ctx, bwd, "bwd"));
    const int E = fwd->Wx.cols, H = fwd->Wh.cols, C = 2 * H;
    if (bwd->Wx.cols != E || bwd->Wh.cols != H) return q8_fail(ctx, Q8_ERR_SHAPE, "directions differ in shape");
    if (l <= 0 || l > kMaxL) return q8_fail(ctx, Q8_ERR_SHAPE, "l = %d outside [1, %d]", l, kMaxL);
    if (E % 4 || H % 4) return q8_fail(ctx, Q8_ERR_ALIGN, "E and H must be multiples of 4");
    TRY(check_vecs(ctx, X, E, E, "X"));
    if (!enc_h) return q8_fail(ctx, Q8_ERR_NULL, "enc_h: NULL");
    if (!aligned16(enc_h)) return q8_fail(ctx, Q8_ERR_ALIGN, "enc_h needs 16-byte alignment");

    Carver cv(ctx);
    int8_t *xq = cv.take<int8_t>((size_t)l * fwd->Wx.ld);
    float *xs = cv.take<float>(l);
    float *gxf = cv.take<float>((size_t)l * 3 * H);
    float *gxb = cv.take<float>((size_t)l * 3 * H);
    float *zero = cv.take<float>(H);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_encode: workspace too small");
    TRY(q8i_fill_u32(ctx, zero, H, 0u));

    // input products for every position at once (the same per-vector quantization as l separate products)
    if (l <= kMaxNarrow) {
        q8i_gemv_desc d[2] = {{&fwd->Wx, X, E, fwd->bx, gxf, 3 * H, nullptr}, {&bwd->Wx, X, E, bwd->bx, gxb, 3 * H, nullptr}};
        TRY(q8i_gemv_jobs(ctx, d, 2, l));
    } else {
        if (fwd->Wx.ld != bwd->Wx.ld) return q8_fail(ctx, Q8_ERR_SHAPE, "q8_encode: the two Wx need the same ld");
        const q8i_quant_job qj = {X, E, E, fwd->Wx.ld, xq, xs, nullptr};            // one quantization serves both
        TRY(q8i_quantize_jobs(ctx, &qj, 1, l));
        const q8i_gemm_job gj[2] = {{&fwd->Wx, xq, xs, fwd->bx, gxf, 3 * H, nullptr, nullptr, nullptr, 0},
                                    {&bwd->Wx, xq, xs, bwd->bx, gxb, 3 * H, nullptr, nullptr, nullptr, 0}};
        TRY(q8i_gemm_jobs(ctx, gj, 2, l));
    }
    // the recurrence: one launch for all positions where the device can hold its blocks at once ...
    if (ctx->enc_one_launch) {
        unsigned long long *xchg = cv.take<unsigned long long>((size_t)4 * H);
        if (cv.ok) {
            int launched = 0;
            TRY(q8i_encode_persistent(ctx, fwd, bwd, gxf, gxb, l, enc_h, xchg, (unsigned *)(ctx->ws + Q8_WS_ENC_ERR),
                                      ctx->enc_spin_limit, &launched));
            if (launched) return Q8_OK;
        }
    }
    // ... else l sequential launches, both directions in each
    for (int t = 0; t < l; ++t) {
        const int pf = t, pb = l - 1 - t;
        q8i_gru_desc d[2];
        d[0] = {fwd, nullptr, 0, t == 0 ? zero : enc_h + (size_t)(pf - 1) * C + H, H, gxf + (size_t)pf * 3 * H, 3 * H,
                enc_h + (size_t)pf * C + H, H, nullptr};
        d[1] = {bwd, nullptr, 0, t == 0 ? zero : enc_h + (size_t)(pb + 1) * C, H, gxb + (size_t)pb * 3 * H, 3 * H,
                enc_h + (size_t)pb * C, H, nullptr};
        TRY(q8i_gru(ctx, d, 2, 1, Q8I_GRU_GX_PRE));
    }
    return Q8_OK;
}

q8_status q8_encoder_options(q8_ctx *ctx, int one_launch, int spin_limit)
{
    if (!ctx) return Q8_ERR_NULL;
    ctx->enc_one_launch = one_launch ? 1 : 0;
    ctx->enc_spin_limit = spin_limit > 0 ? spin_limit : Q8_ENC_SPIN_DEFAULT;
    return Q8_OK;
}

q8_status q8_encode_check(q8_ctx *ctx)
{
    if (!ctx) return Q8_ERR_NULL;
    static_assert(Q8_WS_ATT_ERR == Q8_WS_ENC_ERR + 4, "the two flags are read together");
    unsigned flag[2] = {0, 0};
    hipError_t e = hipMemcpyAsync(flag, ctx->ws + Q8_WS_ENC_ERR, sizeof(flag), hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return q8_fail(ctx, Q8_ERR_DEVICE, "q8_encode_check: %s", hipGetErrorString(e));
    if (flag[0] || flag[1]) {
        q8i_fill_u32(ctx, ctx->ws + Q8_WS_ENC_ERR, 2, 0u);
        // (blocks that were not waited for may have left exchange words set after their reader cleared them)
        q8i_fill_u32(ctx, ctx->ws + Q8_WS_ATT_XCHG, (Q8_WS_HEADER - Q8_WS_ATT_XCHG) / 4, 0u);
        ctx->att_words_set = 0;
        ctx->grup_used[0] = ctx->grup_used[1] = 0;
        if (flag[0])
            return q8_fail(ctx, Q8_ERR_DEVICE, "q8_encode: a wait inside the one-launch recurrence gave up; enc_h is not valid");
        return q8_fail(ctx, Q8_ERR_DEVICE, "decoder step: a wait between the blocks of the attention, the selection or the panel GRU kernel gave up; "
                                           "the results since the last check are not valid");
    }
    return Q8_OK;
}

q8_status q8_attention_options(q8_ctx *ctx, int exchange, int spin_limit)
{
    if (!ctx) return Q8_ERR_NULL;
    ctx->att_split = exchange ? 1 : 0;
    ctx->att_spin_limit = spin_limit > 0 ? spin_limit : Q8_ENC_SPIN_DEFAULT;
    return Q8_OK;
}

size_t q8_encode_batch_bytes(const q8_gru_weights *fwd, int total_l, int n_sent)
{
    if (!fwd || total_l < 1 || n_sent < 1) return 0;
    const size_t H = fwd->Wh.cols, panel = total_l < kMaxMfmaN ? total_l : kMaxMfmaN;
    return 2 * up256((size_t)total_l * 3 * H * 4) + up256(panel * fwd->Wx.ld) + up256(panel * 4) +
           2 * (up256((size_t)n_sent * fwd->Wh.ld) + up256((size_t)n_sent * 4) + up256((size_t)n_sent * 3 * H * 4)) + 4096;
}

q8_status q8_encode_batch(q8_ctx *ctx, const q8_gru_weights *fwd, const q8_gru_weights *bwd, const float *X,
                          const int32_t *sent_off, const int32_t *sent_off_host, int n_sent, float *enc_h)
{
    if (!ctx) return Q8_ERR_NULL;
    TRY(check_gru(ctx, fwd, "fwd"));
    TRY(check_gru(ctx, bwd, "bwd"));
    const int E = fwd->Wx.cols, H = fwd->Wh.cols;
    if (bwd->Wx.cols != E || bwd->Wh.cols != H || fwd->Wx.ld != bwd->Wx.ld || fwd->Wh.ld != bwd->Wh.ld)
        return q8_fail(ctx, Q8_ERR_SHAPE, "directions differ in shape");
    if (E % 4 || H % 4) return q8_fail(ctx, Q8_ERR_ALIGN, "E and H must be multiples of 4");
    if (!sent_off || !sent_off_host || !enc_h) return q8_fail(ctx, Q8_ERR_NULL, "q8_encode_batch: NULL argument");
    if (n_sent <= 0 || n_sent > kMaxMfmaN) return q8_fail(ctx, Q8_ERR_SHAPE, "n_sent = %d outside [1, %d]", n_sent, kMaxMfmaN);
    if (sent_off_host[0] != 0) return q8_fail(ctx, Q8_ERR_SHAPE, "sent_off[0] must be 0");
    int max_l = 0;
    for (int s = 0; s < n_sent; ++s) {
        const int l = sent_off_host[s + 1] - sent_off_host[s];
        if (l <= 0 || l > kMaxL) return q8_fail(ctx, Q8_ERR_SHAPE, "sentence %d: length %d outside [1, %d]", s, l, kMaxL);
        if (l > max_l) max_l = l;
    }
    const int total_l = sent_off_host[n_sent];
    TRY(check_vecs(ctx, X, E, E, "X"));
    if (!aligned16(enc_h)) return q8_fail(ctx, Q8_ERR_ALIGN, "enc_h needs 16-byte alignment");

    Carver cv(ctx);
    const int panel = total_l < kMaxMfmaN ? total_l : kMaxMfmaN;
    float *gxf = cv.take<float>((size_t)total_l * 3 * H), *gxb = cv.take<float>((size_t)total_l * 3 * H);
    int8_t *xq = cv.take<int8_t>((size_t)panel * fwd->Wx.ld);
    float *xs = cv.take<float>(panel);
    int8_t *hqf = cv.take<int8_t>((size_t)n_sent * fwd->Wh.ld), *hqb = cv.take<int8_t>((size_t)n_sent * fwd->Wh.ld);
    float *hsf = cv.take<float>(n_sent), *hsb = cv.take<float>(n_sent);
    float *ghf = cv.take<float>((size_t)n_sent * 3 * H), *ghb = cv.take<float>((size_t)n_sent * 3 * H);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_encode_batch: workspace too small");
    // input products of every position of every sentence, both directions per launch
    for (int o = 0; o < total_l; o += kMaxMfmaN) {
        const int cnt = total_l - o < kMaxMfmaN ? total_l - o : kMaxMfmaN;
        const q8i_quant_job qj = {X + (size_t)o * E, E, E, fwd->Wx.ld, xq, xs, nullptr};
        TRY(q8i_quantize_jobs(ctx, &qj, 1, cnt));
        const q8i_gemm_job gj[2] = {{&fwd->Wx, xq, xs, fwd->bx, gxf + (size_t)o * 3 * H, 3 * H, nullptr, nullptr, nullptr, 0},
                                    {&bwd->Wx, xq, xs, bwd->bx, gxb + (size_t)o * 3 * H, 3 * H, nullptr, nullptr, nullptr, 0}};
        TRY(q8i_gemm_jobs(ctx, gj, 2, cnt));
    }
    // the recurrences, all sentences and both directions per time step
    for (int t = 0; t < max_l; ++t) {
        TRY(q8i_enc_step(ctx, 0, sent_off, n_sent, t, H, fwd->Wh.ld, enc_h, gxf, gxb, ghf, ghb, hqf, hqb, hsf, hsb));
        const q8i_gemm_job gj[2] = {{&fwd->Wh, hqf, hsf, fwd->bh, ghf, 3 * H, nullptr, nullptr, nullptr, 0},
                                    {&bwd->Wh, hqb, hsb, bwd->bh, ghb, 3 * H, nullptr, nullptr, nullptr, 0}};
        TRY(q8i_gemm_jobs(ctx, gj, 2, n_sent));
        TRY(q8i_enc_step(ctx, 1, sent_off, n_sent, t, H, fwd->Wh.ld, enc_h, gxf, gxb, ghf, ghb, hqf, hqb, hsf, hsb));
    }
    return Q8_OK;
}

size_t q8_beam_state_bytes(int max_steps) { return q8i_beam_state_bytes(max_steps < 1 ? 1 : max_steps); }

q8_status q8_beam_init(q8_ctx *ctx, void *state, int beam, int max_steps, const float *s0, const float *E_tgt, int E,
                       int H, float *y_emb, float *s)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!state || !s0 || !E_tgt || !y_emb || !s) return q8_fail(ctx, Q8_ERR_NULL, "q8_beam_init: NULL argument");
    if (beam <= 0 || beam > Q8_MAX_BEAM || max_steps <= 0 || E <= 0 || H <= 0)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_beam_init: beam %d (max %d), max_steps %d", beam, Q8_MAX_BEAM, max_steps);
    return q8i_beam_init(ctx, state, beam, max_steps, s0, E_tgt, E, H, y_emb, s);
}

q8_status q8_beam_update(q8_ctx *ctx, void *state, const float *topk_logp, const int32_t *topk_idx, int n_beam, int k,
                         const float *s_step, int H, const float *E_tgt, int E, float *y_emb, float *s_next)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!state || !topk_logp || !topk_idx || !s_step || !E_tgt || !y_emb || !s_next)
        return q8_fail(ctx, Q8_ERR_NULL, "q8_beam_update: NULL argument");
    if (n_beam <= 0 || n_beam > Q8_MAX_BEAM || k < n_beam || k > kMaxK || E <= 0 || H <= 0)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_beam_update: need 1 <= n_beam <= %d and n_beam <= k <= %d", Q8_MAX_BEAM, kMaxK);
    if (s_next == s_step) return q8_fail(ctx, Q8_ERR_SHAPE, "s_next must not alias s_step");
    if (!aligned16(s_step) || !aligned16(s_next) || !aligned16(E_tgt) || !aligned16(y_emb))
        return q8_fail(ctx, Q8_ERR_ALIGN, "q8_beam_update: fp32 buffers need 16-byte alignment");
    return q8i_beam_update(ctx, state, topk_logp, topk_idx, n_beam, k, s_step, H, E_tgt, E, y_emb, s_next);
}

q8_status q8_beam_result(q8_ctx *ctx, const void *state, int max_steps, int32_t *tokens_host, int *len_host,
                         float *score_host, int *steps_host, int *done_host)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!state) return q8_fail(ctx, Q8_ERR_NULL, "q8_beam_result: NULL state");
    if (max_steps <= 0) return q8_fail(ctx, Q8_ERR_SHAPE, "max_steps must be positive");
    return q8i_beam_read(ctx, state, max_steps, tokens_host, len_host, score_host, steps_host, done_host);
}

namespace {
struct TranslateBufs {
    size_t X, enc_h, P, y, s0, s1, cv, lp, idx, tok, state, yq, ys, cq, cs, sq, ss, sm0, sm1, total;
};
TranslateBufs translate_layout(const q8_model *m, int l, int beam, int k, int max_steps)
{
    const size_t E = m->E, H = m->dec.r.Wh.cols, C = m->dec.q.Wx.cols, A = m->dec.att_U.rows;
    TranslateBufs b;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += up256(bytes); return at; };
    b.X = take((size_t)l * E * 4); b.enc_h = take((size_t)l * C * 4); b.P = take((size_t)l * A * 4);
    b.y = take((size_t)beam * E * 4); b.s0 = take((size_t)beam * H * 4); b.s1 = take((size_t)beam * H * 4);
    b.cv = take((size_t)beam * C * 4); b.lp = take((size_t)beam * k * 4); b.idx = take((size_t)beam * k * 4);
    b.tok = take((size_t)l * 4);
    b.state = take(q8i_beam_state_bytes(max_steps));
    // codes of y and of the context vectors, handed from the decoder step to the output layer
    b.yq = take((size_t)beam * m->dec.r.Wx.ld); b.ys = take((size_t)beam * 4);
    b.cq = take((size_t)beam * m->dec.q.Wx.ld); b.cs = take((size_t)beam * 4);
    // codes of the surviving states, handed from the search step to the next decoder step
    b.sq = take((size_t)beam * m->dec.r.Wh.ld); b.ss = take((size_t)beam * 4);
    // s' of this step and of the next (the loop with GRU r ahead)
    b.sm0 = take((size_t)beam * H * 4); b.sm1 = take((size_t)beam * H * 4);
    b.total = o;
    return b;
}
}  // namespace

size_t q8_translate_bytes(const q8_model *m, int max_l, int beam, int k, int max_steps)
{
    if (!m || max_l < 1 || beam < 1 || k < 1 || max_steps < 1) return 0;
    return translate_layout(m, max_l, beam, k, max_steps).total;
}

q8_status q8_translate(q8_ctx *ctx, const q8_model *m, const int32_t *src_tokens, int l, int beam, int k,
                       int max_steps, int32_t *tokens_host, int *len_host, float *score_host, int *steps_host)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!m || !src_tokens || !m->E_src || !m->E_tgt) return q8_fail(ctx, Q8_ERR_NULL, "q8_translate: NULL argument");
    TRY(check_gru(ctx, &m->enc_fwd, "enc_fwd"));
    TRY(check_gru(ctx, &m->dec.r, "dec.r"));
    TRY(check_gru(ctx, &m->dec.q, "dec.q"));
    TRY(check_mat(ctx, &m->att_W, "att_W"));
    TRY(check_mat(ctx, &m->dec.att_U, "att_U"));
    const int E = m->E, H = m->dec.r.Wh.cols, C = m->dec.q.Wx.cols, A = m->dec.att_U.rows;
    if (l <= 0 || l > kMaxL) return q8_fail(ctx, Q8_ERR_SHAPE, "l = %d outside [1, %d]", l, kMaxL);
    if (beam <= 0 || beam > Q8_MAX_BEAM || k < beam || k > kMaxK || max_steps <= 0)
        return q8_fail(ctx, Q8_ERR_SHAPE, "need 1 <= beam <= %d, beam <= k <= %d, max_steps > 0", Q8_MAX_BEAM, kMaxK);
    if (m->V_src <= 0 || m->V_tgt != m->W_out.rows)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_translate: need V_src > 0 and V_tgt = rows of W_out");
    if (m->enc_fwd.Wx.cols != E || m->dec.r.Wx.cols != E || 2 * m->enc_fwd.Wh.cols != C || m->att_W.cols != C ||
        m->att_W.rows != A || m->enc_fwd.Wh.cols != H)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_translate: model dimensions are inconsistent");
    if (ctx->ws_reserved_top) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_translate is not re-entrant");
    const TranslateBufs b = translate_layout(m, l, beam, k, max_steps);
    if (b.total + Q8_WS_HEADER > ctx->ws_bytes) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_translate: workspace too small");
    char *top = ctx->ws + ((ctx->ws_bytes - b.total) & ~(size_t)255);
    float *X = (float *)(top + b.X), *enc_h = (float *)(top + b.enc_h), *P = (float *)(top + b.P);
    float *y = (float *)(top + b.y), *s[2] = {(float *)(top + b.s0), (float *)(top + b.s1)};
    float *cv = (float *)(top + b.cv), *lp = (float *)(top + b.lp);
    int32_t *idx = (int32_t *)(top + b.idx);
    void *state = top + b.state;
    q8_codes yc = {(int8_t *)(top + b.yq), (float *)(top + b.ys), m->dec.r.Wx.ld, 0};
    q8_codes cc = {(int8_t *)(top + b.cq), (float *)(top + b.cs), m->dec.q.Wx.ld, 0};
    q8_codes sc = {(int8_t *)(top + b.sq), (float *)(top + b.ss), m->dec.r.Wh.ld, 0};
    const q8_row_codes *Ec = m->E_tgt_codes.q ? &m->E_tgt_codes : nullptr;
    ctx->ws_reserved_top = ctx->ws_bytes - (size_t)(top - ctx->ws);

    q8_status st = q8i_gather_rows(ctx, m->E_src, src_tokens, l, E, m->V_src, X);                        // x_i of Eq. 1
    if (!st) st = q8_encode(ctx, &m->enc_fwd, &m->enc_bwd, X, l, enc_h);                       // Eq. 1
    if (!st) st = q8_gemm_narrow(ctx, &m->att_W, enc_h, l, C, m->att_b, P, A, nullptr);        // w(h_i) of Eq. 6
    // initial decoder state: the backward encoder state at the first source position
    if (!st) st = q8i_beam_init(ctx, state, beam, max_steps, enc_h, m->E_tgt, E, H, y, s[0]);
    int cur = 0, done = 0;
    // With the table of GRU r's input products the loop keeps GRU r off the chain of dependent launches: s' of a step
    // is made by the step before it (the first by a plain GRU call), the states stay where GRU q wrote them.
    float *sm[2] = {(float *)(top + b.sm0), (float *)(top + b.sm1)};
    const bool ahead = m->gx_r != nullptr && aligned16(m->gx_r) && m->V_tgt < (1 << 24);
    if (ahead && !st) st = gru_step_q8(ctx, &m->dec.r, y, s[0], beam, sm[0], nullptr);                  // Eq. 3, first step
    for (int t = 0; ahead && t < max_steps && !st && !done; ++t) {
        st = cgru_decoder_step_ahead_q8(ctx, &m->dec, P, enc_h, l, sm[t & 1], beam, s[1], cv, nullptr, &cc);
        if (!st) st = output_logits_beam_ahead_q8(ctx, &m->ro, &m->W_out, m->b_out, s[1], y, cv, beam, k, state, m->E_tgt, E, lp,
                                                  idx, &yc, &cc, Ec, &m->dec.r, m->gx_r, sm[(t + 1) & 1]);
        if (!st && (t % 8 == 7))
            st = q8i_beam_read(ctx, state, max_steps, nullptr, nullptr, nullptr, nullptr, &done);
    }
    for (int t = 0; !ahead && t < max_steps && !st && !done; ++t) {
        st = cgru_decoder_step_loop_q8(ctx, &m->dec, P, enc_h, l, y, s[cur], beam, s[cur ^ 1], cv, nullptr, nullptr, nullptr,
                                       &yc, &cc, &sc);
        // output layer, top-k and (in block 0 of the selection kernel) the beam update, which gathers the
        // surviving states from s[cur ^ 1] into s[cur] and the new embeddings into y, with their codes
        // where the model brings its embeddings' codes
        if (!st) st = output_logits_beam_loop_q8(ctx, &m->ro, &m->W_out, m->b_out, s[cur ^ 1], y, cv, beam, k, state,
                                                 m->E_tgt, E, s[cur], lp, idx, &yc, &cc, &sc, Ec);
        if (!st && (t % 8 == 7))
            st = q8i_beam_read(ctx, state, max_steps, nullptr, nullptr, nullptr, nullptr, &done);
    }
    if (!st) st = q8i_beam_read(ctx, state, max_steps, tokens_host, len_host, score_host, steps_host, nullptr);
    if (!st) st = q8_encode_check(ctx);                       // (the stream is idle here: one word read back)
    ctx->ws_reserved_top = 0;
    return st;
}

// -------------------------------------------------------------------- the 32-bit engine ----

namespace {
q8_status check_matf(q8_ctx *ctx, const q8_matf *W, const char *name)
{
    if (!W || !W->data) return q8_fail(ctx, Q8_ERR_NULL, "%s: NULL matrix", name);
    if (W->rows <= 0 || W->cols <= 0 || W->ld < W->cols || W->cols > kMaxLd)
        return q8_fail(ctx, Q8_ERR_SHAPE, "%s: bad shape %d x %d (ld %d)", name, W->rows, W->cols, W->ld);
    if (!aligned16(W->data) || W->ld % 4 != 0)
        return q8_fail(ctx, Q8_ERR_ALIGN, "%s: needs a 16-byte aligned base and ld %% 4 == 0", name);
    return Q8_OK;
}
q8_status check_gruf(q8_ctx *ctx, const q8_gru_weights_f32 *g, const char *name)
{
    TRY(check_matf(ctx, &g->Wx, name));
    TRY(check_matf(ctx, &g->Wh, name));
    if (g->Wx.rows != g->Wh.rows || g->Wh.rows != 3 * g->Wh.cols)
        return q8_fail(ctx, Q8_ERR_SHAPE, "%s: expected Wx [3H x I], Wh [3H x H]", name);
    return Q8_OK;
}
// the vectors of one launch sit in LDS as floats
bool f32_fits(int n, int cols) { return (size_t)n * ((cols + 3) & ~3) * 4 <= 65536; }
}  // namespace

q8_status q8_gemv_f32(q8_ctx *ctx, const q8_matf *W, const float *X, int n, int ldx, const float *bias, float *Y, int ldy)
{
    if (!ctx) return Q8_ERR_NULL;
    TRY(check_matf(ctx, W, "W"));
    if (n <= 0 || n > kMaxNarrow) return q8_fail(ctx, Q8_ERR_SHAPE, "n = %d outside [1, %d]", n, kMaxNarrow);
    if (!X || !Y) return q8_fail(ctx, Q8_ERR_NULL, "q8_gemv_f32: NULL argument");
    if (n > 1 && (ldx < W->cols || ldy < W->rows)) return q8_fail(ctx, Q8_ERR_SHAPE, "q8_gemv_f32: leading dimensions too small");
    if (!f32_fits(n, W->cols)) return q8_fail(ctx, Q8_ERR_SHAPE, "n * cols exceeds 16384");
    const q8i_f32_job j = {W, X, ldx, bias, Y, ldy};
    return q8i_gemv_f32(ctx, &j, 1, n);
}

q8_status cgru_decoder_step_f32(q8_ctx *ctx, const q8_cgru_weights_f32 *w, const float *P, const float *enc_h, int l,
                                const float *y_emb, const float *s_prev, int n_beam, float *s_out, float *ctx_out,
                                float *alpha_out, float *s_mid_out)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!w) return q8_fail(ctx, Q8_ERR_NULL, "weights: NULL");
    TRY(check_gruf(ctx, &w->r, "r"));
    TRY(check_gruf(ctx, &w->q, "q"));
    TRY(check_matf(ctx, &w->att_U, "att_U"));
    const int n = n_beam, H = w->r.Wh.cols, E = w->r.Wx.cols, C = w->q.Wx.cols, A = w->att_U.rows;
    if (n <= 0 || n > kMaxNarrow) return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam = %d outside [1, %d]", n, kMaxNarrow);
    if (l <= 0 || l > kMaxL) return q8_fail(ctx, Q8_ERR_SHAPE, "l = %d outside [1, %d]", l, kMaxL);
    if (w->q.Wh.cols != H || w->att_U.cols != H) return q8_fail(ctx, Q8_ERR_SHAPE, "hidden sizes of r, q and att_U differ");
    if (E % 4 || H % 4 || C % 4 || A % 4) return q8_fail(ctx, Q8_ERR_ALIGN, "E, H, C, A must be multiples of 4");
    if (!w->att_v || !P || !enc_h || !y_emb || !s_prev || !s_out || !ctx_out)
        return q8_fail(ctx, Q8_ERR_NULL, "cgru_decoder_step_f32: NULL argument");
    if (!aligned16(w->att_v) || !aligned16(P) || !aligned16(enc_h) || !aligned16(ctx_out))
        return q8_fail(ctx, Q8_ERR_ALIGN, "cgru_decoder_step_f32: fp32 buffers need 16-byte alignment");
    if (s_out == s_prev) return q8_fail(ctx, Q8_ERR_SHAPE, "s_out must not alias s_prev");
    if (!f32_fits(n, C) || !f32_fits(n, H) || !f32_fits(n, E)) return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam * dimension exceeds 16384");

    Carver cv(ctx);
    float *s_mid = s_mid_out ? s_mid_out : cv.take<float>((size_t)n * H);
    float *a = cv.take<float>((size_t)n * A);
    float *gx = cv.take<float>((size_t)n * 3 * H), *gh = cv.take<float>((size_t)n * 3 * H);
    float *e = cv.take<float>((size_t)n * l);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "cgru_decoder_step_f32: workspace too small");
    // Eq. 3: s' = r(y, s_prev)
    const q8i_f32_job j1[2] = {{&w->r.Wx, y_emb, E, w->r.bx, gx, 3 * H}, {&w->r.Wh, s_prev, H, w->r.bh, gh, 3 * H}};
    TRY(q8i_gemv_f32(ctx, j1, 2, n));
    TRY(q8i_gru_gates(ctx, gx, gh, s_prev, H, s_mid, H, H, n));
    // u(s') of Eq. 6 and the recurrent half of GRU q
    const q8i_f32_job j2[2] = {{&w->att_U, s_mid, H, nullptr, a, A}, {&w->q.Wh, s_mid, H, w->q.bh, gh, 3 * H}};
    TRY(q8i_gemv_f32(ctx, j2, 2, n));
    // Eq. 5-6
    TRY(q8i_attention(ctx, P, enc_h, l, A, C, a, w->att_v, n, e, alpha_out, ctx_out, nullptr, 0, nullptr, nullptr, 0, nullptr));
    // Eq. 4: s = q(H_t, s')
    const q8i_f32_job j3 = {&w->q.Wx, ctx_out, C, w->q.bx, gx, 3 * H};
    TRY(q8i_gemv_f32(ctx, &j3, 1, n));
    return q8i_gru_gates(ctx, gx, gh, s_mid, H, s_out, H, H, n);
}

q8_status output_logits_f32(q8_ctx *ctx, const q8_readout_weights_f32 *ro, const q8_matf *W_out, const float *b_out,
                            const float *s, const float *y_emb, const float *ctx_vec, int n_beam, int k, float *logits,
                            float *lse, float *topk_logp, int32_t *topk_idx, float *t_out)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!ro) return q8_fail(ctx, Q8_ERR_NULL, "readout weights: NULL");
    TRY(check_matf(ctx, W_out, "W_out"));
    TRY(check_matf(ctx, &ro->W_s, "W_s"));
    TRY(check_matf(ctx, &ro->W_y, "W_y"));
    TRY(check_matf(ctx, &ro->W_c, "W_c"));
    const int n = n_beam, R = W_out->cols, V = W_out->rows;
    if (n <= 0 || n > kMaxNarrow) return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam = %d outside [1, %d]", n, kMaxNarrow);
    if (k <= 0 || k > kMaxK || k > V) return q8_fail(ctx, Q8_ERR_SHAPE, "k = %d outside [1, min(%d, rows)]", k, kMaxK);
    if (V > q8i_out_max_rows()) return q8_fail(ctx, Q8_ERR_SHAPE, "W_out: more than %d rows", q8i_out_max_rows());
    if (ro->W_s.rows != R || ro->W_y.rows != R || ro->W_c.rows != R)
        return q8_fail(ctx, Q8_ERR_SHAPE, "readout matrices must have %d rows", R);
    if (R % 4) return q8_fail(ctx, Q8_ERR_ALIGN, "R must be a multiple of 4");
    if (!s || !y_emb || !ctx_vec || !topk_logp || !topk_idx) return q8_fail(ctx, Q8_ERR_NULL, "output_logits_f32: NULL argument");
    if (!f32_fits(n, ro->W_c.cols) || !f32_fits(n, ro->W_s.cols) || !f32_fits(n, ro->W_y.cols) || !f32_fits(n, R))
        return q8_fail(ctx, Q8_ERR_SHAPE, "n_beam * dimension exceeds 16384");
    Carver cv(ctx);
    float *part[3];
    for (int u = 0; u < 3; ++u) part[u] = cv.take<float>((size_t)n * R);
    float *t = t_out ? t_out : cv.take<float>((size_t)n * R);
    const size_t ngrp = (size_t)q8i_out_tiles(V);
    float *pm = cv.take<float>(ngrp * n);
    double *ps = cv.take<double>(ngrp * n);
    float *lg = logits ? logits : cv.take<float>((size_t)n * V);
    if (!cv.ok) return q8_fail(ctx, Q8_ERR_WORKSPACE, "output_logits_f32: workspace too small");
    const q8i_f32_job j[3] = {{&ro->W_s, s, ro->W_s.cols, nullptr, part[0], R}, {&ro->W_y, y_emb, ro->W_y.cols, nullptr, part[1], R},
                              {&ro->W_c, ctx_vec, ro->W_c.cols, nullptr, part[2], R}};
    TRY(q8i_gemv_f32(ctx, j, 3, n));
    TRY(q8i_readout_combine(ctx, part[0], part[1], part[2], ro->b_t, R, n, t, 0, nullptr, nullptr, nullptr));
    const q8i_f32_job jo = {W_out, t, R, b_out, lg, V};
    TRY(q8i_gemv_f32(ctx, &jo, 1, n));
    TRY(q8i_logit_stats(ctx, lg, n, V, pm, ps));
    return q8i_select_logits(ctx, pm, ps, lg, V, n, k, lse, topk_logp, topk_idx);
}

// ------------------------------------------------------------------------------ ensembles ----

namespace {
const int kMaxModels = 4;
struct EnsModelBufs {
    size_t X, enc_h, P, y, s0, s1, cv, logits, lse;
};
struct EnsBufs {
    EnsModelBufs m[kMaxModels];
    size_t comb, lp, idx, state, total;
};
EnsBufs ensemble_layout(const q8_model *const *ms, int M, int l, int beam, int k, int max_steps)
{
    EnsBufs b;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += up256(bytes); return at; };
    const size_t V = ms[0]->W_out.rows;
    for (int i = 0; i < M; ++i) {
        const q8_model *m = ms[i];
        const size_t E = m->E, H = m->dec.r.Wh.cols, C = m->dec.q.Wx.cols, A = m->dec.att_U.rows;
        EnsModelBufs &e = b.m[i];
        e.X = take((size_t)l * E * 4); e.enc_h = take((size_t)l * C * 4); e.P = take((size_t)l * A * 4);
        e.y = take((size_t)beam * E * 4); e.s0 = take((size_t)beam * H * 4); e.s1 = take((size_t)beam * H * 4);
        e.cv = take((size_t)beam * C * 4); e.logits = take((size_t)beam * V * 4); e.lse = take((size_t)beam * 4);
    }
    b.comb = take((size_t)beam * V * 4);
    b.lp = take((size_t)beam * k * 4); b.idx = take((size_t)beam * k * 4);
    b.state = take(q8i_beam_state_bytes(max_steps));
    b.total = o;
    return b;
}
}  // namespace

size_t q8_translate_ensemble_bytes(const q8_model *const *models, int n_models, int max_l, int beam, int k, int max_steps)
{
    if (!models || n_models < 1 || n_models > kMaxModels || max_l < 1 || beam < 1 || k < 1 || max_steps < 1) return 0;
    for (int i = 0; i < n_models; ++i)
        if (!models[i]) return 0;
    return ensemble_layout(models, n_models, max_l, beam, k, max_steps).total;
}

q8_status q8_translate_ensemble(q8_ctx *ctx, const q8_model *const *models, int n_models, const int32_t *src_tokens, int l,
                                int beam, int k, int max_steps, int32_t *tokens_host, int *len_host, float *score_host,
                                int *steps_host)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!models || !src_tokens) return q8_fail(ctx, Q8_ERR_NULL, "q8_translate_ensemble: NULL argument");
    if (n_models < 1 || n_models > kMaxModels) return q8_fail(ctx, Q8_ERR_SHAPE, "n_models = %d outside [1, %d]", n_models, kMaxModels);
    for (int i = 0; i < n_models; ++i)
        if (!models[i]) return q8_fail(ctx, Q8_ERR_NULL, "model %d: NULL", i);
    if (n_models == 1)
        return q8_translate(ctx, models[0], src_tokens, l, beam, k, max_steps, tokens_host, len_host, score_host, steps_host);
    const int V = models[0]->W_out.rows;
    for (int i = 0; i < n_models; ++i) {
        const q8_model *m = models[i];
        if (!m->E_src || !m->E_tgt) return q8_fail(ctx, Q8_ERR_NULL, "model %d: NULL embedding table", i);
        TRY(check_gru(ctx, &m->enc_fwd, "enc_fwd"));
        TRY(check_gru(ctx, &m->dec.r, "dec.r"));
        TRY(check_gru(ctx, &m->dec.q, "dec.q"));
        TRY(check_mat(ctx, &m->att_W, "att_W"));
        TRY(check_mat(ctx, &m->dec.att_U, "att_U"));
        TRY(check_mat(ctx, &m->W_out, "W_out"));
        const int E = m->E, H = m->dec.r.Wh.cols, C = m->dec.q.Wx.cols, A = m->dec.att_U.rows;
        if (m->enc_fwd.Wx.cols != E || m->dec.r.Wx.cols != E || 2 * m->enc_fwd.Wh.cols != C || m->att_W.cols != C ||
            m->att_W.rows != A || m->enc_fwd.Wh.cols != H)
            return q8_fail(ctx, Q8_ERR_SHAPE, "model %d: dimensions are inconsistent", i);
        if (m->W_out.rows != V) return q8_fail(ctx, Q8_ERR_SHAPE, "the models must share the target vocabulary");
        if (m->V_src <= 0 || m->V_tgt != V) return q8_fail(ctx, Q8_ERR_SHAPE, "model %d: need V_src > 0 and V_tgt = rows of W_out", i);
    }
    if (l <= 0 || l > kMaxL) return q8_fail(ctx, Q8_ERR_SHAPE, "l = %d outside [1, %d]", l, kMaxL);
    if (beam <= 0 || beam > Q8_MAX_BEAM || k < beam || k > kMaxK || k > V || max_steps <= 0)
        return q8_fail(ctx, Q8_ERR_SHAPE, "need 1 <= beam <= %d, beam <= k <= %d, max_steps > 0", Q8_MAX_BEAM, kMaxK);
    if (ctx->ws_reserved_top) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_translate_ensemble is not re-entrant");
    const EnsBufs b = ensemble_layout(models, n_models, l, beam, k, max_steps);
    const size_t ngrp = (size_t)q8i_out_tiles(V);
    const size_t stats = up256(ngrp * beam * 4) + up256(ngrp * beam * 8);
    if (b.total + stats + Q8_WS_HEADER > ctx->ws_bytes)
        return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_translate_ensemble: workspace too small");
    char *top = ctx->ws + ((ctx->ws_bytes - b.total) & ~(size_t)255);
    ctx->ws_reserved_top = ctx->ws_bytes - (size_t)(top - ctx->ws);
    float *lp = (float *)(top + b.lp), *comb = (float *)(top + b.comb);
    int32_t *idx = (int32_t *)(top + b.idx);
    void *state = top + b.state;
    auto F = [&](size_t off) { return (float *)(top + off); };

    q8_status st = Q8_OK;
    for (int i = 0; i < n_models && !st; ++i) {
        const q8_model *m = models[i];
        const EnsModelBufs &e = b.m[i];
        const int E = m->E, H = m->dec.r.Wh.cols, C = m->dec.q.Wx.cols, A = m->dec.att_U.rows;
        st = q8i_gather_rows(ctx, m->E_src, src_tokens, l, E, m->V_src, F(e.X));
        if (!st) st = q8_encode(ctx, &m->enc_fwd, &m->enc_bwd, F(e.X), l, F(e.enc_h));
        if (!st) st = q8_gemm_narrow(ctx, &m->att_W, F(e.enc_h), l, C, m->att_b, F(e.P), A, nullptr);
        // the same initial search state from every model; each call also fills that model's first inputs
        if (!st) st = q8i_beam_init(ctx, state, beam, max_steps, F(e.enc_h), m->E_tgt, E, H, F(e.y), F(e.s0));
    }
    int cur = 0, done = 0;
    for (int t = 0; t < max_steps && !st && !done; ++t) {
        const float *lg[kMaxModels], *ls[kMaxModels];
        for (int i = 0; i < n_models && !st; ++i) {
            const q8_model *m = models[i];
            const EnsModelBufs &e = b.m[i];
            float *s_in = F(cur ? e.s1 : e.s0), *s_out = F(cur ? e.s0 : e.s1);
            st = cgru_decoder_step_q8(ctx, &m->dec, F(e.P), F(e.enc_h), l, F(e.y), s_in, beam, s_out, F(e.cv), nullptr,
                                      nullptr, nullptr);
            // this model's logits and log-sum-exp (its own top-k is not used)
            if (!st) st = output_impl(ctx, &m->ro, &m->W_out, m->b_out, s_out, F(e.y), F(e.cv), nullptr, beam, k, F(e.logits),
                                      F(e.lse), lp, idx, nullptr, nullptr, nullptr);
            lg[i] = F(e.logits);
            ls[i] = F(e.lse);
        }
        if (st) break;
        // averaged distribution, its k best entries, and the search step (first model's buffers)
        Carver cv(ctx);
        float *pm = cv.take<float>(ngrp * beam);
        double *ps = cv.take<double>(ngrp * beam);
        if (!cv.ok) { st = q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_translate_ensemble: workspace too small"); break; }
        st = q8i_ensemble_combine(ctx, lg, ls, n_models, beam, V, comb, pm, ps);
        const q8_model *m0 = models[0];
        const EnsModelBufs &e0 = b.m[0];
        q8i_beam_desc bd = {state, F(cur ? e0.s0 : e0.s1), m0->E_tgt, F(e0.y), F(cur ? e0.s1 : e0.s0), m0->E,
                            m0->dec.r.Wh.cols};
        if (!st) st = q8i_select_normalized(ctx, pm, ps, comb, V, beam, k, lp, idx, &bd);
        for (int i = 1; i < n_models && !st; ++i) {
            const q8_model *m = models[i];
            const EnsModelBufs &e = b.m[i];
            st = q8i_beam_regather(ctx, state, beam, F(cur ? e.s0 : e.s1), m->dec.r.Wh.cols, m->E_tgt, m->E, F(e.y),
                                   F(cur ? e.s1 : e.s0));
        }
        if (!st && (t % 8 == 7))
            st = q8i_beam_read(ctx, state, max_steps, nullptr, nullptr, nullptr, nullptr, &done);
    }
    if (!st) st = q8i_beam_read(ctx, state, max_steps, tokens_host, len_host, score_host, steps_host, nullptr);
    if (!st) st = q8_encode_check(ctx);                       // (the stream is idle here: one word read back)
    ctx->ws_reserved_top = 0;
    return st;
}

// ---------------------------------------------------------------- sentences side by side ----

q8_status q8_beam_init_batch(q8_ctx *ctx, void *states, int n_sent, int beam, int max_steps, const float *enc_h,
                             const int32_t *sent_off, int C, const float *E_tgt, int E, int H, float *y_emb, float *s,
                             int32_t *done)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!states || !enc_h || !sent_off || !E_tgt || !y_emb || !s || !done)
        return q8_fail(ctx, Q8_ERR_NULL, "q8_beam_init_batch: NULL argument");
    if (n_sent <= 0 || beam <= 0 || beam > Q8_MAX_BEAM || (long long)n_sent * beam > kMaxMfmaN || max_steps <= 0 || E <= 0 ||
        H <= 0 || C < H)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_beam_init_batch: bad sizes");
    return q8i_beam_batch(ctx, 1, states, q8i_beam_state_bytes(max_steps), n_sent, beam, 0, max_steps, nullptr, nullptr,
                          nullptr, E_tgt, E, H, y_emb, s, done, enc_h, sent_off, C, 0);
}

q8_status q8_beam_update_batch(q8_ctx *ctx, void *states, int n_sent, int beam, int k, int max_steps,
                               const float *topk_logp, const int32_t *topk_idx, const float *s_step, int H,
                               const float *E_tgt, int E, float *y_emb, float *s_next, int32_t *done)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!states || !topk_logp || !topk_idx || !s_step || !E_tgt || !y_emb || !s_next || !done)
        return q8_fail(ctx, Q8_ERR_NULL, "q8_beam_update_batch: NULL argument");
    if (n_sent <= 0 || beam <= 0 || beam > Q8_MAX_BEAM || (long long)n_sent * beam > kMaxMfmaN || k < beam || k > kMaxK ||
        max_steps <= 0 || E <= 0 || H <= 0)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_beam_update_batch: bad sizes");
    if (s_next == s_step) return q8_fail(ctx, Q8_ERR_SHAPE, "s_next must not alias s_step");
    return q8i_beam_batch(ctx, 0, states, q8i_beam_state_bytes(max_steps), n_sent, beam, k, max_steps, topk_logp, topk_idx,
                          s_step, E_tgt, E, H, y_emb, s_next, done, nullptr, nullptr, 0, 0);
}

namespace {
// The search step's gather takes the codes of its rows along where there is room for them in its pass
// (see output_logits_beam_loop_q8): fills the descriptor and says whether it did.
bool batch_hand_on(q8i_beam_desc *bd, const q8_row_codes *E_codes, const q8_codes *s_codes, q8_codes *y_next, q8_codes *s_next,
                   int E, int H)
{
    if (!E_codes || !E_codes->q || !E_codes->scale || !aligned16(E_codes->q) || !s_codes || s_codes->valid != 1 || !y_next || !s_next)
        return false;
    const int ldy = E_codes->ld, lds = s_codes->ld;
    if (!codes_usable(s_codes, lds) || !codes_usable(y_next, ldy) || !codes_usable(s_next, lds) || s_next->q == s_codes->q)
        return false;
    if (E % 4 || H % 4 || ldy % 16 || lds % 16 || ldy < E || lds < H || E / 4 + ldy / 16 + lds / 16 > 256) return false;
    bd->Eq = E_codes->q; bd->Es = E_codes->scale; bd->ldy = ldy; bd->lds = lds;
    bd->sq_in = s_codes->q; bd->ss_in = s_codes->scale;
    bd->yq_out = y_next->q; bd->ys_out = y_next->scale; bd->sq_out = s_next->q; bd->ss_out = s_next->scale;
    return true;
}
}  // namespace

q8_status q8_beam_update_batch_loop(q8_ctx *ctx, void *states, int n_sent, int beam, int k, int max_steps,
                                    const float *topk_logp, const int32_t *topk_idx, const float *s_step, int H,
                                    const float *E_tgt, int E, int V, float *y_emb, float *s_next, int32_t *done,
                                    const q8_row_codes *E_codes, const q8_codes *s_codes, q8_codes *y_next_codes,
                                    q8_codes *s_next_codes)
{
    if (y_next_codes) y_next_codes->valid = 0;
    if (s_next_codes) s_next_codes->valid = 0;
    if (!ctx) return Q8_ERR_NULL;
    if (!states || !topk_logp || !topk_idx || !s_step || !E_tgt || !y_emb || !s_next || !done)
        return q8_fail(ctx, Q8_ERR_NULL, "q8_beam_update_batch: NULL argument");
    if (n_sent <= 0 || beam <= 0 || beam > Q8_MAX_BEAM || (long long)n_sent * beam > kMaxMfmaN || k < beam || k > kMaxK ||
        max_steps <= 0 || E <= 0 || H <= 0 || V < 0)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_beam_update_batch: bad sizes");
    if (s_next == s_step) return q8_fail(ctx, Q8_ERR_SHAPE, "s_next must not alias s_step");
    q8i_beam_desc bd = {};
    // (codes are gathered by token id: only with the table's height known, so that every id stays inside it)
    const bool hand_on = V > 0 && batch_hand_on(&bd, E_codes, s_codes, y_next_codes, s_next_codes, E, H);
    const q8_status st = q8i_beam_batch(ctx, 0, states, q8i_beam_state_bytes(max_steps), n_sent, beam, k, max_steps, topk_logp,
                                        topk_idx, s_step, E_tgt, E, H, y_emb, s_next, done, nullptr, nullptr, 0, V,
                                        hand_on ? &bd : nullptr);
    if (!st && hand_on) { y_next_codes->valid = 2; s_next_codes->valid = 2; }
    return st;
}

namespace {
// Output layer of a panel and the sentences' search steps: one launch fewer where the panel selection can run
// the search steps itself, the two calls one after the other everywhere else.  Same results either way.
q8_status output_and_search_batch(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                  const float *s, float *y_emb, const float *ctx_vec, int n_sent, int beam, int k,
                                  int max_steps, void *states, const float *E_tgt, int E, int H, float *s_next, int32_t *done,
                                  float *topk_logp, int32_t *topk_idx, const q8_codes *s_codes, const q8_codes *y_codes,
                                  const q8_codes *ctx_codes, const q8i_beam_desc *hand_on)
{
    const int n = n_sent * beam, V = W_out->rows;
    const BeamBatchArgs bb = q8i_beam_batch_args(states, q8i_beam_state_bytes(max_steps), beam, k, max_steps, topk_logp, topk_idx, s,
                                                 E_tgt, E, H, y_emb, s_next, done, nullptr, nullptr, 0, V, hand_on);
    int fused = 0;
    TRY(output_impl(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, nullptr, n, k, nullptr, nullptr, topk_logp, topk_idx, nullptr,
                    nullptr, nullptr, y_codes, ctx_codes, s_codes, &bb, &fused));
    if (fused) return Q8_OK;
    return q8i_beam_batch(ctx, 0, states, q8i_beam_state_bytes(max_steps), n_sent, beam, k, max_steps, topk_logp, topk_idx, s,
                          E_tgt, E, H, y_emb, s_next, done, nullptr, nullptr, 0, V, hand_on);
}
}  // namespace

q8_status output_logits_beam_batch_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                      const float *s, float *y_emb, const float *ctx_vec, int n_sent, int beam, int k,
                                      int max_steps, void *states, const float *E_tgt, int E, float *s_next, int32_t *done,
                                      float *topk_logp, int32_t *topk_idx, const q8_codes *s_codes, q8_codes *y_codes,
                                      const q8_codes *ctx_codes, q8_codes *s_next_codes, const q8_row_codes *E_codes)
{
    // y_codes as an input: the codes of this step's y_emb for the readout (valid != 0)
    q8_codes y_in = {nullptr, nullptr, 0, 0};
    if (y_codes) { y_in = *y_codes; y_codes->valid = 0; }
    if (s_next_codes) s_next_codes->valid = 0;
    if (!ctx) return Q8_ERR_NULL;
    if (!ro || !W_out || !states || !E_tgt || !s_next || !s || !y_emb || !ctx_vec || !done || !topk_logp || !topk_idx)
        return q8_fail(ctx, Q8_ERR_NULL, "output_logits_beam_batch_q8: NULL argument");
    if (n_sent <= 0 || beam <= 0 || beam > Q8_MAX_BEAM || (long long)n_sent * beam > kMaxMfmaN || k < beam || k > kMaxK ||
        max_steps <= 0 || E <= 0)
        return q8_fail(ctx, Q8_ERR_SHAPE, "output_logits_beam_batch_q8: bad sizes");
    if (s_next == s) return q8_fail(ctx, Q8_ERR_SHAPE, "s_next must not alias s");
    if (!aligned16(E_tgt) || !aligned16(s_next)) return q8_fail(ctx, Q8_ERR_ALIGN, "fp32 buffers need 16-byte alignment");
    if (E != ro->W_y.cols) return q8_fail(ctx, Q8_ERR_SHAPE, "E does not match the readout's embedding width");
    const int H = ro->W_s.cols;
    q8i_beam_desc bd = {};
    // (the codes of s for the gather are the caller's: valid == 1, as cgru_decoder_step_batch_codes_q8 left them)
    const bool hand_on = batch_hand_on(&bd, E_codes, s_codes, y_codes, s_next_codes, E, H);
    const q8_status st = output_and_search_batch(ctx, ro, W_out, b_out, s, y_emb, ctx_vec, n_sent, beam, k, max_steps, states, E_tgt,
                                                 E, H, s_next, done, topk_logp, topk_idx, s_codes, y_codes ? &y_in : nullptr,
                                                 ctx_codes, hand_on ? &bd : nullptr);
    if (!st && hand_on) { y_codes->valid = 2; s_next_codes->valid = 2; }
    return st;
}

q8_status q8_beam_result_batch(q8_ctx *ctx, const void *states, int n_sent, int max_steps, int32_t *tokens_host,
                               int *len_host, float *score_host, int *steps_host)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!states || n_sent <= 0 || max_steps <= 0) return q8_fail(ctx, Q8_ERR_NULL, "q8_beam_result_batch: bad argument");
    return q8i_beam_read_batch(ctx, states, q8i_beam_state_bytes(max_steps), n_sent, max_steps, tokens_host, len_host,
                               score_host, steps_host);
}

namespace {
struct BatchBufs {
    size_t X, enc_h, P, off, y, s0, s1, cv, lp, idx, done, states, yq, ys, cq, cs, sq, ss, pq, ps, total;
};
BatchBufs batch_layout(const q8_model *m, int total_l, int n_sent, int beam, int k, int max_steps)
{
    const size_t E = m->E, H = m->dec.r.Wh.cols, C = m->dec.q.Wx.cols, A = m->dec.att_U.rows, n = (size_t)n_sent * beam;
    BatchBufs b;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += up256(bytes); return at; };
    b.X = take((size_t)total_l * E * 4); b.enc_h = take((size_t)total_l * C * 4); b.P = take((size_t)total_l * A * 4);
    b.off = take((size_t)(n_sent + 1) * 4);
    b.y = take(n * E * 4); b.s0 = take(n * H * 4); b.s1 = take(n * H * 4);
    b.cv = take(n * C * 4); b.lp = take(n * k * 4); b.idx = take(n * k * 4);
    b.done = take((size_t)n_sent * 4);
    b.states = take(q8i_beam_state_bytes(max_steps) * n_sent);
    // codes of y, of the context vectors and of the new states, handed from the decoder step to the output layer
    b.yq = take(n * m->dec.r.Wx.ld); b.ys = take(n * 4);
    b.cq = take(n * m->dec.q.Wx.ld); b.cs = take(n * 4);
    b.sq = take(n * m->ro.W_s.ld); b.ss = take(n * 4);
    // codes of the surviving states, handed from the search step to the next decoder step
    b.pq = take(n * m->dec.r.Wh.ld); b.ps = take(n * 4);
    b.total = o;
    return b;
}
}  // namespace

size_t q8_translate_batch_bytes(const q8_model *m, int total_l, int n_sent, int beam, int k, int max_steps)
{
    if (!m || total_l < 1 || n_sent < 1 || beam < 1 || k < 1 || max_steps < 1) return 0;
    return batch_layout(m, total_l, n_sent, beam, k, max_steps).total;
}

q8_status q8_translate_batch(q8_ctx *ctx, const q8_model *m, const int32_t *src_tokens, const int32_t *sent_off_host,
                             int n_sent, int beam, int k, int max_steps, int32_t *tokens_host, int *len_host,
                             float *score_host, int *steps_host)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!m || !src_tokens || !sent_off_host || !m->E_src || !m->E_tgt)
        return q8_fail(ctx, Q8_ERR_NULL, "q8_translate_batch: NULL argument");
    TRY(check_gru(ctx, &m->enc_fwd, "enc_fwd"));
    TRY(check_gru(ctx, &m->dec.r, "dec.r"));
    TRY(check_gru(ctx, &m->dec.q, "dec.q"));
    TRY(check_mat(ctx, &m->att_W, "att_W"));
    TRY(check_mat(ctx, &m->dec.att_U, "att_U"));
    const int E = m->E, H = m->dec.r.Wh.cols, C = m->dec.q.Wx.cols, A = m->dec.att_U.rows;
    if (beam <= 0 || beam > Q8_MAX_BEAM || k < beam || k > kMaxK || max_steps <= 0)
        return q8_fail(ctx, Q8_ERR_SHAPE, "need 1 <= beam <= %d, beam <= k <= %d, max_steps > 0", Q8_MAX_BEAM, kMaxK);
    if (n_sent <= 0 || (long long)n_sent * beam > kMaxMfmaN)
        return q8_fail(ctx, Q8_ERR_SHAPE, "need 1 <= n_sent and n_sent * beam <= %d", kMaxMfmaN);
    if (m->V_src <= 0 || m->V_tgt != m->W_out.rows)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_translate_batch: need V_src > 0 and V_tgt = rows of W_out");
    if (m->enc_fwd.Wx.cols != E || m->dec.r.Wx.cols != E || 2 * m->enc_fwd.Wh.cols != C || m->att_W.cols != C ||
        m->att_W.rows != A || m->enc_fwd.Wh.cols != H)
        return q8_fail(ctx, Q8_ERR_SHAPE, "q8_translate_batch: model dimensions are inconsistent");
    int max_l = 0;
    if (sent_off_host[0] != 0) return q8_fail(ctx, Q8_ERR_SHAPE, "sent_off[0] must be 0");
    for (int s = 0; s < n_sent; ++s) {
        const int l = sent_off_host[s + 1] - sent_off_host[s];
        if (l <= 0 || l > kMaxL) return q8_fail(ctx, Q8_ERR_SHAPE, "sentence %d: length %d outside [1, %d]", s, l, kMaxL);
        if (l > max_l) max_l = l;
    }
    const int total_l = sent_off_host[n_sent];
    if (ctx->ws_reserved_top) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_translate_batch is not re-entrant");
    const BatchBufs b = batch_layout(m, total_l, n_sent, beam, k, max_steps);
    if (b.total + Q8_WS_HEADER > ctx->ws_bytes) return q8_fail(ctx, Q8_ERR_WORKSPACE, "q8_translate_batch: workspace too small");
    char *top = ctx->ws + ((ctx->ws_bytes - b.total) & ~(size_t)255);
    float *X = (float *)(top + b.X), *enc_h = (float *)(top + b.enc_h), *P = (float *)(top + b.P);
    int32_t *off = (int32_t *)(top + b.off), *done = (int32_t *)(top + b.done);
    float *y = (float *)(top + b.y), *sv[2] = {(float *)(top + b.s0), (float *)(top + b.s1)};
    float *cvec = (float *)(top + b.cv), *lp = (float *)(top + b.lp);
    int32_t *idx = (int32_t *)(top + b.idx);
    void *states = top + b.states;
    const int n = n_sent * beam;
    q8_codes yc = {(int8_t *)(top + b.yq), (float *)(top + b.ys), m->dec.r.Wx.ld, 0};
    q8_codes cc = {(int8_t *)(top + b.cq), (float *)(top + b.cs), m->dec.q.Wx.ld, 0};
    q8_codes sc = {(int8_t *)(top + b.sq), (float *)(top + b.ss), m->ro.W_s.ld, 0};
    q8_codes pc = {(int8_t *)(top + b.pq), (float *)(top + b.ps), m->dec.r.Wh.ld, 0};
    const q8_row_codes *Ec = m->E_tgt_codes.q ? &m->E_tgt_codes : nullptr;
    ctx->ws_reserved_top = ctx->ws_bytes - (size_t)(top - ctx->ws);

    q8_status st = Q8_OK;
    if (hipMemcpyAsync(off, sent_off_host, sizeof(int32_t) * (n_sent + 1), hipMemcpyHostToDevice, ctx->stream) != hipSuccess)
        st = q8_fail(ctx, Q8_ERR_DEVICE, "q8_translate_batch: offsets copy failed");
    if (!st) st = q8i_gather_rows(ctx, m->E_src, src_tokens, total_l, E, m->V_src, X);                   // x_i of Eq. 1
    if (!st) st = q8_encode_batch(ctx, &m->enc_fwd, &m->enc_bwd, X, off, sent_off_host, n_sent, enc_h);    // Eq. 1
    // w(h_i) of Eq. 6 for every position of every sentence (per-vector quantization: the
    // same values as sentence by sentence), in panels of at most 1024 positions
    for (int o = 0; o < total_l && !st; o += kMaxMfmaN) {
        const int cnt = total_l - o < kMaxMfmaN ? total_l - o : kMaxMfmaN;
        st = q8_gemm_narrow(ctx, &m->att_W, enc_h + (size_t)o * C, cnt, C, m->att_b, P + (size_t)o * A, A, nullptr);
    }
    if (!st) st = q8_beam_init_batch(ctx, states, n_sent, beam, max_steps, enc_h, off, C, m->E_tgt, E, H, y, sv[0], done);
    int cur = 0;
    bool all_done = false;
    int32_t *done_host = (int32_t *)malloc(sizeof(int32_t) * n_sent);
    if (!done_host && !st) st = q8_fail(ctx, Q8_ERR_DEVICE, "out of host memory");
    for (int t = 0; t < max_steps && !st && !all_done; ++t) {
        if (n <= kMaxNarrow && n_sent == 1) {
            st = cgru_decoder_step_codes_q8(ctx, &m->dec, P, enc_h, total_l, y, sv[cur], n, sv[cur ^ 1], cvec, nullptr, nullptr,
                                            nullptr, &yc, &cc);
            sc.valid = 0;
        } else {
            st = cgru_decoder_step_batch_loop_q8(ctx, &m->dec, P, enc_h, off, n_sent, beam, max_l, y, sv[cur], sv[cur ^ 1],
                                                 cvec, nullptr, nullptr, &yc, &cc, &sc, &pc);
        }
        // (the table's height goes along: a token id outside it, which takes non-finite logits, is replaced by 0;
        // where the model brings its embeddings' codes, the codes of the gathered rows go to the next step)
        q8i_beam_desc bd = {};
        const bool hand_on = !st && batch_hand_on(&bd, Ec, &sc, &yc, &pc, E, H);
        const q8_codes y_in = yc;
        yc.valid = 0;
        pc.valid = 0;
        if (!st) st = output_and_search_batch(ctx, &m->ro, &m->W_out, m->b_out, sv[cur ^ 1], y, cvec, n_sent, beam, k, max_steps,
                                              states, m->E_tgt, E, H, sv[cur], done, lp, idx, &sc, &y_in, &cc, hand_on ? &bd : nullptr);
        if (!st && hand_on) { yc.valid = 2; pc.valid = 2; }
        if (!st && (t % 8 == 7)) {
            hipError_t e = hipMemcpyAsync(done_host, done, sizeof(int32_t) * n_sent, hipMemcpyDeviceToHost, ctx->stream);
            if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
            if (e != hipSuccess) st = q8_fail(ctx, Q8_ERR_DEVICE, "q8_translate_batch: %s", hipGetErrorString(e));
            all_done = true;
            for (int s = 0; s < n_sent && !st; ++s) all_done = all_done && done_host[s] != 0;
        }
    }
    free(done_host);
    if (!st) st = q8_beam_result_batch(ctx, states, n_sent, max_steps, tokens_host, len_host, score_host, steps_host);
    ctx->ws_reserved_top = 0;
    return st;
}

}  // extern "C"
