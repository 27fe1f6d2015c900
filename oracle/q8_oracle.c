/*
 * q8_oracle.c -- CPU oracle for 8-bit GRU-NMT decoding.  TEST INFRASTRUCTURE ONLY.
 * See q8_oracle.h for what each function follows in the paper and for the pins.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC q8_oracle.c -lm
 * (no intrinsics, no blocking, no reordering: loops are written as the
 * definitions read).
 */
#include "q8_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* Non-finite inputs: the method has no rule for them (a NaN has no 8-bit code), so the
 * oracle defines no result; it counts them where data enters a product, and the callers
 * turn a non-zero count into an error. */
static long g_nonfinite = 0;

static void note_nonfinite(const float *v, int n)
{
    for (int i = 0; i < n; ++i)
        if (!isfinite(v[i])) ++g_nonfinite;
}

long q8o_nonfinite_count(int reset)
{
    long c = g_nonfinite;
    if (reset) g_nonfinite = 0;
    return c;
}

/* ------------------------------------------------------------------ Section 3 -- */

void q8o_quantize(const float *v, int n, int8_t *q, float *scale)
{
    note_nonfinite(v, n);
    float m = 0.0f;
    for (int i = 0; i < n; ++i) {
        float a = fabsf(v[i]);
        if (a > m) m = a;
    }
    if (m < 0x1p-100f) {
        for (int i = 0; i < n; ++i) q[i] = 0;
        *scale = 1.0f;
        return;
    }
    float s = m / 127.0f;
    float inv = 127.0f / m;
    for (int i = 0; i < n; ++i) {
        float t = v[i] * inv;
        float r = rintf(t);            /* default rounding mode: half to even */
        if (r > 127.0f) r = 127.0f;
        if (r < -127.0f) r = -127.0f;
        q[i] = (int8_t)r;
    }
    *scale = s;
}

void q8o_quantize_matrix(const float *W, int rows, int cols, int ld_in,
                         int8_t *Wq, int ld_out, float *scale)
{
    for (int i = 0; i < rows; ++i) note_nonfinite(W + (size_t)i * ld_in, cols);
    float m = 0.0f;
    for (int i = 0; i < rows; ++i)
        for (int k = 0; k < cols; ++k) {
            float a = fabsf(W[(size_t)i * ld_in + k]);
            if (a > m) m = a;
        }
    int zero = (m < 0x1p-100f);
    float s = zero ? 1.0f : m / 127.0f;
    float inv = zero ? 0.0f : 127.0f / m;
    for (int i = 0; i < rows; ++i) {
        for (int k = 0; k < cols; ++k) {
            float r = 0.0f;
            if (!zero) {
                float t = W[(size_t)i * ld_in + k] * inv;
                r = rintf(t);
                if (r > 127.0f) r = 127.0f;
                if (r < -127.0f) r = -127.0f;
            }
            Wq[(size_t)i * ld_out + k] = (int8_t)r;
        }
        for (int k = cols; k < ld_out; ++k) Wq[(size_t)i * ld_out + k] = 0;
    }
    *scale = s;
}

void q8o_accumulate(const int8_t *Wq, int rows, int cols, int ld, const int8_t *xq, int32_t *acc)
{
    for (int i = 0; i < rows; ++i) {
        int32_t a = 0;
        for (int k = 0; k < cols; ++k)
            a += (int32_t)Wq[(size_t)i * ld + k] * (int32_t)xq[k];
        acc[i] = a;
    }
}

void q8o_dequantize(const int32_t *acc, int rows, float s_w, float s_x, const float *bias, float *y)
{
    float c = s_w * s_x;
    for (int i = 0; i < rows; ++i) {
        float f = (float)acc[i];
        float p = f * c;
        if (bias) p = p + bias[i];
        y[i] = p;
    }
}

void q8o_gemv(const q8o_linear *L, const float *x, float *y,
              int8_t *tap_xq, float *tap_xscale, int32_t *tap_acc)
{
    int8_t *xq = (int8_t *)malloc((size_t)L->cols);
    int32_t *acc = (int32_t *)malloc(sizeof(int32_t) * (size_t)L->rows);
    float sx;
    q8o_quantize(x, L->cols, xq, &sx);
    q8o_accumulate(L->Wq, L->rows, L->cols, L->ldq, xq, acc);
    q8o_dequantize(acc, L->rows, L->scale, sx, L->bias, y);
    if (tap_xq) memcpy(tap_xq, xq, (size_t)L->cols);
    if (tap_xscale) *tap_xscale = sx;
    if (tap_acc) memcpy(tap_acc, acc, sizeof(int32_t) * (size_t)L->rows);
    free(xq);
    free(acc);
}

void q8o_gemm_narrow(const q8o_linear *L, const float *X, int n, int ldx, float *Y, int ldy,
                     int8_t *tap_xq, float *tap_xscale, int32_t *tap_acc)
{
    for (int j = 0; j < n; ++j)
        q8o_gemv(L, X + (size_t)j * ldx, Y + (size_t)j * ldy,
                 tap_xq ? tap_xq + (size_t)j * L->cols : NULL,
                 tap_xscale ? tap_xscale + j : NULL,
                 tap_acc ? tap_acc + (size_t)j * L->rows : NULL);
}

void q8o_quantize_matrix_rows(const float *W, int rows, int cols, int ld_in,
                              int8_t *Wq, int ld_out, float *row_scale)
{
    for (int i = 0; i < rows; ++i) {
        q8o_quantize(W + (size_t)i * ld_in, cols, Wq + (size_t)i * ld_out, row_scale + i);
        for (int k = cols; k < ld_out; ++k) Wq[(size_t)i * ld_out + k] = 0;
    }
}

void q8o_dequantize_rows(const int32_t *acc, int rows, const float *row_scale, float s_x,
                         const float *bias, float *y)
{
    for (int i = 0; i < rows; ++i) {
        float c = row_scale[i] * s_x;
        float f = (float)acc[i];
        float p = f * c;
        if (bias) p = p + bias[i];
        y[i] = p;
    }
}

void q8o_gemm_narrow_rows(const int8_t *Wq, int rows, int cols, int ld, const float *row_scale,
                          const float *bias, const float *X, int n, int ldx, float *Y, int ldy,
                          int8_t *tap_xq, float *tap_xscale, int32_t *tap_acc)
{
    int8_t *xq = (int8_t *)malloc((size_t)cols);
    int32_t *acc = (int32_t *)malloc(sizeof(int32_t) * (size_t)rows);
    for (int j = 0; j < n; ++j) {
        float sx;
        q8o_quantize(X + (size_t)j * ldx, cols, xq, &sx);
        q8o_accumulate(Wq, rows, cols, ld, xq, acc);
        q8o_dequantize_rows(acc, rows, row_scale, sx, bias, Y + (size_t)j * ldy);
        if (tap_xq) memcpy(tap_xq + (size_t)j * cols, xq, (size_t)cols);
        if (tap_xscale) tap_xscale[j] = sx;
        if (tap_acc) memcpy(tap_acc + (size_t)j * rows, acc, sizeof(int32_t) * (size_t)rows);
    }
    free(xq);
    free(acc);
}

void q8o_gemv_fp32(const q8o_linear *L, const float *x, float *y)
{
    note_nonfinite(x, L->cols);
    for (int i = 0; i < L->rows; ++i) {
        double a = 0.0;
        for (int k = 0; k < L->cols; ++k)
            a += (double)L->Wf[(size_t)i * L->ldf + k] * (double)x[k];
        float p = (float)a;
        if (L->bias) p = p + L->bias[i];
        y[i] = p;
    }
}

void q8o_linear_apply(const q8o_linear *L, const float *x, int use_q8, float *y)
{
    if (use_q8) q8o_gemv(L, x, y, NULL, NULL, NULL);
    else q8o_gemv_fp32(L, x, y);
}

/* ------------------------------------------------------------------ Section 2 -- */

static float sigmoid_f(float a)
{
    return (float)(1.0 / (1.0 + exp(-(double)a)));
}

static float tanh_f(float a)
{
    return (float)tanh((double)a);
}

void q8o_gru_gates(const float *gx, const float *gh, const float *h_prev, int H, float *h_out)
{
    for (int j = 0; j < H; ++j) {
        float pr = gx[j] + gh[j];
        float r = sigmoid_f(pr);
        float pz = gx[H + j] + gh[H + j];
        float z = sigmoid_f(pz);
        float rn = r * gh[2 * H + j];
        float pn = gx[2 * H + j] + rn;
        float n = tanh_f(pn);
        float omz = 1.0f - z;
        float t1 = omz * n;
        float t2 = z * h_prev[j];
        h_out[j] = t1 + t2;
    }
}

void q8o_gru_step(const q8o_gru *g, const float *x, const float *h_prev, int use_q8, float *h_out)
{
    int H = g->Wh.cols;
    float *gx = (float *)malloc(sizeof(float) * 3 * (size_t)H);
    float *gh = (float *)malloc(sizeof(float) * 3 * (size_t)H);
    float *hn = (float *)malloc(sizeof(float) * (size_t)H);
    q8o_linear_apply(&g->Wx, x, use_q8, gx);
    q8o_linear_apply(&g->Wh, h_prev, use_q8, gh);
    q8o_gru_gates(gx, gh, h_prev, H, hn);
    memcpy(h_out, hn, sizeof(float) * (size_t)H);   /* h_out may alias h_prev */
    free(gx);
    free(gh);
    free(hn);
}

void q8o_encode(const q8o_model *m, const float *X, int l, int use_q8, float *enc_h)
{
    int H = m->H, E = m->E, C = 2 * m->H;
    float *h = (float *)calloc((size_t)H, sizeof(float));
    /* forward direction: positions 1..l, state from the left, stored in the lower half */
    for (int i = 0; i < l; ++i) {
        q8o_gru_step(&m->enc_fwd, X + (size_t)i * E, h, use_q8, h);
        memcpy(enc_h + (size_t)i * C + H, h, sizeof(float) * (size_t)H);
    }
    /* backward direction: positions l..1, state from the right, stored in the upper half */
    memset(h, 0, sizeof(float) * (size_t)H);
    for (int i = l - 1; i >= 0; --i) {
        q8o_gru_step(&m->enc_bwd, X + (size_t)i * E, h, use_q8, h);
        memcpy(enc_h + (size_t)i * C, h, sizeof(float) * (size_t)H);
    }
    free(h);
}

void q8o_attention_precompute(const q8o_model *m, const float *enc_h, int l, int use_q8, float *P)
{
    for (int i = 0; i < l; ++i)
        q8o_linear_apply(&m->att_W, enc_h + (size_t)i * m->C, use_q8, P + (size_t)i * m->A);
}

void q8o_attention(const float *P, const float *enc_h, int l, int A, int C,
                   const float *a, const float *v, float *e_out, float *alpha, float *ctx)
{
    float *e = (float *)malloc(sizeof(float) * (size_t)l);
    double *w = (double *)malloc(sizeof(double) * (size_t)l);
    for (int i = 0; i < l; ++i) {
        double acc = 0.0;
        for (int j = 0; j < A; ++j) {
            float pre = P[(size_t)i * A + j] + a[j];
            float th = tanh_f(pre);
            acc += (double)v[j] * (double)th;
        }
        e[i] = (float)acc;
    }
    float mx = e[0];
    for (int i = 1; i < l; ++i)
        if (e[i] > mx) mx = e[i];
    double Z = 0.0;
    for (int i = 0; i < l; ++i) {
        w[i] = exp((double)e[i] - (double)mx);
        Z += w[i];
    }
    for (int i = 0; i < l; ++i) alpha[i] = (float)(w[i] / Z);
    for (int c = 0; c < C; ++c) {
        double acc = 0.0;
        for (int i = 0; i < l; ++i)
            acc += (double)alpha[i] * (double)enc_h[(size_t)i * C + c];
        ctx[c] = (float)acc;
    }
    if (e_out) memcpy(e_out, e, sizeof(float) * (size_t)l);
    free(e);
    free(w);
}

void q8o_attention_q8(const float *P, int l, int A, const float *a, const int8_t *vq, float s_v,
                      const int8_t *hTq, int C, int ldq, float s_h,
                      float *e_out, float *alpha, float *ctx)
{
    float *e = (float *)malloc(sizeof(float) * (size_t)l);
    double *w = (double *)malloc(sizeof(double) * (size_t)l);
    float *T = (float *)malloc(sizeof(float) * (size_t)A);
    int8_t *Tq = (int8_t *)malloc((size_t)A);
    int8_t *aq = (int8_t *)malloc((size_t)l);
    int32_t *acc = (int32_t *)malloc(sizeof(int32_t) * (size_t)C);
    for (int i = 0; i < l; ++i) {
        for (int j = 0; j < A; ++j) {
            float pre = P[(size_t)i * A + j] + a[j];
            T[j] = tanh_f(pre);
        }
        float sT;
        int32_t dot;
        q8o_quantize(T, A, Tq, &sT);
        q8o_accumulate(vq, 1, A, A, Tq, &dot);
        q8o_dequantize(&dot, 1, s_v, sT, NULL, &e[i]);
    }
    float mx = e[0];
    for (int i = 1; i < l; ++i)
        if (e[i] > mx) mx = e[i];
    double Z = 0.0;
    for (int i = 0; i < l; ++i) {
        w[i] = exp((double)e[i] - (double)mx);
        Z += w[i];
    }
    for (int i = 0; i < l; ++i) alpha[i] = (float)(w[i] / Z);
    float sa;
    q8o_quantize(alpha, l, aq, &sa);
    q8o_accumulate(hTq, C, l, ldq, aq, acc);
    q8o_dequantize(acc, C, s_h, sa, NULL, ctx);
    if (e_out) memcpy(e_out, e, sizeof(float) * (size_t)l);
    free(e); free(w); free(T); free(Tq); free(aq); free(acc);
}

void q8o_cgru_step(const q8o_model *m, const float *P, const float *enc_h, int l,
                   const float *y_emb, const float *s_prev, int use_q8,
                   float *s_mid, float *alpha, float *ctx, float *s_out)
{
    int H = m->H, A = m->A, C = m->C;
    float *sm = (float *)malloc(sizeof(float) * (size_t)H);
    float *a = (float *)malloc(sizeof(float) * (size_t)A);
    float *al = (float *)malloc(sizeof(float) * (size_t)l);
    float *cx = (float *)malloc(sizeof(float) * (size_t)C);
    q8o_gru_step(&m->dec_r, y_emb, s_prev, use_q8, sm);           /* Eq. 3 */
    q8o_linear_apply(&m->att_U, sm, use_q8, a);                   /* u(s') of Eq. 6 */
    q8o_attention(P, enc_h, l, A, C, a, m->att_v, NULL, al, cx);  /* Eq. 5-6 */
    q8o_gru_step(&m->dec_q, cx, sm, use_q8, s_out);               /* Eq. 4 */
    if (s_mid) memcpy(s_mid, sm, sizeof(float) * (size_t)H);
    if (alpha) memcpy(alpha, al, sizeof(float) * (size_t)l);
    if (ctx) memcpy(ctx, cx, sizeof(float) * (size_t)C);
    free(sm);
    free(a);
    free(al);
    free(cx);
}

void q8o_readout(const q8o_model *m, const float *s, const float *y_emb, const float *ctx,
                 int use_q8, float *t)
{
    int R = m->R;
    float *u1 = (float *)malloc(sizeof(float) * (size_t)R);
    float *u2 = (float *)malloc(sizeof(float) * (size_t)R);
    float *u3 = (float *)malloc(sizeof(float) * (size_t)R);
    q8o_linear ls = m->ro_s;
    const float *bt = ls.bias;
    ls.bias = NULL;                      /* b_t is added after the three products */
    q8o_linear_apply(&ls, s, use_q8, u1);
    q8o_linear_apply(&m->ro_y, y_emb, use_q8, u2);
    q8o_linear_apply(&m->ro_c, ctx, use_q8, u3);
    for (int i = 0; i < R; ++i) {
        float p = u1[i] + u2[i];
        p = p + u3[i];
        if (bt) p = p + bt[i];
        t[i] = tanh_f(p);
    }
    free(u1);
    free(u2);
    free(u3);
}

void q8o_logsoftmax_topk(const float *logits, int V, int k, float *lse, float *topk_logp, int32_t *topk_idx)
{
    float mx = logits[0];
    for (int i = 1; i < V; ++i)
        if (logits[i] > mx) mx = logits[i];
    double S = 0.0;
    for (int i = 0; i < V; ++i) S += exp((double)logits[i] - (double)mx);
    float L = (float)((double)mx + log(S));
    if (lse) *lse = L;
    /* k rounds of selection: each round takes the largest logit not yet taken,
     * the lowest index winning among equals. */
    for (int r = 0; r < k; ++r) {
        int best = -1;
        for (int i = 0; i < V; ++i) {
            int taken = 0;
            for (int p = 0; p < r; ++p)
                if (topk_idx[p] == i) { taken = 1; break; }
            if (taken) continue;
            if (best < 0 || logits[i] > logits[best]) best = i;
        }
        topk_idx[r] = best;
        topk_logp[r] = logits[best] - L;
    }
}

void q8o_output(const q8o_model *m, const float *t, int use_q8, int k,
                float *logits, float *lse, float *topk_logp, int32_t *topk_idx)
{
    int V = m->out.rows;
    float *lg = (float *)malloc(sizeof(float) * (size_t)V);
    q8o_linear_apply(&m->out, t, use_q8, lg);
    q8o_logsoftmax_topk(lg, V, k, lse, topk_logp, topk_idx);
    if (logits) memcpy(logits, lg, sizeof(float) * (size_t)V);
    free(lg);
}

/* ---------------------------------------------------------------- beam search -- */

typedef struct {
    float score;
    int parent;
    int token;
} cand_t;

/* order: score descending, then parent index ascending, then token id ascending */
static int cand_before(const cand_t *a, const cand_t *b)
{
    if (a->score != b->score) return a->score > b->score;
    if (a->parent != b->parent) return a->parent < b->parent;
    return a->token < b->token;
}

/* Ensemble decoding (Section 4: the English-German systems decode with two models): the
 * models' probabilities of the next word are averaged before the k best are taken,
 *   c[v] = log((1/M) sum_m exp(logp_m[v])),  logp_m[v] = logits_m[v] - lse_m,
 * evaluated in double and rounded once. */
void q8o_ensemble_logp(const float *const *logp, int M, int V, float *c)
{
    for (int v = 0; v < V; ++v) {
        double p = 0.0;
        for (int m = 0; m < M; ++m) p += exp((double)logp[m][v]);
        c[v] = (float)log(p / (double)M);
    }
}

/* The k largest entries of v by (value descending, index ascending). */
static void select_topk(const float *v, int V, int k, float *val, int32_t *idx)
{
    for (int r = 0; r < k; ++r) {
        int best = -1;
        for (int i = 0; i < V; ++i) {
            int taken = 0;
            for (int p = 0; p < r; ++p)
                if (idx[p] == i) { taken = 1; break; }
            if (taken) continue;
            if (best < 0 || v[i] > v[best]) best = i;
        }
        idx[r] = best;
        val[r] = v[best];
    }
}

/* Beam search over M models that share the target vocabulary (M = 1: one model, its own
 * top-k of log-probabilities).  Every model keeps its own encoder states, attention
 * pre-computation and decoder state per hypothesis; the search itself is common. */
int q8o_translate_ensemble(const q8o_model *const *ms, int M, const int32_t *src_tokens, int l, int beam, int topk,
                           int max_steps, int use_q8, int32_t *out_tokens, float *out_score, int *out_steps)
{
    const int V = ms[0]->out.rows;
    float **enc_h = (float **)malloc(sizeof(float *) * (size_t)M);
    float **P = (float **)malloc(sizeof(float *) * (size_t)M);
    float **s = (float **)malloc(sizeof(float *) * (size_t)M);
    float **s_new = (float **)malloc(sizeof(float *) * (size_t)M);
    float **s_step = (float **)malloc(sizeof(float *) * (size_t)M);
    float **logp = (float **)malloc(sizeof(float *) * (size_t)M);
    for (int m = 0; m < M; ++m) {
        const q8o_model *mo = ms[m];
        const int H = mo->H, E = mo->E, C = mo->C, A = mo->A;
        float *X = (float *)malloc(sizeof(float) * (size_t)l * E);
        enc_h[m] = (float *)malloc(sizeof(float) * (size_t)l * C);
        P[m] = (float *)malloc(sizeof(float) * (size_t)l * A);
        for (int i = 0; i < l; ++i)
            memcpy(X + (size_t)i * E, mo->E_src + (size_t)src_tokens[i] * E, sizeof(float) * (size_t)E);
        q8o_encode(mo, X, l, use_q8, enc_h[m]);
        q8o_attention_precompute(mo, enc_h[m], l, use_q8, P[m]);
        free(X);
        s[m] = (float *)calloc((size_t)beam * H, sizeof(float));
        s_new[m] = (float *)calloc((size_t)beam * H, sizeof(float));
        s_step[m] = (float *)malloc(sizeof(float) * (size_t)beam * H);
        logp[m] = (float *)malloc(sizeof(float) * (size_t)V);
        /* initial decoder state: the backward encoder state at the first source position */
        memcpy(s[m], enc_h[m], sizeof(float) * (size_t)H);
    }
    /* live hypotheses: last token, score, token history */
    int32_t *hist = (int32_t *)calloc((size_t)beam * max_steps, sizeof(int32_t));
    int32_t *hist_new = (int32_t *)calloc((size_t)beam * max_steps, sizeof(int32_t));
    int32_t *last = (int32_t *)calloc((size_t)beam, sizeof(int32_t));
    float *score = (float *)calloc((size_t)beam, sizeof(float));
    float *tk_logp = (float *)malloc(sizeof(float) * (size_t)beam * topk);
    int32_t *tk_idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)beam * topk);
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)beam * topk);
    float *comb = (float *)malloc(sizeof(float) * (size_t)V);

    int n_live = 1, b_live = beam;
    last[0] = 0;
    score[0] = 0.0f;

    int have_fin = 0, fin_len = 0;
    float fin_score = 0.0f;
    int32_t *fin_tokens = (int32_t *)calloc((size_t)max_steps, sizeof(int32_t));

    int steps = 0;
    for (int step = 0; step < max_steps && b_live > 0 && n_live > 0; ++step) {
        ++steps;
        for (int b = 0; b < n_live; ++b) {
            for (int m = 0; m < M; ++m) {
                const q8o_model *mo = ms[m];
                const int H = mo->H;
                float *ctx = (float *)malloc(sizeof(float) * (size_t)mo->C);
                float *t = (float *)malloc(sizeof(float) * (size_t)mo->R);
                const float *y = mo->E_tgt + (size_t)last[b] * mo->E;
                q8o_cgru_step(mo, P[m], enc_h[m], l, y, s[m] + (size_t)b * H, use_q8, NULL, NULL, ctx,
                              s_step[m] + (size_t)b * H);
                q8o_readout(mo, s_step[m] + (size_t)b * H, y, ctx, use_q8, t);
                if (M == 1) {
                    q8o_output(mo, t, use_q8, topk, NULL, NULL, tk_logp + (size_t)b * topk, tk_idx + (size_t)b * topk);
                } else {
                    float lse;
                    q8o_output(mo, t, use_q8, 0, logp[m], &lse, NULL, NULL);
                    for (int v = 0; v < V; ++v) logp[m][v] = logp[m][v] - lse;
                }
                free(ctx); free(t);
            }
            if (M > 1) {
                q8o_ensemble_logp((const float *const *)logp, M, V, comb);
                select_topk(comb, V, topk, tk_logp + (size_t)b * topk, tk_idx + (size_t)b * topk);
            }
        }
        int nc = n_live * topk;
        for (int b = 0; b < n_live; ++b)
            for (int j = 0; j < topk; ++j) {
                cand_t *c = &cand[b * topk + j];
                c->score = score[b] + tk_logp[b * topk + j];
                c->parent = b;
                c->token = tk_idx[b * topk + j];
            }
        /* selection sort of the first b_live candidates */
        int take = b_live < nc ? b_live : nc;
        for (int r = 0; r < take; ++r) {
            int best = r;
            for (int i = r + 1; i < nc; ++i)
                if (cand_before(&cand[i], &cand[best])) best = i;
            cand_t tmp = cand[r];
            cand[r] = cand[best];
            cand[best] = tmp;
        }
        int n_new = 0;
        for (int r = 0; r < take; ++r) {
            const cand_t *c = &cand[r];
            if (c->token == 0) {         /* hypothesis ends */
                if (!have_fin || c->score > fin_score) {
                    have_fin = 1;
                    fin_score = c->score;
                    fin_len = step;
                    memcpy(fin_tokens, hist + (size_t)c->parent * max_steps, sizeof(int32_t) * (size_t)step);
                }
                --b_live;
            } else {
                memcpy(hist_new + (size_t)n_new * max_steps, hist + (size_t)c->parent * max_steps,
                       sizeof(int32_t) * (size_t)step);
                hist_new[(size_t)n_new * max_steps + step] = c->token;
                for (int m = 0; m < M; ++m) {
                    const int H = ms[m]->H;
                    memcpy(s_new[m] + (size_t)n_new * H, s_step[m] + (size_t)c->parent * H, sizeof(float) * (size_t)H);
                }
                last[n_new] = c->token;
                score[n_new] = c->score;
                ++n_new;
            }
        }
        /* `last` and `score` were overwritten in place: entries [0,n_new) only depend
         * on cand[], which was copied before, so this is safe. */
        for (int m = 0; m < M; ++m) { float *tmpf = s[m]; s[m] = s_new[m]; s_new[m] = tmpf; }
        int32_t *tmpi = hist; hist = hist_new; hist_new = tmpi;
        n_live = n_new;
    }

    int n_out;
    if (have_fin) {
        n_out = fin_len;
        memcpy(out_tokens, fin_tokens, sizeof(int32_t) * (size_t)n_out);
        *out_score = fin_score;
    } else {
        n_out = steps;
        memcpy(out_tokens, hist, sizeof(int32_t) * (size_t)n_out);
        *out_score = n_live > 0 ? score[0] : 0.0f;
    }
    if (out_steps) *out_steps = steps;

    for (int m = 0; m < M; ++m) { free(enc_h[m]); free(P[m]); free(s[m]); free(s_new[m]); free(s_step[m]); free(logp[m]); }
    free(enc_h); free(P); free(s); free(s_new); free(s_step); free(logp);
    free(hist); free(hist_new); free(last); free(score); free(tk_logp); free(tk_idx); free(cand); free(comb);
    free(fin_tokens);
    return n_out;
}

int q8o_translate(const q8o_model *m, const int32_t *src_tokens, int l, int beam, int topk,
                  int max_steps, int use_q8, int32_t *out_tokens, float *out_score, int *out_steps)
{
    return q8o_translate_ensemble(&m, 1, src_tokens, l, beam, topk, max_steps, use_q8, out_tokens, out_score, out_steps);
}
