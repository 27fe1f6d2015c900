/*
 * q8_oracle_selftest.c -- drives every function of the CPU oracle once on a small seeded model.
 * TEST INFRASTRUCTURE ONLY.  Built together with q8_oracle.c under
 * -fsanitize=address,undefined (tests/test_oracle_sanitized.py), it shows that the oracle reads
 * and writes inside its buffers and has no undefined arithmetic on ordinary inputs; it also
 * checks a few invariants (probabilities sum to one, the narrow product is the vector product
 * column by column) so that a run that computes nothing does not pass.  Exit status 0 = clean.
 */
#include "q8_oracle.h"

#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static unsigned long long g_state = 0x9E3779B97F4A7C15ull;

static float rnd(void)                     /* uniform in (-1, 1), a 64-bit LCG */
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(g_state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}

static float *randv(size_t n, float amp)
{
    float *p = (float *)malloc(sizeof(float) * n);
    for (size_t i = 0; i < n; ++i) p[i] = amp * rnd();
    return p;
}

static int pad16(int n) { return (n + 15) / 16 * 16; }

/* a linear map with exactly sized buffers, so that any access past an end is caught */
static q8o_linear make_linear(int rows, int cols, int with_bias, float amp)
{
    q8o_linear L;
    float *Wf = randv((size_t)rows * cols, amp);
    int ld = pad16(cols);
    int8_t *Wq = (int8_t *)malloc((size_t)rows * ld);
    float s;
    q8o_quantize_matrix(Wf, rows, cols, cols, Wq, ld, &s);
    L.rows = rows; L.cols = cols; L.Wf = Wf; L.ldf = cols; L.Wq = Wq; L.ldq = ld; L.scale = s;
    L.bias = with_bias ? randv((size_t)rows, 0.1f) : NULL;
    return L;
}

static void free_linear(q8o_linear *L)
{
    free((void *)L->Wf); free((void *)L->Wq); free((void *)L->bias);
}

static q8o_gru make_gru(int I, int H)
{
    q8o_gru g;
    g.Wx = make_linear(3 * H, I, 1, 0.5f);
    g.Wh = make_linear(3 * H, H, 1, 0.5f);
    return g;
}

static q8o_model make_model(int V, int E, int H, int A, int R)
{
    q8o_model m;
    memset(&m, 0, sizeof(m));
    m.V_src = V; m.V_tgt = V; m.E = E; m.H = H; m.C = 2 * H; m.A = A; m.R = R;
    m.E_src = randv((size_t)V * E, 1.0f);
    m.E_tgt = randv((size_t)V * E, 1.0f);
    m.enc_fwd = make_gru(E, H);
    m.enc_bwd = make_gru(E, H);
    m.att_W = make_linear(A, 2 * H, 1, 0.5f);
    m.att_U = make_linear(A, H, 0, 0.5f);
    m.att_v = randv((size_t)A, 0.5f);
    m.dec_r = make_gru(E, H);
    m.dec_q = make_gru(2 * H, H);
    m.ro_s = make_linear(R, H, 1, 0.5f);
    m.ro_y = make_linear(R, E, 0, 0.5f);
    m.ro_c = make_linear(R, 2 * H, 0, 0.5f);
    m.out = make_linear(V, R, 1, 0.8f);
    ((float *)m.out.bias)[0] += 0.5f;       /* some hypotheses end */
    return m;
}

static void free_model(q8o_model *m)
{
    free((void *)m->E_src); free((void *)m->E_tgt); free((void *)m->att_v);
    q8o_linear *ls[] = {&m->enc_fwd.Wx, &m->enc_fwd.Wh, &m->enc_bwd.Wx, &m->enc_bwd.Wh, &m->att_W, &m->att_U,
                        &m->dec_r.Wx, &m->dec_r.Wh, &m->dec_q.Wx, &m->dec_q.Wh, &m->ro_s, &m->ro_y, &m->ro_c, &m->out};
    for (size_t i = 0; i < sizeof(ls) / sizeof(ls[0]); ++i) free_linear(ls[i]);
}

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "selftest: %s failed (line %d)\n", #cond, __LINE__); return 1; } } while (0)

int main(void)
{
    /* odd sizes on purpose: nothing is a multiple of 16 */
    const int V = 23, E = 7, H = 9, A = 5, R = 6, l = 4, C = 2 * H;
    q8o_model m = make_model(V, E, H, A, R), m2 = make_model(V, E + 2, H + 1, A + 1, R + 3);

    /* Section 3 */
    {
        const int rows = 11, cols = 19, n = 3;
        q8o_linear L = make_linear(rows, cols, 1, 1.0f);
        float *X = randv((size_t)n * cols, 2.0f), *Y = (float *)malloc(sizeof(float) * n * rows), *y1 = (float *)malloc(sizeof(float) * rows);
        int8_t *xq = (int8_t *)malloc((size_t)n * cols);
        float *xs = (float *)malloc(sizeof(float) * n);
        int32_t *acc = (int32_t *)malloc(sizeof(int32_t) * n * rows);
        q8o_gemm_narrow(&L, X, n, cols, Y, rows, xq, xs, acc);
        for (int j = 0; j < n; ++j) {
            q8o_gemv(&L, X + (size_t)j * cols, y1, NULL, NULL, NULL);
            CHECK(memcmp(y1, Y + (size_t)j * rows, sizeof(float) * rows) == 0);
        }
        q8o_gemv_fp32(&L, X, y1);
        for (int i = 0; i < rows; ++i) CHECK(fabsf(y1[i] - Y[i]) < 0.5f);
        int8_t *Wr = (int8_t *)malloc((size_t)rows * pad16(cols));
        float *rs = (float *)malloc(sizeof(float) * rows);
        q8o_quantize_matrix_rows(L.Wf, rows, cols, cols, Wr, pad16(cols), rs);
        q8o_gemm_narrow_rows(Wr, rows, cols, pad16(cols), rs, L.bias, X, n, cols, Y, rows, xq, xs, acc);
        for (int i = 0; i < rows; ++i) CHECK(fabsf(y1[i] - Y[i]) < 0.5f);
        float zero[5] = {0, 0, 0, 0, 0}, sc;
        int8_t zq[5];
        q8o_quantize(zero, 5, zq, &sc);
        CHECK(sc == 1.0f && zq[0] == 0 && zq[4] == 0);
        free(X); free(Y); free(y1); free(xq); free(xs); free(acc); free(Wr); free(rs);
        free_linear(&L);
    }

    /* Section 2, stage by stage */
    int32_t src[4] = {3, 22, 1, 7};
    float *X = (float *)malloc(sizeof(float) * l * E);
    for (int i = 0; i < l; ++i) memcpy(X + (size_t)i * E, m.E_src + (size_t)src[i] * E, sizeof(float) * E);
    float *enc = (float *)malloc(sizeof(float) * l * C), *P = (float *)malloc(sizeof(float) * l * A);
    for (int q8 = 0; q8 < 2; ++q8) {
        q8o_encode(&m, X, l, q8, enc);
        q8o_attention_precompute(&m, enc, l, q8, P);
        float *s_mid = (float *)malloc(sizeof(float) * H), *alpha = (float *)malloc(sizeof(float) * l);
        float *ctx = (float *)malloc(sizeof(float) * C), *s = (float *)malloc(sizeof(float) * H), *t = (float *)malloc(sizeof(float) * R);
        q8o_cgru_step(&m, P, enc, l, m.E_tgt, enc, q8, s_mid, alpha, ctx, s);
        double sum = 0.0;
        for (int i = 0; i < l; ++i) sum += alpha[i];
        CHECK(fabs(sum - 1.0) < 1e-5);
        q8o_readout(&m, s, m.E_tgt, ctx, q8, t);
        float *logits = (float *)malloc(sizeof(float) * V), lse, lp[V];
        int32_t idx[V];
        q8o_output(&m, t, q8, V, logits, &lse, lp, idx);
        sum = 0.0;
        for (int i = 0; i < V; ++i) sum += exp((double)lp[i]);
        CHECK(fabs(sum - 1.0) < 1e-5);
        for (int i = 1; i < V; ++i) CHECK(lp[i] <= lp[i - 1]);
        free(s_mid); free(alpha); free(ctx); free(s); free(t); free(logits);
    }

    /* the attention variant with 8-bit activation products */
    {
        float *a = randv((size_t)A, 1.0f), *e = (float *)malloc(sizeof(float) * l), *alpha = (float *)malloc(sizeof(float) * l);
        float *ctx = (float *)malloc(sizeof(float) * C), *hT = (float *)malloc(sizeof(float) * C * l);
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < l; ++i) hT[(size_t)c * l + i] = enc[(size_t)i * C + c];
        int8_t *vq = (int8_t *)malloc((size_t)A), *hTq = (int8_t *)malloc((size_t)C * pad16(l));
        float s_v, s_h;
        q8o_quantize_matrix(m.att_v, 1, A, A, vq, A, &s_v);
        q8o_quantize_matrix(hT, C, l, l, hTq, pad16(l), &s_h);
        q8o_attention_q8(P, l, A, a, vq, s_v, hTq, C, pad16(l), s_h, e, alpha, ctx);
        double sum = 0.0;
        for (int i = 0; i < l; ++i) sum += alpha[i];
        CHECK(fabs(sum - 1.0) < 1e-5);
        free(a); free(e); free(alpha); free(ctx); free(hT); free(vq); free(hTq);
    }

    /* searches: every beam width below 8, k from beam to V, both engines, and an ensemble */
    for (int beam = 1; beam <= 7; ++beam) {
        const int max_steps = 6, k = beam + (beam % 3) > V ? V : beam + (beam % 3);
        int32_t *out = (int32_t *)malloc(sizeof(int32_t) * max_steps);
        float score;
        int steps;
        int n = q8o_translate(&m, src, l, beam, k, max_steps, beam & 1, out, &score, &steps);
        CHECK(n >= 0 && n <= max_steps && steps >= 1 && steps <= max_steps && score <= 0.0f);
        for (int i = 0; i < n; ++i) CHECK(out[i] > 0 && out[i] < V);
        free(out);
    }
    {
        const q8o_model *both[2] = {&m, &m2};
        const int max_steps = 5;
        int32_t out[5];
        float score;
        int steps;
        int n = q8o_translate_ensemble(both, 2, src, l, 3, 4, max_steps, 1, out, &score, &steps);
        CHECK(n >= 0 && n <= max_steps && score <= 0.0f);
    }
    CHECK(q8o_nonfinite_count(1) == 0);
    float bad[2] = {1.0f, NAN}, sc;
    int8_t bq[2];
    q8o_quantize(bad, 2, bq, &sc);
    CHECK(q8o_nonfinite_count(1) == 1 && q8o_nonfinite_count(0) == 0);

    free(X); free(enc); free(P);
    free_model(&m);
    free_model(&m2);
    puts("q8 oracle selftest: ok");
    return 0;
}
