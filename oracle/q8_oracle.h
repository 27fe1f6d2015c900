/*
 * q8_oracle.h -- CPU oracle for 8-bit GRU-NMT decoding.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar C implementation of the method of "Pieces of Eight: 8-bit
 * Neural Machine Translation" (Quinn & Ballesteros): Section 3 (8-bit operands,
 * integer accumulation, 32-bit float result, one routine for matrix x vector and
 * matrix x narrow matrix, bias / tanh / sigmoid kept in float) applied to the
 * model of Section 2 (Eq. 1-6).  It exists so that the GPU library can be checked
 * against something that can be compared with the paper by eye.  It shares no
 * code with the GPU path and must never be called from it: only the test-suite,
 * the smoke check and the benchmark's cpu_baseline leg may load this library.
 *
 * Precision: the paper fixes the precision of the data (8-bit operands, 32-bit
 * float results), so every stored value is an IEEE fp32 `float`, every integer
 * sum is an exact int32, float arithmetic is written one operation per statement
 * (compile with -ffp-contract=off), and transcendental functions and long float
 * sums are evaluated in double and rounded once to float.
 *
 * Readings where Section 3 leaves the scheme open are listed with each function
 * (symmetric max-abs scale, codes in [-127,127], round-half-to-even, one scale per
 * weight matrix, one scale per activation vector).
 *
 * Pins: every function below is pinned by tests/test_oracle_*.py (closed forms,
 * brute force, library special cases).  End-to-end translations against the
 * paper's trained systems (its Tables 3, 6-9): parity unpinned (no weights, no
 * test sets).
 */
#ifndef Q8_ORACLE_H
#define Q8_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A trained linear map y = W x + b in both of its stored forms. */
typedef struct {
    int rows, cols;
    const float *Wf;    /* fp32 weights, row-major [rows x ldf]; used by the 32-bit engine */
    int ldf;
    const int8_t *Wq;   /* int8 image of Wf, row-major [rows x ldq], pad columns zero */
    int ldq;
    float scale;        /* Wf ~= scale * Wq */
    const float *bias;  /* [rows] or NULL */
} q8o_linear;

typedef struct {        /* one GRU cell: gate row blocks in the order r, z, n */
    q8o_linear Wx;      /* [3H x I] */
    q8o_linear Wh;      /* [3H x H] */
} q8o_gru;

typedef struct {
    int V_src, V_tgt, E, H, C, A, R;     /* C = 2H */
    const float *E_src;                  /* [V_src x E] fp32, gather only */
    const float *E_tgt;                  /* [V_tgt x E] */
    q8o_gru enc_fwd, enc_bwd;            /* Eq. 1 */
    q8o_linear att_W;                    /* w: [A x C], bias b_att   (Eq. 6) */
    q8o_linear att_U;                    /* u: [A x H], no bias      (Eq. 6) */
    const float *att_v;                  /* v: [A] fp32              (Eq. 6) */
    q8o_gru dec_r, dec_q;                /* Eq. 3, Eq. 4: r is [3H x E],[3H x H]; q is [3H x C],[3H x H] */
    q8o_linear ro_s, ro_y, ro_c;         /* first layer of g (Eq. 2): [R x H], [R x E], [R x C]; bias b_t on ro_s */
    q8o_linear out;                      /* second layer of g: [V_tgt x R], bias b_out */
} q8o_model;

/* Non-finite inputs (NaN, +-inf) have no 8-bit code and the method says nothing about
 * them: the oracle defines no result for them.  Every vector or matrix that enters a
 * product (q8o_quantize, q8o_quantize_matrix, q8o_gemv_fp32, and so everything built on
 * them) is checked, and the number of non-finite elements seen since the last reset is
 * returned here; the Python front-end raises FloatingPointError when it is not zero.
 * Not thread-safe beyond a lost count. */
long q8o_nonfinite_count(int reset);

/* ---- Section 3: the 8-bit product, step by step -------------------------------- */

/* O1. Symmetric max-abs quantization of one vector.  m = max|v_i|.  If m < 2^-100
 * (which covers the zero vector): scale = 1, all codes 0.  Otherwise scale = m/127,
 * inv = 127/m (two fp32 divisions), code_i = clamp(rint(v_i * inv), -127, 127) with
 * round-half-to-even.  -128 is never produced. */
void q8o_quantize(const float *v, int n, int8_t *q, float *scale);

/* O1 for a weight matrix: one scale for the whole [rows x cols] matrix; the
 * ld_out - cols pad bytes of every output row are set to zero. */
void q8o_quantize_matrix(const float *W, int rows, int cols, int ld_in,
                         int8_t *Wq, int ld_out, float *scale);

/* O2. Exact integer accumulation: acc_i = sum_k Wq[i,k] * xq[k] in int32. */
void q8o_accumulate(const int8_t *Wq, int rows, int cols, int ld, const int8_t *xq, int32_t *acc);

/* O3. The 32-bit float result: c = s_w * s_x (one fp32 multiply),
 * y_i = (float)acc_i * c, then y_i = y_i + bias_i as a separate add if bias != NULL. */
void q8o_dequantize(const int32_t *acc, int rows, float s_w, float s_x, const float *bias, float *y);

/* O1+O2+O3 for one vector.  tap_* are optional (NULL) outputs of the intermediate
 * integer tensors: xq [cols], xscale [1], acc [rows]. */
void q8o_gemv(const q8o_linear *L, const float *x, float *y,
              int8_t *tap_xq, float *tap_xscale, int32_t *tap_acc);

/* The same routine on a narrow matrix: n vectors X [n x ldx] -> Y [n x ldy]; each
 * vector has its own scale, so the result equals n separate q8o_gemv calls. */
void q8o_gemm_narrow(const q8o_linear *L, const float *X, int n, int ldx, float *Y, int ldy,
                     int8_t *tap_xq, float *tap_xscale, int32_t *tap_acc);

/* Variant of O1-O3 with one weight scale per ROW (Section 3 does not state the granularity
 * of the scale; the per-matrix reading is the default everywhere else).  Row i of W is
 * quantized as a vector of its own: m_i = max_k |W[i,k]|, the rules of O1 with m_i, codes
 * into Wq row i (pad bytes zero), scale into row_scale[i]. */
void q8o_quantize_matrix_rows(const float *W, int rows, int cols, int ld_in,
                              int8_t *Wq, int ld_out, float *row_scale);

/* O3 with per-row weight scales: c_i = row_scale[i] * s_x (one fp32 multiply per row),
 * y_i = (float)acc_i * c_i, then + bias_i as a separate add if bias != NULL. */
void q8o_dequantize_rows(const int32_t *acc, int rows, const float *row_scale, float s_x,
                         const float *bias, float *y);

/* The narrow product with per-row weight scales: per vector j, O1 on X[j], O2, then
 * q8o_dequantize_rows.  Taps as in q8o_gemm_narrow (NULL to skip). */
void q8o_gemm_narrow_rows(const int8_t *Wq, int rows, int cols, int ld, const float *row_scale,
                          const float *bias, const float *X, int n, int ldx, float *Y, int ldy,
                          int8_t *tap_xq, float *tap_xscale, int32_t *tap_acc);

/* The 32-bit engine's product: y_i = (float)(sum_k (double)W[i,k]*(double)x[k]), then + bias. */
void q8o_gemv_fp32(const q8o_linear *L, const float *x, float *y);

/* Either engine: use_q8 != 0 selects q8o_gemv, else q8o_gemv_fp32. */
void q8o_linear_apply(const q8o_linear *L, const float *x, int use_q8, float *y);

/* ---- Section 2: the model ------------------------------------------------------ */

/* O4 (gates).  gx, gh are the two pre-activation vectors [3H] (biases included),
 * row blocks r, z, n.  r = sigmoid(gx_r + gh_r); z = sigmoid(gx_z + gh_z);
 * n = tanh(gx_n + r * gh_n); h' = (1 - z) * n + z * h.  (GRU cell of Cho et al.,
 * which Eq. 1 and Eq. 3-4 use; reset gate applied after the recurrent product.) */
void q8o_gru_gates(const float *gx, const float *gh, const float *h_prev, int H, float *h_out);

/* O4.  One GRU step: gx = Wx q(x) + bx, gh = Wh q(h) + bh (two separate
 * quantizations), then the gates.  The state mixed in by z is the fp32 h_prev. */
void q8o_gru_step(const q8o_gru *g, const float *x, const float *h_prev, int use_q8, float *h_out);

/* O5 (Eq. 1).  Bidirectional encoder over embeddings X [l x E]; writes
 * enc_h [l x 2H] with the backward state in columns [0,H) and the forward state
 * in [H,2H), as Eq. 1 stacks them.  Both recurrences start from the zero state. */
void q8o_encode(const q8o_model *m, const float *X, int l, int use_q8, float *enc_h);

/* O6 (Eq. 6, the part without t).  P_i = w(h_i) + b_att for every source position: P [l x A]. */
void q8o_attention_precompute(const q8o_model *m, const float *enc_h, int l, int use_q8, float *P);

/* O7 attention core (Eq. 5-6), all in float: e_i = sum_j v_j * tanh(P_ij + a_j)
 * (each tanh rounded to float, the sum kept in double, e_i rounded to float);
 * alpha = softmax(e) with the maximum subtracted (double, rounded per element);
 * ctx_c = sum_i alpha_i * h_i[c] (double sum, rounded).  e_out may be NULL. */
void q8o_attention(const float *P, const float *enc_h, int l, int A, int C,
                   const float *a, const float *v, float *e_out, float *alpha, float *ctx);

/* Variant of the attention core in which the two products of Eq. 5-6 that involve no trained
 * matrix also go through O1-O3 (the other reading of "the matrix products are 8-bit"; the
 * default keeps them in float).
 *   energies: T_i = tanh(P_i + a) (each element rounded to float) is the activation vector of
 *     position i, (Tq_i, s_Ti) = O1(T_i); v is a 1 x A weight matrix (vq, s_v), quantized once
 *     by O1's matrix rule; e_i = (float)(vq . Tq_i) * (s_v * s_Ti)        [O2, O3, no bias]
 *   alpha = softmax(e) exactly as in q8o_attention
 *   context: the C x l matrix of encoder states transposed, hTq [C x ldq] with one scale s_h
 *     (O1's matrix rule, once per sentence), times the vector alpha: (aq, s_a) = O1(alpha);
 *     ctx_c = (float)(sum_i hTq[c,i] * aq_i) * (s_h * s_a)                 [O2, O3, no bias]
 * e_out may be NULL. */
void q8o_attention_q8(const float *P, int l, int A, const float *a, const int8_t *vq, float s_v,
                      const int8_t *hTq, int C, int ldq, float s_h,
                      float *e_out, float *alpha, float *ctx);

/* O7 (Eq. 3-6).  One conditional-GRU step for one hypothesis:
 * s' = r(y, s_prev); a = u(q(s')); attention -> H_t; s = q(H_t, s').
 * Outputs: s_mid [H] (= s'), alpha [l], ctx [C] (= H_t), s_out [H]; any may be NULL except s_out. */
void q8o_cgru_step(const q8o_model *m, const float *P, const float *enc_h, int l,
                   const float *y_emb, const float *s_prev, int use_q8,
                   float *s_mid, float *alpha, float *ctx, float *s_out);

/* O8 first layer of g (Eq. 2): t = tanh(((ro_s q(s) + ro_y q(y)) + ro_c q(ctx)) + b_t). */
void q8o_readout(const q8o_model *m, const float *s, const float *y_emb, const float *ctx,
                 int use_q8, float *t);

/* O8 softmax / top-k over one logit vector: lse = max + log(sum exp(x - max)) in
 * double, rounded; the k best entries are the k largest logits ordered by (logit
 * descending, index ascending); their log-probability is logit - lse (one fp32
 * subtraction).  Requires k <= V. */
void q8o_logsoftmax_topk(const float *logits, int V, int k, float *lse, float *topk_logp, int32_t *topk_idx);

/* O8.  Full output layer for one hypothesis from t [R]; logits may be NULL. */
void q8o_output(const q8o_model *m, const float *t, int use_q8, int k,
                float *logits, float *lse, float *topk_logp, int32_t *topk_idx);

/* O9.  Beam search translation of one sentence.  Token 0 is BOS and EOS.
 * Returns the number of target tokens written to out_tokens (EOS excluded, at most
 * max_steps); *out_score is the winning cumulative log-probability; *out_steps the
 * number of decoder steps executed (each step runs one cGRU + output pass per live
 * hypothesis).  scratch-free: allocates with malloc and frees before returning. */
int q8o_translate(const q8o_model *m, const int32_t *src_tokens, int l, int beam, int topk,
                  int max_steps, int use_q8, int32_t *out_tokens, float *out_score, int *out_steps);

/* Ensemble of M models that share the target vocabulary (Section 4: the English-German
 * systems decode with two models).  The models' next-word probabilities are averaged
 * before the k best are taken: c[v] = log((1/M) sum_m exp(logp_m[v])) with
 * logp_m[v] = logits_m[v] - lse_m (fp32), the average evaluated in double and rounded
 * once; candidates are ordered by (c descending, index ascending).  Every model has its
 * own encoder states, attention pre-computation and decoder state per hypothesis; the
 * search is O9's.  M = 1 is q8o_translate. */
void q8o_ensemble_logp(const float *const *logp, int M, int V, float *c);
int q8o_translate_ensemble(const q8o_model *const *ms, int M, const int32_t *src_tokens, int l, int beam, int topk,
                           int max_steps, int use_q8, int32_t *out_tokens, float *out_score, int *out_steps);

#ifdef __cplusplus
}
#endif
#endif
