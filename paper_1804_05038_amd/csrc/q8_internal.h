// q8_internal.h -- host-side context and the launcher interface between the C ABI
// (q8_api.cpp) and the kernels (the .hip files beside it).  Not part of the public interface.
#pragma once

#include <hip/hip_runtime.h>
#ifdef __HIPCC__
#include <hip/hip_ext.h>
#endif
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "q8nmt.h"
#ifdef __HIPCC__
#include "q8_device.h"
#endif

// Workspace header, zeroed by q8_create and zero again after every call that uses it: one attention
// arrival counter per hypothesis in [0, 4096); scratch slots (max bits, scale) at 6144; the flags of waits that gave up; from 8192 the exchange words of the attention kernel without
// a finishing block (2 KiB per hypothesis), at 24576 those of the selection kernel that runs the
// search step, from 32768 those of the one-launch panel GRU.
#define Q8_MAX_BEAM 8
#define Q8_MAX_COLS 1024            // vectors of one batched call
#define Q8_WS_HEADER 262144
#define Q8_GATE_PAUSE_DEFAULT 8      // sleeps of about 0.45 us of the blocks that wait for the search step's decision, before their first poll
                                     // (0 to 14 measured alike; later than that the first poll comes after the decision)
#define Q8_WS_SCRATCH_SLOT 6144
#define Q8_WS_ENC_ERR 6208          // set to 1 by the one-launch encoder if a wait gave up (zeroed before each such launch)
#define Q8_WS_ATT_ERR 6212          // the same for the attention kernel whose blocks wait for each other
#define Q8_WS_ATT_XCHG 8192
#define Q8_WS_ATT_XCHG_PER_HYP 2048
#define Q8_WS_SELECT_XCHG 24576      // 128 words: the top-k entries on their way to the search step
#define Q8_WS_GRUP_XCHG 32768        // 2 x 10752 words: partial maxima of the one-launch panel GRU (two regions that take turns)
#define Q8_WS_GATES_XCHG 118784      // 64 x 8 words: the search step's decision on its way to the blocks that compute the next GRU r
#define Q8_WS_PSEL_XCHG 131072       // 1024 x 16 8-byte words: the same hand-over for a panel of slots (sentences side by side)
#define Q8_ENC_SPIN_DEFAULT (1 << 20)

struct q8_ctx {
    hipStream_t stream;
    char *ws;
    size_t ws_bytes;
    char err[256];
    // kernel timing (q8_profile_begin / q8_profile_end): event pairs attached to dispatches
    hipEvent_t *prof_ev;
    int prof_cap, prof_n, prof_kind;
    // bytes at the top of the workspace held by a composite call (q8_translate) while it
    // issues other calls, which carve from the bottom
    size_t ws_reserved_top;
    // q8_encode: the recurrence in one cooperative launch where possible (q8_encoder_options), and the
    // bound of its internal waits in polls
    int enc_one_launch, enc_spin_limit;
    // attention of one sentence: the form whose blocks exchange energies and finish their own slices
    // (q8_attention_options), the bound of its waits in polls, and how many of its blocks the device
    // holds at once (-1: not asked yet)
    int att_split, att_spin_limit, att_capacity;
    // that form leaves its exchange words set; the GRU that follows it in the step clears them.  1 while
    // a launch's words are waiting for that (the next attention launch would clear them itself first).
    int att_words_set;
    // one-launch panel GRU: unit groups whose exchange words a launch has left set in each of the two regions
    // (0: the region is clear); the launch after it clears them, see q8i_gru_panel
    int grup_used[2];
    // the decoding loop whose GRU r runs ahead (output_logits_beam_ahead_q8): short sleeps of the blocks that
    // wait for the search step's decision before their first poll
    int gate_pause;
};

// Launch of a kernel of class `kind` (a Q8_KERNEL_* value).  While a profile of that class
// is open the dispatch carries an event pair that takes the kernel's own begin and end
// timestamps; otherwise it is an ordinary launch.
#define Q8_LAUNCH(ctx, kind, kernel, grid, block, smem, ...)                                                   \
    do {                                                                                                       \
        q8_ctx *c_ = (ctx);                                                                                    \
        if (c_->prof_ev && c_->prof_kind == (kind) && c_->prof_n < c_->prof_cap) {                             \
            hipEvent_t e0_ = c_->prof_ev[2 * c_->prof_n], e1_ = c_->prof_ev[2 * c_->prof_n + 1];               \
            ++c_->prof_n;                                                                                      \
            hipExtLaunchKernelGGL(kernel, grid, block, smem, c_->stream, e0_, e1_, 0, __VA_ARGS__);            \
        } else {                                                                                               \
            hipLaunchKernelGGL(kernel, grid, block, smem, c_->stream, __VA_ARGS__);                            \
        }                                                                                                      \
    } while (0)

static inline q8_status q8_fail(q8_ctx *ctx, q8_status code, const char *fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

struct q8i_gemv_desc {
    const q8_mat *W;
    const float *X;
    int ldx;
    const float *bias;
    float *Y;
    int ldy;
    const q8_taps *taps;
    const float *row_scale;     // NULL: W->scale; else one weight scale per row (device)
};

struct q8i_gru_desc {
    const q8_gru_weights *g;
    const float *x;      int ldx;
    const float *h_prev; int ldh;
    const float *g_pre;  int ldg;
    float *h_out;        int ldo;
    const q8_taps *taps; // NULL or [2]
    // may be NULL: codes [n x Wx.ld] (pad bytes zero) and scales [n] of x, left by its producer: used with
    // GH_PRE, and with FULL if hq_pre / hs_pre (the same for h_prev, [n x Wh.ld]) are there too
    const int8_t *xq_pre;
    const float *xs_pre;
    // not GX_PRE, may be NULL: where the codes [n x Wx.ld] and scales [n] of x are left for a later consumer
    int8_t *xq_out;
    float *xs_out;
    // of the first job, may be NULL: 8-byte words the kernel zeroes on its way out
    unsigned long long *clear;
    int clear_words;
    const int8_t *hq_pre;
    const float *hs_pre;
};

// beam update run by the last block of the selection kernel (NULL = none)
struct q8i_beam_desc {
    void *state;
    const float *s_step, *E_tgt;
    float *y_emb, *s_next;
    int E, H;
    // optional, all or none: the codes of the gathered rows travel with them (see BeamUpdateArgs)
    const int8_t *Eq, *sq_in;
    const float *Es, *ss_in;
    int8_t *yq_out, *sq_out;
    float *ys_out, *ss_out;
    int ldy, lds;
    // optional, all or none: GRU r of the next step (Eq. 3) computed in the selection kernel's launch from the
    // decision (see out_select_kernel): W_x^r q(E_tgt[v]) + b_x for every token [V x 3H]; the weights of GRU r, whose
    // recurrent product W_h^r q(s_step[j]) + b_h [n x 3H] the readout's launch makes (gh_r: where it is, set by the
    // output layer); and where s' of the next step goes [n x H]
    const float *gx_table, *gh_r;
    const q8_gru_weights *gru_r;
    float *s_mid_next;
};

// Search steps of several sentences side by side: sentence s owns slots [s beam, (s + 1) beam) of every
// per-hypothesis table.
struct BeamBatchArgs {
    char *states;
    size_t stride;               // bytes between the states of consecutive sentences
    const float *topk_logp;
    const int *topk_idx;
    const float *s_step, *E_tgt;
    float *y_emb, *s_next;
    int *done;                   // [S]: 1 once the sentence's search is over
    const float *enc_h;          // initialization: encoder states, sentence s starts at row sent_off[s]
    const int *sent_off;
    int beam, k, E, H, C, max_steps;
    int V;                       // rows of E_tgt when known (token ids are then kept inside the table), else 0
    // optional, all or none (see BeamUpdateArgs): the codes of the gathered rows travel with them; the per-slot
    // tables are those of all sentences, slot-major like y_emb and s_next
    const int8_t *Eq, *sq_in;
    const float *Es, *ss_in;
    int8_t *yq_out, *sq_out;
    float *ys_out, *ss_out;
    int ldy, lds;
};

enum { Q8I_GRU_FULL = 0, Q8I_GRU_GX_PRE = 1, Q8I_GRU_GH_PRE = 2 };

q8_status q8i_fill_u32(q8_ctx *ctx, void *p, int n, unsigned v);   // fill kernel (safe under graph capture)
q8_status q8i_quantize_matrix(q8_ctx *ctx, const float *W, int rows, int cols, int ld_in, int8_t *Wq, int ld_out,
                              float *scale_host);
q8_status q8i_gemv_jobs(q8_ctx *ctx, const q8i_gemv_desc *d, int njobs, int n);
q8_status q8i_gemm_mfma(q8_ctx *ctx, const q8_mat *W, const float *X, int n, int ldx, const float *bias, float *Y,
                        int ldy, const q8_taps *taps, int8_t *xq, float *xscale, const float *row_scale = nullptr);
q8_status q8i_quantize_matrix_rows(q8_ctx *ctx, const float *W, int rows, int cols, int ld_in, int8_t *Wq, int ld_out,
                                   float *row_scale);
struct q8i_quant_job {          // quantization of n vectors X [n x ldx] (K floats each) into xq [n x ld], xscale [n]
    const float *X;
    int K, ldx, ld;
    int8_t *xq;
    float *xscale;
    const q8_taps *taps;
};
struct q8i_gemm_job {           // Y [n x ldy] = dequantize(W . xq) + bias on the matrix cores
    const q8_mat *W;
    const int8_t *xq;
    const float *xscale;
    const float *bias;
    float *Y;
    int ldy;
    int32_t *tap_acc;
    float *part_max;            // vocabulary layer: per-tile softmax statistics [n x ceil(rows / 16)]
    double *part_sum;
    int tiled;                  // 1: Y is written as [ceil(rows / 16)][n][16] (needs that many floats)
    const float *row_scale;     // NULL: W->scale; else one weight scale per row (plain output without statistics only)
};
q8_status q8i_quantize_jobs(q8_ctx *ctx, const q8i_quant_job *d, int njobs, int n);   // njobs <= 3
q8_status q8i_gemm_jobs(q8_ctx *ctx, const q8i_gemm_job *d, int njobs, int n);        // njobs <= 3
// three products with rows of 1024 / 512 / 2048 bytes (the readout's) over the same vectors in one K-resident launch
bool q8i_gemm_ksplit3_ok(const q8i_gemm_job *d, int n);
q8_status q8i_gemm_ksplit3(q8_ctx *ctx, const q8i_gemm_job *d, int n);
// up to two products with rows of 1024 bytes over at most 336 vectors, k split over pairs of waves
bool q8i_gemm_ksplit2_ok(const q8i_gemm_job *d, int njobs, int n);
q8_status q8i_gemm_ksplit2(q8_ctx *ctx, const q8i_gemm_job *d, int njobs, int n);
bool q8i_vocab_panel_ok(const q8_mat *W);
bool q8i_output_codes_keeps_no_logits(const q8_mat *W, int k);
q8_status q8i_vocab_panel(q8_ctx *ctx, const q8_mat *W, const float *bias, const int8_t *xq, const float *xscale, int n,
                          float *part_max, double *part_sum);
q8_status q8i_gru(q8_ctx *ctx, const q8i_gru_desc *d, int njobs, int n, int mode);
// ctx_q / ctx_qscale (may be NULL): where the finishing blocks leave the codes [n x ldq] and scales [n] of the
// context vectors; *codes_written says whether this launch does (C even, ldq <= 8192, panels: ldq <= 2048)
q8_status q8i_attention(q8_ctx *ctx, const float *P, const float *enc_h, int l, int A, int C, const float *a,
                        const float *v, int n, float *e, float *alpha, float *cvec, const int *sent_off, int beam,
                        int8_t *ctx_q, float *ctx_qscale, int ldq, int *codes_written);
// element-wise parts of the attention variant with 8-bit activation products
q8_status q8i_att_tanh(q8_ctx *ctx, const float *P, const float *a, float *T, int l, int A, int n);
q8_status q8i_att_softmax(q8_ctx *ctx, const float *e, int n, int l, int ld_alpha, float *alpha_ws, float *alpha_out,
                          float *e_out);
q8_status q8i_transpose(q8_ctx *ctx, const float *X, int rows, int cols, float *Xt);
q8_status q8i_gru_gates(q8_ctx *ctx, const float *gx, const float *gh, const float *h_prev, int ldh, float *h_out,
                        int ldo, int H, int n);
// the same, also leaving the new states quantized in q1 [n x ld1] / s1 [n] (and q2 / s2 unless q2 is NULL)
bool q8i_gru_gates_q_ok(int H, int ldh, int ldo, int ld1, int ld2);
q8_status q8i_gru_gates_q(q8_ctx *ctx, const float *gx, const float *gh, const float *h_prev, int ldh, float *h_out,
                          int ldo, int H, int n, int8_t *q1, int ld1, float *s1, int8_t *q2, int ld2, float *s2);
// products, gates and the codes of the new states in one launch (panels; shapes: q8i_gru_panel_ok).  gh_pre NULL:
// both products from the codes xq / hq; else the input product alone, the recurrent pre-activations given.
// q1 NULL: no codes.  region 0 or 1: see the launcher.
bool q8i_gru_panel_ok(q8_ctx *ctx, const q8_gru_weights *g, bool gh_pre, int n, int ldp, int ldo, bool codes, int ld1, int ld2, bool have_q2);
q8_status q8i_gru_panel(q8_ctx *ctx, const q8_gru_weights *g, const int8_t *xq, const float *xs, const int8_t *hq,
                        const float *hs, const float *gh_pre, const float *h_prev, int ldp, float *h_out, int ldo, int n,
                        int8_t *q1, int ld1, float *s1, int8_t *q2, int ld2, float *s2, int region);
// one time step of the batched encoder: phase 0 quantizes the previous states, phase 1 applies the gates
q8_status q8i_encode_persistent(q8_ctx *ctx, const q8_gru_weights *fwd, const q8_gru_weights *bwd, const float *gxf,
                                const float *gxb, int l, float *enc_h, unsigned long long *xchg, unsigned *err,
                                int spin_limit, int *launched);
q8_status q8i_enc_step(q8_ctx *ctx, int phase, const int *sent_off, int S, int t, int H, int ld, float *enc_h,
                       const float *gxf, const float *gxb, float *ghf, float *ghb, int8_t *hqf, int8_t *hqb, float *hsf,
                       float *hsb);
q8_status q8i_readout_combine(q8_ctx *ctx, const float *ts, const float *ty, const float *tc, const float *b_t, int R,
                              int n, float *t_out, int ld, int8_t *tq, float *tscale, const q8_taps *tap);
q8_status q8i_output_codes(q8_ctx *ctx, const q8_mat *W, const float *bias, const int8_t *tq, const float *tscale, int n,
                           int k, float *logits, int tiled, float *lse, float *topk_logp, int32_t *topk_idx,
                           int32_t *tap_acc, float *part_max, double *part_sum, const BeamBatchArgs *search = nullptr,
                           int *search_fused = nullptr);
BeamBatchArgs q8i_beam_batch_args(void *states, size_t stride, int beam, int k, int max_steps, const float *topk_logp,
                                  const int *topk_idx, const float *s_step, const float *E_tgt, int E, int H, float *y_emb,
                                  float *s_next, int *done, const float *enc_h, const int *sent_off, int C, int V,
                                  const struct q8i_beam_desc *codes);
q8_status q8i_beam_batch(q8_ctx *ctx, int init, void *states, size_t stride, int S, int beam, int k, int max_steps,
                         const float *topk_logp, const int *topk_idx, const float *s_step, const float *E_tgt, int E,
                         int H, float *y_emb, float *s_next, int *done, const float *enc_h, const int *sent_off, int C, int V,
                         const struct q8i_beam_desc *codes = nullptr);
q8_status q8i_beam_read_batch(q8_ctx *ctx, const void *states, size_t stride, int S, int max_steps, int32_t *tokens_host,
                              int *len_host, float *score_host, int *steps_host);
// y_codes / c_codes (may be NULL): codes of y and c left by their producers; used when both are valid and laid out
// with the pitches of W_y and W_c
q8_status q8i_readout(q8_ctx *ctx, const q8_readout_weights *ro, const float *s, const float *y, const float *c, int n,
                      float *t_out, const q8_taps *taps3, const q8_codes *y_codes = nullptr, const q8_codes *c_codes = nullptr,
                      int8_t *sq_out = nullptr, float *ss_out = nullptr, int *s_exported = nullptr,
                      const struct q8i_gemv_desc *extra = nullptr, int *extra_done = nullptr);
// One product with rows of at most 1024 bytes on the streaming product's fast kernel body, as blocks of another
// kernel (see readout_with_product_kernel): fills the job, its block count and LDS bytes; false if it does not fit.
struct GemvJobs;
bool q8i_gemv_fast_setup(const struct q8i_gemv_desc *d, int n, struct GemvJobs *jobs, int *blocks, size_t *smem);
q8_status q8i_probe_read(q8_ctx *ctx, const void *buf, size_t bytes);
q8_status q8i_math_eval(q8_ctx *ctx, int fn, const void *x, void *y, size_t n);
int q8i_out_tiles(int V);
size_t q8i_tiles_bytes(int rows, int ld);
q8_status q8i_pack_tiles(q8_ctx *ctx, const q8_mat *W, int8_t *tiles);
int q8i_out_max_rows(void);
q8_status q8i_launch_check(q8_ctx *ctx, const char *what);
q8_status q8i_output(q8_ctx *ctx, const q8_mat *W, const float *bias, const float *T, int ldt, int n, int k,
                     float *logits, float *lse, float *topk_logp, int32_t *topk_idx, const q8_taps *taps,
                     float *part_max, double *part_sum, const struct q8i_beam_desc *beam);

q8_status q8i_ensemble_combine(q8_ctx *ctx, const float *const *logits, const float *const *lse, int M, int n, int V,
                               float *c, float *part_max, double *part_sum);
q8_status q8i_select_normalized(q8_ctx *ctx, const float *part_max, const double *part_sum, const float *c, int V, int n,
                                int k, float *topk_logp, int32_t *topk_idx, const struct q8i_beam_desc *beam);
q8_status q8i_beam_regather(q8_ctx *ctx, void *state, int n, const float *s_step, int H, const float *E_tgt, int E,
                            float *y_emb, float *s_next);
struct q8i_f32_job {            // Y [n x ldy] = W . X + bias in fp32 (the 32-bit engine)
    const q8_matf *W;
    const float *X;
    int ldx;
    const float *bias;
    float *Y;
    int ldy;
};
q8_status q8i_gemv_f32(q8_ctx *ctx, const q8i_f32_job *d, int njobs, int n);          // njobs <= 3, n <= 8
q8_status q8i_logit_stats(q8_ctx *ctx, const float *logits, int n, int V, float *part_max, double *part_sum);
q8_status q8i_select_logits(q8_ctx *ctx, const float *part_max, const double *part_sum, const float *logits, int V, int n,
                            int k, float *lse, float *topk_logp, int32_t *topk_idx);
size_t q8i_beam_state_bytes(int max_steps);
q8_status q8i_gather_rows(q8_ctx *ctx, const float *table, const int *idx, int n, int dim, int V, float *out);
q8_status q8i_beam_init(q8_ctx *ctx, void *state, int beam, int max_steps, const float *s0, const float *E_tgt, int E,
                        int H, float *y_emb, float *s);
q8_status q8i_beam_update(q8_ctx *ctx, void *state, const float *topk_logp, const int *topk_idx, int n, int k,
                          const float *s_step, int H, const float *E_tgt, int E, float *y_emb, float *s_next);
q8_status q8i_beam_read(q8_ctx *ctx, const void *state, int max_steps, int32_t *tokens_host, int *len_host,
                        float *score_host, int *steps_host, int *done_host);
