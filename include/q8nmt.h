/*
 * q8nmt.h -- C ABI of the MI355X (gfx950) library for 8-bit GRU-NMT decoding.
 *
 * The library implements the hot path of "Pieces of Eight: 8-bit Neural Machine
 * Translation" (Quinn & Ballesteros): Section 3's product -- weights and inputs as
 * 8-bit integers, integer accumulation, 32-bit float result, one routine for matrix
 * x vector and matrix x narrow matrix, bias / sigmoid / tanh kept in float -- driving
 * Section 2's model: bidirectional GRU encoder (Eq. 1), conditional GRU decoder with
 * attention (Eq. 3-6) and the two-layer output network with softmax (Eq. 2).
 *
 * Quantization (Section 3 leaves the scheme open; this is the fixed reading):
 * symmetric max-abs, scale = max|v| / 127, code = clamp(rint(v * (127 / max|v|)),
 * -127, 127) with round-half-to-even, all in IEEE fp32; if max|v| < 2^-100 the scale
 * is 1 and every code 0.  One scale per weight matrix, one per activation vector
 * (per column of a narrow matrix).  Accumulation is exact int32.  The float result is
 * y_i = (float)acc_i * (s_w * s_x), then + bias_i as a separate fp32 add.  Two variants
 * of the scheme exist beside it as entry points of their own: one weight scale per row
 * (q8_gemm_narrow_rows) and 8-bit products inside the attention (q8_attention_q8).
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless its name ends in _host.  All device
 *    buffers, the workspace included, are owned by the caller and only borrowed for
 *    the duration of the enqueued work.  Structs passed by pointer are read during
 *    the call and need not outlive it.
 *  - Matrices are row-major with the reduction dimension contiguous.  int8 weight
 *    matrices: base 16-byte aligned, ld % 16 == 0, pad columns [cols, ld) zero.
 *    fp32 vectors: 16-byte aligned base, leading dimensions % 4 == 0.  Batches are
 *    vector-major: [n x dim], each vector contiguous.
 *  - Calls enqueue work on the stream given to q8_create and return without waiting,
 *    except q8_quantize_matrix and q8_attention_states_q8 (they return a scale to the
 *    host), the *_result calls and the q8_translate* drivers.
 *  - Every function returns a q8_status.  Argument errors are detected before
 *    anything is launched; nothing aborts or throws.  q8_last_error gives text.
 *  - Limits: 1 <= cols <= ld <= 16384 for products (the int32 sum cannot overflow
 *    below 133143 columns); narrow products take n <= 8 vectors in one pass over the
 *    weights and 8 < n <= 1024 on the matrix cores (blocked int8 GEMM); the same two
 *    regimes hold for gru_step_q8 and output_logits_q8; cgru_decoder_step_q8 takes
 *    n <= 8 hypotheses of one sentence, cgru_decoder_step_batch_q8 up to 1024 slots of
 *    several sentences; source length l <= 1024; top-k <= 16.
 *  - Non-finite inputs give unspecified results (no fault).
 *  - A context is tied to one stream and one workspace and is not thread-safe.  Calls
 *    that use the workspace (everything but q8_gemv and n <= 8 q8_gemm_narrow) must
 *    not overlap on the GPU; on one stream they cannot.
 *  - Taps: optional (NULL) device outputs of the integer tensors of a product, so that
 *    results can be checked bit for bit: xq [n x cols] int8 (ld = cols), xscale [n],
 *    acc [n x rows] int32.
 */
#ifndef Q8NMT_H
#define Q8NMT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int q8_status;
enum {
    Q8_OK = 0,
    Q8_ERR_NULL = 1,       /* a required pointer is NULL */
    Q8_ERR_SHAPE = 2,      /* a dimension is non-positive, inconsistent or above a limit */
    Q8_ERR_ALIGN = 3,      /* base pointer or leading dimension violates the alignment rule */
    Q8_ERR_WORKSPACE = 4,  /* the context's workspace is too small for this call */
    Q8_ERR_DEVICE = 5      /* a HIP call failed; see q8_last_error */
};

typedef struct q8_ctx q8_ctx;

/* An int8 weight matrix: device data, host-side scale (known at load time).  `tiles` is
 * an optional second copy of the same codes in the matrix-core streaming order made by
 * q8_pack_tiles (NULL = none).  Where it is present the matrix-core kernels read it instead of
 * `data`: output_logits_q8, and every product of a panel of more than 8 vectors (GRU, attention
 * and readout products of batched decoding, the encoder's input products).  The kernels for at
 * most 8 vectors always read `data`, so a matrix used both ways keeps both copies. */
typedef struct {
    const int8_t *data;
    int rows, cols, ld;
    float scale;
    const int8_t *tiles;
} q8_mat;

typedef struct {
    int8_t *xq;
    float *xscale;
    int32_t *acc;
} q8_taps;

/* Codes that travel with n fp32 vectors from the entry point that quantized them (Section 3:
 * one scale per vector) to the next one that multiplies the same vectors: int8 codes [n x ld]
 * (bytes past the vector's length zero) and scales [n], device memory of the caller.  The
 * producer sets `valid` (host side, before it returns) to say whether its launches write them;
 * a consumer uses them only if valid and ld is the pitch of the matrix it multiplies, and then
 * produces exactly what it would from the fp32 vectors, which it still needs. */
typedef struct {
    int8_t *q;
    float *scale;
    int ld;
    int valid;
} q8_codes;

/* One GRU cell.  Gate row blocks in the order r, z, n; biases [3H] may be NULL. */
typedef struct {
    q8_mat Wx;             /* [3H x I] */
    q8_mat Wh;             /* [3H x H] */
    const float *bx, *bh;
} q8_gru_weights;

/* The conditional GRU of Eq. 3-6: GRU r, attention (u and v; w enters through P), GRU q. */
typedef struct {
    q8_gru_weights r;      /* Wx [3H x E], Wh [3H x H] */
    q8_mat att_U;          /* u: [A x H] */
    const float *att_v;    /* v: [A] fp32 */
    q8_gru_weights q;      /* Wx [3H x C], Wh [3H x H] */
} q8_cgru_weights;

/* First layer of the output network g of Eq. 2. */
typedef struct {
    q8_mat W_s, W_y, W_c;  /* [R x H], [R x E], [R x C] */
    const float *b_t;      /* [R] or NULL */
} q8_readout_weights;

/* Bytes of workspace that make every call below succeed for n <= max_n vectors,
 * source length <= max_l, matrices of at most max_rows rows and max_ld columns. */
size_t q8_workspace_bytes(int max_n, int max_l, int max_rows, int max_ld);

/* Creates a context bound to hip_stream (a hipStream_t; NULL = the default stream)
 * and to the caller's device workspace (256-byte aligned).  Allocates host memory
 * only.  The first 128 KiB of the workspace (at least that many bytes are required) are
 * zeroed on the stream here and are left zero after every call by the kernels that use
 * them as arrival counters and exchange words. */
q8_status q8_create(q8_ctx **out, void *hip_stream, void *workspace, size_t workspace_bytes);
q8_status q8_destroy(q8_ctx *ctx);
const char *q8_last_error(const q8_ctx *ctx);

/* Section 3, weights ("models as is", Section 1): W fp32 [rows x cols] (ld_in floats)
 * -> Wq int8 [rows x ld_out] with zeroed pad columns, one scale for the matrix written
 * to *scale_out_host.  Synchronous: waits for the stream. */
q8_status q8_quantize_matrix(q8_ctx *ctx, const float *W, int rows, int cols, int ld_in,
                             int8_t *Wq_out, int ld_out, float *scale_out_host);

/* Load-time re-ordering of a quantized matrix for the matrix-core kernels (a layout choice of
 * this library, not an operation of the paper): rows are grouped in tiles of 16 and each
 * 16 x 64-byte block is stored as one contiguous KiB in the lane order of
 * v_mfma_i32_16x16x64_i8's A operand (lane = 16 * (k / 16 % 4) + row % 16, 16 bytes per lane),
 * so that every wave-wide load of a matrix-core operand is one contiguous KiB (16 pieces of
 * rows that lie ld bytes apart arrive about 2.5 times more slowly).  Rows past
 * `rows` in the last tile are zero.  Requires ld % 64 == 0; tiles_out holds
 * q8_tiles_bytes(rows, ld) bytes, 16-byte aligned.  Enqueued on the stream. */
size_t q8_tiles_bytes(int rows, int ld);
q8_status q8_pack_tiles(q8_ctx *ctx, const q8_mat *W, int8_t *tiles_out);

/* Section 3, matrix x vector: y[rows] = (float)(Wq . quantize(x)) * (s_w * s_x) + bias.
 * bias [rows] may be NULL.  One launch; x is quantized inside the kernel. */
q8_status q8_gemv(q8_ctx *ctx, const q8_mat *W, const float *x, const float *bias, float *y,
                  const q8_taps *taps);

/* Section 3, matrix x narrow matrix (the same routine, P small): n vectors X [n x ldx]
 * -> Y [n x ldy], each vector with its own scale; bit-identical to n q8_gemv calls.
 * n <= 8: one streaming pass over W.  n > 8: vectors are quantized into the workspace
 * and the product runs on the int8 matrix cores. */
q8_status q8_gemm_narrow(q8_ctx *ctx, const q8_mat *W, const float *X, int n, int ldx,
                         const float *bias, float *Y, int ldy, const q8_taps *taps);

/* Variant of Section 3's scheme with one weight scale per ROW (the section does not state the
 * granularity of the scale; every other entry point takes one scale per matrix).
 * q8_quantize_matrix_rows: row i of W [rows x cols] (ld_in floats per row) is quantized on its
 * own maximum: codes into Wq_out row i (ld_out bytes per row, pad bytes zero), scale into
 * row_scale_out[i] (DEVICE pointer, rows floats).  Enqueued on the stream, nothing returns to
 * the host.  Same shape and alignment rules as q8_quantize_matrix.
 * q8_gemm_narrow_rows: Y[j][i] = (float)(Wq_i . quantize(X_j)) * (row_scale[i] * s_xj) + bias[i];
 * W->scale is ignored, row_scale is a device pointer to W->rows floats; everything else as
 * q8_gemm_narrow (n = 1 is the matrix x vector product). */
q8_status q8_quantize_matrix_rows(q8_ctx *ctx, const float *W, int rows, int cols, int ld_in,
                                  int8_t *Wq_out, int ld_out, float *row_scale_out);
q8_status q8_gemm_narrow_rows(q8_ctx *ctx, const q8_mat *W, const float *row_scale, const float *X, int n,
                              int ldx, const float *bias, float *Y, int ldy, const q8_taps *taps);

/* GRU cell of Eq. 1 / Eq. 3-4 for n vectors: gx = Wx q(x) + bx, gh = Wh q(h) + bh,
 * r = sigmoid(gx_r + gh_r), z = sigmoid(gx_z + gh_z), n = tanh(gx_n + r * gh_n),
 * h' = (1 - z) * n + z * h (h in fp32).  x [n x I], h_prev [n x H], h_out [n x H]
 * (must not alias h_prev).  taps: NULL or two entries, [0] for the Wx product and
 * [1] for the Wh product.  n <= 8: one fused streaming kernel; 8 < n <= 1024: both
 * products on the matrix cores, then the gates; the values are the same. */
q8_status gru_step_q8(q8_ctx *ctx, const q8_gru_weights *g, const float *x, const float *h_prev,
                      int n, float *h_out, const q8_taps *taps2);

/* One conditional-GRU decoder step (Eq. 3-6) for n_beam hypotheses of one sentence:
 * s' = r(y, s_prev); a = u q(s'); e_i = v . tanh(P_i + a); alpha = softmax(e);
 * H_t = sum_i alpha_i h_i; s = q(H_t, s').  P [l x A] is w(h_i) + b_att for every
 * source position (q8_gemm_narrow over enc_h), enc_h [l x C].  y_emb [n x E],
 * s_prev [n x H] -> s_out [n x H], ctx_out [n x C]; alpha_out [n x l] and
 * s_mid_out [n x H] may be NULL.  taps5: NULL or five entries for the products
 * r.Wx(y), r.Wh(s_prev), att_U(s'), q.Wx(H_t), q.Wh(s'). */
q8_status cgru_decoder_step_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                               int l, const float *y_emb, const float *s_prev, int n_beam,
                               float *s_out, float *ctx_out, float *alpha_out, float *s_mid_out,
                               const q8_taps *taps5);

/* cgru_decoder_step_q8 (without taps) for callers that cannot allocate device memory or hand over
 * a workspace of their own: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Its kernels' scratch (s', u(s'), the recurrent half of GRU q, the attention energies,
 * the context codes, the arrival counters) lives in a static device array of
 * q8_noalloc_scratch_bytes() = 1 MiB that every GPU the library runs on holds until the process
 * ends; the context's own workspace is not touched, and no device memory is allocated or freed.
 * Sizes that need more scratch than the array holds are refused with Q8_ERR_WORKSPACE (with
 * H = A = 1024 every n_beam <= 8 and l <= 1024 fits).  All calls on one GPU share that GPU's array:
 * calls that overlap there (two streams, two contexts) race; calls on one stream do not.
 * q8_noalloc_setup looks the array up on the current device and clears its counters (it waits for
 * the stream); the first cgru_decoder_step_noalloc_q8 on a device does the same if it was not
 * called, and therefore must not be made under stream capture.  Results are bit-identical to
 * cgru_decoder_step_q8. */
size_t q8_noalloc_scratch_bytes(void);
q8_status q8_noalloc_setup(q8_ctx *ctx);
q8_status cgru_decoder_step_noalloc_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                                       int l, const float *y_emb, const float *s_prev, int n_beam,
                                       float *s_out, float *ctx_out, float *alpha_out, float *s_mid_out);

/* Variant of the attention block of Eq. 5-6 in which the two products without a trained matrix
 * are 8-bit as well (the other reading of Section 3; cgru_decoder_step_q8 keeps them in float).
 * q8_attention_states_q8 (once per sentence, synchronous like q8_quantize_matrix): the encoder
 *   states enc_h [l x C] are transposed and quantized with one scale into hT_out, int8
 *   [C x ld_out] (ld_out >= l, ld_out % 16 == 0, pad bytes zero); the scale returns to the host.
 *   Workspace: 4 C l bytes.
 * q8_attention_q8: v is the energy vector as a 1 x A int8 matrix (q8_quantize_matrix of v),
 *   hT the matrix made above (C x l).  For each of the n <= 8 hypotheses, with a [n x A] = u(s'):
 *   T_i = tanh(P_i + a) is quantized per source position, e_i = (float)(vq . Tq_i) * (s_v * s_Ti);
 *   alpha = softmax(e); alpha is quantized per hypothesis,
 *   ctx_c = (float)(hTq_c . alphaq) * (s_h * s_alpha).  P [l x A]; ctx_out [n x C]; e_out and
 *   alpha_out [n x l] may be NULL.  A % 4 == 0, l <= 1024.  Workspace: about n l (4 A + ld(v) + 12) bytes. */
q8_status q8_attention_states_q8(q8_ctx *ctx, const float *enc_h, int l, int C, int8_t *hT_out, int ld_out,
                                 float *scale_out_host);
q8_status q8_attention_q8(q8_ctx *ctx, const q8_mat *v, const q8_mat *hT, const float *P, const float *a, int n,
                          int l, float *e_out, float *alpha_out, float *ctx_out);

/* Output network g of Eq. 2 for n_beam hypotheses.  If ro != NULL:
 * t = tanh(((W_s q(s) + W_y q(y_emb)) + W_c q(ctx)) + b_t), else t = t_in [n x R].
 * logits = W_out q(t) + b_out; lse = log sum exp(logits); the k best entries per
 * hypothesis, ordered by (logit descending, index ascending), are returned as
 * topk_idx [n x k] and topk_logp [n x k] = logit - lse.  logits [n x rows(W_out)],
 * lse [n] and t_out [n x R] may be NULL.  taps4: NULL or four entries for the products
 * W_s(s), W_y(y), W_c(ctx), W_out(t) (the first three unused when ro == NULL).
 * n_beam <= 8: streaming kernels.  8 < n_beam <= 1024 (hypotheses of many sentences): every
 * product on the matrix cores.  With logits == NULL, a tile-packed W_out with rows of 512 or
 * 640 bytes, k <= 16 and no taps, no logits are kept anywhere: only each 16-row tile's
 * (max, sum of exp) per hypothesis, and the selection computes the logits of the few tiles
 * that can hold one of the k best a second time (same results).  Otherwise the [n x rows]
 * logits are materialized, in the workspace when logits == NULL (it must have room for them). */
q8_status output_logits_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                           const float *s, const float *y_emb, const float *ctx_vec, const float *t_in,
                           int n_beam, int k, float *logits, float *lse, float *topk_logp, int32_t *topk_idx,
                           float *t_out, const q8_taps *taps4);

/* The encoder of Eq. 1 for n_sent sentences side by side: X [L x E] holds their embedding
 * vectors back to back, sentence s in rows [sent_off[s], sent_off[s + 1]) (sent_off: device
 * int32 [n_sent + 1]; sent_off_host: the same values on the host, sent_off_host[0] = 0);
 * enc_h [L x 2H] as q8_encode.  All input products run as matrix-core panels; time step t
 * of every sentence that has one, in both directions, runs in one quantize / product /
 * gates launch triple.  Values are those of q8_encode sentence by sentence.  Needs
 * q8_encode_batch_bytes(fwd, L, n_sent) bytes of workspace. */
size_t q8_encode_batch_bytes(const q8_gru_weights *fwd, int total_l, int n_sent);
q8_status q8_encode_batch(q8_ctx *ctx, const q8_gru_weights *fwd, const q8_gru_weights *bwd, const float *X,
                          const int32_t *sent_off, const int32_t *sent_off_host, int n_sent, float *enc_h);

/* The decoder step of Eq. 3-6 for several sentences side by side (batching is the extension
 * Section 6 names).  Sentence s owns hypothesis slots [s beam, (s + 1) beam) of y_emb,
 * s_prev, s_out [n x H], ctx_out [n x C] (n = n_sent * beam <= 1024) and rows
 * [sent_off[s], sent_off[s + 1]) of P [L x A] and enc_h [L x C]; sent_off is a device
 * array of n_sent + 1 int32, max_l the longest sentence (<= 1024).  alpha_out
 * [n x max_l] (row pitch max_l, entries past the sentence's length untouched) and
 * s_mid_out [n x H] may be NULL.  Per-vector quantization makes every slot's result
 * the one cgru_decoder_step_q8 gives for that slot alone. */
q8_status cgru_decoder_step_batch_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                                     const int32_t *sent_off, int n_sent, int beam, int max_l, const float *y_emb,
                                     const float *s_prev, float *s_out, float *ctx_out, float *alpha_out,
                                     float *s_mid_out);

/* Bidirectional GRU encoder of Eq. 1 over l embedding vectors X [l x E]:
 * enc_h [l x 2H], backward state in columns [0,H), forward state in [H,2H); both
 * recurrences start from zero.  The input products for all positions run as one
 * narrow/MFMA product per direction, the l recurrent steps run in sequence. */
q8_status q8_encode(q8_ctx *ctx, const q8_gru_weights *fwd, const q8_gru_weights *bwd,
                    const float *X, int l, float *enc_h);

/* How q8_encode runs the recurrence.  one_launch != 0 (the default): all positions in one
 * launch where the shape is covered (H % 8 == 0, H <= 2048, rows of Wh of at most 2048 bytes,
 * not under stream capture) and the device can hold 2 H / 8 blocks of 512 threads at once;
 * otherwise, and with one_launch == 0, one launch per position.  Both give the same bits.
 * Inside the one-launch kernel blocks wait for each other's results; every such wait gives up
 * after spin_limit polls (<= 0: the default, 2^20) and the kernel then still ends, leaving enc_h
 * invalid and a flag in the workspace that q8_encode_check reports.  The grid fits the device,
 * so every block runs and the waits end; the bound is a safety net.
 * q8_encode_check waits for the stream and returns Q8_ERR_DEVICE if an encoder launch since the
 * last check gave up (q8_translate and q8_translate_ensemble call it themselves). */
q8_status q8_encoder_options(q8_ctx *ctx, int one_launch, int spin_limit);
q8_status q8_encode_check(q8_ctx *ctx);

/* How the attention block of cgru_decoder_step_q8 / _codes_q8 (Eq. 5-6, one sentence, n_beam <= 8)
 * runs.  Both forms launch one kernel of l x n_beam blocks, one energy each, and give the same bits.
 * exchange != 0 (the default): every block publishes its energy, waits for the other l - 1 of its
 * hypothesis, and then sums and quantizes its own slice of the context vector (the slices' largest
 * magnitudes are exchanged the same way); used where l <= 128, C <= 4096 and the device holds all
 * l n_beam blocks of 1024 threads at once.  exchange == 0, and every other shape: the last block
 * of a hypothesis to arrive computes the whole context vector.  The waits of the first form give
 * up after spin_limit polls (<= 0: the default, 2^20); the kernel then still ends, its results and
 * those of later calls are not valid until q8_encode_check (above) has reported it, once, and put
 * the exchange words in the workspace header back to zero.  The same bound and the same report
 * cover the one wait of output_logits_beam_q8, whose selection kernel hands every hypothesis' k
 * best to the block that runs the search step, and the GRU transitions of
 * cgru_decoder_step_batch_q8 at up to 336 hypothesis slots (rows of 512 / 1024 / 2048 bytes, H a
 * multiple of 32 up to 1024): with exchange != 0 each is one kernel (products, gates, codes of the
 * new states) whose blocks exchange the largest magnitudes of their parts of a state; with
 * exchange == 0, and for every other shape, products and gates are separate launches.  Same bits.
 * Contexts whose decoder steps may run at the same time on one device (different streams): the
 * blocks of the exchange form wait for each other, so the attention grids that can be in flight
 * together must fit the device together (l n_beam blocks of 1024 threads each, two per compute
 * unit); give the contexts beyond that exchange = 0.  The same holds for q8_encoder_options'
 * one-launch recurrence (2 H / 8 blocks of 512 threads) and for the batched step's one-kernel
 * GRU (H / 32 x ceil(slots / 48) blocks of 768 threads, one per compute unit).  The waits inside the
 * selection kernels (output_logits_beam_q8 and its forms, output_logits_beam_ahead_q8's blocks that
 * compute the next GRU r, output_logits_beam_batch_q8) are for blocks of lower index in the same
 * launch, which the device has started before the block that waits: they end whatever else runs. */
q8_status q8_attention_options(q8_ctx *ctx, int exchange, int spin_limit);

/* ---- search (Section 3 only says the beam is smaller than 8; these are the rules) ----
 * Token 0 is both begin- and end-of-sentence.  A search starts with one live hypothesis
 * (score 0, previous token 0) and `beam` slots.  Each step every live hypothesis offers its
 * k best continuations (k >= beam), scored cumulative + log-probability (one fp32 add);
 * the b_live best candidates are kept, ordered by (score descending, parent ascending,
 * token ascending); a kept candidate that ends in token 0 is finished (the best finished
 * one is remembered, ties to the earlier) and b_live drops by one, the others become the
 * live hypotheses.  The search is over when b_live is 0 or max_steps steps were made; the
 * result is the best finished hypothesis, else the best live one.  Scores are not
 * length-normalised.  The state lives on the device; slots that are not live carry score
 * -inf and a copy of slot 0 so that the decoder kernels always see finite data. */

/* Bytes of device memory of a search state for up to max_steps target tokens. */
size_t q8_beam_state_bytes(int max_steps);

/* Starts a search: writes the state, y_emb [beam x E] = E_tgt[0] and s [beam x H] = s0. */
q8_status q8_beam_init(q8_ctx *ctx, void *state, int beam, int max_steps, const float *s0, const float *E_tgt,
                       int E, int H, float *y_emb, float *s);

/* One search step from the top-k of output_logits_q8 (topk_logp, topk_idx [n_beam x k]) and
 * the decoder states s_step [n_beam x H] of this step: updates the state and writes the
 * inputs of the next step, s_next [n_beam x H] (must not alias s_step) and y_emb
 * [n_beam x E] = E_tgt[new tokens].  Does nothing once the search is over.  Every topk_idx must
 * be a row of E_tgt: the table's height is not known here and the ids are not checked. */
q8_status q8_beam_update(q8_ctx *ctx, void *state, const float *topk_logp, const int32_t *topk_idx, int n_beam,
                         int k, const float *s_step, int H, const float *E_tgt, int E, float *y_emb, float *s_next);

/* output_logits_q8 followed by q8_beam_update in the same launches (the update runs in the
 * block of the selection kernel that finishes last): logits of the decoder states s
 * [n_beam x H] of this step, their k best entries, then the search step, which writes
 * s_next [n_beam x H] (must not alias s) and overwrites y_emb [n_beam x E] with the
 * embeddings of the new tokens.  topk_logp / topk_idx [n_beam x k] may be NULL (workspace).
 * E_tgt must have W_out->rows rows.  Non-finite inputs give an unspecified search step, with
 * every token id inside the table. */
q8_status output_logits_beam_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                const float *s, float *y_emb, const float *ctx_vec, int n_beam, int k, void *state,
                                const float *E_tgt, int E, float *s_next, float *topk_logp, int32_t *topk_idx);

/* The decoder step with the quantized vectors handed on instead of recomputed (for callers that
 * cannot afford the second quantization: the readout of Eq. 2 multiplies the same y and H_t that
 * GRU r and GRU q multiplied earlier in the step).  cgru_decoder_step_codes_q8 is
 * cgru_decoder_step_q8 and also leaves the codes of y_emb (pitch r.Wx.ld) and of the context
 * vectors (pitch q.Wx.ld) in y_codes / ctx_codes (either may be NULL; q, scale and ld are the
 * caller's, valid is set here).  output_logits_beam_codes_q8 is output_logits_beam_q8 and takes
 * them (either NULL: as output_logits_beam_q8).  Results are bit-identical to the plain calls. */
q8_status cgru_decoder_step_codes_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                                     int l, const float *y_emb, const float *s_prev, int n_beam,
                                     float *s_out, float *ctx_out, float *alpha_out, float *s_mid_out,
                                     const q8_taps *taps5, q8_codes *y_codes, q8_codes *ctx_codes);
q8_status output_logits_beam_codes_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out,
                                      const float *b_out, const float *s, float *y_emb, const float *ctx_vec,
                                      int n_beam, int k, void *state, const float *E_tgt, int E, float *s_next,
                                      float *topk_logp, int32_t *topk_idx, const q8_codes *y_codes,
                                      const q8_codes *ctx_codes);

/* The same pair for a decoding loop, in which the search step's outputs are the next decoder
 * step's inputs: the rows it gathers (embeddings of the new tokens into y_emb, surviving states
 * into s_next) are rows that were, or can be, quantized before (Section 3: a vector's codes
 * depend on the vector alone), so their codes are gathered with them and GRU r of the next step
 * (Eq. 3) multiplies without quantizing.
 * q8_row_codes: every row of the embedding table quantized on its own maximum, once, by
 * q8_quantize_matrix_rows(E_tgt, V, E, E, q, ld, scale) with ld = r.Wx.ld (= the readout's W_y.ld).
 * output_logits_beam_loop_q8 is output_logits_beam_codes_q8 (y_codes with valid == 1 and ctx_codes
 * are this step's, for the readout) and, given E_codes, y_codes and s_next_codes with the pitches of
 * W_y and W_s and E / 4 + W_y.ld / 16 + W_s.ld / 16 <= 256, leaves the codes of the new y_emb in
 * y_codes and those of s_next (copies of the codes the readout made of s) in s_next_codes, both with
 * valid = 2; otherwise valid = 0.  cgru_decoder_step_loop_q8 is cgru_decoder_step_codes_q8 and takes
 * y_codes and s_prev_codes with valid == 2 (pitches r.Wx.ld, r.Wh.ld; no taps) as the codes of
 * y_emb and s_prev; on return y_codes is valid (1) for the readout as before and s_prev_codes is
 * spent (0).  A caller that changes y_emb or s_prev itself (q8_beam_init does) sets valid = 0.
 * Bit-identical to the plain calls. */
typedef struct {
    const int8_t *q;       /* [rows x ld], pad bytes zero */
    const float *scale;    /* [rows] */
    int ld;
} q8_row_codes;
q8_status cgru_decoder_step_loop_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                                    int l, const float *y_emb, const float *s_prev, int n_beam,
                                    float *s_out, float *ctx_out, float *alpha_out, float *s_mid_out,
                                    const q8_taps *taps5, q8_codes *y_codes, q8_codes *ctx_codes,
                                    q8_codes *s_prev_codes);
q8_status output_logits_beam_loop_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out,
                                     const float *b_out, const float *s, float *y_emb, const float *ctx_vec,
                                     int n_beam, int k, void *state, const float *E_tgt, int E, float *s_next,
                                     float *topk_logp, int32_t *topk_idx, q8_codes *y_codes,
                                     const q8_codes *ctx_codes, q8_codes *s_next_codes,
                                     const q8_row_codes *E_codes);

/* The decoding loop of one sentence with GRU r (Eq. 3) taken off the chain of dependent launches.  s' of the next
 * step is r(E_tgt[token], s[parent]) for the token and parent the search step picks.  Its two products do not
 * depend on that decision (Section 3: a vector's codes, and so its 8-bit products, depend on the vector alone):
 * W_x^r q(E_tgt[v]) + b_x is a function of the token, kept as a table gx_table [V x 3H] (device, fp32; made once
 * per model with q8_gemm_narrow over the rows of E_tgt: 614 MB at V = 50000, H = 1024), and W_h^r q(s_j) + b_h of
 * every state s_j of this step is multiplied in the readout's launch.  What is left for after the decision are
 * the gates.
 * cgru_decoder_step_ahead_q8: Eq. 4-6 from a given s' (s_mid [n_beam x H]): writes s_out, ctx_out (alpha_out, ctx_codes
 * as in cgru_decoder_step_codes_q8).
 * output_logits_beam_ahead_q8: output_logits_beam_loop_q8 whose search step moves no state rows; r: the weights of
 * GRU r (r->Wh, r->bh are used; rows of W_h^r of at most 1024 bytes ride in the readout's launch, longer ones take a
 * launch of their own); blocks of the selection kernel wait (bounded, reported as q8_attention_options says) for
 * the search step's decision and write s_mid_next [n_beam x H] = gates(gx_table[token], W_h^r q(s[parent]) + b_h,
 * s[parent]), the s' of the next step.  y_codes: in, the codes of this step's y_emb (valid != 0; else quantized
 * here); out, with E_codes, those of the new y_emb (valid = 2).  The first s' of a search is
 * gru_step_q8(r, y_emb, s).  Bit-identical to cgru_decoder_step_q8 + output_logits_beam_q8. */
q8_status cgru_decoder_step_ahead_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h, int l,
                                     const float *s_mid, int n_beam, float *s_out, float *ctx_out, float *alpha_out,
                                     q8_codes *ctx_codes);
q8_status output_logits_beam_ahead_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                      const float *s, float *y_emb, const float *ctx_vec, int n_beam, int k, void *state,
                                      const float *E_tgt, int E, float *topk_logp, int32_t *topk_idx, q8_codes *y_codes,
                                      const q8_codes *ctx_codes, const q8_row_codes *E_codes, const q8_gru_weights *r,
                                      const float *gx_table, float *s_mid_next);

/* The same for panels of hypothesis slots: cgru_decoder_step_batch_codes_q8 is
 * cgru_decoder_step_batch_q8 and also leaves the codes of y_emb (pitch r.Wx.ld), of the context
 * vectors (pitch q.Wx.ld) and of the new states s_out (any pitch ld >= H that is a multiple of
 * 16: the readout's W_s.ld) with the caller; output_logits_codes_q8 is output_logits_q8 with the
 * readout (ro must not be NULL, no taps) and takes the three: when all are valid and have the
 * pitches of W_s, W_y and W_c, a panel of more than 8 slots skips its quantization launch; up to
 * 8 slots use y and the context as output_logits_beam_codes_q8 does.  Bit-identical results. */
q8_status cgru_decoder_step_batch_codes_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                                           const int32_t *sent_off, int n_sent, int beam, int max_l,
                                           const float *y_emb, const float *s_prev, float *s_out, float *ctx_out,
                                           float *alpha_out, float *s_mid_out, q8_codes *y_codes,
                                           q8_codes *ctx_codes, q8_codes *s_codes);
q8_status output_logits_codes_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                 const float *s, const float *y_emb, const float *ctx_vec, int n_beam, int k,
                                 float *logits, float *lse, float *topk_logp, int32_t *topk_idx, float *t_out,
                                 const q8_codes *s_codes, const q8_codes *y_codes, const q8_codes *ctx_codes);

/* The loop forms for panels (see cgru_decoder_step_loop_q8): q8_beam_update_batch_loop is q8_beam_update_batch
 * with the height V of E_tgt (token ids are kept inside it) and, given E_codes, the codes s_codes of s_step
 * (valid == 1, as cgru_decoder_step_batch_codes_q8 left them) and y_next_codes / s_next_codes with the pitches of
 * E_codes and s_codes (s_next_codes not the buffers of s_codes), it leaves the codes of the new y_emb and of s_next
 * there with valid = 2 (where E / 4 + E_codes->ld / 16 + s_codes->ld / 16 <= 256; otherwise valid = 0).
 * cgru_decoder_step_batch_loop_q8 is cgru_decoder_step_batch_codes_q8 and takes y_codes and s_prev_codes with
 * valid == 2 (pitches r.Wx.ld, r.Wh.ld) in place of quantizing y_emb and s_prev.  Bit-identical results. */
q8_status cgru_decoder_step_batch_loop_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h,
                                          const int32_t *sent_off, int n_sent, int beam, int max_l,
                                          const float *y_emb, const float *s_prev, float *s_out, float *ctx_out,
                                          float *alpha_out, float *s_mid_out, q8_codes *y_codes,
                                          q8_codes *ctx_codes, q8_codes *s_codes, q8_codes *s_prev_codes);
q8_status q8_beam_update_batch_loop(q8_ctx *ctx, void *states, int n_sent, int beam, int k, int max_steps,
                                    const float *topk_logp, const int32_t *topk_idx, const float *s_step, int H,
                                    const float *E_tgt, int E, int V, float *y_emb, float *s_next, int32_t *done,
                                    const q8_row_codes *E_codes, const q8_codes *s_codes, q8_codes *y_next_codes,
                                    q8_codes *s_next_codes);

/* output_logits_codes_q8 for a panel of n_sent beams followed by q8_beam_update_batch_loop (V = W_out->rows), as
 * output_logits_beam_loop_q8 is for one sentence (Eq. 2, then the search rules above): logits of the decoder states
 * s [n_sent beam x H] of this step, their k best entries into topk_logp / topk_idx [n_sent beam x k] (device, not
 * NULL), then every sentence's search step, which writes s_next (must not alias s), overwrites y_emb with the
 * embeddings of the new tokens and sets done [n_sent].  With tile-packed W_out of pitch 512 or 640 and more than 8
 * slots the search steps run inside the selection kernel's launch (the block of a sentence's last slot waits for the
 * k best of the sentence's other slots; the wait is bounded and reported as q8_attention_options says); every other
 * shape runs the two calls one after the other.  s_codes / y_codes / ctx_codes: this step's codes for the readout
 * (any may be NULL or not valid: quantized here); given E_codes, s_codes with valid == 1, y_codes and s_next_codes
 * (pitches of E_codes and s_codes, s_next_codes not the buffers of s_codes), the codes of the new y_emb and of
 * s_next are left in y_codes and s_next_codes with valid = 2 (otherwise valid = 0).  Bit-identical to the two calls. */
q8_status output_logits_beam_batch_q8(q8_ctx *ctx, const q8_readout_weights *ro, const q8_mat *W_out, const float *b_out,
                                      const float *s, float *y_emb, const float *ctx_vec, int n_sent, int beam, int k,
                                      int max_steps, void *states, const float *E_tgt, int E, float *s_next, int32_t *done,
                                      float *topk_logp, int32_t *topk_idx, const q8_codes *s_codes, q8_codes *y_codes,
                                      const q8_codes *ctx_codes, q8_codes *s_next_codes, const q8_row_codes *E_codes);

/* Waits for the stream and copies the result to the host: tokens (without the final
 * token 0), their number, the cumulative log-probability, the steps made, and whether
 * the search is over.  Host pointers; any may be NULL. */
q8_status q8_beam_result(q8_ctx *ctx, const void *state, int max_steps, int32_t *tokens_host, int *len_host,
                         float *score_host, int *steps_host, int *done_host);

/* The whole model of Section 2. */
typedef struct {
    const float *E_src, *E_tgt;      /* fp32 embedding tables [V_src x E], [V_tgt x E]: gather only */
    int V_src, V_tgt, E;
    q8_gru_weights enc_fwd, enc_bwd; /* Eq. 1 */
    q8_mat att_W;                    /* w of Eq. 6: [A x C] */
    const float *att_b;              /* its bias [A] or NULL */
    q8_cgru_weights dec;             /* Eq. 3-6 */
    q8_readout_weights ro;           /* Eq. 2, first layer */
    q8_mat W_out;                    /* Eq. 2, second layer [V_tgt x R] */
    const float *b_out;
    q8_row_codes E_tgt_codes;        /* optional (q == NULL: none): E_tgt row by row at pitch dec.r.Wx.ld; q8_translate
                                        then hands codes from the search step to the next decoder step */
    const float *gx_r;               /* optional (NULL: none): the table of cgru_decoder_step_ahead_q8, W_x^r q(E_tgt[v]) + b_x
                                        [V_tgt x 3H] fp32; q8_translate then decodes with GRU r off the chain of launches */
} q8_model;

/* Workspace bytes that q8_translate needs on top of q8_workspace_bytes(beam, max_l, ...). */
size_t q8_translate_bytes(const q8_model *m, int max_l, int beam, int k, int max_steps);

/* Translates one sentence: embedding lookup, encoder (Eq. 1), attention pre-computation
 * w(h_i), initial decoder state = backward encoder state at the first position, then up
 * to max_steps steps of cgru_decoder_step_q8 + output_logits_q8 + q8_beam_update, all
 * enqueued without reading anything back except a 4-byte "search over" flag every 8
 * steps.  src_tokens: l device int32 ids in [0, V_src); the library never reads them on the
 * host, and an id outside that range is looked up as a zero embedding vector (no fault).
 * m->V_src must be positive and m->V_tgt the number of rows of W_out.  Results as q8_beam_result. */
q8_status q8_translate(q8_ctx *ctx, const q8_model *m, const int32_t *src_tokens, int l, int beam, int k,
                       int max_steps, int32_t *tokens_host, int *len_host, float *score_host, int *steps_host);

/* Beam search for n_sent sentences side by side: states = n_sent consecutive search states
 * of q8_beam_state_bytes(max_steps) bytes each; per-hypothesis tables hold sentence s in
 * slots [s beam, (s + 1) beam).  The rules per sentence are those of q8_beam_update.
 * done [n_sent] (device int32) is set to 1 for a sentence once its search is over; such a
 * sentence's slots keep finite contents and are ignored.
 * q8_beam_init_batch: sentence s starts from the backward encoder state at its first
 * position, enc_h[sent_off[s], 0 .. H) (row pitch C), and token 0. */
q8_status q8_beam_init_batch(q8_ctx *ctx, void *states, int n_sent, int beam, int max_steps, const float *enc_h,
                             const int32_t *sent_off, int C, const float *E_tgt, int E, int H, float *y_emb, float *s,
                             int32_t *done);
q8_status q8_beam_update_batch(q8_ctx *ctx, void *states, int n_sent, int beam, int k, int max_steps,
                               const float *topk_logp, const int32_t *topk_idx, const float *s_step, int H,
                               const float *E_tgt, int E, float *y_emb, float *s_next, int32_t *done);
/* Waits for the stream; sentence s's tokens go to tokens_host + s * max_steps; len_host,
 * score_host, steps_host [n_sent] (host pointers, each may be NULL). */
q8_status q8_beam_result_batch(q8_ctx *ctx, const void *states, int n_sent, int max_steps, int32_t *tokens_host,
                               int *len_host, float *score_host, int *steps_host);

/* Translates n_sent sentences together: src_tokens = their ids back to back (device),
 * sent_off_host [n_sent + 1] their offsets (host, sent_off_host[0] = 0).  Encoder
 * (q8_encode_batch) and decoder steps run for all sentences at once (n_sent * beam <= 1024
 * slots) until every search is over or max_steps is reached.  Results as
 * q8_beam_result_batch; each sentence's translation is the one q8_translate gives for it.
 * Needs q8_translate_batch_bytes + q8_encode_batch_bytes more workspace than
 * q8_workspace_bytes(n_sent * beam, ...). */
size_t q8_translate_batch_bytes(const q8_model *m, int total_l, int n_sent, int beam, int k, int max_steps);
q8_status q8_translate_batch(q8_ctx *ctx, const q8_model *m, const int32_t *src_tokens, const int32_t *sent_off_host,
                             int n_sent, int beam, int k, int max_steps, int32_t *tokens_host, int *len_host,
                             float *score_host, int *steps_host);

/* Ensemble decoding (Section 4: the English-German systems use two models): n_models <= 4
 * models that share the target vocabulary.  Each step runs every model's decoder step and
 * output layer, averages the models' next-word probabilities,
 * c[v] = log((1 / n_models) sum_m exp(logits_m[v] - lse_m)) (double, rounded once), takes the
 * k best entries of c and makes one search step; every model keeps its own encoder states
 * and decoder state per hypothesis.  Arguments and results as q8_translate.  Needs
 * q8_translate_ensemble_bytes more workspace than q8_workspace_bytes(beam, ...). */
size_t q8_translate_ensemble_bytes(const q8_model *const *models, int n_models, int max_l, int beam, int k,
                                   int max_steps);
q8_status q8_translate_ensemble(q8_ctx *ctx, const q8_model *const *models, int n_models, const int32_t *src_tokens,
                                int l, int beam, int k, int max_steps, int32_t *tokens_host, int *len_host,
                                float *score_host, int *steps_host);

/* ---- The 32-bit engine (Section 4 compares the 8-bit engine with it, Tables 3 and 6) ----
 * The same model with fp32 weights and no quantization: a product is
 * y = (float)(sum_k W[i,k] x[k], accumulated in double) + bias.  Everything else (gates,
 * attention, softmax, top-k, search) is shared with the 8-bit path.  fp32 matrices are
 * row-major [rows x ld] with ld % 4 == 0 and a 16-byte aligned base; n <= 8 vectors. */
typedef struct { const float *data; int rows, cols, ld; } q8_matf;
typedef struct { q8_matf Wx, Wh; const float *bx, *bh; } q8_gru_weights_f32;
typedef struct { q8_gru_weights_f32 r; q8_matf att_U; const float *att_v; q8_gru_weights_f32 q; } q8_cgru_weights_f32;
typedef struct { q8_matf W_s, W_y, W_c; const float *b_t; } q8_readout_weights_f32;

q8_status q8_gemv_f32(q8_ctx *ctx, const q8_matf *W, const float *X, int n, int ldx, const float *bias, float *Y,
                      int ldy);
/* As cgru_decoder_step_q8 / output_logits_q8 (ro must not be NULL), without taps. */
q8_status cgru_decoder_step_f32(q8_ctx *ctx, const q8_cgru_weights_f32 *w, const float *P, const float *enc_h, int l,
                                const float *y_emb, const float *s_prev, int n_beam, float *s_out, float *ctx_out,
                                float *alpha_out, float *s_mid_out);
q8_status output_logits_f32(q8_ctx *ctx, const q8_readout_weights_f32 *ro, const q8_matf *W_out, const float *b_out,
                            const float *s, const float *y_emb, const float *ctx_vec, int n_beam, int k, float *logits,
                            float *lse, float *topk_logp, int32_t *topk_idx, float *t_out);

/* Measurement helpers (not operations of the paper).
 *
 * Between q8_profile_begin and q8_profile_end, up to max_samples launches of the
 * kernels of one class carry a pair of HIP events that take the kernel's own begin
 * and end timestamps.  q8_profile_end waits for the stream and returns the average
 * kernel duration in milliseconds and the number of samples (host pointers, may be
 * NULL).  Not for use under stream capture. */
enum {
    Q8_KERNEL_VOCAB = 0,     /* vocabulary projection of output_logits_q8 (Eq. 2) */
    Q8_KERNEL_SELECT = 1,    /* log-softmax + top-k (+ fused beam update) */
    Q8_KERNEL_GEMV = 2,      /* streaming product of q8_gemv / q8_gemm_narrow, n <= 8 */
    Q8_KERNEL_GRU = 3,       /* GRU transition (encoder cell, decoder r and q) */
    Q8_KERNEL_ATTENTION = 4, /* energies, softmax, context (Eqs. 5-6) */
    Q8_KERNEL_READOUT = 5,   /* hidden layer g of Eq. 2 */
    Q8_KERNEL_MFMA = 6,      /* matrix-core product of q8_gemm_narrow, n > 8 */
    Q8_KERNEL_PROBE = 7,     /* q8_probe_read */
    Q8_KERNEL_CLASSES = 8
};
q8_status q8_profile_begin(q8_ctx *ctx, int kernel_class, int max_samples);
q8_status q8_profile_end(q8_ctx *ctx, float *avg_ms_host, int *samples_host);

/* Enqueues a plain read stream over buf (device pointer, 16-byte aligned, bytes a
 * positive multiple of 16): nothing is computed or written.  Timed with the profile
 * calls above it gives the read bandwidth of whichever memory level holds buf, the
 * ceiling the streaming kernels are compared with.  Uses 8 KiB of the workspace. */
q8_status q8_probe_read(q8_ctx *ctx, const void *buf, size_t bytes);

/* Verification aid: evaluates the library's own device functions for the float parts of the
 * model (Section 3 keeps sigmoid, tanh and the exponentials in floating point) on an array of
 * n values, so that they can be compared with a reference on the device they run on.
 * fn = 0: tanh, 1: sigmoid (x, y: n floats); fn = 2: exp for |x| <= 700 (x, y: n doubles);
 * fn = 3: every group of 64 consecutive floats sorted in descending order (the wave-wide sort
 * from which the top-k selection derives its threshold; n a multiple of 256).
 * x, y: device pointers, y may equal x.  Enqueues one launch on the context's stream. */
q8_status q8_math_eval(q8_ctx *ctx, int fn, const void *x, void *y, size_t n);

#ifdef __cplusplus
}
#endif
#endif
