// q8_search.hip -- the search around the decoder of "Pieces of Eight: 8-bit Neural Machine
// Translation": Section 3 only says that the beam is smaller than 8, so the rules are this
// library's (stated with q8_beam_update in q8nmt.h).  Everything runs on the device: the
// host never reads a score or a token inside the step loop.
#include "q8_beam.h"

// Rows of a table of V rows: out[i, :] = table[idx[i], :] (embedding lookup, Eq. 1).  The ids live on
// the device and were never seen by the host: an id outside [0, V) reads nothing and gives a zero row.
__global__ __launch_bounds__(256) void gather_rows_kernel(const float *__restrict__ table, const int *__restrict__ idx,
                                                          int n, int dim, int V, float *__restrict__ out)
{
    const int i = blockIdx.x;
    if (i >= n) return;
    const int id = idx[i];
    const bool ok = (unsigned)id < (unsigned)V;
    const float *src = table + (size_t)(ok ? id : 0) * dim;
    for (int c = threadIdx.x; c < dim; c += blockDim.x) out[(size_t)i * dim + c] = ok ? src[c] : 0.0f;
}

__global__ __launch_bounds__(256) void beam_update_kernel(BeamUpdateArgs a)
{
    beam_update_body(a);
}

size_t q8i_beam_state_bytes(int max_steps)
{
    return sizeof(BeamState) + sizeof(int) * (size_t)Q8_MAX_BEAM * max_steps;
}

struct BeamInitArgs {
    BeamState *st;
    const float *s0, *E_tgt;
    float *y_emb, *s;
    int beam, max_steps, E, H;
};

__device__ __forceinline__ void beam_init_body(const BeamInitArgs &a)
{
    BeamState *st = a.st;
    if (threadIdx.x == 0) {
        st->n_live = 1; st->b_live = a.beam; st->step = 0; st->done = 0;
        st->have_fin = 0; st->fin_len = 0; st->fin_parent = 0; st->max_steps = a.max_steps; st->beam = a.beam;
        st->gathered = 0;
        st->fin_score = -INFINITY;
        for (int b = 0; b < Q8_MAX_BEAM; ++b) { st->score[b] = b == 0 ? 0.0f : -INFINITY; st->last[b] = 0; }
    }
    // every slot starts from the initial state and the embedding of token 0 (slots beyond
    // the first are not live; they only need finite contents)
    for (int e = threadIdx.x; e < a.beam * a.E; e += blockDim.x) a.y_emb[e] = a.E_tgt[e % a.E];
    for (int e = threadIdx.x; e < a.beam * a.H; e += blockDim.x) a.s[e] = a.s0[e % a.H];
}

__global__ __launch_bounds__(256) void beam_init_kernel(BeamInitArgs a)
{
    beam_init_body(a);
}

// Ensembles: the search state was updated from the first model's call; every further model
// gathers its own decoder states and embeddings along the same back-pointers.
__global__ __launch_bounds__(256) void beam_regather_kernel(BeamUpdateArgs a)
{
    __shared__ int s_parent[Q8_MAX_BEAM], s_token[Q8_MAX_BEAM];
    const BeamState *st = a.st;
    if (!st->gathered) return;
    if (threadIdx.x < Q8_MAX_BEAM) {
        const int *link = st->link + (size_t)(st->step - 1) * Q8_MAX_BEAM;
        const int n_live = st->n_live, q = threadIdx.x < n_live ? threadIdx.x : 0;
        const int e = n_live > 0 ? link[q] : 0;
        s_parent[threadIdx.x] = (e >> 24) & 0xF;
        s_token[threadIdx.x] = e & 0xFFFFFF;
    }
    __syncthreads();
    beam_gather(a, s_parent, s_token);
}

// Several sentences side by side: block s runs sentence s (BeamBatchArgs).
__global__ __launch_bounds__(256) void beam_update_batch_kernel(BeamBatchArgs b)
{
    const int s = blockIdx.x;
    const BeamUpdateArgs a = beam_batch_sentence(b, s);
    beam_update_body(a);
    __syncthreads();
    if (threadIdx.x == 0) b.done[s] = a.st->done;
}

__global__ __launch_bounds__(256) void beam_init_batch_kernel(BeamBatchArgs b)
{
    const int s = blockIdx.x;
    const size_t slot = (size_t)s * b.beam;
    // initial decoder state: the backward encoder state at the sentence's first position
    BeamInitArgs a = {(BeamState *)(b.states + (size_t)s * b.stride), b.enc_h + (size_t)b.sent_off[s] * b.C, b.E_tgt,
                      b.y_emb + slot * b.E, b.s_next + slot * b.H, b.beam, b.max_steps, b.E, b.H};
    beam_init_body(a);
    if (threadIdx.x == 0) b.done[s] = 0;
}

// =================================================================== host launchers ==

q8_status q8i_gather_rows(q8_ctx *ctx, const float *table, const int *idx, int n, int dim, int V, float *out)
{
    hipLaunchKernelGGL(gather_rows_kernel, dim3(n), dim3(256), 0, ctx->stream, table, idx, n, dim, V, out);
    return q8i_launch_check(ctx, "gather");
}

q8_status q8i_beam_init(q8_ctx *ctx, void *state, int beam, int max_steps, const float *s0, const float *E_tgt, int E,
                        int H, float *y_emb, float *s)
{
    BeamInitArgs a = {(BeamState *)state, s0, E_tgt, y_emb, s, beam, max_steps, E, H};
    hipLaunchKernelGGL(beam_init_kernel, dim3(1), dim3(256), 0, ctx->stream, a);
    return q8i_launch_check(ctx, "beam_init");
}

q8_status q8i_beam_update(q8_ctx *ctx, void *state, const float *topk_logp, const int *topk_idx, int n, int k,
                          const float *s_step, int H, const float *E_tgt, int E, float *y_emb, float *s_next)
{
    BeamUpdateArgs a = {(BeamState *)state, topk_logp, topk_idx, s_step, E_tgt, y_emb, s_next, n, k, E, H};
    hipLaunchKernelGGL(beam_update_kernel, dim3(1), dim3(256), 0, ctx->stream, a);
    return q8i_launch_check(ctx, "beam_update");
}

BeamBatchArgs q8i_beam_batch_args(void *states, size_t stride, int beam, int k, int max_steps, const float *topk_logp,
                                  const int *topk_idx, const float *s_step, const float *E_tgt, int E, int H, float *y_emb,
                                  float *s_next, int *done, const float *enc_h, const int *sent_off, int C, int V,
                                  const q8i_beam_desc *codes)
{
    BeamBatchArgs b = {(char *)states, stride, topk_logp, topk_idx, s_step, E_tgt, y_emb, s_next, done, enc_h, sent_off,
                       beam, k, E, H, C, max_steps, V};
    if (codes && codes->Eq) {
        b.Eq = codes->Eq; b.Es = codes->Es; b.sq_in = codes->sq_in; b.ss_in = codes->ss_in;
        b.yq_out = codes->yq_out; b.ys_out = codes->ys_out; b.sq_out = codes->sq_out; b.ss_out = codes->ss_out;
        b.ldy = codes->ldy; b.lds = codes->lds;
    }
    return b;
}

q8_status q8i_beam_batch(q8_ctx *ctx, int init, void *states, size_t stride, int S, int beam, int k, int max_steps,
                         const float *topk_logp, const int *topk_idx, const float *s_step, const float *E_tgt, int E,
                         int H, float *y_emb, float *s_next, int *done, const float *enc_h, const int *sent_off, int C, int V,
                         const q8i_beam_desc *codes)
{
    const BeamBatchArgs b = q8i_beam_batch_args(states, stride, beam, k, max_steps, topk_logp, topk_idx, s_step, E_tgt, E, H, y_emb,
                                                s_next, done, enc_h, sent_off, C, V, codes);
    if (init) hipLaunchKernelGGL(beam_init_batch_kernel, dim3(S), dim3(256), 0, ctx->stream, b);
    else hipLaunchKernelGGL(beam_update_batch_kernel, dim3(S), dim3(256), 0, ctx->stream, b);
    return q8i_launch_check(ctx, init ? "beam init (batch)" : "beam update (batch)");
}

q8_status q8i_beam_regather(q8_ctx *ctx, void *state, int n, const float *s_step, int H, const float *E_tgt, int E,
                            float *y_emb, float *s_next)
{
    BeamUpdateArgs a = {(BeamState *)state, nullptr, nullptr, s_step, E_tgt, y_emb, s_next, n, 0, E, H};
    hipLaunchKernelGGL(beam_regather_kernel, dim3(1), dim3(256), 0, ctx->stream, a);
    return q8i_launch_check(ctx, "beam regather");
}

// Rebuilds a finished search from a host copy of its state: the best finished hypothesis,
// else the best live one, by following the back-pointers from its last token.
static void parse_state(const BeamState *h, int32_t *tokens_host, int *len_host, float *score_host, int *steps_host,
                        int *done_host)
{
    int len, slot;
    if (h->have_fin) {
        len = h->fin_len;
        slot = h->fin_parent;
        if (score_host) *score_host = h->fin_score;
    } else {
        len = h->step;
        slot = 0;
        if (score_host) *score_host = h->n_live > 0 ? h->score[0] : 0.0f;
    }
    for (int t = len - 1; t >= 0; --t) {
        const int e = h->link[(size_t)t * Q8_MAX_BEAM + slot];
        if (tokens_host) tokens_host[t] = e & 0xFFFFFF;
        slot = (e >> 24) & 0xF;
    }
    if (len_host) *len_host = len;
    if (steps_host) *steps_host = h->step;
    if (done_host) *done_host = h->done;
}

// All S states in one copy; sentence s's tokens go to tokens_host + s * max_steps.
q8_status q8i_beam_read_batch(q8_ctx *ctx, const void *states, size_t stride, int S, int max_steps, int32_t *tokens_host,
                              int *len_host, float *score_host, int *steps_host)
{
    char *h = (char *)malloc(stride * S);
    if (!h) return q8_fail(ctx, Q8_ERR_DEVICE, "out of host memory");
    hipError_t e = hipMemcpyAsync(h, states, stride * S, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) { free(h); return q8_fail(ctx, Q8_ERR_DEVICE, "beam read: %s", hipGetErrorString(e)); }
    for (int s = 0; s < S; ++s)
        parse_state((const BeamState *)(h + (size_t)s * stride), tokens_host ? tokens_host + (size_t)s * max_steps : nullptr,
                    len_host ? len_host + s : nullptr, score_host ? score_host + s : nullptr,
                    steps_host ? steps_host + s : nullptr, nullptr);
    free(h);
    return Q8_OK;
}

q8_status q8i_beam_read(q8_ctx *ctx, const void *state, int max_steps, int32_t *tokens_host, int *len_host,
                        float *score_host, int *steps_host, int *done_host)
{
    const size_t bytes = q8i_beam_state_bytes(max_steps);
    BeamState *h = (BeamState *)malloc(bytes);
    if (!h) return q8_fail(ctx, Q8_ERR_DEVICE, "out of host memory");
    hipError_t e = hipMemcpyAsync(h, state, bytes, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) { free(h); return q8_fail(ctx, Q8_ERR_DEVICE, "beam read: %s", hipGetErrorString(e)); }
    parse_state(h, tokens_host, len_host, score_host, steps_host, done_host);
    free(h);
    return Q8_OK;
}
