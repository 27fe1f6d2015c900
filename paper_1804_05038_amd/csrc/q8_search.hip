// q8_search.hip -- the search around the decoder of "Pieces of Eight: 8-bit Neural Machine
// Translation": Section 3 only says that the beam is smaller than 8, so the rules are this
// library's (stated with q8_beam_update in q8nmt.h).  Everything runs on the device: the
// host never reads a score or a token inside the step loop.
#include "q8_internal.h"

// Rows of a table: out[i, :] = table[idx[i], :] (embedding lookup, Eq. 1).
__global__ __launch_bounds__(256) void gather_rows_kernel(const float *__restrict__ table, const int *__restrict__ idx,
                                                          int n, int dim, float *__restrict__ out)
{
    const int i = blockIdx.x;
    if (i >= n) return;
    const float *src = table + (size_t)idx[i] * dim;
    for (int c = threadIdx.x; c < dim; c += blockDim.x) out[(size_t)i * dim + c] = src[c];
}

// Device-resident search state.  Hypotheses are kept as back-pointers: link[t][q] =
// (parent slot << 24) | token of live slot q after step t, so a step costs O(beam) and the
// token sequences are rebuilt on the host when the result is read.
struct BeamState {
    int n_live, b_live, step, done;
    int have_fin, fin_len, fin_parent, max_steps;
    float fin_score;
    int beam;
    float score[Q8_MAX_BEAM];
    int last[Q8_MAX_BEAM];
    int link[1];            // [max_steps][Q8_MAX_BEAM]
};

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

__global__ __launch_bounds__(256) void beam_init_kernel(BeamInitArgs a)
{
    BeamState *st = a.st;
    if (threadIdx.x == 0) {
        st->n_live = 1; st->b_live = a.beam; st->step = 0; st->done = 0;
        st->have_fin = 0; st->fin_len = 0; st->fin_parent = 0; st->max_steps = a.max_steps; st->beam = a.beam;
        st->fin_score = -INFINITY;
        for (int b = 0; b < Q8_MAX_BEAM; ++b) { st->score[b] = b == 0 ? 0.0f : -INFINITY; st->last[b] = 0; }
    }
    // every slot starts from the initial state and the embedding of token 0 (slots beyond
    // the first are not live; they only need finite contents)
    for (int e = threadIdx.x; e < a.beam * a.E; e += blockDim.x) a.y_emb[e] = a.E_tgt[e % a.E];
    for (int e = threadIdx.x; e < a.beam * a.H; e += blockDim.x) a.s[e] = a.s0[e % a.H];
}

struct BeamUpdateArgs {
    BeamState *st;
    const float *topk_logp;
    const int *topk_idx;
    const float *s_step, *E_tgt;
    float *y_emb, *s_next;
    int n, k, E, H;
};

// key: larger score first, then lower parent, then lower token id
__device__ __forceinline__ unsigned long long cand_key(float score, int parent, int token)
{
    unsigned u = __float_as_uint(score + 0.0f);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((unsigned long long)u << 32) | ((unsigned)(15 - parent) << 20) | (unsigned)(0xFFFFF - token);
}

// One block.  Wave 0 selects the b_live best continuations and rewrites the state; all
// threads then gather the surviving decoder states and the embeddings of the new tokens.
__global__ __launch_bounds__(256) void beam_update_kernel(BeamUpdateArgs a)
{
    __shared__ int s_parent[Q8_MAX_BEAM], s_token[Q8_MAX_BEAM];
    __shared__ float s_score[Q8_MAX_BEAM];
    __shared__ int s_skip;
    BeamState *st = a.st;
    const int tid = threadIdx.x, lane = tid & 63;
    const int max_steps = st->max_steps;
    if (tid < 64) {
        const int n_live = st->n_live, b_live = st->b_live, step = st->step;
        const bool skip = st->done != 0;
        if (!skip) {
            int *link = st->link + (size_t)step * Q8_MAX_BEAM;
            // two candidates per lane: c = lane, lane + 64 over [n_live x k]
            unsigned long long key[2];
            float csc[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int c = lane + 64 * t;
                key[t] = 0ull;
                csc[t] = -INFINITY;
                if (c < n_live * a.k) {
                    const int b = c / a.k;
                    const float sc = st->score[b] + a.topk_logp[c];
                    csc[t] = sc;
                    key[t] = cand_key(sc, b, a.topk_idx[c]);
                }
            }
            const int take = min(b_live, n_live * a.k);
            int n_new = 0, b_left = b_live;
            int have_fin = st->have_fin, fin_len = st->fin_len, fin_parent = st->fin_parent;
            float fin_score = st->fin_score;
            for (int r = 0; r < take; ++r) {
                const unsigned long long best = wave_max_u64(key[0] > key[1] ? key[0] : key[1]);
                const int parent = 15 - (int)((best >> 20) & 0xF);
                const int token = 0xFFFFF - (int)(best & 0xFFFFF);
                // the owner lane supplies the exact score
                float sc = -INFINITY;
                if (key[0] == best) { sc = csc[0]; key[0] = 0ull; }
                if (key[1] == best) { sc = csc[1]; key[1] = 0ull; }
                sc = wave_max_f(sc);
                if (token == 0) {                      // end of sentence: the hypothesis is finished
                    if (!have_fin || sc > fin_score) {
                        have_fin = 1; fin_score = sc; fin_len = step; fin_parent = parent;
                    }
                    --b_left;
                } else {
                    if (lane == 0) { s_score[n_new] = sc; s_token[n_new] = token; s_parent[n_new] = parent; }
                    ++n_new;
                }
            }
            if (lane == 0) {
                for (int q = 0; q < Q8_MAX_BEAM; ++q) {
                    st->score[q] = q < n_new ? s_score[q] : -INFINITY;
                    st->last[q] = q < n_new ? s_token[q] : 0;
                    if (q < n_new) link[q] = (s_parent[q] << 24) | s_token[q];
                    if (q >= n_new) {               // dead slots repeat survivor 0: finite data for the next step
                        s_parent[q] = n_new ? s_parent[0] : 0;
                        s_token[q] = n_new ? s_token[0] : 0;
                    }
                }
                st->have_fin = have_fin; st->fin_score = fin_score; st->fin_len = fin_len; st->fin_parent = fin_parent;
                st->n_live = n_new; st->b_live = b_left; st->step = step + 1;
                if (b_left == 0 || n_new == 0 || step + 1 >= max_steps) st->done = 1;
            }
        }
        if (lane == 0) s_skip = skip;
    }
    __syncthreads();
    if (s_skip) return;
    // Gather the surviving decoder states and the embeddings of the new tokens (slots beyond
    // the survivors repeat survivor 0).  All loads of a thread are issued before its stores.
    if (((a.H | a.E) & 3) == 0) {
        const int H4 = a.H >> 2, E4 = a.E >> 2, nH4 = a.n * H4, total4 = nH4 + a.n * E4;
        for (int base = tid; base < total4; base += 256 * 8) {
            float4 v[8];
            float4 *dst[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + 256 * u;
                dst[u] = nullptr;
                if (idx < nH4) {
                    const int q = idx / H4, c = idx - q * H4;
                    v[u] = ((const float4 *)(a.s_step + (size_t)s_parent[q] * a.H))[c];
                    dst[u] = (float4 *)a.s_next + idx;
                } else if (idx < total4) {
                    const int r = idx - nH4, q = r / E4, c = r - q * E4;
                    v[u] = ((const float4 *)(a.E_tgt + (size_t)s_token[q] * a.E))[c];
                    dst[u] = (float4 *)a.y_emb + r;
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (dst[u]) *dst[u] = v[u];
        }
    } else {
        for (int e = tid; e < a.n * a.H; e += blockDim.x) {
            const int q = e / a.H, c = e - q * a.H;
            a.s_next[e] = a.s_step[(size_t)s_parent[q] * a.H + c];
        }
        for (int e = tid; e < a.n * a.E; e += blockDim.x) {
            const int q = e / a.E, c = e - q * a.E;
            a.y_emb[e] = a.E_tgt[(size_t)s_token[q] * a.E + c];
        }
    }
}

// =================================================================== host launchers ==

q8_status q8i_gather_rows(q8_ctx *ctx, const float *table, const int *idx, int n, int dim, float *out)
{
    hipLaunchKernelGGL(gather_rows_kernel, dim3(n), dim3(256), 0, ctx->stream, table, idx, n, dim, out);
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

q8_status q8i_beam_read(q8_ctx *ctx, const void *state, int max_steps, int32_t *tokens_host, int *len_host,
                        float *score_host, int *steps_host, int *done_host)
{
    const size_t bytes = q8i_beam_state_bytes(max_steps);
    BeamState *h = (BeamState *)malloc(bytes);
    if (!h) return q8_fail(ctx, Q8_ERR_DEVICE, "out of host memory");
    hipError_t e = hipMemcpyAsync(h, state, bytes, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) { free(h); return q8_fail(ctx, Q8_ERR_DEVICE, "beam read: %s", hipGetErrorString(e)); }
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
    for (int t = len - 1; t >= 0; --t) {          // follow the back-pointers from the last token
        const int e = h->link[(size_t)t * Q8_MAX_BEAM + slot];
        if (tokens_host) tokens_host[t] = e & 0xFFFFFF;
        slot = (e >> 24) & 0xF;
    }
    if (len_host) *len_host = len;
    if (steps_host) *steps_host = h->step;
    if (done_host) *done_host = h->done;
    free(h);
    return Q8_OK;
}
