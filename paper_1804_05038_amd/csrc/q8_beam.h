// q8_beam.h -- device-resident beam-search state and the update step, shared by the
// stand-alone update kernel and the selection kernel that can run it in its last block.
// Section 3 of "Pieces of Eight: 8-bit Neural Machine Translation" only says that the beam
// is smaller than 8; the rules are stated with q8_beam_update in q8nmt.h.
#pragma once

#include "q8_internal.h"

// Device-resident search state.  Hypotheses are kept as back-pointers: link[t][q] =
// (parent slot << 24) | token of live slot q after step t, so a step costs O(beam) and the
// token sequences are rebuilt on the host when the result is read.
struct BeamState {
    int n_live, b_live, step, done;
    int have_fin, fin_len, fin_parent, max_steps;
    float fin_score;
    int beam;
    int gathered;           // 1 if the last update ran (and gathered the next step's inputs), 0 if the search was over
    float score[Q8_MAX_BEAM];
    int last[Q8_MAX_BEAM];
    int link[1];            // [max_steps][Q8_MAX_BEAM]
};

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

__device__ __forceinline__ void beam_gather(const BeamUpdateArgs &a, const int *s_parent, const int *s_token);

// One block of 256 threads.  Wave 0 selects the b_live best continuations and rewrites the
// state; all threads then gather the surviving decoder states and the embeddings of the new
// tokens.  COHERENT: the top-k tables were written by other blocks of the same kernel with
// device-coherent stores and are read with device-coherent loads.
template <bool COHERENT>
__device__ __forceinline__ void beam_update_body(const BeamUpdateArgs &a)
{
    __shared__ int s_parent[Q8_MAX_BEAM], s_token[Q8_MAX_BEAM];
    __shared__ float s_score[Q8_MAX_BEAM];
    __shared__ int s_skip;
    BeamState *st = a.st;
    const int tid = threadIdx.x, lane = tid & 63;
    if (tid < 64) {
        // Everything the selection needs is requested at once, before any of it is looked at:
        // the state words, and this lane's two candidates of the [n x k] tables (whether their
        // hypothesis is live is decided afterwards).
        float lp[2], sc0[2];
        int tk[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int c = lane + 64 * t;
            lp[t] = 0.0f; tk[t] = 0; sc0[t] = 0.0f;
            if (c < a.n * a.k) {
                lp[t] = COHERENT ? __hip_atomic_load(a.topk_logp + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                 : a.topk_logp[c];
                tk[t] = COHERENT ? __hip_atomic_load(a.topk_idx + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                 : a.topk_idx[c];
                sc0[t] = st->score[c / a.k];
            }
        }
        const int n_live = st->n_live, b_live = st->b_live, step = st->step, max_steps = st->max_steps;
        const bool skip = st->done != 0;
        int have_fin = st->have_fin, fin_len = st->fin_len, fin_parent = st->fin_parent;
        float fin_score = st->fin_score;
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
                    const float sc = sc0[t] + lp[t];
                    csc[t] = sc;
                    key[t] = cand_key(sc, c / a.k, tk[t]);
                }
            }
            const int take = min(b_live, n_live * a.k);
            int n_new = 0, b_left = b_live;
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
        if (lane == 0) { s_skip = skip; st->gathered = skip ? 0 : 1; }
    }
    __syncthreads();
    if (s_skip) return;
    beam_gather(a, s_parent, s_token);
}

// Gathers the surviving decoder states and the embeddings of the new tokens: slot q of the
// next step continues slot s_parent[q] with token s_token[q] (slots beyond the survivors
// repeat survivor 0).  All loads of a thread are issued before its stores.
__device__ __forceinline__ void beam_gather(const BeamUpdateArgs &a, const int *s_parent, const int *s_token)
{
    const int tid = threadIdx.x;
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
