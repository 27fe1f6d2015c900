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
    int V;                  // rows of E_tgt when known (token ids are then kept inside the table), else 0
};

// key: larger score first, then lower parent, then lower token id
__device__ __forceinline__ unsigned long long cand_key(float score, int parent, int token)
{
    unsigned u = __float_as_uint(score + 0.0f);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((unsigned long long)u << 32) | ((unsigned)(15 - parent) << 20) | (unsigned)(0xFFFFF - token);
}

__device__ __forceinline__ void beam_gather(const BeamUpdateArgs &a, const int *s_parent, const int *s_token);

// One block of 256 threads.  The (at most 128) candidates are ranked by counting: thread
// (c, half) counts how many of one half of the keys beat candidate c, so a candidate's rank is
// known after two barriers; thread 0 then walks the best b_live in order (finished hypotheses
// leave the beam, the others become the next step's slots) and rewrites the state; all threads
// gather the surviving decoder states and the embeddings of the new tokens.  COHERENT: the top-k
// tables were written by other blocks of the same kernel with device-coherent stores and are
// read with device-coherent loads.
template <bool COHERENT>
__device__ __forceinline__ void beam_update_body(const BeamUpdateArgs &a)
{
    __shared__ int s_parent[Q8_MAX_BEAM], s_token[Q8_MAX_BEAM];
    __shared__ __align__(16) unsigned long long s_key[128];
    __shared__ int s_rank[128];
    __shared__ float s_rscore[Q8_MAX_BEAM];
    __shared__ int s_rtoken[Q8_MAX_BEAM], s_rparent[Q8_MAX_BEAM];
    __shared__ int s_skip;
    BeamState *st = a.st;
    const int tid = threadIdx.x;
    // everything the selection needs is requested at once, before any of it is looked at
    const int c = tid & 127, half = tid >> 7;
    float lp = 0.0f, sc0 = 0.0f;
    int tk = 0;
    if (c < a.n * a.k) {
        lp = COHERENT ? __hip_atomic_load(a.topk_logp + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : a.topk_logp[c];
        tk = COHERENT ? __hip_atomic_load(a.topk_idx + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : a.topk_idx[c];
        sc0 = st->score[c / a.k];
    }
    const int n_live = st->n_live, b_live = st->b_live, step = st->step, max_steps = st->max_steps;
    const bool skip = st->done != 0;
    const int have_fin0 = st->have_fin, fin_len0 = st->fin_len, fin_parent0 = st->fin_parent;
    const float fin_score0 = st->fin_score;
    const int ncand = skip ? 0 : n_live * a.k;
    const int take = min(b_live, ncand);
    unsigned long long key = 0ull;
    float csc = -INFINITY;
    if (c < ncand) {
        csc = sc0 + lp;
        key = cand_key(csc, c / a.k, tk);
    }
    if (half == 0) {
        s_key[c] = key;
        s_rank[c] = 0;
    }
    __syncthreads();
    if (c < ncand) {
        // keys are distinct (they contain parent and token), so the counts are a permutation
        const int lo = half * 64;
        int cnt = 0;
#pragma unroll 4
        for (int u = lo; u < lo + 64 && u < ncand; u += 2) {
            const ulonglong2 p2 = *(const ulonglong2 *)&s_key[u];
            cnt += (p2.x > key) + (p2.y > key);
        }
        if (cnt) atomicAdd(&s_rank[c], cnt);
    }
    __syncthreads();
    if (half == 0 && c < ncand) {
        const int r = s_rank[c];
        if (r < take) { s_rscore[r] = csc; s_rtoken[r] = tk; s_rparent[r] = c / a.k; }
    }
    __syncthreads();
    __shared__ float s_nscore[Q8_MAX_BEAM];
    __shared__ int s_nnew;
    if (tid == 0) {
        int n_new = 0;
        if (!skip) {
            int have_fin = have_fin0, fin_len = fin_len0, fin_parent = fin_parent0;
            float fin_score = fin_score0;
            int b_left = b_live;
            for (int r = 0; r < take; ++r) {
                const float sc = s_rscore[r];
                int token = s_rtoken[r], parent = s_rparent[r];
                // non-finite scores can leave fewer than k valid candidates per hypothesis: whatever
                // the tables then hold, the gather below stays inside s_step and E_tgt
                if (a.V > 0 && (unsigned)token >= (unsigned)a.V) token = 0;
                if ((unsigned)parent >= (unsigned)a.n) parent = 0;
                if (token == 0) {                      // end of sentence: the hypothesis is finished
                    if (!have_fin || sc > fin_score) {
                        have_fin = 1; fin_score = sc; fin_len = step; fin_parent = parent;
                    }
                    --b_left;
                } else {
                    s_nscore[n_new] = sc; s_token[n_new] = token; s_parent[n_new] = parent;
                    ++n_new;
                }
            }
            st->have_fin = have_fin; st->fin_score = fin_score; st->fin_len = fin_len; st->fin_parent = fin_parent;
            st->n_live = n_new; st->b_live = b_left; st->step = step + 1;
            if (b_left == 0 || n_new == 0 || step + 1 >= max_steps) st->done = 1;
        }
        s_nnew = n_new;
        s_skip = skip;
        st->gathered = skip ? 0 : 1;
    }
    __syncthreads();
    if (!skip && tid < Q8_MAX_BEAM) {                   // slot tid of the state, one thread each
        const int n_new = s_nnew, q = tid;
        st->score[q] = q < n_new ? s_nscore[q] : -INFINITY;
        st->last[q] = q < n_new ? s_token[q] : 0;
        if (q < n_new) st->link[(size_t)step * Q8_MAX_BEAM + q] = (s_parent[q] << 24) | s_token[q];
    }
    __syncthreads();
    if (!skip && tid < Q8_MAX_BEAM && tid >= s_nnew) {  // dead slots repeat survivor 0: finite data for the next step
        const int p0 = s_nnew ? s_parent[0] : 0, t0 = s_nnew ? s_token[0] : 0;
        s_parent[tid] = p0;
        s_token[tid] = t0;
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
        // Thread tid moves 16-byte piece tid (+ 256 per pass) of every row: eight state rows and eight
        // embedding rows per pass, rows past n repeating row n - 1 and pieces past a row's end repeating
        // its last piece (same value to the same place).  So there is no division in the addressing and no
        // branch around a load or a store: inside a branch the compiler waits for each of them on the
        // spot, and a thread's loads and stores become as many memory round trips in a row.
        // (Moved as plain 16-byte vectors: nothing here looks inside the values.)
        const int H4 = a.H >> 2, E4 = a.E >> 2;
        const v4i *s4 = (const v4i *)a.s_step, *e4 = (const v4i *)a.E_tgt;
        v4i *sn4 = (v4i *)a.s_next, *y4 = (v4i *)a.y_emb;
        for (int c0 = 0; c0 < max(H4, E4); c0 += 256) {
            const int ch = min(c0 + tid, H4 - 1), ce = min(c0 + tid, E4 - 1);
            v4i vs[Q8_MAX_BEAM], ve[Q8_MAX_BEAM];
#pragma unroll
            for (int q = 0; q < Q8_MAX_BEAM; ++q) {
                const int qq = min(q, a.n - 1);
                vs[q] = s4[(size_t)s_parent[qq] * H4 + ch];
                ve[q] = e4[(size_t)s_token[qq] * E4 + ce];
            }
#pragma unroll
            for (int q = 0; q < Q8_MAX_BEAM; ++q) {
                const int qq = min(q, a.n - 1);
                sn4[(size_t)qq * H4 + ch] = vs[q];
                y4[(size_t)qq * E4 + ce] = ve[q];
            }
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
