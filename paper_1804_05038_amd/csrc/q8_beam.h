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
    // Optional (all or none; E / 4 + ldy / 16 + lds / 16 <= 256): the codes of the gathered rows travel with
    // them, so that the next decoder step need not quantize its inputs again.  Eq [V x ldy], Es [V]: every
    // embedding row quantized on its own maximum; sq_in [n x lds], ss_in [n]: the codes of s_step as the readout
    // quantized them.  Out: yq_out [n x ldy], ys_out [n] for y_emb; sq_out [n x lds], ss_out [n] for s_next.
    const int8_t *Eq, *sq_in;
    const float *Es, *ss_in;
    int8_t *yq_out, *sq_out;
    float *ys_out, *ss_out;
    int ldy, lds;
    // Optional: the decision goes to blocks that compute GRU r of the next step from it (see out_select_kernel).
    // xg: gate_blocks x 8 8-byte words, zero on entry; word 8 b + q = (present bit, parent slot, token) of slot q
    // for block b, which clears it.  s_next may then be NULL (no state rows are gathered), and with Eq given
    // sq_in / sq_out may be NULL (lds = 0: only the embedding rows' codes travel).
    unsigned long long *xg;
    int gate_blocks;
};

// key: larger score first, then lower parent, then lower token id
__device__ __forceinline__ unsigned long long cand_key(float score, int parent, int token)
{
    unsigned u = __float_as_uint(score + 0.0f);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((unsigned long long)u << 32) | ((unsigned)(15 - parent) << 20) | (unsigned)(0xFFFFF - token);
}

// What a search step reads of the state before it decides (lane q & 7 holds the score of slot q).
struct BeamStateRead {
    float sc_slot, fin_score;
    int n_live, b_live, step, max_steps, done, have_fin;
};
__device__ __forceinline__ BeamStateRead beam_state_read(const BeamState *st, int lane)
{
    BeamStateRead r;
    r.sc_slot = st->score[lane & (Q8_MAX_BEAM - 1)];
    r.n_live = st->n_live; r.b_live = st->b_live; r.step = st->step; r.max_steps = st->max_steps;
    r.done = st->done; r.have_fin = st->have_fin; r.fin_score = st->fin_score;
    return r;
}

__device__ __forceinline__ void beam_gather(const BeamUpdateArgs &a, const int *s_parent, const int *s_token);
template <bool GIVEN>
__device__ __forceinline__ void beam_update_body(const BeamUpdateArgs &a, const float (&lp_in)[2], const int (&tk_in)[2],
                                                 const BeamStateRead &pre);
// The tables as they lie in memory (written by an earlier kernel).
__device__ __forceinline__ void beam_update_body(const BeamUpdateArgs &a)
{
    const float no_lp[2] = {0.0f, 0.0f};
    const int no_tk[2] = {0, 0};
    const BeamStateRead none = {};
    beam_update_body<false>(a, no_lp, no_tk, none);
}

// One block of at least 64 threads.  The decisions of a search step are taken by the block's first
// wave alone, without barriers: lane L holds candidates L and L + 64 of the (at most 128) n_live x k
// candidates as 64-bit keys (score, parent, token); b_live rounds of a wave-wide maximum hand the
// best b_live of them, in order, to lanes 0, 1, ...; ballots over those lanes give every survivor its
// slot, the number of hypotheses that ended and the best of them; lane q then writes slot q of the
// state.  Only then does the block meet, and all threads gather the surviving decoder states and the
// embeddings of the new tokens.  GIVEN: lanes of the first wave bring their two candidates (entries
// lane and lane + 64 of the top-k tables, the last entry repeated past the end) in lp_in / tk_in
// and what beam_state_read returned (requested while they waited for the candidates), and
// neither the tables nor the state are read here.
template <bool GIVEN>
__device__ __forceinline__ void beam_update_body(const BeamUpdateArgs &a, const float (&lp_in)[2], const int (&tk_in)[2],
                                                 const BeamStateRead &pre)
{
    __shared__ int s_parent[Q8_MAX_BEAM], s_token[Q8_MAX_BEAM];
    __shared__ int s_skip;
    BeamState *st = a.st;
    const int tid = threadIdx.x;
    if (tid < 64) {
        const int lane = tid;
        // everything the decisions need is requested at once, before any of it is looked at
        float lp[2];
        int tk[2];
        const int nk = a.n * a.k;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int c = min(lane + 64 * u, nk - 1);      // (a lane past the tables reads their last entry and drops it)
            lp[u] = GIVEN ? lp_in[u] : a.topk_logp[c];
            tk[u] = GIVEN ? tk_in[u] : a.topk_idx[c];
        }
        const BeamStateRead sr = GIVEN ? pre : beam_state_read(st, lane);
        const float sc_slot = sr.sc_slot;                                // lane q < 8: score of slot q
        const int n_live = sr.n_live, b_live = sr.b_live, step = sr.step, max_steps = sr.max_steps;
        const bool skip = sr.done != 0;
        const int have_fin0 = sr.have_fin;
        const float fin_score0 = sr.fin_score;
        const int ncand = skip ? 0 : n_live * a.k;
        const int take = min(b_live, ncand);
        // candidate c = parent * k + rank in the parent's list; parent = floor((c + 0.5) / k) in float
        // (the quotient is at least 1 / (2 k) away from an integer, far more than the reciprocal's error)
        const float rk = __builtin_amdgcn_rcpf((float)a.k);
        unsigned long long key[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int c = lane + 64 * u;
            const int p = (int)(((float)c + 0.5f) * rk);
            const float sp = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (p & (Q8_MAX_BEAM - 1)), __float_as_int(sc_slot)));
            key[u] = c < ncand ? cand_key(sp + lp[u], p, tk[u]) : 0ull;
        }
        // the best `take` keys, in order, into lanes 0 .. take - 1 (keys are distinct: they contain parent and
        // token).  Rounds of a wave-wide maximum: counting ranks through LDS was measured slower (1.3 against 1.0 us).
        unsigned long long mine = 0ull;
        for (int r = 0; r < take; ++r) {
            const unsigned long long best = wave_max_u64(key[0] > key[1] ? key[0] : key[1]);
            if (key[0] == best) key[0] = 0ull;
            if (key[1] == best) key[1] = 0ull;
            if (lane == r) mine = best;
        }
        const bool kept = lane < take;
        unsigned ub = (unsigned)(mine >> 32);
        ub = (ub & 0x80000000u) ? (ub & 0x7fffffffu) : ~ub;
        const float sc = __uint_as_float(ub);
        int parent = 15 - (int)((mine >> 20) & 0xFFFu), token = 0xFFFFF - (int)(mine & 0xFFFFFu);
        // non-finite scores can leave fewer than k valid candidates per hypothesis: whatever the tables
        // then hold, the gather below stays inside s_step and E_tgt
        if (a.V > 0 && (unsigned)token >= (unsigned)a.V) token = 0;
        if ((unsigned)parent >= (unsigned)a.n) parent = 0;
        const unsigned long long ended = __ballot(kept && token == 0), alive = __ballot(kept && token != 0);
        const int n_new = __popcll(alive), b_left = b_live - __popcll(ended);
        const int slot = __popcll(alive & ((1ull << lane) - 1ull));
        if (kept && token != 0) { s_parent[slot] = parent; s_token[slot] = token; }
        // the hypotheses that ended: the first in order has the highest score; it replaces the remembered
        // one only if it is better (ties to the earlier)
        const int first_end = ended ? (int)__ffsll((long long)ended) - 1 : 0;
        const float end_sc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sc), first_end));
        const int end_parent = __builtin_amdgcn_readlane(parent, first_end);
        const int first_alive = alive ? (int)__ffsll((long long)alive) - 1 : 0;
        const int parent0 = n_new ? __builtin_amdgcn_readlane(parent, first_alive) : 0;
        const int token0 = n_new ? __builtin_amdgcn_readlane(token, first_alive) : 0;
        __builtin_amdgcn_wave_barrier();
        if (!skip) {
            // slot q of the new state, lane q: its score and last token come from the survivor that took slot q
            if (kept && token != 0) {
                st->score[slot] = sc;
                st->last[slot] = token;
                st->link[(size_t)step * Q8_MAX_BEAM + slot] = (parent << 24) | token;
            }
            if (lane >= n_new && lane < Q8_MAX_BEAM) { st->score[lane] = -INFINITY; st->last[lane] = 0; }
            if (lane == 0) {
                if (ended && (!have_fin0 || end_sc > fin_score0)) {
                    st->have_fin = 1; st->fin_score = end_sc; st->fin_len = step; st->fin_parent = end_parent;
                }
                st->n_live = n_new; st->b_live = b_left; st->step = step + 1;
                if (b_left == 0 || n_new == 0 || step + 1 >= max_steps) st->done = 1;
            }
        }
        if (lane == 0) { st->gathered = skip ? 0 : 1; s_skip = skip; }
        // dead slots repeat survivor 0 (slot 0 of the tables if nothing survived): finite data for the next step
        if (!skip && lane >= n_new && lane < Q8_MAX_BEAM) {
            s_parent[lane] = parent0;
            s_token[lane] = token0;
        }
        if (a.xg) {
            // (the entries of s_parent / s_token were written by lanes of this wave)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            for (int w = lane; w < a.gate_blocks * Q8_MAX_BEAM; w += 64) {
                const int q = w & (Q8_MAX_BEAM - 1);
                const int par = skip ? 0 : s_parent[q], tok = skip ? 0 : s_token[q];
                if (q < a.n)
                    __hip_atomic_store(a.xg + w, (1ull << 63) | ((unsigned long long)(unsigned)par << 32) | (unsigned)tok,
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
    __syncthreads();
    if (s_skip) return;
    beam_gather(a, s_parent, s_token);
}

// Gathers the surviving decoder states and the embeddings of the new tokens: slot q of the
// next step continues slot s_parent[q] with token s_token[q] (slots beyond the survivors
// repeat survivor 0).  All loads of a thread are issued before its stores.
// Thread tid moves 16-byte piece tid (+ 256 per pass) of every row: ROWS state rows and ROWS
// embedding rows per pass, rows past n repeating row n - 1 and pieces past a row's end repeating
// its last piece (same value to the same place).  So there is no division in the addressing and no
// branch around a load or a store: inside a branch the compiler waits for each of them on the
// spot, and a thread's loads and stores become as many memory round trips in a row.
// (Moved as plain 16-byte vectors: nothing here looks inside the values.)
template <int ROWS, bool STATES>
__device__ __forceinline__ void beam_gather_rows(const BeamUpdateArgs &a, const int *s_parent, const int *s_token)
{
    const int tid = threadIdx.x;
    const int H4 = a.H >> 2, E4 = a.E >> 2;
    const v4i *s4 = (const v4i *)a.s_step;
    v4i *sn4 = (v4i *)a.s_next;
    // The embedding rows are shorter than a pass of 256 pieces; the threads past their end move the rows'
    // codes instead (first pass only): pieces [E4, E4 + ldy / 16) of a "row" are the embedding row's codes,
    // the next lds / 16 the codes of the parent's state.  Each thread has one source and one destination
    // (base, pieces per row, piece) and, per row, the index its source is gathered by.
    const int Y16 = a.Eq ? a.ldy >> 4 : 0, S16 = a.Eq ? a.lds >> 4 : 0;
    const bool is_y = tid >= E4 && tid < E4 + Y16, is_s = tid >= E4 + Y16 && tid < E4 + Y16 + S16;
    const v4i *src0 = is_y ? (const v4i *)a.Eq : is_s ? (const v4i *)a.sq_in : (const v4i *)a.E_tgt;
    v4i *dst0 = is_y ? (v4i *)a.yq_out : is_s ? (v4i *)a.sq_out : (v4i *)a.y_emb;
    const int pitch0 = is_y ? Y16 : is_s ? S16 : E4;
    const int piece0 = is_y ? tid - E4 : is_s ? tid - E4 - Y16 : min(tid, E4 - 1);
    // their scales: thread q & 7 of every wave fetches those of row q (the same words for all waves), thread q stores them
    // (unconditional loads: without codes they read the first floats of the tables and drop them)
    const int qs = min(tid & 7, a.n - 1);
    const float ys = *(a.Eq ? a.Es + s_token[qs] : a.E_tgt), ss = *(a.Eq && a.ss_in ? a.ss_in + s_parent[qs] : a.s_step);
    for (int c0 = 0; c0 < (STATES ? max(H4, E4) : E4); c0 += 256) {
        const int ch = min(c0 + tid, H4 - 1);
        const bool first = c0 == 0;
        const v4i *src = first ? src0 : (const v4i *)a.E_tgt;
        v4i *dst = first ? dst0 : (v4i *)a.y_emb;
        const int pitch = first ? pitch0 : E4, piece = first ? piece0 : min(c0 + tid, E4 - 1);
        const bool by_parent = first && is_s;
        v4i vs[ROWS], ve[ROWS];
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
            const int qq = min(q, a.n - 1);
            const int par = s_parent[qq], tok = s_token[qq];
            if (STATES) vs[q] = s4[(size_t)par * H4 + ch];
            ve[q] = src[(size_t)(by_parent ? par : tok) * pitch + piece];
        }
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
            const int qq = min(q, a.n - 1);
            if (STATES) sn4[(size_t)qq * H4 + ch] = vs[q];
            dst[(size_t)qq * pitch + piece] = ve[q];
        }
    }
    if (a.Eq && tid < a.n) {
        a.ys_out[tid] = ys;
        if (a.ss_out) a.ss_out[tid] = ss;
    }
}

__device__ __forceinline__ void beam_gather(const BeamUpdateArgs &a, const int *s_parent, const int *s_token)
{
    const int tid = threadIdx.x;
    if (((a.H | a.E) & 3) == 0) {
        // (a compute unit moves these rows at about 50 GB/s: rows that only repeat the last one cost as much
        // as the others, so the row count follows the beam in three steps)
        if (!a.s_next) {
            if (a.n <= 4) beam_gather_rows<4, false>(a, s_parent, s_token);
            else if (a.n <= 6) beam_gather_rows<6, false>(a, s_parent, s_token);
            else beam_gather_rows<Q8_MAX_BEAM, false>(a, s_parent, s_token);
        } else if (a.n <= 4) beam_gather_rows<4, true>(a, s_parent, s_token);
        else if (a.n <= 6) beam_gather_rows<6, true>(a, s_parent, s_token);
        else beam_gather_rows<Q8_MAX_BEAM, true>(a, s_parent, s_token);
    } else {
        for (int e = tid; a.s_next && e < a.n * a.H; e += blockDim.x) {
            const int q = e / a.H, c = e - q * a.H;
            a.s_next[e] = a.s_step[(size_t)s_parent[q] * a.H + c];
        }
        for (int e = tid; e < a.n * a.E; e += blockDim.x) {
            const int q = e / a.E, c = e - q * a.E;
            a.y_emb[e] = a.E_tgt[(size_t)s_token[q] * a.E + c];
        }
    }
}

// The search step's arguments for sentence s of a panel.
__device__ __forceinline__ BeamUpdateArgs beam_batch_sentence(const BeamBatchArgs &b, int s)
{
    const size_t slot = (size_t)s * b.beam;
    BeamUpdateArgs a = {(BeamState *)(b.states + (size_t)s * b.stride), b.topk_logp + slot * b.k, b.topk_idx + slot * b.k,
                        b.s_step + slot * b.H, b.E_tgt, b.y_emb + slot * b.E, b.s_next + slot * b.H, b.beam, b.k, b.E, b.H, b.V};
    if (b.Eq) {
        a.Eq = b.Eq; a.Es = b.Es; a.ldy = b.ldy; a.lds = b.lds;
        a.sq_in = b.sq_in + slot * b.lds; a.ss_in = b.ss_in + slot;
        a.yq_out = b.yq_out + slot * b.ldy; a.ys_out = b.ys_out + slot;
        a.sq_out = b.sq_out + slot * b.lds; a.ss_out = b.ss_out + slot;
    }
    return a;
}
