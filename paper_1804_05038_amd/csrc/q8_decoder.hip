// q8_decoder.hip -- the float part of the attention of Eq. 5-6 and the first layer of the
// output network g of Eq. 2 ("Pieces of Eight: 8-bit Neural Machine Translation").
#include "q8_internal.h"
#include "q8_gemv_fast.h"

// ======================================================================== attention ==

struct AttArgs {
    const float *P, *enc_h, *a, *v;
    float *e, *alpha, *ctx;
    unsigned *counters;     // one arrival counter per hypothesis (cstride words apart), zero on entry and on exit
    int cstride;
    int l, A, C;
    // several sentences side by side: hypothesis b belongs to sentence b / beam, whose rows of
    // P and enc_h are [sent_off[s], sent_off[s + 1]); NULL = one sentence of l positions
    const int *sent_off;
    int beam, lde;          // lde: row pitch of e and alpha
    // optional: codes [n x ldq] (bytes [C, ldq) zero) and scales [n] of the context vectors, so that
    // the consumer (GRU q) does not quantize them again; needs C even, ldq <= 2 ATT_PAIRS blockDim
    int8_t *ctx_q;
    float *ctx_qscale;
    int ldq;
    // attention_split_kernel: per hypothesis ATTS_L tagged energies then ATTS_L tagged slice maxima
    // (8-byte words: value bits below, 1 above when present), zero on entry and left set; the flag a
    // wait that gave up sets, the bound of a wait in polls, column pairs per block and its reciprocal
    unsigned long long *xchg;
    unsigned *wait_err;
    int spin_limit, ppb;
    float inv_ppb;
};

// Rows of P and enc_h that hypothesis b attends over, and how many.
__device__ __forceinline__ int att_sentence(const AttArgs &a, int b, const float *&P, const float *&enc_h)
{
    P = a.P;
    enc_h = a.enc_h;
    if (!a.sent_off) return a.l;
    const int s = b / a.beam, o = a.sent_off[s];
    P += (size_t)o * a.A;
    enc_h += (size_t)o * a.C;
    return a.sent_off[s + 1] - o;
}

#define ATT_MAX_THREADS 1024
#define ATT_PAIRS 4
// Run by the last block to arrive for hypothesis b (all its l energies are in a.e, written
// with device-coherent stores): softmax over the energies in one wave, then the context
// vector H_t (Eq. 5), a thread owning two adjacent columns and walking the source positions
// in order.  Sums run in double; every stored value is rounded once.
template <bool HANDOFF>
__device__ __forceinline__ void att_finish(const AttArgs &a, int b, int l, const float *enc_h, double *s_alpha)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nt = blockDim.x;
    if (wave == 0) {
        const float *e = a.e + (size_t)b * a.lde;
        float mx = -INFINITY;
        for (int t = lane; t < l; t += 64) {
            // (inside the energy kernel the energies were written by other blocks of the same launch: device-coherent
            // loads; in a launch of its own they are ordinary data)
            const float ev = HANDOFF ? __hip_atomic_load(e + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : e[t];
            s_alpha[t] = (double)ev;
            mx = fmaxf(mx, ev);
        }
        mx = wave_max_f(mx);
        double Z = 0.0, ex0 = 0.0;               // ex0: the lane's first term, kept for the division below
        for (int t = lane; t < l; t += 64) {
            const double ex = q8_exp_d(fmax(s_alpha[t] - (double)mx, -700.0));
            if (t == lane) ex0 = ex;
            Z += ex;
        }
        Z = wave_sum_d(Z);
        for (int t = lane; t < l; t += 64) {
            const float al = (float)((t == lane ? ex0 : q8_exp_d(fmax(s_alpha[t] - (double)mx, -700.0))) / Z);
            s_alpha[t] = (double)al;          // the weight as the context sum uses it: converted once, not per column
            if (a.alpha) a.alpha[(size_t)b * a.lde + t] = al;
        }
        if (HANDOFF && lane == 0) __hip_atomic_store(&a.counters[b * a.cstride], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (a.ctx_q) {
        // up to ATT_PAIRS pairs of columns per thread, kept in registers: the vector's codes come from
        // the rounded values (C <= 2 ATT_PAIRS blockDim)
        __shared__ float s_m[ATT_MAX_THREADS / 64];
        float f[ATT_PAIRS][2];
        float m = 0.0f;
#pragma unroll
        for (int it = 0; it < ATT_PAIRS; ++it) {
            const int c = (it * nt + tid) * 2;
            f[it][0] = f[it][1] = 0.0f;
            if (c < a.C) {
                double s0 = 0.0, s1 = 0.0;
                const float *h = enc_h + c;
#pragma unroll 10
                for (int t = 0; t < l; ++t) {
                    const float2 hv = *(const float2 *)(h + (size_t)t * a.C);
                    const double al = s_alpha[t];
                    s0 += al * (double)hv.x;
                    s1 += al * (double)hv.y;
                }
                f[it][0] = (float)s0;
                f[it][1] = (float)s1;
                *(float2 *)(a.ctx + (size_t)b * a.C + c) = make_float2(f[it][0], f[it][1]);
            }
            m = fmaxf(m, fmaxf(fabsf(f[it][0]), fabsf(f[it][1])));
        }
        m = wave_max_f(m);
        if (lane == 0) s_m[wave] = m;
        __syncthreads();
        m = 0.0f;
        for (int w = 0; w < nt / 64; ++w) m = fmaxf(m, s_m[w]);
        float scale, inv;
        q8_scale_of(m, scale, inv);
#pragma unroll
        for (int it = 0; it < ATT_PAIRS; ++it) {
            const int c = (it * nt + tid) * 2;
            if (c < a.ldq) *(short *)(a.ctx_q + (size_t)b * a.ldq + c) = (short)q8_pack2(f[it][0], f[it][1], inv);   // zeros past C
        }
        if (tid == 0) a.ctx_qscale[b] = scale;
    } else if ((a.C & 1) == 0) {
        for (int c = tid * 2; c < a.C; c += 2 * nt) {
            double s0 = 0.0, s1 = 0.0;
            const float *h = enc_h + c;
#pragma unroll 10
            for (int t = 0; t < l; ++t) {
                const float2 hv = *(const float2 *)(h + (size_t)t * a.C);
                const double al = s_alpha[t];
                s0 += al * (double)hv.x;
                s1 += al * (double)hv.y;
            }
            *(float2 *)(a.ctx + (size_t)b * a.C + c) = make_float2((float)s0, (float)s1);
        }
    } else {
        for (int c = tid; c < a.C; c += nt) {
            double s = 0.0;
            for (int t = 0; t < l; ++t) s += s_alpha[t] * (double)enc_h[(size_t)t * a.C + c];
            a.ctx[(size_t)b * a.C + c] = (float)s;
        }
    }
}

// One sentence, a handful of hypotheses: block (i, b) of 1024 threads computes one energy
// e[b, i] = sum_j v_j tanh(P[i, j] + a[b, j]) (Eq. 6), so that the l n blocks run side by side;
// the last block to arrive for hypothesis b finishes (att_finish).
#define ATT_THREADS 1024
__global__ __launch_bounds__(ATT_THREADS) void attention_kernel(AttArgs a)
{
    __shared__ double s_red[ATT_THREADS / 64];
    __shared__ double s_alpha[1024];
    __shared__ int s_last;
    const int i = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *P, *enc_h;
    const int l = att_sentence(a, b, P, enc_h);
    if (i >= l) return;                      // the grid spans the longest sentence
    const float *Pi = P + (size_t)i * a.A;
    const float *ab = a.a + (size_t)b * a.A;
    double acc = 0.0;
    for (int j = tid; j < a.A; j += ATT_THREADS) acc += (double)a.v[j] * (double)tanh_rn(Pi[j] + ab[j]);
    acc = wave_sum_d(acc);
    if (lane == 0) s_red[wave] = acc;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < ATT_THREADS / 64; ++w) tot += s_red[w];
        // Publish the energy with a device-coherent store, wait until it has been performed,
        // then count the arrival with a device-coherent atomic: the block that sees the last
        // count can read every energy with device-coherent loads, no cache flush needed.
        __hip_atomic_store(&a.e[(size_t)b * a.lde + i], (float)tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        q8_stores_performed();
        const unsigned prev = __hip_atomic_fetch_add(&a.counters[b * a.cstride], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == (unsigned)l - 1u);
    }
    __syncthreads();
    if (!s_last) return;
    att_finish<true>(a, b, l, enc_h, s_alpha);
}

// The same result without the single finishing block: every block needs all l energies of its
// hypothesis anyway, so each publishes its own as a tagged 8-byte word (value, "present") with one
// device-coherent store and polls the l words; each then derives the attention weights itself and
// sums its own slice of ceil(C / 2 / l) column pairs of the context vector (Eq. 5).  The slice's
// encoder states are requested while the energies are exchanged; once the weights are known, the
// thread that fetched an entry forms its two products (exact in double), and one thread per
// column adds them up over the positions in order, exactly the sum att_finish forms.  The scale
// of the vector's codes needs its largest magnitude: the slices' maxima are exchanged the same
// way, and every block quantizes its own slice.  Nobody pulls the l x C states through one
// compute unit, and an exchange costs a store and a poll (0.6-0.8 us) instead of store, wait,
// atomic, and a block that starts from nothing.  Timeline at l = 30, beam 5 (us after the first
// block starts): energies summed 0.9, published 1.6, all 30 seen 2.7, weights 3.2, products in
// LDS 3.6, columns summed 4.3, maxima published 4.5, seen 5.3, codes stored and last block gone
// 6.0 (the kernel with the finishing block: 8.6-8.9).
// The words stay set when the kernel ends (a block cannot know when the others have read them
// without another exchange, which would cost a microsecond at the end): the next kernel of the
// decoder step zeroes them, and the host keeps track that one does before this kernel runs again.
// All l blocks of a hypothesis must be resident together (the host checks that the whole grid is);
// every wait is bounded, a wait that gives up sets *wait_err and the block goes on with what it has
// (finite values, wrong result).  Measured and not kept: a pause before the first poll (it helped
// while the column sums were slower, 0.3 us, and does nothing now), requesting the slice before
// the energies (they are then published 0.3 us later), a departure count with the last
// block clearing the words (+ 1.2 us at the kernel's end).
#define ATTS_L 128            // source positions at most
static_assert(2 * ATTS_L * 8 == Q8_WS_ATT_XCHG_PER_HYP, "energies and maxima of a hypothesis fill its part of the header");
#define ATTS_SLICE 2304       // entries of LDS for a block's slice: l ceil(C / 2 / l) < C / 2 + l
#define ATTS_SLICE_LOADS 3    // ceil(ATTS_SLICE / ATT_THREADS)
__device__ __forceinline__ void atts_poll(const unsigned long long *w, int l, int lane, int limit, unsigned *wait_err,
                                          float &v0, float &v1)
{
    unsigned long long x0 = 0ull, x1 = 0ull;
    bool ok = false;
    for (int spin = 0; spin < limit; ++spin) {
        x0 = __hip_atomic_load(w + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);        // 128 words per hypothesis: in range
        if (l > 64) x1 = __hip_atomic_load(w + 64 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool mine = (lane >= l || (x0 >> 32) != 0ull) && (lane + 64 >= l || (x1 >> 32) != 0ull);
        if (__all(mine)) { ok = true; break; }
        __builtin_amdgcn_s_sleep(1);
    }
    if (!ok && lane == 0) __hip_atomic_store(wait_err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v0 = __uint_as_float((unsigned)x0);
    v1 = __uint_as_float((unsigned)x1);
}

__global__ __launch_bounds__(ATT_THREADS) void attention_split_kernel(AttArgs a)
{
    __shared__ double s_red[ATT_THREADS / 64];
    __shared__ double s_alpha[ATTS_L];
    __shared__ double2 s_p[ATTS_SLICE];
    __shared__ float s_m[ATT_THREADS / 64];
    __shared__ float s_sc[2];
    const int i = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l = a.l, ppb = a.ppb, C = a.C;
    unsigned long long *xe = a.xchg + (size_t)b * (Q8_WS_ATT_XCHG_PER_HYP / 8), *xm = xe + ATTS_L;

    // Eq. 6: e[b, i] = sum_j v_j tanh(P[i, j] + a[b, j])
    const float *Pi = a.P + (size_t)i * a.A;
    const float *ab = a.a + (size_t)b * a.A;
    double acc = 0.0;
    for (int j = tid; j < a.A; j += ATT_THREADS) acc += (double)a.v[j] * (double)tanh_rn(Pi[j] + ab[j]);
    acc = wave_sum_d(acc);
    if (lane == 0) s_red[wave] = acc;
    __syncthreads();
    // This block's slice of the encoder states: entry e = t ppb + q is position t, column pair i ppb + q.
    // Requested after the energy's barrier and, in the wave that publishes, after the energy is on its
    // way (the requests' address arithmetic ahead of the energy delayed it by 0.3 us); needed when the
    // weights are known.
    float2 hv[ATTS_SLICE_LOADS];
    int tv[ATTS_SLICE_LOADS];
    auto slice_request = [&]() {
        const __amdgpu_buffer_rsrc_t rh = q8_rsrc(a.enc_h, (size_t)l * C * sizeof(float));
#pragma unroll
        for (int u = 0; u < ATTS_SLICE_LOADS; ++u) {
            const int e = u * ATT_THREADS + tid;
            const int t = (int)(((float)e + 0.5f) * a.inv_ppb);      // e / ppb: exact, both far below 2^12
            const int c = 2 * (i * ppb + (e - t * ppb));
            const unsigned off = (t < l && c < C) ? ((unsigned)t * (unsigned)C + (unsigned)c) * 4u : Q8_OOB;
            hv[u] = __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(rh, (int)off, 0, 0));
            tv[u] = min(t, l - 1);
        }
    };
    if (wave != 0) slice_request();
    if (wave == 0) {
        if (lane == 0) {
            double tot = 0.0;
#pragma unroll
            for (int w = 0; w < ATT_THREADS / 64; ++w) tot += s_red[w];
            const float ev = (float)tot;
            __hip_atomic_store(xe + i, (1ull << 32) | (unsigned long long)__float_as_uint(ev), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            a.e[(size_t)b * a.lde + i] = ev;
        }
        slice_request();
        float e0, e1;
        atts_poll(xe, l, lane, a.spin_limit, a.wait_err, e0, e1);
        // softmax over the l energies, as in att_finish
        if (lane < l) s_alpha[lane] = (double)e0;
        if (lane + 64 < l) s_alpha[lane + 64] = (double)e1;
        float mx = -INFINITY;
        for (int t = lane; t < l; t += 64) mx = fmaxf(mx, (float)s_alpha[t]);
        mx = wave_max_f(mx);
        double Z = 0.0, ex0 = 0.0;
        for (int t = lane; t < l; t += 64) {
            const double ex = q8_exp_d(fmax(s_alpha[t] - (double)mx, -700.0));
            if (t == lane) ex0 = ex;
            Z += ex;
        }
        Z = wave_sum_d(Z);
        for (int t = lane; t < l; t += 64) {
            const float al = (float)((t == lane ? ex0 : q8_exp_d(fmax(s_alpha[t] - (double)mx, -700.0))) / Z);
            s_alpha[t] = (double)al;
            if (a.alpha && i == 0) a.alpha[(size_t)b * a.lde + t] = al;
        }
    }
    __syncthreads();
    // Eq. 5.  The products alpha_t h of every entry, by the thread that fetched it (exact in double: 24 x 24
    // bits), so that the sum over the positions, which has to run in order, is additions alone ...
#pragma unroll
    for (int u = 0; u < ATTS_SLICE_LOADS; ++u) {
        const int e = u * ATT_THREADS + tid;
        const double al = s_alpha[tv[u]];
        if (e < ATTS_SLICE) s_p[e] = make_double2(al * (double)hv[u].x, al * (double)hv[u].y);
    }
    __syncthreads();
    // ... by thread c < 2 ppb for column 2 i ppb + c, positions in order as att_finish adds them
    const int c = 2 * i * ppb + tid;
    const bool own = tid < 2 * ppb && c < C;
    float f = 0.0f;
    if (own) {
        const double *pc = (const double *)s_p + tid;
        double sum = 0.0;
#pragma unroll 8
        for (int t = 0; t < l; ++t) sum += pc[(size_t)t * 2 * ppb];
        f = (float)sum;
        a.ctx[(size_t)b * C + c] = f;
    }
    float m = wave_max_f(fabsf(f));
    if (lane == 0) s_m[wave] = m;
    __syncthreads();
    if (wave == 0) {
        if (lane == 0) {
            m = 0.0f;
#pragma unroll
            for (int w = 0; w < ATT_THREADS / 64; ++w) m = fmaxf(m, s_m[w]);
            __hip_atomic_store(xm + i, (1ull << 32) | (unsigned long long)__float_as_uint(m), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
        float m0, m1;
        atts_poll(xm, l, lane, a.spin_limit, a.wait_err, m0, m1);
        m = fmaxf(lane < l ? m0 : 0.0f, lane + 64 < l ? m1 : 0.0f);
        m = wave_max_f(m);
        float scale, inv;
        q8_scale_of(m, scale, inv);
        if (lane == 0) {
            s_sc[0] = scale;
            s_sc[1] = inv;
            if (i == 0) a.ctx_qscale[b] = scale;
        }
    }
    __syncthreads();
    {
        const float inv = s_sc[1];
        if (own) a.ctx_q[(size_t)b * a.ldq + c] = (int8_t)(q8_pack2(f, 0.0f, inv) & 0xff);
        if (i == 0)                                               // pad bytes [C, ldq) are zero
            for (int z = C + 2 * tid; z < a.ldq; z += 2 * ATT_THREADS) *(short *)(a.ctx_q + (size_t)b * a.ldq + z) = 0;
    }
}

// Many hypotheses (sentences side by side): throughput matters, not the latency of one
// energy, and the work is split over two kernels.  First the energies: block (g, b) of 256
// threads takes source positions 8 g .. 8 g + 7 of hypothesis b; thread (p, c) =
// (tid / 32, tid % 32) sums columns 4 c + 128 u, u = 0, 1, ..., of position 8 g + p, and the
// 32 partial sums of a position are added across lanes.
#define ATTP_POS 8
__global__ __launch_bounds__(256) void attention_panel_kernel(AttArgs a)
{
    const int b = blockIdx.y, tid = threadIdx.x;
    const float *P, *enc_h;
    const int l = att_sentence(a, b, P, enc_h);
    const int i0 = blockIdx.x * ATTP_POS;
    if (i0 >= l) return;
    const int p = tid >> 5, c = tid & 31, i = i0 + p;
    double acc = 0.0;
    if (i < l) {
        const float *Pi = P + (size_t)i * a.A;
        const float *ab = a.a + (size_t)b * a.A;
        if ((a.A & 3) == 0) {
            for (int j = 4 * c; j < a.A; j += 128) {
                const float4 pv = *(const float4 *)(Pi + j), av = *(const float4 *)(ab + j), vv = *(const float4 *)(a.v + j);
                acc += (double)vv.x * (double)tanh_rn(pv.x + av.x);
                acc += (double)vv.y * (double)tanh_rn(pv.y + av.y);
                acc += (double)vv.z * (double)tanh_rn(pv.z + av.z);
                acc += (double)vv.w * (double)tanh_rn(pv.w + av.w);
            }
        } else {
            for (int j = c; j < a.A; j += 32) acc += (double)a.v[j] * (double)tanh_rn(Pi[j] + ab[j]);
        }
    }
#pragma unroll
    for (int m = 16; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);     // within the position's 32 lanes
    if (c == 0 && i < l) a.e[(size_t)b * a.lde + i] = (float)acc;
}

// Then softmax and context vector (Eq. 5) of every hypothesis: att_finish as a kernel of its own, one
// block of 1024 threads per hypothesis (a thread owns one pair of columns at C = 2048 and has all
// its loads in flight at once).  Measured at 320 hypotheses of 64 sentences: 256-thread blocks
// finishing inside the energy kernel held that kernel at 34 us (each thread walked the positions
// four times over); one block per sentence for all its hypotheses read every encoder state once
// but kept a single compute unit busy for 17 us; four blocks of 256 threads per sentence, each with a
// quarter of the columns for all hypotheses and the last to arrive quantizing the vectors, took 18 us
// (one wave per SIMD: nothing hides the latency of its loads, and the hand-off adds 5 us at the end)
// against 11 us for this kernel, and 28 us against 20-24 us at 1000 hypotheses.
//
// Workgroups are handed to the eight XCDs in turn, each with an L2 of its own.  The hypotheses of a
// sentence read the same encoder states, so they are given block numbers that fall on one XCD
// (sentence s on XCD s % 8, its hypotheses in consecutive rounds): the first of them brings the
// states into that L2 and the others find them there.  With consecutive block numbers per sentence
// the same states were fetched once per hypothesis (78 MB at 320 hypotheses, 15.7 us).  Only the
// speed depends on how the hardware deals the blocks out.
__global__ __launch_bounds__(ATT_MAX_THREADS) void attention_finish_kernel(AttArgs a, int n)
{
    __shared__ double s_alpha[1024];
    int b = blockIdx.x;
    if (a.sent_off) {
        const int xcd = b & 7, q = b >> 3;
        b = ((q / a.beam) * 8 + xcd) * a.beam + q % a.beam;
    }
    if (b >= n) return;
    const float *P, *enc_h;
    const int l = att_sentence(a, b, P, enc_h);
    att_finish<false>(a, b, l, enc_h, s_alpha);
}

// ========================================================================== readout ==

struct ReadoutArgs {
    const int8_t *Ws, *Wy, *Wc;
    const float *b_t, *s, *y, *c;
    float *t_out;
    q8_taps ts, ty, tc;
    int R, H, E, C, lds, ldy, ldc, lpr;
    float ss_w, sy_w, sc_w;
    // fast kernel with PRE: codes [n x ldy], [n x ldc] (pad bytes zero) and scales [n] of y and c from their producers
    const int8_t *yq_pre, *cq_pre;
    const float *ys_pre, *cs_pre;
    // fast kernel, may be NULL: where block 0 leaves the codes [n x lds] and scales [n] of s (the search step hands
    // the survivors' on to the next decoder step)
    int8_t *sq_out;
    float *ss_out;
};

template <int N>
__device__ __forceinline__ void readout_x_taps(const ReadoutArgs &a, const int8_t *sq, const int8_t *yq, const int8_t *cq,
                                               const float *s_scale)
{
    const q8_taps *tp[3] = {&a.ts, &a.ty, &a.tc};
    const int8_t *src[3] = {sq, yq, cq};
    const int dim[3] = {a.H, a.E, a.C}, ldq[3] = {a.lds, a.ldy, a.ldc};
    for (int m = 0; m < 3; ++m) {
        if (tp[m]->xq)
            for (int e = threadIdx.x; e < N * dim[m]; e += blockDim.x)
                tp[m]->xq[e] = src[m][(e / dim[m]) * ldq[m] + e % dim[m]];
        if (tp[m]->xscale && threadIdx.x < N) tp[m]->xscale[threadIdx.x] = s_scale[8 * m + threadIdx.x];
    }
}

// t = tanh(((W_s q(s) + W_y q(y)) + W_c q(ctx)) + b_t): first layer of g (Eq. 2).  General shapes.
template <int N>
__global__ __launch_bounds__(256) void readout_kernel(ReadoutArgs a)
{
    extern __shared__ __align__(16) int8_t smem[];
    __shared__ float s_scale[24];
    __shared__ float s_red[8 * 4];
    int8_t *sq = smem, *yq = sq + N * a.lds, *cq = yq + N * a.ldy;
    block_quantize<N>(a.s, N, a.H, a.H, a.lds, sq, s_scale, s_red);
    block_quantize<N>(a.y, N, a.E, a.E, a.ldy, yq, s_scale + 8, s_red);
    block_quantize<N>(a.c, N, a.C, a.C, a.ldc, cq, s_scale + 16, s_red);
    if (blockIdx.x == 0) readout_x_taps<N>(a, sq, yq, cq, s_scale);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lpr = a.lpr, lir = lane & (lpr - 1), sg = lane / lpr, upw = 64 / lpr;
    float cs = 0.0f, cy = 0.0f, cc = 0.0f;
    if (lir < N) {
        cs = a.ss_w * s_scale[lir];
        cy = a.sy_w * s_scale[8 + lir];
        cc = a.sc_w * s_scale[16 + lir];
    }
    for (int u0 = (blockIdx.x * 4 + wave) * upw; u0 < a.R; u0 += gridDim.x * 4 * upw) {
        const int unit = u0 + sg;
        const bool ok = unit < a.R;
        int as[1][N], ay[1][N], ac[1][N];
        const int8_t *w1[1];
        w1[0] = ok ? a.Ws + (size_t)unit * a.lds : nullptr;
        wave_dot<N, 1>(w1, a.lds, lpr, lir, sq, as);
        w1[0] = ok ? a.Wy + (size_t)unit * a.ldy : nullptr;
        wave_dot<N, 1>(w1, a.ldy, lpr, lir, yq, ay);
        w1[0] = ok ? a.Wc + (size_t)unit * a.ldc : nullptr;
        wave_dot<N, 1>(w1, a.ldc, lpr, lir, cq, ac);
        if (ok && lir < N) {
            int vs = 0, vy = 0, vc = 0;
#pragma unroll
            for (int jj = 0; jj < N; ++jj) {
                vs = (lir == jj) ? as[0][jj] : vs;
                vy = (lir == jj) ? ay[0][jj] : vy;
                vc = (lir == jj) ? ac[0][jj] : vc;
            }
            const float u1 = (float)vs * cs, u2 = (float)vy * cy, u3 = (float)vc * cc;
            float p = u1 + u2;
            p = p + u3;
            if (a.b_t) p = p + a.b_t[unit];
            a.t_out[(size_t)lir * a.R + unit] = tanh_rn(p);
            if (a.ts.acc) a.ts.acc[(size_t)lir * a.R + unit] = vs;
            if (a.ty.acc) a.ty.acc[(size_t)lir * a.R + unit] = vy;
            if (a.tc.acc) a.tc.acc[(size_t)lir * a.R + unit] = vc;
        }
    }
}

// Rows of at most 1024 * CH bytes, dims % 4 == 0, one output unit per wave: everything is
// requested up front, then quantized and dotted.  PRE: y and c arrive as the codes and scales
// their producers left (the GRU that multiplied y at the start of the step, the attention block
// that finished c); they are copied into LDS and s alone is quantized here.
template <int N, int CH, bool PRE>
__device__ __forceinline__ void readout_fast_body(const ReadoutArgs &a, int bid, int8_t *smem)
{
    __shared__ float s_scale[24];
    __shared__ float s_red[3 * 8 * 4];
    __shared__ int s_t[4][3 * N];
    int8_t *sq = smem, *yq = sq + N * a.lds, *cq = yq + N * a.ldy;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int unit = bid * 4 + wave;
    const bool ok = unit < a.R;

    // PRE: the codes as 16-byte pieces (thread tid takes pieces tid, tid + 256, ... of each input; a piece
    // past the end reads as zero through the descriptor) and the scales, requested first
    constexpr int NPRE = PRE ? (N * CH * 64 + 255) / 256 : 1;
    v4i pre_y[NPRE], pre_c[NPRE];
    float pre_sy = 0.0f, pre_sc = 0.0f;      // thread j < N: the scales of vector j
    if (PRE) {
        const int t = threadIdx.x;
        const int so = (int)(t < N ? (unsigned)t * 4u : Q8_OOB);
        pre_sy = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(q8_rsrc(a.ys_pre, (size_t)N * sizeof(float)), so, 0, 0));
        pre_sc = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(q8_rsrc(a.cs_pre, (size_t)N * sizeof(float)), so, 0, 0));
        const __amdgpu_buffer_rsrc_t ry = q8_rsrc(a.yq_pre, (size_t)N * a.ldy), rc = q8_rsrc(a.cq_pre, (size_t)N * a.ldc);
#pragma unroll
        for (int u = 0; u < NPRE; ++u) {
            pre_y[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(ry, (u * 256 + t) * 16, 0, 0));
            pre_c[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rc, (u * 256 + t) * 16, 0, 0));
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    XRegs<N, CH> rin[3];                     // s, y, ctx
    x_load<N, CH>(rin[0], a.s, N, a.H, a.H);
    if (!PRE) {
        x_load<N, CH>(rin[1], a.y, N, a.E, a.E);
        x_load<N, CH>(rin[2], a.c, N, a.C, a.C);
    }
    v4i ws[1][CH], wy[1][CH], wc[1][CH];
    {
        const int row[1] = {ok ? unit : -1};
        rows_load<1, CH>(ws, q8_rsrc(a.Ws, (size_t)a.R * a.lds), row, a.lds, lane);
        rows_load<1, CH>(wy, q8_rsrc(a.Wy, (size_t)a.R * a.ldy), row, a.ldy, lane);
        rows_load<1, CH>(wc, q8_rsrc(a.Wc, (size_t)a.R * a.ldc), row, a.ldc, lane);
    }
    const float bt = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
        q8_rsrc(a.b_t, a.b_t ? (size_t)a.R * sizeof(float) : 0), (int)(ok ? (unsigned)unit * 4u : Q8_OOB), 0, 0));
    if (PRE) {
#pragma unroll
        for (int u = 0; u < NPRE; ++u) {
            const int o = (u * 256 + (int)threadIdx.x) * 16;
            if (o < N * a.ldy) *(v4i *)(yq + o) = pre_y[u];
            if (o < N * a.ldc) *(v4i *)(cq + o) = pre_c[u];
        }
        if (threadIdx.x < N) { s_scale[8 + threadIdx.x] = pre_sy; s_scale[16 + threadIdx.x] = pre_sc; }
        x_finish<N, CH>(rin[0], N, a.lds, sq, s_scale, s_red);       // scales of s in s_scale[0, N); ends with a barrier
    } else {
        const int lds3[3] = {a.lds, a.ldy, a.ldc};
        int8_t *const dst[3] = {sq, yq, cq};
        x_finish_multi<N, CH, 3>(rin, lds3, dst, s_scale, s_red);
    }
    if (bid == 0) readout_x_taps<N>(a, sq, yq, cq, s_scale);
    if (bid == 0 && a.sq_out) {
        for (int p = threadIdx.x; p < N * a.lds / 16; p += 256) *(v4i *)(a.sq_out + 16 * p) = *(const v4i *)(sq + 16 * p);
        if (threadIdx.x < N) a.ss_out[threadIdx.x] = s_scale[threadIdx.x];
    }

    // the three rows' partial sums against their vectors, totalled over the wave in one pass;
    // lane j < N receives the totals of hypothesis j
    int part[3][N], mine[3];
    {
        int p1[1][N];
        rows_dot_part<N, 1, CH>(ws, a.lds, lane, sq, p1);
#pragma unroll
        for (int jj = 0; jj < N; ++jj) part[0][jj] = p1[0][jj];
        rows_dot_part<N, 1, CH>(wy, a.ldy, lane, yq, p1);
#pragma unroll
        for (int jj = 0; jj < N; ++jj) part[1][jj] = p1[0][jj];
        rows_dot_part<N, 1, CH>(wc, a.ldc, lane, cq, p1);
#pragma unroll
        for (int jj = 0; jj < N; ++jj) part[2][jj] = p1[0][jj];
    }
    sums_to_lanes<N, 3>(part, lane, s_t[wave], mine);
    if (ok && lane < N) {
        const int vs = mine[0], vy = mine[1], vc = mine[2];
        const float cs = a.ss_w * s_scale[lane], cy = a.sy_w * s_scale[8 + lane], cc = a.sc_w * s_scale[16 + lane];
        const float u1 = (float)vs * cs, u2 = (float)vy * cy, u3 = (float)vc * cc;
        float p = u1 + u2;
        p = p + u3;
        if (a.b_t) p = p + bt;
        a.t_out[(size_t)lane * a.R + unit] = tanh_rn(p);
        if (a.ts.acc) a.ts.acc[(size_t)lane * a.R + unit] = vs;
        if (a.ty.acc) a.ty.acc[(size_t)lane * a.R + unit] = vy;
        if (a.tc.acc) a.tc.acc[(size_t)lane * a.R + unit] = vc;
    }
}

template <int N, int CH, bool PRE>
__global__ __launch_bounds__(256) void readout_fast_kernel(ReadoutArgs a)
{
    extern __shared__ __align__(16) int8_t smem[];
    readout_fast_body<N, CH, PRE>(a, blockIdx.x, smem);
}

// The readout and, in the blocks after its own, a streaming product that reads the same new states: the
// recurrent half of the next step's GRU r, W_h^r q(s) + b_h (rows of at most 1024 bytes), which then costs no
// launch of its own on the chain of dependent launches.
template <int N, int CH, bool PRE>
__global__ __launch_bounds__(256) void readout_with_product_kernel(ReadoutArgs a, GemvJobs jobs, int readout_blocks)
{
    extern __shared__ __align__(16) int8_t smem[];
    if ((int)blockIdx.x < readout_blocks) readout_fast_body<N, CH, PRE>(a, blockIdx.x, smem);
    else gemv_fast_body<N, 1, false, 2, true>(jobs, (int)blockIdx.x - readout_blocks, smem);
}

// Panels of more than 8 hypotheses: the three products of g's first layer came from the
// matrix cores (no bias); block j adds them in the order of the fused kernels, applies tanh,
// and quantizes t_j for the vocabulary product.
__global__ __launch_bounds__(256) void readout_combine_kernel(const float *__restrict__ ts, const float *__restrict__ ty,
                                                              const float *__restrict__ tc, const float *__restrict__ b_t,
                                                              int R, float *t_out, int ld, int8_t *tq, float *tscale,
                                                              int8_t *tap_xq, float *tap_scale)
{
    __shared__ float s_scale[1];
    __shared__ float s_red[4];
    const int j = blockIdx.x;
    for (int u = threadIdx.x; u < R; u += 256) {
        const size_t o = (size_t)j * R + u;
        float p = ts[o] + ty[o];
        p = p + tc[o];
        if (b_t) p = p + b_t[u];
        t_out[o] = tanh_rn(p);
    }
    if (!tq) return;                          // the 32-bit engine stops at t
    __syncthreads();                          // this block's t_j is read back below
    block_quantize<1>(t_out + (size_t)j * R, 1, R, R, ld, tq + (size_t)j * ld, s_scale, s_red);
    if (threadIdx.x == 0) {
        tscale[j] = s_scale[0];
        if (tap_scale) tap_scale[j] = s_scale[0];
    }
    if (tap_xq) {
        __syncthreads();
        for (int k = threadIdx.x; k < R; k += 256) tap_xq[(size_t)j * R + k] = tq[(size_t)j * ld + k];
    }
}

// =================================================================== host launchers ==

q8_status q8i_readout_combine(q8_ctx *ctx, const float *ts, const float *ty, const float *tc, const float *b_t, int R,
                              int n, float *t_out, int ld, int8_t *tq, float *tscale, const q8_taps *tap)
{
    Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, readout_combine_kernel, dim3(n), dim3(256), 0, ts, ty, tc, b_t, R, t_out, ld, tq,
              tscale, tap ? tap->xq : nullptr, tap ? tap->xscale : nullptr);
    return q8i_launch_check(ctx, "readout combine");
}


q8_status q8i_attention(q8_ctx *ctx, const float *P, const float *enc_h, int l, int A, int C, const float *a,
                        const float *v, int n, float *e, float *alpha, float *cvec, const int *sent_off, int beam,
                        int8_t *ctx_q, float *ctx_qscale, int ldq, int *codes_written)
{
    AttArgs t;
    t.P = P; t.enc_h = enc_h; t.a = a; t.v = v; t.e = e; t.alpha = alpha; t.ctx = cvec;
    t.counters = (unsigned *)ctx->ws;
    t.cstride = n <= Q8_MAX_BEAM ? Q8_COUNTER_STRIDE : 1;        // header: 1024 words of counters
    t.l = l; t.A = A; t.C = C;
    t.sent_off = sent_off; t.beam = beam; t.lde = l;
    const bool panel = n > Q8_MAX_BEAM;
    const bool codes = ctx_q && ctx_qscale && C % 2 == 0 && ldq >= C && ldq % 2 == 0 && ldq <= 2 * ATT_PAIRS * ATT_THREADS;
    t.ctx_q = codes ? ctx_q : nullptr; t.ctx_qscale = ctx_qscale; t.ldq = ldq;
    t.xchg = nullptr; t.wait_err = nullptr; t.spin_limit = 0; t.ppb = 0; t.inv_ppb = 0.0f;
    if (codes_written) *codes_written = codes ? 1 : 0;
    // One sentence: the form whose blocks exchange their energies and finish their own slices, where
    // its shape limits hold, the consumer takes the codes, and the device holds the whole grid at once
    // (its blocks wait for each other).
    if (!panel && !sent_off && codes && ctx->att_split && l <= ATTS_L && C <= 4096) {
        if (ctx->att_capacity < 0) {
            int dev = 0, cus = 0, per_cu = 0;
            if (hipGetDevice(&dev) == hipSuccess &&
                hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
                hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)attention_split_kernel, ATT_THREADS, 0) == hipSuccess)
                ctx->att_capacity = per_cu * cus;
            else {
                (void)hipGetLastError();
                ctx->att_capacity = 0;
            }
        }
        const int ppb = (C / 2 + l - 1) / l;
        if ((long long)l * n <= ctx->att_capacity && 2 * ppb <= ATT_THREADS && l * ppb <= ATTS_SLICE) {
            t.xchg = (unsigned long long *)(ctx->ws + Q8_WS_ATT_XCHG);
            if (ctx->att_words_set) {          // nobody cleared the last launch's words (its step ended early): do it now
                const q8_status st = q8i_fill_u32(ctx, t.xchg, Q8_MAX_BEAM * (Q8_WS_ATT_XCHG_PER_HYP / 4), 0u);
                if (st) return st;
            }
            ctx->att_words_set = 1;
            t.wait_err = (unsigned *)(ctx->ws + Q8_WS_ATT_ERR);
            t.spin_limit = ctx->att_spin_limit;
            t.ppb = ppb;
            t.inv_ppb = 1.0f / (float)ppb;
            Q8_LAUNCH(ctx, Q8_KERNEL_ATTENTION, attention_split_kernel, dim3(l, n), dim3(ATT_THREADS), 0, t);
            return q8i_launch_check(ctx, "attention");
        }
    }
    if (panel) {
        Q8_LAUNCH(ctx, Q8_KERNEL_ATTENTION, attention_panel_kernel, dim3((l + ATTP_POS - 1) / ATTP_POS, n), dim3(256), 0, t);
        // (block numbers are dealt to sentences in groups of eight, see the kernel: the grid covers whole groups)
        const int nsent = sent_off ? (n + beam - 1) / beam : 0;
        const int fin_blocks = sent_off ? (nsent + 7) / 8 * 8 * beam : n;
        Q8_LAUNCH(ctx, Q8_KERNEL_ATTENTION, attention_finish_kernel, dim3(fin_blocks), dim3(ATT_MAX_THREADS), 0, t, n);
    } else {
        Q8_LAUNCH(ctx, Q8_KERNEL_ATTENTION, attention_kernel, dim3(l, n), dim3(ATT_THREADS), 0, t);
    }
    return q8i_launch_check(ctx, "attention");
}

template <int N>
static void launch_readout_n(q8_ctx *ctx, const ReadoutArgs &a, int blocks, size_t smem, int ch, bool pre, const GemvJobs *extra,
                             int extra_blocks, size_t extra_smem)
{
    if (extra) {
        const size_t sm = smem > extra_smem ? smem : extra_smem;
        const dim3 grid(blocks + extra_blocks);
        if (ch == 1 && pre) Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, (readout_with_product_kernel<N, 1, true>), grid, dim3(256), sm, a, *extra, blocks);
        else if (ch == 2 && pre) Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, (readout_with_product_kernel<N, 2, true>), grid, dim3(256), sm, a, *extra, blocks);
        else if (ch == 1) Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, (readout_with_product_kernel<N, 1, false>), grid, dim3(256), sm, a, *extra, blocks);
        else Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, (readout_with_product_kernel<N, 2, false>), grid, dim3(256), sm, a, *extra, blocks);
        return;
    }
    if (ch == 1 && pre) Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, (readout_fast_kernel<N, 1, true>), dim3(blocks), dim3(256), smem, a);
    else if (ch == 2 && pre) Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, (readout_fast_kernel<N, 2, true>), dim3(blocks), dim3(256), smem, a);
    else if (ch == 1) Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, (readout_fast_kernel<N, 1, false>), dim3(blocks), dim3(256), smem, a);
    else if (ch == 2) Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, (readout_fast_kernel<N, 2, false>), dim3(blocks), dim3(256), smem, a);
    else Q8_LAUNCH(ctx, Q8_KERNEL_READOUT, readout_kernel<N>, dim3(blocks), dim3(256), smem, a);
}

q8_status q8i_readout(q8_ctx *ctx, const q8_readout_weights *ro, const float *s, const float *y, const float *c, int n,
                      float *t_out, const q8_taps *taps3, const q8_codes *y_codes, const q8_codes *c_codes,
                      int8_t *sq_out, float *ss_out, int *s_exported, const q8i_gemv_desc *extra, int *extra_done)
{
    ReadoutArgs a;
    if (s_exported) *s_exported = 0;
    if (extra_done) *extra_done = 0;
    // codes from the producers: both or neither, and only in the layout the kernel copies (the matrices' own pitches)
    const bool pre = y_codes && c_codes && y_codes->valid && c_codes->valid && y_codes->q && c_codes->q && y_codes->scale &&
                     c_codes->scale && y_codes->ld == ro->W_y.ld && c_codes->ld == ro->W_c.ld;
    a.yq_pre = pre ? y_codes->q : nullptr; a.cq_pre = pre ? c_codes->q : nullptr;
    a.ys_pre = pre ? y_codes->scale : nullptr; a.cs_pre = pre ? c_codes->scale : nullptr;
    a.Ws = ro->W_s.data; a.Wy = ro->W_y.data; a.Wc = ro->W_c.data; a.b_t = ro->b_t;
    a.s = s; a.y = y; a.c = c; a.t_out = t_out;
    q8_taps none = {nullptr, nullptr, nullptr};
    a.ts = taps3 ? taps3[0] : none; a.ty = taps3 ? taps3[1] : none; a.tc = taps3 ? taps3[2] : none;
    a.R = ro->W_s.rows; a.H = ro->W_s.cols; a.E = ro->W_y.cols; a.C = ro->W_c.cols;
    a.lds = ro->W_s.ld; a.ldy = ro->W_y.ld; a.ldc = ro->W_c.ld;
    int ldmin = a.lds < a.ldy ? a.lds : a.ldy, ldmax = a.lds > a.ldy ? a.lds : a.ldy;
    if (a.ldc < ldmin) ldmin = a.ldc;
    if (a.ldc > ldmax) ldmax = a.ldc;
    a.lpr = q8_lanes_per_row(ldmin);
    a.ss_w = ro->W_s.scale; a.sy_w = ro->W_y.scale; a.sc_w = ro->W_c.scale;
    int ch = q8_fast_ch(ldmax);                 // dims % 4 == 0 is checked by the caller
    if (ch == 4) ch = 0;
    if ((size_t)a.R * ldmax >= (1u << 31)) ch = 0;      // the fast kernel addresses the matrices with 32-bit offsets
    const int upb = ch ? 4 : 4 * (64 / a.lpr);
    const int blocks = (a.R + upb - 1) / upb;
    const size_t smem = (size_t)n * (a.lds + a.ldy + a.ldc);
    const bool exporting = ch != 0 && sq_out && ss_out;             // (the general kernel does not export)
    a.sq_out = exporting ? sq_out : nullptr; a.ss_out = ss_out;
    if (s_exported) *s_exported = exporting ? 1 : 0;
    // a product of the same states in the blocks after the readout's own (fast kernels of both, rows of <= 1024 bytes)
    GemvJobs xj;
    int xblocks = 0;
    size_t xsmem = 0;
    const bool with_extra = extra && (ch == 1 || ch == 2) && q8i_gemv_fast_setup(extra, n, &xj, &xblocks, &xsmem);
    if (with_extra && extra_done) *extra_done = 1;
    const GemvJobs *xp = with_extra ? &xj : nullptr;
    switch (n) {
    case 1: launch_readout_n<1>(ctx, a, blocks, smem, ch, pre && ch != 0, xp, xblocks, xsmem); break;
    case 2: launch_readout_n<2>(ctx, a, blocks, smem, ch, pre && ch != 0, xp, xblocks, xsmem); break;
    case 3: launch_readout_n<3>(ctx, a, blocks, smem, ch, pre && ch != 0, xp, xblocks, xsmem); break;
    case 4: launch_readout_n<4>(ctx, a, blocks, smem, ch, pre && ch != 0, xp, xblocks, xsmem); break;
    case 5: launch_readout_n<5>(ctx, a, blocks, smem, ch, pre && ch != 0, xp, xblocks, xsmem); break;
    case 6: launch_readout_n<6>(ctx, a, blocks, smem, ch, pre && ch != 0, xp, xblocks, xsmem); break;
    case 7: launch_readout_n<7>(ctx, a, blocks, smem, ch, pre && ch != 0, xp, xblocks, xsmem); break;
    default: launch_readout_n<8>(ctx, a, blocks, smem, ch, pre && ch != 0, xp, xblocks, xsmem); break;
    }
    return q8i_launch_check(ctx, "readout");
}

// ============================ attention with 8-bit activation products (a variant) ==
// Under the other reading of Section 3 for Eq. 5-6 the products with v and with the encoder
// states are 8-bit too.  Both are then ordinary narrow products and run on the product kernels
// (v as a 1 x A matrix against the tanh vectors of all positions, the transposed states as a
// C x l matrix against the attention weights); what is left are three element-wise kernels.

// T[(b l + i) A + j] = tanh(P[i A + j] + a[b A + j])
__global__ __launch_bounds__(256) void att_tanh_kernel(const float *__restrict__ P, const float *__restrict__ a,
                                                       float *__restrict__ T, int l, int A, int n)
{
    const size_t total = (size_t)n * l * A;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const size_t bi = e / A;
        const int j = (int)(e - bi * A), b = (int)(bi / l), i = (int)(bi - (size_t)b * l);
        const float pre = P[(size_t)i * A + j] + a[(size_t)b * A + j];
        T[e] = q8_tanh_rn(pre);
    }
}

// alpha = softmax(e) per hypothesis (one wave each), written with leading dimension ld_alpha
// (pad zero) for the product that follows and, if asked for, densely to alpha_out / e_out.
__global__ __launch_bounds__(64) void att_softmax_kernel(const float *__restrict__ e, int l, int ld_alpha,
                                                         float *__restrict__ alpha_ws, float *__restrict__ alpha_out,
                                                         float *__restrict__ e_out)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const float *eb = e + (size_t)b * l;
    float mx = -INFINITY;
    for (int i = lane; i < l; i += 64) mx = fmaxf(mx, eb[i]);
    mx = wave_max_f(mx);
    double z = 0.0;
    for (int i = lane; i < l; i += 64) z += q8_exp_d(fmax((double)eb[i] - (double)mx, -700.0));
    z = wave_sum_d(z);
    for (int i = lane; i < ld_alpha; i += 64) {
        float al = 0.0f;
        if (i < l) {
            al = (float)(q8_exp_d(fmax((double)eb[i] - (double)mx, -700.0)) / z);
            if (alpha_out) alpha_out[(size_t)b * l + i] = al;
            if (e_out) e_out[(size_t)b * l + i] = eb[i];
        }
        alpha_ws[(size_t)b * ld_alpha + i] = al;
    }
}

// Xt[c rows + r] = X[r cols + c]
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ X, int rows, int cols, float *__restrict__ Xt)
{
    const size_t total = (size_t)rows * cols;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const size_t c = e / rows, r = e - c * rows;
        Xt[e] = X[r * cols + c];
    }
}

static int blocks_for(size_t total)
{
    const size_t b = (total + 255) / 256;
    return (int)(b < 4096 ? b : 4096);
}

q8_status q8i_att_tanh(q8_ctx *ctx, const float *P, const float *a, float *T, int l, int A, int n)
{
    hipLaunchKernelGGL(att_tanh_kernel, dim3(blocks_for((size_t)n * l * A)), dim3(256), 0, ctx->stream, P, a, T, l, A, n);
    return q8i_launch_check(ctx, "attention tanh");
}

q8_status q8i_att_softmax(q8_ctx *ctx, const float *e, int n, int l, int ld_alpha, float *alpha_ws, float *alpha_out,
                          float *e_out)
{
    hipLaunchKernelGGL(att_softmax_kernel, dim3(n), dim3(64), 0, ctx->stream, e, l, ld_alpha, alpha_ws, alpha_out, e_out);
    return q8i_launch_check(ctx, "attention softmax");
}

q8_status q8i_transpose(q8_ctx *ctx, const float *X, int rows, int cols, float *Xt)
{
    hipLaunchKernelGGL(transpose_kernel, dim3(blocks_for((size_t)rows * cols)), dim3(256), 0, ctx->stream, X, rows, cols, Xt);
    return q8i_launch_check(ctx, "transpose");
}
