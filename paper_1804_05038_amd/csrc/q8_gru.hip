// q8_gru.hip -- the GRU cell that Eq. 1 (encoder) and Eq. 3-4 (decoder r and q) of "Pieces
// of Eight: 8-bit Neural Machine Translation" apply, with Section 3's 8-bit products:
// one launch computes both products of a cell for the block's hidden units and fuses
// dequantization, bias, sigmoid / tanh and the state mix.
#include "q8_internal.h"

#define GRU_FULL 0     // both products computed here
#define GRU_GX_PRE 1   // gx = Wx q(x) + bx supplied in g_pre (encoder: all positions at once)
#define GRU_GH_PRE 2   // gh = Wh q(h) + bh supplied in g_pre (decoder GRU q: depends on s' only)

struct GruJob {
    const int8_t *Wx, *Wh;
    const float *bx, *bh;
    const float *x, *h_prev, *g_pre;
    const int8_t *xq_pre;      // kernels with XPRE: codes [N x ldwx] and scales [N] of x from its producer
    const float *xs_pre;
    const int8_t *hq_pre;      // GRU_FULL kernels with XPRE: the same for h_prev, [N x ldwh]
    const float *hs_pre;
    int8_t *xq_out;            // may be NULL: where block 0 leaves the codes [N x ldwx] and scales [N] of x for a later consumer
    float *xs_out;
    float *h_out;
    q8_taps tx, th;
    int I, ldwx, H, ldwh, ldx, ldh, ldo, ldg, lpr;
    float sx_w, sh_w;
};
struct GruJobs {
    GruJob j[2];
    // 8-byte words that an earlier kernel of the step left set and wants zero at its next launch (NULL: none)
    unsigned long long *clear;
    int clear_words;
};

// The grid's first row of blocks zeroes them, as the last thing it does (nothing waits for the stores).
__device__ __forceinline__ void gru_clear_words(const GruJobs &jobs)
{
    if (jobs.clear && blockIdx.y == 0)
        for (unsigned w = blockIdx.x * 256u + threadIdx.x; w < (unsigned)jobs.clear_words; w += gridDim.x * 256u)
            jobs.clear[w] = 0ull;
}

template <int N, int MODE>
__device__ __forceinline__ void gru_x_taps(const GruJob &J, const int8_t *xq, const int8_t *hq, const float *s_scale)
{
    if (MODE != GRU_GX_PRE) {
        if (J.tx.xq)
            for (int e = threadIdx.x; e < N * J.I; e += blockDim.x) J.tx.xq[e] = xq[(e / J.I) * J.ldwx + e % J.I];
        if (J.tx.xscale && threadIdx.x < N) J.tx.xscale[threadIdx.x] = s_scale[threadIdx.x];
    }
    if (MODE != GRU_GH_PRE) {
        if (J.th.xq)
            for (int e = threadIdx.x; e < N * J.H; e += blockDim.x) J.th.xq[e] = hq[(e / J.H) * J.ldwh + e % J.H];
        if (J.th.xscale && threadIdx.x < N) J.th.xscale[threadIdx.x] = s_scale[8 + threadIdx.x];
    }
}

// Block 0 hands the codes and scales of x on to whoever multiplies the same vectors next.
template <int N>
__device__ __forceinline__ void gru_x_export(const GruJob &J, const int8_t *xq, const float *s_scale)
{
    if (!J.xq_out) return;
    for (int p = threadIdx.x; p < N * J.ldwx / 16; p += blockDim.x) *(v4i *)(J.xq_out + 16 * p) = *(const v4i *)(xq + 16 * p);
    if (threadIdx.x < N) J.xs_out[threadIdx.x] = s_scale[threadIdx.x];
}

// General shapes.
template <int N, int MODE>
__global__ __launch_bounds__(256) void gru_kernel(GruJobs jobs)
{
    extern __shared__ __align__(16) int8_t smem[];
    __shared__ float s_scale[16];
    __shared__ float s_red[8 * 4];
    const GruJob &J = jobs.j[blockIdx.y];
    const int H = J.H;
    int8_t *xq = smem;
    int8_t *hq = smem + (MODE == GRU_GX_PRE ? 0 : N * J.ldwx);
    if (MODE != GRU_GX_PRE) block_quantize<N>(J.x, N, J.I, J.ldx, J.ldwx, xq, s_scale, s_red);
    if (MODE != GRU_GH_PRE) block_quantize<N>(J.h_prev, N, H, J.ldh, J.ldwh, hq, s_scale + 8, s_red);
    if (blockIdx.x == 0) gru_x_taps<N, MODE>(J, xq, hq, s_scale);
    if (blockIdx.x == 0 && MODE != GRU_GX_PRE) gru_x_export<N>(J, xq, s_scale);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lpr = J.lpr, lir = lane & (lpr - 1), sg = lane / lpr, upw = 64 / lpr;
    float cx = 0.0f, ch = 0.0f;
    if (lir < N) {
        if (MODE != GRU_GX_PRE) cx = J.sx_w * s_scale[lir];
        if (MODE != GRU_GH_PRE) ch = J.sh_w * s_scale[8 + lir];
    }

    for (int u0 = (blockIdx.x * 4 + wave) * upw; u0 < H; u0 += gridDim.x * 4 * upw) {
        const int unit = u0 + sg;
        const bool ok = unit < H;
        int ax[3][N], ah[3][N];
        if (MODE != GRU_GX_PRE) {
            const int8_t *wrow[3];
#pragma unroll
            for (int gt = 0; gt < 3; ++gt) wrow[gt] = ok ? J.Wx + (size_t)(gt * H + unit) * J.ldwx : nullptr;
            wave_dot<N, 3>(wrow, J.ldwx, lpr, lir, xq, ax);
        }
        if (MODE != GRU_GH_PRE) {
            const int8_t *wrow[3];
#pragma unroll
            for (int gt = 0; gt < 3; ++gt) wrow[gt] = ok ? J.Wh + (size_t)(gt * H + unit) * J.ldwh : nullptr;
            wave_dot<N, 3>(wrow, J.ldwh, lpr, lir, hq, ah);
        }
        if (ok && lir < N) {
            const int j = lir;
            float gx[3], gh[3];
#pragma unroll
            for (int gt = 0; gt < 3; ++gt) {
                const int row = gt * H + unit;
                if (MODE == GRU_GX_PRE) {
                    gx[gt] = J.g_pre[(size_t)j * J.ldg + row];
                } else {
                    int a = 0;
#pragma unroll
                    for (int jj = 0; jj < N; ++jj) a = (j == jj) ? ax[gt][jj] : a;
                    float y = (float)a * cx;
                    if (J.bx) y = y + J.bx[row];
                    gx[gt] = y;
                    if (J.tx.acc) J.tx.acc[(size_t)j * 3 * H + row] = a;
                }
                if (MODE == GRU_GH_PRE) {
                    gh[gt] = J.g_pre[(size_t)j * J.ldg + row];
                } else {
                    int a = 0;
#pragma unroll
                    for (int jj = 0; jj < N; ++jj) a = (j == jj) ? ah[gt][jj] : a;
                    float y = (float)a * ch;
                    if (J.bh) y = y + J.bh[row];
                    gh[gt] = y;
                    if (J.th.acc) J.th.acc[(size_t)j * 3 * H + row] = a;
                }
            }
            J.h_out[(size_t)j * J.ldo + unit] = gru_gates(gx, gh, J.h_prev[(size_t)j * J.ldh + unit]);
        }
    }
    gru_clear_words(jobs);
}

// Rows of at most 1024 * CH bytes, I % 4 == 0, H % 4 == 0, one hidden unit per wave
// (grid.x * 4 >= H).  Activations, the unit's six (or three) weight rows and the
// epilogue's operands are all requested before the block first waits.  XPRE: the vectors
// that are multiplied here arrive as codes and scales from whoever produced them (x with
// GRU_GH_PRE; x and h_prev with GRU_FULL) and are copied to LDS instead of quantized.
template <int N, int MODE, int CH, bool XPRE = false>
__global__ __launch_bounds__(256) void gru_fast_kernel(GruJobs jobs)
{
    static_assert(!XPRE || MODE != GRU_GX_PRE, "codes are taken for x, or for x and h_prev");
    constexpr bool HPRE = XPRE && MODE == GRU_FULL;
    extern __shared__ __align__(16) int8_t smem[];
    __shared__ float s_scale[16];
    __shared__ float s_red[2 * 8 * 4];
    __shared__ int s_t[4][6 * N];
    const GruJob &J = jobs.j[blockIdx.y];
    const int H = J.H;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int unit = blockIdx.x * 4 + wave;
    const bool ok = unit < H;
    int8_t *xq = smem;
    int8_t *hq = smem + (MODE == GRU_GX_PRE ? 0 : N * J.ldwx);

    XRegs<N, CH> xh[2];                      // [0]: x, [1]: h_prev
    XRegs<N, CH> &xr = xh[0], &hr = xh[1];
    // XPRE: N * ldwx code bytes in 16-byte pieces, thread tid takes pieces tid, tid + 256, ...; a piece
    // past the end is read through the descriptor as zero, so the loads need no branch
    constexpr int NPRE = XPRE ? (N * CH * 64 + 255) / 256 : 1;
    v4i pre_q[NPRE], pre_hq[HPRE ? NPRE : 1];
    float pre_s = 0.0f, pre_hs = 0.0f;       // XPRE: scales of vector tid, requested first so that they are not waited for behind the weights
    if (XPRE) {
        const int so = (int)(threadIdx.x < N ? threadIdx.x * 4u : Q8_OOB);
        pre_s = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(q8_rsrc(J.xs_pre, (size_t)N * sizeof(float)), so, 0, 0));
        if (HPRE)
            pre_hs = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(q8_rsrc(J.hs_pre, (size_t)N * sizeof(float)), so, 0, 0));
        const __amdgpu_buffer_rsrc_t rq = q8_rsrc(J.xq_pre, (size_t)N * J.ldwx);
#pragma unroll
        for (int t = 0; t < NPRE; ++t)
            pre_q[t] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rq, (t * 256 + (int)threadIdx.x) * 16, 0, 0));
        if (HPRE) {
            const __amdgpu_buffer_rsrc_t rhq = q8_rsrc(J.hq_pre, (size_t)N * J.ldwh);
#pragma unroll
            for (int t = 0; t < NPRE; ++t)
                pre_hq[t] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rhq, (t * 256 + (int)threadIdx.x) * 16, 0, 0));
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if (MODE != GRU_GX_PRE && !XPRE) x_load<N, CH>(xr, J.x, N, J.I, J.ldx);
    if (MODE != GRU_GH_PRE && !HPRE) x_load<N, CH>(hr, J.h_prev, N, H, J.ldh);
    v4i wx[3][CH], wh[3][CH];
    {
        int row[3];
#pragma unroll
        for (int gt = 0; gt < 3; ++gt) row[gt] = ok ? gt * H + unit : -1;
        if (MODE != GRU_GX_PRE) rows_load<3, CH>(wx, q8_rsrc(J.Wx, (size_t)3 * H * J.ldwx), row, J.ldwx, lane);
        if (MODE != GRU_GH_PRE) rows_load<3, CH>(wh, q8_rsrc(J.Wh, (size_t)3 * H * J.ldwh), row, J.ldwh, lane);
    }
    // Epilogue operands (biases, previous state, supplied pre-activations) in one load instruction, two
    // with pre-activations: lane 8 k + j reads slot k for vector j (k = 0..2: bx of gate k, 3..5: bh of
    // gate k - 3, 6: h_prev of vector j; second load, k = 0..2: pre-activation of gate k for vector j).
    // Lanes with nothing to read (absent arrays, vectors past N, units past H) read the first float of
    // h_prev and drop it.  Every further load instruction per wave costs more than moving the values
    // between lanes afterwards.
    float pre[3] = {0.f, 0.f, 0.f}, bxv[3] = {0.f, 0.f, 0.f}, bhv[3] = {0.f, 0.f, 0.f}, hp = 0.f;
    float ev, pv = 0.0f;
    bool ev_used, pv_used = false;
    typedef const __attribute__((address_space(1))) float *gfp;
    {
        const int k = lane >> 3, j = lane & 7;
        const int gt = k < 3 ? k : (k < 6 ? k - 3 : 0);
        const size_t row = (size_t)gt * H + (ok ? unit : 0);
        const bool use_bx = ok && k < 3 && MODE != GRU_GX_PRE && J.bx != nullptr;
        const bool use_bh = ok && k >= 3 && k < 6 && MODE != GRU_GH_PRE && J.bh != nullptr;
        const bool use_h = ok && k == 6 && j < N;
        const float *p = J.h_prev;
        p = use_bx ? J.bx + row : p;
        p = use_bh ? J.bh + row : p;
        p = use_h ? J.h_prev + (size_t)j * J.ldh + unit : p;
        uintptr_t addr = (uintptr_t)p;
        asm volatile("" : "+v"(addr));                   // one load from the chosen address, not a load per choice
        ev = *(gfp)addr;
        ev_used = use_bx || use_bh || use_h;             // applied where the value is first needed: not here, where it would be waited for
        if (MODE != GRU_FULL) {
            const bool use_p = ok && k < 3 && j < N;
            const float *pp = use_p ? J.g_pre + (size_t)j * J.ldg + row : J.h_prev;
            uintptr_t addr2 = (uintptr_t)pp;
            asm volatile("" : "+v"(addr2));
            pv = *(gfp)addr2;
            pv_used = use_p;
        }
    }

    if (XPRE) {
#pragma unroll
        for (int t = 0; t < NPRE; ++t) {
            const int o = (t * 256 + (int)threadIdx.x) * 16;
            if (o < N * J.ldwx) *(v4i *)(xq + o) = pre_q[t];
            if (HPRE && o < N * J.ldwh) *(v4i *)(hq + o) = pre_hq[t];
        }
        if (threadIdx.x < N) {
            s_scale[threadIdx.x] = pre_s;
            if (HPRE) s_scale[8 + threadIdx.x] = pre_hs;
        }
        __syncthreads();
    } else if (MODE == GRU_FULL) {
        const int lds[2] = {J.ldwx, J.ldwh};
        int8_t *const dst[2] = {xq, hq};
        x_finish_multi<N, CH, 2>(xh, lds, dst, s_scale, s_red);
    } else if (MODE == GRU_GH_PRE) {
        x_finish<N, CH>(xr, N, J.ldwx, xq, s_scale, s_red);
    } else {
        x_finish<N, CH>(hr, N, J.ldwh, hq, s_scale + 8, s_red);
    }
    if (blockIdx.x == 0) gru_x_taps<N, MODE>(J, xq, hq, s_scale);
    if (blockIdx.x == 0 && MODE != GRU_GX_PRE && !XPRE) gru_x_export<N>(J, xq, s_scale);

    // partial sums of the unit's rows against every vector, totalled over the wave in one pass;
    // lane j < N receives the totals of vector j: [0, 3) input product, [3, 6) recurrent product
    constexpr int UT = MODE == GRU_FULL ? 6 : 3;
    int part[UT][N], mine[UT];
    {
        int px[3][N], ph[3][N];
        if (MODE != GRU_GX_PRE) rows_dot_part<N, 3, CH>(wx, J.ldwx, lane, xq, px);
        if (MODE != GRU_GH_PRE) rows_dot_part<N, 3, CH>(wh, J.ldwh, lane, hq, ph);
#pragma unroll
        for (int gt = 0; gt < 3; ++gt)
#pragma unroll
            for (int jj = 0; jj < N; ++jj) {
                if (MODE == GRU_FULL) { part[gt][jj] = px[gt][jj]; part[3 + gt][jj] = ph[gt][jj]; }
                else part[gt][jj] = MODE == GRU_GH_PRE ? px[gt][jj] : ph[gt][jj];
            }
    }
    sums_to_lanes<N, UT>(part, lane, s_t[wave], mine);
    // the epilogue operands to the lanes that use them: biases are the same for every vector (read from
    // the slot's first lane), the rest comes from lane 8 k + j
    ev = ev_used ? ev : 0.0f;
    pv = pv_used ? pv : 0.0f;
#pragma unroll
    for (int gt = 0; gt < 3; ++gt) {
        bxv[gt] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ev), 8 * gt));
        bhv[gt] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ev), 24 + 8 * gt));
        if (MODE != GRU_FULL) pre[gt] = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (8 * gt + (lane & 7)), __float_as_int(pv)));
    }
    hp = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (48 + (lane & 7)), __float_as_int(ev)));
    if (ok && lane < N) {
        const int j = lane;
        float cx = 0.f, ch = 0.f;
        if (MODE != GRU_GX_PRE) cx = J.sx_w * s_scale[j];
        if (MODE != GRU_GH_PRE) ch = J.sh_w * s_scale[8 + j];
        float gx[3], gh[3];
#pragma unroll
        for (int gt = 0; gt < 3; ++gt) {
            const int row = gt * H + unit;
            if (MODE == GRU_GX_PRE) {
                gx[gt] = pre[gt];
            } else {
                const int a = mine[gt];
                float y = (float)a * cx;
                if (J.bx) y = y + bxv[gt];
                gx[gt] = y;
                if (J.tx.acc) J.tx.acc[(size_t)j * 3 * H + row] = a;
            }
            if (MODE == GRU_GH_PRE) {
                gh[gt] = pre[gt];
            } else {
                const int a = mine[MODE == GRU_FULL ? 3 + gt : gt];
                float y = (float)a * ch;
                if (J.bh) y = y + bhv[gt];
                gh[gt] = y;
                if (J.th.acc) J.th.acc[(size_t)j * 3 * H + row] = a;
            }
        }
        J.h_out[(size_t)j * J.ldo + unit] = gru_gates(gx, gh, hp);
    }
    gru_clear_words(jobs);
}

// Gates alone, for panels of more than 8 vectors whose two products came from the matrix
// cores: gx, gh [n x 3H] (biases included), one thread per (vector, hidden unit).
__global__ __launch_bounds__(256) void gru_gates_kernel(const float *__restrict__ gx, const float *__restrict__ gh,
                                                        const float *__restrict__ h_prev, int ldh, float *h_out, int ldo,
                                                        int H, int n)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)n * H) return;
    const int j = (int)(idx / H), u = (int)(idx - (size_t)j * H);
    const float *x = gx + (size_t)j * 3 * H + u, *h = gh + (size_t)j * 3 * H + u;
    const float xv[3] = {x[0], x[H], x[2 * H]}, hv[3] = {h[0], h[H], h[2 * H]};
    h_out[(size_t)j * ldo + u] = gru_gates(xv, hv, h_prev[(size_t)j * ldh + u]);
}

// The same gates, one block per vector, which also leaves the new state quantized for the products
// that consume it next (up to two code buffers with their own row pitch, pad bytes zero): the block
// holds the whole vector, so its max |h| costs one exchange.  Thread t owns units 4 t .. 4 t + 3 of
// every 1024 (G groups: H <= 1024 G, H % 4 == 0).
struct GatesQArgs {
    const float *gx, *gh, *h_prev;
    float *h_out;
    int8_t *q1, *q2;            // q2 may be NULL
    float *s1, *s2;
    int ldh, ldo, H, ld1, ld2;
};
template <int G>
__global__ __launch_bounds__(256) void gru_gates_q_kernel(GatesQArgs a)
{
    __shared__ float s_m[4];
    const int j = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, H = a.H;
    const float *x = a.gx + (size_t)j * 3 * H, *h = a.gh + (size_t)j * 3 * H, *hp = a.h_prev + (size_t)j * a.ldh;
    float4 hv[G];
    float m = 0.0f;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int u = (g * 256 + tid) * 4;
        hv[g] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (u < H) {
            const float4 x0 = *(const float4 *)(x + u), x1 = *(const float4 *)(x + H + u), x2 = *(const float4 *)(x + 2 * H + u);
            const float4 h0 = *(const float4 *)(h + u), h1 = *(const float4 *)(h + H + u), h2 = *(const float4 *)(h + 2 * H + u);
            const float4 p = *(const float4 *)(hp + u);
            const float xa[3] = {x0.x, x1.x, x2.x}, ha[3] = {h0.x, h1.x, h2.x};
            const float xb[3] = {x0.y, x1.y, x2.y}, hb[3] = {h0.y, h1.y, h2.y};
            const float xc[3] = {x0.z, x1.z, x2.z}, hc[3] = {h0.z, h1.z, h2.z};
            const float xd[3] = {x0.w, x1.w, x2.w}, hd[3] = {h0.w, h1.w, h2.w};
            hv[g] = make_float4(gru_gates(xa, ha, p.x), gru_gates(xb, hb, p.y), gru_gates(xc, hc, p.z), gru_gates(xd, hd, p.w));
            *(float4 *)(a.h_out + (size_t)j * a.ldo + u) = hv[g];
        }
        m = fmaxf(m, fmaxf(fmaxf(fabsf(hv[g].x), fabsf(hv[g].y)), fmaxf(fabsf(hv[g].z), fabsf(hv[g].w))));
    }
    m = wave_max_f(m);
    if (lane == 0) s_m[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
    float scale, inv;
    q8_scale_of(m, scale, inv);
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int u = (g * 256 + tid) * 4;
        const int code = q8_pack4(hv[g].x, hv[g].y, hv[g].z, hv[g].w, inv);       // zero past H
        if (u < a.ld1) *(int *)(a.q1 + (size_t)j * a.ld1 + u) = code;
        if (a.q2 && u < a.ld2) *(int *)(a.q2 + (size_t)j * a.ld2 + u) = code;
    }
    if (tid == 0) {
        a.s1[j] = scale;
        if (a.q2) a.s2[j] = scale;
    }
}

// Encoder recurrences of many sentences side by side (Eq. 1), one launch pair per time
// step.  Direction d = 0: forward state, columns [H, 2H) of enc_h, step t works on position
// t; d = 1: backward state, columns [0, H), position l - 1 - t.  Sentence s occupies rows
// [sent_off[s], sent_off[s + 1]) of enc_h [L x 2H] and of the input pre-activations
// gx[d] [L x 3H]; sentences shorter than t + 1 positions are skipped.
struct EncStepArgs {
    const int *sent_off;
    float *enc_h;
    const float *gx[2];          // Wx q(x_i) + bx for every position
    const float *gh[2];          // [S x 3H] recurrent products of this step
    int8_t *hq[2];               // [S x ld] codes of the previous states
    float *hs[2];                // [S] their scales
    int t, H, ld;
};

__device__ __forceinline__ bool enc_rows(const EncStepArgs &a, int s, int d, int &pos, int &prev)
{
    const int o = a.sent_off[s], l = a.sent_off[s + 1] - o;
    if (a.t >= l) return false;
    pos = d == 0 ? o + a.t : o + l - 1 - a.t;
    prev = d == 0 ? pos - 1 : pos + 1;
    return true;
}

// Block (s, d): quantizes the previous state of sentence s, direction d (zero at t = 0).
__global__ __launch_bounds__(256) void enc_quantize_kernel(EncStepArgs a)
{
    __shared__ float s_scale[1];
    __shared__ float s_red[4];
    const int s = blockIdx.x, d = blockIdx.y;
    int pos, prev;
    if (!enc_rows(a, s, d, pos, prev)) return;
    int8_t *xq = a.hq[d] + (size_t)s * a.ld;
    if (a.t == 0) {
        for (int k = threadIdx.x * 4; k < a.ld; k += 1024) *(int *)(xq + k) = 0;
        if (threadIdx.x == 0) a.hs[d][s] = 1.0f;
        return;
    }
    const float *h = a.enc_h + (size_t)prev * 2 * a.H + (d == 0 ? a.H : 0);
    block_quantize<1>(h, 1, a.H, a.H, a.ld, xq, s_scale, s_red);
    if (threadIdx.x == 0) a.hs[d][s] = s_scale[0];
}

// One thread per (direction, sentence, hidden unit): gates and the new state.
__global__ __launch_bounds__(256) void enc_gates_kernel(EncStepArgs a, int S)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int H = a.H;
    if (idx >= (size_t)2 * S * H) return;
    const int d = (int)(idx / ((size_t)S * H));
    const size_t rest = idx - (size_t)d * S * H;
    const int s = (int)(rest / H), u = (int)(rest - (size_t)s * H);
    int pos, prev;
    if (!enc_rows(a, s, d, pos, prev)) return;
    const float *x = a.gx[d] + (size_t)pos * 3 * H + u, *h = a.gh[d] + (size_t)s * 3 * H + u;
    const float xv[3] = {x[0], x[H], x[2 * H]}, hv[3] = {h[0], h[H], h[2 * H]};
    const int col = (d == 0 ? H : 0) + u;
    const float hp = a.t == 0 ? 0.0f : a.enc_h[(size_t)prev * 2 * H + col];
    a.enc_h[(size_t)pos * 2 * H + col] = gru_gates(xv, hv, hp);
}

// ============================================= encoder recurrence in one launch ==
// Eq. 1 for one sentence, both directions, all l positions in ONE launch whose blocks are all
// resident at once (the launcher checks that the device can hold them; otherwise the caller
// launches per position).  Block b
// of 512 threads owns eight hidden units of one direction, a wave one unit: its three recurrent
// weight rows stay in registers for the whole sentence.  Per position every block needs the whole
// previous state of its direction (H floats from all blocks of that direction).  There is no grid
// barrier: a unit's new value is published as one 8-byte word (float, step tag) with a
// device-coherent store into a double-buffered exchange array, and a consumer polls the words it
// needs with device-coherent loads until their tags are this step's.  Buffer t & 1 can only be
// overwritten (at step t + 2) by a block that has read all of step t + 1, which no block has written
// before it had read all of step t: two buffers suffice.  Every wait is bounded: after spin_limit
// polls (or as soon as another block has given up) a block sets the error word and goes on with
// what it has, so the kernel always ends; the error word is the caller's to check.
// Arithmetic per unit and position as in gru_fast_kernel<1, GRU_GX_PRE>: max-abs codes of the
// previous state, exact int32 sums, one scale product, bias, gates in fp32 with the double-precision
// sigmoid / tanh.  H % 8 == 0, H <= 2048, ld <= 2048, the exchange array zeroed before the launch.
struct EncPArgs {
    const int8_t *Wh[2];
    const float *bh[2];
    const float *gx[2];                  // [l x 3H] input pre-activations, biases included
    float *enc_h;                        // [l x 2H]: backward state in columns [0, H), forward in [H, 2H)
    unsigned long long *xchg;            // [2 buffers][2 directions][H] (value bits | tag << 32)
    unsigned *err;
    int l, H, ld, spin_limit;
    float sh_w[2];
};

#define ENCP_THREADS 512
template <int CH>           // 1024-byte chunks per weight row
__global__ __launch_bounds__(ENCP_THREADS) void encoder_persistent_kernel(EncPArgs a)
{
    __shared__ __align__(16) int8_t s_q[2048 + 16];
    __shared__ float s_max[ENCP_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int H = a.H, bpd = H / 8;                       // blocks per direction
    const int d = (int)blockIdx.x / bpd, u = ((int)blockIdx.x - d * bpd) * 8 + wave;
    const int col0 = d == 0 ? H : 0;

    // this wave's rows r, z, n of unit u, for the whole sentence
    v4i w[3][CH];
    {
        const int row[3] = {u, H + u, 2 * H + u};
        rows_load<3, CH, false>(w, q8_rsrc(a.Wh[d], (size_t)3 * H * a.ld), row, a.ld, lane);
    }
    float bh[3] = {0.f, 0.f, 0.f};
    if (a.bh[d]) {
#pragma unroll
        for (int g = 0; g < 3; ++g) bh[g] = a.bh[d][g * H + u];
    }
    float h_prev = 0.0f;

    for (int t = 0; t < a.l; ++t) {
        const int pos = d == 0 ? t : a.l - 1 - t;
        // the unit's input pre-activations of this position: lanes 0..2, requested before the wait
        const float gxl = lane < 3 ? a.gx[d][(size_t)pos * 3 * H + lane * H + u] : 0.0f;
        float scale = 1.0f;
        if (t > 0) {
            // previous state of this direction: thread tid takes units 2 tid, 2 tid + 1 (and + 1024 for H > 1024)
            const unsigned want = (unsigned)t;
            float v[CH][2], m = 0.0f;
            // A poll that comes too early costs a whole round trip to the device-coherent level and its loads
            // (2 per thread, 256 blocks) slow the stores everybody is waiting for.  The new values need about as
            // long to become visible as this pause of 8 x 64 cycles; measured at 50 positions: no pause 161 us,
            // 2: 143, 4: 108, 6: 102, 8: 102, 10: 105, 12: 108, 16: 112, 24: 123 (a pause between failed polls
            // instead: 193 us).
            __builtin_amdgcn_s_sleep(8);
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int i0 = c * 2 * ENCP_THREADS + 2 * tid;
                v[c][0] = v[c][1] = 0.0f;
                if (i0 < H) {
                    const unsigned long long *src = a.xchg + (size_t)(((t - 1) & 1) * 2 + d) * H + i0;
                    int spins = 0;
                    for (;;) {
                        // two published words, each read whole by an 8-byte device-coherent load
                        const unsigned long long r0 = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        const unsigned long long r1 = __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        v[c][0] = __uint_as_float((unsigned)r0);
                        v[c][1] = __uint_as_float((unsigned)r1);
                        if ((unsigned)(r0 >> 32) == want && (unsigned)(r1 >> 32) == want) break;
                        if (++spins >= a.spin_limit ||
                            ((spins & 63) == 0 && __hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
                            __hip_atomic_store(a.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                    }
                }
                m = fmaxf(m, fmaxf(fabsf(v[c][0]), fabsf(v[c][1])));
            }
            m = wave_max_f(m);
            if (lane == 0) s_max[wave] = m;
            __syncthreads();                     // (also: every wave has finished reading the previous step's codes)
            m = s_max[0];
#pragma unroll
            for (int ww = 1; ww < ENCP_THREADS / 64; ++ww) m = fmaxf(m, s_max[ww]);
            float inv;
            q8_scale_of(m, scale, inv);
#pragma unroll
            for (int c = 0; c < CH; ++c)         // codes of the units this thread read; zero past H
                *(short *)(s_q + c * 2 * ENCP_THREADS + 2 * tid) = (short)q8_pack2(v[c][0], v[c][1], inv);
            __syncthreads();
        }
        int acc[3] = {0, 0, 0};
        if (t > 0) {
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const v4i x = *(const v4i *)(s_q + (c * 64 + lane) * 16);
#pragma unroll
                for (int g = 0; g < 3; ++g) acc[g] = dot16(w[g][c], x, acc[g]);
            }
#pragma unroll
            for (int g = 0; g < 3; ++g) acc[g] = group_sum_i(acc[g], 64);
        }
        float gx[3], gh[3];
        const float ch = a.sh_w[d] * scale;
#pragma unroll
        for (int g = 0; g < 3; ++g) {
            gx[g] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(gxl), g));
            float y = (float)acc[g] * ch;
            if (a.bh[d]) y = y + bh[g];
            gh[g] = y;
        }
        // the gates of gru_gates, operation by operation, with the two sigmoids evaluated side by side in lanes 0 and 1
        const float pr = gx[0] + gh[0], pz = gx[1] + gh[1];
        const float sg = sigmoid_rn(lane == 1 ? pz : pr);
        const float r = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sg), 0));
        const float z = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(sg), 1));
        const float rn = r * gh[2];
        const float pn = gx[2] + rn;
        const float nn = tanh_rn(pn);
        const float omz = 1.0f - z;
        const float t1 = omz * nn;
        const float t2 = z * h_prev;
        const float h_new = t1 + t2;
        if (lane == 0) {
            // published first: the other blocks are waiting for it
            const unsigned long long word = (unsigned long long)__float_as_uint(h_new) | ((unsigned long long)(unsigned)(t + 1) << 32);
            __hip_atomic_store(a.xchg + (size_t)((t & 1) * 2 + d) * H + u, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            a.enc_h[(size_t)pos * 2 * H + col0 + u] = h_new;
        }
        h_prev = h_new;                          // (the same value in every lane of the wave)
        // The block's waves start to poll together.  Without this barrier the waves that are done early poll
        // while the last one still computes, and the extra device-coherent loads of 256 blocks slow every
        // exchange down (measured before the pause above was added: 217 us for 50 positions against 153 us).
        __syncthreads();
    }
}

// =================================================================== host launchers ==

q8_status q8i_enc_step(q8_ctx *ctx, int phase, const int *sent_off, int S, int t, int H, int ld, float *enc_h,
                       const float *gxf, const float *gxb, float *ghf, float *ghb, int8_t *hqf, int8_t *hqb, float *hsf,
                       float *hsb)
{
    EncStepArgs a = {sent_off, enc_h, {gxf, gxb}, {ghf, ghb}, {hqf, hqb}, {hsf, hsb}, t, H, ld};
    if (phase == 0) {
        hipLaunchKernelGGL(enc_quantize_kernel, dim3(S, 2), dim3(256), 0, ctx->stream, a);
    } else {
        const size_t total = (size_t)2 * S * H;
        Q8_LAUNCH(ctx, Q8_KERNEL_GRU, enc_gates_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, a, S);
    }
    return q8i_launch_check(ctx, "encoder step");
}


q8_status q8i_gru_gates(q8_ctx *ctx, const float *gx, const float *gh, const float *h_prev, int ldh, float *h_out,
                        int ldo, int H, int n)
{
    const size_t total = (size_t)n * H;
    Q8_LAUNCH(ctx, Q8_KERNEL_GRU, gru_gates_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, gx, gh, h_prev, ldh,
              h_out, ldo, H, n);
    return q8i_launch_check(ctx, "gru gates");
}


// gates + codes of the new states; false if the shape is not covered (the caller then runs the
// gates and the quantization as two launches)
bool q8i_gru_gates_q_ok(int H, int ldh, int ldo, int ld1, int ld2)
{
    const int G = (H + 1023) / 1024;
    return H % 4 == 0 && ldh % 4 == 0 && ldo % 4 == 0 && G <= 4 && ld1 <= 1024 * G && ld2 <= 1024 * G && ld1 % 4 == 0 && ld2 % 4 == 0;
}

q8_status q8i_gru_gates_q(q8_ctx *ctx, const float *gx, const float *gh, const float *h_prev, int ldh, float *h_out,
                          int ldo, int H, int n, int8_t *q1, int ld1, float *s1, int8_t *q2, int ld2, float *s2)
{
    GatesQArgs a = {gx, gh, h_prev, h_out, q1, q2, s1, s2, ldh, ldo, H, ld1, q2 ? ld2 : 0};
    const int G = (H + 1023) / 1024;
    if (G == 1) Q8_LAUNCH(ctx, Q8_KERNEL_GRU, gru_gates_q_kernel<1>, dim3(n), dim3(256), 0, a);
    else if (G == 2) Q8_LAUNCH(ctx, Q8_KERNEL_GRU, gru_gates_q_kernel<2>, dim3(n), dim3(256), 0, a);
    else Q8_LAUNCH(ctx, Q8_KERNEL_GRU, gru_gates_q_kernel<4>, dim3(n), dim3(256), 0, a);
    return q8i_launch_check(ctx, "gru gates + codes");
}

// ================================= products and gates of a panel in one launch ==
// One GRU transition (Eq. 1, 3, 4) for a panel of hypothesis slots without the two [n x 3H] arrays
// of pre-activations ever reaching memory: the matrix-core products of the block kernels above and
// the gates of gru_gates_q_kernel, value for value, in one kernel.  Block (ug, cg) of twelve waves
// owns hidden units 32 ug .. 32 ug + 31 and slots 48 cg .. 48 cg + 47.  Wave (rt, kp), rt = 2 gate +
// unit tile, kp = 0 / 1, multiplies the 16 weight rows of its gate and unit tile over one part of
// the k range against the block's slots (codes parked in LDS, 48 slots whole):
//   both products here (GH_PRE false): kp = 0 is W_x (KS0 k steps of 64 bytes), kp = 1 is W_h (KS1);
//   recurrent product given (GH_PRE true): W_x alone, kp = 0 its first KS0 k steps, kp = 1 the next
//   KS1; the two exact int32 partial sums are added before the one dequantization.
// The accumulators cross to the threads that apply the gates through LDS; thread -> (slot, unit)
// with consecutive threads on consecutive units, two pairs per thread.
// The codes of the new state need max |h| over all H units of a slot, which the H / 32 blocks of a
// column group hold between them.  Each block publishes its 48 partial maxima as 4-byte words
// (float bits + 1, so that zero means "not there yet") with device-coherent stores and polls the
// group's words; with all of them it quantizes the values it still holds in registers.  The waits
// are bounded (a wait that gives up raises the context's flag and the kernel still ends), and the
// launcher checks that the device holds all blocks at once.  Words must be zero on entry: two regions
// take turns (GRU r of a decoder step uses one, GRU q the other) and every launch clears the region it
// does not use, which the launch before it has finished with; the host keeps track and clears by
// a fill where that order is broken.
#define GP_UNITS 32
#define GP_SLOTS 48
#define GP_WAVES 12
#define GP_MAX_CG 7          // column groups of a launch whose blocks exchange maxima (336 slots)
#define GP_REGION_WORDS (GP_MAX_CG * 32 * GP_SLOTS)
struct GruPanelArgs {
    const int8_t *Wx, *Wh;      // [3H x ldx], [3H x ldh] (Wh unused with GH_PRE)
    const int8_t *Wxt, *Wht;    // the same tile-packed (q8_pack_tiles) or NULL: one contiguous KiB per matrix-core operand
    const float *bx, *bh;       // [3H] or NULL
    const int8_t *xq, *hq;      // codes [n x ldx], [n x ldh]
    const float *xs, *hs;       // [n]
    const float *gh_pre;        // GH_PRE: [n x 3H], bias included
    const float *h_prev;        // [n x ldp]
    float *h_out;               // [n x ldo]
    int8_t *q1, *q2;            // codes of h_out [n x ld1], [n x ld2] (q2 may be NULL), pad bytes zero
    float *s1, *s2;
    unsigned *xw;               // exchange words [2 regions][GP_MAX_CG][32 unit groups][48 slots]
    unsigned *wait_err;
    int region, spin_limit;
    int H, n, ldx, ldh, ldp, ldo, ld1, ld2;
    float wx_scale, wh_scale;
};

template <int KS0, int KS1, bool GH_PRE>
__global__ __launch_bounds__(64 * GP_WAVES) void gru_panel_kernel(GruPanelArgs a)
{
    extern __shared__ __align__(16) int8_t s_gp[];
    __shared__ float s_mx[2 * 64 * GP_WAVES];          // the column group's maxima [unit group][slot]
    constexpr int KSM = KS0 > KS1 ? KS0 : KS1;
    constexpr int NT = 64 * GP_WAVES;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave-uniform, and known to be
    const int i = lane & 15, g = lane >> 4;
    const int ug = blockIdx.x, cg = blockIdx.y;
    const int H = a.H, n = a.n, c0 = cg * GP_SLOTS, u0 = ug * GP_UNITS;
    constexpr int ldx = GH_PRE ? 64 * (KS0 + KS1) : 64 * KS0, ldh = GH_PRE ? 0 : 64 * KS1;     // the launcher checks a.ldx, a.ldh
    constexpr int px = ldx + 16, ph = ldh + 16;                  // LDS pitches of the two code regions
    int8_t *s_x = s_gp, *s_h = s_gp + GP_SLOTS * px;
    int *s_e = (int *)(s_gp + GP_SLOTS * px + (GH_PRE ? 0 : GP_SLOTS * ph));     // [12 waves][3 tiles][16 slots][16 units]
    // the exchange words of the region this launch does not use, for this block's unit group: its own
    // column group, and the last column group also those beyond the grid
    if (a.q1 && tid < GP_SLOTS) {
        unsigned *other = a.xw + (size_t)(1 - a.region) * GP_REGION_WORDS + ug * GP_SLOTS + tid;
        const int last = cg == (int)gridDim.y - 1 ? GP_MAX_CG : cg + 1;
        for (int c2 = cg; c2 < last; ++c2) other[(size_t)c2 * 32 * GP_SLOTS] = 0u;
    }

    // ---- every load of the products, requested before the first wait (outside the arrays: zero) ----
    // the slots' codes in 16-byte pieces: UX rounds of the block's threads for x, UH for h
    constexpr int PCX = ldx / 16, PCH = ldh / 16, UX = GP_SLOTS * PCX / NT, UH = GP_SLOTS * PCH / NT;
    static_assert(GP_SLOTS * PCX % NT == 0 && GP_SLOTS * PCH % NT == 0, "pieces divide among the threads");
    const __amdgpu_buffer_rsrc_t rxq = q8_rsrc(a.xq, (size_t)n * ldx);
    const __amdgpu_buffer_rsrc_t rhq = q8_rsrc(GH_PRE ? a.xq : a.hq, GH_PRE ? 0 : (size_t)n * ldh);
    v4i bqx[UX], bqh[UH > 0 ? UH : 1];
#pragma unroll
    for (int u = 0; u < UX; ++u) {
        const int p = u * NT + tid, slot = p / PCX, piece = p - slot * PCX;
        const unsigned off = c0 + slot < n ? (unsigned)(c0 + slot) * (unsigned)ldx + 16u * piece : Q8_OOB;
        bqx[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rxq, (int)off, 0, 0));
    }
#pragma unroll
    for (int u = 0; u < UH; ++u) {
        const int p = u * NT + tid, slot = p / (PCH > 0 ? PCH : 1), piece = p - slot * PCH;
        const unsigned off = c0 + slot < n ? (unsigned)(c0 + slot) * (unsigned)ldh + 16u * piece : Q8_OOB;
        bqh[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rhq, (int)off, 0, 0));
    }
    // this wave's 16 weight rows over its part of the k range
    const int rt = wave % 6, kp = wave / 6, gate = rt >> 1, ut = rt & 1;
    const bool from_h = !GH_PRE && kp == 1;
    const int ks = kp == 0 ? KS0 : KS1;                           // k steps of this wave
    const int kbase = GH_PRE && kp == 1 ? 64 * KS0 : 0;           // first k byte within the matrix's rows
    const int ldw = from_h ? ldh : ldx;
    const int8_t *wt = from_h ? a.Wht : a.Wxt;
    const __amdgpu_buffer_rsrc_t rw = q8_rsrc(wt ? wt : (from_h ? a.Wh : a.Wx), (size_t)3 * H * ldw);
    const int row0 = gate * H + u0 + 16 * ut, row = row0 + i;             // H % 16 == 0: row0 starts a tile
    v4i av[KSM];
#pragma unroll
    for (int s = 0; s < KSM; ++s) {
        const int k = kbase + 64 * s + 16 * g;
        unsigned off = (s < ks && k < ldw) ? (unsigned)row * (unsigned)ldw + (unsigned)k : Q8_OOB;
        if (wt) off = s < ks ? (((unsigned)(row0 >> 4) * (unsigned)(ldw >> 6) + (unsigned)((kbase >> 6) + s)) << 10) + 16u * lane : Q8_OOB;
        av[s] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rw, (int)off, 0, 0));
    }
    // what the gates need per (slot, unit) pair: pairs tid and tid + NT of 48 x 32
    const __amdgpu_buffer_rsrc_t rxs = q8_rsrc(a.xs, (size_t)n * 4), rhs = q8_rsrc(GH_PRE ? a.xs : a.hs, GH_PRE ? 0 : (size_t)n * 4);
    const __amdgpu_buffer_rsrc_t rbx = q8_rsrc(a.bx, a.bx ? (size_t)3 * H * 4 : 0), rbh = q8_rsrc(a.bh, (!GH_PRE && a.bh) ? (size_t)3 * H * 4 : 0);
    const __amdgpu_buffer_rsrc_t rgh = q8_rsrc(a.gh_pre, GH_PRE ? (size_t)n * 3 * H * 4 : 0);
    const __amdgpu_buffer_rsrc_t rhp = q8_rsrc(a.h_prev, ((size_t)(n - 1) * a.ldp + H) * 4);
    float xsv[2], hsv[2], hpv[2], bxv[2][3], bhv[2][3];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int pr = e * NT + tid, c = pr >> 5, u = pr & 31, col = c0 + c, unit = u0 + u;
        const bool ok = col < n;
        xsv[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rxs, (int)(ok ? (unsigned)col * 4u : Q8_OOB), 0, 0));
        hsv[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rhs, (int)(ok ? (unsigned)col * 4u : Q8_OOB), 0, 0));
        hpv[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rhp, (int)(ok ? ((unsigned)col * (unsigned)a.ldp + (unsigned)unit) * 4u : Q8_OOB), 0, 0));
#pragma unroll
        for (int gt = 0; gt < 3; ++gt) {
            const unsigned r4 = (unsigned)(gt * H + unit) * 4u;
            bxv[e][gt] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rbx, (int)r4, 0, 0));
            // GH_PRE: the given recurrent pre-activation takes the place of (product, bias)
            bhv[e][gt] = GH_PRE ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rgh, (int)(ok ? ((unsigned)col * 3u * (unsigned)H) * 4u + r4 : Q8_OOB), 0, 0))
                                : __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rbh, (int)r4, 0, 0));
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- codes into LDS ----
#pragma unroll
    for (int u = 0; u < UX; ++u) {
        const int p = u * NT + tid, slot = p / PCX, piece = p - slot * PCX;
        *(v4i *)(s_x + slot * px + 16 * piece) = bqx[u];
    }
#pragma unroll
    for (int u = 0; u < UH; ++u) {
        const int p = u * NT + tid, slot = p / (PCH > 0 ? PCH : 1), piece = p - slot * PCH;
        *(v4i *)(s_h + slot * ph + 16 * piece) = bqh[u];
    }
    __syncthreads();

    // ---- products: three column tiles, independent accumulation chains ----
    v4i acc[3];
#pragma unroll
    for (int t = 0; t < 3; ++t) acc[t] = (v4i){0, 0, 0, 0};
    {
        const int8_t *bp = (from_h ? s_h + i * ph : s_x + i * px + kbase) + 16 * g;
        const int pitch = from_h ? ph : px;
#pragma unroll
        for (int s = 0; s < KSM; ++s) {
            if (s < ks) {                                           // wave-uniform
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    const v4i bv = *(const v4i *)(bp + t * 16 * pitch + 64 * s);
                    acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[s], bv, acc[t], 0, 0, 0);
                }
            }
        }
    }
    // lane (i, g) holds units 4 g + r, r = 0..3, of slot i of each tile
#pragma unroll
    for (int t = 0; t < 3; ++t) *(v4i *)(s_e + (((wave * 3 + t) * 16 + i) * 16 + 4 * g)) = acc[t];
    __syncthreads();

    // ---- gates ----
    float hn[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int pr = e * NT + tid, c = pr >> 5, u = pr & 31, col = c0 + c, unit = u0 + u;
        const float cx = a.wx_scale * xsv[e], ch = a.wh_scale * hsv[e];
        float gx[3], gh[3];
#pragma unroll
        for (int gt = 0; gt < 3; ++gt) {
            const int w0 = gt * 2 + (u >> 4);
            const int e0 = s_e[(((w0 * 3 + (c >> 4)) * 16 + (c & 15)) * 16 + (u & 15))];
            const int e1 = s_e[((((6 + w0) * 3 + (c >> 4)) * 16 + (c & 15)) * 16 + (u & 15))];
            if (GH_PRE) {
                float y = (float)(e0 + e1) * cx;
                if (a.bx) y = y + bxv[e][gt];
                gx[gt] = y;
                gh[gt] = bhv[e][gt];
            } else {
                float y = (float)e0 * cx;
                if (a.bx) y = y + bxv[e][gt];
                gx[gt] = y;
                float z = (float)e1 * ch;
                if (a.bh) z = z + bhv[e][gt];
                gh[gt] = z;
            }
        }
        hn[e] = gru_gates(gx, gh, hpv[e]);
        if (col < n) a.h_out[(size_t)col * a.ldo + unit] = hn[e];
    }
    if (!a.q1) return;

    // ---- codes: this block's maxima out, the column group's in ----
    unsigned *mine = a.xw + (size_t)a.region * GP_REGION_WORDS + (size_t)cg * 32 * GP_SLOTS;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int pr = e * NT + tid, c = pr >> 5, col = c0 + c;
        float m = col < n ? fmaxf(0.0f, fabsf(hn[e])) : 0.0f;
        // over the 32 lanes that share the slot
        m = fmaxf(m, __int_as_float(dpp_mov_i<DPP_XOR1>(__float_as_int(m))));
        m = fmaxf(m, __int_as_float(dpp_mov_i<DPP_XOR2>(__float_as_int(m))));
        m = fmaxf(m, __int_as_float(dpp_mov_i<DPP_HALF_MIRROR>(__float_as_int(m))));
        m = fmaxf(m, __int_as_float(dpp_mov_i<DPP_MIRROR>(__float_as_int(m))));
        m = fmaxf(m, __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(m), SWZ_XOR16)));
        if ((lane & 31) == 0)
            __hip_atomic_store(mine + ug * GP_SLOTS + c, __float_as_uint(m) + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    {
        // thread t polls words t and t + NT of the group's gridDim.x * 48
        const int nw = (int)gridDim.x * GP_SLOTS;
        unsigned w0 = tid < nw ? 0u : 1u, w1 = tid + NT < nw ? 0u : 1u;
        bool ok = false;
        // A poll is a round trip to the device-coherent level, 1.4 us and more while 224 blocks publish and poll
        // 43 KB of words at once; the blocks publish within 0.6 us of each other, so the first poll waits that
        // long (6 x 256 clocks) and then finds everything (measured: no failed first polls, 0.9 us less per decoder
        // step at 64 sentences than polling at once).
        // (A bound of one poll means no waiting at all, pause included: the give-up path under test.)
        if (a.spin_limit > 1)
            for (int p = 0; p < 6; ++p) __builtin_amdgcn_s_sleep(4);
        for (int spin = 0; spin < a.spin_limit; ++spin) {
            if (!w0) w0 = __hip_atomic_load(mine + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (!w1) w1 = __hip_atomic_load(mine + NT + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (w0 && w1) { ok = true; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        if (!ok) __hip_atomic_store(a.wait_err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_mx[tid] = w0 ? __uint_as_float(w0 - 1u) : 0.0f;
        s_mx[NT + tid] = w1 ? __uint_as_float(w1 - 1u) : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int pr = e * NT + tid, c = pr >> 5, u = pr & 31, col = c0 + c, unit = u0 + u;
        float m = 0.0f;
        for (int g2 = 0; g2 < (int)gridDim.x; ++g2) m = fmaxf(m, s_mx[g2 * GP_SLOTS + c]);
        float scale, inv;
        q8_scale_of(m, scale, inv);
        const int8_t code = (int8_t)(q8_pack2(hn[e], 0.0f, inv) & 0xff);
        if (col < n) {
            a.q1[(size_t)col * a.ld1 + unit] = code;
            if (a.q2) a.q2[(size_t)col * a.ld2 + unit] = code;
            if (ug == 0 && u == 0) {
                a.s1[col] = scale;
                if (a.q2) a.s2[col] = scale;
            }
        }
    }
}

// Whether the one-launch panel GRU takes this shape (rows of 512 + 1024 bytes for both products, or rows of
// 2048 bytes for the input product alone; H a multiple of 32, at most 1024; code rows of exactly H bytes), and,
// where codes are wanted (its blocks then wait for each other), whether the context allows such kernels
// and the device holds the whole grid at once.
bool q8i_gru_panel_ok(q8_ctx *ctx, const q8_gru_weights *g, bool gh_pre, int n, int ldp, int ldo, bool codes, int ld1, int ld2, bool have_q2)
{
    const int H = g->Wh.cols;
    if (H % GP_UNITS || H > 1024 || n < 1 || n > Q8_MAX_COLS) return false;
    if (ldp % 4 || ldo % 4) return false;
    if (g->Wx.rows != 3 * H || (size_t)3 * H * g->Wx.ld >= (1u << 31) || (size_t)n * g->Wx.ld >= (1u << 31)) return false;
    if (gh_pre ? g->Wx.ld != 2048 : (g->Wx.ld != 512 || g->Wh.ld != 1024 || g->Wh.rows != 3 * H)) return false;
    if (!codes) return true;
    if (ld1 != H || (have_q2 && ld2 != H) || !ctx->att_split) return false;
    const int ncg = (n + GP_SLOTS - 1) / GP_SLOTS;
    if (ncg > GP_MAX_CG) return false;
    static int capacity[2] = {-1, -1};
    const int v = gh_pre ? 1 : 0;
    if (capacity[v] < 0) {
        int per_cu = 0, dev = 0, cus = 0;
        const size_t smem = (size_t)GP_SLOTS * (gh_pre ? 2048 + 16 : 512 + 16 + 1024 + 16) + (size_t)GP_WAVES * 3 * 256 * sizeof(int);
        hipError_t e = gh_pre ? hipFuncSetAttribute((const void *)gru_panel_kernel<16, 16, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem)
                              : hipFuncSetAttribute((const void *)gru_panel_kernel<8, 16, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e == hipSuccess)
            e = gh_pre ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gru_panel_kernel<16, 16, true>, 64 * GP_WAVES, smem)
                       : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gru_panel_kernel<8, 16, false>, 64 * GP_WAVES, smem);
        if (e == hipSuccess) e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) { (void)hipGetLastError(); return false; }
        capacity[v] = per_cu * cus;
    }
    return (H / GP_UNITS) * ncg <= capacity[v];
}

// region: which of the two sets of exchange words this launch uses (0: GRU r of a decoder step and single
// transitions, 1: GRU q), the other being cleared by it.
q8_status q8i_gru_panel(q8_ctx *ctx, const q8_gru_weights *g, const int8_t *xq, const float *xs, const int8_t *hq,
                        const float *hs, const float *gh_pre, const float *h_prev, int ldp, float *h_out, int ldo, int n,
                        int8_t *q1, int ld1, float *s1, int8_t *q2, int ld2, float *s2, int region)
{
    GruPanelArgs a;
    a.Wx = g->Wx.data; a.Wh = g->Wh.data; a.bx = g->bx; a.bh = g->bh;
    a.Wxt = g->Wx.tiles; a.Wht = g->Wh.tiles;
    a.xq = xq; a.hq = hq; a.xs = xs; a.hs = hs; a.gh_pre = gh_pre; a.h_prev = h_prev; a.h_out = h_out;
    a.q1 = q1; a.q2 = q2; a.s1 = s1; a.s2 = s2;
    a.xw = (unsigned *)(ctx->ws + Q8_WS_GRUP_XCHG);
    a.wait_err = (unsigned *)(ctx->ws + Q8_WS_ATT_ERR);
    a.region = region ? 1 : 0; a.spin_limit = ctx->att_spin_limit;
    a.H = g->Wh.cols; a.n = n; a.ldx = g->Wx.ld; a.ldh = g->Wh.ld; a.ldp = ldp; a.ldo = ldo; a.ld1 = ld1; a.ld2 = q2 ? ld2 : 0;
    a.wx_scale = g->Wx.scale; a.wh_scale = g->Wh.scale;
    const dim3 grid(a.H / GP_UNITS, (n + GP_SLOTS - 1) / GP_SLOTS);
    if (q1) {
        // the region this launch uses must be clear, and the launch clears the other one for its own unit
        // groups: anything beyond that (a launch before this one with more unit groups, or two launches in
        // a row on one region) is cleared here
        const int r = a.region, ugs = (int)grid.x;
        q8_status st = Q8_OK;
        if (ctx->grup_used[r]) st = q8i_fill_u32(ctx, a.xw + (size_t)r * GP_REGION_WORDS, GP_REGION_WORDS, 0u);
        if (!st && ctx->grup_used[1 - r] > ugs) st = q8i_fill_u32(ctx, a.xw + (size_t)(1 - r) * GP_REGION_WORDS, GP_REGION_WORDS, 0u);
        if (st) return st;
        ctx->grup_used[1 - r] = 0;
        ctx->grup_used[r] = ugs;
    }
    const size_t e_bytes = (size_t)GP_WAVES * 3 * 256 * sizeof(int);
    static bool attr_set[2] = {false, false};
    if (gh_pre) {
        const size_t smem = (size_t)GP_SLOTS * (a.ldx + 16) + e_bytes;
        if (!attr_set[1]) {
            const hipError_t e = hipFuncSetAttribute((const void *)gru_panel_kernel<16, 16, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return q8_fail(ctx, Q8_ERR_DEVICE, "panel GRU kernel: %s", hipGetErrorString(e));
            attr_set[1] = true;
        }
        Q8_LAUNCH(ctx, Q8_KERNEL_GRU, (gru_panel_kernel<16, 16, true>), grid, dim3(64 * GP_WAVES), smem, a);
    } else {
        const size_t smem = (size_t)GP_SLOTS * (a.ldx + 16 + a.ldh + 16) + e_bytes;
        if (!attr_set[0]) {
            const hipError_t e = hipFuncSetAttribute((const void *)gru_panel_kernel<8, 16, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return q8_fail(ctx, Q8_ERR_DEVICE, "panel GRU kernel: %s", hipGetErrorString(e));
            attr_set[0] = true;
        }
        Q8_LAUNCH(ctx, Q8_KERNEL_GRU, (gru_panel_kernel<8, 16, false>), grid, dim3(64 * GP_WAVES), smem, a);
    }
    return q8i_launch_check(ctx, "panel GRU");
}

template <int N, int MODE>
static void launch_gru_nm(q8_ctx *ctx, const GruJobs &jobs, int njobs, int blocks, size_t smem, int ch, bool xpre)
{
    dim3 grid(blocks, njobs);
    if constexpr (MODE != GRU_GX_PRE) {
        if (xpre && (ch == 1 || ch == 2)) {
            if (ch == 1) Q8_LAUNCH(ctx, Q8_KERNEL_GRU, (gru_fast_kernel<N, MODE, 1, true>), grid, dim3(256), smem, jobs);
            else Q8_LAUNCH(ctx, Q8_KERNEL_GRU, (gru_fast_kernel<N, MODE, 2, true>), grid, dim3(256), smem, jobs);
            return;
        }
    }
    if (ch == 1) Q8_LAUNCH(ctx, Q8_KERNEL_GRU, (gru_fast_kernel<N, MODE, 1>), grid, dim3(256), smem, jobs);
    else if (ch == 2) Q8_LAUNCH(ctx, Q8_KERNEL_GRU, (gru_fast_kernel<N, MODE, 2>), grid, dim3(256), smem, jobs);
    else Q8_LAUNCH(ctx, Q8_KERNEL_GRU, (gru_kernel<N, MODE>), grid, dim3(256), smem, jobs);
}

template <int N>
static void launch_gru_n(q8_ctx *ctx, const GruJobs &jobs, int njobs, int mode, int blocks, size_t smem, int ch, bool xpre)
{
    if (mode == GRU_FULL) launch_gru_nm<N, GRU_FULL>(ctx, jobs, njobs, blocks, smem, ch, xpre);
    else if (mode == GRU_GX_PRE) launch_gru_nm<N, GRU_GX_PRE>(ctx, jobs, njobs, blocks, smem, ch, false);
    else launch_gru_nm<N, GRU_GH_PRE>(ctx, jobs, njobs, blocks, smem, ch, xpre);
}

q8_status q8i_gru(q8_ctx *ctx, const q8i_gru_desc *d, int njobs, int n, int mode)
{
    GruJobs jobs;
    jobs.clear = d[0].clear;
    jobs.clear_words = d[0].clear ? d[0].clear_words : 0;
    size_t smem = 0;
    int max_ld = 0, maxH = 0;
    // codes in place of the vectors that are multiplied here (x; with both products also h_prev): only if every job brings them
    bool fast = true, xpre = mode != GRU_GX_PRE;
    for (int t = 0; t < njobs; ++t) {
        GruJob &J = jobs.j[t];
        const q8_gru_weights *g = d[t].g;
        J.Wx = g->Wx.data; J.Wh = g->Wh.data; J.bx = g->bx; J.bh = g->bh;
        J.x = d[t].x; J.h_prev = d[t].h_prev; J.g_pre = d[t].g_pre; J.h_out = d[t].h_out;
        J.xq_pre = d[t].xq_pre; J.xs_pre = d[t].xs_pre;
        J.hq_pre = d[t].hq_pre; J.hs_pre = d[t].hs_pre;
        J.xq_out = d[t].xs_out ? d[t].xq_out : nullptr; J.xs_out = d[t].xs_out;
        if (!J.xq_pre || !J.xs_pre) xpre = false;
        if (mode == GRU_FULL && (!J.hq_pre || !J.hs_pre)) xpre = false;
        q8_taps none = {nullptr, nullptr, nullptr};
        J.tx = d[t].taps ? d[t].taps[0] : none;
        J.th = d[t].taps ? d[t].taps[1] : none;
        J.I = g->Wx.cols; J.ldwx = g->Wx.ld; J.H = g->Wh.cols; J.ldwh = g->Wh.ld;
        J.ldx = d[t].ldx; J.ldh = d[t].ldh; J.ldo = d[t].ldo; J.ldg = d[t].ldg;
        J.sx_w = g->Wx.scale; J.sh_w = g->Wh.scale;
        const int lx = mode == GRU_GX_PRE ? 0 : J.ldwx, lh = mode == GRU_GH_PRE ? 0 : J.ldwh;
        if (lx > max_ld) max_ld = lx;
        if (lh > max_ld) max_ld = lh;
        if (J.H > maxH) maxH = J.H;
        if ((mode != GRU_GX_PRE && J.I % 4) || J.H % 4) fast = false;
        if ((size_t)3 * J.H * J.ldwx >= (1u << 31) || (size_t)3 * J.H * J.ldwh >= (1u << 31)) fast = false;   // 32-bit offsets
        int ldmin = mode == GRU_GX_PRE ? J.ldwh : (mode == GRU_GH_PRE ? J.ldwx : (J.ldwx < J.ldwh ? J.ldwx : J.ldwh));
        J.lpr = q8_lanes_per_row(ldmin);
        const size_t s = (size_t)n * (lx + lh);
        if (s > smem) smem = s;
    }
    int ch = fast ? q8_fast_ch(max_ld) : 0;
    if (ch == 4) ch = 0;                           // rows beyond 2048 bytes take the general kernel
    int blocks = 0;
    for (int t = 0; t < njobs; ++t) {
        const GruJob &J = jobs.j[t];
        const int upb = ch ? 4 : 4 * (64 / J.lpr);
        const int b = (J.H + upb - 1) / upb;
        if (b > blocks) blocks = b;
    }
    switch (n) {
    case 1: launch_gru_n<1>(ctx, jobs, njobs, mode, blocks, smem, ch, xpre); break;
    case 2: launch_gru_n<2>(ctx, jobs, njobs, mode, blocks, smem, ch, xpre); break;
    case 3: launch_gru_n<3>(ctx, jobs, njobs, mode, blocks, smem, ch, xpre); break;
    case 4: launch_gru_n<4>(ctx, jobs, njobs, mode, blocks, smem, ch, xpre); break;
    case 5: launch_gru_n<5>(ctx, jobs, njobs, mode, blocks, smem, ch, xpre); break;
    case 6: launch_gru_n<6>(ctx, jobs, njobs, mode, blocks, smem, ch, xpre); break;
    case 7: launch_gru_n<7>(ctx, jobs, njobs, mode, blocks, smem, ch, xpre); break;
    default: launch_gru_n<8>(ctx, jobs, njobs, mode, blocks, smem, ch, xpre); break;
    }
    return q8i_launch_check(ctx, "gru");
}

// The encoder recurrence of one sentence in one launch.  Returns Q8_OK with *launched = 0
// when the shape is not covered or the device cannot hold all blocks at once (the caller then
// launches per position).  xchg: 4 H words of 8 bytes, zeroed here; err: one word, set to 1 by the
// kernel if a wait gave up.
q8_status q8i_encode_persistent(q8_ctx *ctx, const q8_gru_weights *fwd, const q8_gru_weights *bwd, const float *gxf,
                                const float *gxb, int l, float *enc_h, unsigned long long *xchg, unsigned *err,
                                int spin_limit, int *launched)
{
    *launched = 0;
    const int H = fwd->Wh.cols, ld = fwd->Wh.ld;
    if (H % 8 || H > 2048 || ld > 2048 || bwd->Wh.ld != ld || bwd->Wh.cols != H || l < 1) return Q8_OK;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(ctx->stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return Q8_OK;
    const int ch = ld <= 1024 ? 1 : 2;
    const void *kern = ch == 1 ? (const void *)encoder_persistent_kernel<1> : (const void *)encoder_persistent_kernel<2>;
    const int blocks = 2 * (H / 8);
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, ENCP_THREADS, 0) != hipSuccess ||
        (long long)per_cu * cus < blocks) {
        (void)hipGetLastError();
        return Q8_OK;
    }
    // (the error word is zero between calls: the workspace header starts zeroed and q8_encode_check clears it)
    q8_status st = q8i_fill_u32(ctx, xchg, 4 * H * 2, 0u);
    if (st) return st;
    EncPArgs a;
    a.Wh[0] = fwd->Wh.data; a.Wh[1] = bwd->Wh.data; a.bh[0] = fwd->bh; a.bh[1] = bwd->bh;
    a.gx[0] = gxf; a.gx[1] = gxb; a.enc_h = enc_h; a.xchg = xchg; a.err = err;
    a.l = l; a.H = H; a.ld = ld; a.spin_limit = spin_limit;
    a.sh_w[0] = fwd->Wh.scale; a.sh_w[1] = bwd->Wh.scale;
    // An ordinary launch: the grid fits the device (checked above), earlier work of this stream has ended when
    // it starts, and work of other streams ends without needing this kernel, so every block becomes resident;
    // a cooperative launch, which promises that, costs about 15 us more per call here.
    if (ch == 1) Q8_LAUNCH(ctx, Q8_KERNEL_GRU, encoder_persistent_kernel<1>, dim3(blocks), dim3(ENCP_THREADS), 0, a);
    else Q8_LAUNCH(ctx, Q8_KERNEL_GRU, encoder_persistent_kernel<2>, dim3(blocks), dim3(ENCP_THREADS), 0, a);
    st = q8i_launch_check(ctx, "encoder recurrence");
    if (st) return st;
    *launched = 1;
    return Q8_OK;
}
