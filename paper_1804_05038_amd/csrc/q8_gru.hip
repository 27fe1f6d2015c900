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

// Gates of one hidden unit from its six pre-activations (fp32, one operation per
// statement, transcendental functions in double rounded once).
__device__ __forceinline__ float gru_gates(const float (&gx)[3], const float (&gh)[3], float h_prev)
{
    const float pr = gx[0] + gh[0];
    const float r = sigmoid_rn(pr);
    const float pz = gx[1] + gh[1];
    const float z = sigmoid_rn(pz);
    const float rn = r * gh[2];
    const float pn = gx[2] + rn;
    const float nn = tanh_rn(pn);
    const float omz = 1.0f - z;
    const float t1 = omz * nn;
    const float t2 = z * h_prev;
    return t1 + t2;
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
