// q8_output.hip -- second layer of the output network g of Eq. 2 ("Pieces of Eight: 8-bit
// Neural Machine Translation"): the vocabulary projection as Section 3's narrow product
// on the int8 matrix cores, fused with bias, log-sum-exp partials and a per-block top-k;
// a small second kernel merges the partials.
#include "q8_internal.h"

#include <hip/hip_ext.h>

#define OUT_TPW 3                    // 16-row tiles per wave
#define OUT_RB (4 * OUT_TPW * 16)    // vocabulary rows per block

struct OutArgs {
    const int8_t *W;
    const float *T, *bias;
    float *logits;
    float *part_max;
    double *part_sum;
    float *cand_val;
    int *cand_idx;
    q8_taps taps;
    int V, K, ld, ldt, n, k, ldl;
    float w_scale;
};

// One pass over W_out for all n <= 8 hypotheses.  Operand A of v_mfma_i32_16x16x64_i8 =
// 16 weight rows x 64 k (lane: row lane%16, 16 consecutive k at 16*(lane/16)), operand B =
// the quantized hidden vectors with the same k split; the result leaves rows
// 4*(lane/16)+r, r = 0..3, of hypothesis lane%16 in the lane.  Work is cut into items of
// 16 rows x 512 k; the loads of item i+1 are in flight while item i is multiplied.
template <int CH>
__global__ __launch_bounds__(256) void out_logits_kernel(OutArgs a)
{
    extern __shared__ __align__(16) int8_t smem[];
    __shared__ float s_scale[8];
    __shared__ float s_red[8 * 4];
    __shared__ float s_log[8][OUT_RB];
    const int ld = a.ld, n = a.n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int brow0 = blockIdx.x * OUT_RB;
    const int kchunks = (ld + 511) / 512;
    const int items = OUT_TPW * kchunks;

    XRegs<8, CH> xr;
    x_load<8, CH>(xr, a.T, n, a.K, a.ldt);

    auto load_item = [&](int it, v4i (&av)[8]) {
        const int tile = it / kchunks, kc = it - tile * kchunks;
        const int row = brow0 + (wave * OUT_TPW + tile) * 16 + i;
        const int8_t *wp = a.W + (size_t)row * ld + kc * 512 + 16 * g;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            av[s] = (v4i){0, 0, 0, 0};
            if (row < a.V && kc * 512 + 64 * s + 16 * g < ld) av[s] = *(const v4i *)(wp + 64 * s);
        }
    };
    v4i cur[8], nxt[8];
    load_item(0, cur);

    x_finish<8, CH>(xr, n, ld, smem, s_scale, s_red);
    if (blockIdx.x == 0) {
        if (a.taps.xq)
            for (int e = threadIdx.x; e < n * a.K; e += blockDim.x) a.taps.xq[e] = smem[(e / a.K) * ld + e % a.K];
        if (a.taps.xscale && threadIdx.x < n) a.taps.xscale[threadIdx.x] = s_scale[threadIdx.x];
    }
    const float cj = i < n ? a.w_scale * s_scale[i] : 0.0f;
    const int8_t *xb = smem + (size_t)i * ld + 16 * g;

    v4i acc = (v4i){0, 0, 0, 0};
    for (int it = 0; it < items; ++it) {
        if (it + 1 < items) load_item(it + 1, nxt);
        const int tile = it / kchunks, kc = it - tile * kchunks;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            v4i bv = (v4i){0, 0, 0, 0};
            if (i < n && kc * 512 + 64 * s + 16 * g < ld) bv = *(const v4i *)(xb + kc * 512 + 64 * s);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(cur[s], bv, acc, 0, 0, 0);
        }
        if (kc == kchunks - 1) {
            const int r0 = brow0 + (wave * OUT_TPW + tile) * 16;
            if (i < n) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = r0 + 4 * g + r;
                    float y = -INFINITY;
                    if (row < a.V) {
                        y = (float)acc[r] * cj;
                        if (a.bias) y = y + a.bias[row];
                        if (a.logits) a.logits[(size_t)i * a.ldl + row] = y;
                        if (a.taps.acc) a.taps.acc[(size_t)i * a.V + row] = acc[r];
                    }
                    s_log[i][row - brow0] = y;
                }
            }
            acc = (v4i){0, 0, 0, 0};
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) cur[s] = nxt[s];
    }
    __syncthreads();

    // per hypothesis: block maximum, sum of exp, and the k best (value, row) pairs
    for (int j = wave; j < n; j += 4) {
        float v[OUT_RB / 64];
        float m = -INFINITY;
#pragma unroll
        for (int t = 0; t < OUT_RB / 64; ++t) {
            v[t] = s_log[j][lane + 64 * t];
            m = fmaxf(m, v[t]);
        }
        m = wave_max_f(m);
        double s = 0.0;
        unsigned long long key[OUT_RB / 64];
#pragma unroll
        for (int t = 0; t < OUT_RB / 64; ++t) {
            const int row = brow0 + lane + 64 * t;
            key[t] = 0ull;
            if (row < a.V) {
                s += exp((double)v[t] - (double)m);
                key[t] = topk_key(v[t], row);
            }
        }
        s = wave_sum_d(s);
        if (lane == 0) {
            a.part_max[(size_t)blockIdx.x * n + j] = m;
            a.part_sum[(size_t)blockIdx.x * n + j] = s;
        }
        for (int r = 0; r < a.k; ++r) {
            unsigned long long best = key[0];
#pragma unroll
            for (int t = 1; t < OUT_RB / 64; ++t) best = key[t] > best ? key[t] : best;
            best = wave_max_u64(best);
            if (lane == 0) {
                const size_t o = ((size_t)blockIdx.x * n + j) * a.k + r;
                a.cand_val[o] = best ? topk_key_val(best) : -INFINITY;
                a.cand_idx[o] = best ? topk_key_idx(best) : -1;
            }
#pragma unroll
            for (int t = 0; t < OUT_RB / 64; ++t)
                if (key[t] == best) key[t] = 0ull;
        }
    }
}

struct MergeArgs {
    const float *part_max;
    const double *part_sum;
    const float *cand_val;
    const int *cand_idx;
    float *lse, *topk_logp;
    int *topk_idx;
    int nblk, n, k;
};

#define MERGE_MAX_KEYS 7168   // candidate keys held in LDS (56 KiB)

// One block per hypothesis.  All threads load the block partials and candidate lists;
// wave 0 then merges the (sorted) lists k times, only the list heads competing.
__global__ __launch_bounds__(256) void out_merge_kernel(MergeArgs a)
{
    __shared__ unsigned long long s_key[MERGE_MAX_KEYS];
    __shared__ unsigned short s_ptr[1024];
    __shared__ float s_m[4];
    __shared__ double s_s[4];
    const int j = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = a.n, k = a.k;
    const int nblk = a.nblk;
    for (int e = tid; e < nblk * k; e += 256) {
        const int b = e / k, r = e - b * k;
        const size_t o = ((size_t)b * n + j) * k + r;
        const int idx = a.cand_idx[o];
        s_key[e] = idx >= 0 ? topk_key(a.cand_val[o], idx) : 0ull;
    }
    for (int b = tid; b < nblk; b += 256) s_ptr[b] = 0;
    float pm[4];
    double ps[4];
    float m = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int b = tid + 256 * t;
        pm[t] = -INFINITY;
        ps[t] = 0.0;
        if (b < nblk) {
            pm[t] = a.part_max[(size_t)b * n + j];
            ps[t] = a.part_sum[(size_t)b * n + j];
        }
        m = fmaxf(m, pm[t]);
    }
    m = wave_max_f(m);
    if (lane == 0) s_m[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
    double S = 0.0;
#pragma unroll
    for (int t = 0; t < 4; ++t)
        if (tid + 256 * t < nblk) S += ps[t] * exp((double)pm[t] - (double)m);
    S = wave_sum_d(S);
    if (lane == 0) s_s[wave] = S;
    __syncthreads();
    if (wave != 0) return;
    S = (s_s[0] + s_s[1]) + (s_s[2] + s_s[3]);
    const float lse = (float)((double)m + log(S));
    if (lane == 0 && a.lse) a.lse[j] = lse;

    for (int r = 0; r < k; ++r) {
        unsigned long long best = 0ull;
        for (int b = lane; b < nblk; b += 64) {
            const int p = s_ptr[b];
            const unsigned long long hk = p < k ? s_key[b * k + p] : 0ull;
            best = hk > best ? hk : best;
        }
        best = wave_max_u64(best);
        const int idx = best ? topk_key_idx(best) : -1;
        if (lane == 0) {
            a.topk_idx[(size_t)j * k + r] = idx;
            a.topk_logp[(size_t)j * k + r] = best ? topk_key_val(best) - lse : -INFINITY;
        }
        if (best) {
            const int b = idx / OUT_RB;
            if ((b & 63) == lane) s_ptr[b] = s_ptr[b] + 1;
        }
    }
}

// =================================================================== host launcher ==

int q8i_out_blocks(int V) { return (V + OUT_RB - 1) / OUT_RB; }
int q8i_out_max_keys(void) { return MERGE_MAX_KEYS; }

template <int CH>
static void launch_out(q8_ctx *ctx, const OutArgs &a, int nblk, size_t smem)
{
    if (ctx->prof_ev && ctx->prof_n < ctx->prof_cap) {
        // timed dispatch: the two events take the kernel's own begin and end timestamps
        hipEvent_t e0 = ctx->prof_ev[2 * ctx->prof_n], e1 = ctx->prof_ev[2 * ctx->prof_n + 1];
        ++ctx->prof_n;
        hipExtLaunchKernelGGL(out_logits_kernel<CH>, dim3(nblk), dim3(256), smem, ctx->stream, e0, e1, 0, a);
    } else {
        hipLaunchKernelGGL(out_logits_kernel<CH>, dim3(nblk), dim3(256), smem, ctx->stream, a);
    }
}

q8_status q8i_output(q8_ctx *ctx, const q8_mat *W, const float *bias, const float *T, int ldt, int n, int k,
                     float *logits, float *lse, float *topk_logp, int32_t *topk_idx, const q8_taps *taps,
                     float *part_max, double *part_sum, float *cand_val, int *cand_idx)
{
    OutArgs a;
    a.W = W->data; a.T = T; a.bias = bias; a.logits = logits;
    a.part_max = part_max; a.part_sum = part_sum; a.cand_val = cand_val; a.cand_idx = cand_idx;
    q8_taps none = {nullptr, nullptr, nullptr};
    a.taps = taps ? *taps : none;
    a.V = W->rows; a.K = W->cols; a.ld = W->ld; a.ldt = ldt; a.n = n; a.k = k; a.ldl = W->rows;
    a.w_scale = W->scale;
    const int nblk = q8i_out_blocks(a.V);
    const size_t smem = (size_t)n * a.ld;
    const int ch = q8_fast_ch(a.ld);
    if (ch == 1) launch_out<1>(ctx, a, nblk, smem);
    else if (ch == 2) launch_out<2>(ctx, a, nblk, smem);
    else launch_out<4>(ctx, a, nblk, smem);
    MergeArgs m;
    m.part_max = part_max; m.part_sum = part_sum; m.cand_val = cand_val; m.cand_idx = cand_idx;
    m.lse = lse; m.topk_logp = topk_logp; m.topk_idx = topk_idx;
    m.nblk = nblk; m.n = n; m.k = k;
    hipLaunchKernelGGL(out_merge_kernel, dim3(n), dim3(256), 0, ctx->stream, m);
    return q8i_launch_check(ctx, "output");
}
