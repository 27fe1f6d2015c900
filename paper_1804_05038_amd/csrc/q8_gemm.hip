// q8_gemm.hip -- the 8-bit product of Section 3 for panels of more than 8 vectors (source
// positions of one sentence, or the hypotheses of many sentences decoded together, which
// Section 6 names as the next step): a blocked int8 GEMM on the gfx950 matrix cores.
// The arithmetic is that of the streaming kernels: per-vector activation codes, exact
// int32 sums, one fp32 scale product, separate bias addition.
#include "q8_internal.h"

struct GemmArgs {
    const int8_t *W;       // [rows x ld] int8
    const int8_t *xq;      // [n x ld] int8 codes of the n vectors
    const float *xscale;   // [n]
    const float *bias;     // [rows] or NULL
    float *Y;              // [n x ldy]
    int32_t *tap_acc;      // [n x rows] or NULL
    float *part_max;       // STATS: [n x ntiles] maximum of each 16-row tile
    double *part_sum;      // STATS: [n x ntiles] sum of exp(y - maximum)
    int rows, ld, n, ldy, ntiles;
    float w_scale;
};
#define GEMM_MAX_JOBS 3
struct GemmJobs {          // products of one launch (blockIdx.z), all over the same number of vectors
    GemmArgs j[GEMM_MAX_JOBS];
};

#define GB_K 128           // k bytes per stage
#define GB_PITCH 144       // LDS bytes per staged vector: 16 lanes x 16 bytes fall on 64 distinct banks

// Block tile: 64 RT rows x 16 NT vectors, four waves, wave w owns row tiles w RT .. w RT + RT - 1.
// The vectors' codes go through LDS (every wave multiplies the same ones), double-buffered,
// one barrier per stage; each wave reads its own weight rows straight from memory, one stage
// ahead.  v_mfma_i32_16x16x64_i8 operands: A = 16 weight rows x 64 k (lane: row lane % 16,
// k bytes 16 (lane / 16) .. + 15), B = the same split for 16 vectors; result: lane holds rows
// 4 (lane / 16) + r, r = 0..3, of vector lane % 16.
template <int RT, int NT, bool STATS>
__global__ __launch_bounds__(256) void gemm_block_kernel(GemmJobs jobs)
{
    const GemmArgs &a = jobs.j[blockIdx.z];
    constexpr int BN = 16 * NT;
    if ((int)blockIdx.x * 64 * RT >= a.rows) return;     // the grid is sized for the largest job
    constexpr int PIECES = BN * (GB_K / 16) / 256;      // 16-byte pieces of a stage per thread
    __shared__ __align__(16) int8_t s_b[2][BN * GB_PITCH];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int r0 = (blockIdx.x * 4 + wave) * 16 * RT;
    const int c0 = blockIdx.y * BN;
    const int ld = a.ld, n = a.n, rows = a.rows;

    const int8_t *wp[RT];
    bool row_ok[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int row = r0 + 16 * rt + i;
        row_ok[rt] = row < rows;
        wp[rt] = a.W + (size_t)(row_ok[rt] ? row : 0) * ld + 16 * g;
    }
    v4i breg[PIECES], anext[RT][2], acur[RT][2];
    auto load_stage = [&](int k0) {
#pragma unroll
        for (int u = 0; u < PIECES; ++u) {
            const int p = u * 256 + tid;
            const int col = c0 + (p >> 3), k = k0 + (p & 7) * 16;
            breg[u] = (v4i){0, 0, 0, 0};
            if (col < n && k < ld) breg[u] = *(const v4i *)(a.xq + (size_t)col * ld + k);
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int kc = 0; kc < 2; ++kc) {
                anext[rt][kc] = (v4i){0, 0, 0, 0};
                if (row_ok[rt] && k0 + 64 * kc + 16 * g < ld) anext[rt][kc] = *(const v4i *)(wp[rt] + k0 + 64 * kc);
            }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int u = 0; u < PIECES; ++u) {
            const int p = u * 256 + tid;
            *(v4i *)(s_b[buf] + (p >> 3) * GB_PITCH + (p & 7) * 16) = breg[u];
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int kc = 0; kc < 2; ++kc) acur[rt][kc] = anext[rt][kc];
    };

    v4i acc[RT][NT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[rt][t] = (v4i){0, 0, 0, 0};

    load_stage(0);
    store_stage(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = 0; k0 < ld; k0 += GB_K, buf ^= 1) {
        const bool more = k0 + GB_K < ld;
        if (more) load_stage(k0 + GB_K);
        const int8_t *bp = s_b[buf] + i * GB_PITCH + 16 * g;
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (c0 + 16 * t >= n) continue;          // block-uniform: vectors past n
                const v4i bv = *(const v4i *)(bp + t * 16 * GB_PITCH + 64 * kc);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    acc[rt][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(acur[rt][kc], bv, acc[rt][t], 0, 0, 0);
            }
        if (more) store_stage(buf ^ 1);   // the other buffer was last read before the previous barrier
        __syncthreads();
    }

    const bool vec_ok = ((a.ldy & 3) == 0) && (((uintptr_t)a.Y & 15) == 0);
    const bool bias_vec = (((uintptr_t)a.bias) & 15) == 0;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int row0 = r0 + 16 * rt + 4 * g;
        if (r0 + 16 * rt >= rows) continue;              // wave-uniform
        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a.bias) {
            if (bias_vec && row0 + 3 < rows) {
                b = *(const float4 *)(a.bias + row0);
            } else {
                if (row0 < rows) b.x = a.bias[row0];
                if (row0 + 1 < rows) b.y = a.bias[row0 + 1];
                if (row0 + 2 < rows) b.z = a.bias[row0 + 2];
                if (row0 + 3 < rows) b.w = a.bias[row0 + 3];
            }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (c0 + 16 * t >= n) continue;
            const int col = c0 + 16 * t + i;
            const bool col_ok = col < n;
            const float c = col_ok ? a.w_scale * a.xscale[col] : 0.0f;
            float y[4];
            float m = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                y[r] = -INFINITY;
                if (col_ok && row0 + r < rows) {
                    y[r] = (float)acc[rt][t][r] * c;
                    if (a.bias) y[r] = y[r] + (r == 0 ? b.x : r == 1 ? b.y : r == 2 ? b.z : b.w);
                    if (a.tap_acc) a.tap_acc[(size_t)col * rows + row0 + r] = acc[rt][t][r];
                }
                m = fmaxf(m, y[r]);
            }
            if (col_ok) {
                if (vec_ok && row0 + 3 < rows) {
                    *(float4 *)(a.Y + (size_t)col * a.ldy + row0) = make_float4(y[0], y[1], y[2], y[3]);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (row0 + r < rows) a.Y[(size_t)col * a.ldy + row0 + r] = y[r];
                }
            }
            if (STATS) {
                // (max, sum of exp) of the tile's 16 rows per vector: lanes i, i+16, i+32, i+48
                m = fmaxf(m, __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(m), SWZ_XOR16)));
                m = fmaxf(m, __shfl_xor(m, 32, 64));
                double sd = 0.0;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (y[r] > -INFINITY) sd += (double)__expf(y[r] - m);
                sd += __shfl_xor(sd, 16, 64);
                sd += __shfl_xor(sd, 32, 64);
                if (col_ok && g == 0) {
                    const int tile = (r0 + 16 * rt) >> 4;
                    a.part_max[(size_t)col * a.ntiles + tile] = m;
                    a.part_sum[(size_t)col * a.ntiles + tile] = sd;
                }
            }
        }
    }
}

// Block (j, job): max-abs quantization of vector j's K floats into ld code bytes (pad bytes
// zero), Section 3's "8-bit approximation" of an activation.
struct QuantJob {
    const float *X;
    int K, ldx, ld;
    int8_t *xq;            // [n x ld]
    float *xscale;         // [n]
    int8_t *tap_xq;        // [n x K] or NULL
    float *tap_scale;      // [n] or NULL
};
struct QuantJobs {
    QuantJob j[GEMM_MAX_JOBS];
};

__global__ __launch_bounds__(256) void quantize_rows_kernel(QuantJobs jobs)
{
    __shared__ float s_scale[1];
    __shared__ float s_red[4];
    const QuantJob &J = jobs.j[blockIdx.y];
    const int j = blockIdx.x;
    block_quantize<1>(J.X + (size_t)j * J.ldx, 1, J.K, J.ldx, J.ld, J.xq + (size_t)j * J.ld, s_scale, s_red);
    if (threadIdx.x == 0) {
        J.xscale[j] = s_scale[0];
        if (J.tap_scale) J.tap_scale[j] = s_scale[0];
    }
    if (J.tap_xq) {
        __syncthreads();
        for (int k = threadIdx.x; k < J.K; k += blockDim.x) J.tap_xq[(size_t)j * J.K + k] = J.xq[(size_t)j * J.ld + k];
    }
}

q8_status q8i_quantize_jobs(q8_ctx *ctx, const q8i_quant_job *d, int njobs, int n)
{
    QuantJobs jobs;
    for (int t = 0; t < GEMM_MAX_JOBS; ++t) {
        const q8i_quant_job &q = d[t < njobs ? t : 0];
        jobs.j[t] = {q.X, q.K, q.ldx, q.ld, q.xq, q.xscale, q.taps ? q.taps->xq : nullptr, q.taps ? q.taps->xscale : nullptr};
    }
    hipLaunchKernelGGL(quantize_rows_kernel, dim3(n, njobs), dim3(256), 0, ctx->stream, jobs);
    return q8i_launch_check(ctx, "quantize rows");
}

// Y = dequantize(W . codes) + bias for n already-quantized vectors, up to three products in
// one launch.  part_max / part_sum non-NULL (first job only is looked at): also the per-tile
// softmax statistics of the vocabulary layer.
q8_status q8i_gemm_jobs(q8_ctx *ctx, const q8i_gemm_job *d, int njobs, int n)
{
    GemmJobs jobs;
    int max_rows = 0;
    for (int t = 0; t < GEMM_MAX_JOBS; ++t) {
        const q8i_gemm_job &q = d[t < njobs ? t : 0];
        GemmArgs &a = jobs.j[t];
        a.W = q.W->data; a.xq = q.xq; a.xscale = q.xscale; a.bias = q.bias; a.Y = q.Y; a.tap_acc = q.tap_acc;
        a.part_max = q.part_max; a.part_sum = q.part_sum;
        a.rows = q.W->rows; a.ld = q.W->ld; a.n = n; a.ldy = q.ldy; a.ntiles = (q.W->rows + 15) / 16;
        a.w_scale = q.W->scale;
        if (a.rows > max_rows) max_rows = a.rows;
    }
    const bool stats = d[0].part_max != nullptr;
    if (max_rows > 8192) {
        const dim3 grid((max_rows + 127) / 128, (n + 127) / 128, njobs);
        if (stats) Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, (gemm_block_kernel<2, 8, true>), grid, dim3(256), 0, jobs);
        else Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, (gemm_block_kernel<2, 8, false>), grid, dim3(256), 0, jobs);
    } else {
        const dim3 grid((max_rows + 63) / 64, (n + 63) / 64, njobs);
        if (stats) Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, (gemm_block_kernel<1, 4, true>), grid, dim3(256), 0, jobs);
        else Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, (gemm_block_kernel<1, 4, false>), grid, dim3(256), 0, jobs);
    }
    return q8i_launch_check(ctx, "gemm");
}

q8_status q8i_gemm_mfma(q8_ctx *ctx, const q8_mat *W, const float *X, int n, int ldx, const float *bias, float *Y,
                        int ldy, const q8_taps *taps, int8_t *xq, float *xscale)
{
    q8i_quant_job qj = {X, W->cols, ldx, W->ld, xq, xscale, taps};
    q8_status st = q8i_quantize_jobs(ctx, &qj, 1, n);
    if (st) return st;
    q8i_gemm_job gj = {W, xq, xscale, bias, Y, ldy, taps ? taps->acc : nullptr, nullptr, nullptr};
    return q8i_gemm_jobs(ctx, &gj, 1, n);
}
