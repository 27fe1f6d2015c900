// q8_fp32.hip -- the 32-bit engine that the paper measures its 8-bit engine against
// (Section 4, Tables 3 and 6: "32-bit" columns): the same model with fp32 weights and no
// quantization anywhere.  Only the products differ; gates, attention, softmax, top-k and the
// search are the kernels of the 8-bit path.  A product is y = (float)(sum in double) + bias.
#include "q8_internal.h"

struct F32Job {
    const float *W;        // [rows x ld] fp32
    const float *X;        // [n x ldx]
    const float *bias;     // [rows] or NULL
    float *Y;              // [n x ldy]
    int rows, cols, ld, ldx, ldy;
};
#define F32_MAX_JOBS 3
struct F32Jobs {
    F32Job j[F32_MAX_JOBS];
    int nblk[F32_MAX_JOBS + 1];      // job t owns blocks [nblk[t], nblk[t + 1])
};

// Streaming matrix x (up to 8) vectors in fp32: the block keeps the vectors in LDS, a wave
// owns two rows at a time, each lane 16-byte pieces of them (one contiguous KiB per wave-wide
// load), products and sums in double, wave reduction, one rounding.
template <int N>
__global__ __launch_bounds__(256) void gemv_f32_kernel(F32Jobs jobs)
{
    extern __shared__ __align__(16) float s_x[];       // [N x cols4], cols4 = cols rounded up to 4
    int t = 0;
    while (t + 1 < F32_MAX_JOBS && (int)blockIdx.x >= jobs.nblk[t + 1]) ++t;
    const F32Job &J = jobs.j[t];
    const int blk = blockIdx.x - jobs.nblk[t], nblk = jobs.nblk[t + 1] - jobs.nblk[t];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cols4 = (J.cols + 3) & ~3;
    for (int e = tid; e < N * cols4; e += 256) {
        const int j = e / cols4, k = e - j * cols4;
        s_x[e] = k < J.cols ? J.X[(size_t)j * J.ldx + k] : 0.0f;
    }
    __syncthreads();
    const int nchunk = (J.cols + 255) >> 8;            // float4 pieces per lane and row
    auto load_w = [&](const float *w, int k) {
        float4 wv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k + 3 < J.cols) {
            wv = *(const float4 *)(w + k);
        } else {
            if (k < J.cols) wv.x = w[k];
            if (k + 1 < J.cols) wv.y = w[k + 1];
            if (k + 2 < J.cols) wv.z = w[k + 2];
        }
        return wv;
    };
    // two rows per pass: rows r and r + 4 nblk of this wave
    for (int row = blk * 4 + wave; row < J.rows; row += nblk * 8) {
        const int row2 = row + nblk * 4;
        const bool two = row2 < J.rows;
        const float *w0 = J.W + (size_t)row * J.ld, *w1 = J.W + (size_t)(two ? row2 : row) * J.ld;
        double acc[2][N];
#pragma unroll
        for (int j = 0; j < N; ++j) acc[0][j] = acc[1][j] = 0.0;
        for (int c = 0; c < nchunk; ++c) {
            const int k = (c * 64 + lane) * 4;
            const float4 wa = load_w(w0, k), wb = load_w(w1, k);
            if (k < cols4) {
#pragma unroll
                for (int j = 0; j < N; ++j) {
                    const float4 xv = *(const float4 *)(s_x + j * cols4 + k);
                    acc[0][j] += (double)wa.x * (double)xv.x;
                    acc[0][j] += (double)wa.y * (double)xv.y;
                    acc[0][j] += (double)wa.z * (double)xv.z;
                    acc[0][j] += (double)wa.w * (double)xv.w;
                    acc[1][j] += (double)wb.x * (double)xv.x;
                    acc[1][j] += (double)wb.y * (double)xv.y;
                    acc[1][j] += (double)wb.z * (double)xv.z;
                    acc[1][j] += (double)wb.w * (double)xv.w;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (u == 1 && !two) break;
            const int r = u ? row2 : row;
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const double tot = wave_sum_d(acc[u][j]);
                if (lane == 0) {
                    float y = (float)tot;
                    if (J.bias) y = y + J.bias[r];
                    J.Y[(size_t)j * J.ldy + r] = y;
                }
            }
        }
    }
}

// (max, sum of exp) of every 16-row tile of stored logits [n x V]: the statistics the selection
// kernel starts from (the 8-bit vocabulary kernel produces them in its epilogue).
__global__ __launch_bounds__(256) void logit_stats_kernel(const float *__restrict__ logits, int n, int V, int ntiles,
                                                          float *part_max, double *part_sum)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= n * ntiles) return;
    const int j = idx / ntiles, tile = idx - j * ntiles, r0 = tile * 16;
    const float *lg = logits + (size_t)j * V + r0;
    float v[16], m = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        v[r] = r0 + r < V ? lg[r] : -INFINITY;
        m = fmaxf(m, v[r]);
    }
    double sd = 0.0;
#pragma unroll
    for (int r = 0; r < 16; ++r)
        if (v[r] > -INFINITY) sd += (double)exp_le0(v[r] - m);
    part_max[idx] = m;
    part_sum[idx] = sd;
}

template <int N>
static void launch_f32(q8_ctx *ctx, const F32Jobs &jobs, int blocks, size_t smem)
{
    Q8_LAUNCH(ctx, Q8_KERNEL_GEMV, gemv_f32_kernel<N>, dim3(blocks), dim3(256), smem, jobs);
}

q8_status q8i_gemv_f32(q8_ctx *ctx, const q8i_f32_job *d, int njobs, int n)
{
    F32Jobs jobs;
    int blocks = 0, max_cols4 = 0;
    for (int t = 0; t < F32_MAX_JOBS; ++t) {
        const q8i_f32_job &q = d[t < njobs ? t : 0];
        jobs.j[t] = {q.W->data, q.X, q.bias, q.Y, q.W->rows, q.W->cols, q.W->ld, q.ldx, q.ldy};
        jobs.nblk[t] = blocks;
        if (t < njobs) {
            int b = (q.W->rows + 3) / 4;
            if (b > 1024) b = 1024;
            blocks += b;
            const int c4 = (q.W->cols + 3) & ~3;
            if (c4 > max_cols4) max_cols4 = c4;
        }
    }
    jobs.nblk[F32_MAX_JOBS] = blocks;
    for (int t = njobs; t < F32_MAX_JOBS; ++t) jobs.nblk[t] = blocks;
    const size_t smem = (size_t)n * max_cols4 * sizeof(float);
    switch (n) {
    case 1: launch_f32<1>(ctx, jobs, blocks, smem); break;
    case 2: launch_f32<2>(ctx, jobs, blocks, smem); break;
    case 3: launch_f32<3>(ctx, jobs, blocks, smem); break;
    case 4: launch_f32<4>(ctx, jobs, blocks, smem); break;
    case 5: launch_f32<5>(ctx, jobs, blocks, smem); break;
    case 6: launch_f32<6>(ctx, jobs, blocks, smem); break;
    case 7: launch_f32<7>(ctx, jobs, blocks, smem); break;
    default: launch_f32<8>(ctx, jobs, blocks, smem); break;
    }
    return q8i_launch_check(ctx, "gemv_f32");
}

q8_status q8i_logit_stats(q8_ctx *ctx, const float *logits, int n, int V, float *part_max, double *part_sum)
{
    const int ntiles = q8i_out_tiles(V), total = n * ntiles;
    hipLaunchKernelGGL(logit_stats_kernel, dim3((total + 255) / 256), dim3(256), 0, ctx->stream, logits, n, V, ntiles,
                       part_max, part_sum);
    return q8i_launch_check(ctx, "logit stats");
}
