// q8_products.hip -- Section 3 of "Pieces of Eight: 8-bit Neural Machine Translation" as
// gfx950 kernels: weight quantization, the streaming int8 matrix x vector / narrow-matrix
// product (16-byte loads, 4-way int8 dots, DPP reductions), and the narrow product on the
// int8 matrix cores for more than 8 vectors.
#include "q8_internal.h"
#include "q8_gemv_fast.h"

// =============================================================== weight quantization ==

// max |W| over a [rows x cols] matrix into *out_bits (bit pattern of a non-negative
// float, combined with an unsigned atomic max; *out_bits must start at 0).
__global__ __launch_bounds__(256) void absmax_kernel(const float *__restrict__ W, int rows, int cols, int ld,
                                                     unsigned *out_bits)
{
    __shared__ float s_red[4];
    float m = 0.0f;
    const size_t total = (size_t)rows * cols;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const size_t r = e / cols, c = e - r * cols;
        m = fmaxf(m, fabsf(W[r * ld + c]));
    }
    m = wave_max_f(m);
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
        atomicMax(out_bits, __float_as_uint(m));
    }
}

__global__ __launch_bounds__(256) void quantize_matrix_kernel(const float *__restrict__ W, int rows, int cols, int ld_in,
                                                              int8_t *__restrict__ Wq, int ld_out,
                                                              const unsigned *max_bits, float *scale_out)
{
    float scale, inv;
    q8_scale_of(__uint_as_float(*max_bits), scale, inv);
    if (blockIdx.x == 0 && threadIdx.x == 0) *scale_out = scale;
    const int groups = ld_out / 4;
    const size_t total = (size_t)rows * groups;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
        const size_t r = e / groups;
        const int k = (int)(e - r * groups) * 4;
        const float *w = W + r * ld_in;
        float a = k < cols ? w[k] : 0.0f, b = k + 1 < cols ? w[k + 1] : 0.0f;
        float c = k + 2 < cols ? w[k + 2] : 0.0f, d = k + 3 < cols ? w[k + 3] : 0.0f;
        *(int *)(Wq + r * ld_out + k) = q8_pack4(a, b, c, d, inv);
    }
}

// One scale per row: a wave per row finds the row's maximum and writes its codes.
__global__ __launch_bounds__(256) void quantize_matrix_rows_kernel(const float *__restrict__ W, int rows, int cols, int ld_in,
                                                                   int8_t *__restrict__ Wq, int ld_out, float *__restrict__ row_scale)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;                               // wave-uniform
    const float *w = W + (size_t)r * ld_in;
    float m = 0.0f;
    for (int k = lane; k < cols; k += 64) m = fmaxf(m, fabsf(w[k]));
    m = wave_max_f(m);
    float scale, inv;
    q8_scale_of(m, scale, inv);
    if (lane == 0) row_scale[r] = scale;
    for (int k = 4 * lane; k < ld_out; k += 256) {
        float a = k < cols ? w[k] : 0.0f, b = k + 1 < cols ? w[k + 1] : 0.0f;
        float c = k + 2 < cols ? w[k + 2] : 0.0f, d = k + 3 < cols ? w[k + 3] : 0.0f;
        *(int *)(Wq + (size_t)r * ld_out + k) = q8_pack4(a, b, c, d, inv);
    }
}

__global__ void fill_u32_kernel(unsigned *p, int n, unsigned v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ====================================================== streaming matrix x vector(s) ==

// General shapes.  Up to Q8_MAX_JOBS independent products in one launch, each with
// N <= 8 vectors.  A block belongs to one job, quantizes that job's vectors into LDS
// and streams its slice of rows.
template <int N>
__global__ __launch_bounds__(256) void gemv_jobs_kernel(GemvJobs jobs)
{
    extern __shared__ __align__(16) int8_t smem[];
    __shared__ float s_scale[8];
    __shared__ float s_red[8 * 4];
    const GemvJob &J = jobs.j[pick_job(jobs, blockIdx.x)];
    const int blk = blockIdx.x - J.block0;
    const int ld = J.ld;

    block_quantize<N>(J.X, N, J.cols, J.ldx, ld, smem, s_scale, s_red);
    if (blk == 0) write_x_taps<N>(J, smem, s_scale);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lpr = J.lpr, lir = lane & (lpr - 1), sg = lane / lpr, rpp = 64 / lpr;
    constexpr int U = 4;
    const int r_begin = blk * J.rpb;
    const int r_end = min(J.rows, r_begin + J.rpb);
    float cj = 0.0f, sxj = 0.0f;              // lane lir < N owns vector lir in the epilogue
    if (lir < N) { sxj = s_scale[lir]; cj = J.w_scale * sxj; }

    for (int r = r_begin + wave * rpp * U; r < r_end; r += 4 * rpp * U) {
        const int8_t *wrow[U];
        int row[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            row[u] = r + u * rpp + sg;
            wrow[u] = row[u] < r_end ? J.W + (size_t)row[u] * ld : nullptr;
        }
        int acc[U][N];
        wave_dot<N, U>(wrow, ld, lpr, lir, smem, acc);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int a = 0;
#pragma unroll
            for (int j = 0; j < N; ++j) a = (lir == j) ? acc[u][j] : a;
            if (lir < N && row[u] < r_end) {
                float y = (float)a * (J.row_scale ? J.row_scale[row[u]] * sxj : cj);
                if (J.bias) y = y + J.bias[row[u]];
                J.Y[(size_t)lir * J.ldy + row[u]] = y;
                if (J.tap_acc) J.tap_acc[(size_t)lir * J.rows + row[u]] = a;
            }
        }
    }
}

template <int N, int CH, bool ROWS, int U, bool STREAM>
__global__ __launch_bounds__(256) void gemv_fast_kernel(GemvJobs jobs)
{
    extern __shared__ __align__(16) int8_t smem[];
    gemv_fast_body<N, CH, ROWS, U, STREAM>(jobs, blockIdx.x, smem);
}

// ================================================== one pass over a large matrix ==
// Rows of 256, 512 or 1024 bytes (LPR = 16, 32, 64 lanes per row), a matrix of several MB, one
// product (one weight scale per matrix or per row), no taps: nothing loops.  A wave takes 8 KB of consecutive rows (8 wave-wide loads of
// one contiguous KiB each, 64 / LPR rows per load), so the whole matrix is requested in the
// kernel's first microsecond, as in the vocabulary kernel; the lane's 16 code bytes of every
// vector stay in registers; the 8 N partial sums per lane are totalled over the LPR lanes of a
// row by the transposed reduction restricted to its first log2(LPR) stages, staged in LDS and
// finished (scale, bias, store) by consecutive lanes for consecutive rows.
#define GEMV1_LOADS 8
template <int N, int LPR>
__global__ __launch_bounds__(256) void gemv_onepass_kernel(GemvJobs jobs)
{
    extern __shared__ __align__(16) int8_t smem[];
    __shared__ float s_scale[8];
    __shared__ float s_red[8 * 4];
    constexpr int RPL = 64 / LPR, RW = GEMV1_LOADS * RPL;          // rows per load, rows per wave
    constexpr int CNT = GEMV1_LOADS * N, M = t_pow2(CNT), LG = t_log2(LPR);
    constexpr int KEEP = M > LPR ? M / LPR : 1;                    // totals a lane is left with
    __shared__ int s_t[4][RW * N];
    const GemvJob &J = jobs.j[0];
    const int ld = J.ld, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r0 = ((int)blockIdx.x * 4 + wave) * RW;

    XRegs<N, 1> xr;
    x_load<N, 1>(xr, J.X, N, J.cols, J.ldx);
    const __amdgpu_buffer_rsrc_t rw = q8_rsrc(J.W, (size_t)J.rows * ld);
    v4i w[GEMV1_LOADS];
    {
        const size_t base = (size_t)r0 * ld + (size_t)lane * 16;   // below 2^31 (checked by the launcher)
#pragma unroll
        for (int l = 0; l < GEMV1_LOADS; ++l) {
            const size_t off = base + (size_t)l * 1024;
            w[l] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rw, (int)(r0 < J.rows ? (unsigned)off : Q8_OOB), 0, 0));
        }
    }
    // the bias of row r0 + lane % RW: the row this lane finishes in every pass of the epilogue
    const __amdgpu_buffer_rsrc_t rb = q8_rsrc(J.bias, J.bias ? (size_t)J.rows * sizeof(float) : 0);
    const int my_row = r0 + (lane & (RW - 1));
    const float bias = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, (int)(my_row < J.rows ? (unsigned)my_row * 4u : Q8_OOB), 0, 0));
    // ... and its weight scale where there is one per row (an absent array reads as zero and is not used)
    const __amdgpu_buffer_rsrc_t rs = q8_rsrc(J.row_scale, J.row_scale ? (size_t)J.rows * sizeof(float) : 0);
    const float row_scale = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(my_row < J.rows ? (unsigned)my_row * 4u : Q8_OOB), 0, 0));
    x_finish<N, 1>(xr, N, ld, smem, s_scale, s_red);

    const int lir = lane & (LPR - 1), g = lane / LPR;
    int v[M];
#pragma unroll
    for (int e = 0; e < M; ++e) v[e] = 0;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const v4i x = *(const v4i *)(smem + (size_t)j * ld + lir * 16);
#pragma unroll
        for (int l = 0; l < GEMV1_LOADS; ++l) v[l * N + j] = dot16(w[l], x, 0);
    }
    // totals over the LPR lanes of a row group: the stages that pair lanes within 16, 32 or 64
    t_stage<0, M, TSumI>(v, lane);
    t_stage<1, M, TSumI>(v, lane);
    t_stage<2, M, TSumI>(v, lane);
    t_stage<3, M, TSumI>(v, lane);
    if constexpr (LG > 4) t_stage<4, M, TSumI>(v, lane);
    if constexpr (LG > 5) t_stage<5, M, TSumI>(v, lane);
    // the lane now holds values first .. first + KEEP - 1; lanes that differ only in bits no splitting stage used hold copies
    int first = 0, used = 0;
#pragma unroll
    for (int st = 0; st < (t_log2(M) < LG ? t_log2(M) : LG); ++st) {
        first |= ((lane >> t_bit(st)) & 1) * (M >> (st + 1));
        used |= 1 << t_bit(st);
    }
    const bool owner = (lir & ~used) == 0;
#pragma unroll
    for (int i = 0; i < KEEP; ++i) {
        const int e = first + i;                                   // e = l * N + j
        if (owner && e < CNT) {
            const int l = e / N, j = e - l * N;
            s_t[wave][(l * RPL + g) * N + j] = v[i];
        }
    }
    __builtin_amdgcn_wave_barrier();
    const bool has_bias = J.bias != nullptr, has_rows = J.row_scale != nullptr;
#pragma unroll
    for (int o0 = 0; o0 < RW * N; o0 += 64) {
        const int o = o0 + lane, j = o / RW, rr = o & (RW - 1);     // consecutive lanes, consecutive rows (rr = lane % RW)
        if (o < RW * N && r0 + rr < J.rows) {
            const int a = s_t[wave][rr * N + j];
            float y = (float)a * ((has_rows ? row_scale : J.w_scale) * s_scale[j]);
            if (has_bias) y = y + bias;
            J.Y[(size_t)j * J.ldy + r0 + rr] = y;
        }
    }
}

// ================================================ narrow product on the matrix cores ==

// ==================================================================== read probe ==
// Measurement aid: a plain read stream over `chunks` 16-byte pieces, every wave-wide
// load one contiguous KiB, eight loads in flight per lane, nothing computed but an xor.
// Its duration for a buffer of a kernel's size is the ceiling that kernel is priced
// against for the memory level the buffer sits in.
#define PROBE_BLOCKS 2048
__global__ __launch_bounds__(256) void read_probe_kernel(const int4 *buf, size_t chunks, unsigned *sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    int4 acc = {0, 0, 0, 0};
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < chunks; i += 8 * stride) {
        int4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = buf[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    }
    for (; i < chunks; i += stride) {
        const int4 v = buf[i];
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    const unsigned r = (unsigned)(acc.x ^ acc.y ^ acc.z ^ acc.w);
    if (r == 0x9e3779b9u) sink[blockIdx.x] = r;    // keeps the loads alive; practically never taken
}

// ============================================================ device math, evaluated ==
// Verification aid: the device's own sigmoid / tanh (float in, float out) and exp (double in, double
// out) on an array, so that the functions the kernels call can be compared with a reference value by
// value on the device they run on; and the wave-wide sort of the selection's threshold on groups of 64.
__global__ __launch_bounds__(256) void math_eval_kernel(int fn, const void *x, void *y, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    if (fn == 3) {                                   // (n is a multiple of 256: every wave is complete)
        ((float *)y)[i] = wave_sort_desc_f(((const float *)x)[i], threadIdx.x & 63);
        return;
    }
    if (fn == 0) ((float *)y)[i] = q8_tanh_rn(((const float *)x)[i]);
    else if (fn == 1) ((float *)y)[i] = q8_sigmoid_rn(((const float *)x)[i]);
    else ((double *)y)[i] = q8_exp_d(((const double *)x)[i]);
}

q8_status q8i_math_eval(q8_ctx *ctx, int fn, const void *x, void *y, size_t n)
{
    hipLaunchKernelGGL(math_eval_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, fn, x, y, n);
    return q8i_launch_check(ctx, "math eval");
}

// =================================================================== host launchers ==

q8_status q8i_probe_read(q8_ctx *ctx, const void *buf, size_t bytes)
{
    const size_t chunks = bytes / 16;
    size_t blocks = (chunks + 255) / 256;
    if (blocks > PROBE_BLOCKS) blocks = PROBE_BLOCKS;
    unsigned *sink = (unsigned *)(ctx->ws + Q8_WS_HEADER);          // PROBE_BLOCKS words of scratch
    Q8_LAUNCH(ctx, Q8_KERNEL_PROBE, read_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, (const int4 *)buf, chunks, sink);
    return q8i_launch_check(ctx, "read probe");
}


q8_status q8i_launch_check(q8_ctx *ctx, const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return q8_fail(ctx, Q8_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
    return Q8_OK;
}

q8_status q8i_quantize_matrix(q8_ctx *ctx, const float *W, int rows, int cols, int ld_in, int8_t *Wq, int ld_out,
                              float *scale_host)
{
    unsigned *slot = (unsigned *)(ctx->ws + Q8_WS_SCRATCH_SLOT);
    float *scale_dev = (float *)(slot + 1);
    const size_t total = (size_t)rows * cols;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(absmax_kernel, dim3(blocks), dim3(256), 0, ctx->stream, W, rows, cols, ld_in, slot);
    hipLaunchKernelGGL(quantize_matrix_kernel, dim3(blocks), dim3(256), 0, ctx->stream, W, rows, cols, ld_in, Wq,
                       ld_out, slot, scale_dev);
    q8_status st = q8i_launch_check(ctx, "q8_quantize_matrix");
    if (st) return st;
    hipError_t e = hipMemcpyAsync(scale_host, scale_dev, sizeof(float), hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, ctx->stream, slot, 2, 0u);
        e = hipStreamSynchronize(ctx->stream);
    }
    if (e != hipSuccess) return q8_fail(ctx, Q8_ERR_DEVICE, "q8_quantize_matrix: %s", hipGetErrorString(e));
    return Q8_OK;
}

q8_status q8i_quantize_matrix_rows(q8_ctx *ctx, const float *W, int rows, int cols, int ld_in, int8_t *Wq, int ld_out,
                                   float *row_scale)
{
    hipLaunchKernelGGL(quantize_matrix_rows_kernel, dim3((rows + 3) / 4), dim3(256), 0, ctx->stream, W, rows, cols, ld_in,
                       Wq, ld_out, row_scale);
    return q8i_launch_check(ctx, "q8_quantize_matrix_rows");
}

q8_status q8i_fill_u32(q8_ctx *ctx, void *p, int n, unsigned v)
{
    hipLaunchKernelGGL(fill_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, ctx->stream, (unsigned *)p, n, v);
    return q8i_launch_check(ctx, "fill");
}

template <int N>
static void launch_gemv_onepass_n(q8_ctx *ctx, const GemvJobs &jobs, size_t smem)
{
    const int ld = jobs.j[0].ld, rw = GEMV1_LOADS * 1024 / ld;                 // rows per wave
    const int blocks = (jobs.j[0].rows + 4 * rw - 1) / (4 * rw);
    if (ld == 256) Q8_LAUNCH(ctx, Q8_KERNEL_GEMV, (gemv_onepass_kernel<N, 16>), dim3(blocks), dim3(256), smem, jobs);
    else if (ld == 512) Q8_LAUNCH(ctx, Q8_KERNEL_GEMV, (gemv_onepass_kernel<N, 32>), dim3(blocks), dim3(256), smem, jobs);
    else Q8_LAUNCH(ctx, Q8_KERNEL_GEMV, (gemv_onepass_kernel<N, 64>), dim3(blocks), dim3(256), smem, jobs);
}

static bool launch_gemv_onepass(q8_ctx *ctx, const GemvJobs &jobs, int n, size_t smem)
{
    switch (n) {
    case 1: launch_gemv_onepass_n<1>(ctx, jobs, smem); break;
    case 2: launch_gemv_onepass_n<2>(ctx, jobs, smem); break;
    case 3: launch_gemv_onepass_n<3>(ctx, jobs, smem); break;
    case 4: launch_gemv_onepass_n<4>(ctx, jobs, smem); break;
    case 5: launch_gemv_onepass_n<5>(ctx, jobs, smem); break;
    case 6: launch_gemv_onepass_n<6>(ctx, jobs, smem); break;
    case 7: launch_gemv_onepass_n<7>(ctx, jobs, smem); break;
    case 8: launch_gemv_onepass_n<8>(ctx, jobs, smem); break;
    default: return false;
    }
    return true;
}

template <int N, bool ROWS, int U, bool STREAM>
static void launch_gemv_nu(q8_ctx *ctx, const GemvJobs &jobs, int blocks, size_t smem, int ch)
{
    if (ch == 1) Q8_LAUNCH(ctx, Q8_KERNEL_GEMV, (gemv_fast_kernel<N, 1, ROWS, U, STREAM>), dim3(blocks), dim3(256), smem, jobs);
    else if (ch == 2) Q8_LAUNCH(ctx, Q8_KERNEL_GEMV, (gemv_fast_kernel<N, 2, ROWS, U, STREAM>), dim3(blocks), dim3(256), smem, jobs);
    else Q8_LAUNCH(ctx, Q8_KERNEL_GEMV, (gemv_fast_kernel<N, 4, ROWS, U, STREAM>), dim3(blocks), dim3(256), smem, jobs);
}

template <int N>
static void launch_gemv_n(q8_ctx *ctx, const GemvJobs &jobs, int blocks, size_t smem, int ch, bool rows, bool stream)
{
    if (ch == 0) Q8_LAUNCH(ctx, Q8_KERNEL_GEMV, gemv_jobs_kernel<N>, dim3(blocks), dim3(256), smem, jobs);
    else if (rows) launch_gemv_nu<N, true, 2, false>(ctx, jobs, blocks, smem, ch);
    else if (stream) launch_gemv_nu<N, false, 2, true>(ctx, jobs, blocks, smem, ch);
    else launch_gemv_nu<N, false, 2, false>(ctx, jobs, blocks, smem, ch);
}

bool q8i_gemv_fast_setup(const q8i_gemv_desc *d, int n, GemvJobs *jobs, int *blocks, size_t *smem)
{
    if (d->row_scale || d->taps || d->W->cols % 4 != 0 || (size_t)d->W->rows * d->W->ld >= (1u << 31) || q8_fast_ch(d->W->ld) != 1)
        return false;
    memset(jobs, 0, sizeof(*jobs));
    jobs->njobs = 1;
    GemvJob &J = jobs->j[0];
    J.W = d->W->data; J.X = d->X; J.bias = d->bias; J.Y = d->Y;
    J.rows = d->W->rows; J.cols = d->W->cols; J.ld = d->W->ld;
    J.ldx = d->ldx; J.ldy = d->ldy; J.w_scale = d->W->scale;
    J.lpr = q8_lanes_per_row(J.ld);
    const int pass = 4 * 2;                       // rows per block and pass of the fast kernel (four waves, two rows each)
    int rpb = (J.rows + 2047) / 2048;
    rpb = (rpb + pass - 1) / pass * pass;
    J.rpb = rpb;
    J.block0 = 0;
    *blocks = (J.rows + rpb - 1) / rpb;
    *smem = (size_t)n * J.ld;
    return true;
}

q8_status q8i_gemv_jobs(q8_ctx *ctx, const q8i_gemv_desc *d, int njobs, int n)
{
    GemvJobs jobs;
    jobs.njobs = njobs;
    int max_ld = 0, with_rows = 0;
    bool fast = true;
    for (int t = 0; t < njobs; ++t) {
        GemvJob &J = jobs.j[t];
        with_rows += d[t].row_scale != nullptr;
        J.W = d[t].W->data; J.X = d[t].X; J.bias = d[t].bias; J.Y = d[t].Y;
        J.tap_xq = d[t].taps ? d[t].taps->xq : nullptr;
        J.tap_xscale = d[t].taps ? d[t].taps->xscale : nullptr;
        J.tap_acc = d[t].taps ? d[t].taps->acc : nullptr;
        J.rows = d[t].W->rows; J.cols = d[t].W->cols; J.ld = d[t].W->ld;
        J.ldx = d[t].ldx; J.ldy = d[t].ldy; J.w_scale = d[t].W->scale; J.row_scale = d[t].row_scale;
        if (J.ld > max_ld) max_ld = J.ld;
        if (J.cols % 4 != 0) fast = false;
        if ((size_t)J.rows * J.ld >= (1u << 31)) fast = false;       // the fast kernel addresses the matrix with 32-bit offsets
    }
    if (with_rows != 0 && with_rows != njobs) fast = false;         // mixed launches run on the general kernel
    const bool rows = with_rows != 0;
    const int ch = fast ? q8_fast_ch(max_ld) : 0;
    size_t all_bytes = 0;
    for (int t = 0; t < njobs; ++t) all_bytes += (size_t)jobs.j[t].rows * jobs.j[t].ld;
    const int u = 2;                              // rows per wave and pass of the fast kernel
    int blocks = 0;
    for (int t = 0; t < njobs; ++t) {
        GemvJob &J = jobs.j[t];
        J.lpr = q8_lanes_per_row(J.ld);
        // rows covered by one block iteration; large matrices spread over at most ~2048 blocks
        const int pass = ch ? 4 * u : 4 * (64 / J.lpr) * 4;
        int rpb = (J.rows + 2047) / 2048;
        rpb = (rpb + pass - 1) / pass * pass;
        J.rpb = rpb;
        J.block0 = blocks;
        blocks += (J.rows + rpb - 1) / rpb;
    }
    const size_t smem = (size_t)n * max_ld;
    // one product over a matrix of several MB with rows of 256, 512 or 1024 bytes: the kernel without a loop
    if (fast && njobs == 1 && !jobs.j[0].tap_xq && !jobs.j[0].tap_xscale && !jobs.j[0].tap_acc && all_bytes >= ((size_t)8 << 20) &&
        (max_ld == 256 || max_ld == 512 || max_ld == 1024) && launch_gemv_onepass(ctx, jobs, n, smem))
        return q8i_launch_check(ctx, "gemv");
    size_t bytes = 0;
    for (int t = 0; t < njobs; ++t) bytes += (size_t)jobs.j[t].rows * jobs.j[t].ld;
    const bool stream = bytes < ((size_t)8 << 20);          // the products inside a decoder step
    switch (n) {
    case 1: launch_gemv_n<1>(ctx, jobs, blocks, smem, ch, rows, stream); break;
    case 2: launch_gemv_n<2>(ctx, jobs, blocks, smem, ch, rows, stream); break;
    case 3: launch_gemv_n<3>(ctx, jobs, blocks, smem, ch, rows, stream); break;
    case 4: launch_gemv_n<4>(ctx, jobs, blocks, smem, ch, rows, stream); break;
    case 5: launch_gemv_n<5>(ctx, jobs, blocks, smem, ch, rows, stream); break;
    case 6: launch_gemv_n<6>(ctx, jobs, blocks, smem, ch, rows, stream); break;
    case 7: launch_gemv_n<7>(ctx, jobs, blocks, smem, ch, rows, stream); break;
    default: launch_gemv_n<8>(ctx, jobs, blocks, smem, ch, rows, stream); break;
    }
    return q8i_launch_check(ctx, "gemv");
}
