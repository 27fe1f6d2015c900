// q8_gemv_fast.h -- the streaming product's fast kernel as a body that other kernels can run in some
// of their blocks (the readout kernel runs it for the recurrent half of the next step's GRU r).
#pragma once

#include "q8_device.h"

struct GemvJob {
    const int8_t *W;
    const float *X;
    const float *bias;
    float *Y;
    int8_t *tap_xq;
    float *tap_xscale;
    int32_t *tap_acc;
    int rows, cols, ld, ldx, ldy, lpr, block0, rpb;
    float w_scale;
    const float *row_scale;     // NULL, or one weight scale per row in place of w_scale
};
#define Q8_MAX_JOBS 3
struct GemvJobs {
    GemvJob j[Q8_MAX_JOBS];
    int njobs;
};

__device__ __forceinline__ int pick_job(const GemvJobs &jobs, int bid)
{
    int ji = 0;
    for (int t = 1; t < jobs.njobs; ++t)
        if (bid >= jobs.j[t].block0) ji = t;
    return ji;
}

template <int N>
__device__ __forceinline__ void write_x_taps(const GemvJob &J, const int8_t *xq, const float *s_scale)
{
    if (J.tap_xq)
        for (int e = threadIdx.x; e < N * J.cols; e += blockDim.x) {
            const int j = e / J.cols, k = e - j * J.cols;
            J.tap_xq[e] = xq[j * J.ld + k];
        }
    if (J.tap_xscale && threadIdx.x < N) J.tap_xscale[threadIdx.x] = s_scale[threadIdx.x];
}

// The lane's partial sums of U staged rows against the N quantized vectors in LDS, without a
// branch: a lane whose 16 bytes lie past the row holds zeros (the loader read them from nowhere)
// and multiplies them with the row's last 16 codes.
template <int N, int U, int CH>
__device__ __forceinline__ void rows_dot_part_nb(const v4i (&w)[U][CH], int ld, int lane, const int8_t *xq, int (&acc)[U][N])
{
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int j = 0; j < N; ++j) acc[u][j] = 0;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int off = min((c * 64 + lane) * 16, ld - 16);
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const v4i x = *(const v4i *)(xq + (size_t)j * ld + off);
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u][j] = dot16(w[u][c], x, acc[u][j]);
        }
    }
}

// Rows of at most 1024 * CH bytes and cols % 4 == 0: activations and the first U rows of every
// wave are requested before anything is waited for; after that two register sets take turns, one
// pass's rows being multiplied while the next pass's are in flight (U rows per wave and pass).
// ROWS: every job has one weight scale per row (requested with the row's bias).
// STREAM: small matrices (a decoder step's) are read with the non-temporal hint, large ones plainly,
// so that a matrix of the size of the L2 that is multiplied again and again stays there.
// (bid: the block's index among the blocks of these jobs; a kernel that runs this body beside another passes
// its block index less the other's blocks.)
template <int N, int CH, bool ROWS, int U, bool STREAM>
__device__ __forceinline__ void gemv_fast_body(const GemvJobs &jobs, int bid, int8_t *smem)
{
    __shared__ float s_scale[8];
    __shared__ float s_red[8 * 4];
    __shared__ int s_t[4][U * N];
    const GemvJob &J = jobs.j[pick_job(jobs, bid)];
    const int blk = bid - J.block0;
    const int ld = J.ld;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r_begin = blk * J.rpb;
    const int r_end = min(J.rows, r_begin + J.rpb);

    XRegs<N, CH> xr;
    x_load<N, CH>(xr, J.X, N, J.cols, J.ldx);
    int r = r_begin + wave * U;
    const __amdgpu_buffer_rsrc_t rw = q8_rsrc(J.W, (size_t)J.rows * ld);
    const __amdgpu_buffer_rsrc_t rb = q8_rsrc(J.bias, J.bias ? (size_t)J.rows * sizeof(float) : 0);
    const __amdgpu_buffer_rsrc_t rs = q8_rsrc(J.row_scale, ROWS ? (size_t)J.rows * sizeof(float) : 0);
    const int last_row = J.rows - 1;
    // A pass's rows, their biases and (ROWS) their scales, all requested without a branch: rows past
    // the block's end read from nowhere (zeros); the per-row floats take one load instruction per
    // pass, lane u reading row u's (from a clamped row; absent arrays read as zero): a load
    // instruction per row would double the kernel's count of them.
    auto request = [&](v4i (&wr)[U][CH], float (&b)[2], int r0) {
        int row[U];
#pragma unroll
        for (int u = 0; u < U; ++u) row[u] = r0 + u < r_end ? r0 + u : -1;
        rows_load<U, CH, STREAM>(wr, rw, row, ld, lane);
        const int off = min(r0 + (lane & (U - 1)), last_row) * 4;
        b[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, off, 0, 0));
        b[1] = ROWS ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, off, 0, 0)) : 0.0f;
    };
    v4i w[U][CH], w2[U][CH];
    float bw[2], bw2[2];
    request(w, bw, r);
    x_finish<N, CH>(xr, N, ld, smem, s_scale, s_red);
    if (blk == 0) write_x_taps<N>(J, smem, s_scale);
    float cj = 0.0f, sxj = 0.0f;
    if (lane < N) { sxj = s_scale[lane]; cj = J.w_scale * sxj; }
    const bool has_bias = J.bias != nullptr;

    auto finish = [&](const v4i (&wr)[U][CH], const float (&b)[2], int r0) {
        int part[U][N], mine[U];
        rows_dot_part_nb<N, U, CH>(wr, ld, lane, smem, part);
        sums_to_lanes<N, U>(part, lane, s_t[wave], mine);      // lane j < N: the totals of vector j
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int a = mine[u];
            const float bu = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(b[0]), u));
            const float su = ROWS ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(b[1]), u)) : 0.0f;
            float y = (float)a * (ROWS ? su * sxj : cj);
            const float yb = y + bu;
            y = has_bias ? yb : y;
            if (lane < N && r0 + u < r_end) {
                J.Y[(size_t)lane * J.ldy + r0 + u] = y;
                if (J.tap_acc) J.tap_acc[(size_t)lane * J.rows + r0 + u] = a;
            }
        }
    };
    while (r < r_end) {
        request(w2, bw2, r + 4 * U);
        finish(w, bw, r);
        r += 4 * U;
        if (r >= r_end) break;
        request(w, bw, r + 4 * U);
        finish(w2, bw2, r);
        r += 4 * U;
    }
}
