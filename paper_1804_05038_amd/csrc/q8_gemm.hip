// q8_gemm.hip -- the 8-bit product of Section 3 for panels of more than 8 vectors (source
// positions of one sentence, or the hypotheses of many sentences decoded together, which
// Section 6 names as the next step): a blocked int8 GEMM on the gfx950 matrix cores.
// The arithmetic is that of the streaming kernels: per-vector activation codes, exact
// int32 sums, one fp32 scale product, separate bias addition.
#include "q8_internal.h"

struct GemmArgs {
    const int8_t *W;       // [rows x ld] int8
    const int8_t *Wt;      // the same matrix tile-packed (q8_pack_tiles), or NULL: every matrix-core operand of 16 rows x 64 k
                           // bytes is then one contiguous KiB instead of 16 pieces of rows that lie ld bytes apart, which the
                           // memory system delivers about 2.5 times as fast (measured: 192 KB per block, 2.1 against 5.3 us)
    const int8_t *xq;      // [n x ld] int8 codes of the n vectors
    const float *xscale;   // [n]
    const float *bias;     // [rows] or NULL
    float *Y;              // [n x ldy]
    int32_t *tap_acc;      // [n x rows] or NULL
    float *part_max;       // STATS: [n x ntiles] maximum of each 16-row tile
    double *part_sum;      // STATS: [n x ntiles] sum of exp(y - maximum)
    int rows, ld, n, ldy, ntiles;
    int tiled;             // Y as [ntiles][n][16]: every 16 x 16 result tile is one contiguous KiB
    float w_scale;
    const float *row_scale; // NULL, or one weight scale per row in place of w_scale
};
#define GEMM_MAX_JOBS 3
struct GemmJobs {          // products of one launch (blockIdx.z), all over the same number of vectors
    GemmArgs j[GEMM_MAX_JOBS];
};

// Block tiles (row tiles per wave, vector tiles): matrices of more than 8192 rows (the
// vocabulary) and the rest.
#ifndef GB_BIG_RT
#define GB_BIG_RT 2
#define GB_BIG_NT 8
#endif
#ifndef GB_SMALL_RT
#define GB_SMALL_RT 1
#define GB_SMALL_NT 4
#endif
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
    const int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    const GemmArgs &a = jobs.j[bz];
    constexpr int BN = 16 * NT;
    if (bx * 64 * RT >= a.rows) return;                  // the grid is sized for the largest job
    constexpr int PIECES = BN * (GB_K / 16) / 256;      // 16-byte pieces of a stage per thread
    __shared__ __align__(16) int8_t s_b[2][BN * GB_PITCH];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int r0 = (bx * 4 + wave) * 16 * RT;
    const int c0 = by * BN;
    const int ld = a.ld, n = a.n, rows = a.rows;

    // Every load below is unconditional and in bounds (rows, vectors and k offsets are clamped);
    // what lies outside the matrix is replaced by zeros when a stage is consumed.  That keeps the
    // number of loads per step fixed, so that waiting for one stage leaves the later ones in flight.
    const int8_t *wp[RT];
    bool row_ok[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int row = r0 + 16 * rt + i;
        row_ok[rt] = row < rows;
        wp[rt] = a.W + (size_t)(row_ok[rt] ? row : rows - 1) * ld;
        if (a.Wt) {            // this lane's 16 bytes of the row tile's first k step (tiles past the matrix: the last one, dropped below)
            const int tile = min((r0 + 16 * rt) >> 4, a.ntiles - 1);
            wp[rt] = a.Wt + (size_t)tile * (ld >> 6) * 1024 + lane * 16;
        }
    }
    const bool tiled = a.Wt != nullptr;
    const int kc_last = (ld >> 6) - 1;
    const int8_t *bp_g[PIECES];
    bool col_ok[PIECES];
#pragma unroll
    for (int u = 0; u < PIECES; ++u) {
        const int col = c0 + ((u * 256 + tid) >> 3);
        col_ok[u] = col < n;
        bp_g[u] = a.xq + (size_t)(col_ok[u] ? col : n - 1) * ld;
    }
    const int kb = (tid & 7) * 16;            // k offset of this thread's pieces within a stage
    const int klast = ld - 16;

    // Software pipeline over stages of GB_K k bytes, loads two stages ahead: while stage s is
    // multiplied out of LDS, stage s + 1 sits in one register set (or is still arriving) and
    // stage s + 2 is in flight into the other.
    struct Stage {
        v4i b[PIECES];       // this thread's pieces of the vectors' codes
        v4i a[RT][2];        // this lane's weight operands
    };
    Stage R0, R1;
    v4i acur[RT][2];
    const v4i zero4 = (v4i){0, 0, 0, 0};
    auto load_stage = [&](Stage &R, int k0) {
        const int kB = min(k0 + kb, klast);
#pragma unroll
        for (int u = 0; u < PIECES; ++u) R.b[u] = *(const v4i *)(bp_g[u] + kB);
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            const int kA = tiled ? min((k0 >> 6) + kc, kc_last) * 1024 : min(k0 + 64 * kc + 16 * g, klast);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) R.a[rt][kc] = *(const v4i *)(wp[rt] + kA);
        }
    };
    auto store_stage = [&](const Stage &R, int buf, int k0) {
        const bool kB_ok = k0 + kb < ld;
#pragma unroll
        for (int u = 0; u < PIECES; ++u) {
            const int p = u * 256 + tid;
            *(v4i *)(s_b[buf] + (p >> 3) * GB_PITCH + (p & 7) * 16) = (col_ok[u] && kB_ok) ? R.b[u] : zero4;
        }
#pragma unroll
        for (int kc = 0; kc < 2; ++kc) {
            const bool kA_ok = k0 + 64 * kc + 16 * g < ld;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) acur[rt][kc] = (row_ok[rt] && kA_ok) ? R.a[rt][kc] : zero4;
        }
    };

    v4i acc[RT][NT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[rt][t] = zero4;

    const int nst = (ld + GB_K - 1) / GB_K;
    load_stage(R0, 0);
    load_stage(R1, GB_K);                      // past the last stage: a clamped, unused reload
    store_stage(R0, 0, 0);
    load_stage(R0, 2 * GB_K);
    __syncthreads();
    // step s: multiply stage s (LDS buffer s & 1), move stage s + 1 from Rn to the other buffer,
    // which was last read before the previous barrier, and reuse Rn for stage s + 3
    auto step = [&](Stage &Rn, int s) {
        const int8_t *bp = s_b[s & 1] + i * GB_PITCH + 16 * g;
        v4i av[RT][2];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int kc = 0; kc < 2; ++kc) av[rt][kc] = acur[rt][kc];
        store_stage(Rn, (s + 1) & 1, (s + 1) * GB_K);
        load_stage(Rn, (s + 3) * GB_K);
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const v4i bv = *(const v4i *)(bp + t * 16 * GB_PITCH + 64 * kc);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    acc[rt][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[rt][kc], bv, acc[rt][t], 0, 0, 0);
            }
        __syncthreads();
    };
    int s = 0;
    for (; s + 1 < nst; s += 2) {                // always both halves: the load counts per path stay fixed
        step(R1, s);
        step(R0, s + 1);
    }
    if (s < nst) step(R1, s);

    // Epilogue, written so that the loads and the cross-lane steps of all NT tiles of a row tile
    // are issued together instead of one tile after the other.
    const bool vec_ok = ((a.ldy & 3) == 0) && (((uintptr_t)a.Y & 15) == 0);
    const bool bias_vec = (((uintptr_t)a.bias) & 15) == 0;
    float cs[NT], xs[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int col = c0 + 16 * t + i;
        xs[t] = col < n ? a.xscale[col] : 0.0f;
        cs[t] = a.w_scale * xs[t];
    }
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
        float rsv[4] = {0.f, 0.f, 0.f, 0.f};
        if (a.row_scale) {
#pragma unroll
            for (int r = 0; r < 4; ++r) rsv[r] = a.row_scale[min(row0 + r, rows - 1)];
        }
        float y[NT][4], m[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int col = c0 + 16 * t + i;
            const bool col_ok = col < n;
            m[t] = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                y[t][r] = -INFINITY;
                if (col_ok && row0 + r < rows) {
                    y[t][r] = (float)acc[rt][t][r] * (a.row_scale ? rsv[r] * xs[t] : cs[t]);
                    if (a.bias) y[t][r] = y[t][r] + (r == 0 ? b.x : r == 1 ? b.y : r == 2 ? b.z : b.w);
                    if (a.tap_acc) a.tap_acc[(size_t)col * rows + row0 + r] = acc[rt][t][r];
                }
                m[t] = fmaxf(m[t], y[t][r]);
            }
            if (a.tiled) {
                // rows past the matrix carry -inf; whoever reads the tile skips them
                if (col_ok)
                    *(float4 *)(a.Y + ((size_t)((r0 + 16 * rt) >> 4) * n + col) * 16 + 4 * g) =
                        make_float4(y[t][0], y[t][1], y[t][2], y[t][3]);
            } else if (col_ok) {
                if (vec_ok && row0 + 3 < rows) {
                    *(float4 *)(a.Y + (size_t)col * a.ldy + row0) = make_float4(y[t][0], y[t][1], y[t][2], y[t][3]);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (row0 + r < rows) a.Y[(size_t)col * a.ldy + row0 + r] = y[t][r];
                }
            }
        }
        if (STATS) {
            // (max, sum of exp) of the tile's 16 rows per vector: lanes i, i+16, i+32, i+48
#pragma unroll
            for (int t = 0; t < NT; ++t)
                m[t] = fmaxf(m[t], __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(m[t]), SWZ_XOR16)));
#pragma unroll
            for (int t = 0; t < NT; ++t) m[t] = fmaxf(m[t], __shfl_xor(m[t], 32, 64));
            double sd[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                sd[t] = 0.0;
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (y[t][r] > -INFINITY) sd[t] += (double)exp_le0(y[t][r] - m[t]);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) sd[t] += __shfl_xor(sd[t], 16, 64);
#pragma unroll
            for (int t = 0; t < NT; ++t) sd[t] += __shfl_xor(sd[t], 32, 64);
            const int tile = (r0 + 16 * rt) >> 4;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int col = c0 + 16 * t + i;
                if (col < n && g == 0) {
                    a.part_max[(size_t)col * a.ntiles + tile] = m[t];
                    a.part_sum[(size_t)col * a.ntiles + tile] = sd[t];
                }
            }
        }
    }
}

// ============================================================== K-resident blocks ==
// Rows of at most 64 KS bytes (KS = 8 or 16): nothing is staged.  A block of four waves takes
// 64 rows x 64 vectors; every wave requests its 16 rows whole (KS operands per lane), the block
// requests the 64 vectors' codes whole (one vector row per wave-wide load) and parks them in LDS
// at pitch 64 KS + 16 (16 lanes x 16 bytes then fall on distinct banks); one barrier; 4 KS
// matrix-core instructions per wave in four independent chains.  All loads go through
// bounds-checked descriptors without branches (what lies outside reads as zero), so they are all
// in flight before the first wait.  Matrices and panels below 2 GiB, no taps, no statistics.
template <int KS>
__global__ __launch_bounds__(256) void gemm_resident_kernel(GemmJobs jobs)
{
    extern __shared__ __align__(16) int8_t s_v[];        // [64 x pitch]
    const GemmArgs &a = jobs.j[blockIdx.z];
    if ((int)blockIdx.x * 64 >= a.rows) return;          // the grid is sized for the largest job
    constexpr int pitch = 64 * KS + 16, PCS = 4 * KS;    // 16-byte pieces per (padded) vector
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int r0 = ((int)blockIdx.x * 4 + wave) * 16, c0 = (int)blockIdx.y * 64;
    const int ld = a.ld, n = a.n, rows = a.rows;

    // the vectors' codes: thread (v, pc) = (tid / PCS, tid % PCS) takes piece pc of vectors v, v + 256 / PCS, ...
    const __amdgpu_buffer_rsrc_t rx = q8_rsrc(a.xq, (size_t)n * ld);
    const int pc = tid & (PCS - 1), v0 = tid / PCS;
    v4i bq[KS];
#pragma unroll
    for (int u = 0; u < KS; ++u) {
        const int col = c0 + v0 + u * (256 / PCS);
        const unsigned off = (col < n && pc * 16 < ld) ? (unsigned)col * (unsigned)ld + pc * 16u : Q8_OOB;
        bq[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rx, (int)off, 0, 0));
    }
    // this wave's 16 rows
    const bool tiled = a.Wt != nullptr;
    const __amdgpu_buffer_rsrc_t rw = tiled ? q8_rsrc(a.Wt, (size_t)a.ntiles * 16 * ld) : q8_rsrc(a.W, (size_t)rows * ld);
    const int row = r0 + i;
    v4i av[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const int k = 64 * s + 16 * g;
        unsigned off = (row < rows && k < ld) ? (unsigned)row * (unsigned)ld + (unsigned)k : Q8_OOB;
        // tile-packed: operand (row tile, k step) is one KiB, lane by lane (rows past the matrix are zero in it)
        if (tiled) off = (r0 < rows && 64 * s < ld) ? (((unsigned)(r0 >> 4) * (unsigned)(ld >> 6) + (unsigned)s) << 10) + 16u * lane : Q8_OOB;
        av[s] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rw, (int)off, 0, 0));
    }
    // epilogue operands: dequantization factors and biases
    float cs[4];
    const __amdgpu_buffer_rsrc_t rs = q8_rsrc(a.xscale, (size_t)n * sizeof(float));
#pragma unroll
    for (int t = 0; t < 4; ++t)
        cs[t] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(c0 + 16 * t + i < n ? (unsigned)(c0 + 16 * t + i) * 4u : Q8_OOB), 0, 0));
    const int row0 = r0 + 4 * g;
    const __amdgpu_buffer_rsrc_t rb = q8_rsrc(a.bias, a.bias ? (size_t)rows * sizeof(float) : 0);
    const __amdgpu_buffer_rsrc_t rr = q8_rsrc(a.row_scale, a.row_scale ? (size_t)rows * sizeof(float) : 0);
    float bias[4], rsv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int off = (int)(row0 + r < rows ? (unsigned)(row0 + r) * 4u : Q8_OOB);
        bias[r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, off, 0, 0));
        rsv[r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rr, off, 0, 0));
    }
    __builtin_amdgcn_sched_barrier(0);

#pragma unroll
    for (int u = 0; u < KS; ++u) *(v4i *)(s_v + (v0 + u * (256 / PCS)) * pitch + pc * 16) = bq[u];
    __syncthreads();
    if (r0 >= rows) return;                              // wave-uniform, after the only barrier

    v4i acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = (v4i){0, 0, 0, 0};
    const int8_t *bp = s_v + i * pitch + 16 * g;
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const v4i bv = *(const v4i *)(bp + t * 16 * pitch + 64 * s);
            acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[s], bv, acc[t], 0, 0, 0);
        }

    const bool vec_ok = ((a.ldy & 3) == 0) && (((uintptr_t)a.Y & 15) == 0);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int col = c0 + 16 * t + i;
        if (col >= n) continue;
        const float c = a.w_scale * cs[t];
        float y[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            y[r] = (float)acc[t][r] * (a.row_scale ? rsv[r] * cs[t] : c);
            if (a.bias) y[r] = y[r] + bias[r];
        }
        if (vec_ok && row0 + 3 < rows) {
            *(float4 *)(a.Y + (size_t)col * a.ldy + row0) = make_float4(y[0], y[1], y[2], y[3]);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (row0 + r < rows) a.Y[(size_t)col * a.ldy + row0 + r] = y[r];
        }
    }
}

// ===================================================== three products, k split over waves ==
// The readout's three partial products (Eq. 2's first layer: W_s q(s), W_y q(y), W_c q(H_t), 512 rows
// each, rows of 1024 / 512 / 2048 bytes) for a panel of slots in one K-resident launch.  The block
// kernel above needs ten staged steps for the longest rows and fills 120 blocks (10 us); here block
// (rg, cg) owns rows 32 rg .. 32 rg + 31 of all three matrices and slots 32 cg .. 32 cg + 31, whose codes
// for all three products sit in LDS (3632 bytes per slot), and the 3584 k bytes are cut into seven
// chunks of 512: wave (ut, chunk) multiplies one tile of 16 rows over one chunk against the two slot
// tiles, every load requested up front.  The exact int32 partial sums of a product's chunks meet in LDS
// and are dequantized once, as the block kernel does it.  Rows of other lengths take the block kernel.
#define KS3_ROWS 32
#define KS3_SLOTS 32
#define KS3_WAVES 14
struct Ksplit3Args {
    const int8_t *W[3], *Wt[3];    // [R x ld], and tile-packed or NULL
    const int8_t *xq[3];           // codes [n x ld]
    const float *xs[3];            // [n]
    float *Y[3];                   // [n x ldy]
    float w_scale[3];
    int R, n, ldy;
};

__global__ __launch_bounds__(64 * KS3_WAVES) void gemm_ksplit3_kernel(Ksplit3Args a)
{
    extern __shared__ __align__(16) int8_t s_k3[];
    constexpr int NT = 64 * KS3_WAVES;
    constexpr int LD0 = 1024, LD1 = 512, LD2 = 2048;
    constexpr int P0 = LD0 + 16, P1 = LD1 + 16, P2 = LD2 + 16;           // LDS pitches
    int8_t *s_x0 = s_k3, *s_x1 = s_x0 + KS3_SLOTS * P0, *s_x2 = s_x1 + KS3_SLOTS * P1;
    int *s_e = (int *)(s_x2 + KS3_SLOTS * P2);                           // [14 waves][2 slot tiles][16 slots][16 rows]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int rg = blockIdx.x, cg = blockIdx.y, n = a.n, c0 = cg * KS3_SLOTS, r0 = rg * KS3_ROWS;

    // ---- all loads up front (outside the arrays: zero) ----
    constexpr int U0 = (KS3_SLOTS * LD0 / 16 + NT - 1) / NT, U1 = (KS3_SLOTS * LD1 / 16 + NT - 1) / NT, U2 = (KS3_SLOTS * LD2 / 16 + NT - 1) / NT;
    const __amdgpu_buffer_rsrc_t rq0 = q8_rsrc(a.xq[0], (size_t)n * LD0), rq1 = q8_rsrc(a.xq[1], (size_t)n * LD1), rq2 = q8_rsrc(a.xq[2], (size_t)n * LD2);
    v4i b0[U0], b1[U1], b2[U2];
#pragma unroll
    for (int u = 0; u < U0; ++u) {
        const int p = u * NT + tid, slot = p / (LD0 / 16), piece = p - slot * (LD0 / 16);
        const unsigned off = (p < KS3_SLOTS * LD0 / 16 && c0 + slot < n) ? (unsigned)(c0 + slot) * LD0 + 16u * piece : Q8_OOB;
        b0[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rq0, (int)off, 0, 0));
    }
#pragma unroll
    for (int u = 0; u < U1; ++u) {
        const int p = u * NT + tid, slot = p / (LD1 / 16), piece = p - slot * (LD1 / 16);
        const unsigned off = (p < KS3_SLOTS * LD1 / 16 && c0 + slot < n) ? (unsigned)(c0 + slot) * LD1 + 16u * piece : Q8_OOB;
        b1[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rq1, (int)off, 0, 0));
    }
#pragma unroll
    for (int u = 0; u < U2; ++u) {
        const int p = u * NT + tid, slot = p / (LD2 / 16), piece = p - slot * (LD2 / 16);
        const unsigned off = (p < KS3_SLOTS * LD2 / 16 && c0 + slot < n) ? (unsigned)(c0 + slot) * LD2 + 16u * piece : Q8_OOB;
        b2[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rq2, (int)off, 0, 0));
    }
    // this wave: row tile ut, chunk ch -> product j, first k byte kbase
    const int ut = wave / 7, ch = wave % 7;
    const int j = ch < 2 ? 0 : ch == 2 ? 1 : 2;
    const int kbase = 512 * (ch < 2 ? ch : ch == 2 ? 0 : ch - 3);
    const int ldw = j == 0 ? LD0 : j == 1 ? LD1 : LD2;
    const int8_t *wt = a.Wt[j];
    const __amdgpu_buffer_rsrc_t rw = q8_rsrc(wt ? wt : a.W[j], (size_t)a.R * ldw);
    const int row0 = r0 + 16 * ut;                                       // R % 32 == 0: a whole tile inside the matrix
    v4i av[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        unsigned off = (unsigned)(row0 + i) * (unsigned)ldw + (unsigned)(kbase + 64 * s + 16 * g);
        if (wt) off = (((unsigned)(row0 >> 4) * (unsigned)(ldw >> 6) + (unsigned)((kbase >> 6) + s)) << 10) + 16u * lane;
        av[s] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rw, (int)off, 0, 0));
    }
    // dequantization factors of the (slot, row) pairs tid and tid + NT of 32 x 32
    const __amdgpu_buffer_rsrc_t rs0 = q8_rsrc(a.xs[0], (size_t)n * 4), rs1 = q8_rsrc(a.xs[1], (size_t)n * 4), rs2 = q8_rsrc(a.xs[2], (size_t)n * 4);
    float xs[2][3];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int pr = e * NT + tid, col = c0 + (pr >> 5);
        const int off = (int)((pr < KS3_SLOTS * KS3_ROWS && col < n) ? (unsigned)col * 4u : Q8_OOB);
        xs[e][0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs0, off, 0, 0));
        xs[e][1] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs1, off, 0, 0));
        xs[e][2] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs2, off, 0, 0));
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- codes into LDS ----
#pragma unroll
    for (int u = 0; u < U0; ++u) {
        const int p = u * NT + tid, slot = p / (LD0 / 16), piece = p - slot * (LD0 / 16);
        if (p < KS3_SLOTS * LD0 / 16) *(v4i *)(s_x0 + slot * P0 + 16 * piece) = b0[u];
    }
#pragma unroll
    for (int u = 0; u < U1; ++u) {
        const int p = u * NT + tid, slot = p / (LD1 / 16), piece = p - slot * (LD1 / 16);
        if (p < KS3_SLOTS * LD1 / 16) *(v4i *)(s_x1 + slot * P1 + 16 * piece) = b1[u];
    }
#pragma unroll
    for (int u = 0; u < U2; ++u) {
        const int p = u * NT + tid, slot = p / (LD2 / 16), piece = p - slot * (LD2 / 16);
        if (p < KS3_SLOTS * LD2 / 16) *(v4i *)(s_x2 + slot * P2 + 16 * piece) = b2[u];
    }
    __syncthreads();

    // ---- products ----
    v4i acc[2] = {(v4i){0, 0, 0, 0}, (v4i){0, 0, 0, 0}};
    {
        const int pitch = j == 0 ? P0 : j == 1 ? P1 : P2;
        const int8_t *bp = (j == 0 ? s_x0 : j == 1 ? s_x1 : s_x2) + i * pitch + kbase + 16 * g;
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const v4i bv = *(const v4i *)(bp + t * 16 * pitch + 64 * s);
                acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[s], bv, acc[t], 0, 0, 0);
            }
    }
    // lane (i, g) holds rows 4 g + r, r = 0..3, of slot i of each tile
#pragma unroll
    for (int t = 0; t < 2; ++t) *(v4i *)(s_e + (((wave * 2 + t) * 16 + i) * 16 + 4 * g)) = acc[t];
    __syncthreads();

    // ---- chunks summed, dequantized, stored: consecutive threads, consecutive rows of a slot ----
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int pr = e * NT + tid;
        if (pr >= KS3_SLOTS * KS3_ROWS) break;
        const int c = pr >> 5, r = pr & 31, col = c0 + c;
        const int at = ((c >> 4) * 16 + (c & 15)) * 16 + (r & 15), w0 = (r >> 4) * 7;        // wave (ut, chunk) = 7 ut + chunk
        const int e0 = s_e[(w0 + 0) * 512 + at] + s_e[(w0 + 1) * 512 + at];
        const int e1 = s_e[(w0 + 2) * 512 + at];
        const int e2 = ((s_e[(w0 + 3) * 512 + at] + s_e[(w0 + 4) * 512 + at]) + s_e[(w0 + 5) * 512 + at]) + s_e[(w0 + 6) * 512 + at];
        if (col < n) {
            const size_t o = (size_t)col * a.ldy + r0 + r;
            a.Y[0][o] = (float)e0 * (a.w_scale[0] * xs[e][0]);
            a.Y[1][o] = (float)e1 * (a.w_scale[1] * xs[e][1]);
            a.Y[2][o] = (float)e2 * (a.w_scale[2] * xs[e][2]);
        }
    }
}

// Whether the three products W[u] . xq[u] (no bias, no taps, plain output at pitch ldy) take the kernel above.
bool q8i_gemm_ksplit3_ok(const q8i_gemm_job *d, int n)
{
    const int R = d[0].W->rows;
    if (R % KS3_ROWS || n < 1 || (R / KS3_ROWS) * ((n + KS3_SLOTS - 1) / KS3_SLOTS) > 256) return false;
    static const int want[3] = {1024, 512, 2048};
    for (int u = 0; u < 3; ++u) {
        if (d[u].W->rows != R || d[u].W->ld != want[u] || d[u].bias || d[u].tap_acc || d[u].part_max || d[u].tiled || d[u].row_scale ||
            d[u].ldy != d[0].ldy || (size_t)n * want[u] >= (1u << 31))
            return false;
    }
    return true;
}

q8_status q8i_gemm_ksplit3(q8_ctx *ctx, const q8i_gemm_job *d, int n)
{
    Ksplit3Args a;
    for (int u = 0; u < 3; ++u) {
        a.W[u] = d[u].W->data; a.Wt[u] = d[u].W->tiles; a.xq[u] = d[u].xq; a.xs[u] = d[u].xscale; a.Y[u] = d[u].Y;
        a.w_scale[u] = d[u].W->scale;
    }
    a.R = d[0].W->rows; a.n = n; a.ldy = d[0].ldy;
    const size_t smem = (size_t)KS3_SLOTS * (1024 + 16 + 512 + 16 + 2048 + 16) + (size_t)KS3_WAVES * 2 * 1024;
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute((const void *)gemm_ksplit3_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return q8_fail(ctx, Q8_ERR_DEVICE, "three-product kernel: %s", hipGetErrorString(e));
        attr_set = true;
    }
    Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, gemm_ksplit3_kernel, dim3(a.R / KS3_ROWS, (n + KS3_SLOTS - 1) / KS3_SLOTS), dim3(64 * KS3_WAVES), smem, a);
    return q8i_launch_check(ctx, "three products");
}

// ============================================ rows of 1024 bytes, k split over two waves ==
// Products with rows of exactly 1024 bytes over a panel of at most 336 slots (u(s') of Eq. 6 and the
// recurrent product of GRU q, which share a launch): block (rg, cg, job) owns 128 rows and 48 slots;
// wave (row tile, half) multiplies 16 rows over 512 k bytes against the three slot tiles, the two exact
// int32 halves meet in LDS and are dequantized once, and a slot's 128 results leave as 512 contiguous
// bytes.  Against the 64 x 64 blocks of gemm_resident_kernel a compute unit takes in 178 KB instead of
// 2 x 128 KB, and the results leave in whole lines.
#define KS2_ROWS 128
#define KS2_SLOTS 48
struct Ksplit2Args {
    GemmArgs j[2];
};

__global__ __launch_bounds__(1024) void gemm_ksplit2_kernel(Ksplit2Args jobs)
{
    extern __shared__ __align__(16) int8_t s_k2[];
    constexpr int NT = 1024, LD = 1024, PITCH = LD + 16;
    const GemmArgs &a = jobs.j[blockIdx.z];
    if ((int)blockIdx.x * KS2_ROWS >= a.rows) return;            // the grid is sized for the larger job
    int8_t *s_x = s_k2;
    int *s_e = (int *)(s_k2 + KS2_SLOTS * PITCH);                // [16 waves][3 slot tiles][16 slots][16 rows]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int n = a.n, c0 = (int)blockIdx.y * KS2_SLOTS, r0 = (int)blockIdx.x * KS2_ROWS;

    // ---- all loads up front ----
    constexpr int UX = KS2_SLOTS * (LD / 16) / NT;              // 3 pieces per thread
    static_assert(KS2_SLOTS * (LD / 16) % NT == 0, "pieces divide among the threads");
    const __amdgpu_buffer_rsrc_t rq = q8_rsrc(a.xq, (size_t)n * LD);
    v4i bq[UX];
#pragma unroll
    for (int u = 0; u < UX; ++u) {
        const int p = u * NT + tid, slot = p / (LD / 16), piece = p - slot * (LD / 16);
        const unsigned off = c0 + slot < n ? (unsigned)(c0 + slot) * LD + 16u * piece : Q8_OOB;
        bq[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rq, (int)off, 0, 0));
    }
    const int rt = wave >> 1, half = wave & 1, kbase = 512 * half;
    const __amdgpu_buffer_rsrc_t rw = q8_rsrc(a.Wt ? a.Wt : a.W, (size_t)a.rows * LD);      // rows % 128 == 0
    const int row0 = r0 + 16 * rt;
    v4i av[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        unsigned off = (unsigned)(row0 + i) * (unsigned)LD + (unsigned)(kbase + 64 * s + 16 * g);
        if (a.Wt) off = (((unsigned)(row0 >> 4) * (unsigned)(LD >> 6) + (unsigned)((kbase >> 6) + s)) << 10) + 16u * lane;
        av[s] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rw, (int)off, 0, 0));
    }
    // per (slot, row) pair tid + 1024 e, e = 0..5: row = pair % 128 is the same for all six
    const int row = r0 + (tid & 127);
    const __amdgpu_buffer_rsrc_t rs = q8_rsrc(a.xscale, (size_t)n * 4), rb = q8_rsrc(a.bias, a.bias ? (size_t)a.rows * 4 : 0);
    const float bias = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, (int)((unsigned)row * 4u), 0, 0));
    float xs[6];
#pragma unroll
    for (int e = 0; e < 6; ++e) {
        const int col = c0 + ((e * NT + tid) >> 7);
        xs[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, (int)(col < n ? (unsigned)col * 4u : Q8_OOB), 0, 0));
    }
    __builtin_amdgcn_sched_barrier(0);

#pragma unroll
    for (int u = 0; u < UX; ++u) {
        const int p = u * NT + tid, slot = p / (LD / 16), piece = p - slot * (LD / 16);
        *(v4i *)(s_x + slot * PITCH + 16 * piece) = bq[u];
    }
    __syncthreads();

    v4i acc[3] = {(v4i){0, 0, 0, 0}, (v4i){0, 0, 0, 0}, (v4i){0, 0, 0, 0}};
    {
        const int8_t *bp = s_x + i * PITCH + kbase + 16 * g;
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                const v4i bv = *(const v4i *)(bp + t * 16 * PITCH + 64 * s);
                acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[s], bv, acc[t], 0, 0, 0);
            }
    }
#pragma unroll
    for (int t = 0; t < 3; ++t) *(v4i *)(s_e + (((wave * 3 + t) * 16 + i) * 16 + 4 * g)) = acc[t];
    __syncthreads();

#pragma unroll
    for (int e = 0; e < 6; ++e) {
        const int pr = e * NT + tid, c = pr >> 7, r = pr & 127, col = c0 + c;
        const int at = ((c >> 4) * 16 + (c & 15)) * 16 + (r & 15), w0 = (r >> 4) * 2;        // wave (row tile, half) = 2 rt + half
        const int sum = s_e[w0 * 768 + at] + s_e[(w0 + 1) * 768 + at];
        float y = (float)sum * (a.w_scale * xs[e]);
        if (a.bias) y = y + bias;
        if (col < n) a.Y[(size_t)col * a.ldy + row] = y;
    }
}

// Whether the products d[0 .. njobs) (njobs <= 2; plain output, no taps) take the kernel above.
bool q8i_gemm_ksplit2_ok(const q8i_gemm_job *d, int njobs, int n)
{
    if (njobs < 1 || njobs > 2 || n < 1 || (n + KS2_SLOTS - 1) / KS2_SLOTS > 7) return false;
    int blocks = 0;
    for (int u = 0; u < njobs; ++u) {
        if (d[u].W->ld != 1024 || d[u].W->rows % KS2_ROWS || d[u].tap_acc || d[u].part_max || d[u].tiled || d[u].row_scale ||
            (size_t)d[u].W->rows * 1024 >= (1u << 31))
            return false;
        blocks += d[u].W->rows / KS2_ROWS;
    }
    return blocks * ((n + KS2_SLOTS - 1) / KS2_SLOTS) <= 256;
}

q8_status q8i_gemm_ksplit2(q8_ctx *ctx, const q8i_gemm_job *d, int njobs, int n)
{
    Ksplit2Args jobs;
    int max_rows = 0;
    for (int t = 0; t < 2; ++t) {
        const q8i_gemm_job &q = d[t < njobs ? t : 0];
        GemmArgs &a = jobs.j[t];
        a.W = q.W->data; a.Wt = q.W->tiles; a.xq = q.xq; a.xscale = q.xscale; a.bias = q.bias; a.Y = q.Y; a.tap_acc = nullptr;
        a.part_max = nullptr; a.part_sum = nullptr;
        a.rows = q.W->rows; a.ld = q.W->ld; a.n = n; a.ldy = q.ldy; a.ntiles = (q.W->rows + 15) / 16; a.tiled = 0;
        a.w_scale = q.W->scale; a.row_scale = nullptr;
        if (a.rows > max_rows) max_rows = a.rows;
    }
    const size_t smem = (size_t)KS2_SLOTS * (1024 + 16) + (size_t)16 * 3 * 1024;
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute((const void *)gemm_ksplit2_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return q8_fail(ctx, Q8_ERR_DEVICE, "k-split product kernel: %s", hipGetErrorString(e));
        attr_set = true;
    }
    Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, gemm_ksplit2_kernel, dim3(max_rows / KS2_ROWS, (n + KS2_SLOTS - 1) / KS2_SLOTS, njobs), dim3(1024), smem, jobs);
    return q8i_launch_check(ctx, "k-split products");
}

// ================================================================ vocabulary panel ==
// The vocabulary product for a panel of hypothesis slots (many sentences side by side).  Unlike
// the block kernel above, a block keeps its share of the vectors' codes in LDS for its whole
// life (up to 160 KB per workgroup on gfx950) and streams tile-packed 16-row weight tiles past
// them, one tile ahead in registers: no barrier after the prologue, every weight byte read once
// per column group.  Per (row tile, column tile): KC matrix-core steps, then dequantize, bias,
// and the tile's (max, sum of exp) per slot with the cross-lane steps on v_permlane16/32_swap.
// The logits themselves are not kept (64 MB per step at 320 slots): the selection computes
// those of the few tiles that can hold one of the k best again.
struct PanelArgs {
    const int8_t *tiles;   // tile-packed weights (q8_pack_tiles)
    const int8_t *xq;      // [n x ld] codes
    const float *xscale, *bias;
    float *part_max;       // [n x ntiles]
    double *part_sum;
    int rows, ld, n, ntiles, cols_per_group;
    float w_scale;
};

#define VP_WAVES 16        // at most; the launch picks the number of waves that divides the row tiles most evenly
#define VP_MAX_NT 16

// One row tile against U column tiles starting at column tile t0: U independent accumulation
// chains keep the matrix core busy (a single chain waits ~44 cycles per step) and their
// epilogues interleave.  FULL: all 16 rows and all 16 U columns exist, nothing is masked (the
// masked form costs about twice the vector instructions, which are what bounds this kernel:
// per result tile 8 matrix-core steps stand against some 50 vector instructions).
template <int KC, int U, bool FULL>
__device__ __forceinline__ void panel_tiles(const PanelArgs &a, const v4i (&A)[KC], const int8_t *bt, int pitch, const float *s_c,
                                            int tile, int t0, int nt, int cols, int c_base, float4 b, int i, int g)
{
    v4i acc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) acc[u] = (v4i){0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < KC; ++s)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // column tiles past the panel read the first tile of the group again (in bounds); their results are dropped
            const v4i bv = *(const v4i *)(bt + ((FULL || t0 + u < nt) ? u : 0) * 16 * pitch + 64 * s);
            acc[u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[s], bv, acc[u], 0, 0, 0);
        }
    const int row0 = tile * 16 + 4 * g;
    const float bias[4] = {b.x, b.y, b.z, b.w};
    float y[U][4], m[U];
    double sd[U];
    if (FULL) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float c = s_c[16 * (t0 + u) + i];
#pragma unroll
            for (int r = 0; r < 4; ++r) y[u][r] = (float)acc[u][r] * c;
            if (a.bias) {
#pragma unroll
                for (int r = 0; r < 4; ++r) y[u][r] = y[u][r] + bias[r];
            }
            m[u] = fmaxf(fmaxf(y[u][0], y[u][1]), fmaxf(y[u][2], y[u][3]));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) m[u] = quad_rows_max(m[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            sd[u] = (double)exp_le0(y[u][0] - m[u]);
#pragma unroll
            for (int r = 1; r < 4; ++r) sd[u] += (double)exp_le0(y[u][r] - m[u]);
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int colr = 16 * (t0 + u) + i;                  // column within the panel
            const bool col_ok = t0 + u < nt && colr < cols;
            const float c = col_ok ? s_c[colr] : 0.0f;
            m[u] = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                y[u][r] = -INFINITY;
                if (col_ok && row0 + r < a.rows) {
                    y[u][r] = (float)acc[u][r] * c;
                    if (a.bias) y[u][r] = y[u][r] + bias[r];
                }
                m[u] = fmaxf(m[u], y[u][r]);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) m[u] = quad_rows_max(m[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            sd[u] = 0.0;
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (y[u][r] > -INFINITY) sd[u] += (double)exp_le0(y[u][r] - m[u]);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) sd[u] = quad_rows_sum(sd[u]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int colr = 16 * (t0 + u) + i;
        if ((FULL || (t0 + u < nt && colr < cols)) && g == 0) {
            a.part_max[(size_t)(c_base + colr) * a.ntiles + tile] = m[u];
            a.part_sum[(size_t)(c_base + colr) * a.ntiles + tile] = sd[u];
        }
    }
}

template <int KC, int U>      // 64-byte k steps per row: ld = 64 KC; column tiles per inner step
__global__ __launch_bounds__(64 * VP_WAVES) void vocab_panel_kernel(PanelArgs a)
{
    extern __shared__ __align__(16) int8_t s_x[];        // [cols x pitch]
    constexpr int ld = 64 * KC, pitch = ld + 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nthr = blockDim.x, nwave = nthr >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int n = a.n, c_base = blockIdx.y * a.cols_per_group;
    const int cols = min(a.cols_per_group, n - c_base);       // > 0 by construction of the grid
    const int nt = (cols + 15) >> 4;
    // this wave's row tiles: gw, gw + stride, ...
    const int gw = blockIdx.x * nwave + wave, stride = gridDim.x * nwave;

    v4i A0[KC], A1[KC];
    auto load_tile = [&](v4i (&A)[KC], int tile) {
        const int8_t *p = a.tiles + ((size_t)(tile < a.ntiles ? tile : a.ntiles - 1) * KC) * 1024 + lane * 16;
#pragma unroll
        for (int s = 0; s < KC; ++s) A[s] = *(const v4i *)(p + 1024 * s);
    };
    load_tile(A0, gw);
    // the codes of this block's slots into LDS (slots past the panel are zero): eight 16-byte pieces per
    // thread and round, requested together through a bounds-checked descriptor (no branch around a
    // load: inside one, every piece would be a memory round trip of its own)
    {
        const __amdgpu_buffer_rsrc_t rx = q8_rsrc(a.xq + (size_t)c_base * ld, (size_t)cols * ld);
        const int total = nt * 16 * (ld / 16);
        for (int p0 = 0; p0 < total; p0 += 8 * nthr) {
            v4i v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + u * nthr + tid;               // piece p: slot p / (ld / 16), bytes 16 (p % (ld / 16)) ..
                v[u] = __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(p < total ? (unsigned)p * 16u : Q8_OOB), 0, 0));
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + u * nthr + tid;
                const int col = p / (ld / 16), ch = p - col * (ld / 16);
                if (p < total) *(v4i *)(s_x + col * pitch + ch * 16) = v[u];
            }
        }
    }
    float *s_c = (float *)(s_x + (size_t)a.cols_per_group * pitch);      // dequantization factor of every slot
    for (int c = tid; c < nt * 16; c += nthr) s_c[c] = c < cols ? a.w_scale * a.xscale[c_base + c] : 0.0f;
    __syncthreads();

    const bool bias_vec = (((uintptr_t)a.bias) & 15) == 0;
    const int8_t *bp = s_x + i * pitch + 16 * g;
    const int nt_full = cols >> 4;                           // column tiles without a missing slot
    auto do_tile = [&](const v4i (&A)[KC], int tile) {
        const int row0 = tile * 16 + 4 * g;
        const bool rows_full = tile * 16 + 16 <= a.rows;
        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a.bias) {
            if (bias_vec && row0 + 3 < a.rows) {
                b = *(const float4 *)(a.bias + row0);
            } else {
                if (row0 < a.rows) b.x = a.bias[row0];
                if (row0 + 1 < a.rows) b.y = a.bias[row0 + 1];
                if (row0 + 2 < a.rows) b.z = a.bias[row0 + 2];
                if (row0 + 3 < a.rows) b.w = a.bias[row0 + 3];
            }
        }
        for (int t0 = 0; t0 < nt; t0 += U) {
            const int8_t *bt = bp + t0 * 16 * pitch;
            if (rows_full && t0 + U <= nt_full) panel_tiles<KC, U, true>(a, A, bt, pitch, s_c, tile, t0, nt, cols, c_base, b, i, g);
            else panel_tiles<KC, U, false>(a, A, bt, pitch, s_c, tile, t0, nt, cols, c_base, b, i, g);
        }
    };
    for (int tile = gw; tile < a.ntiles; tile += 2 * stride) {
        load_tile(A1, tile + stride);
        do_tile(A0, tile);
        if (tile + stride < a.ntiles) {
            load_tile(A0, tile + 2 * stride);
            do_tile(A1, tile + stride);
        }
    }
}

// Whether the panel kernel takes this product: tile-packed weights with rows of 512 or 640 bytes.
bool q8i_vocab_panel_ok(const q8_mat *W) { return W->tiles != nullptr && (W->ld == 512 || W->ld == 640); }

q8_status q8i_vocab_panel(q8_ctx *ctx, const q8_mat *W, const float *bias, const int8_t *xq, const float *xscale, int n,
                          float *part_max, double *part_sum)
{
    PanelArgs a;
    a.tiles = W->tiles; a.xq = xq; a.xscale = xscale; a.bias = bias;
    a.part_max = part_max; a.part_sum = part_sum;
    a.rows = W->rows; a.ld = W->ld; a.n = n; a.ntiles = (W->rows + 15) / 16; a.w_scale = W->scale;
    // column groups of equal size, as many slots as fit the LDS (codes at pitch ld + 16, one float
    // per slot) and VP_MAX_NT column tiles; about one block per compute unit
    int max_cols = (int)((160 * 1024) / (size_t)(W->ld + 16 + 4)) & ~15;
    if (max_cols > 16 * VP_MAX_NT) max_cols = 16 * VP_MAX_NT;
    const int ngroups = (n + max_cols - 1) / max_cols;
    a.cols_per_group = ((n + ngroups - 1) / ngroups + 15) & ~15;
    int gx = 256 / ngroups;
    if (gx < 1) gx = 1;
    if (gx * 8 > a.ntiles) gx = (a.ntiles + 7) / 8;
    const int gy = (n + a.cols_per_group - 1) / a.cols_per_group;
    // waves per block (8..16): the count for which the busiest wave's row tiles exceed the average least
    int nw = 8;
    double best = 1e30;
    for (int w = 8; w <= VP_WAVES; ++w) {
        const int waves = gx * w, most = (a.ntiles + waves - 1) / waves;
        const double ratio = (double)most * waves / a.ntiles;
        if (ratio < best - 1e-9) { best = ratio; nw = w; }
    }
    const size_t smem = (size_t)a.cols_per_group * (W->ld + 16 + 4);
    // column tiles per inner step: five when they divide the group's tiles and four do not (rows of 512
    // bytes only: with ten k steps per row five chains no longer fit the registers of 16 waves)
    const int ntg = a.cols_per_group / 16;
    const bool five = W->ld == 512 && ntg % 5 == 0 && ntg % 4 != 0;
    typedef void (*kern_t)(PanelArgs);
    const kern_t kern = W->ld == 512 ? (five ? vocab_panel_kernel<8, 5> : vocab_panel_kernel<8, 4>) : vocab_panel_kernel<10, 4>;
    static bool attr_set[3] = {false, false, false};
    const int which = W->ld == 512 ? (five ? 1 : 0) : 2;
    if (!attr_set[which]) {
        const hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return q8_fail(ctx, Q8_ERR_DEVICE, "vocabulary panel kernel: %s", hipGetErrorString(e));
        attr_set[which] = true;
    }
    Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, kern, dim3(gx, gy), dim3(64 * nw), smem, a);
    return q8i_launch_check(ctx, "vocabulary panel");
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
        a.W = q.W->data; a.Wt = (q.W->tiles && q.W->ld % 64 == 0) ? q.W->tiles : nullptr; a.xq = q.xq; a.xscale = q.xscale; a.bias = q.bias; a.Y = q.Y; a.tap_acc = q.tap_acc;
        a.part_max = q.part_max; a.part_sum = q.part_sum;
        a.rows = q.W->rows; a.ld = q.W->ld; a.n = n; a.ldy = q.ldy; a.ntiles = (q.W->rows + 15) / 16;
        a.tiled = q.tiled;
        a.w_scale = q.W->scale;
        a.row_scale = q.row_scale;
        if (a.rows > max_rows) max_rows = a.rows;
    }
    const bool stats = d[0].part_max != nullptr;
    // K-resident blocks: every product with rows of at most 1024 bytes, plain output, no taps
    bool resident = !stats && n > 8;
    int max_ld = 0;
    for (int t = 0; t < njobs; ++t) {
        const GemmArgs &a = jobs.j[t];
        if (a.ld > 1024 || a.tap_acc || a.tiled || (size_t)a.ntiles * 16 * a.ld >= (1u << 31) || (size_t)n * a.ld >= (1u << 31)) resident = false;
        if (a.ld > max_ld) max_ld = a.ld;
    }
    if (resident) {
        const dim3 grid((max_rows + 63) / 64, (n + 63) / 64, njobs);
        static bool attr_set[2] = {false, false};
        const int which = max_ld <= 512 ? 0 : 1;
        const size_t smem = (size_t)64 * (which == 0 ? 64 * 8 + 16 : 64 * 16 + 16);
        if (!attr_set[which]) {
            const hipError_t e = which == 0
                ? hipFuncSetAttribute((const void *)gemm_resident_kernel<8>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem)
                : hipFuncSetAttribute((const void *)gemm_resident_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return q8_fail(ctx, Q8_ERR_DEVICE, "resident product kernel: %s", hipGetErrorString(e));
            attr_set[which] = true;
        }
        if (which == 0) Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, gemm_resident_kernel<8>, grid, dim3(256), smem, jobs);
        else Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, gemm_resident_kernel<16>, grid, dim3(256), smem, jobs);
        return q8i_launch_check(ctx, "gemm");
    }
    if (max_rows > 8192) {
        const dim3 grid((max_rows + 64 * GB_BIG_RT - 1) / (64 * GB_BIG_RT), (n + 16 * GB_BIG_NT - 1) / (16 * GB_BIG_NT), njobs);
        if (stats) Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, (gemm_block_kernel<GB_BIG_RT, GB_BIG_NT, true>), grid, dim3(256), 0, jobs);
        else Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, (gemm_block_kernel<GB_BIG_RT, GB_BIG_NT, false>), grid, dim3(256), 0, jobs);
    } else {
        const dim3 grid((max_rows + 64 * GB_SMALL_RT - 1) / (64 * GB_SMALL_RT), (n + 16 * GB_SMALL_NT - 1) / (16 * GB_SMALL_NT), njobs);
        if (stats) Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, (gemm_block_kernel<GB_SMALL_RT, GB_SMALL_NT, true>), grid, dim3(256), 0, jobs);
        else Q8_LAUNCH(ctx, Q8_KERNEL_MFMA, (gemm_block_kernel<GB_SMALL_RT, GB_SMALL_NT, false>), grid, dim3(256), 0, jobs);
    }
    return q8i_launch_check(ctx, "gemm");
}

q8_status q8i_gemm_mfma(q8_ctx *ctx, const q8_mat *W, const float *X, int n, int ldx, const float *bias, float *Y,
                        int ldy, const q8_taps *taps, int8_t *xq, float *xscale, const float *row_scale)
{
    q8i_quant_job qj = {X, W->cols, ldx, W->ld, xq, xscale, taps};
    q8_status st = q8i_quantize_jobs(ctx, &qj, 1, n);
    if (st) return st;
    q8i_gemm_job gj = {W, xq, xscale, bias, Y, ldy, taps ? taps->acc : nullptr, nullptr, nullptr, 0, row_scale};
    return q8i_gemm_jobs(ctx, &gj, 1, n);
}
