// q8_output.hip -- second layer of the output network g of Eq. 2 ("Pieces of Eight: 8-bit
// Neural Machine Translation"): the vocabulary projection as Section 3's narrow product
// on the int8 matrix cores, fused with bias and log-sum-exp partials; a second kernel
// finishes the log-sum-exp and selects the k best entries of every hypothesis.
#include "q8_beam.h"

#include <hip/hip_ext.h>

// The vocabulary matrix (25.6 MB at V = 50000) is read with the non-temporal hint: every byte
// is used once per step, and not letting it displace the kernel's other streams (hidden
// vectors, bias, logits, statistics) in the caches measured 2 us per decoder step.
#define Q8_WLOAD(p) __builtin_nontemporal_load(p)

#define OUT_TILE 16                  // vocabulary rows per matrix-core tile = one selection group
#define OUT_SB 16                    // tiles per thread of the selection kernel (256 threads)
#ifndef OUT_BLOCKS
#define OUT_BLOCKS 512               // blocks of 4 waves; tile t belongs to block t % OUT_BLOCKS
#endif
#define OUT_MAX_TILES 4096           // 65536 vocabulary rows

// tiles[((t * ksteps + s) * 64 + lane) * 16 ..] = W[(16 t + lane % 16) * ld + 64 s + 16 * (lane / 16) ..], 16 bytes
__global__ __launch_bounds__(256) void pack_tiles_kernel(const int8_t *__restrict__ W, int rows, int ld,
                                                         int8_t *__restrict__ tiles, size_t chunks)
{
    const int ksteps = ld / 64;
    for (size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x; o < chunks; o += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(o & 63);
        const size_t blk = o >> 6;
        const int s = (int)(blk % ksteps);
        const size_t t = blk / ksteps;
        const size_t row = t * 16 + (lane & 15);
        v4i v = (v4i){0, 0, 0, 0};
        if (row < (size_t)rows) v = *(const v4i *)(W + row * ld + 64 * s + 16 * (lane >> 4));
        *(v4i *)(tiles + o * 16) = v;
    }
}

struct OutArgs {
    const int8_t *W;
    const int8_t *tiles;    // matrix-core streaming order, or NULL
    const float *T, *bias;
    float *logits;          // [n x ldl], always written
    float *part_max;        // [n x tiles]
    double *part_sum;       // [n x tiles]: sum of exp(logit - part_max)
    q8_taps taps;
    int V, K, ld, ldt, n, ldl, ntiles;
    float w_scale;
};

// One pass over W_out for all n <= 8 hypotheses.  Operand A of v_mfma_i32_16x16x64_i8 =
// 16 weight rows x 64 k (lane: row lane%16, 16 consecutive k at 16*(lane/16)), operand B =
// the quantized hidden vectors with the same k split; the result leaves rows
// 4*(lane/16)+r, r = 0..3, of hypothesis lane%16 in the lane.  Tiles of 16 rows are dealt
// round-robin to blocks and, within a block, to waves, so every CU streams the same
// number of bytes.  Work is cut into items of 16 rows x 512 k; two items are in flight
// per wave.  Each tile's (max, sum of exp) per hypothesis is reduced in registers.
// The hidden vectors of all hypotheses, quantized by ONE wave (rows of at most 1024
// columns): the wave loads every vector (KPL float4 per lane and vector), reduces max|x|
// without leaving the wave, and writes the codes and scales to LDS.  The streaming waves
// of the block meanwhile have their weight loads in flight and meet this wave at a barrier.
template <int KPL>
__device__ __forceinline__ void wave_quantize(const float *__restrict__ X, int n, int K, int ldx, int ld, int8_t *xq,
                                              float *s_scale, int lane)
{
    float4 v[8][KPL];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int t = 0; t < KPL; ++t) {
            const int k = (t * 64 + lane) * 4;
            v[j][t] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (j < n && k < K) v[j][t] = *(const float4 *)(X + (size_t)j * ldx + k);
        }
    float m[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        m[j] = 0.0f;
#pragma unroll
        for (int t = 0; t < KPL; ++t)
            m[j] = fmaxf(m[j], fmaxf(fmaxf(fabsf(v[j][t].x), fabsf(v[j][t].y)), fmaxf(fabsf(v[j][t].z), fabsf(v[j][t].w))));
    }
    wave_max_multi<8>(m);
    float mine = 0.0f;                       // lane j owns vector j's two divisions
#pragma unroll
    for (int j = 0; j < 8; ++j) mine = (lane == j) ? m[j] : mine;
    float scale, inv;
    q8_scale_of(mine, scale, inv);
    if (lane < 8) s_scale[lane] = scale;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (j < n) {
            const float invj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(inv), j));
#pragma unroll
            for (int t = 0; t < KPL; ++t) {
                const int k = (t * 64 + lane) * 4;
                if (k < ld) *(int *)(xq + (size_t)j * ld + k) = q8_pack4(v[j][t].x, v[j][t].y, v[j][t].z, v[j][t].w, invj);
            }
        }
    }
}

#define OUT_STREAM_WAVES 4

// QKPL = 0: four waves, all of them quantize and stream.  QKPL = 1, 2, 4: blocks of five waves,
// the fifth only quantizes (QKPL float4 per lane and vector; rows of at most 256 * QKPL columns).
template <int CH, bool PACKED, int QKPL>
__device__ __forceinline__ void out_logits_body(const OutArgs &a)
{
    constexpr bool QW = QKPL != 0;
    extern __shared__ __align__(16) int8_t smem[];
    __shared__ float s_scale[8];
    __shared__ float s_red[8 * 4];
    const int ld = a.ld, n = a.n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    // five-wave blocks only run rows of at most 512 bytes: one k chunk, no index divisions
    const int kchunks = QW ? 1 : (ld + 511) / 512;
    if (QW && wave == OUT_STREAM_WAVES) {
        // ahead of the streaming waves at instruction issue: its few loads then leave before their
        // many, and the block's barrier opens 1.4 us earlier (measured)
        __builtin_amdgcn_s_setprio(3);
        wave_quantize<QW ? QKPL : 1>(a.T, n, a.K, a.ldt, ld, smem, s_scale, lane);
        __syncthreads();
        if (blockIdx.x == 0) {
            if (a.taps.xq)
                for (int e = lane; e < n * a.K; e += 64) a.taps.xq[e] = smem[(e / a.K) * ld + e % a.K];
            if (a.taps.xscale && lane < n) a.taps.xscale[lane] = s_scale[lane];
        }
        return;
    }
    // tiles of this wave: blockIdx + (wave + 4 q) * gridDim, q = 0, 1, ...
    const int tstride = 4 * gridDim.x;
    const int tile0 = blockIdx.x + wave * gridDim.x;
    const int ntw = tile0 < a.ntiles ? (a.ntiles - tile0 + tstride - 1) / tstride : 0;
    const int items = ntw * kchunks;
    const bool bias_vec = (((uintptr_t)a.bias) & 15) == 0;

    XRegs<8, QW ? 1 : CH> xr;
    if (!QW) x_load<8, CH>(xr, a.T, n, a.K, a.ldt);

    auto load_item = [&](int it, v4i (&av)[8]) {
        const int q = it / kchunks, kc = it - q * kchunks;
        const int tile = tile0 + q * tstride;
        if (PACKED) {
            // one contiguous KiB per wave-wide load
            const int8_t *wp = a.tiles + ((size_t)tile * (ld >> 6) + kc * 8) * 1024 + lane * 16;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                av[s] = (v4i){0, 0, 0, 0};
                if (it < items && kc * 512 + 64 * s < ld) av[s] = Q8_WLOAD((const v4i *)(wp + 1024 * s));
            }
        } else {
            const int row = tile * OUT_TILE + i;
            const int8_t *wp = a.W + (size_t)row * ld + kc * 512 + 16 * g;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                av[s] = (v4i){0, 0, 0, 0};
                if (it < items && row < a.V && kc * 512 + 64 * s + 16 * g < ld) av[s] = Q8_WLOAD((const v4i *)(wp + 64 * s));
            }
        }
    };
    // wait for the hidden vectors alone, then put the whole weight stream (and the biases of
    // the wave's first two tiles) in flight; the reduction and packing below overlap it
    float xm[8];
    if (!QW) x_absmax<8, QW ? 1 : CH>(xr, xm);
    // bias of the four rows this lane finishes in the tile of item `it` (needed when the
    // tile's last k chunk is multiplied); rows past V read as zero
    auto load_bias = [&](int it) {
        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
        const int q = it / kchunks;
        const int row0 = (tile0 + q * tstride) * OUT_TILE + 4 * g;
        if (a.bias && it < items && i < n) {
            if (bias_vec && row0 + 3 < a.V) {
                b = *(const float4 *)(a.bias + row0);
            } else {
                if (row0 < a.V) b.x = a.bias[row0];
                if (row0 + 1 < a.V) b.y = a.bias[row0 + 1];
                if (row0 + 2 < a.V) b.z = a.bias[row0 + 2];
                if (row0 + 3 < a.V) b.w = a.bias[row0 + 3];
            }
        }
        return b;
    };
    v4i bufA[8], bufB[8];
    load_item(0, bufA);
    load_item(1, bufB);
    float4 bias_cur = load_bias(0), bias_nxt = load_bias(kchunks);   // this wave's first and second tile
    __builtin_amdgcn_sched_barrier(0);
    if (QW) __syncthreads();                 // the quantizing wave has filled smem and s_scale
    else x_finish_m<8, QW ? 1 : CH>(xr, xm, n, ld, smem, s_scale, s_red);
    if (!QW && blockIdx.x == 0) {
        if (a.taps.xq)
            for (int e = threadIdx.x; e < n * a.K; e += blockDim.x) a.taps.xq[e] = smem[(e / a.K) * ld + e % a.K];
        if (a.taps.xscale && threadIdx.x < n) a.taps.xscale[threadIdx.x] = s_scale[threadIdx.x];
    }
    const float cj = i < n ? a.w_scale * s_scale[i] : 0.0f;
    const int8_t *xb = smem + (size_t)i * ld + 16 * g;
    const bool vec_ok = ((a.ldl & 3) == 0) && (((uintptr_t)a.logits & 15) == 0);

    v4i acc = (v4i){0, 0, 0, 0};
    auto compute_item = [&](int it, const v4i (&av)[8]) {
        const int q = it / kchunks, kc = it - q * kchunks;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            v4i bv = (v4i){0, 0, 0, 0};
            if (i < n && kc * 512 + 64 * s + 16 * g < ld) bv = *(const v4i *)(xb + kc * 512 + 64 * s);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[s], bv, acc, 0, 0, 0);
        }
        if (kc != kchunks - 1) return;
        const int tile = tile0 + q * tstride;
        const int row0 = tile * OUT_TILE + 4 * g;
        float y[4];
        float m = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            y[r] = -INFINITY;
            if (i < n && row0 + r < a.V) {
                y[r] = (float)acc[r] * cj;
                if (a.bias) y[r] = y[r] + (r == 0 ? bias_cur.x : r == 1 ? bias_cur.y : r == 2 ? bias_cur.z : bias_cur.w);
                if (a.taps.acc) a.taps.acc[(size_t)i * a.V + row0 + r] = acc[r];
            }
            m = fmaxf(m, y[r]);
        }
        if (i < n) {
            if (vec_ok && row0 + 3 < a.V) {
                *(float4 *)(a.logits + (size_t)i * a.ldl + row0) = make_float4(y[0], y[1], y[2], y[3]);
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (row0 + r < a.V) a.logits[(size_t)i * a.ldl + row0 + r] = y[r];
            }
        }
        // (max, sum of exp) of the tile's 16 rows per hypothesis: lanes i, i+16, i+32, i+48
        m = fmaxf(m, __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(m), SWZ_XOR16)));
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        double sd = 0.0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (y[r] > -INFINITY) sd += (double)exp_le0(y[r] - m);
        sd += __shfl_xor(sd, 16, 64);
        sd += __shfl_xor(sd, 32, 64);
        if (i < n && g == 0) {
            a.part_max[(size_t)i * a.ntiles + tile] = m;
            a.part_sum[(size_t)i * a.ntiles + tile] = sd;
        }
        acc = (v4i){0, 0, 0, 0};
        bias_cur = bias_nxt;                       // tiles finish in order: q, q + 1, ...
        bias_nxt = load_bias((q + 2) * kchunks);
    };
    for (int it = 0; it < items; it += 2) {
        compute_item(it, bufA);
        load_item(it + 2, bufA);
        if (it + 1 < items) {
            compute_item(it + 1, bufB);
            load_item(it + 3, bufB);
        }
    }
}

template <int CH, bool PACKED>
__global__ __launch_bounds__(256) void out_logits_kernel(OutArgs a)
{
    out_logits_body<CH, PACKED, 0>(a);
}

// Five-wave blocks.  At most 128 registers per lane (four waves per SIMD): the fifth waves of
// two blocks land on the same SIMD, and with fewer waves per SIMD the second block of a CU
// could not start before the first block's fifth wave has left.
template <bool PACKED, int QKPL>
__global__ __launch_bounds__(320) __attribute__((amdgpu_waves_per_eu(4, 8))) void out_logits5_kernel(OutArgs a)
{
    out_logits_body<1, PACKED, QKPL>(a);
}

// The kernel for tile-packed matrices with rows of at most 64 KS bytes (KS = 8 or 10): one tile per wave, eight
// waves per block, two blocks per compute unit, so that all of the matrix is requested within
// the first microsecond and nothing loops.  Wave j < n requests hidden vector j first (its
// data comes back ahead of the weights, which every wave requests next), quantizes it alone
// (no exchange between waves) and leaves the codes in LDS; after the one barrier every wave
// holds the codes of all vectors as operand B in registers.  KPL float4 per lane and vector.
// RESIDENT: the matrix fits the L2 (32 MB over the eight XCDs; a block reads the same tiles every
// step and lands on the same XCD) and is read plainly, so that it stays there from one step to the
// next; the other matrices of the step are streamed past it.  A larger matrix is streamed itself.
template <int KPL, int KS, bool RESIDENT>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 8))) void out_logits8_kernel(OutArgs a)
{
    extern __shared__ __align__(16) int8_t smem[];     // [n x pitch] codes of the hidden vectors
    __shared__ float s_scale[8];
    const int ld = a.ld, n = a.n, pitch = ld + 16, ksteps = ld >> 6;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int tile = blockIdx.x + wave * gridDim.x;
    const bool have = tile < a.ntiles;

    // The block's barrier waits for the waves that quantize; the compute unit's sixteen waves share one
    // vector-memory queue, which takes about a microsecond to accept all their loads.  Raised priority
    // puts the quantizing waves' requests in first (measured: barrier reached 0.25 us earlier).
    if (wave < n) __builtin_amdgcn_s_setprio(3);
    const __amdgpu_buffer_rsrc_t rT = q8_rsrc(a.T, ((size_t)(n - 1) * a.ldt + a.K) * sizeof(float));
    float4 tv[KPL];
#pragma unroll
    for (int t = 0; t < KPL; ++t) tv[t] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (wave < n) {                              // (the other waves would only add requests that fetch nothing to the queue)
#pragma unroll
        for (int t = 0; t < KPL; ++t) {
            const int k = (t * 64 + lane) * 4;
            const unsigned off = (k < a.K) ? (unsigned)(wave * a.ldt + k) * 4u : Q8_OOB;
            tv[t] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rT, (int)off, 0, 0));
        }
    }
    // the tile: up to KS wave-wide loads of one contiguous KiB each
    const __amdgpu_buffer_rsrc_t rW = q8_rsrc(a.tiles, (size_t)a.ntiles * ld * OUT_TILE);
    const unsigned woff = have ? (unsigned)tile * (unsigned)(ld * OUT_TILE) + lane * 16u : Q8_OOB;
    v4i av[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const unsigned off = s < ksteps ? woff + 1024u * s : Q8_OOB;
        av[s] = RESIDENT ? __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rW, (int)off, 0, 0))
                         : __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rW, (int)off, 0, 2));
    }
    // bias of the four rows this lane finishes
    const int row0 = tile * OUT_TILE + 4 * g;
    const __amdgpu_buffer_rsrc_t rB = q8_rsrc(a.bias, a.bias ? (size_t)a.V * sizeof(float) : 0);
    float bias[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const unsigned off = (have && i < n) ? (unsigned)(row0 + r) * 4u : Q8_OOB;
        bias[r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rB, (int)off, 0, 0));
    }
    __builtin_amdgcn_sched_barrier(0);

    if (wave < n) {
        float m = 0.0f;
#pragma unroll
        for (int t = 0; t < KPL; ++t)
            m = fmaxf(m, fmaxf(fmaxf(fabsf(tv[t].x), fabsf(tv[t].y)), fmaxf(fabsf(tv[t].z), fabsf(tv[t].w))));
        m = wave_max_f(m);
        float scale, inv;
        q8_scale_of(m, scale, inv);
#pragma unroll
        for (int t = 0; t < KPL; ++t) {
            const int k = (t * 64 + lane) * 4;         // values beyond K are zero, so the pad bytes come out zero
            if (k < ld) *(int *)(smem + (size_t)wave * pitch + k) = q8_pack4(tv[t].x, tv[t].y, tv[t].z, tv[t].w, inv);
        }
        if (lane == 0) s_scale[wave] = scale;
        __builtin_amdgcn_s_setprio(0);
    }
    __syncthreads();
    if (blockIdx.x == 0) {
        if (a.taps.xq)
            for (int e = threadIdx.x; e < n * a.K; e += blockDim.x) a.taps.xq[e] = smem[(e / a.K) * pitch + e % a.K];
        if (a.taps.xscale && threadIdx.x < n) a.taps.xscale[threadIdx.x] = s_scale[threadIdx.x];
    }
    if (!have) return;

    // operand B: hypothesis i's codes, k = 64 s + 16 g ..
    v4i bv[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        bv[s] = (v4i){0, 0, 0, 0};
        if (i < n && s < ksteps) bv[s] = *(const v4i *)(smem + (size_t)i * pitch + 64 * s + 16 * g);
    }
    const float cj = i < n ? a.w_scale * s_scale[i] : 0.0f;
    v4i acc0 = (v4i){0, 0, 0, 0}, acc1 = (v4i){0, 0, 0, 0};     // two chains: a dependent matrix-core op waits twice as long
#pragma unroll
    for (int s = 0; s < KS; s += 2) {
        acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[s], bv[s], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[s + 1], bv[s + 1], acc1, 0, 0, 0);
    }
    const v4i acc = acc0 + acc1;

    float y[4];
    float m = -INFINITY;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        y[r] = -INFINITY;
        if (i < n && row0 + r < a.V) {
            y[r] = (float)acc[r] * cj;
            if (a.bias) y[r] = y[r] + bias[r];
            if (a.taps.acc) a.taps.acc[(size_t)i * a.V + row0 + r] = acc[r];
        }
        m = fmaxf(m, y[r]);
    }
    if (i < n) {
        const bool vec_ok = ((a.ldl & 3) == 0) && (((uintptr_t)a.logits & 15) == 0);
        if (vec_ok && row0 + 3 < a.V) {
            *(float4 *)(a.logits + (size_t)i * a.ldl + row0) = make_float4(y[0], y[1], y[2], y[3]);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (row0 + r < a.V) a.logits[(size_t)i * a.ldl + row0 + r] = y[r];
        }
    }
    // (max, sum of exp) of the tile's 16 rows per hypothesis: lanes i, i + 16, i + 32, i + 48
    m = quad_rows_max(m);
    double sd = 0.0;
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (y[r] > -INFINITY) sd += (double)exp_le0(y[r] - m);
    sd = quad_rows_sum(sd);
    if (i < n && g == 0) {
        a.part_max[(size_t)i * a.ntiles + tile] = m;
        a.part_sum[(size_t)i * a.ntiles + tile] = sd;
    }
}

struct SelectArgs {
    const float *part_max;
    const double *part_sum;
    const float *logits;
    float *lse, *topk_logp;
    int *topk_idx;
    int ntiles, n, k, V, ldl;
    int tiled;              // logits kept as [ntiles][n][16] instead of [n][ldl]
    int normalized;         // the "logits" are log-probabilities already: nothing is subtracted
    int fuse_update;        // 1: block 0 also runs the beam update, once every block's k best are there
    // for that: n k 8-byte words, one per top-k entry (bit 63 "present", token id, log-probability), zero on
    // entry and on exit; the flag a wait that gave up sets; the bound of the wait in polls
    unsigned long long *xw;
    unsigned *wait_err;
    int spin_limit;
    BeamUpdateArgs bu;
    // with bu.xg: blocks n .. n + bu.gate_blocks - 1 compute s' of the next step (Eq. 3) once block 0 has decided
    const float *gx_table, *gh_r;
    float *s_mid_next;
    int gate_pause;         // short sleeps before the first poll for the decision
};

#define SEL_CAP 2048
#define SEL_GATE_BLOCKS_MAX 64

// GRU r of the next decoder step (Eq. 3) ahead of its launch.  Its two products do not wait for the search
// step's decision: W_x^r q(y) + b_x depends on the token alone (a table over the vocabulary, gx_table), and
// W_h^r q(s) + b_h of every state of this step was computed in the readout's launch (gh_r).  What is left, the
// gates of slot q from row token[q] of the one and row parent[q] of the other, is done here, by blocks of the
// selection kernel that wait for the decision: block 0 publishes it as tagged words, eight per gate block,
// and each block clears its own.  The wait is bounded; a block that gives up sets wait_err and goes on with
// indices kept inside the tables.
__device__ __forceinline__ void ahead_gates_block(const SelectArgs &a)
{
    __shared__ int s_par[Q8_MAX_BEAM], s_tok[Q8_MAX_BEAM];
    const int gb = blockIdx.x - a.n, tid = threadIdx.x, n = a.n, H = a.bu.H;
    if (tid < 64) {
        unsigned long long *xg = a.bu.xg + gb * Q8_MAX_BEAM;
        // (polls that come long before the decision only disturb the blocks that work towards it)
        for (int i = 0; i < a.gate_pause; ++i) __builtin_amdgcn_s_sleep(16);
        const int q = min(tid, n - 1);
        unsigned long long x = 0ull;
        bool ok = false;
        for (int spin = 0; spin < a.spin_limit; ++spin) {
            x = __hip_atomic_load(xg + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (__all((x >> 63) != 0ull)) { ok = true; break; }
            __builtin_amdgcn_s_sleep(4);
        }
        if (!ok && tid == 0) __hip_atomic_store(a.wait_err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (tid < n) {
            const int par = (int)((x >> 32) & 0xFull), tok = (int)(x & 0xFFFFFFull);
            s_par[tid] = par < n ? par : 0;
            s_tok[tid] = tok < a.V ? tok : 0;
            xg[tid] = 0ull;
        }
    }
    __syncthreads();
    for (int e = gb * 256 + tid; e < n * H; e += a.bu.gate_blocks * 256) {
        const int q = e / H, u = e - q * H;
        const float *x = a.gx_table + (size_t)s_tok[q] * 3 * H + u, *h = a.gh_r + (size_t)s_par[q] * 3 * H + u;
        const float xv[3] = {x[0], x[H], x[2 * H]}, hv[3] = {h[0], h[H], h[2 * H]};
        a.s_mid_next[(size_t)q * H + u] = gru_gates(xv, hv, a.bu.s_step[(size_t)s_par[q] * H + u]);
    }
}
          // survivors held in LDS

// One block of 256 threads per hypothesis; thread t owns tiles t, t + 256, ... (up to 16).
// (1) log-sum-exp from the tile partials.  (2) Each wave sorts its 64 threads' maxima; the
// wave's k-th largest has at least k logits at or above it, and T is the largest of the four
// such values: at least k logits are >= T, so each of the k best logits is >= T and lies in
// a tile whose maximum is >= T.  (3) Those tiles are read back, logits >= T
// collected (a few dozen unless many logits tie) and ranked by (value descending, index
// ascending).  If ties overflow the survivor list, k exact rounds of arg-max over the
// whole row run instead.  The k results are collected in LDS (a rank that found no candidate,
// which takes non-finite logits, keeps an entry of token 0 with log-probability -inf) and stored
// by k threads.
// With the search step fused in, every block also publishes its k entries as tagged 8-byte words
// with device-coherent stores and is done; block 0 polls the n k words (two per lane of one wave),
// clears them for the next launch (it is their only reader) and goes on with the values in
// registers: one store and a poll between "ranked" and "keys formed", where a count of arrivals
// (stores performed, atomic, the last block reading the tables back) took 1.7 us.
__global__ __launch_bounds__(256) void out_select_kernel(SelectArgs a)
{
    __shared__ unsigned short s_q[OUT_MAX_TILES];
    __shared__ __align__(16) unsigned long long s_key[SEL_CAP + 4];
    __shared__ float s_f[4];
    __shared__ double s_d[4];
    __shared__ unsigned long long s_u[4];
    __shared__ float s_t4[4];
    __shared__ int s_nq, s_ns;
    __shared__ unsigned long long s_top[16];
    const int j = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = a.n, k = a.k;
    const int ntiles = a.ntiles;
    if (j >= n) { ahead_gates_block(a); return; }
    if (tid == 0) { s_nq = 0; s_ns = 0; }
    if (tid < 16) s_top[tid] = topk_key(-INFINITY, 0);

    float pm[OUT_SB];
    double ps[OUT_SB];
#pragma unroll
    for (int t = 0; t < OUT_SB; ++t) {
        const int tile = tid + 256 * t;            // consecutive threads, consecutive tiles
        pm[t] = -INFINITY;
        ps[t] = 0.0;
        if (tile < ntiles) {
            pm[t] = a.part_max[(size_t)j * ntiles + tile];
            ps[t] = a.part_sum[(size_t)j * ntiles + tile];
        }
    }
    float bm = -INFINITY;
#pragma unroll
    for (int t = 0; t < OUT_SB; ++t) bm = fmaxf(bm, pm[t]);
    // the wave's maxima in descending order: lane 0 holds the largest, lane k - 1 the k-th
    const float sorted = wave_sort_desc_f(bm, lane);
    if (lane == 0) s_f[wave] = sorted;
    if (lane == k - 1) s_t4[wave] = sorted;       // -inf if the wave has fewer than k non-empty threads
    __syncthreads();
    const float m = fmaxf(fmaxf(s_f[0], s_f[1]), fmaxf(s_f[2], s_f[3]));
    const float T = fmaxf(fmaxf(s_t4[0], s_t4[1]), fmaxf(s_t4[2], s_t4[3]));   // -inf: everything qualifies

    // ---- tiles that can hold a logit >= T
#pragma unroll
    for (int t = 0; t < OUT_SB; ++t)
        if (tid + 256 * t < ntiles && pm[t] >= T) s_q[atomicAdd(&s_nq, 1)] = (unsigned short)(tid + 256 * t);
    __syncthreads();
    const int total = s_nq * OUT_TILE;
    // logit of vocabulary row r of this hypothesis, in either layout
    const float *lg = a.tiled ? a.logits + (size_t)j * OUT_TILE : a.logits + (size_t)j * a.ldl;
    const size_t tile_pitch = a.tiled ? (size_t)a.n * OUT_TILE - OUT_TILE : 0;     // extra floats per tile boundary
    auto logit = [&](int r) { return lg[(size_t)r + (size_t)(r / OUT_TILE) * tile_pitch]; };
    // The first 1024 logits of those tiles are requested now, without branches (an entry past the end
    // reads some valid row and is dropped), and the log-sum-exp is summed while they are on their way.
    float v0[4];
    int row0[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int c = tid + 256 * t, cc = min(c, max(total, 1) - 1);
        const int r = (int)s_q[cc / OUT_TILE] * OUT_TILE + cc % OUT_TILE;
        row0[t] = (c < total && r < a.V) ? r : -1;
        v0[t] = logit(min(r, a.V - 1));
    }
    // ---- log-sum-exp (1): this wave's share of the sum
    double S = 0.0;
#pragma unroll
    for (int t = 0; t < OUT_SB; ++t)
        if (pm[t] > -INFINITY) S += ps[t] * (double)exp_le0(pm[t] - m);
    S = wave_sum_d(S);
    if (lane == 0) s_d[wave] = S;
    // ---- logits >= T of the qualifying tiles
    bool overflow = total > 16 * SEL_CAP;
    if (!overflow) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (row0[t] >= 0 && v0[t] >= T) {
                const int pos = atomicAdd(&s_ns, 1);
                if (pos < SEL_CAP) s_key[pos] = topk_key(v0[t], row0[t]);
            }
        for (int c0 = tid + 1024; c0 < total; c0 += 1024) {
            float v[4];
            int row[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int c = c0 + 256 * t;
                row[t] = -1;
                v[t] = -INFINITY;
                if (c < total) {
                    const int r = (int)s_q[c / OUT_TILE] * OUT_TILE + c % OUT_TILE;
                    if (r < a.V) { row[t] = r; v[t] = logit(r); }
                }
            }
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (row[t] >= 0 && v[t] >= T) {
                    const int pos = atomicAdd(&s_ns, 1);
                    if (pos < SEL_CAP) s_key[pos] = topk_key(v[t], row[t]);
                }
        }
    }
    __syncthreads();
    overflow = overflow || s_ns > SEL_CAP;
    // ---- log-sum-exp (2)
    S = (s_d[0] + s_d[1]) + (s_d[2] + s_d[3]);
    const float lse = a.normalized ? 0.0f : (float)((double)m + log(S));
    if (tid == 0 && a.lse) a.lse[j] = lse;

    if (!overflow) {
        // rank every survivor among the survivors; ranks below k are the answer
        const int ns = s_ns;
        if (tid < 4) s_key[ns + tid] = 0ull;     // pad to a multiple of four with keys that are never greater
        __syncthreads();
        for (int t = tid; t < ns; t += 256) {
            const unsigned long long key = s_key[t];
            int rank = 0;
#pragma unroll 2
            for (int u = 0; u < ns; u += 4) {
                const ulonglong2 p0 = *(const ulonglong2 *)&s_key[u], p1 = *(const ulonglong2 *)&s_key[u + 2];
                rank += (p0.x > key) + (p0.y > key) + (p1.x > key) + (p1.y > key);
            }
            if (rank < k) s_top[rank] = key;
        }
    } else {
    // ---- heavily tied logits: k exact rounds of arg-max over the whole row
    unsigned long long prev = ~0ull;
    for (int r = 0; r < k; ++r) {
        unsigned long long best = 0ull;
        for (int row = tid; row < a.V; row += 256) {
            const unsigned long long key = topk_key(logit(row), row);
            if (key < prev && key > best) best = key;
        }
        best = wave_max_u64(best);
        __syncthreads();
        if (lane == 0) s_u[wave] = best;
        __syncthreads();
        best = s_u[0];
#pragma unroll
        for (int w = 1; w < 4; ++w) best = s_u[w] > best ? s_u[w] : best;
        if (tid == 0) s_top[r] = best;
        prev = best;
    }
    }
    __syncthreads();
    if (tid < k) {
        const unsigned long long key = s_top[tid];
        // (a round of the exact fallback that finds no candidate decodes to an index past the table;
        // whoever gathers an embedding row by it must find a row)
        int idx = topk_key_idx(key);
        idx = (unsigned)idx < (unsigned)a.V ? idx : 0;
        const float logp = topk_key_val(key) - lse;
        const size_t o = (size_t)j * k + tid;
        a.topk_idx[o] = idx;
        a.topk_logp[o] = logp;
        if (a.fuse_update)
            __hip_atomic_store(a.xw + o, (1ull << 63) | ((unsigned long long)(unsigned)idx << 32) | __float_as_uint(logp),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    if (!a.fuse_update || j != 0) return;
    // ---- block 0 continues with the search step once all n k entries are there
    float lp[2] = {0.0f, 0.0f};
    int tk[2] = {0, 0};
    BeamStateRead sr = {};
    if (tid < 64) {
        sr = beam_state_read(a.bu.st, lane);       // (on its way while the candidates are waited for)
        const int nk = n * k;                      // at most 128
        const int c0 = min(lane, nk - 1), c1 = min(lane + 64, nk - 1);
        unsigned long long x0 = 0ull, x1 = 0ull;
        bool ok = false;
        for (int spin = 0; spin < a.spin_limit; ++spin) {
            x0 = __hip_atomic_load(a.xw + c0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            x1 = __hip_atomic_load(a.xw + c1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (__all((x0 >> 63) != 0ull && (x1 >> 63) != 0ull)) { ok = true; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        if (!ok && lane == 0) __hip_atomic_store(a.wait_err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lp[0] = __uint_as_float((unsigned)x0); tk[0] = (int)((x0 >> 32) & 0x7fffffffull);
        lp[1] = __uint_as_float((unsigned)x1); tk[1] = (int)((x1 >> 32) & 0x7fffffffull);
        if (lane < nk) a.xw[lane] = 0ull;
        if (lane + 64 < nk) a.xw[lane + 64] = 0ull;
    }
    beam_update_body<true>(a.bu, lp, tk, sr);
}

// ========================================== selection for panels, logits recomputed ==
// Many hypothesis slots (sentences side by side): the vocabulary panel kernel keeps no logits
// (at 320 slots they would be 64 MB per step, written once and almost never read), only each
// tile's (max, sum of exp).  This kernel, one block per slot, derives the log-sum-exp and the
// threshold T from those, and computes the logits of the few tiles whose maximum reaches T a
// second time: the same matrix-core instruction on the same tile-packed weights with the
// slot's codes in column 0 of the second operand, so the int32 sums, and with the same
// dequantization and bias steps the logits, are those the panel kernel saw.
struct PanelSelectArgs {
    const float *part_max;
    const double *part_sum;
    const int8_t *tiles;    // tile-packed weights (q8_pack_tiles)
    const int8_t *xq;       // [n x 64 KC] codes of t
    const float *xscale, *bias;
    float *lse, *topk_logp;
    int *topk_idx;
    int ntiles, n, k, V;
    float w_scale;
    // FUSE: the search steps of the sentences run in this launch (see the kernel); xw: n k 8-byte words, zero
    // on entry and on exit; the flag a wait that gave up sets; the bound of the wait in polls
    unsigned long long *xw;
    unsigned *wait_err;
    int spin_limit;
    BeamBatchArgs bb;
};

#define PSEL_BATCH 4          // tiles per wave whose weights are requested together

// FUSE: the search step of every sentence runs here too, as in out_select_kernel: each block publishes its
// k entries as tagged 8-byte words (present bit, token id, log-probability) with device-coherent stores; the
// block of a sentence's last slot polls the beam k words of its sentence (two per lane of one wave), clears
// them (it is their only reader) and runs the sentence's search step with the candidates in registers.  The
// blocks it waits for have lower indices and were dispatched before it, so the wait ends whatever the
// device holds at once; it is bounded all the same, and a wait that gives up sets wait_err.
template <int KC, bool FUSE>
__global__ __launch_bounds__(256) void panel_select_kernel(PanelSelectArgs a)
{
    __shared__ unsigned long long s_best[16];
    __shared__ unsigned short s_q[OUT_MAX_TILES];
    __shared__ __align__(16) unsigned long long s_key[SEL_CAP + 4];
    __shared__ float s_f[4];
    __shared__ double s_d[4];
    __shared__ unsigned long long s_u[4];
    __shared__ float s_top[64];
    __shared__ float s_T;
    __shared__ int s_nq, s_ns;
    constexpr int ld = 64 * KC;
    const int j = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, k = a.k;
    const int i = lane & 15, g = lane >> 4;
    const int ntiles = a.ntiles;
    if (tid == 0) { s_nq = 0; s_ns = 0; }
    if (tid < 64) s_top[tid] = -INFINITY;
    if (FUSE && tid < 16) s_best[tid] = topk_key(-INFINITY, 0);

    // the slot's codes as second operand: column 0 carries them, columns 1..15 are zero
    v4i bv[KC];
    {
        const int8_t *xj = a.xq + (size_t)j * ld + 16 * g;
#pragma unroll
        for (int s = 0; s < KC; ++s) bv[s] = i == 0 ? *(const v4i *)(xj + 64 * s) : (v4i){0, 0, 0, 0};
    }
    const float c = a.w_scale * a.xscale[j];

    float pm[OUT_SB];
    double ps[OUT_SB];
#pragma unroll
    for (int t = 0; t < OUT_SB; ++t) {
        const int tile = tid + 256 * t;
        pm[t] = -INFINITY;
        ps[t] = 0.0;
        if (tile < ntiles) {
            pm[t] = a.part_max[(size_t)j * ntiles + tile];
            ps[t] = a.part_sum[(size_t)j * ntiles + tile];
        }
    }
    float bm = -INFINITY;
#pragma unroll
    for (int t = 0; t < OUT_SB; ++t) bm = fmaxf(bm, pm[t]);
    // T = the k-th largest of the 256 threads' maxima (each the largest logit of up to 16 tiles of
    // its own, so at least k logits are >= T): every wave sorts its 64, the k best of each wave are
    // sorted once more.  k <= 16 (four waves' candidates fill one wave).
    __syncthreads();
    const float sorted = wave_sort_desc_f(bm, lane);
    if (lane == 0) s_f[wave] = sorted;
    if (lane < 16) s_top[16 * wave + lane] = lane < k ? sorted : -INFINITY;
    __syncthreads();
    const float m = fmaxf(fmaxf(s_f[0], s_f[1]), fmaxf(s_f[2], s_f[3]));
    if (wave == 0) {
        const float again = wave_sort_desc_f(s_top[lane], lane);
        if (lane == k - 1) s_T = again;              // -inf if fewer than k threads own a tile: everything qualifies
    }
    __syncthreads();
    const float T = s_T;

#pragma unroll
    for (int t = 0; t < OUT_SB; ++t)
        if (tid + 256 * t < ntiles && pm[t] >= T) s_q[atomicAdd(&s_nq, 1)] = (unsigned short)(tid + 256 * t);
    __syncthreads();
    const int nq = s_nq;

    // logits of tile `tile` for this slot: lanes 0, 16, 32, 48 (column 0) end up with rows 4 g .. 4 g + 3
    auto tile_loads = [&](v4i (&A)[KC], int tile) {
        const int8_t *p = a.tiles + (size_t)tile * KC * 1024 + lane * 16;
#pragma unroll
        for (int s = 0; s < KC; ++s) A[s] = *(const v4i *)(p + 1024 * s);
    };
    // (the biases of the lane's four rows are requested with the tile, not after the products)
    // (unconditional loads: without biases the slot's scale is read instead and not used)
    const float *bias_p = a.bias ? a.bias : a.xscale + j;
    const int bias_last = a.bias ? a.V - 1 : 0;
    auto tile_bias = [&](float (&bb)[4], int tile) {
#pragma unroll
        for (int r = 0; r < 4; ++r) bb[r] = bias_p[min(tile * OUT_TILE + 4 * g + r, bias_last)];
    };
    auto tile_logits = [&](const v4i (&A)[KC], const float (&bb)[4], int tile, float (&y)[4]) {
        v4i acc = (v4i){0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KC; ++s) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[s], bv[s], acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = tile * OUT_TILE + 4 * g + r;
            y[r] = -INFINITY;
            if (row < a.V) {
                y[r] = (float)acc[r] * c;
                if (a.bias) y[r] = y[r] + bb[r];
            }
        }
    };

    // this wave's share of the log-sum-exp from the tile partials
    auto lse_share = [&]() {
        double S = 0.0;
#pragma unroll
        for (int t = 0; t < OUT_SB; ++t)
            if (pm[t] > -INFINITY) S += ps[t] * (double)exp_le0(pm[t] - m);
        S = wave_sum_d(S);
        if (lane == 0) s_d[wave] = S;
    };
    lse_share();
    bool overflow = nq * OUT_TILE > 16 * SEL_CAP;
    if (!overflow) {
        for (int q0 = 0; q0 < nq; q0 += 4 * PSEL_BATCH) {
            v4i A[PSEL_BATCH][KC];
            float bb[PSEL_BATCH][4];
            int tile[PSEL_BATCH];
#pragma unroll
            for (int u = 0; u < PSEL_BATCH; ++u) {
                const int q = q0 + 4 * u + wave;
                tile[u] = q < nq ? (int)s_q[q] : -1;
                tile_loads(A[u], tile[u] < 0 ? 0 : tile[u]);         // a slot past the list reads tile 0 and drops it
                tile_bias(bb[u], tile[u] < 0 ? 0 : tile[u]);
            }
#pragma unroll
            for (int u = 0; u < PSEL_BATCH; ++u) {
                float y[4];
                tile_logits(A[u], bb[u], tile[u] < 0 ? 0 : tile[u], y);
                if (tile[u] >= 0 && i == 0) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (y[r] >= T) {                             // -inf (a row past the matrix) only if T is -inf too
                            const int row = tile[u] * OUT_TILE + 4 * g + r;
                            if (row < a.V) {
                                const int pos = atomicAdd(&s_ns, 1);
                                if (pos < SEL_CAP) s_key[pos] = topk_key(y[r], row);
                            }
                        }
                }
            }
        }
    }
    __syncthreads();
    overflow = overflow || s_ns > SEL_CAP;
    const double S = (s_d[0] + s_d[1]) + (s_d[2] + s_d[3]);
    const float lse = (float)((double)m + log(S));
    if (tid == 0 && a.lse) a.lse[j] = lse;

    if (!overflow) {
        const int ns = s_ns;
        if (tid < 4) s_key[ns + tid] = 0ull;
        __syncthreads();
        for (int t = tid; t < ns; t += 256) {
            const unsigned long long key = s_key[t];
            int rank = 0;
#pragma unroll 2
            for (int u = 0; u < ns; u += 4) {
                const ulonglong2 p0 = *(const ulonglong2 *)&s_key[u], p1 = *(const ulonglong2 *)&s_key[u + 2];
                rank += (p0.x > key) + (p0.y > key) + (p1.x > key) + (p1.y > key);
            }
            if (rank < k) {
                if (FUSE) {
                    s_best[rank] = key;
                } else {
                    a.topk_idx[(size_t)j * k + rank] = topk_key_idx(key);
                    a.topk_logp[(size_t)j * k + rank] = topk_key_val(key) - lse;
                }
            }
        }
        if (!FUSE) return;
    } else {
    // heavily tied logits (more than SEL_CAP at or above T): k exact rounds of arg-max over every tile
    unsigned long long prev = ~0ull;
    for (int r = 0; r < k; ++r) {
        unsigned long long best = 0ull;
        for (int tile = wave; tile < ntiles; tile += 4) {
            v4i A[KC];
            float y[4], bb[4];
            tile_loads(A, tile);
            tile_bias(bb, tile);
            tile_logits(A, bb, tile, y);
            if (i == 0) {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int row = tile * OUT_TILE + 4 * g + rr;
                    if (row < a.V) {
                        const unsigned long long key = topk_key(y[rr], row);
                        if (key < prev && key > best) best = key;
                    }
                }
            }
        }
        best = wave_max_u64(best);
        __syncthreads();
        if (lane == 0) s_u[wave] = best;
        __syncthreads();
        best = s_u[0];
#pragma unroll
        for (int w = 1; w < 4; ++w) best = s_u[w] > best ? s_u[w] : best;
        if (tid == 0) {
            const int idx = topk_key_idx(best);              // past the table if the round found no candidate (non-finite logits)
            if (FUSE) {
                s_best[r] = best;
            } else {
                a.topk_idx[(size_t)j * k + r] = (unsigned)idx < (unsigned)a.V ? idx : 0;
                a.topk_logp[(size_t)j * k + r] = topk_key_val(best) - lse;
            }
        }
        prev = best;
    }
    }
    if (!FUSE) return;
    // ---- the k entries: stored, and published for the block that runs this sentence's search step
    __syncthreads();
    if (tid < k) {
        const unsigned long long key = s_best[tid];
        int idx = topk_key_idx(key);
        idx = (unsigned)idx < (unsigned)a.V ? idx : 0;       // (a rank without a candidate: token 0 at -inf)
        const float logp = topk_key_val(key) - lse;
        const size_t o = (size_t)j * k + tid;
        a.topk_idx[o] = idx;
        a.topk_logp[o] = logp;
        __hip_atomic_store(a.xw + o, (1ull << 63) | ((unsigned long long)(unsigned)idx << 32) | __float_as_uint(logp),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const int beam = a.bb.beam, sent = j / beam;
    if (j != sent * beam + beam - 1) return;
    const BeamUpdateArgs bu = beam_batch_sentence(a.bb, sent);
    float lp[2] = {0.0f, 0.0f};
    int tk[2] = {0, 0};
    BeamStateRead sr = {};
    if (tid < 64) {
        sr = beam_state_read(bu.st, lane);                   // (on its way while the candidates are waited for)
        const int nk = beam * k;                             // at most 128
        unsigned long long *xw = a.xw + (size_t)sent * nk;
        const int c0 = min(lane, nk - 1), c1 = min(lane + 64, nk - 1);
        unsigned long long x0 = 0ull, x1 = 0ull;
        bool ok = false;
        for (int spin = 0; spin < a.spin_limit; ++spin) {
            x0 = __hip_atomic_load(xw + c0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            x1 = __hip_atomic_load(xw + c1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (__all((x0 >> 63) != 0ull && (x1 >> 63) != 0ull)) { ok = true; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        if (!ok && lane == 0) __hip_atomic_store(a.wait_err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        lp[0] = __uint_as_float((unsigned)x0); tk[0] = (int)((x0 >> 32) & 0x7fffffffull);
        lp[1] = __uint_as_float((unsigned)x1); tk[1] = (int)((x1 >> 32) & 0x7fffffffull);
        if (lane < nk) xw[lane] = 0ull;
        if (lane + 64 < nk) xw[lane + 64] = 0ull;
    }
    beam_update_body<true>(bu, lp, tk, sr);
    __syncthreads();
    if (tid == 0) a.bb.done[sent] = bu.st->done;
}

// =================================================================== host launcher ==

int q8i_out_tiles(int V) { return (V + OUT_TILE - 1) / OUT_TILE; }
int q8i_out_max_rows(void) { return OUT_MAX_TILES * OUT_TILE; }

template <bool PACKED>
static void launch_out_packed(q8_ctx *ctx, const OutArgs &a, int nblk, size_t smem, int ch)
{
    if (ch == 1 && a.ld <= 256) Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits5_kernel<PACKED, 1>), dim3(nblk), dim3(320), smem, a);
    else if (ch == 1 && a.ld <= 512) Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits5_kernel<PACKED, 2>), dim3(nblk), dim3(320), smem, a);
    else if (ch == 1) Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits_kernel<1, PACKED>), dim3(nblk), dim3(256), smem, a);
    else if (ch == 2) Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits_kernel<2, PACKED>), dim3(nblk), dim3(256), smem, a);
    else Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits_kernel<4, PACKED>), dim3(nblk), dim3(256), smem, a);
}

size_t q8i_tiles_bytes(int rows, int ld) { return (size_t)q8i_out_tiles(rows) * OUT_TILE * (size_t)ld; }

q8_status q8i_pack_tiles(q8_ctx *ctx, const q8_mat *W, int8_t *tiles)
{
    const size_t chunks = q8i_tiles_bytes(W->rows, W->ld) / 16;
    int blocks = (int)((chunks + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(pack_tiles_kernel, dim3(blocks), dim3(256), 0, ctx->stream, W->data, W->rows, W->ld, tiles, chunks);
    return q8i_launch_check(ctx, "pack_tiles");
}

// Ensemble (Section 4): c[j, v] = log(mean over the models of exp(logits_m[j, v] - lse_m[j])), in
// double, rounded once; one thread per (hypothesis, 16-row tile) also leaves the tile's maximum
// and sum of exponentials for the selection kernel.
#define ENS_MAX_MODELS 4
struct CombineArgs {
    const float *logits[ENS_MAX_MODELS];
    const float *lse[ENS_MAX_MODELS];
    float *c, *part_max;
    double *part_sum;
    int M, n, V, ntiles;
};

__global__ __launch_bounds__(256) void ensemble_combine_kernel(CombineArgs a)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= a.n * a.ntiles) return;
    const int j = idx / a.ntiles, tile = idx - j * a.ntiles;
    const int r0 = tile * OUT_TILE, rows = min(OUT_TILE, a.V - r0);
    float ls[ENS_MAX_MODELS];
#pragma unroll
    for (int m = 0; m < ENS_MAX_MODELS; ++m) ls[m] = m < a.M ? a.lse[m][j] : 0.0f;
    const double inv_m = 1.0 / (double)a.M;
    float c[OUT_TILE], mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < OUT_TILE; ++r) {
        c[r] = -INFINITY;
        if (r < rows) {
            double p = 0.0;
#pragma unroll
            for (int m = 0; m < ENS_MAX_MODELS; ++m)
                if (m < a.M) {
                    const float lp = a.logits[m][(size_t)j * a.V + r0 + r] - ls[m];
                    p += q8_exp_d(fmax((double)lp, -700.0));
                }
            c[r] = (float)log(p * inv_m);
            a.c[(size_t)j * a.V + r0 + r] = c[r];
        }
        mx = fmaxf(mx, c[r]);
    }
    double sd = 0.0;
#pragma unroll
    for (int r = 0; r < OUT_TILE; ++r)
        if (r < rows) sd += (double)exp_le0(c[r] - mx);
    a.part_max[(size_t)j * a.ntiles + tile] = mx;
    a.part_sum[(size_t)j * a.ntiles + tile] = sd;
}

q8_status q8i_ensemble_combine(q8_ctx *ctx, const float *const *logits, const float *const *lse, int M, int n, int V,
                               float *c, float *part_max, double *part_sum)
{
    CombineArgs a;
    for (int m = 0; m < ENS_MAX_MODELS; ++m) {
        a.logits[m] = logits[m < M ? m : 0];
        a.lse[m] = lse[m < M ? m : 0];
    }
    a.c = c; a.part_max = part_max; a.part_sum = part_sum;
    a.M = M; a.n = n; a.V = V; a.ntiles = q8i_out_tiles(V);
    const int total = n * a.ntiles;
    hipLaunchKernelGGL(ensemble_combine_kernel, dim3((total + 255) / 256), dim3(256), 0, ctx->stream, a);
    return q8i_launch_check(ctx, "ensemble combine");
}

static q8_status launch_select(q8_ctx *ctx, const float *part_max, const double *part_sum, const float *logits, int tiled,
                               int V, int n, int k, float *lse, float *topk_logp, int32_t *topk_idx,
                               const q8i_beam_desc *beam, int normalized = 0)
{
    SelectArgs s;
    s.part_max = part_max; s.part_sum = part_sum; s.logits = logits;
    s.lse = lse; s.topk_logp = topk_logp; s.topk_idx = topk_idx;
    s.ntiles = q8i_out_tiles(V); s.n = n; s.k = k; s.V = V; s.ldl = V; s.tiled = tiled; s.normalized = normalized;
    s.fuse_update = beam ? 1 : 0;
    s.xw = (unsigned long long *)(ctx->ws + Q8_WS_SELECT_XCHG);
    s.wait_err = (unsigned *)(ctx->ws + Q8_WS_ATT_ERR);
    s.spin_limit = ctx->att_spin_limit;
    if (beam) {
        BeamUpdateArgs bu = {(BeamState *)beam->state, topk_logp, topk_idx, beam->s_step, beam->E_tgt, beam->y_emb,
                             beam->s_next, n, k, beam->E, beam->H, V};
        if (beam->Eq) {
            bu.Eq = beam->Eq; bu.Es = beam->Es; bu.sq_in = beam->sq_in; bu.ss_in = beam->ss_in;
            bu.yq_out = beam->yq_out; bu.ys_out = beam->ys_out; bu.sq_out = beam->sq_out; bu.ss_out = beam->ss_out;
            bu.ldy = beam->ldy; bu.lds = beam->lds;
        }
        s.bu = bu;
    } else {
        memset(&s.bu, 0, sizeof(s.bu));
    }
    int gate_blocks = 0;
    s.gx_table = nullptr; s.gh_r = nullptr; s.s_mid_next = nullptr; s.gate_pause = ctx->gate_pause;
    if (beam && beam->gx_table) {
        gate_blocks = (n * beam->H + 255) / 256;
        if (gate_blocks > SEL_GATE_BLOCKS_MAX) gate_blocks = SEL_GATE_BLOCKS_MAX;
        s.gx_table = beam->gx_table; s.gh_r = beam->gh_r; s.s_mid_next = beam->s_mid_next;
        s.bu.xg = (unsigned long long *)(ctx->ws + Q8_WS_GATES_XCHG);
        s.bu.gate_blocks = gate_blocks;
    }
    Q8_LAUNCH(ctx, Q8_KERNEL_SELECT, out_select_kernel, dim3(n + gate_blocks), dim3(256), 0, s);
    return q8i_launch_check(ctx, "output");
}

// Selection alone over values that are log-probabilities already (the ensemble's averaged
// distribution), row-major [n x V], with their tile statistics; optional fused beam update.
q8_status q8i_select_normalized(q8_ctx *ctx, const float *part_max, const double *part_sum, const float *c, int V, int n,
                                int k, float *topk_logp, int32_t *topk_idx, const q8i_beam_desc *beam)
{
    return launch_select(ctx, part_max, part_sum, c, 0, V, n, k, nullptr, topk_logp, topk_idx, beam, 1);
}

// Selection alone over stored row-major logits [n x V] and their tile statistics.
q8_status q8i_select_logits(q8_ctx *ctx, const float *part_max, const double *part_sum, const float *logits, int V, int n,
                            int k, float *lse, float *topk_logp, int32_t *topk_idx)
{
    return launch_select(ctx, part_max, part_sum, logits, 0, V, n, k, lse, topk_logp, topk_idx, nullptr, 0);
}

q8_status q8i_output(q8_ctx *ctx, const q8_mat *W, const float *bias, const float *T, int ldt, int n, int k,
                     float *logits, float *lse, float *topk_logp, int32_t *topk_idx, const q8_taps *taps,
                     float *part_max, double *part_sum, const q8i_beam_desc *beam)
{
    OutArgs a;
    a.W = W->data; a.tiles = (W->ld % 64 == 0) ? W->tiles : nullptr; a.T = T; a.bias = bias; a.logits = logits;
    a.part_max = part_max; a.part_sum = part_sum;
    q8_taps none = {nullptr, nullptr, nullptr};
    a.taps = taps ? *taps : none;
    a.V = W->rows; a.K = W->cols; a.ld = W->ld; a.ldt = ldt; a.n = n; a.ldl = W->rows;
    a.w_scale = W->scale;
    a.ntiles = q8i_out_tiles(a.V);
    const int nblk = a.ntiles < 4 * OUT_BLOCKS ? (a.ntiles + 3) / 4 : OUT_BLOCKS;
    const size_t smem = (size_t)n * a.ld;
    const int ch = q8_fast_ch(a.ld);
    if (a.tiles && a.ld <= 640) {
        // one tile per wave: a.ntiles <= OUT_MAX_TILES = 8 * OUT_BLOCKS
        // (at most 256 blocks' worth of tiles: one block per compute unit; more: two each, evenly filled)
        const int nblk8 = a.ntiles <= 8 * (OUT_BLOCKS / 2) ? (a.ntiles + 7) / 8 : OUT_BLOCKS;
        const size_t smem8 = (size_t)n * (a.ld + 16);
        const bool resident = (size_t)a.ntiles * OUT_TILE * a.ld <= ((size_t)27 << 20);
        if (a.ld > 512 && resident) Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits8_kernel<3, 10, true>), dim3(nblk8), dim3(512), smem8, a);
        else if (a.ld > 512) Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits8_kernel<3, 10, false>), dim3(nblk8), dim3(512), smem8, a);
        else if (a.K <= 256 && resident) Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits8_kernel<1, 8, true>), dim3(nblk8), dim3(512), smem8, a);
        else if (a.K <= 256) Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits8_kernel<1, 8, false>), dim3(nblk8), dim3(512), smem8, a);
        else if (resident) Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits8_kernel<2, 8, true>), dim3(nblk8), dim3(512), smem8, a);
        else Q8_LAUNCH(ctx, Q8_KERNEL_VOCAB, (out_logits8_kernel<2, 8, false>), dim3(nblk8), dim3(512), smem8, a);
    } else if (a.tiles) {
        launch_out_packed<true>(ctx, a, nblk, smem, ch);
    } else {
        launch_out_packed<false>(ctx, a, nblk, smem, ch);
    }
    return launch_select(ctx, part_max, part_sum, logits, 0, a.V, n, k, lse, topk_logp, topk_idx, beam);
}

// Whether q8i_output_codes, asked for tiled logits and no taps, runs the panel kernel and keeps no logits.
bool q8i_output_codes_keeps_no_logits(const q8_mat *W, int k) { return q8i_vocab_panel_ok(W) && k <= 16; }

// Vocabulary layer for more than 8 hypotheses, from the codes of t: the blocked matrix-core
// product (which also leaves the per-tile softmax statistics), then the same selection.
// tiled: the logits go to the workspace tile by tile (see GemmArgs) instead of row-major.
q8_status q8i_output_codes(q8_ctx *ctx, const q8_mat *W, const float *bias, const int8_t *tq, const float *tscale, int n,
                           int k, float *logits, int tiled, float *lse, float *topk_logp, int32_t *topk_idx,
                           int32_t *tap_acc, float *part_max, double *part_sum, const BeamBatchArgs *search, int *search_fused)
{
    q8_status st;
    if (search_fused) *search_fused = 0;
    if (tiled && !tap_acc && q8i_output_codes_keeps_no_logits(W, k)) {
        // no logits are kept: the selection computes those of the few tiles it needs again
        st = q8i_vocab_panel(ctx, W, bias, tq, tscale, n, part_max, part_sum);
        if (st) return st;
        PanelSelectArgs s;
        s.part_max = part_max; s.part_sum = part_sum; s.tiles = W->tiles; s.xq = tq; s.xscale = tscale; s.bias = bias;
        s.lse = lse; s.topk_logp = topk_logp; s.topk_idx = topk_idx;
        s.ntiles = q8i_out_tiles(W->rows); s.n = n; s.k = k; s.V = W->rows; s.w_scale = W->scale;
        s.xw = (unsigned long long *)(ctx->ws + Q8_WS_PSEL_XCHG);
        s.wait_err = (unsigned *)(ctx->ws + Q8_WS_ATT_ERR);
        s.spin_limit = ctx->att_spin_limit;
        // the sentences' search steps in the same launch: n = whole beams of at most 8, beam k <= 128 candidates
        const bool fuse = search && search->beam >= 1 && search->beam <= Q8_MAX_BEAM && n % search->beam == 0 &&
                          search->beam * k <= 128 && (size_t)n * k * 8 <= Q8_WS_HEADER - Q8_WS_PSEL_XCHG;
        if (fuse) {
            s.bb = *search;
            s.bb.topk_logp = topk_logp; s.bb.topk_idx = topk_idx; s.bb.k = k;
            if (W->ld == 512) Q8_LAUNCH(ctx, Q8_KERNEL_SELECT, (panel_select_kernel<8, true>), dim3(n), dim3(256), 0, s);
            else Q8_LAUNCH(ctx, Q8_KERNEL_SELECT, (panel_select_kernel<10, true>), dim3(n), dim3(256), 0, s);
            if (search_fused) *search_fused = 1;
        } else {
            memset(&s.bb, 0, sizeof(s.bb));
            if (W->ld == 512) Q8_LAUNCH(ctx, Q8_KERNEL_SELECT, (panel_select_kernel<8, false>), dim3(n), dim3(256), 0, s);
            else Q8_LAUNCH(ctx, Q8_KERNEL_SELECT, (panel_select_kernel<10, false>), dim3(n), dim3(256), 0, s);
        }
        return q8i_launch_check(ctx, "panel selection");
    } else {
        const q8i_gemm_job gj = {W, tq, tscale, bias, logits, W->rows, tap_acc, part_max, part_sum, tiled};
        st = q8i_gemm_jobs(ctx, &gj, 1, n);
    }
    if (st) return st;
    return launch_select(ctx, part_max, part_sum, logits, tiled, W->rows, n, k, lse, topk_logp, topk_idx, nullptr);
}

