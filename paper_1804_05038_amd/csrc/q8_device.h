// q8_device.h -- wave64 device helpers shared by the gfx950 kernels: cross-lane
// reductions on DPP / swizzle, block-level activation quantization into LDS, and the
// int8 row-streaming dot product (16-byte loads + 4-way int8 dot instructions).
//
// The arithmetic follows Section 3 of "Pieces of Eight: 8-bit Neural Machine
// Translation": both operands 8-bit integers, integer accumulation, float result.
#pragma once

#include <hip/hip_runtime.h>
#include "q8_math.h"
#include <stdint.h>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));

#define Q8_WAVE 64

// ------------------------------------------------------ hand-off between blocks ----
// "The last block to arrive finishes": blocks of one kernel leave results for the block that comes
// last.  On gfx950 the L2 caches of the eight XCDs are not coherent with each other, so the ordering
// is built from operations that act at agent scope by themselves, not from fences (a release fence
// writes the whole L2 back and an acquire fence invalidates it: 1.5 us each, measured, and the
// invalidation would also drop the vocabulary matrix that is kept resident there):
//   writer: agent-scope relaxed atomic stores of the data (performed in memory, past the L2), then
//           q8_stores_performed(), then one agent-scope relaxed atomic add on the arrival counter;
//   reader: sees the last count (its own add returned it), then reads the data with agent-scope
//           relaxed atomic loads, which are served from memory and cannot hit a stale line.
// q8_stores_performed: the wave waits until every store it has issued has been acknowledged
// (s_waitcnt vmcnt(0); gfx950 counts stores in vmcnt), and the compiler may not move memory
// operations across it.  The counter's add is program-ordered after it, so it cannot be performed
// before the data.  Block-wide: every wave calls it, then __syncthreads(), then one thread counts.
__device__ __forceinline__ void q8_stores_performed()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}
// Arrival counters of concurrent hand-offs sit 256 bytes apart when there are few of them: atomics
// on one address (and on neighbours in one line) are performed one after the other, about 10 ns each.
#define Q8_COUNTER_STRIDE 64

// ---------------------------------------------------------------- cross-lane ----

template <int CTRL>
__device__ __forceinline__ int dpp_mov_i(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}

#define DPP_XOR1 0xB1         // quad_perm [1,0,3,2]
#define DPP_XOR2 0x4E         // quad_perm [2,3,0,1]
#define DPP_HALF_MIRROR 0x141 // lane <-> 7 - lane within 8
#define DPP_MIRROR 0x140      // lane <-> 15 - lane within 16
#define SWZ_XOR16 0x401F      // ds_swizzle bit mode: and 0x1f, or 0, xor 0x10

// Sum over groups of `lpr` consecutive lanes (lpr in {16, 32, 64}, wave-uniform).
// Every lane of a group ends up holding the group's sum.
__device__ __forceinline__ int group_sum_i(int v, int lpr)
{
    v += dpp_mov_i<DPP_XOR1>(v);
    v += dpp_mov_i<DPP_XOR2>(v);
    v += dpp_mov_i<DPP_HALF_MIRROR>(v);
    v += dpp_mov_i<DPP_MIRROR>(v);
    if (lpr >= 32) v += __builtin_amdgcn_ds_swizzle(v, SWZ_XOR16);
    if (lpr >= 64) v = __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 32);
    return v;
}

__device__ __forceinline__ float wave_max_f(float v)
{
    v = fmaxf(v, __int_as_float(dpp_mov_i<DPP_XOR1>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_mov_i<DPP_XOR2>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_mov_i<DPP_HALF_MIRROR>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_mov_i<DPP_MIRROR>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), SWZ_XOR16)));
    return fmaxf(__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0)),
                 __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32)));
}

template <int CTRL>
__device__ __forceinline__ double dpp_mov_d(double v)
{
    const long long b = __double_as_longlong(v);
    const unsigned lo = dpp_mov_i<CTRL>((int)(unsigned)b), hi = dpp_mov_i<CTRL>((int)(unsigned)(b >> 32));
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// Sum of a double over the wave (fixed tree order), result in every lane.
__device__ __forceinline__ double wave_sum_d(double v)
{
    v += dpp_mov_d<DPP_XOR1>(v);
    v += dpp_mov_d<DPP_XOR2>(v);
    v += dpp_mov_d<DPP_HALF_MIRROR>(v);
    v += dpp_mov_d<DPP_MIRROR>(v);
    {
        const long long b = __double_as_longlong(v);
        const unsigned lo = __builtin_amdgcn_ds_swizzle((int)(unsigned)b, SWZ_XOR16);
        const unsigned hi = __builtin_amdgcn_ds_swizzle((int)(unsigned)(b >> 32), SWZ_XOR16);
        v += __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
    }
    const long long b = __double_as_longlong(v);
    const unsigned lo0 = __builtin_amdgcn_readlane((int)(unsigned)b, 0), hi0 = __builtin_amdgcn_readlane((int)(unsigned)(b >> 32), 0);
    const unsigned lo1 = __builtin_amdgcn_readlane((int)(unsigned)b, 32), hi1 = __builtin_amdgcn_readlane((int)(unsigned)(b >> 32), 32);
    return __longlong_as_double((long long)(((unsigned long long)hi0 << 32) | lo0)) +
           __longlong_as_double((long long)(((unsigned long long)hi1 << 32) | lo1));
}

template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_max_u64(unsigned long long v)
{
    const unsigned lo = dpp_mov_i<CTRL>((int)(unsigned)v), hi = dpp_mov_i<CTRL>((int)(unsigned)(v >> 32));
    const unsigned long long o = ((unsigned long long)hi << 32) | lo;
    return o > v ? o : v;
}

// Maximum of a 64-bit key over the wave, result in every lane.
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v)
{
    v = dpp_max_u64<DPP_XOR1>(v);
    v = dpp_max_u64<DPP_XOR2>(v);
    v = dpp_max_u64<DPP_HALF_MIRROR>(v);
    v = dpp_max_u64<DPP_MIRROR>(v);
    {
        const unsigned lo = __builtin_amdgcn_ds_swizzle((int)(unsigned)v, SWZ_XOR16);
        const unsigned hi = __builtin_amdgcn_ds_swizzle((int)(unsigned)(v >> 32), SWZ_XOR16);
        const unsigned long long o = ((unsigned long long)hi << 32) | lo;
        v = o > v ? o : v;
    }
    const unsigned long long a = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), 0) << 32) |
                                 (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, 0);
    const unsigned long long b = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), 32) << 32) |
                                 (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, 32);
    return a > b ? a : b;
}

// Order-preserving unsigned image of a float (-0.0 counts as +0.0): a < b  <=>  image(a) < image(b).
__device__ __forceinline__ unsigned ordered_bits(float v)
{
    const unsigned u = __float_as_uint(v + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_value(unsigned u)
{
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}

// The value of lane (lane ^ J), J a power of two below 64, without going through LDS: quad permutations
// (1, 2), two row shifts that write alternate banks of four lanes (4), a row rotation (8), and the lane
// swaps of rows (16) and wave halves (32).
template <int J>
__device__ __forceinline__ int lane_xor_i(int v, int lane)
{
    if constexpr (J == 1) return dpp_mov_i<DPP_XOR1>(v);
    else if constexpr (J == 2) return dpp_mov_i<DPP_XOR2>(v);
    else if constexpr (J == 4) {
        // row_shl:4 (lane L reads L + 4) into banks 0 and 2, row_shr:4 (L reads L - 4) into banks 1 and 3
        int t = __builtin_amdgcn_update_dpp(v, v, 0x104, 0xf, 0x5, false);
        return __builtin_amdgcn_update_dpp(t, v, 0x114, 0xf, 0xa, false);
    } else if constexpr (J == 8) return dpp_mov_i<0x128>(v);                       // row_ror:8
    else if constexpr (J == 16) {
        auto q = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);   // {rows 0 0 2 2, rows 1 1 3 3}
        return (int)((lane & 16) ? q[0] : q[1]);
    } else {
        auto q = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);   // {low half twice, high half twice}
        return (int)((lane & 32) ? q[0] : q[1]);
    }
}

template <int K2, int J>
__device__ __forceinline__ float sort_stage_f(float v, int lane)
{
    const float o = __int_as_float(lane_xor_i<J>(__float_as_int(v), lane));
    const bool up = (lane & K2) == 0;              // this block of K2 lanes is sorted descending
    const bool low = (lane & J) == 0;              // lower lane of the pair
    v = (up == low) ? fmaxf(v, o) : fminf(v, o);
    if constexpr (J > 1) return sort_stage_f<K2, J / 2>(v, lane);
    else return v;
}

// Bitonic sort of one float per lane across the wave, descending: lane r ends up holding
// the (r+1)-th largest value (with multiplicity).  21 compare-exchange stages on the cross-lane
// moves above: 0.35 us at one wave per SIMD, against 1.0 us with the partner fetched by
// ds_bpermute.  (Finding the k-th largest bit by bit with one ballot per bit, 32 scalar steps,
// took 1.2 us.)
__device__ __forceinline__ float wave_sort_desc_f(float v, int lane)
{
    v = sort_stage_f<2, 1>(v, lane);
    v = sort_stage_f<4, 2>(v, lane);
    v = sort_stage_f<8, 4>(v, lane);
    v = sort_stage_f<16, 8>(v, lane);
    v = sort_stage_f<32, 16>(v, lane);
    v = sort_stage_f<64, 32>(v, lane);
    return v;
}

// Order-preserving key: larger value first, then lower index.  -0.0 is folded into +0.0
// so that equal floats compare equal.
__device__ __forceinline__ unsigned long long topk_key(float val, int idx)
{
    return ((unsigned long long)ordered_bits(val) << 32) | (unsigned)(0x7fffffff - idx);
}
__device__ __forceinline__ int topk_key_idx(unsigned long long k) { return 0x7fffffff - (int)(k & 0xffffffffu); }
__device__ __forceinline__ float topk_key_val(unsigned long long k) { return ordered_value((unsigned)(k >> 32)); }

// ------------------------------------------------------ activation quantization ----

// Scale and reciprocal of the symmetric max-abs quantizer: scale = m / 127,
// inv = 127 / m, or (1, 0) when m < 2^-100.
__device__ __forceinline__ void q8_scale_of(float m, float &scale, float &inv)
{
    if (m < 0x1p-100f) {
        scale = 1.0f;
        inv = 0.0f;
    } else {
        scale = m / 127.0f;
        inv = 127.0f / m;
    }
}

__device__ __forceinline__ int q8_code(float v, float inv)
{
    float r = __builtin_rintf(v * inv);   // round half to even
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

// Four codes in a dword, for values whose largest magnitude produced inv: then |v * inv| <= 127.00002
// and q8_code's clamp never acts (non-finite inputs give unspecified codes).  Adding 1.5 * 2^23
// rounds the product to the nearest integer, ties to even (the sum's unit in the last place is 1
// and the constant is even), and leaves the two's-complement code in the low byte of the sum's
// bits: two instructions per value instead of four, and byte selects instead of masks and shifts.
__device__ __forceinline__ int q8_pack4(float a, float b, float c, float d, float inv)
{
    const float magic = 12582912.0f;
    const unsigned ua = __float_as_uint(__fadd_rn(__fmul_rn(a, inv), magic));
    const unsigned ub = __float_as_uint(__fadd_rn(__fmul_rn(b, inv), magic));
    const unsigned uc = __float_as_uint(__fadd_rn(__fmul_rn(c, inv), magic));
    const unsigned ud = __float_as_uint(__fadd_rn(__fmul_rn(d, inv), magic));
    // v_perm_b32: selector 0-3 = bytes of the second operand, 4-7 = bytes of the first, 0x0c = zero
    const unsigned lo = __builtin_amdgcn_perm(ub, ua, 0x0c0c0400u);
    const unsigned hi = __builtin_amdgcn_perm(ud, uc, 0x04000c0cu);
    return (int)(lo | hi);
}

// Two codes in the low half of a dword (same rounding as q8_pack4).
__device__ __forceinline__ int q8_pack2(float a, float b, float inv)
{
    const float magic = 12582912.0f;
    const unsigned ua = __float_as_uint(__fadd_rn(__fmul_rn(a, inv), magic));
    const unsigned ub = __float_as_uint(__fadd_rn(__fmul_rn(b, inv), magic));
    return (int)__builtin_amdgcn_perm(ub, ua, 0x0c0c0400u);
}

// Buffer descriptor over [base, base + bytes): a load through it at an offset at or past
// `bytes` returns zero without touching memory.  A load that has nothing to fetch is then
// still an unconditional instruction, and the counts the compiler waits on stay exact
// (a load inside a branch makes it wait for everything in flight).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t q8_rsrc(const void *base, size_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)bytes, 0x00020000);
}
#define Q8_OOB 0x80000000u           // past the end of every descriptor used here (sizes stay below 2^31)

// Quantizes n (<= NMAX) fp32 vectors X[j * ldx + k], k < K, into LDS bytes
// xq[j * ld + k] (ld % 16 == 0, bytes [K, ld) zeroed) and their scales into s_scale[j].
// s_red needs NMAX * (blockDim.x / 64) floats.  Ends with a block barrier.
template <int NMAX>
__device__ __forceinline__ void block_quantize(const float *__restrict__ X, int n, int K, int ldx, int ld,
                                               int8_t *xq, float *s_scale, float *s_red)
{
    const int tid = threadIdx.x, nt = blockDim.x, nw = nt >> 6, wave = tid >> 6, lane = tid & 63;
    float m[NMAX];
#pragma unroll
    for (int j = 0; j < NMAX; ++j) {
        m[j] = 0.0f;
        if (j < n) {
            const float *x = X + (size_t)j * ldx;
            for (int k = tid * 4; k < K; k += nt * 4) {
                if (k + 4 <= K) {
                    float4 v = *(const float4 *)(x + k);
                    m[j] = fmaxf(m[j], fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
                } else {
                    for (int t = k; t < K; ++t) m[j] = fmaxf(m[j], fabsf(x[t]));
                }
            }
            m[j] = wave_max_f(m[j]);
            if (lane == 0) s_red[j * nw + wave] = m[j];
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NMAX; ++j) {
        if (j < n) {
            float mm = 0.0f;
            for (int w = 0; w < nw; ++w) mm = fmaxf(mm, s_red[j * nw + w]);
            float scale, inv;
            q8_scale_of(mm, scale, inv);
            if (tid == 0) s_scale[j] = scale;
            const float *x = X + (size_t)j * ldx;
            for (int k = tid * 4; k < ld; k += nt * 4) {
                int packed;
                if (k + 4 <= K) {
                    float4 v = *(const float4 *)(x + k);
                    packed = q8_pack4(v.x, v.y, v.z, v.w, inv);
                } else {
                    float a = k < K ? x[k] : 0.0f, b = k + 1 < K ? x[k + 1] : 0.0f;
                    float c = k + 2 < K ? x[k + 2] : 0.0f, d = k + 3 < K ? x[k + 3] : 0.0f;
                    packed = q8_pack4(a, b, c, d, inv);
                }
                *(int *)(xq + (size_t)j * ld + k) = packed;
            }
        }
    }
    __syncthreads();
}

// ------------------------------------------------------------ row streaming dot ----

__device__ __forceinline__ int dot16(v4i w, v4i x, int acc)
{
    acc = __builtin_amdgcn_sdot4(w.x, x.x, acc, false);
    acc = __builtin_amdgcn_sdot4(w.y, x.y, acc, false);
    acc = __builtin_amdgcn_sdot4(w.z, x.z, acc, false);
    acc = __builtin_amdgcn_sdot4(w.w, x.w, acc, false);
    return acc;
}

// Integer dot products of U weight rows with N quantized vectors held in LDS.
//   wrow[u]: this lane's row base pointer (NULL = no row: contributes zeros).  Lanes are
//            split into groups of `lpr` consecutive lanes; all lanes of a group pass
//            the same row, different groups may pass different rows.
//   lir:     lane index within its group; the lane covers bytes [(c*lpr + lir)*16, +16)
//            of the row for c = 0, 1, ...
//   xq:      LDS, vector j at xq + j * ld (same ld as the weight rows).
// On return acc[u][j] holds, in every lane of a group, the full int32 sum for that
// group's row u and vector j.
template <int N, int U>
__device__ __forceinline__ void wave_dot(const int8_t *const (&wrow)[U], int ld, int lpr, int lir,
                                         const int8_t *xq, int (&acc)[U][N])
{
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int j = 0; j < N; ++j) acc[u][j] = 0;
    const int step = lpr * 16;
    int off = lir * 16;
    v4i w[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        w[u] = (v4i){0, 0, 0, 0};
        if (wrow[u] != nullptr && off < ld) w[u] = *(const v4i *)(wrow[u] + off);
    }
    while (off < ld) {                       // uniform trip count would be nicer; lanes past ld idle
        const int offn = off + step;
        v4i wn[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            wn[u] = (v4i){0, 0, 0, 0};
            if (wrow[u] != nullptr && offn < ld) wn[u] = *(const v4i *)(wrow[u] + offn);
        }
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const v4i x = *(const v4i *)(xq + (size_t)j * ld + off);
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u][j] = dot16(w[u], x, acc[u][j]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) w[u] = wn[u];
        off = offn;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int j = 0; j < N; ++j) acc[u][j] = group_sum_i(acc[u][j], lpr);
}

// ------------------------------------------------ fast path: everything in registers ----
//
// For the latency-bound products of a decoder step the order of issue decides the time:
// the fp32 activations are requested first (short, L2-resident), then every weight byte
// the wave will need, and only then does the block wait, reduce max|x| and write the int8
// codes to LDS -- the weight loads stay in flight behind that work.  Requires 256-thread
// blocks, K % 4 == 0, ld <= 1024 * CH.

template <int N, int CH>
struct XRegs {
    float4 v[N][CH];
};

// (Unconditional loads through a bounds-checked descriptor: a slice with nothing to fetch reads as
// zero.  A load inside a branch costs a dozen instructions of mask handling and makes the compiler
// wait for it before anything else.)
template <int N, int CH>
__device__ __forceinline__ void x_load(XRegs<N, CH> &R, const float *__restrict__ X, int n, int K, int ldx)
{
    const __amdgpu_buffer_rsrc_t rx = q8_rsrc(X, ((size_t)(n - 1) * ldx + K) * sizeof(float));
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
        for (int t = 0; t < CH; ++t) {
            const int k = (t * 256 + (int)threadIdx.x) * 4;
            const unsigned off = (j < n && k < K) ? (unsigned)(j * ldx + k) * 4u : Q8_OOB;
            R.v[j][t] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(rx, (int)off, 0, 0));
        }
    // loads return in issue order: nothing issued later may be moved ahead of these
    __builtin_amdgcn_sched_barrier(0);
}

// ---------------------------------------------------------- transposed wave reductions ----
// M values per lane (M a power of two, at most 64) reduced over the wave's 64 lanes.  In the first
// log2(M) exchange stages the two partners split the values between them: each keeps one half,
// hands the other half over and combines what it receives, so the work halves from stage to
// stage; the stages that are left run on the single remaining value.  About 4 M instructions
// instead of the 12 M of M separate reductions.  Stage s pairs lane L with L ^ 7, ^ 1, ^ 2, ^ 8,
// ^ 16, ^ 32 and lets lane bit 2, 0, 1, 3, 4, 5 choose the half that is kept (the first stage
// flips bits 0 and 1 as well, which is harmless while every lane still holds every value).
// Afterwards lane L holds the total of value t_index<M>(L).
__host__ __device__ constexpr int t_bit(int s) { return s == 0 ? 2 : s == 1 ? 0 : s == 2 ? 1 : s; }
__host__ __device__ constexpr int t_log2(int m) { return m <= 1 ? 0 : 1 + t_log2(m >> 1); }
__host__ __device__ constexpr int t_pow2(int n) { return n <= 1 ? 1 : 2 * t_pow2((n + 1) >> 1); }

template <int S>
__device__ __forceinline__ int t_xchg(int v, int lane)
{
    if constexpr (S == 0) return dpp_mov_i<DPP_HALF_MIRROR>(v);
    else if constexpr (S == 1) return dpp_mov_i<DPP_XOR1>(v);
    else if constexpr (S == 2) return dpp_mov_i<DPP_XOR2>(v);
    else if constexpr (S == 3) return dpp_mov_i<0x128>(v);                        // row_ror:8 = lane ^ 8 within 16
    else if constexpr (S == 4) {
        // (x, x) -> {rows 0 0 2 2, rows 1 1 3 3} of x
        auto q = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
        return (int)((lane & 16) ? q[0] : q[1]);
    } else {
        auto q = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);   // {low half twice, high half twice}
        return (int)((lane & 32) ? q[0] : q[1]);
    }
}

struct TSumI { static __device__ __forceinline__ int op(int a, int b) { return a + b; } };
struct TMaxF {
    static __device__ __forceinline__ int op(int a, int b) { return __float_as_int(fmaxf(__int_as_float(a), __int_as_float(b))); }
};

template <int S, int M, class Op>
__device__ __forceinline__ void t_stage(int (&v)[M], int lane)
{
    if constexpr (S < t_log2(M)) {
        constexpr int half = M >> (S + 1);
        const bool up = (lane >> t_bit(S)) & 1;
#pragma unroll
        for (int i = 0; i < half; ++i) {
            const int give = up ? v[i] : v[i + half];
            const int keep = up ? v[i + half] : v[i];
            v[i] = Op::op(keep, t_xchg<S>(give, lane));
        }
    } else {
        v[0] = Op::op(v[0], t_xchg<S>(v[0], lane));
    }
}

template <int M, class Op>
__device__ __forceinline__ int wave_reduce_t(int (&v)[M], int lane)
{
    static_assert(M >= 1 && M <= 64 && (M & (M - 1)) == 0, "power of two up to 64");
    t_stage<0, M, Op>(v, lane);
    t_stage<1, M, Op>(v, lane);
    t_stage<2, M, Op>(v, lane);
    t_stage<3, M, Op>(v, lane);
    t_stage<4, M, Op>(v, lane);
    t_stage<5, M, Op>(v, lane);
    return v[0];
}

// Index of the value whose total lane `lane` holds after wave_reduce_t<M>, and whether the lane
// is the first of the 64 / M lanes that hold that same total.
template <int M>
__device__ __forceinline__ int t_index(int lane)
{
    int idx = 0;
#pragma unroll
    for (int s = 0; s < t_log2(M); ++s) idx |= ((lane >> t_bit(s)) & 1) * (M >> (s + 1));
    return idx;
}
template <int M>
__device__ __forceinline__ bool t_first(int lane)
{
    int used = 0;
#pragma unroll
    for (int s = 0; s < t_log2(M); ++s) used |= 1 << t_bit(s);
    return (lane & (63 & ~used)) == 0;
}

// Totals of CNT = UT * N partial sums per lane, handed to the lanes that finish them: lane j < N
// receives the UT totals of vector j (part[u][j] summed over the wave) in mine[u].  s_t: CNT
// ints of LDS owned by this wave.
template <int N, int UT>
__device__ __forceinline__ void sums_to_lanes(const int (&part)[UT][N], int lane, int *s_t, int (&mine)[UT])
{
    constexpr int CNT = UT * N, M = t_pow2(CNT);
    int v[M];
#pragma unroll
    for (int e = 0; e < M; ++e) v[e] = e < CNT ? part[e / N][e % N] : 0;
    const int tot = wave_reduce_t<M, TSumI>(v, lane);
    const int idx = t_index<M>(lane);
    if (idx < CNT && t_first<M>(lane)) s_t[idx] = tot;
    __builtin_amdgcn_wave_barrier();             // same wave: the reads below are issued after the writes
#pragma unroll
    for (int u = 0; u < UT; ++u) mine[u] = lane < N ? s_t[u * N + lane] : 0;
}

// Wave maxima of N independent values, the cross-lane steps of all N interleaved so that
// their latencies overlap.
template <int N>
__device__ __forceinline__ void wave_max_multi(float (&m)[N])
{
#pragma unroll
    for (int j = 0; j < N; ++j) m[j] = fmaxf(m[j], __int_as_float(dpp_mov_i<DPP_XOR1>(__float_as_int(m[j]))));
#pragma unroll
    for (int j = 0; j < N; ++j) m[j] = fmaxf(m[j], __int_as_float(dpp_mov_i<DPP_XOR2>(__float_as_int(m[j]))));
#pragma unroll
    for (int j = 0; j < N; ++j) m[j] = fmaxf(m[j], __int_as_float(dpp_mov_i<DPP_HALF_MIRROR>(__float_as_int(m[j]))));
#pragma unroll
    for (int j = 0; j < N; ++j) m[j] = fmaxf(m[j], __int_as_float(dpp_mov_i<DPP_MIRROR>(__float_as_int(m[j]))));
#pragma unroll
    for (int j = 0; j < N; ++j) m[j] = fmaxf(m[j], __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(m[j]), SWZ_XOR16)));
#pragma unroll
    for (int j = 0; j < N; ++j)
        m[j] = fmaxf(__int_as_float(__builtin_amdgcn_readlane(__float_as_int(m[j]), 0)),
                     __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m[j]), 32)));
}

// Turns the staged vectors into int8 codes in LDS (xq[j * ld + k], bytes [K, ld) zero) and
// scales in s_scale[j].  s_red: N * 4 floats.  Ends with a block barrier.  The two
// divisions per vector are done once per wave, by lane j for vector j, and broadcast.
// Thread-local max |x| of every staged vector: the first use of the loaded values.  Calling
// this before the weight loads are issued makes the block wait for the (short) activation
// loads alone; the rest of the quantization then overlaps the weight stream.
template <int N, int CH>
__device__ __forceinline__ void x_absmax(const XRegs<N, CH> &R, float (&m)[N])
{
#pragma unroll
    for (int j = 0; j < N; ++j) {
        m[j] = 0.0f;
#pragma unroll
        for (int t = 0; t < CH; ++t) {
            const float4 v = R.v[j][t];
            m[j] = fmaxf(m[j], fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
        }
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <int N, int CH>
__device__ __forceinline__ void x_finish_m(const XRegs<N, CH> &R, float (&m)[N], int n, int ld, int8_t *xq, float *s_scale,
                                           float *s_red);

template <int N, int CH>
__device__ __forceinline__ void x_finish(const XRegs<N, CH> &R, int n, int ld, int8_t *xq, float *s_scale, float *s_red)
{
    float m[N];
    x_absmax<N, CH>(R, m);
    x_finish_m<N, CH>(R, m, n, ld, xq, s_scale, s_red);
}

template <int N, int CH>
__device__ __forceinline__ void x_finish_m(const XRegs<N, CH> &R, float (&m)[N], int n, int ld, int8_t *xq, float *s_scale,
                                           float *s_red)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    {
        constexpr int M = t_pow2(N);
        int mv[M];
#pragma unroll
        for (int e = 0; e < M; ++e) mv[e] = e < N ? __float_as_int(m[e]) : 0;
        const int tot = wave_reduce_t<M, TMaxF>(mv, lane);
        const int idx = t_index<M>(lane);
        if (idx < N && t_first<M>(lane)) s_red[idx * 4 + wave] = __int_as_float(tot);
    }
    __syncthreads();
    float scale = 1.0f, inv = 0.0f;
    if (lane < N) {
        const float mm = fmaxf(fmaxf(s_red[lane * 4], s_red[lane * 4 + 1]), fmaxf(s_red[lane * 4 + 2], s_red[lane * 4 + 3]));
        q8_scale_of(mm, scale, inv);
        if (wave == 0) s_scale[lane] = scale;
    }
#pragma unroll
    for (int j = 0; j < N; ++j) {
        if (j < n) {
            const float invj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(inv), j));
#pragma unroll
            for (int t = 0; t < CH; ++t) {
                const int k = (t * 256 + tid) * 4;
                const float4 v = R.v[j][t];      // zero beyond K, so pad bytes come out zero
                if (k < ld) *(int *)(xq + (size_t)j * ld + k) = q8_pack4(v.x, v.y, v.z, v.w, invj);
            }
        }
    }
    __syncthreads();
}

// The same for NIN staged inputs at once (different widths allowed): one pair of barriers
// for all of them, their reductions interleaved.  Input i uses s_scale[8 * i + j];
// s_red needs NIN * N * 4 floats.
template <int N, int CH, int NIN>
__device__ __forceinline__ void x_finish_multi(const XRegs<N, CH> (&R)[NIN], const int (&ld)[NIN], int8_t *const (&xq)[NIN],
                                               float *s_scale, float *s_red)
{
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    float m[NIN * N];
#pragma unroll
    for (int i = 0; i < NIN; ++i)
#pragma unroll
        for (int j = 0; j < N; ++j) {
            float mm = 0.0f;
#pragma unroll
            for (int t = 0; t < CH; ++t) {
                const float4 v = R[i].v[j][t];
                mm = fmaxf(mm, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
            }
            m[i * N + j] = mm;
        }
    {
        constexpr int M = t_pow2(NIN * N);
        int mv[M];
#pragma unroll
        for (int e = 0; e < M; ++e) mv[e] = e < NIN * N ? __float_as_int(m[e]) : 0;
        const int tot = wave_reduce_t<M, TMaxF>(mv, lane);
        const int idx = t_index<M>(lane);
        if (idx < NIN * N && t_first<M>(lane)) s_red[idx * 4 + wave] = __int_as_float(tot);
    }
    __syncthreads();
    float scale = 1.0f, inv = 0.0f;          // lane 8 i + j owns vector j of input i
    if (lane < 8 * NIN && (lane & 7) < N) {
        const int e = (lane >> 3) * N + (lane & 7);
        const float mm = fmaxf(fmaxf(s_red[e * 4], s_red[e * 4 + 1]), fmaxf(s_red[e * 4 + 2], s_red[e * 4 + 3]));
        q8_scale_of(mm, scale, inv);
        if (wave == 0) s_scale[lane] = scale;
    }
#pragma unroll
    for (int i = 0; i < NIN; ++i)
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const float invj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(inv), 8 * i + j));
#pragma unroll
            for (int t = 0; t < CH; ++t) {
                const int k = (t * 256 + tid) * 4;
                const float4 v = R[i].v[j][t];
                if (k < ld[i]) *(int *)(xq[i] + (size_t)j * ld[i] + k) = q8_pack4(v.x, v.y, v.z, v.w, invj);
            }
        }
    __syncthreads();
}

// Requests U weight rows for this wave: lane covers bytes [(c * 64 + lane) * 16, +16) of a row.
// rw: descriptor over the whole matrix (below 2 GiB); row[u] < 0: no such row, reads as zero.
// STREAM: the loads carry the non-temporal hint.  The matrices of a decoder step other than the
// vocabulary matrix are read once per step by kernels that are bound by latency wherever the
// bytes come from; streaming them leaves the 32 MB of L2 to the vocabulary matrix.
template <int U, int CH, bool STREAM = true>
__device__ __forceinline__ void rows_load(v4i (&w)[U][CH], __amdgpu_buffer_rsrc_t rw, const int (&row)[U], int ld, int lane)
{
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int off = (c * 64 + lane) * 16;
            const unsigned o = (row[u] >= 0 && off < ld) ? (unsigned)row[u] * (unsigned)ld + (unsigned)off : Q8_OOB;
            w[u][c] = STREAM ? __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rw, (int)o, 0, 2))
                             : __builtin_bit_cast(v4i, __builtin_amdgcn_raw_buffer_load_b128(rw, (int)o, 0, 0));
        }
}

// Dots the staged rows with the N quantized vectors in LDS: the lane's partial sums (its 16 bytes
// of every chunk), to be totalled over the wave by sums_to_lanes.
template <int N, int U, int CH>
__device__ __forceinline__ void rows_dot_part(const v4i (&w)[U][CH], int ld, int lane, const int8_t *xq, int (&acc)[U][N])
{
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int j = 0; j < N; ++j) acc[u][j] = 0;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int off = (c * 64 + lane) * 16;
        if (off < ld) {
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const v4i x = *(const v4i *)(xq + (size_t)j * ld + off);
#pragma unroll
                for (int u = 0; u < U; ++u) acc[u][j] = dot16(w[u][c], x, acc[u][j]);
            }
        }
    }
}

// Chunks per lane of the fast path for a row of ld bytes (0 = not covered).
static inline int q8_fast_ch(int ld) { return ld <= 1024 ? 1 : (ld <= 2048 ? 2 : (ld <= 4096 ? 4 : 0)); }

// Group width for rows of `ld` bytes: the smallest of 16, 32, 64 lanes whose single
// 16-byte-per-lane pass covers the row, 64 for longer rows.
static inline int q8_lanes_per_row(int ld)
{
    return ld <= 256 ? 16 : (ld <= 512 ? 32 : 64);
}

// combine lanes i, i + 16, i + 32, i + 48 (the four row groups of a result tile), all lanes get the result
__device__ __forceinline__ float quad_rows_max(float v)
{
    auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ double quad_rows_sum(double v)
{
    unsigned lo = (unsigned)__double2loint(v), hi = (unsigned)__double2hiint(v);
    auto ql = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    auto qh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    v = __hiloint2double((int)qh[0], (int)ql[0]) + __hiloint2double((int)qh[1], (int)ql[1]);
    lo = (unsigned)__double2loint(v); hi = (unsigned)__double2hiint(v);
    auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __hiloint2double((int)rh[0], (int)rl[0]) + __hiloint2double((int)rh[1], (int)rl[1]);
}

// e^x for x <= 0 (a logit minus the maximum of its group) by the hardware's 2^x on x log2(e), the
// product and the 2^x that the fast library exponential takes for results in the normal range;
// without its rescaling of denormal results (four more instructions per value): below 2^-126 this
// returns zero, which a sum that also holds e^0 = 1 cannot tell from the denormal value.
__device__ __forceinline__ float exp_le0(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896340736f); }

// fp32 nonlinearities of the gates, evaluated in double and rounded once (q8_math.h).
__device__ __forceinline__ float sigmoid_rn(float a) { return q8_sigmoid_rn(a); }
__device__ __forceinline__ float tanh_rn(float a) { return q8_tanh_rn(a); }

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
