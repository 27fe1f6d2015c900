// q8_noalloc.hip -- the decoder step for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the kernels of
// cgru_decoder_step_q8 with their scratch (s', u(s'), the recurrent half of GRU q, the attention
// energies, the context codes and the arrival counters) in a static device array instead of the
// caller's workspace.  Nothing here, or in what it calls, allocates or frees device memory.
#include "q8_internal.h"

#include <mutex>

#define Q8_STATIC_SCRATCH_BYTES (1u << 20)
#define Q8_STATIC_MAX_DEVICES 64

// Each GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[Q8_STATIC_SCRATCH_BYTES];

namespace {

std::mutex g_lock;
void *g_ptr[Q8_STATIC_MAX_DEVICES];          // per device: the array's address there, NULL = not set up

// Address of the array on the current device; the first call on a device looks it up and clears the
// arrival counters at its head (the kernels leave them zero after every call).  That first call waits
// for the stream, so it cannot run under stream capture.
q8_status scratch_of_current_device(q8_ctx *ctx, char **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= Q8_STATIC_MAX_DEVICES)
        return q8_fail(ctx, Q8_ERR_DEVICE, "static scratch: no current device below %d", Q8_STATIC_MAX_DEVICES);
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_ptr[dev]) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(ctx->stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone)
            return q8_fail(ctx, Q8_ERR_DEVICE, "static scratch: call q8_noalloc_setup on this device before capturing");
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return q8_fail(ctx, Q8_ERR_DEVICE, "static scratch: hipGetSymbolAddress: %s", hipGetErrorString(e));
        q8_status st = q8i_fill_u32(ctx, p, Q8_WS_HEADER / 4, 0u);
        if (st) return st;
        if (hipStreamSynchronize(ctx->stream) != hipSuccess)
            return q8_fail(ctx, Q8_ERR_DEVICE, "static scratch: clearing the counters failed");
        g_ptr[dev] = p;
    }
    *out = (char *)g_ptr[dev];
    return Q8_OK;
}

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

extern "C" {

size_t q8_noalloc_scratch_bytes(void) { return Q8_STATIC_SCRATCH_BYTES; }

q8_status q8_noalloc_setup(q8_ctx *ctx)
{
    if (!ctx) return Q8_ERR_NULL;
    char *p = nullptr;
    return scratch_of_current_device(ctx, &p);
}

q8_status cgru_decoder_step_noalloc_q8(q8_ctx *ctx, const q8_cgru_weights *w, const float *P, const float *enc_h, int l,
                                       const float *y_emb, const float *s_prev, int n_beam, float *s_out, float *ctx_out,
                                       float *alpha_out, float *s_mid_out)
{
    if (!ctx) return Q8_ERR_NULL;
    if (!w) return q8_fail(ctx, Q8_ERR_NULL, "weights: NULL");
    // what cgru_decoder_step_q8 carves from its workspace, for these sizes (its own checks of the
    // arguments follow; here only the size against the array)
    const long long n = n_beam, H = w->r.Wh.cols, A = w->att_U.rows, ldq = w->q.Wx.ld;
    if (n <= 0 || n > Q8_MAX_BEAM || l <= 0 || l > 1024 || H <= 0 || A <= 0 || ldq <= 0 || H > 16384 || A > 65536 || ldq > 16384)
        return q8_fail(ctx, Q8_ERR_SHAPE, "cgru_decoder_step_noalloc_q8: bad sizes");
    const size_t need = Q8_WS_HEADER + up256((size_t)n * H * 4) + up256((size_t)n * A * 4) + up256((size_t)n * 3 * H * 4) +
                        up256((size_t)n * l * 4) + up256((size_t)n * ldq) + up256((size_t)n * 4);
    if (need > Q8_STATIC_SCRATCH_BYTES)
        return q8_fail(ctx, Q8_ERR_WORKSPACE, "cgru_decoder_step_noalloc_q8: these sizes need %zu bytes of scratch, the static array has %u",
                       need, Q8_STATIC_SCRATCH_BYTES);
    char *p = nullptr;
    q8_status st = scratch_of_current_device(ctx, &p);
    if (st) return st;
    // the same launches as cgru_decoder_step_q8, against a view of the context whose workspace is the array
    q8_ctx view = *ctx;
    view.ws = p;
    view.ws_bytes = Q8_STATIC_SCRATCH_BYTES;
    view.ws_reserved_top = 0;
    view.att_split = 0;                      // (its waits report through a flag in the context's own workspace)
    st = cgru_decoder_step_q8(&view, w, P, enc_h, l, y_emb, s_prev, n_beam, s_out, ctx_out, alpha_out, s_mid_out, nullptr);
    ctx->prof_n = view.prof_n;               // event pairs of an open profile were taken from the shared list
    if (st) memcpy(ctx->err, view.err, sizeof(ctx->err));
    return st;
}

}  // extern "C"
