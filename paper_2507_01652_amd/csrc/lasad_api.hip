// C ABI of liblasad: argument validation on the host, then dispatch to the
// kernel launchers.  Nothing here allocates device memory or synchronises.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "lasad_internal.h"

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(const char *what, hipError_t e)
{
    return fail(LASAD_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

bool supported_d(int d) { return d == 32 || d == 64 || d == 128; }

bool force_generic()
{
    static const bool v = [] {
        const char *e = getenv("LASAD_FORCE_GENERIC");
        return e && e[0] == '1';
    }();
    return v;
}

int check_grid(int grid_h, int grid_w, int mode)
{
    if (grid_h < 1 || grid_w < 1) return fail(LASAD_ERR_INVALID_ARG, "grid %d x %d: both sides must be >= 1", grid_h, grid_w);
    if ((int64_t)grid_h * grid_w > (int64_t)1 << 30) return fail(LASAD_ERR_INVALID_ARG, "grid %d x %d is too large", grid_h, grid_w);
    if (mode < 0 || mode > 2) return fail(LASAD_ERR_INVALID_ARG, "boundary_mode %d is not a lasad_boundary_t", mode);
    return LASAD_OK;
}

}  // namespace

// Scratch of lasad_forward_chunked_static: the per-segment partial states of the segment plan
// (at most 512 workgroup slots x one 64 x 64 fp32 state).  One copy per GPU, held until the
// process ends; its device address is looked up once per device (the array's name is only a
// host-side handle).
constexpr size_t kStaticScratchBytes = (size_t)512 * 64 * 64 * sizeof(float);   // 8 MiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (looked up on the first call per device)
int static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail("hipGetDevice", e);
    if (dev < 0 || dev >= kMaxDevices) return fail(LASAD_ERR_UNSUPPORTED, "device index %d", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail("hipGetSymbolAddress(scratch)", e);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LASAD_OK;
}

}  // namespace

extern "C" {

const char *lasad_last_error(void) { return g_err; }

const char *lasad_version(void) { return "lasad 0.1 gfx950"; }

int lasad_decay_factors(const float *gamma, int n_heads, int grid_h, int grid_w,
                        int start_pos, int n_tokens, int boundary_mode,
                        float *lambda_out, int32_t *cum_exp_out, void *hip_stream)
{
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "n_heads = %d", n_heads);
    if (start_pos < 0 || n_tokens < 0 || (int64_t)start_pos + n_tokens > (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "positions %d+1..%d+%d leave the %d x %d grid", start_pos, start_pos, n_tokens, grid_h, grid_w);
    if (lambda_out && !gamma) return fail(LASAD_ERR_INVALID_ARG, "gamma is NULL");
    hipError_t e = lasad::launch_decay_factors(gamma, n_heads, grid_w, start_pos, n_tokens, boundary_mode,
                                               lambda_out, cum_exp_out, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail("lasad_decay_factors launch", e);
    return LASAD_OK;
}

size_t lasad_forward_workspace_bytes(int B, int n_heads, int n_tokens, int d, int io_dtype)
{
    if (B < 1 || n_heads < 1 || n_tokens < 1) return 0;
    if (io_dtype == LASAD_BF16 && d == 64 && !force_generic())
        return lasad::forward_mfma_workspace_bytes((int64_t)B * n_heads, n_tokens);
    return 0;   // the fp32 kernel keeps everything in registers and LDS
}

// static_ws: the workspace is the library's own scratch array (looked up after the arguments have passed)
static int forward_chunked_impl(const void *q, const void *k, const void *v, void *o,
                                const lasad_layout_t *qkv_layout, const lasad_layout_t *o_layout,
                                int io_dtype, int out_dtype,
                                int B, int n_heads, int d, int grid_h, int grid_w,
                                int start_pos, int n_tokens,
                                const float *gamma, int boundary_mode, float q_scale,
                                const float *state_in, float *state_out,
                                void *workspace, size_t workspace_bytes, bool static_ws, void *hip_stream)
{
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x7fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (!supported_d(d)) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (supported: 32, 64, 128)", d);
    if (start_pos < 0 || n_tokens < 0 || (int64_t)start_pos + n_tokens > (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "positions %d+1..%d+%d leave the %d x %d grid", start_pos, start_pos, n_tokens, grid_h, grid_w);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (out_dtype != LASAD_F32 && out_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "out_dtype %d", out_dtype);
    if (io_dtype == LASAD_F32 && out_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 output");
    if (!gamma) return fail(LASAD_ERR_INVALID_ARG, "gamma is NULL");
    if (!qkv_layout || !o_layout) return fail(LASAD_ERR_INVALID_ARG, "layout is NULL");
    if (n_tokens > 0 && (!q || !k || !v || !o)) return fail(LASAD_ERR_INVALID_ARG, "q, k, v or o is NULL");
    const int vec = io_dtype == LASAD_BF16 ? 8 : 4;   // elements per 16 bytes
    const int ovec = out_dtype == LASAD_BF16 ? 8 : 4;
    if (qkv_layout->stride_b % vec || qkv_layout->stride_n % vec || qkv_layout->stride_h % vec ||
        qkv_layout->stride_b < 0 || qkv_layout->stride_n < 0 || qkv_layout->stride_h < 0)
        return fail(LASAD_ERR_INVALID_ARG, "q/k/v strides must be non-negative multiples of %d elements", vec);
    if (o_layout->stride_b % ovec || o_layout->stride_n % ovec || o_layout->stride_h % ovec ||
        o_layout->stride_b < 0 || o_layout->stride_n < 0 || o_layout->stride_h < 0)
        return fail(LASAD_ERR_INVALID_ARG, "o strides must be non-negative multiples of %d elements", ovec);
    if (n_tokens > 0 && (qkv_layout->stride_n < d || o_layout->stride_n < d))
        return fail(LASAD_ERR_INVALID_ARG, "token stride smaller than the head dim");
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) ||
        !aligned(state_in, 16) || !aligned(state_out, 16))
        return fail(LASAD_ERR_INVALID_ARG, "q, k, v, o and the states must be 16-byte aligned");
    if (n_tokens > 0 && (o == q || o == k || o == v)) return fail(LASAD_ERR_INVALID_ARG, "o aliases an input");

    lasad::ForwardArgs a;
    a.q = q; a.k = k; a.v = v; a.o = o; a.lam = nullptr;
    a.in = *qkv_layout; a.out = *o_layout;
    a.io_dtype = io_dtype; a.out_dtype = out_dtype;
    a.B = B; a.Hh = n_heads; a.d = d;
    a.grid_w = grid_w;
    a.start_pos = start_pos; a.n_tokens = n_tokens;
    a.gamma = gamma; a.mode = boundary_mode; a.q_scale = q_scale;
    a.state_in = state_in; a.state_out = state_out;
    a.seg_states = nullptr; a.n_segments = 1; a.seg_chunks = 0;
    a.fused_act = 0; a.norm = 0; a.norm_eps = 0.f; a.norm_w = nullptr;
    if (static_ws && n_tokens > 0) {
        if (lasad_forward_workspace_bytes(B, n_heads, n_tokens, d, io_dtype) > kStaticScratchBytes)
            return fail(LASAD_ERR_WORKSPACE, "the call wants %zu bytes of scratch, the built-in array holds %zu",
                        lasad_forward_workspace_bytes(B, n_heads, n_tokens, d, io_dtype), kStaticScratchBytes);
        if (int rc = static_scratch(&workspace)) return rc;
        workspace_bytes = kStaticScratchBytes;
    }
    if (workspace) {
        const size_t need = lasad_forward_workspace_bytes(B, n_heads, n_tokens, d, io_dtype);
        if (workspace_bytes < need)
            return fail(LASAD_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed", workspace_bytes, need);
        if (!aligned(workspace, 16)) return fail(LASAD_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
        if (need > 0) a.seg_states = (float *)workspace;
    }

    if (n_tokens == 0 && (!state_out || state_out == state_in)) return LASAD_OK;   // nothing to do

    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e;
    if (io_dtype == LASAD_BF16 && d == 64 && n_tokens > 0 && !force_generic())
        e = lasad::launch_forward_mfma(a, s);
    else
        e = lasad::launch_forward_generic(a, s);
    if (e != hipSuccess) return hip_fail("lasad_forward_chunked launch", e);
    return LASAD_OK;
}

int lasad_forward_chunked(const void *q, const void *k, const void *v, void *o,
                          const lasad_layout_t *qkv_layout, const lasad_layout_t *o_layout,
                          int io_dtype, int out_dtype,
                          int B, int n_heads, int d, int grid_h, int grid_w,
                          int start_pos, int n_tokens,
                          const float *gamma, int boundary_mode, float q_scale,
                          const float *state_in, float *state_out,
                          void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return forward_chunked_impl(q, k, v, o, qkv_layout, o_layout, io_dtype, out_dtype, B, n_heads, d, grid_h, grid_w,
                                start_pos, n_tokens, gamma, boundary_mode, q_scale, state_in, state_out,
                                workspace, workspace_bytes, false, hip_stream);
}

size_t lasad_forward_static_scratch_bytes(void) { return kStaticScratchBytes; }

int lasad_forward_chunked_static(const void *q, const void *k, const void *v, void *o,
                                 const lasad_layout_t *qkv_layout, const lasad_layout_t *o_layout,
                                 int io_dtype, int out_dtype,
                                 int B, int n_heads, int d, int grid_h, int grid_w,
                                 int start_pos, int n_tokens,
                                 const float *gamma, int boundary_mode, float q_scale,
                                 const float *state_in, float *state_out, void *hip_stream)
{
    return forward_chunked_impl(q, k, v, o, qkv_layout, o_layout, io_dtype, out_dtype, B, n_heads, d, grid_h, grid_w,
                                start_pos, n_tokens, gamma, boundary_mode, q_scale, state_in, state_out,
                                nullptr, 0, true, hip_stream);
}

int lasad_decode_step(const void *q, const void *k, const void *v, void *o,
                      int io_dtype, int out_dtype, int B, int n_heads, int d,
                      int grid_h, int grid_w, int pos,
                      const float *gamma, int boundary_mode, float q_scale,
                      float *state, void *hip_stream)
{
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x7fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (!supported_d(d)) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (supported: 32, 64, 128)", d);
    if (pos < 0 || (int64_t)pos >= (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "pos %d is outside the %d x %d grid", pos, grid_h, grid_w);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (out_dtype != LASAD_F32 && out_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "out_dtype %d", out_dtype);
    if (io_dtype == LASAD_F32 && out_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 output");
    if (!q || !k || !v || !o || !gamma || !state) return fail(LASAD_ERR_INVALID_ARG, "a required pointer is NULL");
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(state, 16))
        return fail(LASAD_ERR_INVALID_ARG, "q, k, v, o and state must be 16-byte aligned");
    if (o == q || o == k || o == v) return fail(LASAD_ERR_INVALID_ARG, "o aliases an input");

    lasad::DecodeArgs a;
    a.q = q; a.k = k; a.v = v; a.o = o; a.lam = nullptr;
    a.io_dtype = io_dtype; a.out_dtype = out_dtype;
    a.B = B; a.Hh = n_heads; a.d = d;
    a.grid_w = grid_w; a.pos = pos; a.pos_rows = nullptr; a.grid_n = grid_h * grid_w;
    a.fused_act = 0; a.norm = 0; a.norm_eps = 0.f; a.norm_w = nullptr;
    a.gamma = gamma; a.mode = boundary_mode; a.q_scale = q_scale;
    a.state = state;
    hipError_t e = lasad::launch_decode(a, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail("lasad_decode_step launch", e);
    return LASAD_OK;
}

int lasad_decode_step_cached(const void *q, const void *k, const void *v, void *o,
                             void *k_cache, void *v_cache, int cache_tokens,
                             int io_dtype, int out_dtype, int B, int n_heads, int d,
                             int grid_h, int grid_w, int pos,
                             const float *gamma, int boundary_mode, float q_scale,
                             void *hip_stream)
{
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x7fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (!supported_d(d)) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (supported: 32, 64, 128)", d);
    if (pos < 0 || (int64_t)pos >= (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "pos %d is outside the %d x %d grid", pos, grid_h, grid_w);
    if (cache_tokens < 1 || pos >= cache_tokens)
        return fail(LASAD_ERR_INVALID_ARG, "pos %d does not fit a cache of %d tokens", pos, cache_tokens);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (out_dtype != LASAD_F32 && out_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "out_dtype %d", out_dtype);
    if (io_dtype == LASAD_F32 && out_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 output");
    if (!q || !k || !v || !o || !gamma || !k_cache || !v_cache) return fail(LASAD_ERR_INVALID_ARG, "a required pointer is NULL");
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16))
        return fail(LASAD_ERR_INVALID_ARG, "q, k, v, o and the caches must be 16-byte aligned");
    if (o == q || o == k || o == v || k_cache == v_cache) return fail(LASAD_ERR_INVALID_ARG, "buffers alias");

    lasad::CachedDecodeArgs a;
    a.q = q; a.k = k; a.v = v; a.o = o; a.k_cache = k_cache; a.v_cache = v_cache;
    a.io_dtype = io_dtype; a.out_dtype = out_dtype;
    a.B = B; a.Hh = n_heads; a.d = d; a.cache_tokens = cache_tokens;
    a.grid_w = grid_w; a.pos = pos;
    a.gamma = gamma; a.mode = boundary_mode; a.q_scale = q_scale;
    hipError_t e = lasad::launch_decode_cached(a, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail("lasad_decode_step_cached launch", e);
    return LASAD_OK;
}

int lasad_decode_step_gated_cached(const void *q, const void *lam, const void *k, const void *v, void *o,
                                   void *lam_cache, void *k_cache, void *v_cache, int cache_tokens,
                                   int io_dtype, int out_dtype, int B, int n_heads, int d,
                                   int grid_h, int grid_w, int pos, int boundary_mode, float q_scale,
                                   void *hip_stream)
{
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x7fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (!supported_d(d)) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (supported: 32, 64, 128)", d);
    if (pos < 0 || (int64_t)pos >= (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "pos %d is outside the %d x %d grid", pos, grid_h, grid_w);
    if (cache_tokens < 1 || pos >= cache_tokens)
        return fail(LASAD_ERR_INVALID_ARG, "pos %d does not fit a cache of %d tokens", pos, cache_tokens);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (out_dtype != LASAD_F32 && out_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "out_dtype %d", out_dtype);
    if (io_dtype == LASAD_F32 && out_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 output");
    if (!q || !lam || !v || !o || !lam_cache || !v_cache) return fail(LASAD_ERR_INVALID_ARG, "a required pointer is NULL");
    if ((k == nullptr) != (k_cache == nullptr))
        return fail(LASAD_ERR_INVALID_ARG, "k and k_cache must be given together (own key) or both be NULL (tied key)");
    if (!aligned(q, 16) || !aligned(lam, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) ||
        !aligned(lam_cache, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16))
        return fail(LASAD_ERR_INVALID_ARG, "q, lam, k, v, o and the caches must be 16-byte aligned");
    if (o == q || o == lam || o == v || (k && o == k) || lam_cache == v_cache || (k_cache && (k_cache == v_cache || k_cache == lam_cache)))
        return fail(LASAD_ERR_INVALID_ARG, "buffers alias");

    lasad::CachedDecodeArgs a;
    a.q = q; a.lam = lam; a.k = k; a.v = v; a.o = o;
    a.lam_cache = lam_cache; a.k_cache = k_cache; a.v_cache = v_cache;
    a.io_dtype = io_dtype; a.out_dtype = out_dtype;
    a.B = B; a.Hh = n_heads; a.d = d; a.cache_tokens = cache_tokens;
    a.grid_w = grid_w; a.pos = pos;
    a.gamma = nullptr; a.mode = boundary_mode; a.q_scale = q_scale;
    hipError_t e = lasad::launch_decode_cached(a, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail("lasad_decode_step_gated_cached launch", e);
    return LASAD_OK;
}

static int forward_gated_common(const void *q, const void *lam, const void *k, const void *v, void *o,
                                const lasad_layout_t *in_layout, const lasad_layout_t *o_layout,
                                int io_dtype, int out_dtype,
                                int B, int n_heads, int d, int grid_h, int grid_w,
                                int start_pos, int n_tokens, int boundary_mode, float q_scale,
                                const float *state_in, float *state_out, void *hip_stream,
                                int layer, const float *norm_weight, float norm_eps)
{
    if (layer && d != 64) return fail(LASAD_ERR_UNSUPPORTED, "the fused layer needs head dim 64 (got %d)", d);
    if (layer && !aligned(norm_weight, 16)) return fail(LASAD_ERR_INVALID_ARG, "norm_weight must be 16-byte aligned");
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x7fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (!supported_d(d)) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (supported: 32, 64, 128)", d);
    if (start_pos < 0 || n_tokens < 0 || (int64_t)start_pos + n_tokens > (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "positions %d+1..%d+%d leave the %d x %d grid", start_pos, start_pos, n_tokens, grid_h, grid_w);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (out_dtype != LASAD_F32 && out_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "out_dtype %d", out_dtype);
    if (io_dtype == LASAD_F32 && out_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 output");
    if (!in_layout || !o_layout) return fail(LASAD_ERR_INVALID_ARG, "layout is NULL");
    if (n_tokens > 0 && (!q || !lam || !v || !o)) return fail(LASAD_ERR_INVALID_ARG, "q, lam, v or o is NULL");
    const int vec = io_dtype == LASAD_BF16 ? 8 : 4, ovec = out_dtype == LASAD_BF16 ? 8 : 4;
    if (in_layout->stride_b % vec || in_layout->stride_n % vec || in_layout->stride_h % vec ||
        in_layout->stride_b < 0 || in_layout->stride_n < 0 || in_layout->stride_h < 0)
        return fail(LASAD_ERR_INVALID_ARG, "input strides must be non-negative multiples of %d elements", vec);
    if (o_layout->stride_b % ovec || o_layout->stride_n % ovec || o_layout->stride_h % ovec ||
        o_layout->stride_b < 0 || o_layout->stride_n < 0 || o_layout->stride_h < 0)
        return fail(LASAD_ERR_INVALID_ARG, "o strides must be non-negative multiples of %d elements", ovec);
    if (n_tokens > 0 && (in_layout->stride_n < d || o_layout->stride_n < d))
        return fail(LASAD_ERR_INVALID_ARG, "token stride smaller than the head dim");
    if (!aligned(q, 16) || !aligned(lam, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) ||
        !aligned(state_in, 16) || !aligned(state_out, 16))
        return fail(LASAD_ERR_INVALID_ARG, "q, lam, k, v, o and the states must be 16-byte aligned");
    if (n_tokens > 0 && (o == q || o == lam || o == v || (k && o == k))) return fail(LASAD_ERR_INVALID_ARG, "o aliases an input");

    lasad::ForwardArgs a;
    a.q = q; a.k = k; a.v = v; a.o = o; a.lam = lam;
    a.in = *in_layout; a.out = *o_layout;
    a.io_dtype = io_dtype; a.out_dtype = out_dtype;
    a.B = B; a.Hh = n_heads; a.d = d;
    a.grid_w = grid_w;
    a.start_pos = start_pos; a.n_tokens = n_tokens;
    a.gamma = nullptr; a.mode = boundary_mode; a.q_scale = q_scale;
    a.state_in = state_in; a.state_out = state_out;
    a.seg_states = nullptr; a.n_segments = 1; a.seg_chunks = 0;
    a.fused_act = layer ? 1 : 0; a.norm = (layer && norm_eps >= 0.f) ? 1 : 0;
    a.norm_eps = norm_eps; a.norm_w = norm_weight;
    if (n_tokens == 0 && (!state_out || state_out == state_in)) return LASAD_OK;
    hipError_t e;
    if (io_dtype == LASAD_BF16 && d == 64 && n_tokens > 0 && !force_generic())
        e = lasad::launch_forward_gated_mfma(a, (hipStream_t)hip_stream);
    else
        e = lasad::launch_forward_generic(a, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail("lasad_forward_gated launch", e);
    return LASAD_OK;
}

size_t lasad_backward_workspace_bytes(int B, int n_heads, int n_tokens, int d, int io_dtype)
{
    if (B < 1 || n_heads < 1 || n_tokens < 1 || d < 1) return 0;
    return lasad::backward_workspace_bytes((int64_t)B * n_heads, n_tokens, d, force_generic() ? LASAD_F32 : io_dtype);
}

size_t lasad_backward_carried_workspace_bytes(int B, int n_heads, int n_tokens, int d, int io_dtype)
{
    if (B < 1 || n_heads < 1 || n_tokens < 1 || d < 1) return 0;
    return lasad_backward_workspace_bytes(B, n_heads, n_tokens, d, io_dtype) +
           lasad::backward_carried_extra_bytes((int64_t)B * n_heads, d);
}

static int backward_chunked_impl(const void *q, const void *k, const void *v, const void *d_o,
                           const float *state_in, const float *d_state_out, float *d_state_in, bool carried,
                           void *dq, void *dk, void *dv, float *dgamma,
                           const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                           int io_dtype, int grad_dtype,
                           int B, int n_heads, int d, int grid_h, int grid_w,
                           int start_pos, int n_tokens,
                           const float *gamma, int boundary_mode, float q_scale,
                           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x3fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (!supported_d(d)) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (supported: 32, 64, 128)", d);
    if (start_pos < 0 || n_tokens < 0 || (int64_t)start_pos + n_tokens > (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "positions %d+1..%d+%d leave the %d x %d grid", start_pos, start_pos, n_tokens, grid_h, grid_w);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (grad_dtype != LASAD_F32 && grad_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "grad_dtype %d", grad_dtype);
    if (io_dtype == LASAD_F32 && grad_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 gradients");
    if (!gamma || !dgamma) return fail(LASAD_ERR_INVALID_ARG, "gamma or dgamma is NULL");
    if (!in_layout || !grad_layout) return fail(LASAD_ERR_INVALID_ARG, "layout is NULL");
    if (n_tokens > 0 && (!q || !k || !v || !d_o || !dq || !dk || !dv)) return fail(LASAD_ERR_INVALID_ARG, "a tensor pointer is NULL");
    const int vec = io_dtype == LASAD_BF16 ? 8 : 4, gvec = grad_dtype == LASAD_BF16 ? 8 : 4;
    if (in_layout->stride_b % vec || in_layout->stride_n % vec || in_layout->stride_h % vec ||
        in_layout->stride_b < 0 || in_layout->stride_n < 0 || in_layout->stride_h < 0)
        return fail(LASAD_ERR_INVALID_ARG, "input strides must be non-negative multiples of %d elements", vec);
    if (grad_layout->stride_b % gvec || grad_layout->stride_n % gvec || grad_layout->stride_h % gvec ||
        grad_layout->stride_b < 0 || grad_layout->stride_n < 0 || grad_layout->stride_h < 0)
        return fail(LASAD_ERR_INVALID_ARG, "gradient strides must be non-negative multiples of %d elements", gvec);
    if (n_tokens > 0 && (in_layout->stride_n < d || grad_layout->stride_n < d))
        return fail(LASAD_ERR_INVALID_ARG, "token stride smaller than the head dim");
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(d_o, 16) ||
        !aligned(dq, 16) || !aligned(dk, 16) || !aligned(dv, 16) || !aligned(workspace, 256))
        return fail(LASAD_ERR_INVALID_ARG, "tensors must be 16-byte aligned, the workspace 256-byte aligned");
    if (!aligned(state_in, 16) || !aligned(d_state_out, 16) || !aligned(d_state_in, 16))
        return fail(LASAD_ERR_INVALID_ARG, "the states must be 16-byte aligned");
    if (d_state_in && (d_state_in == state_in || d_state_in == d_state_out))
        return fail(LASAD_ERR_INVALID_ARG, "d_state_in aliases an input state");
    if (d_state_out && !(q_scale != 0.f))
        return fail(LASAD_ERR_UNSUPPORTED, "q_scale = 0 with a gradient of the final state");
    const void *ins[4] = {q, k, v, d_o};
    void *outs[3] = {dq, dk, dv};
    for (int i = 0; n_tokens > 0 && i < 3; ++i) {
        for (int j = 0; j < 4; ++j)
            if (outs[i] == ins[j]) return fail(LASAD_ERR_INVALID_ARG, "a gradient buffer aliases an input");
        for (int j = i + 1; j < 3; ++j)
            if (outs[i] == outs[j]) return fail(LASAD_ERR_INVALID_ARG, "two gradient buffers alias");
    }
    hipStream_t s = (hipStream_t)hip_stream;
    if (n_tokens == 0) {                                  // no token: the state passes through, so does its gradient
        hipError_t e = lasad::launch_zero_f32(dgamma, n_heads, s);
        if (e == hipSuccess && d_state_in)
            e = lasad::launch_copy_state(d_state_out, d_state_in, (int64_t)B * n_heads * d * d, s);
        if (e != hipSuccess) return hip_fail("lasad_backward_chunked", e);
        return LASAD_OK;
    }
    const size_t need = carried ? lasad_backward_carried_workspace_bytes(B, n_heads, n_tokens, d, io_dtype)
                                : lasad_backward_workspace_bytes(B, n_heads, n_tokens, d, io_dtype);
    if (!workspace || workspace_bytes < need)
        return fail(LASAD_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : (size_t)0, need);

    lasad::BackwardArgs a;
    a.q = q; a.k = k; a.v = v; a.d_o = d_o; a.dq = dq; a.dk = dk; a.dv = dv; a.dgamma = dgamma;
    a.in = *in_layout; a.grad = *grad_layout;
    a.io_dtype = io_dtype; a.grad_dtype = grad_dtype;
    a.B = B; a.Hh = n_heads; a.d = d; a.grid_w = grid_w;
    a.start_pos = start_pos; a.n_tokens = n_tokens;
    a.gamma = gamma; a.mode = boundary_mode; a.q_scale = q_scale;
    a.workspace = workspace; a.dq32 = a.dk32 = a.seq_sums = nullptr;
    a.state_in = state_in; a.d_state_out = d_state_out; a.d_state_in = d_state_in;
    const bool use_mfma = io_dtype == LASAD_BF16 && d == 64 && !force_generic();
    hipError_t e = lasad::launch_backward(a, use_mfma, s);
    if (e != hipSuccess) return hip_fail("lasad_backward_chunked launch", e);
    return LASAD_OK;
}

int lasad_backward_chunked(const void *q, const void *k, const void *v, const void *d_o,
                           void *dq, void *dk, void *dv, float *dgamma,
                           const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                           int io_dtype, int grad_dtype,
                           int B, int n_heads, int d, int grid_h, int grid_w,
                           int start_pos, int n_tokens,
                           const float *gamma, int boundary_mode, float q_scale,
                           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return backward_chunked_impl(q, k, v, d_o, nullptr, nullptr, nullptr, false, dq, dk, dv, dgamma, in_layout, grad_layout,
                                 io_dtype, grad_dtype, B, n_heads, d, grid_h, grid_w, start_pos, n_tokens, gamma,
                                 boundary_mode, q_scale, workspace, workspace_bytes, hip_stream);
}

int lasad_backward_chunked_carried(const void *q, const void *k, const void *v, const void *d_o,
                                   const float *state_in, const float *d_state_out,
                                   void *dq, void *dk, void *dv, float *dgamma, float *d_state_in,
                                   const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                                   int io_dtype, int grad_dtype,
                                   int B, int n_heads, int d, int grid_h, int grid_w,
                                   int start_pos, int n_tokens,
                                   const float *gamma, int boundary_mode, float q_scale,
                                   void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return backward_chunked_impl(q, k, v, d_o, state_in, d_state_out, d_state_in, true, dq, dk, dv, dgamma, in_layout,
                                 grad_layout, io_dtype, grad_dtype, B, n_heads, d, grid_h, grid_w, start_pos, n_tokens,
                                 gamma, boundary_mode, q_scale, workspace, workspace_bytes, hip_stream);
}

size_t lasad_backward_gated_workspace_bytes(int B, int n_heads, int n_tokens, int d)
{
    if (B < 1 || n_heads < 1 || n_tokens < 1 || d < 1) return 0;
    return lasad::backward_gated_workspace_bytes((int64_t)B * n_heads, n_tokens, d);
}

size_t lasad_backward_gated_carried_workspace_bytes(int B, int n_heads, int n_tokens, int d)
{
    if (B < 1 || n_heads < 1 || n_tokens < 1 || d < 1) return 0;
    return lasad_backward_gated_workspace_bytes(B, n_heads, n_tokens, d) +
           lasad::backward_gated_carried_extra_bytes((int64_t)B * n_heads, d);
}

static int backward_gated_impl(const void *q, const void *lam, const void *k, const void *v, const void *d_o,
                         const float *state_in, const float *d_state_out, float *d_state_in, bool carried,
                         void *dq, void *dlam, void *dk, void *dv,
                         const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                         int io_dtype, int grad_dtype,
                         int B, int n_heads, int d, int grid_h, int grid_w,
                         int start_pos, int n_tokens, int boundary_mode, float q_scale,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x3fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (!supported_d(d)) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (supported: 32, 64, 128)", d);
    if (start_pos < 0 || n_tokens < 0 || (int64_t)start_pos + n_tokens > (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "positions %d+1..%d+%d leave the %d x %d grid", start_pos, start_pos, n_tokens, grid_h, grid_w);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (grad_dtype != LASAD_F32 && grad_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "grad_dtype %d", grad_dtype);
    if (io_dtype == LASAD_F32 && grad_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 gradients");
    if (!in_layout || !grad_layout) return fail(LASAD_ERR_INVALID_ARG, "layout is NULL");
    if ((k != nullptr) != (dk != nullptr)) return fail(LASAD_ERR_INVALID_ARG, "dk must be given exactly when k is");
    if (n_tokens > 0 && (!q || !lam || !v || !d_o || !dq || !dlam || !dv)) return fail(LASAD_ERR_INVALID_ARG, "a tensor pointer is NULL");
    const int vec = io_dtype == LASAD_BF16 ? 8 : 4, gvec = grad_dtype == LASAD_BF16 ? 8 : 4;
    if (in_layout->stride_b % vec || in_layout->stride_n % vec || in_layout->stride_h % vec ||
        in_layout->stride_b < 0 || in_layout->stride_n < 0 || in_layout->stride_h < 0)
        return fail(LASAD_ERR_INVALID_ARG, "input strides must be non-negative multiples of %d elements", vec);
    if (grad_layout->stride_b % gvec || grad_layout->stride_n % gvec || grad_layout->stride_h % gvec ||
        grad_layout->stride_b < 0 || grad_layout->stride_n < 0 || grad_layout->stride_h < 0)
        return fail(LASAD_ERR_INVALID_ARG, "gradient strides must be non-negative multiples of %d elements", gvec);
    if (n_tokens > 0 && (in_layout->stride_n < d || grad_layout->stride_n < d))
        return fail(LASAD_ERR_INVALID_ARG, "token stride smaller than the head dim");
    if (!aligned(q, 16) || !aligned(lam, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(d_o, 16) ||
        !aligned(dq, 16) || !aligned(dlam, 16) || !aligned(dk, 16) || !aligned(dv, 16) || !aligned(workspace, 256))
        return fail(LASAD_ERR_INVALID_ARG, "tensors must be 16-byte aligned, the workspace 256-byte aligned");
    if (!aligned(state_in, 16) || !aligned(d_state_out, 16) || !aligned(d_state_in, 16))
        return fail(LASAD_ERR_INVALID_ARG, "the states must be 16-byte aligned");
    if (d_state_in && (d_state_in == state_in || d_state_in == d_state_out))
        return fail(LASAD_ERR_INVALID_ARG, "d_state_in aliases an input state");
    if (d_state_out && !(q_scale != 0.f))
        return fail(LASAD_ERR_UNSUPPORTED, "q_scale = 0 with a gradient of the final state");
    const void *ins[5] = {q, lam, k, v, d_o};
    void *outs[4] = {dq, dlam, dk, dv};
    for (int i = 0; n_tokens > 0 && i < 4; ++i) {
        if (!outs[i]) continue;
        for (int j = 0; j < 5; ++j)
            if (outs[i] == ins[j]) return fail(LASAD_ERR_INVALID_ARG, "a gradient buffer aliases an input");
        for (int j = i + 1; j < 4; ++j)
            if (outs[i] == outs[j]) return fail(LASAD_ERR_INVALID_ARG, "two gradient buffers alias");
    }
    if (n_tokens == 0) {                                  // no token: the state passes through, so does its gradient
        if (d_state_in) {
            hipError_t e0 = lasad::launch_copy_state(d_state_out, d_state_in, (int64_t)B * n_heads * d * d, (hipStream_t)hip_stream);
            if (e0 != hipSuccess) return hip_fail("lasad_backward_gated", e0);
        }
        return LASAD_OK;
    }
    const size_t need = carried ? lasad_backward_gated_carried_workspace_bytes(B, n_heads, n_tokens, d)
                                : lasad_backward_gated_workspace_bytes(B, n_heads, n_tokens, d);
    if (!workspace || workspace_bytes < need)
        return fail(LASAD_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : (size_t)0, need);

    lasad::GatedBackwardArgs a;
    a.q = q; a.lam = lam; a.k = k; a.v = v; a.d_o = d_o;
    a.dq = dq; a.dlam = dlam; a.dk = dk; a.dv = dv;
    a.in = *in_layout; a.grad = *grad_layout;
    a.io_dtype = io_dtype; a.grad_dtype = grad_dtype;
    a.B = B; a.Hh = n_heads; a.d = d; a.grid_w = grid_w;
    a.start_pos = start_pos; a.n_tokens = n_tokens;
    a.mode = boundary_mode; a.q_scale = q_scale;
    a.workspace = workspace;
    a.fused_act = 0; a.d_o_lo = nullptr;
    a.state_in = state_in; a.d_state_out = d_state_out; a.d_state_in = d_state_in;
    hipError_t e = lasad::launch_backward_gated(a, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail("lasad_backward_gated launch", e);
    return LASAD_OK;
}

int lasad_backward_gated(const void *q, const void *lam, const void *k, const void *v, const void *d_o,
                         void *dq, void *dlam, void *dk, void *dv,
                         const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                         int io_dtype, int grad_dtype,
                         int B, int n_heads, int d, int grid_h, int grid_w,
                         int start_pos, int n_tokens, int boundary_mode, float q_scale,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return backward_gated_impl(q, lam, k, v, d_o, nullptr, nullptr, nullptr, false, dq, dlam, dk, dv, in_layout, grad_layout,
                               io_dtype, grad_dtype, B, n_heads, d, grid_h, grid_w, start_pos, n_tokens, boundary_mode,
                               q_scale, workspace, workspace_bytes, hip_stream);
}

int lasad_backward_gated_carried(const void *q, const void *lam, const void *k, const void *v, const void *d_o,
                                 const float *state_in, const float *d_state_out,
                                 void *dq, void *dlam, void *dk, void *dv, float *d_state_in,
                                 const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                                 int io_dtype, int grad_dtype,
                                 int B, int n_heads, int d, int grid_h, int grid_w,
                                 int start_pos, int n_tokens, int boundary_mode, float q_scale,
                                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return backward_gated_impl(q, lam, k, v, d_o, state_in, d_state_out, d_state_in, true, dq, dlam, dk, dv, in_layout,
                               grad_layout, io_dtype, grad_dtype, B, n_heads, d, grid_h, grid_w, start_pos, n_tokens,
                               boundary_mode, q_scale, workspace, workspace_bytes, hip_stream);
}

static bool bad_strides(const lasad_layout_t *l, int vec)
{
    return l->stride_b % vec || l->stride_n % vec || l->stride_h % vec || l->stride_b < 0 || l->stride_n < 0 || l->stride_h < 0;
}

size_t lasad_backward_layer_workspace_bytes(int B, int n_heads, int n_tokens, int d, int io_dtype,
                                            const lasad_layout_t *in_layout)
{
    if (B < 1 || n_heads < 1 || n_tokens < 1 || d < 1 || !in_layout) return 0;
    if (in_layout->stride_b < 0 || in_layout->stride_n < 0 || in_layout->stride_h < 0) return 0;
    return lasad::backward_layer_workspace_bytes(B, n_heads, n_tokens, d, io_dtype, *in_layout);
}

// d_o_out NULL: the whole backward (gradients dq_pre, dz, dv with grad_layout / grad_dtype);
// else only the normalisation's part: d_o_out (grad_layout, grad_dtype) and dweight.
static int backward_layer_common(const void *q_pre, const void *z, const void *v, const void *d_out,
                                 void *dq_pre, void *dz, void *dv, void *d_o_out, float *dweight,
                                 const lasad_layout_t *in_layout, const lasad_layout_t *dout_layout,
                                 const lasad_layout_t *grad_layout,
                                 int io_dtype, int grad_dtype,
                                 int B, int n_heads, int d, int grid_h, int grid_w,
                                 int start_pos, int n_tokens, int boundary_mode, float q_scale,
                                 const float *norm_weight, float norm_eps,
                                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const bool norm_only = d_o_out != nullptr;
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x3fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (d != 64) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (the layer backward supports 64)", d);
    if (start_pos < 0 || n_tokens < 0 || (int64_t)start_pos + n_tokens > (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "positions %d+1..%d+%d leave the %d x %d grid", start_pos, start_pos, n_tokens, grid_h, grid_w);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (grad_dtype != LASAD_F32 && grad_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "grad_dtype %d", grad_dtype);
    if (io_dtype == LASAD_F32 && grad_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 gradients");
    if (!in_layout || !dout_layout || !grad_layout) return fail(LASAD_ERR_INVALID_ARG, "layout is NULL");
    if (n_tokens > 0 && (!q_pre || !z || !v || !d_out)) return fail(LASAD_ERR_INVALID_ARG, "a tensor pointer is NULL");
    if (norm_only && norm_eps < 0.f) return fail(LASAD_ERR_INVALID_ARG, "norm_eps < 0: there is no normalisation to differentiate");
    const int vec = io_dtype == LASAD_BF16 ? 8 : 4, gvec = grad_dtype == LASAD_BF16 ? 8 : 4;
    if (bad_strides(in_layout, vec) || bad_strides(dout_layout, vec))
        return fail(LASAD_ERR_INVALID_ARG, "input strides must be non-negative multiples of %d elements", vec);
    if (bad_strides(grad_layout, gvec))
        return fail(LASAD_ERR_INVALID_ARG, "gradient strides must be non-negative multiples of %d elements", gvec);
    if (n_tokens > 0 && (in_layout->stride_n < d || dout_layout->stride_n < d || grad_layout->stride_n < d))
        return fail(LASAD_ERR_INVALID_ARG, "token stride smaller than the head dim");
    if (!aligned(q_pre, 16) || !aligned(z, 16) || !aligned(v, 16) || !aligned(d_out, 16) || !aligned(dq_pre, 16) ||
        !aligned(dz, 16) || !aligned(dv, 16) || !aligned(d_o_out, 16) || !aligned(dweight, 16) || !aligned(norm_weight, 16) || !aligned(workspace, 256))
        return fail(LASAD_ERR_INVALID_ARG, "tensors must be 16-byte aligned, the workspace 256-byte aligned");
    const void *ins[4] = {q_pre, z, v, d_out};
    void *outs[3] = {norm_only ? d_o_out : dq_pre, dz, dv};
    const int n_outs = norm_only ? 1 : 3;
    for (int i = 0; n_tokens > 0 && i < n_outs; ++i) {
        for (int j = 0; j < 4; ++j)
            if (outs[i] == ins[j]) return fail(LASAD_ERR_INVALID_ARG, "a gradient buffer aliases an input");
        for (int j = i + 1; j < n_outs; ++j)
            if (outs[i] == outs[j]) return fail(LASAD_ERR_INVALID_ARG, "two gradient buffers alias");
    }
    if (n_tokens == 0) {
        if (dweight) {
            hipError_t e0 = lasad::launch_zero_f32(dweight, n_heads * d, (hipStream_t)hip_stream);
            if (e0 != hipSuccess) return hip_fail("lasad_backward_layer launch", e0);
        }
        return LASAD_OK;
    }
    const size_t need = lasad_backward_layer_workspace_bytes(B, n_heads, n_tokens, d, io_dtype, in_layout);
    if (!workspace || workspace_bytes < need)
        return fail(LASAD_ERR_WORKSPACE, "workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : (size_t)0, need);

    lasad::LayerBackwardArgs a;
    a.q_pre = q_pre; a.z = z; a.v = v; a.d_out = d_out;
    a.dq_pre = dq_pre; a.dz = dz; a.dv = dv; a.dweight = dweight;
    a.d_o_out = d_o_out; a.d_o_l = *grad_layout; a.d_o_f32 = (norm_only && grad_dtype == LASAD_F32) ? 1 : 0;
    a.in = *in_layout; a.dout = *dout_layout; a.grad = *grad_layout;
    a.io_dtype = io_dtype; a.grad_dtype = grad_dtype;
    a.B = B; a.Hh = n_heads; a.d = d; a.grid_w = grid_w;
    a.start_pos = start_pos; a.n_tokens = n_tokens;
    a.mode = boundary_mode; a.q_scale = q_scale;
    a.norm_w = norm_weight; a.norm_eps = norm_eps;
    a.workspace = workspace;
    hipError_t e = lasad::launch_backward_layer(a, !force_generic(), (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail("lasad_backward_layer launch", e);
    return LASAD_OK;
}

int lasad_backward_layer(const void *q_pre, const void *z, const void *v, const void *d_out,
                         void *dq_pre, void *dz, void *dv, float *dweight,
                         const lasad_layout_t *in_layout, const lasad_layout_t *dout_layout,
                         const lasad_layout_t *grad_layout,
                         int io_dtype, int grad_dtype,
                         int B, int n_heads, int d, int grid_h, int grid_w,
                         int start_pos, int n_tokens, int boundary_mode, float q_scale,
                         const float *norm_weight, float norm_eps,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (n_tokens > 0 && (!dq_pre || !dz || !dv)) return fail(LASAD_ERR_INVALID_ARG, "a tensor pointer is NULL");
    return backward_layer_common(q_pre, z, v, d_out, dq_pre, dz, dv, nullptr, dweight, in_layout, dout_layout, grad_layout,
                                 io_dtype, grad_dtype, B, n_heads, d, grid_h, grid_w, start_pos, n_tokens, boundary_mode,
                                 q_scale, norm_weight, norm_eps, workspace, workspace_bytes, hip_stream);
}

int lasad_backward_layer_norm(const void *q_pre, const void *z, const void *v, const void *d_out,
                              void *d_o, float *dweight,
                              const lasad_layout_t *in_layout, const lasad_layout_t *dout_layout,
                              const lasad_layout_t *d_o_layout, int io_dtype, int d_o_dtype,
                              int B, int n_heads, int d, int grid_h, int grid_w,
                              int start_pos, int n_tokens, int boundary_mode, float q_scale,
                              const float *norm_weight, float norm_eps,
                              void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!d_o) return fail(LASAD_ERR_INVALID_ARG, "d_o is NULL");
    return backward_layer_common(q_pre, z, v, d_out, nullptr, nullptr, nullptr, d_o, dweight, in_layout, dout_layout, d_o_layout,
                                 io_dtype, d_o_dtype, B, n_heads, d, grid_h, grid_w, start_pos, n_tokens, boundary_mode,
                                 q_scale, norm_weight, norm_eps, workspace, workspace_bytes, hip_stream);
}

int lasad_forward_gated(const void *q, const void *lam, const void *k, const void *v, void *o,
                        const lasad_layout_t *in_layout, const lasad_layout_t *o_layout,
                        int io_dtype, int out_dtype,
                        int B, int n_heads, int d, int grid_h, int grid_w,
                        int start_pos, int n_tokens, int boundary_mode, float q_scale,
                        const float *state_in, float *state_out, void *hip_stream)
{
    return forward_gated_common(q, lam, k, v, o, in_layout, o_layout, io_dtype, out_dtype, B, n_heads, d, grid_h, grid_w,
                                start_pos, n_tokens, boundary_mode, q_scale, state_in, state_out, hip_stream,
                                0, nullptr, -1.f);
}

int lasad_forward_layer(const void *q_pre, const void *z, const void *v, void *o,
                        const lasad_layout_t *in_layout, const lasad_layout_t *o_layout,
                        int io_dtype, int out_dtype,
                        int B, int n_heads, int d, int grid_h, int grid_w,
                        int start_pos, int n_tokens, int boundary_mode, float q_scale,
                        const float *norm_weight, float norm_eps,
                        const float *state_in, float *state_out, void *hip_stream)
{
    return forward_gated_common(q_pre, z, nullptr, v, o, in_layout, o_layout, io_dtype, out_dtype, B, n_heads, d, grid_h, grid_w,
                                start_pos, n_tokens, boundary_mode, q_scale, state_in, state_out, hip_stream,
                                1, norm_weight, norm_eps);
}

static int decode_gated_common(const void *q, const void *lam, const void *k, const void *v, void *o,
                               int io_dtype, int out_dtype, int B, int n_heads, int d,
                               int grid_h, int grid_w, int pos, int boundary_mode, float q_scale,
                               float *state, void *hip_stream,
                               int layer, const float *norm_weight, float norm_eps)
{
    if (layer && !aligned(norm_weight, 16)) return fail(LASAD_ERR_INVALID_ARG, "norm_weight must be 16-byte aligned");
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x7fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (!supported_d(d)) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (supported: 32, 64, 128)", d);
    if (pos < 0 || (int64_t)pos >= (int64_t)grid_h * grid_w)
        return fail(LASAD_ERR_INVALID_ARG, "pos %d is outside the %d x %d grid", pos, grid_h, grid_w);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (out_dtype != LASAD_F32 && out_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "out_dtype %d", out_dtype);
    if (io_dtype == LASAD_F32 && out_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 output");
    if (!q || !lam || !v || !o || !state) return fail(LASAD_ERR_INVALID_ARG, "a required pointer is NULL");
    if (!aligned(q, 16) || !aligned(lam, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) || !aligned(state, 16))
        return fail(LASAD_ERR_INVALID_ARG, "q, lam, k, v, o and state must be 16-byte aligned");
    if (o == q || o == lam || o == v || (k && o == k)) return fail(LASAD_ERR_INVALID_ARG, "o aliases an input");

    lasad::DecodeArgs a;
    a.q = q; a.k = k; a.v = v; a.o = o; a.lam = lam;
    a.io_dtype = io_dtype; a.out_dtype = out_dtype;
    a.B = B; a.Hh = n_heads; a.d = d;
    a.grid_w = grid_w; a.pos = pos; a.pos_rows = nullptr; a.grid_n = grid_h * grid_w;
    a.fused_act = 0; a.norm = 0; a.norm_eps = 0.f; a.norm_w = nullptr;
    a.gamma = nullptr; a.mode = boundary_mode; a.q_scale = q_scale;
    a.state = state;
    a.fused_act = layer ? 1 : 0; a.norm = (layer && norm_eps >= 0.f) ? 1 : 0;
    a.norm_eps = norm_eps; a.norm_w = norm_weight;
    hipError_t e = lasad::launch_decode(a, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail("lasad_decode_step_gated launch", e);
    return LASAD_OK;
}

int lasad_decode_step_gated(const void *q, const void *lam, const void *k, const void *v, void *o,
                            int io_dtype, int out_dtype, int B, int n_heads, int d,
                            int grid_h, int grid_w, int pos, int boundary_mode, float q_scale,
                            float *state, void *hip_stream)
{
    return decode_gated_common(q, lam, k, v, o, io_dtype, out_dtype, B, n_heads, d, grid_h, grid_w, pos, boundary_mode,
                               q_scale, state, hip_stream, 0, nullptr, -1.f);
}

int lasad_decode_step_layer(const void *q_pre, const void *z, const void *v, void *o,
                            int io_dtype, int out_dtype, int B, int n_heads, int d,
                            int grid_h, int grid_w, int pos, int boundary_mode, float q_scale,
                            const float *norm_weight, float norm_eps,
                            float *state, void *hip_stream)
{
    return decode_gated_common(q_pre, z, nullptr, v, o, io_dtype, out_dtype, B, n_heads, d, grid_h, grid_w, pos, boundary_mode,
                               q_scale, state, hip_stream, 1, norm_weight, norm_eps);
}

int lasad_decode_step_rows(const void *q, const void *lam, const void *k, const void *v, void *o,
                           int io_dtype, int out_dtype, int B, int n_heads, int d,
                           int grid_h, int grid_w, const int32_t *pos_rows,
                           const float *gamma, int boundary_mode, float q_scale,
                           float *state, void *hip_stream)
{
    if (int rc = check_grid(grid_h, grid_w, boundary_mode)) return rc;
    if (B < 1 || n_heads < 1) return fail(LASAD_ERR_INVALID_ARG, "B = %d, n_heads = %d", B, n_heads);
    if ((int64_t)B * n_heads > 0x7fffffff) return fail(LASAD_ERR_INVALID_ARG, "B * n_heads overflows the launch grid");
    if (!supported_d(d)) return fail(LASAD_ERR_UNSUPPORTED, "head dim %d (supported: 32, 64, 128)", d);
    if (io_dtype != LASAD_F32 && io_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "io_dtype %d", io_dtype);
    if (out_dtype != LASAD_F32 && out_dtype != LASAD_BF16) return fail(LASAD_ERR_INVALID_ARG, "out_dtype %d", out_dtype);
    if (io_dtype == LASAD_F32 && out_dtype == LASAD_BF16) return fail(LASAD_ERR_UNSUPPORTED, "fp32 inputs with bf16 output");
    if (!q || !v || !o || !state || !pos_rows) return fail(LASAD_ERR_INVALID_ARG, "a required pointer is NULL");
    if (lam && gamma) return fail(LASAD_ERR_INVALID_ARG, "give either lam (vector decay) or gamma (scalar decay), not both");
    if (!lam && (!gamma || !k)) return fail(LASAD_ERR_INVALID_ARG, "the scalar-decay step needs gamma and k");
    if (!aligned(q, 16) || !aligned(lam, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(o, 16) ||
        !aligned(state, 16) || !aligned(pos_rows, 4))
        return fail(LASAD_ERR_INVALID_ARG, "q, lam, k, v, o and state must be 16-byte aligned");
    if (o == q || o == v || (lam && o == lam) || (k && o == k)) return fail(LASAD_ERR_INVALID_ARG, "o aliases an input");

    lasad::DecodeArgs a;
    a.q = q; a.k = k; a.v = v; a.o = o; a.lam = lam;
    a.io_dtype = io_dtype; a.out_dtype = out_dtype;
    a.B = B; a.Hh = n_heads; a.d = d;
    a.grid_w = grid_w; a.pos = 0; a.pos_rows = pos_rows; a.grid_n = grid_h * grid_w;
    a.fused_act = 0; a.norm = 0; a.norm_eps = 0.f; a.norm_w = nullptr;
    a.gamma = gamma; a.mode = boundary_mode; a.q_scale = q_scale;
    a.state = state;
    hipError_t e = lasad::launch_decode(a, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail("lasad_decode_step_rows launch", e);
    return LASAD_OK;
}

}  // extern "C"
