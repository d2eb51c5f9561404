// Backward pass of the scalar-decay forward (gradients of the Section 3.4 recurrence from a zero
// state): dq, dk, dv and the gradient of the per-head base decay.
//
// With M[i][j] = prod_{s=j+1..i} lambda_s (j <= i) and g_i = dL/do_i, the forward
// o_i = q_scale sum_{j<=i} M[i][j] (q_i . k_j) v_j gives
//
//   dq_i = q_scale sum_{j<=i} M[i][j] (g_i . v_j) k_j      -- the forward itself with (q, k, v) := (g, v, k)
//   dv_j = q_scale sum_{i>=j} M[i][j] (q_i . k_j) g_i      -- the forward over the REVERSED sequence, (k, q, g)
//   dk_j = q_scale sum_{i>=j} M[i][j] (g_i . v_j) q_i      -- the forward over the reversed sequence, (v, g, q)
//
// In reversed token order m = n-1-t the decay between two tokens is still a product of the
// lambdas of the steps between them, with the decay of original token s now applied at
// reversed step n-s: the boundary pattern is the original one mirrored and shifted by one, which
// for a raster grid is again "every W-th position" and is obtained by giving the forward
// kernels a different start column.  Reversal itself costs nothing: the kernels address tokens
// as base + token * stride, so the reversed passes get a base pointer at the last token and a
// negative token stride.  The three passes therefore run the forward kernels unchanged (bf16
// matrix-core kernel, fp32 scan kernel or generic kernel, as the forward would choose).
//
// Decay gradient.  Write the decay applied at token t as exp(a_t) and G_i = a_1 + .. + a_i; L
// depends on the a's only through G_i - G_j, and dL/dG_i = q_i . dq_i - k_i . dk_i.  Every
// non-boundary token has a_t = log gamma_h, so with E_i = number of non-boundary tokens among the
// first i tokens of the call
//
//   dL/dgamma_h = (1 / gamma_h) sum_b sum_i E_i (q_i . dq_i - k_i . dk_i).
//
// bf16 inputs, head dim 64, enough sequences (or sequences too short to be cut into segments):
// ONE launch of the wave-specialised forward kernel runs the three passes side by side.  Each
// pass stores its gradient in the caller's type and layout, and the dq and dk passes add up
// E_i (q_i . dq_i) and -E_i (k_i . dk_i) from their fp32 output tiles before those are rounded
// (a per-wave partial sum per sequence, fixed order); a small kernel (one workgroup per head)
// adds the partial sums in a fixed order (no atomics) and divides by gamma.
//
// Otherwise (fp32 inputs, other head dims, few long sequences): three separate passes; dq and dk
// are produced in fp32 into the workspace, a finishing kernel (one workgroup per 64 tokens of a
// sequence) forms its part of the sum above (fp32, fixed order) and stores dq, dk in the caller's
// type and layout, and a last small kernel (one wave per head) adds the partial sums.
//
// Carried states.  When the call starts from a state s_0 and the loss also depends on the final state s_n
// (H = dL/ds_n given), the three passes keep their form: the dq pass is the forward recurrence on S^T, so it
// starts from s_0^T (and ends with s_n^T); the reversed passes run the recurrence of the state gradient
// g_t = lambda_{t+1} g_{t+1} + q_scale q_t d_o_t^T, g_n = H + q_scale q_n d_o_n^T, so they start from H (dv pass)
// and H^T (dk pass) with NO decay at their first step; the dv pass ends with g_1, and dL/ds_0 = lambda_1 g_1.
// The decay gradient gains one term: L depends on the cumulative decays also through s_n, which adds
// E_n <H, s_n> to the sum above (E_n: non-boundary tokens of the call).  A preparation kernel makes the
// transposed copies (H divided by q_scale: the kernels multiply their outputs by it, and g_t carries it only on
// the q d_o^T part), a finishing kernel forms dL/ds_0 and <H, s_n> per sequence.
#include "lasad_internal.h"

namespace lasad {

namespace {

constexpr int kFinThreads = 256;
constexpr int kFinTokens = 64;       // tokens per workgroup of the finishing kernel

template <int IN_BF16, int OUT_BF16>
__global__ void __launch_bounds__(kFinThreads)
backward_finish_kernel(BackwardArgs a)
{
    __shared__ float red[kFinThreads / 64];
    const int nblk = (a.n_tokens + kFinTokens - 1) / kFinTokens;
    const int bh = blockIdx.x / nblk, blk = blockIdx.x - bh * nblk;
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const int d = a.d;
    const int tb = blk * kFinTokens, n = min(kFinTokens, a.n_tokens - tb);   // this workgroup's tokens
    const int vec_per_tok = d / 4;                       // 4 channels per thread and step
    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    const int64_t g_base = (int64_t)b * a.grad.stride_b + (int64_t)h * a.grad.stride_h;
    const int64_t w_base = ((int64_t)b * a.n_tokens * a.Hh + h) * d;      // workspace: [B][n][Hh][d] fp32
    const int64_t w_stride_n = (int64_t)a.Hh * d;
    const int e0 = cum_exp(a.start_pos, a.grid_w, a.mode);

    float acc = 0.f;
    for (int i = threadIdx.x; i < n * vec_per_tok; i += kFinThreads) {
        const int t = tb + i / vec_per_tok, c = (i % vec_per_tok) * 4;
        const float4 dq4 = *(const float4 *)(a.dq32 + w_base + t * w_stride_n + c);
        const float4 dk4 = *(const float4 *)(a.dk32 + w_base + t * w_stride_n + c);
        const int64_t ii = in_base + (int64_t)t * a.in.stride_n + c;
        float q4[4], k4[4];
        if (IN_BF16) {
            const uint2 qr = *(const uint2 *)((const uint16_t *)a.q + ii);
            const uint2 kr = *(const uint2 *)((const uint16_t *)a.k + ii);
            q4[0] = __uint_as_float(qr.x << 16); q4[1] = __uint_as_float(qr.x & 0xffff0000u);
            q4[2] = __uint_as_float(qr.y << 16); q4[3] = __uint_as_float(qr.y & 0xffff0000u);
            k4[0] = __uint_as_float(kr.x << 16); k4[1] = __uint_as_float(kr.x & 0xffff0000u);
            k4[2] = __uint_as_float(kr.y << 16); k4[3] = __uint_as_float(kr.y & 0xffff0000u);
        } else {
            const float4 qr = *(const float4 *)((const float *)a.q + ii);
            const float4 kr = *(const float4 *)((const float *)a.k + ii);
            q4[0] = qr.x; q4[1] = qr.y; q4[2] = qr.z; q4[3] = qr.w;
            k4[0] = kr.x; k4[1] = kr.y; k4[2] = kr.z; k4[3] = kr.w;
        }
        const float dot = (q4[0] * dq4.x - k4[0] * dk4.x) + (q4[1] * dq4.y - k4[1] * dk4.y) +
                          (q4[2] * dq4.z - k4[2] * dk4.z) + (q4[3] * dq4.w - k4[3] * dk4.w);
        const int e = cum_exp(a.start_pos + t + 1, a.grid_w, a.mode) - e0;
        acc = fmaf((float)e, dot, acc);
        const int64_t gi = g_base + (int64_t)t * a.grad.stride_n + c;
        if (OUT_BF16) {
            uint2 w;
            w.x = (uint32_t)float_to_bf16_bits(dq4.x) | ((uint32_t)float_to_bf16_bits(dq4.y) << 16);
            w.y = (uint32_t)float_to_bf16_bits(dq4.z) | ((uint32_t)float_to_bf16_bits(dq4.w) << 16);
            *(uint2 *)((uint16_t *)a.dq + gi) = w;
            w.x = (uint32_t)float_to_bf16_bits(dk4.x) | ((uint32_t)float_to_bf16_bits(dk4.y) << 16);
            w.y = (uint32_t)float_to_bf16_bits(dk4.z) | ((uint32_t)float_to_bf16_bits(dk4.w) << 16);
            *(uint2 *)((uint16_t *)a.dk + gi) = w;
        } else {
            *(float4 *)((float *)a.dq + gi) = dq4;
            *(float4 *)((float *)a.dk + gi) = dk4;
        }
    }
    // fixed-order reduction: lanes of a wave (xor butterflies), then the four waves
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) a.seq_sums[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// dgamma[h] = (1 / gamma[h]) * sum over the batch and the token blocks of the partial sums of head h.
// One wave per head: lane l adds entries l, l + 64, ... in order, then a butterfly over the lanes.
__global__ void __launch_bounds__(64)
backward_dgamma_kernel(const float *sums, const float *extra, const float *gamma, float *dgamma, int B, int Hh, int nblk)
{
    const int h = blockIdx.x;
    float acc = 0.f;
    for (int i = threadIdx.x; i < B * nblk; i += 64) {
        const int b = i / nblk, blk = i - b * nblk;
        acc += sums[((int64_t)b * Hh + h) * nblk + blk];
    }
    if (extra)                                            // E_n <dL/ds_n, s_n> of every sequence of this head
        for (int b = threadIdx.x; b < B; b += 64) acc += extra[(int64_t)b * Hh + h];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if (threadIdx.x == 0) dgamma[h] = acc / gamma[h];     // gamma = 0: the formula does not apply (inf or NaN)
}

// The same from the sums the forward kernels left: [pass (3)][B][Hh][kDotSlots]; pass 1 (dv) has none.
__global__ void __launch_bounds__(256)
backward_dgamma_slots_kernel(const float *sums, const float *extra, const float *gamma, float *dgamma, int B, int Hh)
{
    __shared__ float red[4];
    const int h = blockIdx.x;
    float acc = 0.f;
    for (int i = threadIdx.x; i < 2 * B * kDotSlots; i += 256) {
        const int pass = (i / (B * kDotSlots)) * 2, r = i % (B * kDotSlots);
        const int b = r / kDotSlots, slot = r - b * kDotSlots;
        acc += sums[(((int64_t)pass * B + b) * Hh + h) * kDotSlots + slot];
    }
    if (extra)
        for (int b = threadIdx.x; b < B; b += 256) acc += extra[(int64_t)b * Hh + h];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) dgamma[h] = ((red[0] + red[1]) + (red[2] + red[3])) / gamma[h];
}

// Per sequence: s0T = s_0^T; hS = H / q_scale and hT = H^T / q_scale (either source may be NULL).  The kernels
// multiply every output by q_scale, the state gradient g_t = H-part + q_scale (q d_o^T)-part carries q_scale only on
// its second part: the reversed passes therefore run on g_t / q_scale.
__global__ void __launch_bounds__(256)
carried_prep_kernel(const float *s0, float *s0T, const float *H, float *hS, float *hT, float inv_q_scale, int d)
{
    const int64_t off = (int64_t)blockIdx.x * d * d;
    for (int e = threadIdx.x; e < d * d; e += 256) {
        const int i = e / d, j = e - i * d;
        if (s0) s0T[off + (int64_t)j * d + i] = s0[off + e];
        if (H) {
            const float x = H[off + e] * inv_q_scale;
            hS[off + e] = x;
            hT[off + (int64_t)j * d + i] = x;
        }
    }
}

// One workgroup per sequence: dL/ds_0 = lambda_1 g_1 (g_1 / q_scale: final state of the reversed dv pass) and
// extra[bh] = E_n <H, s_n> with s_n^T the final state of the dq pass.  Fixed summation order.
__global__ void __launch_bounds__(256)
carried_finish_kernel(BackwardArgs a, const float *g1, const float *snT, float *extra)
{
    __shared__ float red[4];
    const int bh = blockIdx.x, h = bh % a.Hh, d = a.d;
    const int64_t off = (int64_t)bh * d * d;
    const float lam1 = is_boundary(a.start_pos + 1, a.grid_w, a.mode) ? 1.0f : a.gamma[h];
    float acc = 0.f;
    for (int e = threadIdx.x; e < d * d; e += 256) {
        if (a.d_state_in) a.d_state_in[off + e] = (lam1 * a.q_scale) * g1[off + e];
        if (extra) {
            const int i = e / d, j = e - i * d;
            acc = fmaf(a.d_state_out[off + e], snT[off + (int64_t)j * d + i], acc);
        }
    }
    if (!extra) return;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int en = cum_exp(a.start_pos + a.n_tokens, a.grid_w, a.mode) - cum_exp(a.start_pos, a.grid_w, a.mode);
        extra[bh] = (float)en * ((red[0] + red[1]) + (red[2] + red[3]));
    }
}

// dst = src (d_state_in of a call without tokens)
__global__ void copy_f32_kernel(const float *src, float *dst, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src ? src[i] : 0.f;
}

}  // namespace

// partial sums of the decay gradient: one per 64-token block of a sequence (finishing kernel) or
// kDotSlots per pass and sequence (sums taken inside the forward kernels), whichever is more
namespace {
__global__ void zero_f32_kernel(float *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}
}  // namespace

// p[0..n) = 0 by a kernel (a memset node in a captured graph is best avoided on this platform)
hipError_t launch_zero_f32(float *p, int n, hipStream_t s)
{
    if (n < 1) return hipSuccess;
    hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

static size_t sums_bytes(int64_t n_seq, int n_tokens)
{
    size_t per_seq = (size_t)(n_tokens + kFinTokens - 1) / kFinTokens;
    if (per_seq < 3 * kDotSlots) per_seq = 3 * kDotSlots;
    return ((size_t)n_seq * per_seq * sizeof(float) + 255) / 256 * 256;
}

size_t backward_carried_extra_bytes(int64_t n_seq, int d)
{
    // s_0^T, H / q_scale, its transpose, s_n^T (dq pass), g_1 / q_scale (dv pass), one sum per sequence
    return 5 * (size_t)n_seq * d * d * sizeof(float) + (((size_t)n_seq * sizeof(float) + 255) / 256 * 256);
}

hipError_t launch_copy_state(const float *src, float *dst, int64_t n, hipStream_t s)
{
    if (n < 1) return hipSuccess;
    hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, dst, n);
    return hipGetLastError();
}

size_t backward_workspace_bytes(int64_t n_seq, int n_tokens, int d, int io_dtype)
{
    const size_t grads = 2 * (size_t)n_seq * n_tokens * d * sizeof(float);
    const size_t sums = sums_bytes(n_seq, n_tokens);
    const size_t fwd = (io_dtype == LASAD_BF16 && d == 64) ? forward_mfma_workspace_bytes(n_seq, n_tokens) : 0;
    return grads + sums + fwd;
}

hipError_t launch_backward(const BackwardArgs &b_in, bool use_mfma, hipStream_t s)
{
    BackwardArgs b = b_in;
    const int64_t n_seq = (int64_t)b.B * b.Hh;
    const int n = b.n_tokens;
    const int elt = b.io_dtype == LASAD_BF16 ? 2 : 4;
    const int gelt = b.grad_dtype == LASAD_BF16 ? 2 : 4;
    // workspace: dq32, dk32 ([B][n][Hh][d] fp32), partial sums, forward-kernel workspace
    char *ws = (char *)b.workspace;
    const size_t one = (size_t)n_seq * n * b.d * sizeof(float);
    b.dq32 = (float *)ws;
    b.dk32 = (float *)(ws + one);
    b.seq_sums = (float *)(ws + 2 * one);
    float *fwd_ws = (float *)(ws + 2 * one + sums_bytes(n_seq, n));
    const bool has_fwd_ws = use_mfma && forward_mfma_workspace_bytes(n_seq, n) > 0;
    // carried states: transposed copies and the passes' final states follow the forward kernels' workspace
    const bool carried = b.state_in || b.d_state_out || b.d_state_in;
    const size_t mat = (size_t)n_seq * b.d * b.d;
    float *cw = (float *)((char *)fwd_ws + (use_mfma ? forward_mfma_workspace_bytes(n_seq, n) : 0));
    float *s0T = cw, *hS = cw + mat, *hT = cw + 2 * mat, *snT = cw + 3 * mat, *g1 = cw + 4 * mat, *extra = cw + 5 * mat;
    const float *st_in[3] = {nullptr, nullptr, nullptr};      // per pass (dq, dv, dk)
    float *st_out[3] = {nullptr, nullptr, nullptr};
    if (carried) {
        if (b.state_in || b.d_state_out) {
            hipLaunchKernelGGL(carried_prep_kernel, dim3((unsigned)n_seq), dim3(256), 0, s,
                               b.state_in, s0T, b.d_state_out, hS, hT, 1.0f / b.q_scale, b.d);
            hipError_t e0 = hipGetLastError();
            if (e0 != hipSuccess) return e0;
        }
        st_in[0] = b.state_in ? s0T : nullptr;
        st_out[0] = b.d_state_out ? snT : nullptr;            // s_n^T, for the decay gradient only
        st_in[1] = b.d_state_out ? hS : nullptr;
        st_out[1] = b.d_state_in ? g1 : nullptr;
        st_in[2] = b.d_state_out ? hT : nullptr;
    }
    const float *extra_sum = (carried && b.d_state_out) ? extra : nullptr;
    auto finish_carried = [&]() -> hipError_t {
        if (!carried || (!b.d_state_in && !extra_sum)) return hipSuccess;
        hipLaunchKernelGGL(carried_finish_kernel, dim3((unsigned)n_seq), dim3(256), 0, s, b, g1, snT, (float *)extra_sum);
        return hipGetLastError();
    };
    // The three passes are independent: one launch runs them side by side when that alone fills
    // the chip or when a pass would not be cut into segments anyway.  The passes then store dq, dv
    // and dk in the caller's type themselves and take the decay-gradient sums from their fp32
    // output tiles, so nothing but those sums goes through the workspace.
    const bool merged = use_mfma && (n_seq * 3 >= 192 || !has_fwd_ws);

    lasad_layout_t wl;                                   // layout of dq32 / dk32
    wl.stride_b = (int64_t)n * b.Hh * b.d; wl.stride_n = (int64_t)b.Hh * b.d; wl.stride_h = b.d;
    lasad_layout_t in_rev = b.in, grad_rev = b.grad, wl_rev = wl;
    in_rev.stride_n = -b.in.stride_n; grad_rev.stride_n = -b.grad.stride_n; wl_rev.stride_n = -wl.stride_n;

    ForwardArgs f;
    f.lam = nullptr;
    f.fused_act = 0; f.norm = 0; f.norm_eps = 0.f; f.norm_w = nullptr;
    f.io_dtype = b.io_dtype;
    f.B = b.B; f.Hh = b.Hh; f.d = b.d;
    f.grid_w = b.grid_w; f.n_tokens = n;
    f.gamma = b.gamma; f.mode = b.mode; f.q_scale = b.q_scale;
    f.state_in = nullptr; f.state_out = nullptr;
    f.seg_states = has_fwd_ws ? fwd_ws : nullptr; f.n_segments = 1; f.seg_chunks = 0;
    auto run = [&](const ForwardArgs &fa) { return use_mfma ? launch_forward_mfma(fa, s) : launch_forward_generic(fa, s); };

    const int rev_start = reversed_start(b.start_pos, n, b.grid_w, b.mode);
    hipError_t e;
    if (merged) {
        MultiPass m;
        m.n_pass = 3;
        // dq: forward order, (q, k, v) := (d_o, v, k); sum + E_t (q_t . dq_t)
        m.q[0] = b.d_o; m.k[0] = b.v; m.v[0] = b.k; m.o[0] = b.dq;
        m.in[0] = b.in; m.out[0] = b.grad; m.start_pos[0] = b.start_pos;
        m.x[0] = b.q; m.x_sign[0] = 1.f; m.x_rev[0] = 0;
        // dv: reversed order, (q, k, v) := (k, q, d_o)
        m.q[1] = last_token(b.k, b.in, n, elt); m.k[1] = last_token(b.q, b.in, n, elt); m.v[1] = last_token(b.d_o, b.in, n, elt);
        m.o[1] = (void *)last_token(b.dv, b.grad, n, gelt);
        m.in[1] = in_rev; m.out[1] = grad_rev; m.start_pos[1] = rev_start;
        m.x[1] = nullptr; m.x_sign[1] = 0.f; m.x_rev[1] = 1;
        // dk: reversed order, (q, k, v) := (v, d_o, q); sum - E_t (k_t . dk_t)
        m.q[2] = last_token(b.v, b.in, n, elt); m.k[2] = last_token(b.d_o, b.in, n, elt); m.v[2] = last_token(b.q, b.in, n, elt);
        m.o[2] = (void *)last_token(b.dk, b.grad, n, gelt);
        m.in[2] = in_rev; m.out[2] = grad_rev; m.start_pos[2] = rev_start;
        m.x[2] = last_token(b.k, b.in, n, elt); m.x_sign[2] = -1.f; m.x_rev[2] = 1;
        m.x_start_pos = b.start_pos;
        m.x_sums = b.seq_sums;
        for (int y = 0; y < 3; ++y) {
            m.state_in[y] = st_in[y]; m.state_out[y] = st_out[y];
            m.first_decay_off[y] = y > 0;                 // the reversed passes take their incoming state undecayed
        }
        f.q = m.q[0]; f.k = m.k[0]; f.v = m.v[0]; f.o = m.o[0];
        f.in = m.in[0]; f.out = m.out[0]; f.out_dtype = b.grad_dtype; f.start_pos = b.start_pos;
        f.seg_states = nullptr; f.seg_chunks = (n + 63) / 64;
        e = launch_forward_mfma_multi(f, m, s);
        if (e != hipSuccess) return e;
        e = finish_carried();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(backward_dgamma_slots_kernel, dim3((unsigned)b.Hh), dim3(256), 0, s,
                           b.seq_sums, extra_sum, b.gamma, b.dgamma, b.B, b.Hh);
        return hipGetLastError();
    } else {
        // dq (fp32, workspace): forward order, (q, k, v) := (d_o, v, k)
        f.q = b.d_o; f.k = b.v; f.v = b.k; f.o = b.dq32;
        f.in = b.in; f.out = wl; f.out_dtype = LASAD_F32; f.start_pos = b.start_pos;
        f.state_in = st_in[0]; f.state_out = st_out[0]; f.first_decay_off = 0;
        e = run(f);
        if (e != hipSuccess) return e;

        // dv (caller's buffer): reversed order, (q, k, v) := (k, q, d_o)
        f.q = last_token(b.k, b.in, n, elt); f.k = last_token(b.q, b.in, n, elt); f.v = last_token(b.d_o, b.in, n, elt);
        f.o = (void *)last_token(b.dv, b.grad, n, gelt);
        f.in = in_rev; f.out = grad_rev; f.out_dtype = b.grad_dtype;
        f.start_pos = rev_start;
        f.state_in = st_in[1]; f.state_out = st_out[1]; f.first_decay_off = 1;
        e = run(f);
        if (e != hipSuccess) return e;

        // dk (fp32, workspace): reversed order, (q, k, v) := (v, d_o, q)
        f.q = last_token(b.v, b.in, n, elt); f.k = last_token(b.d_o, b.in, n, elt); f.v = last_token(b.q, b.in, n, elt);
        f.o = (void *)last_token(b.dk32, wl, n, 4);
        f.out = wl_rev; f.out_dtype = LASAD_F32;
        f.state_in = st_in[2]; f.state_out = st_out[2]; f.first_decay_off = 1;
        e = run(f);
        if (e != hipSuccess) return e;
    }

    const int nblk = (n + kFinTokens - 1) / kFinTokens;
    if (n_seq * nblk > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(n_seq * nblk)), block(kFinThreads);
    const bool in16 = b.io_dtype == LASAD_BF16, out16 = b.grad_dtype == LASAD_BF16;
    if (in16 && out16) hipLaunchKernelGGL((backward_finish_kernel<1, 1>), grid, block, 0, s, b);
    else if (in16) hipLaunchKernelGGL((backward_finish_kernel<1, 0>), grid, block, 0, s, b);
    else if (out16) hipLaunchKernelGGL((backward_finish_kernel<0, 1>), grid, block, 0, s, b);
    else hipLaunchKernelGGL((backward_finish_kernel<0, 0>), grid, block, 0, s, b);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = finish_carried();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(backward_dgamma_kernel, dim3((unsigned)b.Hh), dim3(64), 0, s,
                       b.seq_sums, extra_sum, b.gamma, b.dgamma, b.B, b.Hh, nblk);
    return hipGetLastError();
}

}  // namespace lasad
