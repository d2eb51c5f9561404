// Backward pass of the vector-decay recurrence (Section 3.4 / Algorithm 1, zero initial state):
// dq, dv, the gradient of the decay input lambda and, with an own key, dk.  First version: fp32
// token-serial walks on the vector ALUs (lasad_scan.h), head dim 64.
//
// With l_t the decay actually applied (1 in every channel at a row boundary, lambda_t elsewhere),
// k_t the key (1 - lambda_t if tied) and g_t = dL/do_t:
//
//   forward state   S_t = diag(l_t) S_{t-1} + k_t v_t^T             dq_t = q_scale S_t g_t
//   adjoint state   G_t = diag(l_{t+1}) G_{t+1} + q_scale q_t g_t^T  dk_t = G_t v_t,  dv_t = G_t^T k_t
//
// Each of the three is the forward walk "state <- decay * state + (row operand)(column operand)^T,
// output = (row operand)^T state" with the tensors in other roles:
//
//   dq:  state S^T, decay per COLUMN l_t;      update v_t k_t^T;   output g_t^T S^T          (forward order)
//   dk:  state G^T, decay per COLUMN l_{t+1};  update g_t q_t^T;   output v_t^T G^T          (reversed order)
//   dv:  state G,   decay per ROW l_{t+1};     update q_t g_t^T;   output k_t^T G            (reversed order)
//
// Reversed order is a base pointer at the last token and a negative token stride; in that order the
// decay of step m is the lambda of the token one step EARLIER in walking order (l_{t+1}), read with a
// token shift of -1, and the row-boundary pattern is the forward one mirrored and shifted, i.e. that
// of another start column (as in the scalar-decay backward).  The three walks run in one launch.
// With bf16 inputs the three passes run on the matrix cores instead, chunk by chunk
// (lasad_backward_gated_mfma.hip, one launch per pass); the walks remain the path for fp32 inputs
// and the range fallback of those kernels (LASAD_GATED_BWD=walk forces them).
//
// Decay gradient.  L depends on l only through the products prod_{s=j+1..i} l_s[c] between a key
// j and a query i, so with r_i[c] = q_i[c] dq_i[c] - k_i[c] dk_i[c]
//
//   l_t[c] * dL/dl_t[c] = sum_{i >= t} r_i[c]            (every pair with j < t <= i, once)
//
// and dlam_t = (t a boundary or the first token ? 0 : that suffix sum / lambda_t) - (tied key: dk_t).
// The suffix sums cancel heavily, so dq and dk go through the workspace in fp32; the finishing kernel
// (one workgroup of 16 waves per sequence, lane = channel, each wave a contiguous token range: range
// sums first, then the walk down its range) forms them in a fixed order and stores dq, dk, dlam in
// the caller's type.  lambda must be > 0 where it is applied, and the result loses precision like
// 1 / lambda for very small decays (the quotient of a rounded sum).
#include <stdlib.h>
#include <string.h>

#include "lasad_scan.h"

namespace lasad {

hipError_t launch_backward_gated_pass(const ForwardArgs &a, const scan::ScanRoles &roles, int kind, int shift,
                                      int q_one_minus, hipStream_t s);

namespace {

using namespace scan;

struct WalkArgs {
    ForwardArgs common;
    ScanRoles roles[3];            // pass 0 dq, 1 dv, 2 dk
    void *o[3];
    lasad_layout_t in[3], out[3];
    int start_pos[3];
};

template <int IN_BF16, int OUT_BF16, int NJ>
__global__ void __launch_bounds__(kThreads)
backward_gated_walk_kernel(WalkArgs w)
{
    constexpr int JS = kD / NJ;            // workgroups per sequence and pass
    __shared__ __attribute__((aligned(16))) float lds[lds_floats<ROLES_ROW>()];
    const int pass = blockIdx.y;
    const int bh = blockIdx.x / JS, j0 = (blockIdx.x - bh * JS) * NJ;
    ForwardArgs a = w.common;
    a.o = w.o[pass]; a.in = w.in[pass]; a.out = w.out[pass]; a.start_pos = w.start_pos[pass];
    if (pass == 1) scan_sequence<IN_BF16, OUT_BF16, ROLES_ROW, NJ>(a, bh, j0, lds, &w.roles[1]);
    else scan_sequence<IN_BF16, 0, ROLES_COL, NJ>(a, bh, j0, lds, &w.roles[pass]);     // fp32 into the workspace
}

constexpr int kFinWaves = 16;

template <int IN_BF16, int OUT_BF16>
__global__ void __launch_bounds__(kFinWaves * 64)
backward_gated_finish_kernel(GatedBackwardArgs a, const float *dq32, const float *dk32)
{
    __shared__ float part[kFinWaves][kD];
    const int bh = blockIdx.x, b = bh / a.Hh, h = bh - b * a.Hh;
    const int wave = threadIdx.x >> 6, c = threadIdx.x & 63;
    const int n = a.n_tokens;
    const int per = (n + kFinWaves - 1) / kFinWaves;
    const int t_lo = min(wave * per, n), t_hi = min(t_lo + per, n);     // this wave's tokens
    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h + c;
    const int64_t g_base = (int64_t)b * a.grad.stride_b + (int64_t)h * a.grad.stride_h + c;
    const int64_t w_base = ((int64_t)b * n * a.Hh + h) * kD + c;         // workspace: [B][n][Hh][d] fp32
    const int64_t w_stride_n = (int64_t)a.Hh * kD;
    auto in_val = [&](const void *p, int t) {
        const int64_t i = in_base + (int64_t)t * a.in.stride_n;
        return IN_BF16 ? bf16_bits_to_float(((const uint16_t *)p)[i]) : ((const float *)p)[i];
    };
    auto put = [&](void *p, int t, float x) {
        const int64_t i = g_base + (int64_t)t * a.grad.stride_n;
        if (OUT_BF16) ((uint16_t *)p)[i] = float_to_bf16_bits(x);
        else ((float *)p)[i] = x;
    };
    auto r_term = [&](int t, float &lam, float &dk) {
        lam = in_val(a.lam, t);
        const float k = a.k ? in_val(a.k, t) : 1.0f - lam;
        dk = dk32[w_base + t * w_stride_n];
        return in_val(a.q, t) * dq32[w_base + t * w_stride_n] - k * dk;
    };
    // sum of this wave's token range, top down (the order of the walk below)
    float sum = 0.f;
    for (int t = t_hi - 1; t >= t_lo; --t) {
        float lam, dk;
        sum += r_term(t, lam, dk);
    }
    part[wave][c] = sum;
    __syncthreads();
    float suffix = 0.f;                    // sum over the tokens after this wave's range
    for (int w2 = kFinWaves - 1; w2 > wave; --w2) suffix += part[w2][c];
    for (int t = t_hi - 1; t >= t_lo; --t) {
        float lam, dk;
        suffix += r_term(t, lam, dk);
        const bool no_decay = t == 0 || is_boundary(a.start_pos + t + 1, a.grid_w, a.mode);
        float dl = no_decay ? 0.f : suffix / lam;
        if (!a.k) dl -= dk;
        put(a.dlam, t, dl);
        put(a.dq, t, dq32[w_base + t * w_stride_n]);
        if (a.k) put(a.dk, t, dk);
    }
}

int reversed_start(int start_pos, int n, int grid_w, int mode)
{
    const int64_t W = grid_w;
    int64_t s = 0;
    if (mode == LASAD_RESET_LAST_COL) s = -((int64_t)start_pos + n + 2);
    else if (mode == LASAD_RESET_FIRST_COL) s = -((int64_t)start_pos + n);
    s %= W;
    if (s < 0) s += W;
    return (int)s;
}

const void *last_token(const void *p, const lasad_layout_t &l, int n, int elt)
{
    return p ? (const char *)p + (int64_t)(n - 1) * l.stride_n * elt : nullptr;
}

template <int IN_BF16, int OUT_BF16>
void launch_walks(const WalkArgs &w, int64_t n_seq, hipStream_t s)
{
    // two workgroups per sequence and pass while that still leaves workgroup slots free on 256 CUs
    if (n_seq * 3 * 2 <= 1024)
        hipLaunchKernelGGL((backward_gated_walk_kernel<IN_BF16, OUT_BF16, 32>), dim3((unsigned)(n_seq * 2), 3), dim3(kThreads), 0, s, w);
    else
        hipLaunchKernelGGL((backward_gated_walk_kernel<IN_BF16, OUT_BF16, 64>), dim3((unsigned)n_seq, 3), dim3(kThreads), 0, s, w);
}

}  // namespace

size_t backward_gated_workspace_bytes(int64_t n_seq, int n_tokens, int d)
{
    return 2 * (size_t)n_seq * n_tokens * d * sizeof(float);
}

hipError_t launch_backward_gated(const GatedBackwardArgs &b, hipStream_t s)
{
    if (b.d != kD || b.n_tokens < 1) return hipErrorInvalidValue;
    const int64_t n_seq = (int64_t)b.B * b.Hh;
    if (n_seq * 2 > 0x7fffffff) return hipErrorInvalidValue;
    const int n = b.n_tokens;
    const int elt = b.io_dtype == LASAD_BF16 ? 2 : 4;
    const int gelt = b.grad_dtype == LASAD_BF16 ? 2 : 4;
    float *dq32 = (float *)b.workspace;
    float *dk32 = dq32 + (size_t)n_seq * n * b.d;

    lasad_layout_t wl;                                   // layout of dq32 / dk32
    wl.stride_b = (int64_t)n * b.Hh * b.d; wl.stride_n = (int64_t)b.Hh * b.d; wl.stride_h = b.d;
    lasad_layout_t in_rev = b.in, grad_rev = b.grad, wl_rev = wl;
    in_rev.stride_n = -b.in.stride_n; grad_rev.stride_n = -b.grad.stride_n; wl_rev.stride_n = -wl.stride_n;
    const int rev_start = reversed_start(b.start_pos, n, b.grid_w, b.mode);
    const void *q_l = last_token(b.q, b.in, n, elt), *lam_l = last_token(b.lam, b.in, n, elt);
    const void *k_l = last_token(b.k, b.in, n, elt), *v_l = last_token(b.v, b.in, n, elt);
    const void *g_l = last_token(b.d_o, b.in, n, elt);

    WalkArgs w;
    ForwardArgs &f = w.common;
    f.q = f.k = f.v = f.lam = nullptr; f.o = nullptr;
    f.fused_act = 0; f.norm = 0; f.norm_eps = 0.f; f.norm_w = nullptr;
    f.io_dtype = b.io_dtype; f.out_dtype = b.grad_dtype;
    f.in = b.in; f.out = b.grad;
    f.B = b.B; f.Hh = b.Hh; f.d = b.d;
    f.grid_w = b.grid_w; f.start_pos = b.start_pos; f.n_tokens = n;
    f.gamma = nullptr; f.mode = b.mode; f.q_scale = b.q_scale;
    f.state_in = nullptr; f.state_out = nullptr;
    f.seg_states = nullptr; f.n_segments = 1; f.seg_chunks = 0;
    // planes: PQ (output row operand), PK (update row operand), PV (update column operand), PL (decay)
    // dq, forward order: g, v, k, lambda
    w.roles[0] = ScanRoles{{b.d_o, b.v, b.k ? b.k : b.lam, b.lam}, {0, 0, 0, 0}, {0, 0, b.k ? 0 : 1, 0}};
    w.o[0] = dq32; w.in[0] = b.in; w.out[0] = wl; w.start_pos[0] = b.start_pos;
    // dv, reversed order: k, q, g, lambda of the step before
    w.roles[1] = ScanRoles{{b.k ? k_l : lam_l, q_l, g_l, lam_l}, {0, 0, 0, -1}, {b.k ? 0 : 1, 0, 0, 0}};
    w.o[1] = (void *)last_token(b.dv, b.grad, n, gelt); w.in[1] = in_rev; w.out[1] = grad_rev; w.start_pos[1] = rev_start;
    // dk, reversed order: v, g, q, lambda of the step before
    w.roles[2] = ScanRoles{{v_l, g_l, q_l, lam_l}, {0, 0, 0, -1}, {0, 0, 0, 0}};
    w.o[2] = (void *)last_token(dk32, wl, n, 4); w.in[2] = in_rev; w.out[2] = wl_rev; w.start_pos[2] = rev_start;

    const bool in16 = b.io_dtype == LASAD_BF16, out16 = b.grad_dtype == LASAD_BF16;
    static const bool force_walk = [] { const char *e = getenv("LASAD_GATED_BWD"); return e && !strcmp(e, "walk"); }();
    hipError_t e;
    if (in16 && !force_walk) {
        // matrix-core passes: the pass's operands in the forward's fields
        ForwardArgs p = f;
        p.q = b.d_o; p.lam = b.lam; p.k = b.k; p.v = b.v; p.o = dq32;                      // dq
        p.in = b.in; p.out = wl; p.out_dtype = LASAD_F32; p.start_pos = b.start_pos;
        e = launch_backward_gated_pass(p, w.roles[0], 1, 0, 0, s);
        if (e != hipSuccess) return e;
        p.q = b.k ? k_l : lam_l; p.lam = lam_l; p.k = q_l; p.v = g_l; p.o = w.o[1];         // dv
        p.in = in_rev; p.out = grad_rev; p.out_dtype = b.grad_dtype; p.start_pos = rev_start;
        e = launch_backward_gated_pass(p, w.roles[1], 0, 1, b.k ? 0 : 1, s);
        if (e != hipSuccess) return e;
        p.q = v_l; p.lam = lam_l; p.k = q_l; p.v = g_l; p.o = w.o[2];                       // dk
        p.out = wl_rev; p.out_dtype = LASAD_F32;
        e = launch_backward_gated_pass(p, w.roles[2], 1, 1, 0, s);
        if (e != hipSuccess) return e;
    } else {
        if (in16 && out16) launch_walks<1, 1>(w, n_seq, s);
        else if (in16) launch_walks<1, 0>(w, n_seq, s);
        else if (!out16) launch_walks<0, 0>(w, n_seq, s);
        else return hipErrorInvalidValue;
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }

    const dim3 grid((unsigned)n_seq), block(kFinWaves * 64);
    if (in16 && out16) hipLaunchKernelGGL((backward_gated_finish_kernel<1, 1>), grid, block, 0, s, b, dq32, dk32);
    else if (in16) hipLaunchKernelGGL((backward_gated_finish_kernel<1, 0>), grid, block, 0, s, b, dq32, dk32);
    else hipLaunchKernelGGL((backward_gated_finish_kernel<0, 0>), grid, block, 0, s, b, dq32, dk32);
    return hipGetLastError();
}

}  // namespace lasad
