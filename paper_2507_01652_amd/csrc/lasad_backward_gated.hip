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
// (lasad_backward_gated_mfma.hip, again one launch); the walks remain the path for fp32 inputs
// and the range fallback of those kernels (LASAD_GATED_BWD=walk forces them).
//
// Decay gradient.  L depends on l only through the products prod_{s=j+1..i} l_s[c] between a key
// j and a query i, so with r_i[c] = q_i[c] dq_i[c] - k_i[c] dk_i[c]
//
//   l_t[c] * dL/dl_t[c] = sum_{i >= t} r_i[c]            (every pair with j < t <= i, once)
//
// and dlam_t = (t a boundary or the first token ? 0 : that suffix sum / lambda_t) - (tied key: dk_t).
// The suffix sums cancel heavily, so dq and dk go through the workspace in fp32; the finishing kernel
// (one workgroup per sequence, blocks of 64 tokens from the last to the first) forms them in a fixed
// order and stores dq, dk, dlam in the caller's type.  lambda must be > 0 where it is applied, and the result loses precision like
// 1 / lambda for very small decays (the quotient of a rounded sum).
#include <stdlib.h>
#include <string.h>

#include "lasad_recurrence.h"
#include "lasad_scan.h"

namespace lasad {

hipError_t launch_backward_gated_passes(const ForwardArgs *a, const scan::ScanRoles *roles, bool tied, hipStream_t s);

namespace {

using namespace scan;

struct WalkArgs {
    ForwardArgs common;
    ScanRoles roles[3];            // pass 0 dq, 1 dv, 2 dk
    void *o[3];
    lasad_layout_t in[3], out[3];
    int start_pos[3];
    const float *state_in[3];      // per pass, [B, Hh, d, d] in the layout [decayed channel][other index], or NULL
    float *state_out[3];
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
    a.state_in = w.state_in[pass]; a.state_out = w.state_out[pass];
    if (pass == 1) scan_sequence<IN_BF16, OUT_BF16, ROLES_ROW, NJ>(a, bh, j0, lds, &w.roles[1]);
    else scan_sequence<IN_BF16, 0, ROLES_COL, NJ>(a, bh, j0, lds, &w.roles[pass]);     // fp32 into the workspace
}

// The same walks for the other head dims (32, 128): the plain fp32 recurrence of lasad_recurrence.h with the
// tensors in the roles of ScanRoles (shift and 1 - x; no activations: the fused layer is a head-dim-64 path).
// Thread (g, j) owns column j and rows g R .. g R + R - 1 of the walk's state [update row operand][update column
// operand]; COL: the decay is per column, and the state's memory layout is [decayed channel][other index], as in
// scan_sequence.  smem: (4 + G) x kRecT x D floats.
template <int D>
constexpr int roles_lds_floats() { return (4 + kRecThreads / D) * kRecT * D; }

template <int D, int IN_BF16, int OUT_BF16, int COL>
__device__ void recurrence_roles(const ForwardArgs &a, const ScanRoles &ro, int bh, float *smem)
{
    constexpr int G = kRecThreads / D;
    constexpr int R = D / G;
    float (*pl)[kRecT][D] = (float (*)[kRecT][D])smem;               // planes PQ, PK, PV, PL
    float (*red)[G][D] = (float (*)[G][D])(smem + 4 * kRecT * D);
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const int tid = threadIdx.x;
    const int j = tid % D, g = tid / D;

    float S[R];
    if (a.state_in) {
        const float *s0 = a.state_in + (int64_t)bh * D * D;
#pragma unroll
        for (int r = 0; r < R; ++r) S[r] = COL ? s0[(int64_t)j * D + g * R + r] : s0[(int64_t)(g * R + r) * D + j];
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) S[r] = 0.f;
    }
    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    const int64_t out_base = (int64_t)b * a.out.stride_b + (int64_t)h * a.out.stride_h;

    for (int t0 = 0; t0 < a.n_tokens; t0 += kRecT) {
        const int nt = min(kRecT, a.n_tokens - t0);
        for (int e = tid; e < 4 * kRecT * D; e += kRecThreads) {
            const int p = e / (kRecT * D), w = e - p * (kRecT * D);
            const int tt = w / D, c = w - tt * D;
            float x = p == PL ? 1.0f : 0.0f;                         // rows past the end (never walked)
            if (tt < nt) {
                const int t = t0 + tt + ro.shift[p];                  // the plane of token m holds the tensor's token m + shift
                const bool before = t < 0;                            // a shifted read before the first token is neutral
                if (!before) {
                    x = rec_load<IN_BF16>(ro.ptr[p], in_base + (int64_t)t * a.in.stride_n + c);
                    if (ro.one_minus[p]) x = 1.0f - x;
                }
                if (p == PL) {
                    if (before || is_boundary(a.start_pos + t0 + tt + 1, a.grid_w, a.mode)) x = 1.0f;
                } else if (before) {
                    x = 0.0f;
                }
                if (p == PQ) x *= a.q_scale;
            }
            pl[p][tt][c] = x;
        }
        __syncthreads();
        for (int tt = 0; tt < nt; ++tt) {
            const float vj = pl[PV][tt][j];
            const float lj = pl[PL][tt][j];
            float part = 0.f;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float lr = COL ? lj : pl[PL][tt][g * R + r];
                S[r] = fmaf(lr, S[r], pl[PK][tt][g * R + r] * vj);
                part = fmaf(pl[PQ][tt][g * R + r], S[r], part);
            }
            red[tt][g][j] = part;
        }
        __syncthreads();
        for (int e = tid; e < nt * D; e += kRecThreads) {
            const int tt = e / D, c = e - tt * D;
            float acc = 0.f;
#pragma unroll
            for (int gg = 0; gg < G; ++gg) acc += red[tt][gg][c];
            rec_store<OUT_BF16>(a.o, out_base + (int64_t)(t0 + tt) * a.out.stride_n + c, acc);
        }
        // (the next round's staging writes the planes, not red; its first barrier orders them against these reads)
    }
    if (a.state_out) {
        float *s1 = a.state_out + (int64_t)bh * D * D;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (COL) s1[(int64_t)j * D + g * R + r] = S[r];
            else s1[(int64_t)(g * R + r) * D + j] = S[r];
        }
    }
}

template <int D, int IN_BF16, int OUT_BF16>
__global__ void __launch_bounds__(kRecThreads)
backward_gated_generic_walk_kernel(WalkArgs w)
{
    __shared__ __attribute__((aligned(16))) float lds[roles_lds_floats<D>()];
    const int pass = blockIdx.y;
    ForwardArgs a = w.common;
    a.o = w.o[pass]; a.in = w.in[pass]; a.out = w.out[pass]; a.start_pos = w.start_pos[pass];
    a.state_in = w.state_in[pass]; a.state_out = w.state_out[pass];
    if (pass == 1) recurrence_roles<D, IN_BF16, OUT_BF16, 0>(a, w.roles[1], blockIdx.x, lds);
    else recurrence_roles<D, IN_BF16, 0, 1>(a, w.roles[pass], blockIdx.x, lds);     // fp32 into the workspace
}

constexpr int kFinBlock = 64;          // tokens per step of the finishing kernel

// One workgroup per sequence walks it in blocks of 64 tokens from the last block to the first,
// every thread holding four channels of one token (16-byte loads; the next block's loads are in
// flight while this one is worked on).  Per block: r = q dq - k dk into LDS, suffix sums down the
// block's tokens per channel (four 16-token quarters side by side, then their totals), outputs,
// and the block's total joins the carry.  Every input is read once; the order of all sums is fixed.
// Few long sequences are cut into n_seg segments of seg_blocks blocks with a workgroup each
// (blockIdx.y): a first launch (TOTALS) only adds up r over each segment, the second starts every
// segment from the totals of the segments after it.  seg_totals: [sequence][segment][d] fp32.
// The channels are independent: with few workgroups a sequence's channels are further divided between
// 64 / CH workgroups (blockIdx.z) of 16 CH threads, which shortens nothing of the chain of blocks but
// puts more of them in flight.
// (fp64 sums were tried: no gain in accuracy, the error left is that of the fp32 dq and dk.)
template <int IN_BF16, int OUT_BF16, int TOTALS, int CH>
__global__ void __launch_bounds__(16 * CH)
backward_gated_finish_kernel(GatedBackwardArgs a, const float *dq32, const float *dk32,
                             float *seg_totals, int n_seg, int seg_blocks, const float *sink)
{
    // sink [sequence][d] (or NULL): per key channel, sum_n H[c][n] s_n[c][n] for H = dL/d(final state): the products of
    // decays that end in the final state pass through EVERY step of the call, so every suffix sum starts from it
    constexpr int LPR = CH / 4;            // threads per token
    __shared__ __attribute__((aligned(16))) float sR[kFinBlock][CH + 4];
    __shared__ __attribute__((aligned(16))) float sQtr[4][CH];
    __shared__ __attribute__((aligned(16))) float sCarry[CH];
    const int bh = blockIdx.x, b = bh / a.Hh, h = bh - b * a.Hh;
    const int tid = threadIdx.x;
    const int ch0 = blockIdx.z * CH;       // this workgroup's first channel
    const int row = tid / LPR, c4l = (tid % LPR) * 4, c4 = ch0 + c4l;
    const int n = a.n_tokens;
    const int nblk = (n + kFinBlock - 1) / kFinBlock;
    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h + c4;
    const int64_t g_base = (int64_t)b * a.grad.stride_b + (int64_t)h * a.grad.stride_h + c4;
    const int64_t w_base = ((int64_t)b * n * a.Hh + h) * a.d + c4;       // workspace: [B][n][Hh][d] fp32
    const int64_t w_stride_n = (int64_t)a.Hh * a.d;

    struct Item { f4 q, k, lam, dq, dk, dact; };     // dact: d(activation)/d(input) of q, fused activations only
    auto in4 = [&](const void *p, int t) {
        const int64_t i = in_base + (int64_t)t * a.in.stride_n;
        if (IN_BF16) {
            const uint2 w = *(const uint2 *)((const uint16_t *)p + i);
            return f4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u),
                      __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xffff0000u)};
        }
        return *(const f4 *)((const float *)p + i);
    };
    auto load = [&](int blk, Item &it) {
        const int t = min(blk * kFinBlock + row, n - 1);
        it.q = in4(a.q, t);
        it.lam = in4(a.lam, t);
        if (a.fused_act) {                 // q = SiLU(x), SiLU'(x) = s (1 + x (1 - s)) with s = sigmoid(x); lambda = sigmoid(z)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x = it.q[e], sg = sigmoid_f32(x);
                it.q[e] = x * sg;
                it.dact[e] = sg * (1.0f + x * (1.0f - sg));
                it.lam[e] = sigmoid_f32(it.lam[e]);
            }
        }
        if (a.k) it.k = in4(a.k, t);
        else it.k = f4{1.0f, 1.0f, 1.0f, 1.0f} - it.lam;
        it.dq = *(const f4 *)(dq32 + w_base + t * w_stride_n);
        it.dk = *(const f4 *)(dk32 + w_base + t * w_stride_n);
    };
    auto put4 = [&](void *p, int t, f4 x) {
        const int64_t i = g_base + (int64_t)t * a.grad.stride_n;
        if (OUT_BF16) {
            uint2 w;
            w.x = (uint32_t)float_to_bf16_bits(x[0]) | ((uint32_t)float_to_bf16_bits(x[1]) << 16);
            w.y = (uint32_t)float_to_bf16_bits(x[2]) | ((uint32_t)float_to_bf16_bits(x[3]) << 16);
            *(uint2 *)((uint16_t *)p + i) = w;
        } else {
            *(f4 *)((float *)p + i) = x;
        }
    };

    const int seg = blockIdx.y;
    const int blk_lo = seg * seg_blocks, blk_hi = min(blk_lo + seg_blocks, nblk) - 1;     // this workgroup's blocks
    float *totals = seg_totals + ((int64_t)bh * n_seg) * a.d + ch0;
    if (TOTALS) {
        f4 sum = f4{0.f, 0.f, 0.f, 0.f};
        for (int blk = blk_hi; blk >= blk_lo; --blk) {
            Item it;
            load(blk, it);
            if (blk * kFinBlock + row < n) sum += it.q * it.dq - it.k * it.dk;
        }
        *(f4 *)&sR[row][c4l] = sum;
        __syncthreads();
        if (tid < CH) {
            float acc = 0.f;
            for (int r2 = kFinBlock - 1; r2 >= 0; --r2) acc += sR[r2][tid];
            totals[seg * a.d + tid] = acc;
        }
        return;
    }
    if (tid < CH) {
        float carry = sink ? sink[(int64_t)bh * a.d + ch0 + tid] : 0.f;
        for (int s2 = n_seg - 1; s2 > seg; --s2) carry += totals[s2 * a.d + tid];
        sCarry[tid] = carry;
    }
    Item cur;
    load(blk_hi, cur);
    for (int blk = blk_hi; blk >= blk_lo; --blk) {
        Item nxt = cur;
        if (blk > blk_lo) load(blk - 1, nxt);
        const int t = blk * kFinBlock + row;
        const bool live = t < n;
        f4 r = cur.q * cur.dq - cur.k * cur.dk;
        if (!live) r = f4{0.f, 0.f, 0.f, 0.f};
        *(f4 *)&sR[row][c4l] = r;
        __syncthreads();
        if (tid < 4 * CH) {                // suffix sums inside a quarter of the block, top down
            const int c = tid % CH, qtr = tid / CH;
            float acc = 0.f;
#pragma unroll
            for (int tt = 15; tt >= 0; --tt) {
                acc += sR[16 * qtr + tt][c];
                sR[16 * qtr + tt][c] = acc;
            }
            sQtr[qtr][c] = acc;
        }
        __syncthreads();
        {
            f4 suffix = *(const f4 *)&sR[row][c4l] + *(const f4 *)&sCarry[c4l];
            for (int q2 = 3; q2 > (row >> 4); --q2) suffix += *(const f4 *)&sQtr[q2][c4l];
            // (from a zero state the first token's decay multiplies nothing)
            const bool no_decay = (t == 0 && !a.state_in) || is_boundary(a.start_pos + t + 1, a.grid_w, a.mode);
            f4 dl = suffix / cur.lam;
            if (no_decay) dl = f4{0.f, 0.f, 0.f, 0.f};
            if (!a.k) dl -= cur.dk;
            f4 dqo = cur.dq;
            if (a.fused_act) {             // chain rule to the pre-activation inputs; sigmoid' = lambda (1 - lambda)
                dl = dl * cur.lam * (f4{1.0f, 1.0f, 1.0f, 1.0f} - cur.lam);
                dqo = dqo * cur.dact;
            }
            if (live) {
                put4(a.dlam, t, dl);
                put4(a.dq, t, dqo);
                if (a.k) put4(a.dk, t, cur.dk);
            }
        }
        __syncthreads();
        if (tid < CH) sCarry[tid] += (sQtr[3][tid] + sQtr[2][tid]) + (sQtr[1][tid] + sQtr[0][tid]);
        cur = nxt;
    }
}

// hS = H / q_scale for the reversed passes (the kernels multiply their outputs by q_scale; the state gradient carries it
// only on its q d_o^T part).
__global__ void __launch_bounds__(256)
gated_carried_prep_kernel(const float *H, float *hS, float inv_q_scale, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) hS[i] = H[i] * inv_q_scale;
}

// One workgroup per sequence: dL/ds_0 = diag(l_1) g_1 (g_1 / q_scale: final state of the reversed dv pass; l_1: the decay
// applied at the call's first token) and sink[bh][c] = sum_n H[c][n] s_n[c][n] (s_n: final state of the dq pass).
template <int IN_BF16>
__global__ void __launch_bounds__(256)
gated_carried_finish_kernel(GatedBackwardArgs a, const float *g1, const float *sn, float *sink)
{
    const int bh = blockIdx.x, b = bh / a.Hh, h = bh - b * a.Hh;
    const int64_t off = (int64_t)bh * kD * kD;
    const int c = threadIdx.x >> 2, part = threadIdx.x & 3;          // four threads per key channel, 16 columns each
    float l1 = 1.0f;
    if (!is_boundary(a.start_pos + 1, a.grid_w, a.mode)) {
        const int64_t i = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h + c;
        l1 = IN_BF16 ? bf16_bits_to_float(((const uint16_t *)a.lam)[i]) : ((const float *)a.lam)[i];
        if (a.fused_act) l1 = sigmoid_f32(l1);
    }
    float acc = 0.f;
    for (int n = part * 16; n < part * 16 + 16; ++n) {
        if (a.d_state_in) a.d_state_in[off + c * kD + n] = (l1 * a.q_scale) * g1[off + c * kD + n];
        if (sink) acc = fmaf(a.d_state_out[off + c * kD + n], sn[off + c * kD + n], acc);
    }
    if (sink) {
        acc += __shfl_xor(acc, 1);
        acc += __shfl_xor(acc, 2);
        if (part == 0) sink[(int64_t)bh * kD + c] = acc;
    }
}

// The same for the other head dims: thread c < d takes key channel c.
template <int IN_BF16>
__global__ void __launch_bounds__(128)
gated_carried_finish_generic_kernel(GatedBackwardArgs a, const float *g1, const float *sn, float *sink)
{
    const int bh = blockIdx.x, b = bh / a.Hh, h = bh - b * a.Hh;
    const int d = a.d, c = threadIdx.x;
    if (c >= d) return;
    const int64_t off = (int64_t)bh * d * d + (int64_t)c * d;
    float l1 = 1.0f;
    if (!is_boundary(a.start_pos + 1, a.grid_w, a.mode)) {
        const int64_t i = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h + c;
        l1 = IN_BF16 ? bf16_bits_to_float(((const uint16_t *)a.lam)[i]) : ((const float *)a.lam)[i];
    }
    float acc = 0.f;
    for (int n = 0; n < d; ++n) {
        if (a.d_state_in) a.d_state_in[off + n] = (l1 * a.q_scale) * g1[off + n];
        if (sink) acc = fmaf(a.d_state_out[off + n], sn[off + n], acc);
    }
    if (sink) sink[(int64_t)bh * d + c] = acc;
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

size_t backward_gated_carried_extra_bytes(int64_t n_seq, int d)
{
    // H / q_scale, s_n (dq pass), g_1 / q_scale (dv pass), one sum per sequence and key channel
    return 3 * (size_t)n_seq * d * d * sizeof(float) + (size_t)n_seq * d * sizeof(float);
}

size_t backward_gated_workspace_bytes(int64_t n_seq, int n_tokens, int d)
{
    // dq and dk in fp32, then the finishing kernel's segment totals (at most 8 segments per sequence)
    return 2 * (size_t)n_seq * n_tokens * d * sizeof(float) + (size_t)n_seq * 8 * d * sizeof(float);
}

hipError_t launch_backward_gated(const GatedBackwardArgs &b, hipStream_t s)
{
    if ((b.d != 32 && b.d != 64 && b.d != 128) || b.n_tokens < 1) return hipErrorInvalidValue;
    if (b.d != kD && (b.fused_act || b.d_o_lo)) return hipErrorInvalidValue;     // the fused layer is a head-dim-64 path
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

    // carried states: the dq pass runs the forward recurrence itself (state [dk][dv], starts from state_in, ends with
    // s_n); the reversed passes run the recurrence of the state gradient from H / q_scale (no decay at their first
    // step: the shifted decay of step 0 is neutral); the dv pass ends with g_1 / q_scale
    const bool carried = b.state_in || b.d_state_out || b.d_state_in;
    const size_t mat = (size_t)n_seq * b.d * b.d;
    float *cw = dk32 + (size_t)n_seq * n * b.d + (size_t)n_seq * 8 * b.d;      // after the gradients and the segment totals
    float *hS = cw, *sn = cw + mat, *g1 = cw + 2 * mat, *sink_buf = cw + 3 * mat;
    const float *sink = (carried && b.d_state_out) ? sink_buf : nullptr;
    if (carried && b.d_state_out) {
        hipLaunchKernelGGL(gated_carried_prep_kernel, dim3((unsigned)((mat + 255) / 256)), dim3(256), 0, s,
                           b.d_state_out, hS, 1.0f / b.q_scale, (int64_t)mat);
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    const float *st_in[3] = {b.state_in, b.d_state_out ? hS : nullptr, b.d_state_out ? hS : nullptr};
    float *st_out[3] = {b.d_state_out ? sn : nullptr, b.d_state_in ? g1 : nullptr, nullptr};

    WalkArgs w;
    for (int y = 0; y < 3; ++y) { w.state_in[y] = st_in[y]; w.state_out[y] = st_out[y]; }
    ForwardArgs &f = w.common;
    f.q = f.k = f.v = f.lam = nullptr; f.o = nullptr;
    if (b.fused_act && b.k) return hipErrorInvalidValue;
    f.fused_act = b.fused_act; f.norm = 0; f.norm_eps = 0.f; f.norm_w = nullptr;
    f.io_dtype = b.io_dtype; f.out_dtype = b.grad_dtype;
    f.in = b.in; f.out = b.grad;
    f.B = b.B; f.Hh = b.Hh; f.d = b.d;
    f.grid_w = b.grid_w; f.start_pos = b.start_pos; f.n_tokens = n;
    f.gamma = nullptr; f.mode = b.mode; f.q_scale = b.q_scale;
    f.state_in = nullptr; f.state_out = nullptr;
    f.seg_states = nullptr; f.n_segments = 1; f.seg_chunks = 0;
    // planes: PQ (output row operand), PK (update row operand), PV (update column operand), PL (decay)
    // dq, forward order: g, v, k, lambda
    const int sg = b.fused_act ? ACT_SIGMOID : ACT_NONE, si = b.fused_act ? ACT_SILU : ACT_NONE;
    const void *gl_l = last_token(b.d_o_lo, b.in, n, elt);              // low-order part of d_o (layer backward, bf16)
    w.roles[0] = ScanRoles{{b.d_o, b.v, b.k ? b.k : b.lam, b.lam}, {0, 0, 0, 0}, {0, 0, b.k ? 0 : 1, 0}, {0, 0, b.k ? 0 : sg, sg},
                           {b.d_o_lo, nullptr, nullptr, nullptr}};
    w.o[0] = dq32; w.in[0] = b.in; w.out[0] = wl; w.start_pos[0] = b.start_pos;
    // dv, reversed order: k, q, g, lambda of the step before
    w.roles[1] = ScanRoles{{b.k ? k_l : lam_l, q_l, g_l, lam_l}, {0, 0, 0, -1}, {b.k ? 0 : 1, 0, 0, 0}, {b.k ? 0 : sg, si, 0, sg},
                           {nullptr, nullptr, gl_l, nullptr}};
    w.o[1] = (void *)last_token(b.dv, b.grad, n, gelt); w.in[1] = in_rev; w.out[1] = grad_rev; w.start_pos[1] = rev_start;
    // dk, reversed order: v, g, q, lambda of the step before
    w.roles[2] = ScanRoles{{v_l, g_l, q_l, lam_l}, {0, 0, 0, -1}, {0, 0, 0, 0}, {0, 0, si, sg}, {nullptr, gl_l, nullptr, nullptr}};
    w.o[2] = (void *)last_token(dk32, wl, n, 4); w.in[2] = in_rev; w.out[2] = wl_rev; w.start_pos[2] = rev_start;

    const bool in16 = b.io_dtype == LASAD_BF16, out16 = b.grad_dtype == LASAD_BF16;
    static const bool force_walk = [] { const char *e = getenv("LASAD_GATED_BWD"); return e && !strcmp(e, "walk"); }();
    hipError_t e;
    if (b.d != kD) {
        // other head dims: the plain fp32 recurrence with the tensors in their roles, one workgroup per sequence and pass
        const dim3 grid((unsigned)n_seq, 3), block(kRecThreads);
#define LASAD_GEN_WALK(D) do { \
            if (in16 && out16) hipLaunchKernelGGL((backward_gated_generic_walk_kernel<D, 1, 1>), grid, block, 0, s, w); \
            else if (in16) hipLaunchKernelGGL((backward_gated_generic_walk_kernel<D, 1, 0>), grid, block, 0, s, w); \
            else if (!out16) hipLaunchKernelGGL((backward_gated_generic_walk_kernel<D, 0, 0>), grid, block, 0, s, w); \
            else return hipErrorInvalidValue; \
        } while (0)
        if (b.d == 32) LASAD_GEN_WALK(32); else LASAD_GEN_WALK(128);
#undef LASAD_GEN_WALK
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else if (in16 && !force_walk) {
        // matrix-core passes: the pass's operands in the forward's fields
        ForwardArgs p[3] = {f, f, f};
        p[0].q = b.d_o; p[0].lam = b.lam; p[0].k = b.k; p[0].v = b.v; p[0].o = dq32;                  // dq
        p[0].in = b.in; p[0].out = wl; p[0].out_dtype = LASAD_F32; p[0].start_pos = b.start_pos;
        p[0].q_lo = b.d_o_lo;
        p[1].q = b.k ? k_l : lam_l; p[1].lam = lam_l; p[1].k = q_l; p[1].v = g_l; p[1].o = w.o[1];     // dv
        p[1].in = in_rev; p[1].out = grad_rev; p[1].out_dtype = b.grad_dtype; p[1].start_pos = rev_start;
        p[2] = p[1];
        p[1].v_lo = gl_l;
        p[2].q = v_l; p[2].o = w.o[2]; p[2].out = wl_rev; p[2].out_dtype = LASAD_F32;                  // dk
        p[2].v_lo = gl_l;
        for (int y = 0; y < 3; ++y) { p[y].state_in = st_in[y]; p[y].state_out = st_out[y]; }
        e = launch_backward_gated_passes(p, w.roles, b.k == nullptr, s);
        if (e != hipSuccess) return e;
    } else {
        if (in16 && out16) launch_walks<1, 1>(w, n_seq, s);
        else if (in16) launch_walks<1, 0>(w, n_seq, s);
        else if (!out16) launch_walks<0, 0>(w, n_seq, s);
        else return hipErrorInvalidValue;
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }

    if (carried && (b.d_state_in || sink)) {
        if (b.d != kD) {
            if (in16) hipLaunchKernelGGL((gated_carried_finish_generic_kernel<1>), dim3((unsigned)n_seq), dim3(128), 0, s, b, g1, sn, (float *)sink);
            else hipLaunchKernelGGL((gated_carried_finish_generic_kernel<0>), dim3((unsigned)n_seq), dim3(128), 0, s, b, g1, sn, (float *)sink);
        } else if (in16) hipLaunchKernelGGL((gated_carried_finish_kernel<1>), dim3((unsigned)n_seq), dim3(256), 0, s, b, g1, sn, (float *)sink);
        else hipLaunchKernelGGL((gated_carried_finish_kernel<0>), dim3((unsigned)n_seq), dim3(256), 0, s, b, g1, sn, (float *)sink);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // finishing kernel: one workgroup per sequence, or several segments per sequence when there are
    // few long ones (then a first launch for the segment totals)
    const int nblk = (n + kFinBlock - 1) / kFinBlock;
    int n_seg = 1;
    if (n_seq < 256 && nblk >= 8) {
        n_seg = (int)(512 / n_seq);
        if (n_seg > 8) n_seg = 8;
        if (n_seg > nblk / 4) n_seg = nblk / 4;
        if (n_seg < 1) n_seg = 1;
    }
    const int seg_blocks = (nblk + n_seg - 1) / n_seg;
    n_seg = (nblk + seg_blocks - 1) / seg_blocks;
    float *seg_totals = dk32 + (size_t)n_seq * n * b.d;          // after the two gradient tensors
    // few workgroups: 16 channels per workgroup (four workgroups of 256 threads per sequence and segment)
    const bool narrow = b.d == kD && n_seq * n_seg < 256;      // (at 480 workgroups the narrow rows already cost more than they gain)
    // head dim 32: one workgroup of 32 channels; 128: two of 64; 64: one of 64 or four of 16
    const dim3 grid((unsigned)n_seq, (unsigned)n_seg, narrow ? 4 : b.d == 128 ? 2 : 1), block(narrow ? 256 : b.d == 32 ? 512 : 1024);
#define LASAD_FIN_LAUNCH(I, O, T) do { \
        if (b.d == 32) hipLaunchKernelGGL((backward_gated_finish_kernel<I, O, T, 32>), grid, block, 0, s, b, dq32, dk32, seg_totals, n_seg, seg_blocks, sink); \
        else if (narrow) hipLaunchKernelGGL((backward_gated_finish_kernel<I, O, T, 16>), grid, block, 0, s, b, dq32, dk32, seg_totals, n_seg, seg_blocks, sink); \
        else hipLaunchKernelGGL((backward_gated_finish_kernel<I, O, T, 64>), grid, block, 0, s, b, dq32, dk32, seg_totals, n_seg, seg_blocks, sink); \
    } while (0)
    if (n_seg > 1) {
        if (in16) LASAD_FIN_LAUNCH(1, 0, 1); else LASAD_FIN_LAUNCH(0, 0, 1);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (in16 && out16) LASAD_FIN_LAUNCH(1, 1, 0);
    else if (in16) LASAD_FIN_LAUNCH(1, 0, 0);
    else LASAD_FIN_LAUNCH(0, 0, 0);
#undef LASAD_FIN_LAUNCH
    return hipGetLastError();
}

}  // namespace lasad
