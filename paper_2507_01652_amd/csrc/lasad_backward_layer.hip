// Backward pass of the fused layer (Algorithm 1 between its two Linear maps, zero initial state):
//     q = SiLU(q_pre),  lambda = sigmoid(z),  k = 1 - lambda,  o = recurrence(q, lambda, k, v),
//     y = o * rstd * w,  rstd = (mean_c(o^2) + eps)^(-1/2)        (per token and head)
// given d_out = dL/dy.  Composition of existing pieces around two small kernels of this file:
//
//   1. o is recomputed by the forward kernels (activations on load, no norm), fp32, into the workspace;
//   2. norm_backward_kernel: with gw = d_out * w,
//          d_o = rstd gw - o rstd^3 mean_c(gw o),      dw[h][c] += d_out o rstd
//      d_o goes to the workspace in the inputs' type and with the inputs' strides (the recurrence
//      kernels read all their operands with one layout); the weight gradient is first summed over
//      the 64 tokens of a workgroup, in a fixed order;
//   3. the vector-decay backward (lasad_backward_gated.hip) with activations on load and the chain
//      rule to q_pre and z in its finishing kernel;
//   4. weight_grad_kernel adds the per-workgroup sums of step 2, again in a fixed order.
//
// Without a normalisation (norm_eps < 0) step 1 is skipped and step 2 only copies d_out.
//
// Precision.  d_o is orthogonal to o (the normalisation ignores the length of o), and early in a
// sequence the state is close to rank one with o along its dominant direction, so dq = S d_o and
// dk are small differences of larger terms: d_o rounded to a single bf16 shows in dq_pre and dz up
// to 0.15 of their RMS.  With bf16 inputs step 2 therefore leaves d_o as a bf16 PAIR hi + lo (two
// tensors), and the two column passes of step 3 use both parts where d_o is their operand (the
// row pass, dv, takes hi alone: no cancellation there).  fp32 inputs keep d_o in fp32.  Steps 1-2
// can be run alone (d_o_out: hi only), step 3 alone is the call without a normalisation.
#include "lasad_scan.h"

namespace lasad {

namespace {

using scan::f4;
constexpr int kD = 64;
constexpr int kNbThreads = 1024;
constexpr int kNbTokens = 64;            // tokens per workgroup of the norm-backward kernel

// Thread (row, c4) holds four channels of one token; a token's 16 threads are neighbours in a wave.
template <int IN_BF16, int NORM>
__global__ void __launch_bounds__(kNbThreads)
norm_backward_kernel(LayerBackwardArgs a, const float *o32, void *d_o, void *d_o_lo, lasad_layout_t dl, float *wpart, int nblk)
{
    __shared__ __attribute__((aligned(16))) float sW[kNbTokens][kD + 4];
    const int bh = blockIdx.x / nblk, blk = blockIdx.x - bh * nblk;
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const int tid = threadIdx.x, row = tid >> 4, c4 = (tid & 15) * 4;
    const int n = a.n_tokens;
    const int t = blk * kNbTokens + row;
    const bool live = t < n;
    const int tc = min(t, n - 1);

    f4 g;
    {
        const int64_t i = (int64_t)b * a.dout.stride_b + (int64_t)tc * a.dout.stride_n + (int64_t)h * a.dout.stride_h + c4;
        if (IN_BF16) {
            const uint2 w = *(const uint2 *)((const uint16_t *)a.d_out + i);
            g = f4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u),
                   __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xffff0000u)};
        } else {
            g = *(const f4 *)((const float *)a.d_out + i);
        }
    }
    f4 res = g;
    if (NORM) {
        const f4 o = *(const f4 *)(o32 + (((int64_t)b * n + tc) * a.Hh + h) * kD + c4);
        const f4 w = a.norm_w ? *(const f4 *)(a.norm_w + h * kD + c4) : f4{1.0f, 1.0f, 1.0f, 1.0f};
        const f4 gw = g * w;
        float ss = (o[0] * o[0] + o[1] * o[1]) + (o[2] * o[2] + o[3] * o[3]);
        float go = (gw[0] * o[0] + gw[1] * o[1]) + (gw[2] * o[2] + gw[3] * o[3]);
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) {             // over the token's 16 threads
            ss += __shfl_xor(ss, m);
            go += __shfl_xor(go, m);
        }
        const float rstd = 1.0f / sqrtf(ss * (1.0f / kD) + a.norm_eps);
        res = gw * rstd - o * (rstd * rstd * rstd * go * (1.0f / kD));
        f4 dw = g * o * rstd;
        if (!live) dw = f4{0.f, 0.f, 0.f, 0.f};
        *(f4 *)&sW[row][c4] = dw;
    }
    if (live) {
        const int64_t i = (int64_t)b * dl.stride_b + (int64_t)t * dl.stride_n + (int64_t)h * dl.stride_h + c4;
        if (IN_BF16 && !a.d_o_f32) {
            uint2 w;
            w.x = (uint32_t)float_to_bf16_bits(res[0]) | ((uint32_t)float_to_bf16_bits(res[1]) << 16);
            w.y = (uint32_t)float_to_bf16_bits(res[2]) | ((uint32_t)float_to_bf16_bits(res[3]) << 16);
            *(uint2 *)((uint16_t *)d_o + i) = w;
            if (d_o_lo) {                  // what the rounding to bf16 left over, again as bf16
                float lo[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t hi = (e & 1) ? ((e < 2 ? w.x : w.y) & 0xffff0000u) : ((e < 2 ? w.x : w.y) << 16);
                    lo[e] = res[e] - __uint_as_float(hi);
                }
                uint2 wl;
                wl.x = (uint32_t)float_to_bf16_bits(lo[0]) | ((uint32_t)float_to_bf16_bits(lo[1]) << 16);
                wl.y = (uint32_t)float_to_bf16_bits(lo[2]) | ((uint32_t)float_to_bf16_bits(lo[3]) << 16);
                *(uint2 *)((uint16_t *)d_o_lo + i) = wl;
            }
        } else {
            *(f4 *)((float *)d_o + i) = res;
        }
    }
    if (NORM && a.dweight) {
        __syncthreads();
        if (tid < kD) {
            float acc = 0.f;
            for (int r = 0; r < kNbTokens; ++r) acc += sW[r][tid];
            wpart[((int64_t)bh * nblk + blk) * kD + tid] = acc;
        }
    }
}

// dweight[h][c] = sum over batch rows and token blocks of the partial sums.  A workgroup owns 16
// channels of one head: 64 threads per channel take every 64th item, then one thread per channel adds
// the 64 in order.
__global__ void __launch_bounds__(1024)
weight_grad_kernel(const float *wpart, float *dweight, int B, int Hh, int nblk)
{
    __shared__ float sP[64][17];
    const int h = blockIdx.x >> 2, c = (blockIdx.x & 3) * 16 + (threadIdx.x & 15), g = threadIdx.x >> 4;
    const int items = B * nblk;
    float acc = 0.f;
    for (int i = g; i < items; i += 64) {
        const int b = i / nblk, blk = i - b * nblk;
        acc += wpart[(((int64_t)b * Hh + h) * nblk + blk) * kD + c];
    }
    sP[g][threadIdx.x & 15] = acc;
    __syncthreads();
    if (threadIdx.x < 16) {
        float s = 0.f;
        for (int i = 0; i < 64; ++i) s += sP[i][threadIdx.x];
        dweight[h * kD + c] = s;
    }
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// elements spanned by a [B, n, Hh, d] view with non-negative strides
size_t extent(const lasad_layout_t &l, int B, int n, int Hh, int d)
{
    return (size_t)((int64_t)(B - 1) * l.stride_b + (int64_t)(n - 1) * l.stride_n + (int64_t)(Hh - 1) * l.stride_h + d);
}

struct Regions { size_t core, o32, d_o, d_o_lo, wpart, total; };

Regions regions(int B, int Hh, int n, int d, int io_dtype, const lasad_layout_t &in)
{
    const int64_t n_seq = (int64_t)B * Hh;
    const int nblk = (n + kNbTokens - 1) / kNbTokens;
    Regions r;
    r.core = 0;
    r.o32 = align256(backward_gated_workspace_bytes(n_seq, n, d));
    r.d_o = r.o32 + align256((size_t)n_seq * n * d * sizeof(float));
    r.d_o_lo = r.d_o + align256(extent(in, B, n, Hh, d) * (io_dtype == LASAD_BF16 ? 2 : 4));
    r.wpart = r.d_o_lo + (io_dtype == LASAD_BF16 ? align256(extent(in, B, n, Hh, d) * 2) : 0);
    r.total = r.wpart + align256((size_t)n_seq * nblk * d * sizeof(float));
    return r;
}

}  // namespace

size_t backward_layer_workspace_bytes(int B, int Hh, int n_tokens, int d, int io_dtype, const lasad_layout_t &in)
{
    return regions(B, Hh, n_tokens, d, io_dtype, in).total;
}

hipError_t launch_backward_layer(const LayerBackwardArgs &a, bool use_mfma, hipStream_t s)
{
    if (a.d != kD || a.n_tokens < 1) return hipErrorInvalidValue;
    const int n = a.n_tokens;
    const int64_t n_seq = (int64_t)a.B * a.Hh;
    const int nblk = (n + kNbTokens - 1) / kNbTokens;
    if (n_seq * nblk > 0x7fffffff) return hipErrorInvalidValue;
    const Regions r = regions(a.B, a.Hh, n, a.d, a.io_dtype, a.in);
    char *ws = (char *)a.workspace;
    float *o32 = (float *)(ws + r.o32);
    void *d_o = a.d_o_out ? a.d_o_out : ws + r.d_o;
    const lasad_layout_t dl = a.d_o_out ? a.d_o_l : a.in;
    // bf16: the whole call keeps what the rounding of d_o to bf16 leaves over as a second bf16 tensor
    void *d_o_lo = (!a.d_o_out && a.io_dtype == LASAD_BF16) ? ws + r.d_o_lo : nullptr;
    float *wpart = (float *)(ws + r.wpart);
    const bool norm = a.norm_eps >= 0.f;
    const bool in16 = a.io_dtype == LASAD_BF16;
    hipError_t e;

    if (norm) {                                                         // 1. o, fp32, [B][n][Hh][d]
        ForwardArgs f;
        f.q = a.q_pre; f.lam = a.z; f.k = nullptr; f.v = a.v; f.o = o32;
        f.in = a.in;
        f.out.stride_b = (int64_t)n * a.Hh * a.d; f.out.stride_n = (int64_t)a.Hh * a.d; f.out.stride_h = a.d;
        f.io_dtype = a.io_dtype; f.out_dtype = LASAD_F32;
        f.B = a.B; f.Hh = a.Hh; f.d = a.d;
        f.grid_w = a.grid_w; f.start_pos = a.start_pos; f.n_tokens = n;
        f.gamma = nullptr; f.mode = a.mode; f.q_scale = a.q_scale;
        f.state_in = nullptr; f.state_out = nullptr;
        f.seg_states = nullptr; f.n_segments = 1; f.seg_chunks = 0;
        f.fused_act = 1; f.norm = 0; f.norm_eps = -1.f; f.norm_w = nullptr;
        e = (in16 && use_mfma) ? launch_forward_gated_mfma(f, s) : launch_forward_generic(f, s);
        if (e != hipSuccess) return e;
    }
    {                                                                   // 2. d_o (and the weight-gradient partial sums)
        const dim3 grid((unsigned)(n_seq * nblk)), block(kNbThreads);
        if (in16 && norm) hipLaunchKernelGGL((norm_backward_kernel<1, 1>), grid, block, 0, s, a, o32, d_o, d_o_lo, dl, wpart, nblk);
        else if (in16) hipLaunchKernelGGL((norm_backward_kernel<1, 0>), grid, block, 0, s, a, o32, d_o, d_o_lo, dl, wpart, nblk);
        else if (norm) hipLaunchKernelGGL((norm_backward_kernel<0, 1>), grid, block, 0, s, a, o32, d_o, d_o_lo, dl, wpart, nblk);
        else hipLaunchKernelGGL((norm_backward_kernel<0, 0>), grid, block, 0, s, a, o32, d_o, d_o_lo, dl, wpart, nblk);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (a.d_o_out) {                                                    // the normalisation's part only
        if (a.dweight) {
            if (norm) hipLaunchKernelGGL(weight_grad_kernel, dim3((unsigned)a.Hh * 4), dim3(1024), 0, s, wpart, a.dweight, a.B, a.Hh, nblk);
            else return launch_zero_f32(a.dweight, a.Hh * a.d, s);
        }
        return hipGetLastError();
    }
    GatedBackwardArgs g;                                                // 3. the recurrence and the activations
    g.q = a.q_pre; g.lam = a.z; g.k = nullptr; g.v = a.v; g.d_o = d_o;
    g.dq = a.dq_pre; g.dlam = a.dz; g.dk = nullptr; g.dv = a.dv;
    g.in = a.in; g.grad = a.grad;
    g.io_dtype = a.io_dtype; g.grad_dtype = a.grad_dtype;
    g.B = a.B; g.Hh = a.Hh; g.d = a.d; g.grid_w = a.grid_w;
    g.start_pos = a.start_pos; g.n_tokens = n;
    g.mode = a.mode; g.q_scale = a.q_scale;
    g.workspace = ws + r.core;
    g.fused_act = 1; g.d_o_lo = d_o_lo;
    e = launch_backward_gated(g, s);
    if (e != hipSuccess) return e;
    if (a.dweight) {                                                    // 4. weight gradient (zero without a norm)
        if (norm) {
            hipLaunchKernelGGL(weight_grad_kernel, dim3((unsigned)a.Hh * 4), dim3(1024), 0, s, wpart, a.dweight, a.B, a.Hh, nblk);
            e = hipGetLastError();
        } else {
            e = launch_zero_f32(a.dweight, a.Hh * a.d, s);
        }
    }
    return e;
}

}  // namespace lasad
