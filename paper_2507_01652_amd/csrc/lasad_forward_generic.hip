// Generic forward kernel: fp32 arithmetic on the vector ALUs, any supported head
// dim (32 / 64 / 128), fp32 or bf16 storage.  It is the path for fp32 inputs (whose
// 1e-5 tolerance rules out bf16 matrix-core operands) and for shapes the MFMA
// kernel does not take.
//
// One workgroup (256 threads) walks one (batch, head) sequence with the d x d
// state of Section 3.4's recurrence held in registers:
//     S <- lambda_t S + k_t v_t^T,   o_t = q_scale * S^T q_t.
// Thread (g, j) owns column j (value channel) and the rows (key channels)
// g*R .. g*R+R-1 of S, R = d*d/256.  Tokens are staged through LDS T at a time;
// each thread writes its partial sum over its rows for each staged token and one
// cross-group reduction per T tokens produces the outputs, so the workgroup
// synchronises twice per T tokens instead of twice per token.
#include "lasad_internal.h"

namespace lasad {

namespace {

constexpr int kThreads = 256;
constexpr int kT = 16;   // tokens staged per round

template <int IN_BF16>
__device__ inline float load_in(const void *p, int64_t idx)
{
    if (IN_BF16) return bf16_bits_to_float(((const uint16_t *)p)[idx]);
    return ((const float *)p)[idx];
}

template <int OUT_BF16>
__device__ inline void store_out(void *p, int64_t idx, float x)
{
    if (OUT_BF16) ((uint16_t *)p)[idx] = float_to_bf16_bits(x);
    else ((float *)p)[idx] = x;
}

template <int D, int IN_BF16, int OUT_BF16>
__global__ void __launch_bounds__(kThreads)
forward_generic_kernel(ForwardArgs a)
{
    constexpr int G = kThreads / D;   // row groups
    constexpr int R = D / G;          // rows of S per thread
    __shared__ float sq[kT][D], sk[kT][D], sv[kT][D];
    __shared__ float red[kT][G][D];

    const int bh = blockIdx.x;
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const int tid = threadIdx.x;
    const int j = tid % D, g = tid / D;
    const float gamma = a.gamma[h];

    float S[R];
    if (a.state_in) {
        const float *s0 = a.state_in + (int64_t)bh * D * D;
#pragma unroll
        for (int r = 0; r < R; ++r) S[r] = s0[(g * R + r) * D + j];
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) S[r] = 0.f;
    }

    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    const int64_t out_base = (int64_t)b * a.out.stride_b + (int64_t)h * a.out.stride_h;

    for (int t0 = 0; t0 < a.n_tokens; t0 += kT) {
        const int nt = min(kT, a.n_tokens - t0);
        // stage q, k, v of tokens t0 .. t0+nt-1
        for (int e = tid; e < kT * D; e += kThreads) {
            const int tt = e / D, c = e - tt * D;
            float fq = 0.f, fk = 0.f, fv = 0.f;
            if (tt < nt) {
                const int64_t idx = in_base + (int64_t)(t0 + tt) * a.in.stride_n + c;
                fq = load_in<IN_BF16>(a.q, idx);
                fk = load_in<IN_BF16>(a.k, idx);
                fv = load_in<IN_BF16>(a.v, idx);
            }
            sq[tt][c] = fq; sk[tt][c] = fk; sv[tt][c] = fv;
        }
        __syncthreads();
        for (int tt = 0; tt < nt; ++tt) {
            const int t = a.start_pos + t0 + tt + 1;   // 1-indexed raster position
            const float lam = is_boundary(t, a.grid_w, a.mode) ? 1.0f : gamma;
            const float vj = sv[tt][j];
            float part = 0.f;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                S[r] = fmaf(lam, S[r], sk[tt][g * R + r] * vj);
                part = fmaf(sq[tt][g * R + r], S[r], part);
            }
            red[tt][g][j] = part;
        }
        __syncthreads();
        for (int e = tid; e < nt * D; e += kThreads) {
            const int tt = e / D, c = e - tt * D;
            float acc = 0.f;
#pragma unroll
            for (int gg = 0; gg < G; ++gg) acc += red[tt][gg][c];
            store_out<OUT_BF16>(a.o, out_base + (int64_t)(t0 + tt) * a.out.stride_n + c,
                                a.q_scale * acc);
        }
        // the next round's staging writes sq/sk/sv (not red), and its first
        // barrier orders those writes against this round's reads of red.
    }
    if (a.state_out) {
        float *s1 = a.state_out + (int64_t)bh * D * D;
#pragma unroll
        for (int r = 0; r < R; ++r) s1[(g * R + r) * D + j] = S[r];
    }
}

template <int D>
hipError_t launch_d(const ForwardArgs &a, hipStream_t s)
{
    const dim3 grid((unsigned)(a.B * a.Hh)), block(kThreads);
    const bool in16 = a.io_dtype == LASAD_BF16, out16 = a.out_dtype == LASAD_BF16;
    if (in16 && out16) hipLaunchKernelGGL((forward_generic_kernel<D, 1, 1>), grid, block, 0, s, a);
    else if (in16) hipLaunchKernelGGL((forward_generic_kernel<D, 1, 0>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((forward_generic_kernel<D, 0, 0>), grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_forward_generic(const ForwardArgs &a, hipStream_t s)
{
    switch (a.d) {
        case 32: return launch_d<32>(a, s);
        case 64: return launch_d<64>(a, s);
        case 128: return launch_d<128>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lasad
