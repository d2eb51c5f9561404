// fp32 recurrence of Section 3.4 for ONE (batch, head) sequence, run by one
// 256-thread workgroup on the vector ALUs:
//     S <- lambda_t S + k_t v_t^T,   o_t = q_scale * S^T q_t.
// Thread (g, j) owns column j (value channel) and rows g*R .. g*R+R-1 (key
// channels) of the d x d state, R = d*d/256, in registers.  Tokens are staged
// through LDS kRecT at a time; each thread writes its partial sum over its rows for
// every staged token and one cross-group reduction per kRecT tokens produces the
// outputs, so the workgroup synchronises twice per kRecT tokens.
//
// Used by the generic kernel (any supported d, fp32 or bf16 storage) and by the
// MFMA kernel for heads whose decay is too small for its separable mask.
//
// GATED = 1 is the recurrence exactly as Section 3.4 / Algorithm 1 write it: a decay
// vector lambda_t per token over the key channels (row r of S is scaled by lambda_t[r],
// or by 1 at a row-boundary position), with the key tied to the base decay,
// k_t = 1 - lambda_t, unless a key tensor is given.
#pragma once

#include "lasad_internal.h"

namespace lasad {

constexpr int kRecThreads = 256;
constexpr int kRecT = 16;   // tokens staged per round

// LDS floats the routine needs for head dim D
template <int D, int GATED = 0>
constexpr int recurrence_lds_floats() { return (3 + GATED) * kRecT * D + kRecT * (kRecThreads / D) * D; }

template <int IN_BF16>
__device__ inline float rec_load(const void *p, int64_t idx)
{
    if (IN_BF16) return bf16_bits_to_float(((const uint16_t *)p)[idx]);
    return ((const float *)p)[idx];
}

template <int OUT_BF16>
__device__ inline void rec_store(void *p, int64_t idx, float x)
{
    if (OUT_BF16) ((uint16_t *)p)[idx] = float_to_bf16_bits(x);
    else ((float *)p)[idx] = x;
}

// hook(token, channel, value) sees every output element (fp32, before it is stored) in the thread that stores it
struct RecNoHook {
    __device__ void operator()(int, int, float) const {}
};

template <int D, int IN_BF16, int OUT_BF16, int GATED = 0, class Hook = RecNoHook>
__device__ void recurrence_sequence(const ForwardArgs &a, int bh, float *smem, Hook hook = Hook())
{
    constexpr int G = kRecThreads / D;   // row groups
    constexpr int R = D / G;             // rows of S per thread
    float (*sq)[D] = (float (*)[D])smem;
    float (*sk)[D] = (float (*)[D])(smem + kRecT * D);
    float (*sv)[D] = (float (*)[D])(smem + 2 * kRecT * D);
    float (*sl)[D] = (float (*)[D])(smem + 3 * kRecT * D);      // GATED only: decay vectors
    float (*red)[G][D] = (float (*)[G][D])(smem + (3 + GATED) * kRecT * D);

    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const int tid = threadIdx.x;
    const int j = tid % D, g = tid / D;
    const float gamma = GATED ? 1.0f : a.gamma[h];

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

    for (int t0 = 0; t0 < a.n_tokens; t0 += kRecT) {
        const int nt = min(kRecT, a.n_tokens - t0);
        for (int e = tid; e < kRecT * D; e += kRecThreads) {
            const int tt = e / D, c = e - tt * D;
            float fq = 0.f, fk = 0.f, fv = 0.f, fl = 1.f;
            if (tt < nt) {
                const int64_t idx = in_base + (int64_t)(t0 + tt) * a.in.stride_n + c;
                fq = rec_load<IN_BF16>(a.q, idx);
                fv = rec_load<IN_BF16>(a.v, idx);
                if (GATED) {
                    fl = rec_load<IN_BF16>(a.lam, idx);
                    fk = a.k ? rec_load<IN_BF16>(a.k, idx) : 1.0f - fl;     // key from the base decay
                    if (is_boundary(a.start_pos + t0 + tt + 1, a.grid_w, a.mode)) fl = 1.0f;
                } else {
                    fk = rec_load<IN_BF16>(a.k, idx);
                }
            }
            sq[tt][c] = fq; sk[tt][c] = fk; sv[tt][c] = fv;
            if (GATED) sl[tt][c] = fl;
        }
        __syncthreads();
        for (int tt = 0; tt < nt; ++tt) {
            const int t = a.start_pos + t0 + tt + 1;   // 1-indexed raster position
            const float lam = (is_boundary(t, a.grid_w, a.mode) || (a.first_decay_off && t0 + tt == 0)) ? 1.0f : gamma;
            const float vj = sv[tt][j];
            float part = 0.f;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float lr = GATED ? sl[tt][g * R + r] : lam;
                S[r] = fmaf(lr, S[r], sk[tt][g * R + r] * vj);
                part = fmaf(sq[tt][g * R + r], S[r], part);
            }
            red[tt][g][j] = part;
        }
        __syncthreads();
        for (int e = tid; e < nt * D; e += kRecThreads) {
            const int tt = e / D, c = e - tt * D;
            float acc = 0.f;
#pragma unroll
            for (int gg = 0; gg < G; ++gg) acc += red[tt][gg][c];
            rec_store<OUT_BF16>(a.o, out_base + (int64_t)(t0 + tt) * a.out.stride_n + c, a.q_scale * acc);
            hook(t0 + tt, c, a.q_scale * acc);
        }
        // the next round's staging writes sq/sk/sv (not red); its first barrier
        // orders those writes against this round's reads of red.
    }
    if (a.state_out) {
        float *s1 = a.state_out + (int64_t)bh * D * D;
#pragma unroll
        for (int r = 0; r < R; ++r) s1[(g * R + r) * D + j] = S[r];
    }
}

}  // namespace lasad
