// Chunked forward on the bf16 matrix cores (gfx950 MFMA), head dim 64, chunk 64.
//
// Unrolling Section 3.4's recurrence over a chunk of C tokens that starts after
// position c0 gives, with e_i = E(i) - E(c0) (number of decaying steps between the
// chunk start and token i; E is the integer prefix of the boundary rule):
//
//   o_i   = gamma^{e_i} q_i^T S_prev  +  sum_{j<=i} gamma^{e_i - e_j} (q_i . k_j) v_j
//   S_new = gamma^{e_C} S_prev        +  sum_j      gamma^{e_C - e_j}  k_j v_j^T
//
// i.e. per chunk four 64x64x64 contractions: K Q^T, (masked P) V, Q S and K^T V.
//
// One workgroup of four wavefronts walks one (batch, head) sequence.  Wave (a, c)
// owns query half a / key-channel half a and value-channel half c (32 x 32 tiles,
// v_mfma_f32_32x32x16_bf16).  Layout choices, all to avoid shuffling data between
// the MFMA accumulator layout and the MFMA operand layout:
//  * the score tile is computed transposed, P^T = K Q^T: a lane then holds, for
//    its query column i, key rows j in groups of four consecutive -- which is
//    exactly an A/B operand fragment of the next MFMA once the reduction index j
//    is enumerated in that same (permuted) order on the V side;
//  * the output tile is computed transposed, O^T = V^T P^T + S^T Q^T, so the
//    per-query decay gamma^{e_i} is one scalar per lane and a lane owns four
//    consecutive value channels of its query (8-byte LDS writes on the way out);
//  * V and K are kept row-major (token, channel) in LDS, as they arrive from
//    HBM; their token-major operand fragments (reduction over tokens) come from
//    the LDS transpose read ds_read_b64_tr_b16;
//  * the fp32 state stays in MFMA accumulators for the whole sequence; a bf16
//    copy S^T goes through LDS once per chunk for the Q S product.
// Precision.  The matrix cores take bf16 operands, but rounding the computed
// operands (masked scores P, state S, decayed values b (.) V) to one bf16 each
// costs about 2^-9 of the local output magnitude per site, which on heavy-tailed
// outputs exceeds a 2e-2-of-RMS budget at the largest element.  Each computed
// operand is therefore split into a bf16 pair hi + lo (lo = the rounding
// residual) and multiplied with two MFMAs; q, k, v themselves are exact bf16.
// The kernel is bound by HBM, not by the matrix cores, so the extra MFMAs hide
// under the memory time.
//
// Decay.  Powers of gamma are only ever formed for in-chunk exponent differences
// (0..64).  For gamma > 0.5 the mask is separable, gamma^{e_i - e_j} =
// gamma^{e_i} * gamma^{-e_j} with gamma^{-e_j} <= 2^64: the column factor is one
// table lookup and multiply per score, the row factor one multiply per output.
// For smaller gamma (where gamma^{-e_j} could overflow) every score gets its own
// exp2((e_i - e_j) log2 gamma).
#include "lasad_internal.h"

namespace lasad {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((__vector_size__(4 * sizeof(short))));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int C = 64;      // chunk length (tokens)
constexpr int D = 64;      // head dim
constexpr int kThreads = 256;
constexpr int RS = 72;     // LDS row stride (elements) of tiles read 16 bytes at a time: 144 B
constexpr int VS = 80;     // LDS row stride of the V tile (transpose reads only): 160 B

struct Frag {              // 8 bf16 = one lane's share of a 32x16 MFMA operand
    union { bf16x8 v; uint4 u; uint2 h[2]; };
};

__device__ inline uint32_t pack2(float lo, float hi)
{
    f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

__device__ inline uint2 tr_read(const uint16_t *p)
{
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
    return __builtin_bit_cast(uint2, r);
}

__device__ inline f32x16 mfma(const Frag &a, const Frag &b, f32x16 acc)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc, 0, 0, 0);
}

// split a pair of fp32 values into packed bf16 hi (round to nearest) and lo (residual)
__device__ inline void split2(float x0, float x1, uint32_t &hi, uint32_t &lo)
{
    hi = pack2(x0, x1);
    const float h0 = __uint_as_float(hi << 16), h1 = __uint_as_float(hi & 0xffff0000u);
    lo = pack2(x0 - h0, x1 - h1);
}

template <int OUT_BF16>
__global__ void __launch_bounds__(kThreads, 2)
forward_mfma_kernel(ForwardArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t sQ[C * RS];
    __shared__ __attribute__((aligned(16))) uint16_t sK[C * RS];
    __shared__ __attribute__((aligned(16))) uint16_t sV[C * VS];
    __shared__ __attribute__((aligned(16))) uint16_t sSt[2][2][D * RS];   // [buffer][hi, lo] bf16 S^T [dv][dk]
    __shared__ __attribute__((aligned(16))) uint16_t sO[OUT_BF16 ? C * RS : 8];   // bf16 output tile [token][dv]
    __shared__ __attribute__((aligned(16))) float tabE[C];   // e_j as float
    __shared__ __attribute__((aligned(16))) float tabC[C];   // gamma^{-e_j} (separable path)
    __shared__ __attribute__((aligned(16))) float tabB[C];   // gamma^{e_end - e_j}, 0 for rows past the end

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wa = wave >> 1, wc = wave & 1;     // query/key-channel half, value-channel half
    const int l32 = lane & 31, g = lane >> 5;    // column inside the 32-wide tile, k-group
    const int bh = blockIdx.x;
    const int b = bh / a.Hh, h = bh - b * a.Hh;

    const float gamma = a.gamma[h];
    const float lg = log2f(gamma);               // -inf for gamma == 0 (guarded where used)
    const bool separable = lg * (float)C > -64.0f;   // gamma^{-64} <= 2^64

    const uint16_t *gq = (const uint16_t *)a.q + (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    const uint16_t *gk = (const uint16_t *)a.k + (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    const uint16_t *gv = (const uint16_t *)a.v + (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    const int64_t o_base = (int64_t)b * a.out.stride_b + (int64_t)h * a.out.stride_h;

    // --- state accumulators: S[dk = wa*32 + 8*(r/4) + 4*g + r%4][dv = wc*32 + l32] ---
    f32x16 accS;
    bool have_state = a.state_in != nullptr;
    if (have_state) {
        const float *s0 = a.state_in + (int64_t)bh * D * D;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            accS[r] = s0[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32];
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) accS[r] = 0.f;
    }
    // bf16 hi/lo copy of S^T for the Q S product of the next chunk
    auto publish_state = [&](int buf) {
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            uint2 hi, lo;
            split2(accS[4 * qd + 0], accS[4 * qd + 1], hi.x, lo.x);
            split2(accS[4 * qd + 2], accS[4 * qd + 3], hi.y, lo.y);
            const int off = (wc * 32 + l32) * RS + wa * 32 + 8 * qd + 4 * g;
            *(uint2 *)&sSt[buf][0][off] = hi;
            *(uint2 *)&sSt[buf][1][off] = lo;
        }
    };
    if (have_state) publish_state(0);

    const int n_chunks = (a.n_tokens + C - 1) / C;

    // global -> register staging: thread loads 16 B pieces (row = tid/8 + 32*it, piece = tid%8)
    uint4 rq[2], rk[2], rv[2];
    auto prefetch = [&](int chunk) {
        const int t0 = chunk * C;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int row = (tid >> 3) + 32 * it;
            const int tok = t0 + row;
            if (tok < a.n_tokens) {
                const int64_t off = (int64_t)tok * a.in.stride_n + (tid & 7) * 8;
                rq[it] = *(const uint4 *)(gq + off);
                rk[it] = *(const uint4 *)(gk + off);
                rv[it] = *(const uint4 *)(gv + off);
            } else {
                rq[it] = rk[it] = rv[it] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    prefetch(0);

    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int t0 = chunk * C;
        const int nt = min(C, a.n_tokens - t0);
        const int c0 = a.start_pos + t0;                 // tokens before this chunk
        const int cur = chunk & 1;

        // ---- stage tiles and per-chunk decay tables into LDS ----
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int row = (tid >> 3) + 32 * it;
            const int col = (tid & 7) * 8;
            *(uint4 *)&sQ[row * RS + col] = rq[it];
            *(uint4 *)&sK[row * RS + col] = rk[it];
            *(uint4 *)&sV[row * VS + col] = rv[it];
        }
        const int e_base = cum_exp(c0, a.grid_w, a.mode);
        const int e_end = cum_exp(c0 + nt, a.grid_w, a.mode) - e_base;
        if (tid < C) {
            const int ej = cum_exp(c0 + 1 + tid, a.grid_w, a.mode) - e_base;
            tabE[tid] = (float)ej;
            tabC[tid] = separable ? __builtin_amdgcn_exp2f(-(float)ej * lg) : 0.f;
            const int de = e_end - ej;
            tabB[tid] = tid < nt ? (de == 0 ? 1.0f : __builtin_amdgcn_exp2f((float)de * lg)) : 0.0f;
        }
        __syncthreads();                                  // (A) tiles, tables and S^T[cur] visible
        if (chunk + 1 < n_chunks) prefetch(chunk + 1);

        // ---- Q fragments of this wave's query half: row i = wa*32 + l32, channels 16*s + 8*g .. +7 ----
        Frag fq[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) fq[s].u = *(const uint4 *)&sQ[(wa * 32 + l32) * RS + 16 * s + 8 * g];

        const int i_row = wa * 32 + l32;                  // this lane's query (column of the transposed tiles)
        const float e_i = tabE[i_row];
        const float r_i = (e_i == 0.f) ? 1.0f : __builtin_amdgcn_exp2f(e_i * lg);   // gamma^{e_i}

        // ---- P^T[j][i] = sum_d K[j][d] Q[i][d]; key block 1 is fully masked for query half 0 ----
        Frag fph[4], fpl[4];                              // bf16 hi / lo fragments of P, reduction index j permuted
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            if (jb <= wa) {
                f32x16 acc;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    Frag fk;
                    fk.u = *(const uint4 *)&sK[(jb * 32 + l32) * RS + 16 * s + 8 * g];
                    acc = mfma(fk, fq[s], acc);
                }
                // decay + causal mask on the fp32 scores, then split to bf16 hi + lo
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    const int j0 = jb * 32 + 8 * qd + 4 * g;
                    float p[4];
                    if (separable) {
                        const float4 c4 = *(const float4 *)&tabC[j0];
                        p[0] = acc[4 * qd + 0] * c4.x; p[1] = acc[4 * qd + 1] * c4.y;
                        p[2] = acc[4 * qd + 2] * c4.z; p[3] = acc[4 * qd + 3] * c4.w;
                    } else {
                        const float4 ej4 = *(const float4 *)&tabE[j0];
                        const float ej[4] = {ej4.x, ej4.y, ej4.z, ej4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float de = e_i - ej[e];
                            p[e] = acc[4 * qd + e] * ((de == 0.f) ? 1.0f : __builtin_amdgcn_exp2f(de * lg));
                        }
                    }
                    if (jb == wa) {                       // diagonal block: causal mask
#pragma unroll
                        for (int e = 0; e < 4; ++e) p[e] = (j0 + e <= i_row) ? p[e] : 0.f;
                    }
                    // fragment for k-step s = 2*jb + qd/2, half qd%2
                    uint2 hi, lo;
                    split2(p[0], p[1], hi.x, lo.x);
                    split2(p[2], p[3], hi.y, lo.y);
                    fph[2 * jb + qd / 2].h[qd % 2] = hi;
                    fpl[2 * jb + qd / 2].h[qd % 2] = lo;
                }
            } else {
                fph[2 * jb].u = fph[2 * jb + 1].u = make_uint4(0, 0, 0, 0);
                fpl[2 * jb].u = fpl[2 * jb + 1].u = make_uint4(0, 0, 0, 0);
            }
        }

        // ---- O^T[n][i] = gamma^{e_i} sum_dk S^T[n][dk] Q[i][dk]  +  sum_j V[j][n] P[i][j] ----
        // (separable path: P lacks the row factor gamma^{e_i}, applied to the whole sum at the end)
        f32x16 accO;
#pragma unroll
        for (int r = 0; r < 16; ++r) accO[r] = 0.f;
        if (have_state) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag fs;
                fs.u = *(const uint4 *)&sSt[cur][0][(wc * 32 + l32) * RS + 16 * s + 8 * g];
                accO = mfma(fs, fq[s], accO);
                fs.u = *(const uint4 *)&sSt[cur][1][(wc * 32 + l32) * RS + 16 * s + 8 * g];
                accO = mfma(fs, fq[s], accO);
            }
            if (!separable) {
#pragma unroll
                for (int r = 0; r < 16; ++r) accO[r] *= r_i;
            }
        }
        // V fragments: value channel n = wc*32 + l32, token rows 16*s + 4*g + {0..3} and + 8
        Frag fv[4];
        {
            const int trow = (lane & 15) >> 2;                       // row inside the 4-row group this lane points at
            const int tcol = wc * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                fv[s].h[0] = tr_read(&sV[(16 * s + 4 * g + trow) * VS + tcol]);
                fv[s].h[1] = tr_read(&sV[(16 * s + 8 + 4 * g + trow) * VS + tcol]);
            }
        }
        const int s_max = wa == 0 ? 2 : 4;               // key rows 32..63 carry zero P for query half 0
#pragma unroll
        for (int s = 0; s < 4; ++s)
            if (s < s_max) {
                accO = mfma(fv[s], fph[s], accO);
                accO = mfma(fv[s], fpl[s], accO);
            }
        {
            const float osc = separable ? a.q_scale * r_i : a.q_scale;
#pragma unroll
            for (int r = 0; r < 16; ++r) accO[r] *= osc;
        }

        // ---- state update: S <- gamma^{e_end} S + K^T (b (.) V) ----
        {
            const float gtot = (e_end == 0) ? 1.0f : __builtin_amdgcn_exp2f((float)e_end * lg);
#pragma unroll
            for (int r = 0; r < 16; ++r) accS[r] *= gtot;
            const int trow = (lane & 15) >> 2;
            const int tcol = wa * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag fkt, fvh, fvl;
                fkt.h[0] = tr_read(&sK[(16 * s + 4 * g + trow) * RS + tcol]);
                fkt.h[1] = tr_read(&sK[(16 * s + 8 + 4 * g + trow) * RS + tcol]);
                // scale V rows by b_j (slot e <-> token 16*s + 8*(e/4) + 4*g + e%4), split hi + lo
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const float4 b4 = *(const float4 *)&tabB[16 * s + 8 * hh + 4 * g];
                    const uint2 raw = fv[s].h[hh];
                    const float v0 = __uint_as_float(raw.x << 16) * b4.x;
                    const float v1 = __uint_as_float(raw.x & 0xffff0000u) * b4.y;
                    const float v2 = __uint_as_float(raw.y << 16) * b4.z;
                    const float v3 = __uint_as_float(raw.y & 0xffff0000u) * b4.w;
                    uint2 hi, lo;
                    split2(v0, v1, hi.x, lo.x);
                    split2(v2, v3, hi.y, lo.y);
                    fvh.h[hh] = hi;
                    fvl.h[hh] = lo;
                }
                accS = mfma(fkt, fvh, accS);             // S[dk][dv] += sum_j K[j][dk] * (b_j V[j][dv])
                accS = mfma(fkt, fvl, accS);
            }
            have_state = true;
        }

        // ---- hand the new S^T to the next chunk; send the output tile out ----
        if (chunk + 1 < n_chunks) publish_state(cur ^ 1);
        if (OUT_BF16) {
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                uint2 w2;
                w2.x = pack2(accO[4 * qd + 0], accO[4 * qd + 1]);
                w2.y = pack2(accO[4 * qd + 2], accO[4 * qd + 3]);
                *(uint2 *)&sO[i_row * RS + wc * 32 + 8 * qd + 4 * g] = w2;
            }
        } else if (i_row < nt) {
            // fp32 output: a lane owns 4 consecutive value channels of its query, 16-byte stores
            float *go = (float *)a.o + o_base + (int64_t)(t0 + i_row) * a.out.stride_n + wc * 32 + 4 * g;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                *(float4 *)(go + 8 * qd) = make_float4(accO[4 * qd + 0], accO[4 * qd + 1],
                                                       accO[4 * qd + 2], accO[4 * qd + 3]);
        }
        __syncthreads();                                  // (B) output tile complete; all tile reads finished

        if (OUT_BF16) {                                   // coalesced 16-byte stores of the bf16 tile
            uint16_t *go = (uint16_t *)a.o + o_base;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = (tid >> 3) + 32 * it;
                if (row < nt)
                    *(uint4 *)(go + (int64_t)(t0 + row) * a.out.stride_n + (tid & 7) * 8) =
                        *(const uint4 *)&sO[row * RS + (tid & 7) * 8];
            }
        }
    }

    if (a.state_out) {
        float *s1 = a.state_out + (int64_t)bh * D * D;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s1[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32] = accS[r];
    }
}

}  // namespace

hipError_t launch_forward_mfma(const ForwardArgs &a, hipStream_t s)
{
    if (a.d != D || a.io_dtype != LASAD_BF16) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(a.B * a.Hh)), block(kThreads);
    if (a.out_dtype == LASAD_BF16) hipLaunchKernelGGL(forward_mfma_kernel<1>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(forward_mfma_kernel<0>, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace lasad
