// Pieces shared by the vector-decay matrix-core kernels (lasad_forward_gated_mfma.hip and its
// wave-specialised variant lasad_forward_gated_ws.hip): tile geometry, the running-product scan
// across lanes, and the in-register preparation of one chunk's operands.
#pragma once

#include "lasad_mfma_util.h"
#include "lasad_internal.h"
#include "lasad_scan.h"

namespace lasad {
namespace gated {

constexpr int C = 64;      // chunk length (tokens)
constexpr int D = 64;      // head dim
constexpr int kThreads = 256;
#ifndef LASAD_GATED_KS
#define LASAD_GATED_KS 80
#endif
constexpr int TS = 80;     // LDS row stride (bf16 elements) of the V tile (transpose reads): 160 B
constexpr int KS = LASAD_GATED_KS;   // of the K~ tiles (16-byte row reads and transpose reads)
constexpr int RS = 72;     // of the Q~, S^T and output tiles (16-byte row reads): 144 B
constexpr float kMinChunkDecay = 7.8886091e-31f;   // 2^-100

// Running products of eight values along the 32 lanes of each half wavefront: on return x[c]
// of lane l holds the product over lanes 0..l of its half (inclusive) and e[c] the product over
// lanes 0..l-1 (1 in lane 0 of a half).  Each DPP step multiplies by the value 1, 2, 4, 8 lanes
// down the 16-lane row (lanes without a source keep their value), the last one by lane 15 of
// the row below (rows 1 and 3 only).  The eight chains are interleaved, so every DPP source
// was written eight instructions earlier; the s_nop covers what preceded the block.
#define SCAN_STEP(ctrl)                                                                           \
    "v_mul_f32_dpp %0, %0, %0 " ctrl "\n v_mul_f32_dpp %1, %1, %1 " ctrl "\n"                     \
    "v_mul_f32_dpp %2, %2, %2 " ctrl "\n v_mul_f32_dpp %3, %3, %3 " ctrl "\n"                     \
    "v_mul_f32_dpp %4, %4, %4 " ctrl "\n v_mul_f32_dpp %5, %5, %5 " ctrl "\n"                     \
    "v_mul_f32_dpp %6, %6, %6 " ctrl "\n v_mul_f32_dpp %7, %7, %7 " ctrl "\n"
__device__ inline void scan_mul32x8(float (&x)[8], float (&e)[8], bool half_start)
{
    asm("s_nop 1\n"
        SCAN_STEP("row_shr:1 row_mask:0xf bank_mask:0xf")
        SCAN_STEP("row_shr:2 row_mask:0xf bank_mask:0xf")
        SCAN_STEP("row_shr:4 row_mask:0xf bank_mask:0xf")
        SCAN_STEP("row_shr:8 row_mask:0xf bank_mask:0xf")
        SCAN_STEP("row_bcast:15 row_mask:0xa bank_mask:0xf")
        : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]));
#pragma unroll
    for (int c = 0; c < 8; ++c) e[c] = 1.0f;
    asm("s_nop 1\n"
        "v_mov_b32_dpp %0, %8 wave_shr:1 row_mask:0xf bank_mask:0xf\n v_mov_b32_dpp %1, %9 wave_shr:1 row_mask:0xf bank_mask:0xf\n"
        "v_mov_b32_dpp %2, %10 wave_shr:1 row_mask:0xf bank_mask:0xf\n v_mov_b32_dpp %3, %11 wave_shr:1 row_mask:0xf bank_mask:0xf\n"
        "v_mov_b32_dpp %4, %12 wave_shr:1 row_mask:0xf bank_mask:0xf\n v_mov_b32_dpp %5, %13 wave_shr:1 row_mask:0xf bank_mask:0xf\n"
        "v_mov_b32_dpp %6, %14 wave_shr:1 row_mask:0xf bank_mask:0xf\n v_mov_b32_dpp %7, %15 wave_shr:1 row_mask:0xf bank_mask:0xf\n"
        : "+v"(e[0]), "+v"(e[1]), "+v"(e[2]), "+v"(e[3]), "+v"(e[4]), "+v"(e[5]), "+v"(e[6]), "+v"(e[7])
        : "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]), "v"(x[4]), "v"(x[5]), "v"(x[6]), "v"(x[7]));
#pragma unroll
    for (int c = 0; c < 8; ++c) e[c] = half_start ? 1.0f : e[c];
}

// x where keep, else every 32-bit word = fill (component-wise, so the values stay in registers)
__device__ inline uint4 keep_or(bool keep, uint4 x, uint32_t fill)
{
    return make_uint4(keep ? x.x : fill, keep ? x.y : fill, keep ? x.z : fill, keep ? x.w : fill);
}

// One chunk of staged inputs and prepared operands of a staging thread: lane (l32, g) of staging
// wave w holds token rows 2*l32, 2*l32 + 1 and channels pcol = 16*w + 8*g .. +7.
// The backward passes (lasad_backward_gated_mfma.hip) stage the same operands from other tensors:
// SHIFT = 1 takes the decay of token m from the decay tensor's token m - 1 (none at token 0: the
// walk runs the sequence backwards and step m applies the decay of the step before it);
// QMODE = 1 stages Q~ = q_scale A (query 1), QMODE = 2 takes the query as 1 - x from its tensor.
// FUSED = 1 reads pre-activation tensors (Algorithm 1): the decay tensor holds gate logits (sigmoid
// on load, also where it feeds the QMODE = 2 query), a QMODE = 0 query and an own key hold the
// pre-activation query (SiLU on load; an own key together with FUSED occurs in the backward passes
// only, whose key operand is the forward's query).
// WITH_V = 0 leaves the V tile to somebody else (the state waves of the twelve-wave kernel).
template <int OWNKEY, int FUSED, int SHIFT = 0, int QMODE = 0, int WITH_V = 1>
struct ChunkStage {
    uint4 rq[2], rl[2], rk[2], rv[2];                 // as fetched: q, lambda (or gate logits), own key, v
    uint4 pkh[2], pkl[2], pqh[2], pql[2], pv[2];      // prepared: K~ hi / lo, Q~ hi / lo, v
    bool trip;                                        // some channel's chunk decay is below the limit
    float lam[2][8], kk[2][8];                        // between the two halves of prepare(): decay (then A) and key, fp32
    uint4 qc[2];                                      // and the fetched query pieces

    // unconditional, clamped 16-byte loads of chunk `chunk` of a sequence of n tokens
    __device__ void fetch(const uint16_t *gq, const uint16_t *gl, const uint16_t *gk, const uint16_t *gv,
                          int chunk, int n, int64_t stride_n, int l32, int pcol)
    {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int tok = min(chunk * C + 2 * l32 + it, n - 1);
            const int64_t off = (int64_t)tok * stride_n + pcol;
            if (QMODE != 1) rq[it] = *(const uint4 *)(gq + off);
            rl[it] = *(const uint4 *)(gl + (SHIFT ? (int64_t)max(tok - 1, 0) * stride_n + pcol : off));
            if (OWNKEY) rk[it] = *(const uint4 *)(gk + off);
            if (WITH_V) rv[it] = *(const uint4 *)(gv + off);
        }
    }

    // K~ = k / A and Q~ = q_scale q A (bf16 hi + lo) for this lane's rows; A_end of the lane's
    // channels goes to sTotN (written by the lanes that hold the last token pair).  Two halves:
    // prepare_begin() consumes the fetched registers (a caller may issue the next fetch() right
    // after it), prepare_end() does the scan, the scaling and the splits.
    __device__ void prepare(const ForwardArgs &a, int chunk, int n, int lane, int pcol, float *sTotN,
                            const SplitConst &sc)
    {
        prepare_begin(a, chunk, n, lane);
        prepare_end(a, lane, pcol, sTotN, sc);
    }

    __device__ void prepare_begin(const ForwardArgs &a, int chunk, int n, int lane)
    {
        const int l32 = lane & 31;
        const int t0 = chunk * C, nt = min(C, n - t0);
        // which of the chunk's 64 tokens sit on a row boundary (bit t), same in every wavefront
        const unsigned long long bmask = __ballot(is_boundary(a.start_pos + t0 + lane + 1, a.grid_w, a.mode));
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int row = 2 * l32 + it;
            const bool bnd = (bmask >> row) & 1ull;
            const uint32_t lw[4] = {rl[it].x, rl[it].y, rl[it].z, rl[it].w};
            const uint32_t kw[4] = {rk[it].x, rk[it].y, rk[it].z, rk[it].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float l0 = __uint_as_float(lw[e] << 16), l1 = __uint_as_float(lw[e] & 0xffff0000u);
                if (FUSED) { l0 = sigmoid_f32(l0); l1 = sigmoid_f32(l1); }
                float k0 = OWNKEY ? __uint_as_float(kw[e] << 16) : 1.0f - l0;
                float k1 = OWNKEY ? __uint_as_float(kw[e] & 0xffff0000u) : 1.0f - l1;
                if (OWNKEY && FUSED) { k0 = silu_f32(k0); k1 = silu_f32(k1); }
                kk[it][2 * e] = k0;
                kk[it][2 * e + 1] = k1;
                const bool no_decay = bnd || (SHIFT && t0 + row == 0);
                lam[it][2 * e] = no_decay ? 1.0f : l0;
                lam[it][2 * e + 1] = no_decay ? 1.0f : l1;
            }
            if (WITH_V) pv[it] = rv[it];
        }
        if (nt < C) {                                      // tail chunk: rows past the end get lambda 1, q = k = v = 0
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const bool live = 2 * l32 + it < nt;
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    kk[it][c] = live ? kk[it][c] : 0.f;
                    lam[it][c] = live ? lam[it][c] : 1.0f;
                }
                if (WITH_V) pv[it] = keep_or(live, pv[it], 0u);
                if (QMODE == 0) rq[it] = keep_or(live, rq[it], 0u);
                // a query of zero: 1 - 1, or 1 - sigmoid(100) (= 1 - 1 in fp32)
                if (QMODE == 2) rq[it] = keep_or(live, rq[it], FUSED ? 0x42c842c8u : 0x3f803f80u);
            }
        }
        if (QMODE != 1) { qc[0] = rq[0]; qc[1] = rq[1]; }
    }

    __device__ void prepare_end(const ForwardArgs &a, int lane, int pcol, float *sTotN, const SplitConst &sc)
    {
        const int l32 = lane & 31;
        // product over the token pairs of lanes 0..l32 (tot) and 0..l32-1 (exc), per channel
        float tot[8], exc[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) tot[c] = lam[0][c] * lam[1][c];
        scan_mul32x8(tot, exc, l32 == 0);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            lam[0][c] *= exc[c];                                // A of token 2*l32
            lam[1][c] *= lam[0][c];                             // A of token 2*l32 + 1
        }
        if (l32 == 31) {                                        // chunk totals A_end of this half's channels
            *(float4 *)&sTotN[pcol] = make_float4(tot[0], tot[1], tot[2], tot[3]);
            *(float4 *)&sTotN[pcol + 4] = make_float4(tot[4], tot[5], tot[6], tot[7]);
        }
        // A decreases along the tokens: the smallest value of each channel sits in lane 31
        float amin = lam[1][0];
#pragma unroll
        for (int c = 1; c < 8; ++c) amin = fminf(amin, lam[1][c]);
        trip = !(amin >= kMinChunkDecay);
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            uint32_t qw[4] = {0u, 0u, 0u, 0u};
            if (QMODE != 1) { qw[0] = qc[it].x; qw[1] = qc[it].y; qw[2] = qc[it].z; qw[3] = qc[it].w; }
            uint32_t kh[4], kl[4], qh[4], ql[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a0 = lam[it][2 * e], a1 = lam[it][2 * e + 1];
                split2(kk[it][2 * e] * __builtin_amdgcn_rcpf(a0), kk[it][2 * e + 1] * __builtin_amdgcn_rcpf(a1), kh[e], kl[e], sc);
                float q0 = 1.0f, q1 = 1.0f;
                if (QMODE != 1) { q0 = __uint_as_float(qw[e] << 16); q1 = __uint_as_float(qw[e] & 0xffff0000u); }
                if (QMODE == 2 && FUSED) { q0 = sigmoid_f32(q0); q1 = sigmoid_f32(q1); }
                if (QMODE == 2) { q0 = 1.0f - q0; q1 = 1.0f - q1; }
                if (QMODE == 0 && FUSED) { q0 = silu_f32(q0); q1 = silu_f32(q1); }
                split2(q0 * (a0 * a.q_scale), q1 * (a1 * a.q_scale), qh[e], ql[e], sc);
            }
            pkh[it] = make_uint4(kh[0], kh[1], kh[2], kh[3]); pkl[it] = make_uint4(kl[0], kl[1], kl[2], kl[3]);
            pqh[it] = make_uint4(qh[0], qh[1], qh[2], qh[3]); pql[it] = make_uint4(ql[0], ql[1], ql[2], ql[3]);
        }
    }

    // the prepared 16-byte tile rows
    __device__ void write(uint16_t *sQh, uint16_t *sQl, uint16_t *sKh, uint16_t *sKl, uint16_t *sV,
                          int l32, int pcol) const
    {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int row = 2 * l32 + it;
            *(uint4 *)&sKh[row * KS + pcol] = pkh[it];
            *(uint4 *)&sKl[row * KS + pcol] = pkl[it];
            *(uint4 *)&sQh[row * RS + pcol] = pqh[it];
            *(uint4 *)&sQl[row * RS + pcol] = pql[it];
            if (WITH_V) *(uint4 *)&sV[row * TS + pcol] = pv[it];
        }
    }
};

// The token-serial redo of one sequence (range fallback of the chunked kernels), as a real call:
// inlined into a kernel it makes the compiler keep the argument block in scratch memory and
// reload fields from there inside the chunk loop of the twelve-wave kernel (measured: 18 instead
// of 11 us at the base shape).  The four-wave kernel is faster with the inlined routine.
template <int OUT_BF16, int OWNKEY>
__device__ __noinline__ void redo_sequence(const ForwardArgs *a, int bh, float *lds)
{
    scan::scan_sequence<1, OUT_BF16, OWNKEY ? scan::OWNKEY : scan::TIED, 64>(*a, bh, 0, lds);
}

}  // namespace gated
}  // namespace lasad
