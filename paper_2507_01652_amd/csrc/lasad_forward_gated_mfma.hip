// Chunked forward for the vector, data-dependent decay of Section 3.4 / Algorithm 1 on the
// bf16 matrix cores (gfx950 MFMA), head dim 64, chunk 64, bf16 storage.
//
// Per token t the state row of key channel c is scaled by lambda_t[c] (1 at a row boundary)
// before k_t v_t^T is added.  With A_i[c] = prod_{s<=i} lambda_s[c] taken over the tokens of
// the chunk (chunk-local cumulative decay), unrolling the recurrence over the chunk gives
//
//   o_i   = (q_i . A_i)^T S_prev + sum_{j<=i} [ (q_i . A_i) . (k_j / A_j) ] v_j
//   S_new = diag(A_end) ( S_prev + sum_j (k_j / A_j) v_j^T )
//
// i.e. with Q~ = q_scale * Q . A and K~ = K / A (elementwise, per token and channel) the same
// four 64x64x64 contractions as the scalar-decay kernel: K~ Q~^T, (masked P) V, Q~ S, K~^T V,
// and one row scaling of S.  All decay sits inside the two operands, so the score tile only
// needs the causal mask.  Tiling, accumulator layouts and the transposed score / output tiles
// are those of lasad_forward_mfma.hip: four wavefronts, wave (a, c) owns key-channel half a and
// value-channel half c of the fp32 state (kept in accumulators), P^T = K~ Q~^T and
// O^T = V^T P^T + S^T Q~^T so that accumulators feed the next MFMA without shuffles.
//
// Chunk preparation, in registers.  Wave w fetches key channels 16w .. 16w+15 of all 64 tokens
// of the chunk: lane (r, p) holds tokens 2r, 2r+1 and channels 16w + 8p .. +7 of q, lambda, (k,)
// v as 16-byte pieces.  The running product of lambda along the tokens is a scan across the 32
// lanes of each half wavefront (DPP row shifts and the row-15 broadcast; no LDS, no barrier);
// the lane then forms K~ and Q~ for its two token rows, splits them into bf16 hi + lo and keeps
// them in registers until the tiles of the previous chunk are free.  This happens one chunk
// ahead, overlapped with the other wavefronts' MFMA work.  The tied key k = 1 - lambda uses
// lambda before the boundary override, as Algorithm 1 does.
//
// Precision: Q~, K~, P and S are computed operands and are each split into bf16 hi + lo (three
// MFMAs for a product of two split operands, two when one side is exact); v is exact bf16.
//
// Range.  K~ grows like 1 / A and Q~ shrinks like A.  Down to a chunk decay of 2^-100 per channel
// both stay normal numbers in fp32 and in their bf16 hi and lo parts for inputs of ordinary size
// (|k| 2^100 < 2^127; q_scale q 2^-100 and its low part, 2^-8 of it, > 2^-126), every valid score is
// a sum of products A_i / A_j <= 1, and a state row mixes only terms of its own channel.  A chunk
// whose total decay of some channel is below that (or zero) cannot be factored this way; the
// workgroup then abandons the chunked walk and redoes its whole sequence with the token-serial
// fp32 routine (lasad_scan.h), which applies each decay step by step.  Independent sigmoid gates
// of logits N(m, 1) stay inside the range for m >= 0.5 (median gate 0.62: worst channel of a
// chunk near 2^-73); at m = 0 the worst channels of a chunk straddle the limit.
#include <stdlib.h>

#include "lasad_forward_gated_common.h"
#include "lasad_scan.h"

namespace lasad {

namespace {

using namespace gated;

// FUSED >= 1 adds Algorithm 1's elementwise steps: q := SiLU(q) and lambda := sigmoid(lambda) while
// the chunk is prepared; FUSED = 2 also the root-mean-square normalisation of every output token
// over its 64 channels before it is stored.
// OCC: workgroups per compute unit the register budget is set for (1: 512 registers per lane).
template <int OUT_BF16, int OWNKEY, int FUSED, int OCC = 2>
__global__ void __launch_bounds__(kThreads, OCC)
forward_gated_mfma_kernel(ForwardArgs a)
{
    // tiles: Q~ hi, Q~ lo, K~ hi, K~ lo, V (stride TS); S^T hi, lo and the bf16 output tile (stride RS)
    constexpr int kTileHalfs = C * TS + 2 * C * KS + 2 * C * RS + 3 * D * RS;
    constexpr int kScanFloats = scan::lds_floats<OWNKEY ? scan::OWNKEY : scan::TIED>();
    constexpr int kLdsBytes = kTileHalfs * 2 > kScanFloats * 4 ? kTileHalfs * 2 : kScanFloats * 4;
    __shared__ __attribute__((aligned(16))) unsigned char smem_raw[kLdsBytes];
    __shared__ __attribute__((aligned(16))) float sTot[2][D];  // A_end per key channel, by chunk parity
    __shared__ __attribute__((aligned(16))) int sTrip[2][4];   // range flag of each wave, by chunk parity
    constexpr bool NORM = FUSED == 2;
    __shared__ float sSS[NORM ? 2 : 1][NORM ? C : 1];          // sum of squares of a token's two channel halves
    uint16_t *sQh = (uint16_t *)smem_raw;
    uint16_t *sQl = sQh + C * RS;
    uint16_t *sKh = sQl + C * RS;
    uint16_t *sKl = sKh + C * KS;
    uint16_t *sV = sKl + C * KS;
    uint16_t *sSh = sV + C * TS;        // S^T [dv][dk]
    uint16_t *sSl = sSh + D * RS;
    uint16_t *sO = sSl + D * RS;        // [token][dv]

    const int bh = blockIdx.x;
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wa = wave >> 1, wc = wave & 1;     // key-channel half, value-channel half
    const int l32 = lane & 31, g = lane >> 5;    // column inside the 32-wide tile, k-group

    const int n = a.n_tokens;
    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    const uint16_t *gq = (const uint16_t *)a.q + in_base;
    const uint16_t *gl = (const uint16_t *)a.lam + in_base;
    const uint16_t *gk = OWNKEY ? (const uint16_t *)a.k + in_base : nullptr;
    const uint16_t *gv = (const uint16_t *)a.v + in_base;
    const int64_t o_base = (int64_t)b * a.out.stride_b + (int64_t)h * a.out.stride_h;

    SplitConst sc;
    sc.init();

    // staging: token rows 2*l32, 2*l32 + 1 of the chunk, channels 16*wave + 8*g .. +7
    const int pcol = 16 * wave + 8 * g;
    ChunkStage<OWNKEY, (FUSED > 0)> stg;
    stg.trip = false;
    stg.fetch(gq, gl, gk, gv, 0, n, a.in.stride_n, l32, pcol);

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
    auto publish_state = [&]() {       // bf16 hi/lo copy of S^T for the Q~ S product of the next chunk
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            uint2 hi, lo;
            split2(accS[4 * qd + 0], accS[4 * qd + 1], hi.x, lo.x, sc);
            split2(accS[4 * qd + 2], accS[4 * qd + 3], hi.y, lo.y, sc);
            const int off = (wc * 32 + l32) * RS + wa * 32 + 8 * qd + 4 * g;
            *(uint2 *)&sSh[off] = hi;
            *(uint2 *)&sSl[off] = lo;
        }
    };
    if (have_state) publish_state();

    // causal mask of a diagonal 32 x 32 score block: key 8*qd + 4*g + e is at or before query l32
    // iff 8*qd + e <= cq
    const int cq = l32 - 4 * g;

    const int n_chunks = (n + C - 1) / C;
    int pending_rows = 0;          // NORM: rows of the output tile in LDS that are not stored yet
    stg.prepare(a, 0, n, lane, pcol, sTot[0], sc);
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int t0 = chunk * C;
        const int nt = min(C, n - t0);
        const int qa = wa ^ (chunk & 1);                  // query half of this wave in this chunk

        // ---- write the prepared tiles (free since barrier B of the previous chunk) ----
        stg.write(sQh, sQl, sKh, sKl, sV, l32, pcol);
        // Range flag: one LDS store per wave before the barrier, four loads after it (an atomic OR by
        // every thread on one LDS word, as __syncthreads_or does it, serialises: 2 us per chunk).
        {
            const bool any = __any(stg.trip);
            if (lane == 0) sTrip[chunk & 1][wave] = any ? 1 : 0;
        }
        __syncthreads();                                      // (A) operand tiles and A_end visible
        const int4 tf = *(const int4 *)sTrip[chunk & 1];
        if ((tf.x | tf.y | tf.z | tf.w) != 0) {               // some chunk left the range: give up the chunked walk
            __syncthreads();
            // every thread has left the tiles; redo the whole sequence step by step
            scan::scan_sequence<1, OUT_BF16, OWNKEY ? scan::OWNKEY : scan::TIED, 64>(a, bh, 0, (float *)smem_raw);
            return;
        }
        if (chunk + 1 < n_chunks) stg.fetch(gq, gl, gk, gv, chunk + 1, n, a.in.stride_n, l32, pcol);
        if (NORM && OUT_BF16 && pending_rows > 0) {       // the previous chunk's normalised tile, 16-byte rows
            uint16_t *go = (uint16_t *)a.o + o_base;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = (tid >> 3) + 32 * it;
                if (row < pending_rows)
                    *(uint4 *)(go + (int64_t)(t0 - C + row) * a.out.stride_n + (tid & 7) * 8) =
                        *(const uint4 *)&sO[row * RS + (tid & 7) * 8];
            }
            pending_rows = 0;
        }

        const int i_row = qa * 32 + l32;                  // this lane's query (column of the transposed tiles)
        Frag fqh[4], fql[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            fqh[s].u = *(const uint4 *)&sQh[(i_row) * RS + 16 * s + 8 * g];
            fql[s].u = *(const uint4 *)&sQl[(i_row) * RS + 16 * s + 8 * g];
        }

        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 acc0, acc1 = zero16, accO = zero16;
        // ---- scores P^T[j][i] = sum_c K~[j][c] Q~[i][c], key block 0 (and 1 for the upper query half) ----
        auto scores = [&](f32x16 &acc, int jb) {
            acc = zero16;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag kh, kl;
                kh.u = *(const uint4 *)&sKh[(jb * 32 + l32) * KS + 16 * s + 8 * g];
                kl.u = *(const uint4 *)&sKl[(jb * 32 + l32) * KS + 16 * s + 8 * g];
                acc = mfma(kh, fqh[s], acc);
                acc = mfma(kl, fqh[s], acc);
                acc = mfma(kh, fql[s], acc);
            }
        };
        scores(acc0, 0);
        // ---- O^T[n][i] += sum_dk S^T[n][dk] Q~[i][dk] ----
        if (have_state) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag sh, sl;
                sh.u = *(const uint4 *)&sSh[(wc * 32 + l32) * RS + 16 * s + 8 * g];
                sl.u = *(const uint4 *)&sSl[(wc * 32 + l32) * RS + 16 * s + 8 * g];
                accO = mfma(sh, fqh[s], accO);
                accO = mfma(sl, fqh[s], accO);
                accO = mfma(sh, fql[s], accO);
            }
        }
        if (qa == 1) scores(acc1, 1);

        // ---- state: S[dk][dv] += sum_j K~[j][dk] V[j][dv], then row dk times A_end[dk] ----
        Frag fv[4];
        {
            const int trow = (lane & 15) >> 2;
            const int vcol = wc * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
            const int kcol = wa * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int r0 = 16 * s + 4 * g + trow, r1 = r0 + 8;
                fv[s].h[0] = tr_read(&sV[r0 * TS + vcol]);
                fv[s].h[1] = tr_read(&sV[r1 * TS + vcol]);
                Frag fk;
                fk.h[0] = tr_read(&sKh[(r0) * KS + kcol]);
                fk.h[1] = tr_read(&sKh[(r1) * KS + kcol]);
                accS = mfma(fk, fv[s], accS);
                fk.h[0] = tr_read(&sKl[(r0) * KS + kcol]);
                fk.h[1] = tr_read(&sKl[(r1) * KS + kcol]);
                accS = mfma(fk, fv[s], accS);
            }
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const float4 t4 = *(const float4 *)&sTot[chunk & 1][wa * 32 + 8 * qd + 4 * g];
                accS[4 * qd + 0] *= t4.x; accS[4 * qd + 1] *= t4.y;
                accS[4 * qd + 2] *= t4.z; accS[4 * qd + 3] *= t4.w;
            }
            have_state = true;
        }

        // ---- causal mask on the fp32 scores, split to bf16 hi + lo, then P V ----
        auto mask_split = [&](const f32x16 &acc, bool diagonal, Frag *ph, Frag *pl) {
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                float p0 = acc[4 * qd + 0], p1 = acc[4 * qd + 1], p2 = acc[4 * qd + 2], p3 = acc[4 * qd + 3];
                if (diagonal) {
                    p0 = 8 * qd + 0 <= cq ? p0 : 0.f;
                    p1 = 8 * qd + 1 <= cq ? p1 : 0.f;
                    p2 = 8 * qd + 2 <= cq ? p2 : 0.f;
                    p3 = 8 * qd + 3 <= cq ? p3 : 0.f;
                }
                uint2 hi, lo;
                split2(p0, p1, hi.x, lo.x, sc);
                split2(p2, p3, hi.y, lo.y, sc);
                ph[qd / 2].h[qd % 2] = hi;
                pl[qd / 2].h[qd % 2] = lo;
            }
        };
        {
            Frag ph[2], pl[2];
            mask_split(acc0, qa == 0, ph, pl);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                accO = mfma(fv[s], ph[s], accO);
                accO = mfma(fv[s], pl[s], accO);
            }
        }
        if (qa == 1) {
            Frag ph[2], pl[2];
            mask_split(acc1, true, ph, pl);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                accO = mfma(fv[2 + s], ph[s], accO);
                accO = mfma(fv[2 + s], pl[s], accO);
            }
        }

        if (NORM) {
            // ---- Norm(o): every token divided by the root mean square of its 64 channels.  The two
            // value-channel waves of a query half exchange their sums of squares through LDS. ----
            float ss = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) ss = fmaf(accO[r], accO[r], ss);
            ss += __shfl_xor(ss, 32);
            if (g == 0) sSS[wc][i_row] = ss;
            __syncthreads();                              // (B) tile and S^T reads finished; sums visible
            const float rstd = __builtin_amdgcn_rsqf((sSS[0][i_row] + sSS[1][i_row]) * (1.0f / D) + a.norm_eps);
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                float4 w4 = make_float4(1.f, 1.f, 1.f, 1.f);
                if (a.norm_w) w4 = *(const float4 *)(a.norm_w + h * D + wc * 32 + 8 * qd + 4 * g);
                accO[4 * qd + 0] *= rstd * w4.x; accO[4 * qd + 1] *= rstd * w4.y;
                accO[4 * qd + 2] *= rstd * w4.z; accO[4 * qd + 3] *= rstd * w4.w;
            }
            pending_rows = nt;                            // a bf16 tile is stored after the next barrier
        }
        // ---- the output tile: a lane owns four consecutive value channels of its query per quad ----
        if (OUT_BF16) {                                   // via LDS for 16-byte coalesced stores
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                uint2 w2;
                w2.x = pack2(accO[4 * qd + 0], accO[4 * qd + 1]);
                w2.y = pack2(accO[4 * qd + 2], accO[4 * qd + 3]);
                *(uint2 *)&sO[i_row * RS + wc * 32 + 8 * qd + 4 * g] = w2;
            }
        } else if (i_row < nt) {
            float *go = (float *)a.o + o_base + (int64_t)(t0 + i_row) * a.out.stride_n + wc * 32 + 4 * g;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                *(float4 *)(go + 8 * qd) = make_float4(accO[4 * qd + 0], accO[4 * qd + 1],
                                                       accO[4 * qd + 2], accO[4 * qd + 3]);
        }
        if (chunk + 1 < n_chunks) stg.prepare(a, chunk + 1, n, lane, pcol, sTot[(chunk + 1) & 1], sc);   // its loads have landed by now
        if (!NORM) {
            __syncthreads();                              // (B) all reads of the tiles and of S^T finished
            if (OUT_BF16) {                               // coalesced 16-byte stores of the bf16 tile
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
        if (chunk + 1 < n_chunks) publish_state();        // read after the next barrier (A)
    }
    if (NORM && OUT_BF16 && pending_rows > 0) {           // the last chunk's normalised tile
        __syncthreads();
        uint16_t *go = (uint16_t *)a.o + o_base;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int row = (tid >> 3) + 32 * it;
            if (row < pending_rows)
                *(uint4 *)(go + (int64_t)((n_chunks - 1) * C + row) * a.out.stride_n + (tid & 7) * 8) =
                    *(const uint4 *)&sO[row * RS + (tid & 7) * 8];
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

hipError_t launch_forward_gated_mfma(const ForwardArgs &a, hipStream_t s)
{
    if (a.d != D || a.io_dtype != LASAD_BF16 || a.n_tokens < 1 || !a.lam) return hipErrorInvalidValue;
    const int64_t n_seq = (int64_t)a.B * a.Hh;
    if (n_seq > 0x7fffffff) return hipErrorInvalidValue;
    // while every sequence gets a compute unit of its own: the twelve-wave kernel (LASAD_GATED_WS=0 / 1 forces the choice)
    static const int ws_env = [] { const char *e = getenv("LASAD_GATED_WS"); return e ? atoi(e) : -1; }();
    // the fused layer with its norm: always (measured 67 against 94 us at 512 sequences; the four-wave
    // variant needs the register budget of one workgroup per compute unit there)
    const bool layer = a.norm && a.fused_act;
    if ((!a.norm || a.fused_act) && (ws_env == 1 || (ws_env < 0 && (n_seq <= 256 || layer)))) return launch_forward_gated_ws(a, s);
    const dim3 grid((unsigned)n_seq), block(kThreads);
    const bool out16 = a.out_dtype == LASAD_BF16;
    if (a.fused_act || a.norm) {
        if (a.k || !a.fused_act) return hipErrorInvalidValue;      // the fused layer ties the key to the gate
        if (a.norm) {
            // The normalised bf16 tile keeps the output accumulators alive across a barrier; at two
            // workgroups per compute unit that spills registers and measures slower (104 vs 87 us at
            // the large shape), so this variant takes the one-workgroup register budget.
            if (out16) hipLaunchKernelGGL((forward_gated_mfma_kernel<1, 0, 2, 1>), grid, block, 0, s, a);
            else hipLaunchKernelGGL((forward_gated_mfma_kernel<0, 0, 2>), grid, block, 0, s, a);
        } else {
            if (out16) hipLaunchKernelGGL((forward_gated_mfma_kernel<1, 0, 1>), grid, block, 0, s, a);
            else hipLaunchKernelGGL((forward_gated_mfma_kernel<0, 0, 1>), grid, block, 0, s, a);
        }
    } else if (a.k) {
        if (out16) hipLaunchKernelGGL((forward_gated_mfma_kernel<1, 1, 0>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((forward_gated_mfma_kernel<0, 1, 0>), grid, block, 0, s, a);
    } else {
        if (out16) hipLaunchKernelGGL((forward_gated_mfma_kernel<1, 0, 0>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((forward_gated_mfma_kernel<0, 0, 0>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace lasad
