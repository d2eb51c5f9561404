// The twelve-wave workgroup of the chunked vector-decay kernels, shared by the forward
// (lasad_forward_gated_ws.hip) and by the passes of the backward (lasad_backward_gated_mfma.hip):
// three groups of four wavefronts on the same four SIMDs, every LDS buffer doubled, one barrier per
// chunk.
//
//   output waves (0-3):  scores, causal mask + split, second product, state term, output tile      (chunk c)
//   state waves  (4-7):  state update K~^T V, row scaling by A_end, bf16 hi/lo copy of S^T,
//                        V tile of chunk c + 1 (a plain copy)                                     (chunk c -> c+1)
//   loader waves (8-11): global loads, running decay products, K~ and Q~ (split), tile writes     (chunk c+1),
//                        16-byte stores of the finished bf16 output tile                          (chunk c-1)
//
// Template switches: FUSED (SiLU / sigmoid while staging), NORM (RMS norm of the output tile: sums
// of squares before the chunk's barrier, the tile scaled after it and stored one chunk later),
// SHIFT and QMODE (staging for the backward passes, see ChunkStage), COL (the column-decay pass of
// the backward: out_i = q_scale A_i (.) [S x_i + sum_{j<=i} (x_i . y_j) Z~_j], scores from the plain
// x and y, x straight from global memory, fp32 output).  A chunk whose decay leaves the range of
// the factorisation is seen by the loader waves one chunk ahead; the barrier carries the flag and
// the workgroup redoes its sequence through fallback_fn (waves 0-3; the others leave).
#pragma once

#include "lasad_forward_gated_common.h"
#include "lasad_scan.h"

namespace lasad {
namespace gated {

constexpr int kWsThreads = 768;
constexpr int kSetHalfs = 2 * C * RS + 2 * C * KS + C * TS + 2 * D * RS + C * RS;   // one set of tiles

// a: the call's (or the pass's) arguments; bh: the sequence; smem: 2 * kSetHalfs bf16 elements;
// sTot: A_end per key channel by chunk parity; sTrip: range flag of each loader wave by barrier
// parity; sSS (NORM only): sums of squares [chunk parity][channel half][token].
template <int OUT_BF16, int OWNKEY, int FUSED, int NORM, int SHIFT, int QMODE, int COL, int XLO = 0, int YLO = 0, class Fallback = void>
__device__ __forceinline__ void gated_ws_body(const ForwardArgs &a, int bh, uint16_t *smem, float (*sTot)[D],
                                              int (*sTrip)[4], float *sSS, Fallback fallback_fn)
{
    static_assert(!COL || (QMODE == 1 && !OUT_BF16 && !NORM), "column passes: query of ones, fp32 output, no norm");
    static_assert(COL || !XLO, "a two-part x: column passes only");
    static_assert(TS >= RS, "the low-order Y tile sits in the output tile's place");
    // the bf16 output tile goes through LDS for 16-byte stores unless its place holds the low-order Y tile (a row pass
    // with a two-part value operand: then a lane stores its 8-byte pieces itself)
    constexpr bool TILE_OUT = OUT_BF16 && !YLO;
    auto sQh = [&](int p) { return smem + p * kSetHalfs; };
    auto sQl = [&](int p) { return smem + p * kSetHalfs + C * RS; };
    auto sKh = [&](int p) { return smem + p * kSetHalfs + 2 * C * RS; };
    auto sKl = [&](int p) { return smem + p * kSetHalfs + 2 * C * RS + C * KS; };
    auto sV = [&](int p) { return smem + p * kSetHalfs + 2 * C * RS + 2 * C * KS; };
    auto sSh = [&](int p) { return smem + p * kSetHalfs + 2 * C * RS + 2 * C * KS + C * TS; };
    auto sSl = [&](int p) { return smem + p * kSetHalfs + 2 * C * RS + 2 * C * KS + C * TS + D * RS; };
    auto sO = [&](int p) { return smem + p * kSetHalfs + 2 * C * RS + 2 * C * KS + C * TS + 2 * D * RS; };
    auto sVl = sO;     // YLO: low-order part of the Y tile, row stride RS (such a pass stores its output from registers)

    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int group = wave >> 2;                 // 0 output, 1 state, 2 loader
    const int w4 = wave & 3;
    const int wa = w4 >> 1, wc = w4 & 1;         // (query half base | key-channel half), value-channel half
    const int l32 = lane & 31, g = lane >> 5;
    const int st = tid & 255;                    // thread index inside its group

    const int n = a.n_tokens;
    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    const uint16_t *gq = (const uint16_t *)a.q + in_base;
    const uint16_t *gl = (const uint16_t *)a.lam + in_base;
    const uint16_t *gk = OWNKEY ? (const uint16_t *)a.k + in_base : nullptr;
    const uint16_t *gv = (const uint16_t *)a.v + in_base;
    const uint16_t *gql = XLO ? (const uint16_t *)a.q_lo + in_base : nullptr;
    const uint16_t *gvl = YLO ? (const uint16_t *)a.v_lo + in_base : nullptr;
    const int64_t o_base = (int64_t)b * a.out.stride_b + (int64_t)h * a.out.stride_h;
    const int n_chunks = (n + C - 1) / C;

    SplitConst sc;
    sc.init();

    // Every wave meets the same 1 + n_chunks barriers; each carries the loader waves' range flag: a
    // loader wave leaves "any lane tripped" in LDS before the barrier (one store per wave -- an
    // atomic OR by every thread of the workgroup on one LDS word serialises and was measured at
    // 2 us per chunk), everybody reads the four flags after it.  Barrier number k uses flag set k & 1;
    // the set is rewritten two barriers later.  On a set flag the workgroup redoes its whole
    // sequence token by token.
    int n_bar = 0;
    auto barrier_flag = [&](bool mine) {
        const int par = n_bar & 1;
        ++n_bar;
        if (group == 2) {
            const bool any = __any(mine);
            if (lane == 0) sTrip[par][w4] = any ? 1 : 0;
        }
        __syncthreads();
        const int4 f = *(const int4 *)sTrip[par];
        return (f.x | f.y | f.z | f.w) != 0;
    };
    auto fallback = [&]() {            // the token-serial redo of the sequence, by the first waves
        if (tid < scan::kThreads) fallback_fn((float *)smem);
    };

    if (group == 2) {
        // ===================================== loader waves =====================================
        const int pcol = 16 * w4 + 8 * g;
        ChunkStage<OWNKEY, FUSED, SHIFT, QMODE, 0> stg;        // (the V tile is the state waves' job)
        stg.trip = false;
        auto store_tile = [&](int chunk) {                // bf16 output tile of a finished chunk, 16-byte rows
            const uint16_t *bO = sO(chunk & 1);
            const int t0 = chunk * C, nt = min(C, n - t0);
            uint16_t *go = (uint16_t *)a.o + o_base;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = (st >> 3) + 32 * it;
                if (row < nt)
                    *(uint4 *)(go + (int64_t)(t0 + row) * a.out.stride_n + (st & 7) * 8) =
                        *(const uint4 *)&bO[row * RS + (st & 7) * 8];
            }
        };
        stg.fetch(gq, gl, gk, gv, 0, n, a.in.stride_n, l32, pcol);
        stg.prepare(a, 0, n, lane, pcol, sTot[0], sc);
        stg.write(sQh(0), sQl(0), sKh(0), sKl(0), sV(0), l32, pcol);
        if (n_chunks > 1) stg.fetch(gq, gl, gk, gv, 1, n, a.in.stride_n, l32, pcol);
        if (barrier_flag(stg.trip)) return;           // (output waves run the fallback)
        for (int chunk = 0; chunk < n_chunks; ++chunk) {
            if (chunk + 1 < n_chunks) {                   // tiles of the next chunk into the other set
                const int p = (chunk + 1) & 1;
                stg.prepare_begin(a, chunk + 1, n, lane);
                // the fetched registers are free again: the loads of chunk + 2 fly during the rest of this chunk
                if (chunk + 2 < n_chunks) stg.fetch(gq, gl, gk, gv, chunk + 2, n, a.in.stride_n, l32, pcol);
                stg.prepare_end(a, lane, pcol, sTot[p], sc);
                stg.write(sQh(p), sQl(p), sKh(p), sKl(p), sV(p), l32, pcol);
            }
            // the output tile last: the wait for the next loads must not include these stores
            if (TILE_OUT && chunk > NORM) store_tile(chunk - 1 - NORM);
            if (barrier_flag(stg.trip)) return;
        }
        if (TILE_OUT) {
            if (NORM) {
                if (n_chunks > 1) store_tile(n_chunks - 2);
                __syncthreads();                          // the output waves have written the last normalised tile
            }
            store_tile(n_chunks - 1);
        }
        return;
    }

    if (group == 1) {
        // ===================================== state waves =====================================
        f32x16 accS;                   // S[dk = wa*32 + 8*(r/4) + 4*g + r%4][dv = wc*32 + l32]
        if (a.state_in) {
            const float *s0 = a.state_in + (int64_t)bh * D * D;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                accS[r] = s0[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32];
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) accS[r] = 0.f;
        }
        auto publish_state = [&](int p) {
            uint16_t *sh = sSh(p), *sl = sSl(p);
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                uint2 hi, lo;
                split2(accS[4 * qd + 0], accS[4 * qd + 1], hi.x, lo.x, sc);
                split2(accS[4 * qd + 2], accS[4 * qd + 3], hi.y, lo.y, sc);
                const int off = (wc * 32 + l32) * RS + wa * 32 + 8 * qd + 4 * g;
                *(uint2 *)&sh[off] = hi;
                *(uint2 *)&sl[off] = lo;
            }
        };
        // The state waves also stage V (a plain copy; they have the time): thread st takes the
        // 16-byte pieces (st & 7) of rows st / 8 and st / 8 + 32, loaded one chunk ahead with
        // clamped addresses, rows past the end zeroed.
        uint4 rvs[2], rvl[2];
        auto load_v = [&](int chunk) {
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int tok = min(chunk * C + (st >> 3) + 32 * it, n - 1);
                rvs[it] = *(const uint4 *)(gv + (int64_t)tok * a.in.stride_n + (st & 7) * 8);
                if (YLO) rvl[it] = *(const uint4 *)(gvl + (int64_t)tok * a.in.stride_n + (st & 7) * 8);
            }
        };
        auto write_v = [&](int chunk) {
            uint16_t *bV = sV(chunk & 1), *bVl = sVl(chunk & 1);
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = (st >> 3) + 32 * it;
                *(uint4 *)&bV[row * TS + (st & 7) * 8] = keep_or(chunk * C + row < n, rvs[it], 0u);
                if (YLO) *(uint4 *)&bVl[row * RS + (st & 7) * 8] = keep_or(chunk * C + row < n, rvl[it], 0u);
            }
        };
        load_v(0);
        publish_state(0);
        write_v(0);
        if (n_chunks > 1) load_v(1);
        if (barrier_flag(false)) return;
        for (int chunk = 0; chunk < n_chunks; ++chunk) {
            const int p = chunk & 1;
            const uint16_t *bKh = sKh(p), *bKl = sKl(p), *bV = sV(p), *bVl = sVl(p);
            // ---- S[dk][dv] += sum_j K~[j][dk] V[j][dv], then row dk times A_end[dk] ----
            const int trow = (lane & 15) >> 2;
            const int vcol = wc * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
            const int kcol = wa * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int r0 = 16 * s + 4 * g + trow, r1 = r0 + 8;
                Frag fv, fk;
                fv.h[0] = tr_read(&bV[r0 * TS + vcol]);
                fv.h[1] = tr_read(&bV[r1 * TS + vcol]);
                fk.h[0] = tr_read(&bKh[r0 * KS + kcol]);
                fk.h[1] = tr_read(&bKh[r1 * KS + kcol]);
                accS = mfma(fk, fv, accS);
                if (YLO) {                                   // K~ hi times the low-order part of V
                    Frag fvl;
                    fvl.h[0] = tr_read(&bVl[r0 * RS + vcol]);
                    fvl.h[1] = tr_read(&bVl[r1 * RS + vcol]);
                    accS = mfma(fk, fvl, accS);
                }
                fk.h[0] = tr_read(&bKl[r0 * KS + kcol]);
                fk.h[1] = tr_read(&bKl[r1 * KS + kcol]);
                accS = mfma(fk, fv, accS);
            }
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const float4 t4 = *(const float4 *)&sTot[p][wa * 32 + 8 * qd + 4 * g];
                accS[4 * qd + 0] *= t4.x; accS[4 * qd + 1] *= t4.y;
                accS[4 * qd + 2] *= t4.z; accS[4 * qd + 3] *= t4.w;
            }
            if (chunk + 1 < n_chunks) {
                publish_state(p ^ 1);                         // the state chunk + 1 starts from
                write_v(chunk + 1);
                if (chunk + 2 < n_chunks) load_v(chunk + 2);
            }
            if (barrier_flag(false)) return;
        }
        if (a.state_out) {
            float *s1 = a.state_out + (int64_t)bh * D * D;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                s1[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32] = accS[r];
        }
        return;
    }

    // ========================================= output waves =========================================
    const int cq = l32 - 4 * g;        // key 8*qd + 4*g + e of a diagonal block is at or before query l32 iff 8*qd + e <= cq
    // the output tile of a chunk: a lane owns four consecutive value channels of its query per quad
    auto put_tile = [&](const f32x16 &acc, int chunk) {
        const int i_row = (wa ^ (chunk & 1)) * 32 + l32;
        if (OUT_BF16 && !TILE_OUT) {                      // bf16 straight from the registers, 8-byte pieces
            if (chunk * C + i_row < n) {
                uint16_t *go = (uint16_t *)a.o + o_base + (int64_t)(chunk * C + i_row) * a.out.stride_n + wc * 32 + 4 * g;
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    uint2 w2;
                    w2.x = pack2(acc[4 * qd + 0], acc[4 * qd + 1]);
                    w2.y = pack2(acc[4 * qd + 2], acc[4 * qd + 3]);
                    *(uint2 *)(go + 8 * qd) = w2;
                }
            }
        } else if (OUT_BF16) {                            // via LDS; the loader waves store it during a later chunk
            uint16_t *bO = sO(chunk & 1);
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                uint2 w2;
                w2.x = pack2(acc[4 * qd + 0], acc[4 * qd + 1]);
                w2.y = pack2(acc[4 * qd + 2], acc[4 * qd + 3]);
                *(uint2 *)&bO[i_row * RS + wc * 32 + 8 * qd + 4 * g] = w2;
            }
        } else if (chunk * C + i_row < n) {
            float *go = (float *)a.o + o_base + (int64_t)(chunk * C + i_row) * a.out.stride_n + wc * 32 + 4 * g;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                *(float4 *)(go + 8 * qd) = make_float4(acc[4 * qd + 0], acc[4 * qd + 1], acc[4 * qd + 2], acc[4 * qd + 3]);
        }
    };
    f32x16 accP;                       // NORM: the fp32 tile of the chunk before, not yet normalised
    auto finish_tile = [&](int chunk) {                   // after that chunk's barrier: both sums of squares are there
        const int p = chunk & 1, i_row = (wa ^ p) * 32 + l32;
        const float rstd = __builtin_amdgcn_rsqf((sSS[(p * 2) * C + i_row] + sSS[(p * 2 + 1) * C + i_row]) * (1.0f / D) + a.norm_eps);
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            float4 w4 = make_float4(1.f, 1.f, 1.f, 1.f);
            if (a.norm_w) w4 = *(const float4 *)(a.norm_w + h * D + wc * 32 + 8 * qd + 4 * g);
            accP[4 * qd + 0] *= rstd * w4.x; accP[4 * qd + 1] *= rstd * w4.y;
            accP[4 * qd + 2] *= rstd * w4.z; accP[4 * qd + 3] *= rstd * w4.w;
        }
        put_tile(accP, chunk);
    };
    // COL: this lane's query x (row of the pass's first operand), straight from memory in operand
    // layout, one chunk ahead (clamped loads; rows past the end are zeroed when taken)
    Frag fxn[4];
    auto prefetch_x = [&](int chunk) {
        const int xtok = min(chunk * C + (wa ^ (chunk & 1)) * 32 + l32, n - 1);
        const uint16_t *p = gq + (int64_t)xtok * a.in.stride_n + 8 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s) fxn[s].u = *(const uint4 *)(p + 16 * s);
    };
    // XLO: the low-order part of x, ONE register set: loaded for the next chunk after this chunk's last use
    Frag fxl[4];
    auto load_xl = [&](int chunk) {
        const int xtok = min(chunk * C + (wa ^ (chunk & 1)) * 32 + l32, n - 1);
        const uint16_t *p = gql + (int64_t)xtok * a.in.stride_n + 8 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s) fxl[s].u = *(const uint4 *)(p + 16 * s);
    };
    if (COL) prefetch_x(0);
    if (XLO) load_xl(0);
    if (barrier_flag(false)) { fallback(); return; }
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int t0 = chunk * C;
        const int nt = min(C, n - t0);
        (void)nt;
        if (NORM && chunk > 0) finish_tile(chunk - 1);
        const int qa = wa ^ (chunk & 1);                  // query half of this wave in this chunk
        const int p = chunk & 1;
        const uint16_t *bQh = sQh(p), *bQl = sQl(p), *bKh = sKh(p), *bKl = sKl(p), *bV = sV(p);
        const uint16_t *bSh = sSh(p), *bSl = sSl(p);
        const int i_row = qa * 32 + l32;                  // this lane's query (column of the transposed tiles)
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const int trow = (lane & 15) >> 2;
        const int tcol = wc * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
        f32x16 accO = zero16;
        if (!COL) {
            Frag fqh[4], fql[4];
    #pragma unroll
            for (int s = 0; s < 4; ++s) {
                fqh[s].u = *(const uint4 *)&bQh[i_row * RS + 16 * s + 8 * g];
                fql[s].u = *(const uint4 *)&bQl[i_row * RS + 16 * s + 8 * g];
            }
            // scores P^T[j][i] = sum_c K~[j][c] Q~[i][c] of key block jb
            auto scores = [&](int jb) {
                f32x16 acc = zero16;
    #pragma unroll
                for (int s = 0; s < 4; ++s) {
                    Frag kh, kl;
                    kh.u = *(const uint4 *)&bKh[(jb * 32 + l32) * KS + 16 * s + 8 * g];
                    kl.u = *(const uint4 *)&bKl[(jb * 32 + l32) * KS + 16 * s + 8 * g];
                    acc = mfma(kh, fqh[s], acc);
                    acc = mfma(kl, fqh[s], acc);
                    acc = mfma(kh, fql[s], acc);
                }
                return acc;
            };
            // O^T += V^T P^T for key block jb: causal mask (diagonal blocks), split, two MFMAs per k-step
            auto intra = [&](f32x16 acc, const f32x16 &sa, int jb, bool diagonal) {
                Frag fv[2];
                const int trow = (lane & 15) >> 2;
                const int tcol = wc * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
    #pragma unroll
                for (int s = 0; s < 2; ++s) {
                    fv[s].h[0] = tr_read(&bV[(32 * jb + 16 * s + 4 * g + trow) * TS + tcol]);
                    fv[s].h[1] = tr_read(&bV[(32 * jb + 16 * s + 8 + 4 * g + trow) * TS + tcol]);
                }
                Frag ph[2], pl[2];
    #pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    float p0 = sa[4 * qd + 0], p1 = sa[4 * qd + 1], p2 = sa[4 * qd + 2], p3 = sa[4 * qd + 3];
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
    #pragma unroll
                for (int s = 0; s < 2; ++s) {
                    acc = mfma(fv[s], ph[s], acc);
                    acc = mfma(fv[s], pl[s], acc);
                    if (YLO) {                                // the low-order part of V times P hi
                        const uint16_t *bVl = sVl(p);
                        Frag fvl;
                        fvl.h[0] = tr_read(&bVl[(32 * jb + 16 * s + 4 * g + trow) * RS + tcol]);
                        fvl.h[1] = tr_read(&bVl[(32 * jb + 16 * s + 8 + 4 * g + trow) * RS + tcol]);
                        acc = mfma(fvl, ph[s], acc);
                    }
                }
                return acc;
            };

            const f32x16 acc0 = scores(0);
            // ---- O^T[n][i] += sum_dk S^T[n][dk] Q~[i][dk] ----
    #pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag sh, sl;
                sh.u = *(const uint4 *)&bSh[(wc * 32 + l32) * RS + 16 * s + 8 * g];
                sl.u = *(const uint4 *)&bSl[(wc * 32 + l32) * RS + 16 * s + 8 * g];
                accO = mfma(sh, fqh[s], accO);
                accO = mfma(sl, fqh[s], accO);
                accO = mfma(sh, fql[s], accO);
            }
            f32x16 acc1 = zero16;
            if (qa == 1) acc1 = scores(1);
            accO = intra(accO, acc0, 0, qa == 0);
            if (qa == 1) accO = intra(accO, acc1, 1, true);
        } else {
            // ---- COL pass: rows of the tile are the key channels c = wc*32 + .., columns the queries ----
            Frag fx[4];
            {
                const bool live = t0 + i_row < n;
#pragma unroll
                for (int s = 0; s < 4; ++s) fx[s].u = keep_or(live, fxn[s].u, 0u);
                if (XLO) {
#pragma unroll
                    for (int s = 0; s < 4; ++s) fxl[s].u = keep_or(live, fxl[s].u, 0u);
                }
            }
            if (chunk + 1 < n_chunks) prefetch_x(chunk + 1);
            const uint16_t *bVl = sVl(p);
            // scores P^T[j][i] = sum_e Y[j][e] X[i][e] of key block jb (plain bf16 operands)
            auto scores = [&](int jb) {
                f32x16 acc = zero16;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    Frag fy;
                    fy.u = *(const uint4 *)&bV[(jb * 32 + l32) * TS + 16 * s + 8 * g];
                    acc = mfma(fy, fx[s], acc);
                    if (XLO) acc = mfma(fy, fxl[s], acc);
                    if (YLO) {
                        fy.u = *(const uint4 *)&bVl[(jb * 32 + l32) * RS + 16 * s + 8 * g];
                        acc = mfma(fy, fx[s], acc);
                    }
                }
                return acc;
            };
            // O^T[c][i] += sum_j Z~[j][c] P^T[j][i] for key block jb: mask, split, three MFMAs per k-step
            auto intra = [&](f32x16 acc, const f32x16 &sa, int jb, bool diagonal) {
                Frag ph[2], pl[2];
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    float p0 = sa[4 * qd + 0], p1 = sa[4 * qd + 1], p2 = sa[4 * qd + 2], p3 = sa[4 * qd + 3];
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
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    Frag zh, zl;
                    zh.h[0] = tr_read(&bKh[(32 * jb + 16 * s + 4 * g + trow) * KS + tcol]);
                    zh.h[1] = tr_read(&bKh[(32 * jb + 16 * s + 8 + 4 * g + trow) * KS + tcol]);
                    zl.h[0] = tr_read(&bKl[(32 * jb + 16 * s + 4 * g + trow) * KS + tcol]);
                    zl.h[1] = tr_read(&bKl[(32 * jb + 16 * s + 8 + 4 * g + trow) * KS + tcol]);
                    acc = mfma(zh, ph[s], acc);
                    acc = mfma(zl, ph[s], acc);
                    acc = mfma(zh, pl[s], acc);
                }
                return acc;
            };
            const f32x16 acc0 = scores(0);
            // ---- O^T[c][i] += sum_e S[c][e] X[i][e]: S rows from the S^T tiles through the transposing read ----
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag sh, sl;
                sh.h[0] = tr_read(&bSh[(16 * s + 8 * g + trow) * RS + tcol]);
                sh.h[1] = tr_read(&bSh[(16 * s + 8 * g + 4 + trow) * RS + tcol]);
                sl.h[0] = tr_read(&bSl[(16 * s + 8 * g + trow) * RS + tcol]);
                sl.h[1] = tr_read(&bSl[(16 * s + 8 * g + 4 + trow) * RS + tcol]);
                accO = mfma(sh, fx[s], accO);
                accO = mfma(sl, fx[s], accO);
                if (XLO) accO = mfma(sh, fxl[s], accO);
            }
            f32x16 acc1 = zero16;
            if (qa == 1) acc1 = scores(1);
            if (XLO && chunk + 1 < n_chunks) load_xl(chunk + 1);      // (its last use in this chunk is behind us)
            accO = intra(accO, acc0, 0, qa == 0);
            if (qa == 1) accO = intra(accO, acc1, 1, true);
            // ---- times q_scale A_i[c] (staged as Q~ of a query of ones, bf16 hi + lo) ----
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const uint2 ah = *(const uint2 *)&bQh[i_row * RS + wc * 32 + 8 * qd + 4 * g];
                const uint2 al = *(const uint2 *)&bQl[i_row * RS + wc * 32 + 8 * qd + 4 * g];
                accO[4 * qd + 0] *= __uint_as_float(ah.x << 16) + __uint_as_float(al.x << 16);
                accO[4 * qd + 1] *= __uint_as_float(ah.x & 0xffff0000u) + __uint_as_float(al.x & 0xffff0000u);
                accO[4 * qd + 2] *= __uint_as_float(ah.y << 16) + __uint_as_float(al.y << 16);
                accO[4 * qd + 3] *= __uint_as_float(ah.y & 0xffff0000u) + __uint_as_float(al.y & 0xffff0000u);
            }
        }

        if (NORM) {                                       // sums of squares now, the tile after the barrier
            float ss = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) ss = fmaf(accO[r], accO[r], ss);
            ss += __shfl_xor(ss, 32);
            if (g == 0) sSS[(p * 2 + wc) * C + i_row] = ss;
            accP = accO;
        } else {
            put_tile(accO, chunk);
        }
        if (barrier_flag(false)) { fallback(); return; }
    }
    if (NORM) {
        finish_tile(n_chunks - 1);
        if (TILE_OUT) __syncthreads();                    // (the loader waves store the tile after it)
    }
}

}  // namespace gated
}  // namespace lasad
