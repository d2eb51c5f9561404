// Chunked matrix-core passes of the vector-decay backward (bf16 inputs, head dim 64): the
// twelve-wave structure of lasad_forward_gated_ws.hip (output / state / loader waves, doubled LDS
// tiles, one barrier per chunk, the same operand preparation and range rule) for the two kinds of
// pass the gradients need (lasad_backward_gated.hip has the derivation):
//
// ROW pass (dv): the forward itself over the reversed sequence, query := the key of the token
//   (1 - lambda if tied), key := q, value := d_o, decay of step m := lambda of step m - 1.
//
// COL pass (dq; dk over the reversed sequence): with A_i the chunk-local running product of the
//   decay and Z~_j = z_j / A_j (z the key for dq, q for dk),
//       out_i = q_scale A_i (.) [ S x_i + sum_{j<=i} (x_i . y_j) Z~_j ],   S <- diag(A_end) (S + Z~^T Y)
//   (x, y: d_o and v for dq, v and d_o for dk).  The state and its update are those of the forward
//   (the state waves are unchanged); the output waves take the scores from the plain x and y
//   (one MFMA per step, no decay inside), contract them with Z~ (bf16 hi + lo on both sides: three
//   MFMAs) and the state with x over the VALUE index (S^T tiles read through the transposing LDS
//   load), and scale the fp32 tile by q_scale A_i, which the loader waves stage as "Q~ of a query
//   of ones".  x comes straight from global memory in operand layout, one chunk ahead.  Output fp32.
//
// A chunk that leaves the range of the factorisation sends the workgroup to the token-serial walk
// of the same pass (lasad_scan.h with operand roles).
#include "lasad_forward_gated_common.h"
#include "lasad_scan.h"

namespace lasad {

namespace {

using namespace gated;

constexpr int kBwdThreads = 768;
constexpr int kBwdSetHalfs = 2 * C * RS + 2 * C * KS + C * TS + 2 * D * RS + C * RS;   // one set of tiles

// The token-serial walk of a pass, out of line.  It is handed the arguments where the launch put
// them (the kernel-argument segment): references to the kernel's by-value parameter, or copies,
// would make every thread of every launch write them to its stack first.
template <int OUT_BF16, int COL>
__device__ __noinline__ void redo_roles(const ForwardArgs *a, const scan::ScanRoles *r, int bh, float *lds)
{
    if (COL) scan::scan_sequence<1, 0, scan::ROLES_COL, 64>(*a, bh, 0, lds, r);
    else scan::scan_sequence<1, OUT_BF16, scan::ROLES_ROW, 64>(*a, bh, 0, lds, r);
}

// One pass for sequence bh by the calling twelve-wave workgroup.  smem: 2 * kBwdSetHalfs bf16 elements.
template <int OUT_BF16, int OWNKEY, int SHIFT, int QMODE, int COL>
__device__ __forceinline__ void pass_body(const ForwardArgs &a, const ForwardArgs *ka, const scan::ScanRoles *kr, int bh,
                                          uint16_t *smem, float (*sTot)[D], int (*sTrip)[4])
{
    static_assert(!COL || (QMODE == 1 && !OUT_BF16), "column passes: query of ones, fp32 output");
    auto sQh = [&](int p) { return smem + p * kBwdSetHalfs; };
    auto sQl = [&](int p) { return smem + p * kBwdSetHalfs + C * RS; };
    auto sKh = [&](int p) { return smem + p * kBwdSetHalfs + 2 * C * RS; };
    auto sKl = [&](int p) { return smem + p * kBwdSetHalfs + 2 * C * RS + C * KS; };
    auto sV = [&](int p) { return smem + p * kBwdSetHalfs + 2 * C * RS + 2 * C * KS; };
    auto sSh = [&](int p) { return smem + p * kBwdSetHalfs + 2 * C * RS + 2 * C * KS + C * TS; };
    auto sSl = [&](int p) { return smem + p * kBwdSetHalfs + 2 * C * RS + 2 * C * KS + C * TS + D * RS; };
    auto sO = [&](int p) { return smem + p * kBwdSetHalfs + 2 * C * RS + 2 * C * KS + C * TS + 2 * D * RS; };

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
    const int64_t o_base = (int64_t)b * a.out.stride_b + (int64_t)h * a.out.stride_h;
    const int n_chunks = (n + C - 1) / C;

    SplitConst sc;
    sc.init();

    // every wave meets the same 1 + n_chunks barriers; each carries the loader waves' range flag
    // (one LDS word per loader wave and barrier parity)
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
    auto fallback = [&]() {
        if (tid < scan::kThreads) redo_roles<OUT_BF16, COL>(ka, kr, bh, (float *)smem);     // ka, kr: in the kernel-argument segment
    };

    if (group == 2) {
        // ===================================== loader waves =====================================
        const int pcol = 16 * w4 + 8 * g;
        ChunkStage<OWNKEY, 0, SHIFT, QMODE, 0> stg;    // (the V tile is the state waves' job)
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
                if (chunk + 2 < n_chunks) stg.fetch(gq, gl, gk, gv, chunk + 2, n, a.in.stride_n, l32, pcol);
                stg.prepare_end(a, lane, pcol, sTot[p], sc);
                stg.write(sQh(p), sQl(p), sKh(p), sKl(p), sV(p), l32, pcol);
            }
            if (OUT_BF16 && chunk > 0) store_tile(chunk - 1);
            if (barrier_flag(stg.trip)) return;
        }
        if (OUT_BF16) store_tile(n_chunks - 1);
        return;
    }

    if (group == 1) {
        // ===================================== state waves =====================================
        f32x16 accS;                   // S[dk = wa*32 + 8*(r/4) + 4*g + r%4][dv = wc*32 + l32]
#pragma unroll
        for (int r = 0; r < 16; ++r) accS[r] = 0.f;
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
        // the state waves also stage the V tile (a plain copy, one chunk ahead, rows past the end zeroed)
        uint4 rvs[2];
        auto load_v = [&](int chunk) {
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int tok = min(chunk * C + (st >> 3) + 32 * it, n - 1);
                rvs[it] = *(const uint4 *)(gv + (int64_t)tok * a.in.stride_n + (st & 7) * 8);
            }
        };
        auto write_v = [&](int chunk) {
            uint16_t *bVw = sV(chunk & 1);
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = (st >> 3) + 32 * it;
                *(uint4 *)&bVw[row * TS + (st & 7) * 8] = keep_or(chunk * C + row < n, rvs[it], 0u);
            }
        };
        load_v(0);
        publish_state(0);
        write_v(0);
        if (n_chunks > 1) load_v(1);
        if (barrier_flag(false)) return;
        for (int chunk = 0; chunk < n_chunks; ++chunk) {
            const int p = chunk & 1;
            const uint16_t *bKh = sKh(p), *bKl = sKl(p), *bV = sV(p);
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
        return;
    }

    // ========================================= output waves =========================================
    const int cq = l32 - 4 * g;        // key 8*qd + 4*g + e of a diagonal block is at or before query l32 iff 8*qd + e <= cq
    // COL: this lane's query x (row of the pass's first operand), straight from memory in operand
    // layout, one chunk ahead (clamped loads; rows past the end are zeroed when taken)
    Frag fxn[4];
    auto prefetch_x = [&](int chunk) {
        const int xtok = min(chunk * C + (wa ^ (chunk & 1)) * 32 + l32, n - 1);
        const uint16_t *p = gq + (int64_t)xtok * a.in.stride_n + 8 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s) fxn[s].u = *(const uint4 *)(p + 16 * s);
    };
    if (COL) prefetch_x(0);
    if (barrier_flag(false)) { fallback(); return; }
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int t0 = chunk * C;
        const int nt = min(C, n - t0);
        const int qa = wa ^ (chunk & 1);                  // query half of this wave in this chunk
        const int p = chunk & 1;
        const uint16_t *bQh = sQh(p), *bQl = sQl(p), *bKh = sKh(p), *bKl = sKl(p), *bV = sV(p);
        const uint16_t *bSh = sSh(p), *bSl = sSl(p);
        uint16_t *bO = sO(p);
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
            }
            if (chunk + 1 < n_chunks) prefetch_x(chunk + 1);
            // scores P^T[j][i] = sum_e Y[j][e] X[i][e] of key block jb (plain bf16 operands)
            auto scores = [&](int jb) {
                f32x16 acc = zero16;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    Frag fy;
                    fy.u = *(const uint4 *)&bV[(jb * 32 + l32) * TS + 16 * s + 8 * g];
                    acc = mfma(fy, fx[s], acc);
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
            }
            f32x16 acc1 = zero16;
            if (qa == 1) acc1 = scores(1);
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

        // ---- the output tile: a lane owns four consecutive channels of its query per quad ----
        if (OUT_BF16) {                                   // via LDS; the loader waves store it during the next chunk
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                uint2 w2;
                w2.x = pack2(accO[4 * qd + 0], accO[4 * qd + 1]);
                w2.y = pack2(accO[4 * qd + 2], accO[4 * qd + 3]);
                *(uint2 *)&bO[i_row * RS + wc * 32 + 8 * qd + 4 * g] = w2;
            }
        } else if (i_row < nt) {
            float *go = (float *)a.o + o_base + (int64_t)(t0 + i_row) * a.out.stride_n + wc * 32 + 4 * g;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                *(float4 *)(go + 8 * qd) = make_float4(accO[4 * qd + 0], accO[4 * qd + 1],
                                                       accO[4 * qd + 2], accO[4 * qd + 3]);
        }
        if (barrier_flag(false)) { fallback(); return; }
    }
}

struct PassSet {
    ForwardArgs a[3];              // dq, dv, dk: the pass's operands in the forward's fields
    scan::ScanRoles roles[3];      // the same passes for the token-serial walk (range fallback)
};

// The three passes of a call in one launch.  Workgroups come in groups of 8 sequences x 3 passes,
// a sequence's passes 8 workgroup ids apart: they start together on the same XCD (ids go round
// the 8 XCDs) and share what they both read through its L2 (dv and dk walk the same q, d_o and
// lambda rows in the same order).  TIED: the key is 1 - lambda.
template <int OUT_BF16, int TIED>
__global__ void __launch_bounds__(kBwdThreads, 1)
backward_gated_passes_kernel(PassSet ps)
{
    constexpr int kScanFloats = scan::lds_floats<scan::ROLES_ROW>();
    static_assert(2 * kBwdSetHalfs * 2 >= kScanFloats * 4, "the fallback needs the LDS block");
    __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kBwdSetHalfs];
    __shared__ __attribute__((aligned(16))) float sTot[2][D];  // A_end per key channel, by chunk parity
    __shared__ __attribute__((aligned(16))) int sTrip[2][4];   // range flag of each loader wave, by barrier parity
    const int grp = blockIdx.x / 24, r = blockIdx.x - grp * 24;
    const int pass = r >> 3, bh = grp * 8 + (r & 7);
    if (bh >= ps.a[0].B * ps.a[0].Hh) return;                  // (the last group may be partly empty)
    const PassSet *kp = (const PassSet *)__builtin_amdgcn_kernarg_segment_ptr();
    if (pass == 0) pass_body<0, TIED ? 0 : 1, 0, 1, 1>(ps.a[0], &kp->a[0], &kp->roles[0], bh, smem, sTot, sTrip);
    else if (pass == 1) pass_body<OUT_BF16, 1, 1, TIED ? 2 : 0, 0>(ps.a[1], &kp->a[1], &kp->roles[1], bh, smem, sTot, sTrip);
    else pass_body<0, 1, 1, 1, 1>(ps.a[2], &kp->a[2], &kp->roles[2], bh, smem, sTot, sTrip);
}

}  // namespace

// The three passes of the vector-decay backward with the matrix-core kernel, one launch.
// a[0..2], roles[0..2]: dq (column pass, forward order), dv (row pass, reversed; its query tensor
// is lambda itself when tied), dk (column pass, reversed), as lasad_backward_gated.hip sets them up.
hipError_t launch_backward_gated_passes(const ForwardArgs *a, const scan::ScanRoles *roles, bool tied, hipStream_t s)
{
    if (a[0].d != D || a[0].io_dtype != LASAD_BF16 || a[0].n_tokens < 1) return hipErrorInvalidValue;
    const int64_t n_seq = (int64_t)a[0].B * a[0].Hh;
    if ((n_seq + 7) / 8 * 24 > 0x7fffffff) return hipErrorInvalidValue;
    PassSet ps;
    for (int i = 0; i < 3; ++i) { ps.a[i] = a[i]; ps.roles[i] = roles[i]; }
    const dim3 grid((unsigned)((n_seq + 7) / 8 * 24)), block(kBwdThreads);
    const bool out16 = a[1].out_dtype == LASAD_BF16;
    if (tied) {
        if (out16) hipLaunchKernelGGL((backward_gated_passes_kernel<1, 1>), grid, block, 0, s, ps);
        else hipLaunchKernelGGL((backward_gated_passes_kernel<0, 1>), grid, block, 0, s, ps);
    } else {
        if (out16) hipLaunchKernelGGL((backward_gated_passes_kernel<1, 0>), grid, block, 0, s, ps);
        else hipLaunchKernelGGL((backward_gated_passes_kernel<0, 0>), grid, block, 0, s, ps);
    }
    return hipGetLastError();
}

}  // namespace lasad
