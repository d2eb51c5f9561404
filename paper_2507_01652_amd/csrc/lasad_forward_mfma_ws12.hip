// Twelve-wave variant of the chunked scalar-decay forward for the case that a sequence has a
// compute unit to itself (at most 256 sequences or segments): three groups of four wavefronts,
// every LDS buffer doubled, ONE barrier per chunk.
//
//   output waves (0-3):  scores, decay + mask + split, P V, Q S, output tile        (chunk c)
//   state waves  (4-7):  state update K~^T V, scaling, bf16 hi/lo copy of S^T       (chunk c -> c+1)
//   loader waves (8-11): global loads of K and V, decayed keys, tile writes         (chunk c+1),
//                        16-byte stores of the finished output tile                (chunk c-1)
//
// During chunk c the loader waves fill the other set of tiles for chunk c+1 and the state waves
// publish the state that chunk c+1 starts from into the other S^T buffer, so nothing is left to
// do between the end of one chunk's reads and the start of the next chunk's: the workgroup meets
// one barrier per chunk and the chunk time is that of the slowest group (measured with cycle
// stamps on the eight-wave kernel: about a third of its chunk time was the serial stretch between
// its two barriers).  LDS: 2 x 67.6 KB.  Algorithm, layouts and precision: lasad_forward_mfma.hip.
//
// With at most 128 workgroups a sequence is split into two workgroups by value-channel half
// (SPLIT = 2), and the output work of a half is spread over FOUR waves: for each query half one
// wave takes the diagonal score block and the low part of Q S, the other the off-diagonal block
// (upper query half only) and the high part of Q S.  Each leaves an fp32 partial tile in LDS; the
// loader waves add the two, convert and store them during the next chunk.
#include <stdlib.h>

#include "lasad_forward_mfma_common.h"
#include "lasad_recurrence.h"

namespace lasad {

namespace {

using namespace fwd;

constexpr int kWs12Threads = 768;     // SPLIT 1: 4 output + 4 state + 4 loader waves
constexpr int kWs10Threads = 640;     // SPLIT 2: 4 output + 2 state + 4 loader waves
constexpr int PS = RS / 2;            // row stride (floats) of an fp32 partial output tile [token][32 channels]

constexpr int kSetHalfs = C * RS + 3 * C * VS + 2 * D * RS + C * RS;   // one set of tiles

__device__ inline int l32_of(int tid) { return tid & 31; }

// SPLIT = 1: one workgroup (twelve waves) per sequence or segment.  SPLIT = 2: two workgroups, one per
// value-channel half, each with four output waves, two state waves and four loader waves (the loader
// work, K and its decayed copies, is done by both); for so few sequences that compute units stay free.
// DOT: the variant for passes of the backward that also take the decay-gradient sums (MultiPass::x)
template <int OUT_BF16, int SPLIT, int DOT>
__global__ void __launch_bounds__(SPLIT == 1 ? kWs12Threads : kWs10Threads, 1)
forward_mfma_ws12_kernel(ForwardArgs a, MultiPass m)
{
    if (m.n_pass > 1) {                // one of several independent passes of this launch
        const int y = blockIdx.y;
        a.q = m.q[y]; a.k = m.k[y]; a.v = m.v[y]; a.o = m.o[y];
        a.in = m.in[y]; a.out = m.out[y]; a.start_pos = m.start_pos[y];
        a.state_in = m.state_in[y]; a.state_out = m.state_out[y]; a.first_decay_off = m.first_decay_off[y];
    }

    // rows touched once per call: non-temporal.  Split workgroups share Q and K through the L2 and the passes of a
    // backward launch read every tensor two or three times: ordinary loads there.
    constexpr bool NT = !DOT && SPLIT == 1;
    constexpr bool NTO = !DOT;                          // output rows
    constexpr int SROWS = SPLIT == 1 ? D : D / 2;       // rows (value channels) of the S^T tiles
    constexpr int oV = C * RS, oKh = oV + C * VS, oKl = oKh + C * VS, oSh = oKl + C * VS;
    constexpr int oSl = oSh + SROWS * RS, oO = oSl + SROWS * RS;
    // output area of a set: a bf16 tile (SPLIT 1) or two fp32 partial tiles of 32 channels (SPLIT 2)
    static_assert(oO + (SPLIT == 1 ? C * RS : 2 * C * PS * 2) == kSetHalfs, "LDS set layout");
    __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kSetHalfs];
    __shared__ __attribute__((aligned(16))) float tabC2[2][C];
    static_assert(kSetHalfs * 4 >= recurrence_lds_floats<D>() * 4, "fallback needs the LDS block");
    // buffer set p: K, V, decayed keys hi / lo, S^T hi / lo, output tile
    auto sK = [&](int p) { return smem + p * kSetHalfs; };
    auto sV = [&](int p) { return smem + p * kSetHalfs + oV; };
    auto sKh = [&](int p) { return smem + p * kSetHalfs + oKh; };
    auto sKl = [&](int p) { return smem + p * kSetHalfs + oKl; };
    auto sSh = [&](int p) { return smem + p * kSetHalfs + oSh; };
    auto sSl = [&](int p) { return smem + p * kSetHalfs + oSl; };
    auto sO = [&](int p) { return smem + p * kSetHalfs + oO; };
    auto sPart = [&](int p, int part) { return (float *)(smem + p * kSetHalfs + oO) + part * C * PS; };

    const int G = a.n_segments;
    // SPLIT 2: the two workgroups of a sequence (half = value-channel half) are 8 workgroup ids apart,
    // so they start together on the same XCD (ids go round the 8 XCDs) and what both read, Q and
    // K, comes from memory once
    int blk = blockIdx.x, half = 0;
    if (SPLIT == 2) {
        const int grp = blockIdx.x >> 4, r = blockIdx.x & 15;
        half = r >> 3;
        blk = grp * 8 + (r & 7);
        if (blk >= a.B * a.Hh * G) return;                // (the last group of 16 may be partly empty)
    }
    const int bh = blk / G, seg = blk - bh * G;
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const float lg = log2f(a.gamma[h]);
    const int tid = threadIdx.x;
    if (!(lg * (float)C > -64.0f)) {   // gamma <= 0.5: separable factors could overflow -> fp32 recurrence
        if (tid >= kRecThreads || seg != 0 || half != 0) return;   // (finished waves no longer count at barriers)
        if (DOT) recurrence_with_dot<OUT_BF16>(a, m, blockIdx.y, bh, (float *)smem);
        else recurrence_sequence<D, 1, OUT_BF16>(a, bh, (float *)smem);     // whole sequence
        return;
    }

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    // SPLIT 1: waves 0-3 output, 4-7 state, 8-11 loader; SPLIT 2: waves 0-3 output, 4-5 state, 6-9 loader
    const int group = SPLIT == 1 ? wave >> 2 : (wave < 4 ? 0 : wave < 6 ? 1 : 2);
    const int wa = SPLIT == 1 ? (wave & 3) >> 1 : wave & 1;      // query half base | key-channel half
    const int wc = SPLIT == 1 ? wave & 1 : half;                 // value-channel half
    const int part = wave >> 1;                                  // SPLIT 2 output waves: 0 off-diagonal, 1 diagonal
    const int srow = SPLIT == 1 ? wc * 32 + l32_of(tid) : l32_of(tid);   // this lane's row of the S^T tiles
    (void)part;
    const int l32 = lane & 31, g = lane >> 5;
    const int st = SPLIT == 1 ? tid & 255 : tid - 384;   // thread index inside the loader group

    const int seg_t0 = seg * a.seg_chunks * C;                 // first token of this segment
    const int n = min(a.seg_chunks * C, a.n_tokens - seg_t0);   // tokens in this segment
    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h + (int64_t)seg_t0 * a.in.stride_n;
    const uint16_t *gq = (const uint16_t *)a.q + in_base;
    const uint16_t *gk = (const uint16_t *)a.k + in_base;
    const uint16_t *gv = (const uint16_t *)a.v + in_base;
    const int64_t o_base = (int64_t)b * a.out.stride_b + (int64_t)h * a.out.stride_h + (int64_t)seg_t0 * a.out.stride_n;
    const int n_chunks = (n + C - 1) / C;

    SplitConst sc;
    sc.init();

    auto store_tile = [&](int chunk) {                    // output tile of a finished chunk, 16-byte pieces
        const int t0 = chunk * C, nt = min(C, n - t0);
        if (SPLIT == 1) {
            const uint16_t *bO = sO(chunk & 1);
            uint16_t *go = (uint16_t *)a.o + o_base;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = (st >> 3) + 32 * it;
                if (row < nt)
                    gstore16<NTO>(go + (int64_t)(t0 + row) * a.out.stride_n + (st & 7) * 8,
                                  *(const uint4 *)&bO[row * RS + (st & 7) * 8]);
            }
        } else {                                          // sum of the two fp32 partial tiles of this channel half
            const float *x = sPart(chunk & 1, 0), *y = sPart(chunk & 1, 1);
            const int row = st >> 2, col = (st & 3) * 8;
            if (row < nt) {
                const float4 x0 = *(const float4 *)&x[row * PS + col], x1 = *(const float4 *)&x[row * PS + col + 4];
                const float4 y0 = *(const float4 *)&y[row * PS + col], y1 = *(const float4 *)&y[row * PS + col + 4];
                const int64_t oi = o_base + (int64_t)(t0 + row) * a.out.stride_n + half * 32 + col;
                if (OUT_BF16) {
                    uint4 w;
                    w.x = pack2(x0.x + y0.x, x0.y + y0.y); w.y = pack2(x0.z + y0.z, x0.w + y0.w);
                    w.z = pack2(x1.x + y1.x, x1.y + y1.y); w.w = pack2(x1.z + y1.z, x1.w + y1.w);
                    gstore16<NTO>((uint16_t *)a.o + oi, w);
                } else {
                    gstore16<NTO>((float *)a.o + oi, x0.x + y0.x, x0.y + y0.y, x0.z + y0.z, x0.w + y0.w);
                    gstore16<NTO>((float *)a.o + oi + 4, x1.x + y1.x, x1.y + y1.y, x1.z + y1.z, x1.w + y1.w);
                }
            }
        }
    };
    if (group == 2) {
        // ===================================== loader waves =====================================
        // K and V rows are loaded one chunk before their tiles are written.  (Deeper rings of register sets were
        // measured: with loads that are issued under a condition the compiler's wait counts collapse the depth to one
        // chunk anyway, and with unconditional loads the depth is real and gains nothing.)
        uint4 rk[2], rv[2];
        StagedKeys sk;
        ChunkPos pos;
        pos.init(a.start_pos + seg_t0, a.grid_w, a.mode);
        load_kv<NT>(rk, rv, gk, gv, 0, n, a.in.stride_n, st);
        prepare_keys(sk, rk, rv, st, min(C, n), pos, lg, sc);
        pos.advance();
        write_tiles<true>(sK(0), sV(0), sKh(0), sKl(0), tabC2[0], rk, rv, sk, st);
        if (1 < n_chunks) load_kv<NT>(rk, rv, gk, gv, C, n, a.in.stride_n, st);
        __syncthreads();
        for (int chunk = 0; chunk < n_chunks; ++chunk) {
            if ((OUT_BF16 || SPLIT == 2) && chunk > 0) store_tile(chunk - 1);   // the output waves' finished tile
            if (chunk + 1 < n_chunks) {                   // tiles of the next chunk into the other set
                const int p = (chunk + 1) & 1;
                prepare_keys(sk, rk, rv, st, min(C, n - (chunk + 1) * C), pos, lg, sc);
                pos.advance();
                write_tiles<true>(sK(p), sV(p), sKh(p), sKl(p), tabC2[p], rk, rv, sk, st);
                if (chunk + 2 < n_chunks) load_kv<NT>(rk, rv, gk, gv, (chunk + 2) * C, n, a.in.stride_n, st);
            }
            __syncthreads();
        }
        if (OUT_BF16 || SPLIT == 2) store_tile(n_chunks - 1);
        return;
    }

    if (group == 1) {
        // ===================================== state waves =====================================
        f32x16 accS;                   // S[dk = wa*32 + 8*(r/4) + 4*g + r%4][dv = wc*32 + l32]
        if (a.state_in) {
            const float *s0 = a.state_in + (int64_t)bh * D * D;
            const float s_in = incoming_state_scale(a, a.gamma[h]);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                accS[r] = s_in * s0[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32];
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) accS[r] = 0.f;
        }
        // incoming state = caller's state folded through the segments before this one
        for (int sp = 0; sp < seg; ++sp) {
            const int begin = a.start_pos + sp * a.seg_chunks * C;
            const int de = range_exponent(begin, begin + a.seg_chunks * C, a.grid_w, a.mode);
            const float dec = de == 0 ? 1.0f : __builtin_amdgcn_exp2f((float)de * lg);
            const float *u = a.seg_states + ((int64_t)bh * (G - 1) + sp) * D * D;
            float ur[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) ur[r] = u[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32];
#pragma unroll
            for (int r = 0; r < 16; ++r) accS[r] = fmaf(dec, accS[r], ur[r]);
        }
        auto publish_state = [&](int p) {
            uint16_t *sh = sSh(p), *sl = sSl(p);
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                uint2 hi, lo;
                split2(accS[4 * qd + 0], accS[4 * qd + 1], hi.x, lo.x, sc);
                split2(accS[4 * qd + 2], accS[4 * qd + 3], hi.y, lo.y, sc);
                const int off = srow * RS + wa * 32 + 8 * qd + 4 * g;
                *(uint2 *)&sh[off] = hi;
                *(uint2 *)&sl[off] = lo;
            }
        };
        publish_state(0);
        __syncthreads();
        for (int chunk = 0; chunk < n_chunks; ++chunk) {
            const int p = chunk & 1;
            const int nt = min(C, n - chunk * C);
            Frag fv[4];
            load_v_frags(fv, sV(p), wc, lane);
            state_update(accS, sKh(p), sKl(p), fv, wa, lane);
            const float r_end = __builtin_amdgcn_rcpf(tabC2[p][nt - 1]);
#pragma unroll
            for (int r = 0; r < 16; ++r) accS[r] *= r_end;
            if (chunk + 1 < n_chunks) publish_state(p ^ 1);   // the state chunk + 1 starts from
            __syncthreads();
        }
        if (a.state_out && seg == G - 1) {
            float *s1 = a.state_out + (int64_t)bh * D * D;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                s1[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32] = accS[r];
        }
        return;
    }

    // ========================================= output waves =========================================
    // Q fragments go through one of two register sets, loaded two chunks ahead (chunk c uses set c & 1)
    Frag fqn[2][4], fq[4];
    auto prefetch_q = [&](Frag (&dst)[4], int chunk) {
        const int qtok = min(chunk * C + (wa ^ (chunk & 1)) * 32 + l32, n - 1);
        const uint16_t *p = gq + (int64_t)qtok * a.in.stride_n + 8 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s) dst[s].u = *(const uint4 *)(p + 16 * s);    // (a row in four pieces: they meet in the cache)
    };
    auto take_q = [&](const Frag (&src)[4], int chunk) {  // prefetched Q fragments -> fq (tail rows zero)
        const bool live = chunk * C + (wa ^ (chunk & 1)) * 32 + l32 < n;
#pragma unroll
        for (int s = 0; s < 4; ++s) fq[s].u = live ? src[s].u : make_uint4(0, 0, 0, 0);
    };
    prefetch_q(fqn[0], 0);
    if (n_chunks > 1) prefetch_q(fqn[1], 1);
    GradDot gd;
    if (DOT) gd.init(a, m, blockIdx.y, in_base);

    // causal mask of a diagonal 32 x 32 score block: key 8*qd + 4*g + e is at or before query l32
    const int cq = l32 - 4 * g;

    __syncthreads();
    for (int c0 = 0; c0 < n_chunks; c0 += 2) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {                         // p = chunk & 1: buffer set and Q register set
        const int chunk = c0 + p;
        if (chunk >= n_chunks) break;
        const int t0 = chunk * C;
        const int nt = min(C, n - t0);
        const int qa = wa ^ p;                            // query half of this wave in this chunk
        const uint16_t *bK = sK(p), *bV = sV(p), *bSh = sSh(p), *bSl = sSl(p);
        uint16_t *bO = sO(p);
        const float *bC = tabC2[p];
        take_q(fqn[p], chunk);
        if (chunk + 2 < n_chunks) prefetch_q(fqn[p], chunk + 2);
        const int i_row = qa * 32 + l32;
        if (DOT) gd.fetch(min(t0 + i_row, n - 1), wc * 32 + 4 * g);
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

        // scores of key block jb: P^T[j][i] = sum_d K[j][d] Q[i][d]
        auto scores = [&](int jb) {
            f32x16 acc = zero16;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag fk;
                fk.u = *(const uint4 *)&bK[(jb * 32 + l32) * RS + 16 * s + 8 * g];
                acc = mfma(fk, fq[s], acc);
            }
            return acc;
        };
        // O^T[n][i] += sum_dk S^T[n][dk] Q[i][dk] with one bf16 part of S^T
        auto inter = [&](f32x16 acc, const uint16_t *bS) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag fs;
                fs.u = *(const uint4 *)&bS[srow * RS + 16 * s + 8 * g];
                acc = mfma(fs, fq[s], acc);
            }
            return acc;
        };
        // O^T += V^T P^T for key block jb (V fragments of that block: 2*jb, 2*jb + 1)
        auto intra = [&](f32x16 acc, const f32x16 &sc_acc, int jb, bool diagonal) {
            Frag fv[2];
            {
                const int trow = (lane & 15) >> 2;
                const int tcol = wc * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    fv[s].h[0] = tr_read(&bV[(32 * jb + 16 * s + 4 * g + trow) * VS + tcol]);
                    fv[s].h[1] = tr_read(&bV[(32 * jb + 16 * s + 8 + 4 * g + trow) * VS + tcol]);
                }
            }
            Frag ph[2], pl[2];
            mask_split(sc_acc, bC, jb, diagonal, cq, g, sc, ph, pl);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                acc = mfma(fv[s], ph[s], acc);
                acc = mfma(fv[s], pl[s], acc);
            }
            return acc;
        };

        f32x16 accO = zero16;
        if (SPLIT == 1) {
            const f32x16 acc0 = scores(0);
            accO = inter(accO, bSh);
            accO = inter(accO, bSl);
            f32x16 acc1 = zero16;
            if (qa == 1) acc1 = scores(1);
            accO = intra(accO, acc0, 0, qa == 0);
            if (qa == 1) accO = intra(accO, acc1, 1, true);
        } else if (part == 1) {                           // diagonal block of this query half, low part of Q S
            const f32x16 accd = scores(qa);
            accO = inter(accO, bSl);
            accO = intra(accO, accd, qa, true);
        } else {                                          // off-diagonal block (upper query half), high part of Q S
            f32x16 acc0 = zero16;
            if (qa == 1) acc0 = scores(0);
            accO = inter(accO, bSh);
            if (qa == 1) accO = intra(accO, acc0, 0, false);
        }
        // ---- row factor r_i = 1 / c_i and the output tile ----
        const float osc = a.q_scale * __builtin_amdgcn_rcpf(bC[i_row]);
#pragma unroll
        for (int r = 0; r < 16; ++r) accO[r] *= osc;
        if (DOT) gd.add(accO, t0 + i_row, i_row < nt);
        if (SPLIT == 2) {                                 // fp32 partial tile [token][32 channels]; the loader waves add the two
            float *bP = sPart(p, part);
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                *(float4 *)&bP[i_row * PS + 8 * qd + 4 * g] = make_float4(accO[4 * qd + 0], accO[4 * qd + 1],
                                                                         accO[4 * qd + 2], accO[4 * qd + 3]);
        } else if (OUT_BF16) {                            // via LDS for 16-byte coalesced stores
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
                gstore16<NTO>(go + 8 * qd, accO[4 * qd + 0], accO[4 * qd + 1], accO[4 * qd + 2], accO[4 * qd + 3]);
        }
        __syncthreads();
    }
    }
    // slots: SPLIT 1 waves 0-3 (4-7 zero); SPLIT 2 channel half * 4 + wave
    if (!DOT) return;
    if (SPLIT == 1) gd.finish(m, blockIdx.y, (int64_t)a.B * a.Hh, bh, wave, wave + 4, lane);
    else gd.finish(m, blockIdx.y, (int64_t)a.B * a.Hh, bh, half * 4 + wave, -1, lane);
}

}  // namespace


hipError_t launch_ws12_passes(const ForwardArgs &a, const MultiPass &m, hipStream_t s);

hipError_t launch_forward_mfma_ws12(const ForwardArgs &a, hipStream_t s)
{
    MultiPass one;
    one.n_pass = 1;
    return launch_ws12_passes(a, one, s);
}

hipError_t launch_ws12_passes(const ForwardArgs &a, const MultiPass &m, hipStream_t s)
{
    if (a.d != D || a.io_dtype != LASAD_BF16 || a.n_tokens < 1) return hipErrorInvalidValue;
    const int64_t n_seq = (int64_t)a.B * a.Hh;
    if (n_seq * a.n_segments > 0x7fffffff) return hipErrorInvalidValue;
    const int64_t n_wg = n_seq * a.n_segments * m.n_pass;      // workgroups before any split
    static const int split_env = [] { const char *e = getenv("LASAD_SPLIT"); return e ? atoi(e) : 0; }();
    const bool split = split_env ? split_env == 2 : n_wg * 2 <= 256;   // two workgroups per sequence while compute units stay free
    const bool dot = m.n_pass > 1 && (m.x[0] || m.x[1] || m.x[2]);
    const bool out16 = a.out_dtype == LASAD_BF16;
    const int64_t n_blk = n_seq * a.n_segments;
    const dim3 grid((unsigned)(split ? (n_blk + 7) / 8 * 16 : n_blk), (unsigned)m.n_pass);
    const dim3 block(split ? kWs10Threads : kWs12Threads);
#define LASAD_WS12_LAUNCH(O, S, X) hipLaunchKernelGGL((forward_mfma_ws12_kernel<O, S, X>), grid, block, 0, s, a, m)
    if (split) {
        if (dot) { if (out16) LASAD_WS12_LAUNCH(1, 2, 1); else LASAD_WS12_LAUNCH(0, 2, 1); }
        else { if (out16) LASAD_WS12_LAUNCH(1, 2, 0); else LASAD_WS12_LAUNCH(0, 2, 0); }
    } else {
        if (dot) { if (out16) LASAD_WS12_LAUNCH(1, 1, 1); else LASAD_WS12_LAUNCH(0, 1, 1); }
        else { if (out16) LASAD_WS12_LAUNCH(1, 1, 0); else LASAD_WS12_LAUNCH(0, 1, 0); }
    }
#undef LASAD_WS12_LAUNCH
    return hipGetLastError();
}

}  // namespace lasad
