// Eight-wave variant of the chunked scalar-decay forward (see lasad_forward_mfma.hip for the
// algorithm, the tile layouts and the hi/lo operand split): the work of one chunk is divided
// between two groups of four wavefronts that run side by side on the same four SIMDs.
//
//   output waves (0-3), wave (query half, value-channel half):
//       scores K Q^T, decay + causal mask + split, P V, Q S, row factors, output tile;
//   state waves (4-7), wave (key-channel half, value-channel half):
//       global loads and staging of K and V, decayed keys (scaled, split), state update
//       K~^T V in accumulators, bf16 hi/lo copy of S^T for the output waves.
//
// A single wavefront issues a vector-ALU instruction only every eight cycles on this chip; with
// one four-wave workgroup per compute unit (few sequences) the chunk time of the four-wave kernel
// is mostly that issue limit.  Two wavefronts per SIMD with independent instruction streams
// overlap their vector, matrix and LDS work, and the serial chain from one chunk to the next
// shrinks to the state waves' part.  With a segment plan the state waves fold the partial states
// of the earlier segments into their incoming state, as in the four-wave kernel.
#include <stdlib.h>

#include "lasad_forward_mfma_common.h"
#include "lasad_recurrence.h"

namespace lasad {

namespace {

using namespace fwd;

constexpr int kWsThreads = 512;


// DOT: the variant for passes of the backward that also take the decay-gradient sums (MultiPass::x)
template <int OUT_BF16, int DOT>
__global__ void __launch_bounds__(kWsThreads, 4)
forward_mfma_ws_kernel(ForwardArgs a, MultiPass m)
{
    // Several independent passes in one launch: workgroups come in groups of 8 sequences x n_pass
    // passes, a sequence's passes 8 workgroup ids apart, so that they run at about the same time on
    // the same XCD (ids go round the 8 XCDs) and share what they both read through its L2.
    int pass = 0, wg = blockIdx.x;
    if (m.n_pass > 1) {
        const int grp = blockIdx.x / (8 * m.n_pass), r = blockIdx.x - grp * (8 * m.n_pass);
        pass = r >> 3;
        wg = grp * 8 + (r & 7);
        if (wg >= a.B * a.Hh) return;  // (n_segments is 1 here; the last group may be partly empty)
        a.q = m.q[pass]; a.k = m.k[pass]; a.v = m.v[pass]; a.o = m.o[pass];
        a.in = m.in[pass]; a.out = m.out[pass]; a.start_pos = m.start_pos[pass];
        a.state_in = m.state_in[pass]; a.state_out = m.state_out[pass]; a.first_decay_off = m.first_decay_off[pass];
    }

    // q, k, v and o rows are touched once by a forward call: non-temporal.  The passes of a backward launch read
    // each tensor two or three times and share it through the L2: ordinary loads there.
    constexpr bool NT = !DOT;
    constexpr int kLdsHalfs = C * RS + 3 * C * VS + 2 * D * RS + C * RS;
    __shared__ __attribute__((aligned(16))) uint16_t smem[kLdsHalfs];
    __shared__ __attribute__((aligned(16))) float tabC[C];
    static_assert(kLdsHalfs * 2 >= recurrence_lds_floats<D>() * 4, "fallback needs the LDS block");
    uint16_t *sK = smem;               // K as loaded [token][channel] (16-byte row reads)
    uint16_t *sV = sK + C * RS;        // V as loaded (transpose reads)
    uint16_t *sKh = sV + C * VS;       // decayed keys, bf16 hi / lo (transpose reads)
    uint16_t *sKl = sKh + C * VS;
    uint16_t *sSh = sKl + C * VS;      // S^T [dv][dk], bf16 hi / lo
    uint16_t *sSl = sSh + D * RS;
    uint16_t *sO = sSl + D * RS;       // bf16 output tile [token][dv]

    const int G = a.n_segments;
    const int bh = wg / G, seg = wg - bh * G;
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const float lg = log2f(a.gamma[h]);
    const int tid = threadIdx.x;
    if (!(lg * (float)C > -64.0f)) {   // gamma <= 0.5: separable factors could overflow -> fp32 recurrence
        if (tid >= kRecThreads || seg != 0) return;       // (finished waves no longer count at barriers)
        if (DOT) recurrence_with_dot<OUT_BF16>(a, m, pass, bh, (float *)smem);
        else recurrence_sequence<D, 1, OUT_BF16>(a, bh, (float *)smem);     // whole sequence
        return;
    }

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const bool state_wave = wave >= 4;
    const int w4 = wave & 3;
    const int wa = w4 >> 1, wc = w4 & 1;         // (query half base | key-channel half), value-channel half
    const int l32 = lane & 31, g = lane >> 5;
    const int st = tid & 255;                    // thread index inside its group

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

    if (state_wave) {
        // ===================================== state waves =====================================
        uint4 rk[2], rv[2];
        load_kv<NT>(rk, rv, gk, gv, 0, n, a.in.stride_n, st);

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
        auto publish_state = [&]() {
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
        publish_state();

        ChunkPos pos;
        pos.init(a.start_pos + seg_t0, a.grid_w, a.mode);
        StagedKeys sk;
        prepare_keys(sk, rk, rv, st, min(C, n), pos, lg, sc);
        pos.advance();

        for (int chunk = 0; chunk < n_chunks; ++chunk) {
            const int t0 = chunk * C;
            const int nt = min(C, n - t0);
            write_tiles<true>(sK, sV, sKh, sKl, tabC, rk, rv, sk, st);
            __syncthreads();                              // (A) tiles, c_j table and S^T visible
            if (chunk + 1 < n_chunks) load_kv<NT>(rk, rv, gk, gv, t0 + C, n, a.in.stride_n, st);
            Frag fv[4];
            load_v_frags(fv, sV, wc, lane);
            state_update(accS, sKh, sKl, fv, wa, lane);
            const float r_end = __builtin_amdgcn_rcpf(tabC[nt - 1]);
#pragma unroll
            for (int r = 0; r < 16; ++r) accS[r] *= r_end;
            if (chunk + 1 < n_chunks) {
                prepare_keys(sk, rk, rv, st, min(C, n - t0 - C), pos, lg, sc);
                pos.advance();
            }
            __syncthreads();                              // (B) all reads of the tiles and of S^T finished
            if (chunk + 1 < n_chunks) publish_state();    // read after the next barrier (A)
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
    Frag fqn[4], fq[4];
    auto prefetch_q = [&](int chunk) {
        const int qtok = min(chunk * C + (wa ^ (chunk & 1)) * 32 + l32, n - 1);
        const uint16_t *p = gq + (int64_t)qtok * a.in.stride_n + 8 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s) fqn[s].u = *(const uint4 *)(p + 16 * s);    // (a row in four pieces: they meet in the cache)
    };
    auto take_q = [&](int chunk) {                        // prefetched Q fragments -> fq (tail rows zero)
        const bool live = chunk * C + (wa ^ (chunk & 1)) * 32 + l32 < n;
#pragma unroll
        for (int s = 0; s < 4; ++s) fq[s].u = live ? fqn[s].u : make_uint4(0, 0, 0, 0);
    };
    prefetch_q(0);
    GradDot gd;
    if (DOT) gd.init(a, m, pass, in_base);

    // causal mask of a diagonal 32 x 32 score block: key 8*qd + 4*g + e is at or before query l32
    const int cq = l32 - 4 * g;

    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int t0 = chunk * C;
        const int nt = min(C, n - t0);
        const int qa = wa ^ (chunk & 1);                  // query half of this wave in this chunk
        take_q(chunk);
        __syncthreads();                                  // (A)
        if (chunk + 1 < n_chunks) prefetch_q(chunk + 1);
        const int i_row = qa * 32 + l32;

        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 acc0 = zero16, acc1 = zero16, accO = zero16;
        // ---- scores of key block 0, P^T[j][i] = sum_d K[j][d] Q[i][d] ----
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            Frag fk;
            fk.u = *(const uint4 *)&sK[l32 * RS + 16 * s + 8 * g];
            acc0 = mfma(fk, fq[s], acc0);
        }
        // ---- O^T[n][i] += sum_dk S^T[n][dk] Q[i][dk] ----
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            Frag fs;
            fs.u = *(const uint4 *)&sSh[(wc * 32 + l32) * RS + 16 * s + 8 * g];
            accO = mfma(fs, fq[s], accO);
            fs.u = *(const uint4 *)&sSl[(wc * 32 + l32) * RS + 16 * s + 8 * g];
            accO = mfma(fs, fq[s], accO);
        }
        // ---- scores of key block 1 (all masked for the lower query half) ----
        if (qa == 1) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag fk;
                fk.u = *(const uint4 *)&sK[(32 + l32) * RS + 16 * s + 8 * g];
                acc1 = mfma(fk, fq[s], acc1);
            }
        }
        if (DOT) gd.fetch(min(t0 + i_row, n - 1), wc * 32 + 4 * g);     // (here the Q fragments' registers are free)
        Frag fv[4];
        load_v_frags(fv, sV, wc, lane);

        {
            Frag ph[2], pl[2];
            mask_split(acc0, tabC, 0, qa == 0, cq, g, sc, ph, pl);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                accO = mfma(fv[s], ph[s], accO);
                accO = mfma(fv[s], pl[s], accO);
            }
        }
        if (qa == 1) {
            Frag ph[2], pl[2];
            mask_split(acc1, tabC, 1, true, cq, g, sc, ph, pl);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                accO = mfma(fv[2 + s], ph[s], accO);
                accO = mfma(fv[2 + s], pl[s], accO);
            }
        }
        // ---- row factor r_i = 1 / c_i and the output tile ----
        const float osc = a.q_scale * __builtin_amdgcn_rcpf(tabC[i_row]);
#pragma unroll
        for (int r = 0; r < 16; ++r) accO[r] *= osc;
        if (DOT) gd.add(accO, t0 + i_row, i_row < nt);
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
                gstore16<NT>(go + 8 * qd, accO[4 * qd + 0], accO[4 * qd + 1], accO[4 * qd + 2], accO[4 * qd + 3]);
        }
        __syncthreads();                                  // (B)
        if (OUT_BF16) {                                   // coalesced 16-byte stores of the bf16 tile
            uint16_t *go = (uint16_t *)a.o + o_base;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = (st >> 3) + 32 * it;
                if (row < nt)
                    gstore16<NT>(go + (int64_t)(t0 + row) * a.out.stride_n + (st & 7) * 8,
                                 *(const uint4 *)&sO[row * RS + (st & 7) * 8]);
            }
        }
    }
    if (DOT) gd.finish(m, pass, (int64_t)a.B * a.Hh, bh, w4, w4 + 4, lane);
}

}  // namespace


static hipError_t launch_ws8(const ForwardArgs &a, const MultiPass &m, hipStream_t s);

hipError_t launch_forward_mfma_ws(const ForwardArgs &a, hipStream_t s)
{
    MultiPass one;
    one.n_pass = 1;
    return launch_ws8(a, one, s);
}

static hipError_t launch_ws8(const ForwardArgs &a, const MultiPass &m, hipStream_t s)
{
    if (a.d != D || a.io_dtype != LASAD_BF16 || a.n_tokens < 1) return hipErrorInvalidValue;
    const int64_t n_seq = (int64_t)a.B * a.Hh;
    if (n_seq * a.n_segments > 0x7fffffff) return hipErrorInvalidValue;
    if (m.n_pass > 1 && a.n_segments != 1) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(m.n_pass > 1 ? (n_seq + 7) / 8 * 8 * m.n_pass : n_seq * a.n_segments)), block(kWsThreads);
    const bool dot = m.n_pass > 1 && (m.x[0] || m.x[1] || m.x[2]);
    const bool out16 = a.out_dtype == LASAD_BF16;
    if (dot && out16) hipLaunchKernelGGL((forward_mfma_ws_kernel<1, 1>), grid, block, 0, s, a, m);
    else if (dot) hipLaunchKernelGGL((forward_mfma_ws_kernel<0, 1>), grid, block, 0, s, a, m);
    else if (out16) hipLaunchKernelGGL((forward_mfma_ws_kernel<1, 0>), grid, block, 0, s, a, m);
    else hipLaunchKernelGGL((forward_mfma_ws_kernel<0, 0>), grid, block, 0, s, a, m);
    return hipGetLastError();
}

hipError_t launch_ws12_passes(const ForwardArgs &a, const MultiPass &m, hipStream_t s);   // lasad_forward_mfma_ws12.hip

// Several whole-sequence passes in one launch: twelve waves per workgroup while all workgroups of
// all passes get a compute unit each, else eight waves (two workgroups per compute unit).
hipError_t launch_forward_mfma_multi(const ForwardArgs &common, const MultiPass &m, hipStream_t s)
{
    if (common.n_segments != 1 || m.n_pass < 1 || m.n_pass > 3) return hipErrorInvalidValue;
    const int64_t n_wg = (int64_t)common.B * common.Hh * m.n_pass;
    static const int ws = [] { const char *e = getenv("LASAD_WS_MULTI"); return e ? atoi(e) : -1; }();
    if (ws == 12 || (ws < 0 && n_wg <= 256)) return launch_ws12_passes(common, m, s);
    return launch_ws8(common, m, s);
}

}  // namespace lasad
