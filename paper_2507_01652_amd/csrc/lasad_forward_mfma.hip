// Chunked forward on the bf16 matrix cores (gfx950 MFMA), head dim 64, chunk 64.
//
// Unrolling Section 3.4's recurrence over a chunk of C tokens that starts after
// position c0 gives, with e_i = E(i) - E(c0) (number of decaying steps between the
// chunk start and token i; E is the integer prefix of the boundary rule) and the
// separable factors r_i = gamma^{e_i}, c_j = gamma^{-e_j}:
//
//   o_i   = r_i   ( q_i^T S_prev + sum_{j<=i} c_j (q_i . k_j) v_j )
//   S_new = r_end ( S_prev       + sum_j      c_j  k_j v_j^T )
//
// i.e. per chunk four 64x64x64 contractions: K Q^T, (masked P) V, Q S and K^T V.
//
// One workgroup of four wavefronts walks one (batch, head) sequence.  Wave (a, c)
// owns key-channel half a and value-channel half c of the state and, in
// alternating chunks, query half a or 1-a (the lower query half has half the
// causal work) -- all 32 x 32 tiles of v_mfma_f32_32x32x16_bf16.  Layout choices,
// all made so that nothing is shuffled between the MFMA accumulator layout and
// the MFMA operand layout:
//  * the score tile is computed transposed, P^T = K Q^T: a lane then holds, for
//    its query column i, key rows j in groups of four consecutive -- which is
//    exactly an operand fragment of the next MFMA once the reduction index j is
//    enumerated in that same (permuted) order on the V side;
//  * the output tile is computed transposed, O^T = V^T P^T + S^T Q^T, so the
//    per-query factor r_i is one scalar per lane and a lane owns four consecutive
//    value channels of its query (8-byte LDS writes on the way out);
//  * K, V and the decayed keys c_j k_j are kept row-major (token, channel) in
//    LDS, as they arrive from HBM; the token-major operand fragments (reduction
//    over tokens) come from the LDS transpose read ds_read_b64_tr_b16;
//  * Q fragments are loaded from global memory straight into operand layout;
//  * the fp32 state stays in MFMA accumulators for the whole sequence; a bf16
//    copy S^T goes through LDS once per chunk for the Q S product.
//
// Precision.  The matrix cores take bf16 operands, but rounding the computed
// operands (masked scores P, state S, decayed keys c (.) K) to one bf16 each
// costs about 2^-9 of the local output magnitude per site, which on heavy-tailed
// outputs exceeds a 2e-2-of-RMS budget at the largest element.  Each computed
// operand is therefore split into a bf16 pair hi + lo (lo = the rounding
// residual) and multiplied with two MFMAs; q, k, v themselves are exact bf16.
// The kernel is bound by instruction issue and HBM, not by the matrix cores, so
// all elementwise work is done once per element (the decayed keys at staging
// time by the thread that loaded them) and the extra MFMAs are cheap.
//
// Few, long sequences.  When there are fewer sequences than the chip has room
// for workgroups, each sequence is cut into segments of whole chunks and the work
// is done in two launches: a state pass in which every segment but the last
// builds, from a zero state, its own contribution U_g to the state (K, V only, no
// scores, no output), written to a workspace; then the full pass, in which the
// workgroup of segment g folds U_0..U_{g-1} (and the caller's initial state) into
// its incoming state, S <- gamma^{E(end_g') - E(begin_g')} S + U_g', and walks its
// own chunks.  The serial chain per sequence shrinks from all chunks to one
// segment's chunks plus a few 16 KB folds.
//
// Decay.  Powers of gamma are only formed for in-chunk exponents (0..64), from
// each token's (row, column) position.  The separable form needs c_j <= 2^64,
// i.e. gamma > 0.5; a head with a smaller gamma is walked with the fp32
// recurrence instead (lasad_recurrence.h), where its decay is applied step by
// step.
#include <stdlib.h>

#include "lasad_forward_mfma_common.h"
#include "lasad_recurrence.h"

namespace lasad {

namespace {


using namespace fwd;

// ------------------------------------------------------------------------------------------
// State pass: segment g < G-1 of every sequence builds U_g = sum_j gamma^{E(end) - E(j)} k_j v_j^T
// from a zero state and writes it (fp32 [dk][dv]) to seg_states[(bh * (G-1) + g)].
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads, 2)
segment_state_kernel(ForwardArgs a)
{
    __shared__ __attribute__((aligned(16))) uint16_t sV[C * VS], sKh[C * VS], sKl[C * VS];
    __shared__ __attribute__((aligned(16))) float tabC[C];

    const int G1 = a.n_segments - 1;
    const int bh = blockIdx.x / G1, seg = blockIdx.x - bh * G1;
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const float lg = log2f(a.gamma[h]);
    if (!(lg * (float)C > -64.0f)) return;        // this head is walked by the fp32 recurrence

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wa = wave >> 1, wc = wave & 1;
    const int l32 = lane & 31, g = lane >> 5;

    const int seg_t0 = seg * a.seg_chunks * C;                 // first token of the segment
    const int n = min(a.seg_chunks * C, a.n_tokens - seg_t0);   // its length (a full segment here)
    const int64_t base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h + (int64_t)seg_t0 * a.in.stride_n;
    const uint16_t *gk = (const uint16_t *)a.k + base;
    const uint16_t *gv = (const uint16_t *)a.v + base;

    ChunkPos pos;
    pos.init(a.start_pos + seg_t0, a.grid_w, a.mode);
    SplitConst sc;
    sc.init();

    f32x16 accS;
#pragma unroll
    for (int r = 0; r < 16; ++r) accS[r] = 0.f;

    uint4 rk[2], rv[2];
    load_kv(rk, rv, gk, gv, 0, n, a.in.stride_n, tid);
    const int n_chunks = (n + C - 1) / C;
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int nt = min(C, n - chunk * C);
        StagedKeys st;
        prepare_keys(st, rk, rv, tid, nt, pos, lg, sc);
        write_tiles<false>(nullptr, sV, sKh, sKl, tabC, rk, rv, st, tid);
        pos.advance();
        __syncthreads();
        if (chunk + 1 < n_chunks) load_kv(rk, rv, gk, gv, (chunk + 1) * C, n, a.in.stride_n, tid);
        Frag fv[4];
        load_v_frags(fv, sV, wc, lane);
        state_update(accS, sKh, sKl, fv, wa, lane);
        const float r_end = __builtin_amdgcn_rcpf(tabC[nt - 1]);
#pragma unroll
        for (int r = 0; r < 16; ++r) accS[r] *= r_end;
        __syncthreads();                                   // tiles free for the next chunk
    }
    float *u = a.seg_states + ((int64_t)bh * G1 + seg) * D * D;
#pragma unroll
    for (int r = 0; r < 16; ++r)
        u[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32] = accS[r];
}

// ------------------------------------------------------------------------------------------
// Full pass: workgroup (bh, seg) walks the chunks of its segment.
//
// Schedule of one chunk (two barriers):
//   write the staged tiles (prepared during the previous chunk) to LDS          | barrier A
//   issue the global loads of the next chunk (K, V pieces, Q fragments)
//   scores K Q^T, Q S, state update K~^T V        (MFMA chains, operands from LDS)
//   decay + causal mask, hi/lo split, P V          (VALU, then MFMA)
//   scale the state and the output tile (bf16 tile into LDS; fp32 rows straight to memory)
//   scale/split the next chunk's keys in registers (its loads have landed by now)  | barrier B
//   16-byte stores of the bf16 tile, bf16 hi/lo copy of the new S^T for the next chunk
// ------------------------------------------------------------------------------------------
template <int OUT_BF16>
__global__ void __launch_bounds__(kThreads, 2)
forward_mfma_kernel(ForwardArgs a)
{
    // LDS: K tile (16-byte reads), V and decayed-K hi/lo tiles (transpose reads), S^T hi/lo, the
    // bf16 output tile, the table of c_j.  The fp32-recurrence fallback reuses the block.
    constexpr int kLdsHalfs = C * RS + 3 * C * VS + 2 * D * RS + C * RS;
    __shared__ __attribute__((aligned(16))) uint16_t smem[kLdsHalfs];
    __shared__ __attribute__((aligned(16))) float tabC[C];
    static_assert(kLdsHalfs * 2 >= recurrence_lds_floats<D>() * 4, "fallback needs the LDS block");
    uint16_t *sK = smem;
    uint16_t *sV = sK + C * RS;
    uint16_t *sKh = sV + C * VS;
    uint16_t *sKl = sKh + C * VS;
    uint16_t *sS = sKl + C * VS;       // S^T [hi, lo][dv][dk]
    uint16_t *sO = sS + 2 * D * RS;   // bf16 output tile [token][dv]

    const int G = a.n_segments;
    const int bh = blockIdx.x / G, seg = blockIdx.x - bh * G;
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const float gamma = a.gamma[h];
    const float lg = log2f(gamma);
    if (!(lg * (float)C > -64.0f)) {   // gamma <= 0.5 (or 0): separable factors could overflow
        if (seg == 0) recurrence_sequence<D, 1, OUT_BF16>(a, bh, (float *)smem);   // whole sequence
        return;
    }

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wa = wave >> 1, wc = wave & 1;     // key-channel half, value-channel half
    const int l32 = lane & 31, g = lane >> 5;    // column inside the 32-wide tile, k-group

    const int seg_t0 = seg * a.seg_chunks * C;                 // first token of this segment
    const int n = min(a.seg_chunks * C, a.n_tokens - seg_t0);   // tokens in this segment
    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h + (int64_t)seg_t0 * a.in.stride_n;
    const uint16_t *gq = (const uint16_t *)a.q + in_base;
    const uint16_t *gk = (const uint16_t *)a.k + in_base;
    const uint16_t *gv = (const uint16_t *)a.v + in_base;
    const int64_t o_base = (int64_t)b * a.out.stride_b + (int64_t)h * a.out.stride_h + (int64_t)seg_t0 * a.out.stride_n;

    SplitConst sc;
    sc.init();

    // first loads go out before the incoming state is assembled
    uint4 rk[2], rv[2];
    Frag fqn[4];
    auto prefetch = [&](int chunk) {
        load_kv(rk, rv, gk, gv, chunk * C, n, a.in.stride_n, tid);
        const int qtok = min(chunk * C + (wa ^ (chunk & 1)) * 32 + l32, n - 1);
        const uint16_t *p = gq + (int64_t)qtok * a.in.stride_n + 8 * g;
#pragma unroll
        for (int s = 0; s < 4; ++s) fqn[s].u = *(const uint4 *)(p + 16 * s);
    };
    prefetch(0);

    // --- state accumulators: S[dk = wa*32 + 8*(r/4) + 4*g + r%4][dv = wc*32 + l32] ---
    // incoming state = caller's state folded through the segments before this one
    f32x16 accS;
    bool have_state = a.state_in != nullptr;
    if (have_state) {
        const float *s0 = a.state_in + (int64_t)bh * D * D;
        const float s_in = incoming_state_scale(a, gamma);
#pragma unroll
        for (int r = 0; r < 16; ++r)
            accS[r] = s_in * s0[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32];
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) accS[r] = 0.f;
    }
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
        have_state = true;
    }
    // bf16 hi/lo copy of S^T for the Q S product of the next chunk, into buffer `buf`
    auto publish_state = [&](int buf) {
        uint16_t *sh = sS + buf * 2 * D * RS, *sl = sh + D * RS;
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
    publish_state(0);          // also when the state is zero: the Q S product below is unconditional

    ChunkPos pos;
    pos.init(a.start_pos + seg_t0, a.grid_w, a.mode);

    // causal mask of a diagonal 32 x 32 score block in block-local coordinates (loop invariant):
    // causal[4*qd + e] says whether key 8*qd + 4*g + e is at or before query l32
    bool causal[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) causal[r] = 8 * (r / 4) + 4 * g + (r % 4) <= l32;

    const int n_chunks = (n + C - 1) / C;

    // keys and Q fragments of chunk 0
    StagedKeys st;
    Frag fq[4];
    auto take_q = [&](int chunk) {                        // prefetched Q fragments -> fq (tail rows zero)
        const bool live = chunk * C + (wa ^ (chunk & 1)) * 32 + l32 < n;
#pragma unroll
        for (int s = 0; s < 4; ++s) fq[s].u = live ? fqn[s].u : make_uint4(0, 0, 0, 0);
    };
    prepare_keys(st, rk, rv, tid, min(C, n), pos, lg, sc);
    pos.advance();
    take_q(0);

    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int t0 = chunk * C;
        const int nt = min(C, n - t0);
        const int qa = wa ^ (chunk & 1);                  // query half of this wave in this chunk
        const uint16_t *sSh = sS, *sSl = sSh + D * RS;

        write_tiles<true>(sK, sV, sKh, sKl, tabC, rk, rv, st, tid);
        __syncthreads();                                  // (A) tiles, c_j table and S^T visible
        if (chunk + 1 < n_chunks) prefetch(chunk + 1);

        const int i_row = qa * 32 + l32;                  // this lane's query (column of the transposed tiles)

        // ---- scores of key block 0, P^T[j][i] = sum_d K[j][d] Q[i][d] ----
        // accumulators start from a constant-zero C operand of their first MFMA (no register clears)
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 acc0 = zero16, acc1 = zero16, accO = zero16;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            Frag fk;
            fk.u = *(const uint4 *)&sK[l32 * RS + 16 * s + 8 * g];
            acc0 = mfma(fk, fq[s], acc0);
        }
        // ---- O^T[n][i] += sum_dk S^T[n][dk] Q[i][dk]  (independent of the scores) ----
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
        // ---- state update (independent of the scores) ----
        Frag fv[4];
        load_v_frags(fv, sV, wc, lane);
        state_update(accS, sKh, sKl, fv, wa, lane);

        // ---- decay + causal mask on the fp32 scores, split to bf16 hi + lo, then P V ----
        // slot e of quad qd of key block jb is key j = jb*32 + 8*qd + 4*g + e; it lands in the
        // fragment of k-step s = 2*jb + qd/2, half qd%2.
        auto mask_split = [&](const f32x16 &acc, int jb, bool diagonal, Frag *ph, Frag *pl) {
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const float4 c4 = *(const float4 *)&tabC[jb * 32 + 8 * qd + 4 * g];
                float p0 = acc[4 * qd + 0] * c4.x, p1 = acc[4 * qd + 1] * c4.y;
                float p2 = acc[4 * qd + 2] * c4.z, p3 = acc[4 * qd + 3] * c4.w;
                if (diagonal) {
                    p0 = causal[4 * qd + 0] ? p0 : 0.f;
                    p1 = causal[4 * qd + 1] ? p1 : 0.f;
                    p2 = causal[4 * qd + 2] ? p2 : 0.f;
                    p3 = causal[4 * qd + 3] ? p3 : 0.f;
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
            mask_split(acc0, 0, qa == 0, ph, pl);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                accO = mfma(fv[s], ph[s], accO);
                accO = mfma(fv[s], pl[s], accO);
            }
        }
        if (qa == 1) {
            Frag ph[2], pl[2];
            mask_split(acc1, 1, true, ph, pl);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                accO = mfma(fv[2 + s], ph[s], accO);
                accO = mfma(fv[2 + s], pl[s], accO);
            }
        }

        // ---- row factors ----
        {
            const float osc = a.q_scale * __builtin_amdgcn_rcpf(tabC[i_row]);
#pragma unroll
            for (int r = 0; r < 16; ++r) accO[r] *= osc;
            const float r_end = __builtin_amdgcn_rcpf(tabC[nt - 1]);
#pragma unroll
            for (int r = 0; r < 16; ++r) accS[r] *= r_end;
            have_state = true;
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
        // ---- the next chunk's keys (scaled and split) and Q fragments, in registers ----
        if (chunk + 1 < n_chunks) {
            prepare_keys(st, rk, rv, tid, min(C, n - t0 - C), pos, lg, sc);
            pos.advance();
            take_q(chunk + 1);
        }
        __syncthreads();                                  // (B) all reads of the tiles and of S^T finished
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
        if (chunk + 1 < n_chunks) publish_state(0);       // read after the next barrier (A)
    }

    if (a.state_out && seg == G - 1) {
        float *s1 = a.state_out + (int64_t)bh * D * D;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s1[(wa * 32 + 8 * (r / 4) + 4 * g + (r % 4)) * D + wc * 32 + l32] = accS[r];
    }
}

}  // namespace

// Segments per sequence for `n_seq` sequences of `n_chunks` chunks: enough workgroups to fill
// the chip's resident slots (2 per compute unit) once.  Short sequences stay whole (two
// launches cost more than their few chunks), and a workgroup folds at most kMaxSegments - 1
// partial states.
constexpr int kMaxSegments = 8;
constexpr int kMinChunksToSplit = 8;
void plan_segments(int64_t n_seq, int n_chunks, int *n_segments, int *seg_chunks)
{
    const int64_t slots = 512;
    int G = (int)(slots / (n_seq > 0 ? n_seq : 1));
    if (n_chunks < kMinChunksToSplit) G = 1;
    if (G > kMaxSegments) G = kMaxSegments;
    if (G > n_chunks / 2) G = n_chunks / 2;          // at least two chunks per segment
    if (G < 1) G = 1;
    const int L = (n_chunks + G - 1) / G;
    *seg_chunks = L > 0 ? L : 1;
    *n_segments = L > 0 ? (n_chunks + L - 1) / L : 1;
}

size_t forward_mfma_workspace_bytes(int64_t n_seq, int n_tokens)
{
    int G, L;
    plan_segments(n_seq, (n_tokens + C - 1) / C, &G, &L);
    return G > 1 ? (size_t)n_seq * (G - 1) * D * D * sizeof(float) : 0;
}

hipError_t launch_forward_mfma(const ForwardArgs &a_in, hipStream_t s)
{
    if (a_in.d != D || a_in.io_dtype != LASAD_BF16 || a_in.n_tokens < 1) return hipErrorInvalidValue;
    ForwardArgs a = a_in;
    const int64_t n_seq = (int64_t)a.B * a.Hh;
    if (a.seg_states) plan_segments(n_seq, (a.n_tokens + C - 1) / C, &a.n_segments, &a.seg_chunks);
    else { a.n_segments = 1; a.seg_chunks = (a.n_tokens + C - 1) / C; }
    if (n_seq * a.n_segments > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 block(kThreads);
    if (a.n_segments > 1) {
        hipLaunchKernelGGL(segment_state_kernel, dim3((unsigned)(n_seq * (a.n_segments - 1))), block, 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // The full pass: the twelve-wave kernel while every workgroup gets a compute unit of its own,
    // else the eight-wave one (LASAD_WS = 12 / 8 / 0 forces one of them or the four-wave kernel).
    static const int ws = [] { const char *e = getenv("LASAD_WS"); return e ? atoi(e) : -1; }();
    if (ws == 12 || (ws < 0 && n_seq * a.n_segments <= 256)) return launch_forward_mfma_ws12(a, s);
    if (ws != 0) return launch_forward_mfma_ws(a, s);
    const dim3 grid((unsigned)(n_seq * a.n_segments));
    if (a.out_dtype == LASAD_BF16) hipLaunchKernelGGL(forward_mfma_kernel<1>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(forward_mfma_kernel<0>, grid, block, 0, s, a);
    return hipGetLastError();
}


}  // namespace lasad
