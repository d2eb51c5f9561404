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
// Chunk preparation.  The 16-byte pieces of q, lambda, (k,) v fetched during the previous chunk
// are written raw (bf16) into the LDS tiles; after a barrier the workgroup re-reads them
// column-wise: thread (channel c, quarter u) owns tokens 16u .. 16u+15 of channel c, forms the
// running product of lambda in fp32, exchanges the quarter totals with the three other lanes
// of its channel (same wavefront, no barrier), and overwrites the tiles in place with the bf16
// hi + lo pairs of K~ and Q~.  The tied key k = 1 - lambda uses lambda before the boundary
// override, as Algorithm 1 does.
//
// Precision: Q~, K~, P and S are computed operands and are each split into bf16 hi + lo (three
// MFMAs for a product of two split operands, two when one side is exact); v is exact bf16.
//
// Range.  K~ grows like 1 / A.  A chunk whose total decay of some channel is below 2^-60 (or
// zero) cannot be factored this way; the workgroup then abandons the chunked walk and redoes
// its whole sequence with the token-serial fp32 routine (lasad_scan.h), which applies each
// decay step by step.  Gates from a sigmoid stay many orders of magnitude above that limit.
#include "lasad_mfma_util.h"
#include "lasad_scan.h"

namespace lasad {

namespace {

constexpr int C = 64;      // chunk length (tokens)
constexpr int D = 64;      // head dim
constexpr int kThreads = 256;
constexpr int TS = 80;     // LDS row stride (bf16 elements) of the operand tiles: 160 B
constexpr int RS = 72;     // LDS row stride of the S^T and output tiles: 144 B
constexpr float kMinChunkDecay = 8.6736174e-19f;   // 2^-60

// Element (row, col) of a 64 x 64 operand tile.  Rows are rotated by 16 channels per 16-row
// band so that the column-wise 2-byte accesses of the four token quarters of a wavefront fall
// into different banks; 8- and 4-element runs stay contiguous.
__device__ inline int tix(int row, int col) { return row * TS + ((col + (row & 48)) & 63); }

// x where keep, else every 32-bit word = fill (component-wise, so the values stay in registers)
__device__ inline uint4 keep_or(bool keep, uint4 x, uint32_t fill)
{
    return make_uint4(keep ? x.x : fill, keep ? x.y : fill, keep ? x.z : fill, keep ? x.w : fill);
}

template <int OUT_BF16, int OWNKEY>
__global__ void __launch_bounds__(kThreads, 2)
forward_gated_mfma_kernel(ForwardArgs a)
{
    // tiles: Q~ hi, Q~ lo, K~ hi, K~ lo, V (stride TS); S^T hi, lo and the bf16 output tile (stride RS)
    constexpr int kTileHalfs = 5 * C * TS + 3 * D * RS;
    constexpr int kScanFloats = scan::lds_floats<OWNKEY ? scan::OWNKEY : scan::TIED>();
    constexpr int kLdsBytes = kTileHalfs * 2 > kScanFloats * 4 ? kTileHalfs * 2 : kScanFloats * 4;
    __shared__ __attribute__((aligned(16))) unsigned char smem_raw[kLdsBytes];
    __shared__ __attribute__((aligned(16))) float sTot[D];     // A_end per key channel
    uint16_t *sQh = (uint16_t *)smem_raw;
    uint16_t *sQl = sQh + C * TS;
    uint16_t *sKh = sQl + C * TS;
    uint16_t *sKl = sKh + C * TS;
    uint16_t *sV = sKl + C * TS;
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

    // staging loads: rows tid/8 and tid/8 + 32 of the chunk, channels (tid%8)*8 .. +7; unconditional, clamped
    uint4 rq[2], rl[2], rk[2], rv[2];
    auto prefetch = [&](int chunk) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int tok = min(chunk * C + (tid >> 3) + 32 * it, n - 1);
            const int64_t off = (int64_t)tok * a.in.stride_n + (tid & 7) * 8;
            rq[it] = *(const uint4 *)(gq + off);
            rl[it] = *(const uint4 *)(gl + off);
            if (OWNKEY) rk[it] = *(const uint4 *)(gk + off);
            rv[it] = *(const uint4 *)(gv + off);
        }
    };
    prefetch(0);

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

    // column-wise preparation: this thread's key channel and token quarter
    const int pc = 16 * wave + (lane & 15), pu = lane >> 4;

    const int n_chunks = (n + C - 1) / C;
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int t0 = chunk * C;
        const int nt = min(C, n - t0);
        const int qa = wa ^ (chunk & 1);                  // query half of this wave in this chunk

        // ---- raw tiles: q -> Q~hi, lambda -> K~hi, own key -> K~lo, v -> V; rows past the end neutral ----
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int row = (tid >> 3) + 32 * it, col = (tid & 7) * 8;
            const bool live = row < nt;
            *(uint4 *)&sQh[tix(row, col)] = keep_or(live, rq[it], 0u);
            *(uint4 *)&sKh[tix(row, col)] = keep_or(live, rl[it], 0x3f803f80u);     // lambda = 1
            if (OWNKEY) *(uint4 *)&sKl[tix(row, col)] = keep_or(live, rk[it], 0u);
            *(uint4 *)&sV[row * TS + col] = keep_or(live, rv[it], 0u);
        }
        // which of the chunk's 64 tokens sit on a row boundary (bit t), same in every wavefront
        const unsigned long long bmask =
            __ballot(is_boundary(a.start_pos + t0 + lane + 1, a.grid_w, a.mode));
        __syncthreads();                                  // (P) raw tiles visible
        if (chunk + 1 < n_chunks) prefetch(chunk + 1);

        // ---- column-wise: running decay, K~ = k / A, Q~ = q_scale q A, split, in place ----
        bool trip;
        {
            float A[16], kk[16];
            const uint32_t bits = (uint32_t)(bmask >> (16 * pu)) & 0xffffu;
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                const int idx = tix(16 * pu + m, pc);
                const float lraw = __uint_as_float((uint32_t)sKh[idx] << 16);
                kk[m] = OWNKEY ? __uint_as_float((uint32_t)sKl[idx] << 16) : 1.0f - lraw;
                A[m] = ((bits >> m) & 1u) ? 1.0f : lraw;
            }
#pragma unroll
            for (int m = 1; m < 16; ++m) A[m] *= A[m - 1];
            // totals of the four quarters of this channel (lanes pc%16 + 16*u of this wavefront)
            const float T = A[15];
            const float T0 = __shfl(T, lane & 15), T1 = __shfl(T, (lane & 15) + 16);
            const float T2 = __shfl(T, (lane & 15) + 32), T3 = __shfl(T, (lane & 15) + 48);
            const float pre = pu == 0 ? 1.0f : pu == 1 ? T0 : pu == 2 ? T0 * T1 : (T0 * T1) * T2;
            const float tot = ((T0 * T1) * T2) * T3;
            trip = !(tot >= kMinChunkDecay);
            if (pu == 0) sTot[pc] = tot;
            const float pq = pre * a.q_scale;
#pragma unroll
            for (int m = 0; m < 16; m += 2) {
                const int i0 = tix(16 * pu + m, pc), i1 = tix(16 * pu + m + 1, pc);
                const float q0 = __uint_as_float((uint32_t)sQh[i0] << 16), q1 = __uint_as_float((uint32_t)sQh[i1] << 16);
                const float a0 = A[m] * pre, a1 = A[m + 1] * pre;
                uint32_t hi, lo;
                split2(kk[m] * __builtin_amdgcn_rcpf(a0), kk[m + 1] * __builtin_amdgcn_rcpf(a1), hi, lo, sc);
                sKh[i0] = (uint16_t)hi; sKh[i1] = (uint16_t)(hi >> 16);
                sKl[i0] = (uint16_t)lo; sKl[i1] = (uint16_t)(lo >> 16);
                split2(q0 * (A[m] * pq), q1 * (A[m + 1] * pq), hi, lo, sc);
                sQh[i0] = (uint16_t)hi; sQh[i1] = (uint16_t)(hi >> 16);
                sQl[i0] = (uint16_t)lo; sQl[i1] = (uint16_t)(lo >> 16);
            }
        }
        if (__syncthreads_or(trip)) {                     // (A) operand tiles visible, or give up
            // every thread has left the tiles; redo the whole sequence step by step
            scan::scan_sequence<1, OUT_BF16, OWNKEY ? scan::OWNKEY : scan::TIED, 64>(a, bh, 0, (float *)smem_raw);
            return;
        }

        const int i_row = qa * 32 + l32;                  // this lane's query (column of the transposed tiles)
        Frag fqh[4], fql[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            fqh[s].u = *(const uint4 *)&sQh[tix(i_row, 16 * s + 8 * g)];
            fql[s].u = *(const uint4 *)&sQl[tix(i_row, 16 * s + 8 * g)];
        }

        f32x16 acc0, acc1, accO;
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; accO[r] = 0.f; }
        // ---- scores P^T[j][i] = sum_c K~[j][c] Q~[i][c], key block 0 (and 1 for the upper query half) ----
        auto scores = [&](f32x16 &acc, int jb) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag kh, kl;
                kh.u = *(const uint4 *)&sKh[tix(jb * 32 + l32, 16 * s + 8 * g)];
                kl.u = *(const uint4 *)&sKl[tix(jb * 32 + l32, 16 * s + 8 * g)];
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
                fk.h[0] = tr_read(&sKh[tix(r0, kcol)]);
                fk.h[1] = tr_read(&sKh[tix(r1, kcol)]);
                accS = mfma(fk, fv[s], accS);
                fk.h[0] = tr_read(&sKl[tix(r0, kcol)]);
                fk.h[1] = tr_read(&sKl[tix(r1, kcol)]);
                accS = mfma(fk, fv[s], accS);
            }
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const float4 t4 = *(const float4 *)&sTot[wa * 32 + 8 * qd + 4 * g];
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
        if (chunk + 1 < n_chunks) publish_state();        // read after the next barrier (A)
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
    const dim3 grid((unsigned)n_seq), block(kThreads);
    const bool out16 = a.out_dtype == LASAD_BF16;
    if (a.k) {
        if (out16) hipLaunchKernelGGL((forward_gated_mfma_kernel<1, 1>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((forward_gated_mfma_kernel<0, 1>), grid, block, 0, s, a);
    } else {
        if (out16) hipLaunchKernelGGL((forward_gated_mfma_kernel<1, 0>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((forward_gated_mfma_kernel<0, 0>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace lasad
