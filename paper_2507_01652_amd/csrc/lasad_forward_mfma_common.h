// Pieces shared by the chunked scalar-decay matrix-core kernels (lasad_forward_mfma.hip and its
// eight-wave variant lasad_forward_mfma_ws.hip): tile geometry, per-chunk position bookkeeping,
// staging of K and V, decayed keys, and the state update.
#pragma once

#include "lasad_mfma_util.h"
#include "lasad_internal.h"
#include "lasad_recurrence.h"

namespace lasad {
namespace fwd {

constexpr int C = 64;      // chunk length (tokens)
constexpr int D = 64;      // head dim
constexpr int kThreads = 256;
#ifndef LASAD_RS
#define LASAD_RS 72
#endif
#ifndef LASAD_VS
#define LASAD_VS 80
#endif
constexpr int RS = LASAD_RS;     // LDS row stride (elements) of tiles read 16 bytes at a time: 144 B
constexpr int VS = LASAD_VS;     // LDS row stride of the V tile (transpose reads only): 160 B


// number of boundary positions among x small offsets: floor(x / W), 0 <= x < W + 128
__device__ inline int small_div(int x, int W, float rcpW)
{
    if (W > 128) return x >= W ? 1 : 0;
    int q = (int)((float)x * rcpW);
    const int r = x - q * W;
    q += (r >= W) ? 1 : 0;
    q -= (r < 0) ? 1 : 0;
    return q;
}

// Per-chunk position bookkeeping.  col0 = (tokens before the chunk) mod W.  The number of
// boundary positions among the first j+1 tokens of the chunk is floor((j + xoff) / W) with a
// small per-chunk offset xoff, so e_j = j + 1 - floor((j + xoff) / W).
struct ChunkPos {
    int W, mode, col0;
    float rcpW;
    __device__ void init(int start, int grid_w, int boundary_mode)
    {
        W = grid_w; mode = boundary_mode; col0 = start % grid_w; rcpW = 1.0f / (float)grid_w;
    }
    __device__ int xoff() const
    {
        if (mode == LASAD_RESET_LAST_COL) return col0 + 1;
        if (mode == LASAD_RESET_FIRST_COL) return col0 ? col0 : W;
        return 0;
    }
    __device__ int e_of(int j, int xo) const     // e_j of chunk-local token j
    {
        return j + 1 - (mode == LASAD_RESET_NONE ? 0 : small_div(j + xo, W, rcpW));
    }
    __device__ void advance()                    // to the next chunk
    {
        col0 += C;
        if (W > 128) col0 -= col0 >= W ? W : 0;
        else col0 -= W * small_div(col0, W, rcpW);
    }
};

// Decayed keys of one chunk, in registers: every thread scales the two 16-byte pieces of K it
// loaded (rows tid/8 and tid/8 + 32) by c_j = gamma^{-e_j} and splits them into bf16 hi + lo.
struct StagedKeys {
    uint4 hi[2], lo[2];
    float cj[2];
};

__device__ inline void prepare_keys(StagedKeys &st, uint4 (&rk)[2], uint4 (&rv)[2], int tid, int nt,
                                    const ChunkPos &pos, float lg, const SplitConst &sc)
{
    const int xo = pos.xoff();
    if (nt < C) {                                   // tail chunk: rows past the end are zero
#pragma unroll
        for (int it = 0; it < 2; ++it)
            if ((tid >> 3) + 32 * it >= nt) rk[it] = rv[it] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int row = (tid >> 3) + 32 * it;
        const float cj = __builtin_amdgcn_exp2f(-(float)pos.e_of(row, xo) * lg);   // gamma^{-e_j}
        st.cj[it] = cj;
        const uint32_t kw[4] = {rk[it].x, rk[it].y, rk[it].z, rk[it].w};
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2)
            split2(__uint_as_float(kw[w2] << 16) * cj, __uint_as_float(kw[w2] & 0xffff0000u) * cj,
                   hi[w2], lo[w2], sc);
        st.hi[it] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        st.lo[it] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
}

// Write one chunk's K, V (as loaded), decayed keys (hi, lo) and the table of c_j to LDS.
template <bool RAW_K>
__device__ inline void write_tiles(uint16_t *sK, uint16_t *sV, uint16_t *sKh, uint16_t *sKl, float *tabC,
                                   const uint4 (&rk)[2], const uint4 (&rv)[2], const StagedKeys &st, int tid)
{
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int row = (tid >> 3) + 32 * it;
        const int col = (tid & 7) * 8;
        if ((tid & 7) == 0) tabC[row] = st.cj[it];
        if (RAW_K) *(uint4 *)&sK[row * RS + col] = rk[it];
        *(uint4 *)&sV[row * VS + col] = rv[it];
        *(uint4 *)&sKh[row * VS + col] = st.hi[it];
        *(uint4 *)&sKl[row * VS + col] = st.lo[it];
    }
}

// Decay and causal mask on the fp32 scores of key block jb (this lane: query column l32, keys
// 8*qd + 4*g + e), split into bf16 hi + lo operand fragments of the next MFMA.  tabC: the chunk's
// c_j table; cq = l32 - 4*g: key 8*qd + 4*g + e of a diagonal block is at or before the query iff
// 8*qd + e <= cq.
__device__ __forceinline__ void mask_split(const f32x16 &acc, const float *tabC, int jb, bool diagonal, int cq, int g,
                                           const SplitConst &sc, Frag *ph, Frag *pl)
{
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
        const float4 c4 = *(const float4 *)&tabC[jb * 32 + 8 * qd + 4 * g];
        float p0 = acc[4 * qd + 0] * c4.x, p1 = acc[4 * qd + 1] * c4.y;
        float p2 = acc[4 * qd + 2] * c4.z, p3 = acc[4 * qd + 3] * c4.w;
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
}

// V fragments of value-channel half wc: channel n = wc*32 + l32, tokens 16*s + 4*g + {0..3}, + 8
__device__ inline void load_v_frags(Frag (&fv)[4], const uint16_t *sV, int wc, int lane)
{
    const int l32 = lane & 31, g = lane >> 5;
    const int trow = (lane & 15) >> 2;               // row inside the 4-row group this lane points at
    const int tcol = wc * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        fv[s].h[0] = tr_read(&sV[(16 * s + 4 * g + trow) * VS + tcol]);
        fv[s].h[1] = tr_read(&sV[(16 * s + 8 + 4 * g + trow) * VS + tcol]);
    }
}

// S[dk][dv] += sum_j (c_j K[j][dk]) V[j][dv] for the wave's 32 x 32 tile (dk half wa)
__device__ inline void state_update(f32x16 &accS, const uint16_t *sKh, const uint16_t *sKl,
                                    const Frag (&fv)[4], int wa, int lane)
{
    const int l32 = lane & 31, g = lane >> 5;
    const int trow = (lane & 15) >> 2;
    const int tcol = wa * 32 + 16 * (l32 >> 4) + 4 * (lane & 3);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        Frag fkt;
        fkt.h[0] = tr_read(&sKh[(16 * s + 4 * g + trow) * VS + tcol]);
        fkt.h[1] = tr_read(&sKh[(16 * s + 8 + 4 * g + trow) * VS + tcol]);
        accS = mfma(fkt, fv[s], accS);
        fkt.h[0] = tr_read(&sKl[(16 * s + 4 * g + trow) * VS + tcol]);
        fkt.h[1] = tr_read(&sKl[(16 * s + 8 + 4 * g + trow) * VS + tcol]);
        accS = mfma(fkt, fv[s], accS);
    }
}

// K/V staging loads of one chunk of a token range [0, n): unconditional, index clamped.
template <bool NT = false>
__device__ inline void load_kv(uint4 (&rk)[2], uint4 (&rv)[2], const uint16_t *gk, const uint16_t *gv,
                               int t0, int n, int64_t stride_n, int tid)
{
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int tok = min(t0 + (tid >> 3) + 32 * it, n - 1);
        const int64_t off = (int64_t)tok * stride_n + (tid & 7) * 8;
        rk[it] = gload16<NT>(gk + off);
        rv[it] = gload16<NT>(gv + off);
    }
}

// exponent E(end) - E(begin) of a token range, begin/end = tokens consumed before / after it
__device__ inline int range_exponent(int begin, int end, int W, int mode)
{
    return cum_exp(end, W, mode) - cum_exp(begin, W, mode);
}


// Decay-gradient term of a backward pass (see MultiPass).  A lane of an output wave holds, in fp32,
// the 16 channels col + 8*qd + e (qd, e = 0..3) of one output row; it adds
// sign * E_t * (x_t . o_t) for that row and those channels, chunk after chunk, and the wave's total
// goes to its slot of x_sums at the end (butterfly over the lanes: fixed order).
struct GradDot {
    const uint16_t *gx;          // x of this sequence, or NULL: no sum asked for
    int64_t stride_n;
    float sign, acc;
    int rev, n_total, start_pos, grid_w, mode, e0;
    uint2 xr[4];

    __device__ void init(const ForwardArgs &a, const MultiPass &m, int y, int64_t in_base)   // y: pass
    {
        gx = nullptr;
        acc = 0.f;
        if (m.n_pass > 1 && m.x[y]) {
            gx = (const uint16_t *)m.x[y] + in_base;
            stride_n = a.in.stride_n;
            sign = m.x_sign[y];
            rev = m.x_rev[y];
            n_total = a.n_tokens;
            start_pos = m.x_start_pos;
            grid_w = a.grid_w;
            mode = a.mode;
            e0 = cum_exp(start_pos, grid_w, mode);
        }
    }
    // x of row tok (the caller clamps it to the sequence), channels col + 8*qd .. + 3
    __device__ void fetch(int tok, int col)
    {
        if (!gx) return;
        const uint16_t *p = gx + (int64_t)tok * stride_n + col;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) xr[qd] = *(const uint2 *)(p + 8 * qd);
    }
    __device__ void add(const f32x16 &o, int tok, bool live)
    {
        if (!gx) return;
        float d = 0.f;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            d = fmaf(__uint_as_float(xr[qd].x << 16), o[4 * qd + 0], d);
            d = fmaf(__uint_as_float(xr[qd].x & 0xffff0000u), o[4 * qd + 1], d);
            d = fmaf(__uint_as_float(xr[qd].y << 16), o[4 * qd + 2], d);
            d = fmaf(__uint_as_float(xr[qd].y & 0xffff0000u), o[4 * qd + 3], d);
        }
        const int t = rev ? n_total - 1 - tok : tok;
        const int e = cum_exp(start_pos + t + 1, grid_w, mode) - e0;
        acc = fmaf(live ? sign * (float)e : 0.f, d, acc);
    }
    // slot (and zero_slot, if >= 0) of this sequence's entries of x_sums
    __device__ void finish(const MultiPass &m, int y, int64_t n_seq, int bh, int slot, int zero_slot, int lane)
    {
        if (!gx) return;
        float v = acc;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0) {
            float *dst = m.x_sums + ((int64_t)y * n_seq + bh) * kDotSlots;
            dst[slot] = v;
            if (zero_slot >= 0) dst[zero_slot] = 0.f;
        }
    }
};

// The fp32 recurrence over a whole sequence (decay outside the range of the factorised form) with
// the same sum, taken from the fp32 output values as they are produced.  Run by the first
// kRecThreads threads of the workgroup; smem as recurrence_sequence wants it.
struct RecDotHook {
    const uint16_t *gx;
    int64_t stride_n;
    int rev, n_total, start_pos, grid_w, mode, e0;
    float *acc;
    __device__ void operator()(int tok, int c, float v) const
    {
        const float x = bf16_bits_to_float(gx[(int64_t)tok * stride_n + c]);
        const int t = rev ? n_total - 1 - tok : tok;
        const int e = cum_exp(start_pos + t + 1, grid_w, mode) - e0;
        *acc = fmaf((float)e * x, v, *acc);
    }
};

template <int OUT_BF16>
__device__ inline void recurrence_with_dot(const ForwardArgs &a, const MultiPass &m, int y, int bh, float *smem)
{
    if (!(m.n_pass > 1 && m.x[y])) {
        recurrence_sequence<D, 1, OUT_BF16>(a, bh, smem);
        return;
    }
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    float acc = 0.f;
    RecDotHook hook;
    hook.gx = (const uint16_t *)m.x[y] + (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    hook.stride_n = a.in.stride_n;
    hook.rev = m.x_rev[y]; hook.n_total = a.n_tokens; hook.start_pos = m.x_start_pos;
    hook.grid_w = a.grid_w; hook.mode = a.mode;
    hook.e0 = cum_exp(m.x_start_pos, a.grid_w, a.mode);
    hook.acc = &acc;
    recurrence_sequence<D, 1, OUT_BF16>(a, bh, smem, hook);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    __syncthreads();                   // the recurrence's last reads of its LDS block
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x < kDotSlots) {     // the total in slot 0, the other slots zero
        float v = 0.f;
        if (threadIdx.x == 0) {
            for (int w = 0; w < kRecThreads / 64; ++w) v += smem[w];
            v *= m.x_sign[y];
        }
        m.x_sums[((int64_t)y * a.B * a.Hh + bh) * kDotSlots + threadIdx.x] = v;
    }
}

}  // namespace fwd
}  // namespace lasad
