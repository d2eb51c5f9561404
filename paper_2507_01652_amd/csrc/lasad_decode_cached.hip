// Decode step from a key / value cache instead of the d x d state, for the first positions of a
// sequence: unrolling the Section 3.4 recurrence from a zero state,
//     o_t = q_scale sum_{j<=t} gamma^(E(t) - E(j)) (q_t . k_j) v_j,    E = non-boundary positions so far,
// touches (t + 1) rows of k and v (2 d elements each) where the state form reads and writes
// d x d fp32 (Section 1 of the paper counts the same trade for softmax attention's cache): fewer
// bytes while t + 1 < 2 d^2 * 4 / (2 d * elt), i.e. the first 128 positions for d = 64 and bf16.
// A caller switches to the state form by building the state from the cache with one
// lasad_forward_chunked call (state_out) over the cached rows.
//
// One wavefront per (batch, head), four to a workgroup (the form is meant for few cached tokens:
// a whole workgroup per sequence spent its time on launch and barriers).  A token's k (and v) row is
// read by D / 8 consecutive lanes (bf16; D / 4 for fp32) with one 16-byte load each, so the
// wavefront takes 64 / (D / 8) tokens per step, four steps in flight.  A lane keeps its 8 query
// entries and 8 output accumulators in registers: partial dot over its channels, butterfly over
// the lanes of the token, decay weight, then score * v into the accumulators; at the end the
// accumulators are added over the token slots by butterflies (fixed order).  No LDS, no barrier.
// The step's own k and v come from the call's arguments and are appended to the cache by the
// same launch.
#include "lasad_internal.h"

namespace lasad {

namespace {

constexpr int kCdThreads = 256;

template <int IN_BF16, int VEC>
__device__ inline void cd_unpack(const uint4 w, float (&f)[VEC])
{
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
    if (IN_BF16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            f[2 * e] = __uint_as_float(ww[e] << 16);
            f[2 * e + 1] = __uint_as_float(ww[e] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = __uint_as_float(ww[e]);
    }
}


// One lane's VEC output values, scaled, as a 16-byte (bf16: VEC = 8) or VEC/4 x 16-byte (fp32) store.
template <int OUT_BF16, int VEC>
__device__ inline void cd_store(void *o, int64_t idx, float q_scale, const float (&acc)[VEC])
{
    if (OUT_BF16) {
        uint4 w;
        w.x = (uint32_t)float_to_bf16_bits(q_scale * acc[0]) | ((uint32_t)float_to_bf16_bits(q_scale * acc[1]) << 16);
        w.y = (uint32_t)float_to_bf16_bits(q_scale * acc[2]) | ((uint32_t)float_to_bf16_bits(q_scale * acc[3]) << 16);
        w.z = (uint32_t)float_to_bf16_bits(q_scale * acc[4 % VEC]) | ((uint32_t)float_to_bf16_bits(q_scale * acc[5 % VEC]) << 16);
        w.w = (uint32_t)float_to_bf16_bits(q_scale * acc[6 % VEC]) | ((uint32_t)float_to_bf16_bits(q_scale * acc[7 % VEC]) << 16);
        *(uint4 *)((uint16_t *)o + idx) = w;             // (bf16 output implies bf16 input: VEC = 8)
    } else {
#pragma unroll
        for (int e = 0; e < VEC; e += 4)
            *(float4 *)((float *)o + idx + e) =
                make_float4(q_scale * acc[e], q_scale * acc[e + 1], q_scale * acc[e + 2], q_scale * acc[e + 3]);
    }
}

template <int IN_BF16, int OUT_BF16, int D>
__global__ void __launch_bounds__(kCdThreads)
decode_cached_kernel(CachedDecodeArgs a)
{
    constexpr int VEC = IN_BF16 ? 8 : 4;                  // elements per 16-byte load
    constexpr int LPT = D / VEC;                          // lanes per token row
    constexpr int TPW = 64 / LPT;                         // tokens per step
    constexpr int UNROLL = 4;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t bh = (int64_t)blockIdx.x * 4 + wave;
    if (bh >= (int64_t)a.B * a.Hh) return;
    const int h = (int)(bh % a.Hh);
    const int piece = lane % LPT, slot = lane / LPT;      // 16-byte piece of the row; token slot in the wavefront
    const int pos = a.pos;
    const int elt = IN_BF16 ? 2 : 4;
    const char *q_row = (const char *)a.q + (bh * D + piece * VEC) * elt;               // q, k, v, o: [B, Hh, d]
    const char *k_row = (const char *)a.k + (bh * D + piece * VEC) * elt;
    const char *v_row = (const char *)a.v + (bh * D + piece * VEC) * elt;
    const int64_t cache_off = (bh * a.cache_tokens * D + piece * VEC) * elt;            // caches: [B, Hh, T, d]
    const char *kc = (const char *)a.k_cache + cache_off, *vc = (const char *)a.v_cache + cache_off;

    float qf[VEC];
    cd_unpack<IN_BF16, VEC>(*(const uint4 *)q_row, qf);
    if (slot < 2) {                                       // append this step's k and v rows
        char *dst = (char *)(slot ? a.v_cache : a.k_cache) + cache_off + (int64_t)pos * D * elt;
        *(uint4 *)dst = *(const uint4 *)(slot ? v_row : k_row);
    }
    const float lg = log2f(a.gamma[h]);
    const int e_now = cum_exp(pos + 1, a.grid_w, a.mode);

    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    for (int j0 = 0; j0 <= pos; j0 += UNROLL * TPW) {
        uint4 kw[UNROLL], vw[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            // (row pos comes from the arguments: the append above is not ordered against these loads)
            const int jc = min(j0 + u * TPW + slot, pos);
            kw[u] = *(const uint4 *)(jc == pos ? k_row : kc + (int64_t)jc * D * elt);
            vw[u] = *(const uint4 *)(jc == pos ? v_row : vc + (int64_t)jc * D * elt);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int j = j0 + u * TPW + slot;
            const int jc = min(j, pos);
            float kf[VEC], vf[VEC];
            cd_unpack<IN_BF16, VEC>(kw[u], kf);
            cd_unpack<IN_BF16, VEC>(vw[u], vf);
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) s = fmaf(qf[e], kf[e], s);
#pragma unroll
            for (int off = LPT / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off);
            const int de = e_now - cum_exp(jc + 1, a.grid_w, a.mode);        // decays applied after token j
            s *= de == 0 ? 1.0f : __builtin_amdgcn_exp2f((float)de * lg);
            s = j <= pos ? s : 0.f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = fmaf(s, vf[e], acc[e]);
        }
    }
    // over the token slots of the wavefront
#pragma unroll
    for (int off = LPT; off < 64; off <<= 1) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += __shfl_xor(acc[e], off);
    }
    if (slot == 0) cd_store<OUT_BF16, VEC>(a.o, bh * D + piece * VEC, a.q_scale, acc);
}

// Vector decay (Section 3.4 as written: a decay vector per token over the key channels, key tied to it unless
// given).  Unrolled from a zero state,
//     o_t = q_scale sum_{j<=t} [ sum_c q_t[c] (prod_{s=j+1..t} l_s[c]) k_j[c] ] v_j,    l_s = 1 at a boundary,
// so the caches hold the gate rows (and v; k only with an own key): with the tied key a cached token is again
// 2 d elements.  The weight of a token is a vector, the running product of the decays of the tokens after it, so
// the cache is walked from the newest token backwards, in blocks of TPW runs: token slot s of the wavefront walks
// R consecutive tokens (newest first) with its product in registers.  First the slot's rows are fetched (they
// stay in registers) and the gates multiplied up, one exclusive product scan over the slots gives every run the
// decays of the runs before it, then the run is walked again with the v rows.  Cross-lane traffic per token is
// the butterfly of the score alone.  Products of numbers in [0, 1] only underflow, which is the right limit.
#ifndef LASAD_CD_RUN
#define LASAD_CD_RUN 4
#endif
constexpr int kCdRun = LASAD_CD_RUN;       // tokens of a run (its rows are held in registers; 4 measured best of 4, 8, 16)

// (t mod W) for the boundary test of a run that is walked towards smaller t: one division per run, then steps
struct RowResidue {
    int r, W;
    __device__ void init(int t, int grid_w) { W = grid_w; r = t % grid_w; }
    __device__ void step_down() { r = r == 0 ? W - 1 : r - 1; }
    __device__ bool boundary(int mode) const      // is the 1-indexed position with residue r a boundary position
    {
        return mode == LASAD_RESET_LAST_COL ? r == 0 : mode == LASAD_RESET_FIRST_COL ? (r == 1 || W == 1) : false;
    }
};

template <int IN_BF16, int OUT_BF16, int D>
__global__ void __launch_bounds__(kCdThreads)
decode_cached_gated_kernel(CachedDecodeArgs a)
{
    constexpr int VEC = IN_BF16 ? 8 : 4;
    constexpr int LPT = D / VEC;
    constexpr int TPW = 64 / LPT;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t bh = (int64_t)blockIdx.x * 4 + wave;
    if (bh >= (int64_t)a.B * a.Hh) return;
    const int piece = lane % LPT, slot = lane / LPT;
    const int pos = a.pos;
    const int elt = IN_BF16 ? 2 : 4;
    const int64_t row_off = (bh * D + piece * VEC) * elt;
    const char *q_row = (const char *)a.q + row_off, *l_row = (const char *)a.lam + row_off;
    const char *k_row = a.k ? (const char *)a.k + row_off : nullptr, *v_row = (const char *)a.v + row_off;
    const int64_t cache_off = (bh * a.cache_tokens * D + piece * VEC) * elt;
    const char *lc = (const char *)a.lam_cache + cache_off, *vc = (const char *)a.v_cache + cache_off;
    const char *kc = a.k ? (const char *)a.k_cache + cache_off : nullptr;
    const int64_t row_bytes = (int64_t)D * elt;

    float qf[VEC];
    cd_unpack<IN_BF16, VEC>(*(const uint4 *)q_row, qf);
    if (slot == 0) {                                      // append this step's gate, v (and k) rows
        const int64_t dst = cache_off + (int64_t)pos * row_bytes;
        *(uint4 *)((char *)a.lam_cache + dst) = *(const uint4 *)l_row;
        *(uint4 *)((char *)a.v_cache + dst) = *(const uint4 *)v_row;
        if (a.k) *(uint4 *)((char *)a.k_cache + dst) = *(const uint4 *)k_row;
    }

    float acc[VEC], carry[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { acc[e] = 0.f; carry[e] = 1.f; }
    for (int top = pos; top >= 0; top -= TPW * kCdRun) {  // block: tokens top, top - 1, ... (at most TPW * kCdRun)
        const int nb = min(top + 1, TPW * kCdRun);
        const int R = (nb + TPW - 1) / TPW;               // run length of this block, the same for every slot
        const int first = top - slot * R;                 // newest token of this lane's run; tokens below 0 are empty
        // (row pos comes from the arguments: the append above is not ordered against these loads)
        uint4 lw[kCdRun];
#pragma unroll
        for (int i = 0; i < kCdRun; ++i) {
            if (i < R) {
                const int jc = max(first - i, 0);
                lw[i] = *(const uint4 *)(jc == pos ? l_row : lc + (int64_t)jc * row_bytes);
            }
        }
        uint4 vw[kCdRun], kw[kCdRun];                     // (issued now, used by the second walk)
#pragma unroll
        for (int i = 0; i < kCdRun; ++i) {
            if (i < R) {
                const int jc = max(first - i, 0);
                vw[i] = *(const uint4 *)(jc == pos ? v_row : vc + (int64_t)jc * row_bytes);
                if (a.k) kw[i] = *(const uint4 *)(jc == pos ? k_row : kc + (int64_t)jc * row_bytes);
            }
        }
        RowResidue rr;
        rr.init(max(first, 0) + 1, a.grid_w);             // (an empty run never looks at it)
        const RowResidue rr0 = rr;
        float w[VEC];                                     // product of the decays applied at the run's tokens
#pragma unroll
        for (int e = 0; e < VEC; ++e) w[e] = 1.f;
#pragma unroll
        for (int i = 0; i < kCdRun; ++i) {
            if (i < R) {
                if (first - i >= 0 && !rr.boundary(a.mode)) {
                    float lf[VEC];
                    cd_unpack<IN_BF16, VEC>(lw[i], lf);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) w[e] *= lf[e];
                }
                rr.step_down();
            }
        }
        // inclusive product over the slots 0..slot; the value of the slot before = decays of the runs after this one
#pragma unroll
        for (int off = LPT; off < 64; off <<= 1) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float up = __shfl_up(w[e], off);
                w[e] *= lane >= off ? up : 1.0f;
            }
        }
        float total[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            total[e] = __shfl(w[e], (TPW - 1) * LPT + piece);             // product over the whole block
            const float excl = __shfl_up(w[e], LPT);
            w[e] = carry[e] * (slot ? excl : 1.0f);                         // weight of the run's newest token
        }
        rr = rr0;
#pragma unroll
        for (int i = 0; i < kCdRun; ++i) {                // the run again, with the v (and k) rows
            if (i < R) {
                const bool live = first - i >= 0;
                float lf[VEC], kf[VEC], vf[VEC];
                cd_unpack<IN_BF16, VEC>(lw[i], lf);
                cd_unpack<IN_BF16, VEC>(vw[i], vf);
                if (a.k) {
                    cd_unpack<IN_BF16, VEC>(kw[i], kf);
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) kf[e] = 1.0f - lf[e];      // key from the base gate, boundary or not
                }
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) s = fmaf(qf[e] * w[e], kf[e], s);
#pragma unroll
                for (int off = LPT / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off);
                s = live ? s : 0.f;
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = fmaf(s, vf[e], acc[e]);
                if (live && !rr.boundary(a.mode)) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) w[e] *= lf[e];
                }
                rr.step_down();
            }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) carry[e] *= total[e];
    }
#pragma unroll
    for (int off = LPT; off < 64; off <<= 1) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += __shfl_xor(acc[e], off);
    }
    if (slot == 0) cd_store<OUT_BF16, VEC>(a.o, bh * D + piece * VEC, a.q_scale, acc);
}

template <int D>
void launch_d(const CachedDecodeArgs &a, hipStream_t s)
{
    const dim3 grid((unsigned)(((int64_t)a.B * a.Hh + 3) / 4)), block(kCdThreads);
    const bool in16 = a.io_dtype == LASAD_BF16, out16 = a.out_dtype == LASAD_BF16;
    if (a.lam) {
        if (in16 && out16) hipLaunchKernelGGL((decode_cached_gated_kernel<1, 1, D>), grid, block, 0, s, a);
        else if (in16) hipLaunchKernelGGL((decode_cached_gated_kernel<1, 0, D>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((decode_cached_gated_kernel<0, 0, D>), grid, block, 0, s, a);
        return;
    }
    if (in16 && out16) hipLaunchKernelGGL((decode_cached_kernel<1, 1, D>), grid, block, 0, s, a);
    else if (in16) hipLaunchKernelGGL((decode_cached_kernel<1, 0, D>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((decode_cached_kernel<0, 0, D>), grid, block, 0, s, a);
}

}  // namespace

hipError_t launch_decode_cached(const CachedDecodeArgs &a, hipStream_t s)
{
    if (a.d == 32) launch_d<32>(a, s);
    else if (a.d == 64) launch_d<64>(a, s);
    else if (a.d == 128) launch_d<128>(a, s);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace lasad
