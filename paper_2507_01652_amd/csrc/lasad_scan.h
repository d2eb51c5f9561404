// Token-serial fp32 forward for head dim 64 on the vector ALUs (Section 3.4 recurrence):
//     S <- diag(lambda_t) S + k_t v_t^T,   o_t = q_scale * S^T q_t,
// with lambda_t either the per-head scalar gamma (1 at a row boundary) or the per-token
// decay vector of Algorithm 1 (key tied to it, k_t = 1 - lambda_t, unless a key is given).
// It is the path for the vector decay and for fp32 inputs; arithmetic is fp32 throughout.
//
// Work split.  One 256-thread workgroup owns NJ value channels (columns of S) of one
// (batch, head) sequence: NJ = 64 (whole head) or 32 (two workgroups per head, chosen when
// there are too few sequences to fill the chip).  Lane j of a key-channel group holds
// S[c][j] for the group's R = NJ/4 key channels c in registers.  A 16-lane row belongs to
// one group, and row lane n holds the token's q, k, lambda entries for key channel
// c = group*R + n%R, so every multiply-add takes its per-channel operand straight from a
// neighbour lane through the DPP row broadcast of the VALU instruction: no LDS read and no
// extra move per operand.  Per token and key channel the inner loop is three VALU
// instructions (decay, rank-1 update, output accumulate).
//
// Tokens move in batches of 16: global loads for batch b+1 are in flight while batch b
// is computed; a batch is converted to fp32 once (q scaled, lambda forced to 1 at row
// boundaries, tied key formed) into a double-buffered LDS stage.  Each key-channel group
// leaves its partial outputs in a double-buffered LDS area and one pass per batch adds the
// groups and stores o, so the workgroup meets one barrier per 16 tokens.
#pragma once

#include "lasad_internal.h"

namespace lasad {
namespace scan {

constexpr int kThreads = 256;
constexpr int kT = 16;          // tokens per batch
constexpr int kD = 64;

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

// decay kind: per-head scalar; vector with k = 1 - lambda; vector with own key; and the two walks of the
// vector-decay BACKWARD passes, which are the same recurrence with the tensors in other roles
// (ScanRoles): decay per key channel (row of S) as in the forward, or per column of S
enum { SCALAR = 0, TIED = 1, OWNKEY = 2, ROLES_ROW = 3, ROLES_COL = 4 };

// Which tensor feeds which operand plane of the walk, for the ROLES kinds: plane PQ (row operand of
// the output contraction, scaled by q_scale), PK (row operand of the rank-1 update), PV (column
// operand of the update), PL (decay; 1 at a row boundary of the pass's start column).
struct ScanRoles {
    const void *ptr[4];
    int shift[4];         // 0, or -1: the plane of token m holds the tensor's token m - 1 (token 0: a neutral value)
    int one_minus[4];     // the plane holds 1 - x (a key tied to the decay)
    int act[4];           // applied to the tensor's value first: 0 nothing, 1 SiLU, 2 sigmoid (Algorithm 1's activations)
    const void *lo[4];    // not NULL (bf16 inputs only): a second tensor of the same layout, added to the first
};
enum { ACT_NONE = 0, ACT_SILU = 1, ACT_SIGMOID = 2 };

// LDS planes of one staged batch
enum { PQ = 0, PK = 1, PV = 2, PL = 3 };

#define DPPS(i) " row_newbcast:" #i " row_mask:0xf bank_mask:0xf bound_ctrl:1\n"

// Eight key channels of one token.  Operands: %0-%7 state entries (in place), %8-%11 output
// accumulators (OP starts or continues them), %12 q, %13 k, %14 lambda (row-broadcast sources), %15 v of this lane's
// column.  Every instruction reads registers written at least four instructions earlier
// (the DPP read-after-VALU-write spacing); the leading s_nop covers whatever preceded the block.
#define SCAN8_GATED(OP, a, b, c, d, e, f, g, h)                                                        \
    "s_nop 1\n"                                                                                  \
    "v_mul_f32_dpp %0, %14, %0" DPPS(a) "v_mul_f32_dpp %1, %14, %1" DPPS(b)                      \
    "v_mul_f32_dpp %2, %14, %2" DPPS(c) "v_mul_f32_dpp %3, %14, %3" DPPS(d)                      \
    "v_mul_f32_dpp %4, %14, %4" DPPS(e) "v_mul_f32_dpp %5, %14, %5" DPPS(f)                      \
    "v_mul_f32_dpp %6, %14, %6" DPPS(g) "v_mul_f32_dpp %7, %14, %7" DPPS(h)                      \
    SCAN8_TAIL(OP, a, b, c, d, e, f, g, h)

#define SCAN8_SCALAR(OP, a, b, c, d, e, f, g, h)                                                       \
    "s_nop 1\n"                                                                                  \
    "v_mul_f32 %0, %14, %0\n v_mul_f32 %1, %14, %1\n v_mul_f32 %2, %14, %2\n v_mul_f32 %3, %14, %3\n" \
    "v_mul_f32 %4, %14, %4\n v_mul_f32 %5, %14, %5\n v_mul_f32 %6, %14, %6\n v_mul_f32 %7, %14, %7\n" \
    SCAN8_TAIL(OP, a, b, c, d, e, f, g, h)

#define SCAN8_TAIL(OP, a, b, c, d, e, f, g, h)                                                     \
    "v_fmac_f32_dpp %0, %13, %15" DPPS(a) "v_fmac_f32_dpp %1, %13, %15" DPPS(b)                  \
    "v_fmac_f32_dpp %2, %13, %15" DPPS(c) "v_fmac_f32_dpp %3, %13, %15" DPPS(d)                  \
    "v_fmac_f32_dpp %4, %13, %15" DPPS(e) "v_fmac_f32_dpp %5, %13, %15" DPPS(f)                  \
    "v_fmac_f32_dpp %6, %13, %15" DPPS(g) "v_fmac_f32_dpp %7, %13, %15" DPPS(h)                  \
    OP " %8, %12, %0" DPPS(a) OP " %9, %12, %1" DPPS(b)                                          \
    OP " %10, %12, %2" DPPS(c) OP " %11, %12, %3" DPPS(d)                                        \
    "v_fmac_f32_dpp %8, %12, %4" DPPS(e) "v_fmac_f32_dpp %9, %12, %5" DPPS(f)                    \
    "v_fmac_f32_dpp %10, %12, %6" DPPS(g) "v_fmac_f32_dpp %11, %12, %7" DPPS(h)

#define SCAN8_STATE(S) "+v"(S[0]), "+v"(S[1]), "+v"(S[2]), "+v"(S[3]), "+v"(S[4]), "+v"(S[5]), "+v"(S[6]), "+v"(S[7])
// first eight channels of a token: the accumulators start here (plain multiply, early-clobber outputs)
#define SCAN8_OPS_FIRST(S, o, q, k, l, v)                                                          \
    : SCAN8_STATE(S), "=&v"(o[0]), "=&v"(o[1]), "=&v"(o[2]), "=&v"(o[3]) : "v"(q), "v"(k), "v"(l), "v"(v)
#define SCAN8_OPS_NEXT(S, o, q, k, l, v)                                                           \
    : SCAN8_STATE(S), "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3]) : "v"(q), "v"(k), "v"(l), "v"(v)

// One token for key channels BASE .. BASE+7 of the group (BASE = 0 or 8).
template <int KIND, int BASE>
__device__ __forceinline__ void scan8(float *S, float *o, float q, float k, float l, float v)
{
    if (KIND == SCALAR || KIND == ROLES_COL) {            // the decay is a per-lane (per-column) factor
        if (BASE == 0) asm(SCAN8_SCALAR("v_mul_f32_dpp", 0, 1, 2, 3, 4, 5, 6, 7) SCAN8_OPS_FIRST(S, o, q, k, l, v));
        else asm(SCAN8_SCALAR("v_fmac_f32_dpp", 8, 9, 10, 11, 12, 13, 14, 15) SCAN8_OPS_NEXT(S, o, q, k, l, v));
    } else {
        if (BASE == 0) asm(SCAN8_GATED("v_mul_f32_dpp", 0, 1, 2, 3, 4, 5, 6, 7) SCAN8_OPS_FIRST(S, o, q, k, l, v));
        else asm(SCAN8_GATED("v_fmac_f32_dpp", 8, 9, 10, 11, 12, 13, 14, 15) SCAN8_OPS_NEXT(S, o, q, k, l, v));
    }
}

template <int IN_BF16, int KIND>
struct Loader {
    static constexpr int VEC = IN_BF16 ? 8 : 4;                 // elements per 16-byte load
    static constexpr int NA = KIND >= OWNKEY ? 4 : 3;           // tensors read from memory
    static constexpr bool ROLES = KIND >= ROLES_ROW;
    const ScanRoles *roles = nullptr;                           // ROLES kinds only
    static constexpr int PER_ARRAY = kT * kD / VEC;             // 16-byte loads per tensor and batch
    static constexpr int TOTAL = NA * PER_ARRAY;
    static constexpr int NL = (TOTAL + kThreads - 1) / kThreads;   // loads per thread and batch
    u4 raw[NL];

    // which tensor the i-th load of this thread reads, and where
    __device__ static void where(int i, int &arr, int &tok, int &c0)
    {
        int idx = threadIdx.x + kThreads * i;
        idx = idx < TOTAL ? idx : TOTAL - 1;
        arr = idx / PER_ARRAY;
        const int w = idx - arr * PER_ARRAY;
        tok = w / (kD / VEC);
        c0 = (w - tok * (kD / VEC)) * VEC;
    }

    __device__ const void *tensor(const ForwardArgs &a, int arr) const
    {
        if (ROLES) return roles->ptr[arr];
        if (KIND == SCALAR) return arr == 0 ? a.q : arr == 1 ? a.k : a.v;
        if (KIND == TIED) return arr == 0 ? a.q : arr == 1 ? a.lam : a.v;
        return arr == 0 ? a.q : arr == 1 ? a.lam : arr == 2 ? a.k : a.v;
    }

    // issue the loads of the batch starting at token t0 (rows past the end re-read the last token;
    // stage() replaces them by neutral tokens)
    __device__ void fetch(const ForwardArgs &a, int64_t in_base, int t0)
    {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            int arr, tok, c0;
            where(i, arr, tok, c0);
            int t = min(t0 + tok, a.n_tokens - 1);
            if (ROLES) t = max(t + roles->shift[arr], 0);
            const int64_t idx = in_base + (int64_t)t * a.in.stride_n + c0;
            const char *p = (const char *)tensor(a, arr) + idx * (IN_BF16 ? 2 : 4);
            raw[i] = *(const u4 *)p;
        }
    }

    // convert the fetched batch to fp32 and write it to the LDS stage [plane][token][channel]
    __device__ void stage(const ForwardArgs &a, int64_t in_base, int t0, float *st) const
    {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            // a thread past the end of the list repeats the last item (same values to the same
            // place), which keeps every load unconditionally used and therefore issued early
            int arr, tok, c0;
            where(i, arr, tok, c0);
            float f[VEC];
            if (IN_BF16) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    f[2 * e] = __uint_as_float(raw[i][e] << 16);
                    f[2 * e + 1] = __uint_as_float(raw[i][e] & 0xffff0000u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) f[e] = __uint_as_float(raw[i][e]);
            }
            if (!ROLES && KIND != SCALAR && a.fused_act && arr <= 1) {   // Algorithm 1: q := SiLU(q), lambda := sigmoid(lambda)
#pragma unroll
                for (int e = 0; e < VEC; ++e) f[e] = arr == 0 ? silu_f32(f[e]) : sigmoid_f32(f[e]);
            }
            const bool past_end = t0 + tok >= a.n_tokens;
            if (ROLES) {
                // plane = tensor index; rows past the end and a shifted read before the first token are neutral
                if (IN_BF16 && roles->lo[arr]) {             // (rare route: loaded here, not ahead)
                    const int t = max(min(t0 + tok, a.n_tokens - 1) + roles->shift[arr], 0);
                    const u4 w = *(const u4 *)((const uint16_t *)roles->lo[arr] + in_base + (int64_t)t * a.in.stride_n + c0);
#pragma unroll
                    for (int e = 0; e < VEC / 2; ++e) {
                        f[2 * e] += __uint_as_float(w[e] << 16);
                        f[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u);
                    }
                }
                if (roles->act[arr]) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) f[e] = roles->act[arr] == ACT_SILU ? silu_f32(f[e]) : sigmoid_f32(f[e]);
                }
                if (roles->one_minus[arr]) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) f[e] = 1.0f - f[e];
                }
                const bool neutral = past_end || t0 + tok + roles->shift[arr] < 0;
                if (arr == PL && (neutral || is_boundary(a.start_pos + t0 + tok + 1, a.grid_w, a.mode))) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) f[e] = 1.0f;
                } else if (neutral) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) f[e] = 0.0f;
                }
                if (arr == PQ) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) f[e] *= a.q_scale;
                }
                float *dst = st + (arr * kT + tok) * kD + c0;
#pragma unroll
                for (int e = 0; e < VEC; e += 4) *(f4 *)(dst + e) = f4{f[e], f[e + 1], f[e + 2], f[e + 3]};
                continue;
            }
            if (past_end) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) f[e] = (KIND != SCALAR && arr == 1) ? 1.0f : 0.0f;
            }
            int plane;
            if (arr == 0) {
                plane = PQ;
#pragma unroll
                for (int e = 0; e < VEC; ++e) f[e] *= a.q_scale;
            } else if (KIND == SCALAR) {
                plane = arr == 1 ? PK : PV;
            } else if (arr == 1) {
                plane = PL;
                if (KIND == TIED) {   // the key comes from the decay before the boundary override
                    float *kd = st + (PK * kT + tok) * kD + c0;
#pragma unroll
                    for (int e = 0; e < VEC; e += 4)
                        *(f4 *)(kd + e) = f4{1.0f - f[e], 1.0f - f[e + 1], 1.0f - f[e + 2], 1.0f - f[e + 3]};
                }
                if (is_boundary(a.start_pos + t0 + tok + 1, a.grid_w, a.mode)) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) f[e] = 1.0f;
                }
            } else {
                plane = (KIND == OWNKEY && arr == 2) ? PK : PV;
            }
            float *dst = st + (plane * kT + tok) * kD + c0;
#pragma unroll
            for (int e = 0; e < VEC; e += 4) *(f4 *)(dst + e) = f4{f[e], f[e + 1], f[e + 2], f[e + 3]};
        }
    }
};

// LDS floats one workgroup needs (stage and partial-sum areas, both double-buffered)
template <int KIND>
constexpr int lds_floats() { return 2 * (KIND == SCALAR ? 3 : 4) * kT * kD + 2 * kT * kThreads; }

// Walk sequence bh, value channels j0 .. j0+NJ-1, with the calling 256-thread workgroup.
// lds: lds_floats<KIND>() floats, 16-byte aligned.
template <int IN_BF16, int OUT_BF16, int KIND, int NJ>
__device__ void scan_sequence(const ForwardArgs &a, int bh, int j0, float *lds, const ScanRoles *roles = nullptr)
{
    constexpr int CG = kThreads / NJ;      // key-channel groups
    constexpr int R = kD / CG;             // key channels per thread (16 or 8)
    constexpr int NP = KIND == SCALAR ? 3 : 4;   // LDS planes per staged batch
    constexpr int STAGE = NP * kT * kD;
    constexpr int RED = kT * CG * NJ;
    float *const s_stage[2] = {lds, lds + STAGE};
    float *const s_red[2] = {lds + 2 * STAGE, lds + 2 * STAGE + RED};
    const int b = bh / a.Hh, h = bh - b * a.Hh;
    const int tid = threadIdx.x;
    const int j = tid % NJ, cg = tid / NJ;
    const int cop = cg * R + (tid % 16) % R;      // key channel whose operands this lane carries
    const float gamma = KIND == SCALAR ? a.gamma[h] : 1.0f;

    // The walk's state is [update row operand][update column operand].  A column-decay walk (ROLES_COL) is the
    // transposed form of a pass whose state is [decayed channel][other index]: in memory its incoming and final
    // states keep THAT layout (the one of the chunked column pass it stands in for), so they are read and
    // written transposed here.
    float S[R];
    if (a.state_in) {
        if (KIND == ROLES_COL) {
            const float *s0 = a.state_in + (int64_t)bh * kD * kD + (int64_t)(j0 + j) * kD;
#pragma unroll
            for (int r = 0; r < R; ++r) S[r] = s0[cg * R + r];
        } else {
            const float *s0 = a.state_in + (int64_t)bh * kD * kD + j0 + j;
#pragma unroll
            for (int r = 0; r < R; ++r) S[r] = s0[(cg * R + r) * kD];
        }
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) S[r] = 0.f;
    }

    // the state's loads complete here, not at their first use inside the token loop
#pragma unroll
    for (int r = 0; r < R; ++r) asm volatile("" : "+v"(S[r]));

    const int64_t in_base = (int64_t)b * a.in.stride_b + (int64_t)h * a.in.stride_h;
    const int64_t out_base = (int64_t)b * a.out.stride_b + (int64_t)h * a.out.stride_h + j0;
    const int nb = (a.n_tokens + kT - 1) / kT;

    Loader<IN_BF16, KIND> ld;
    ld.roles = roles;
    if (nb > 0) {
        ld.fetch(a, in_base, 0);
        ld.stage(a, in_base, 0, s_stage[0]);
    }
    __syncthreads();

    for (int bt = 0; bt < nb; ++bt) {
        const int t0 = bt * kT;
        const int nt = min(kT, a.n_tokens - t0);
        const float *st = s_stage[bt & 1];
        float *red = s_red[bt & 1];
        // The next batch's loads are in flight while this one is computed.  They are issued and
        // consumed in the same iteration, unconditionally (after the last batch they re-read the
        // last token and stage neutral rows nobody uses), so that no register carries a pending
        // load around the loop and the compiler's wait counts stay exact.
        ld.fetch(a, in_base, t0 + kT);
        __builtin_amdgcn_sched_barrier(0);      // keep the loads ahead of the compute block

        // all 16 tokens of the batch, unrolled: rows past the end of the sequence were staged as
        // neutral tokens (lambda 1, k = v = q = 0) and leave the state as it is
#pragma unroll
        for (int tt = 0; tt < kT; ++tt) {
            const float qo = st[(PQ * kT + tt) * kD + cop];
            const float ko = st[(PK * kT + tt) * kD + cop];
            const float vj = st[(PV * kT + tt) * kD + j0 + j];
            float lo;
            if (KIND == SCALAR)
                lo = (t0 + tt >= a.n_tokens || is_boundary(a.start_pos + t0 + tt + 1, a.grid_w, a.mode) ||
                      (a.first_decay_off && t0 + tt == 0)) ? 1.0f : gamma;
            else if (KIND == ROLES_COL) lo = st[(PL * kT + tt) * kD + j0 + j];
            else lo = st[(PL * kT + tt) * kD + cop];
            float o[4];
            scan8<KIND, 0>(S, o, qo, ko, lo, vj);
            if (R == 16) scan8<KIND, 8>(S + 8, o, qo, ko, lo, vj);
            red[(tt * CG + cg) * NJ + j] = (o[0] + o[1]) + (o[2] + o[3]);
        }

        ld.stage(a, in_base, t0 + kT, s_stage[(bt + 1) & 1]);
        __syncthreads();

        // add the groups' partial sums and store o for this batch, two channels per thread and pass
#pragma unroll
        for (int i = 0; i < kT * NJ / 2 / kThreads; ++i) {
            const int e = tid + kThreads * i;
            const int tt = e / (NJ / 2), jp = (e - tt * (NJ / 2)) * 2;
            f2 acc = *(const f2 *)(red + (tt * CG) * NJ + jp);
#pragma unroll
            for (int g = 1; g < CG; ++g) acc += *(const f2 *)(red + (tt * CG + g) * NJ + jp);
            if (NJ == kD && a.norm) {
                // root-mean-square normalisation over the 64 channels of the token: its 32 channel
                // pairs sit in 32 consecutive lanes
                float ss = acc[0] * acc[0] + acc[1] * acc[1];
#pragma unroll
                for (int off = 16; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
                const float rstd = __builtin_amdgcn_rsqf(ss * (1.0f / kD) + a.norm_eps);
                const int hh = bh % a.Hh;
                const float w0 = a.norm_w ? a.norm_w[hh * kD + jp] : 1.0f, w1 = a.norm_w ? a.norm_w[hh * kD + jp + 1] : 1.0f;
                acc[0] *= rstd * w0;
                acc[1] *= rstd * w1;
            }
            if (tt < nt) {
                const int64_t oi = out_base + (int64_t)(t0 + tt) * a.out.stride_n + jp;
                if (OUT_BF16)
                    *(uint32_t *)((uint16_t *)a.o + oi) =
                        (uint32_t)float_to_bf16_bits(acc[0]) | ((uint32_t)float_to_bf16_bits(acc[1]) << 16);
                else
                    *(f2 *)((float *)a.o + oi) = acc;
            }
        }
    }

    if (a.state_out) {
        if (KIND == ROLES_COL) {
            float *s1 = a.state_out + (int64_t)bh * kD * kD + (int64_t)(j0 + j) * kD;
#pragma unroll
            for (int r = 0; r < R; ++r) s1[cg * R + r] = S[r];
        } else {
            float *s1 = a.state_out + (int64_t)bh * kD * kD + j0 + j;
#pragma unroll
            for (int r = 0; r < R; ++r) s1[(cg * R + r) * kD] = S[r];
        }
    }
}

}  // namespace scan
}  // namespace lasad
