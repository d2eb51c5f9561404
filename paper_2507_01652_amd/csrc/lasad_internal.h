// Internal declarations shared by the translation units of liblasad (gfx950 only).
// Host-side launchers live next to their kernels; the C ABI in lasad_api.hip
// validates arguments and calls them.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lasad.h"

namespace lasad {

// Arguments of one forward call, already validated.
struct ForwardArgs {
    const void *q, *k, *v;
    const void *lam;             // vector decay [B, n, Hh, d] (same layout as q), or NULL: per-head gamma.
                                 // With lam, k may be NULL: the key is then 1 - lam.
    void *o;
    lasad_layout_t in, out;      // element strides of q/k/v and of o
    int io_dtype, out_dtype;
    int B, Hh, d;
    int grid_w;
    int start_pos, n_tokens;
    const float *gamma;
    int mode;
    float q_scale;
    const float *state_in;
    float *state_out;
    // Algorithm 1's elementwise steps fused around the vector-decay recurrence (lam given, k NULL):
    int fused_act;               // 1: q := SiLU(q), lam := sigmoid(lam) on load
    int norm;                    // 1: o := o / sqrt(mean_c(o^2) + norm_eps) * norm_w[h][c] on store
    float norm_eps;
    const float *norm_w;         // [Hh][d] fp32, or NULL for ones
    // segment-parallel plan of the MFMA kernel (filled by its launcher)
    float *seg_states;           // workspace: [B*Hh][n_segments-1][d][d] fp32, or NULL
    int n_segments, seg_chunks;
    // column passes of the layer backward only: low-order bf16 parts of the tensors in the q and v fields
    // (the operand is hi + lo; same layout), or NULL
    const void *q_lo = nullptr, *v_lo = nullptr;
    // 1: the decay of the call's first token is NOT applied to the incoming state (the state then enters
    // the first token's update as it is).  Used by the reversed passes of a backward call whose loss also
    // depends on the forward's final state: its gradient joins the state gradient of the last token undecayed.
    int first_decay_off = 0;
};

// Up to three independent forward passes in one launch of the wave-specialised kernels
// (blockIdx.y = pass): the fields below replace those of the common ForwardArgs.
// Several independent passes of the scalar-decay forward kernels in one launch (blockIdx.y = pass):
// per-pass operands, layouts and start column; everything else is shared (ForwardArgs).
// A pass may also accumulate the decay-gradient term of the backward pass,
//   sign * sum_t E_t (x_t . o_t),   E_t = non-boundary tokens among the first t + 1 of the call,
// from its fp32 output tiles: x is a fourth bf16 tensor laid out like the pass's inputs, and with
// x_rev the pass runs the sequence backwards (pass token m is call token n_tokens - 1 - m).  Each
// workgroup leaves its part of the sum in x_sums[((pass * n_seq) + sequence) * kDotSlots + slot];
// slots it does not use are written as zero.
constexpr int kDotSlots = 8;
struct MultiPass {
    int n_pass;                  // 1: the ForwardArgs as they are (no other member is read)
    int start_pos[3];
    const void *q[3], *k[3], *v[3];
    void *o[3];
    lasad_layout_t in[3], out[3];
    const void *x[3];            // NULL: no sum for this pass
    float x_sign[3];
    int x_rev[3];
    int x_start_pos;             // start column of the call (not of the reversed passes)
    float *x_sums;
    // per-pass incoming / final states ([B, Hh, d, d] fp32 or NULL) and first_decay_off, as in ForwardArgs
    const float *state_in[3] = {nullptr, nullptr, nullptr};
    float *state_out[3] = {nullptr, nullptr, nullptr};
    int first_decay_off[3] = {0, 0, 0};
};

struct DecodeArgs {
    const void *q, *k, *v;
    const void *lam;             // vector decay [B, Hh, d], or NULL: per-head gamma (k NULL: key = 1 - lam)
    void *o;
    int io_dtype, out_dtype;
    int B, Hh, d;
    int fused_act, norm;         // as in ForwardArgs
    float norm_eps;
    const float *norm_w;
    int grid_w, pos;
    const int32_t *pos_rows;     // per batch row positions [B] (device), or NULL: every row at `pos`.
                                 // A row whose position is outside 0 .. grid_n-1 is inactive.
    int grid_n;                  // grid_h * grid_w
    const float *gamma;
    int mode;
    float q_scale;
    float *state;
};

// Arguments of one backward call, already validated.
struct BackwardArgs {
    const void *q, *k, *v, *d_o;   // [B, n, Hh, d] views sharing one layout and storage type
    void *dq, *dk, *dv;            // same logical shape, layout `grad`, type grad_dtype
    float *dgamma;                 // [Hh]
    lasad_layout_t in, grad;
    int io_dtype, grad_dtype;
    int B, Hh, d;
    int grid_w;
    int start_pos, n_tokens;
    const float *gamma;
    int mode;
    float q_scale;
    void *workspace;
    // carved out of the workspace by the launcher
    float *dq32, *dk32, *seq_sums;
    // gradients through a carried state (all [B, Hh, d, d] fp32, each may be NULL): the state before the call's
    // first token, dL/d(final state), and the output dL/d(state_in)
    const float *state_in = nullptr, *d_state_out = nullptr;
    float *d_state_in = nullptr;
};

// Arguments of one decode step from a key / value cache, already validated.
struct CachedDecodeArgs {
    const void *q, *k, *v;       // [B, Hh, d]
    const void *lam = nullptr;   // vector decay: this step's gate row (then gamma is unused, and k may be NULL: tied key)
    void *lam_cache = nullptr;   // vector decay: the gate rows, like the other caches
    void *o;
    void *k_cache, *v_cache;     // [B, Hh, cache_tokens, d], type io_dtype; row pos is written, rows 0..pos-1 read
    int io_dtype, out_dtype;
    int B, Hh, d;
    int cache_tokens;
    int grid_w, pos;
    const float *gamma;
    int mode;
    float q_scale;
};
hipError_t launch_decode_cached(const CachedDecodeArgs &a, hipStream_t s);

// Arguments of one backward call of the vector-decay recurrence, already validated (d == 64).
struct GatedBackwardArgs {
    const void *q, *lam, *k, *v, *d_o;   // k NULL: key tied to the decay, k = 1 - lam
    void *dq, *dlam, *dk, *dv;           // dk NULL with the tied key
    lasad_layout_t in, grad;
    int io_dtype, grad_dtype;
    int B, Hh, d;
    int grid_w;
    int start_pos, n_tokens;
    int mode;
    float q_scale;
    void *workspace;
    const void *d_o_lo;                  // fused_act with bf16 inputs: low-order bf16 part of d_o (d_o is hi + lo), else NULL
    int fused_act;                       // 1: q and lam hold Algorithm 1's pre-activation query and gate logits
                                         // (tied key only); dq and dlam are then the gradients of THOSE tensors
    // gradients through a carried state ([B, Hh, d, d] fp32, each may be NULL): the state before the call's first
    // token, dL/d(final state), and the output dL/d(state_in)
    const float *state_in = nullptr, *d_state_out = nullptr;
    float *d_state_in = nullptr;
};
hipError_t launch_backward_gated(const GatedBackwardArgs &a, hipStream_t s);

// Arguments of one backward call of the fused layer (Algorithm 1 between its Linear maps), validated.
struct LayerBackwardArgs {
    const void *q_pre, *z, *v, *d_out;
    void *dq_pre, *dz, *dv;
    void *d_o_out;                       // not NULL: stop after the normalisation's backward and leave the gradient
    lasad_layout_t d_o_l;                //   that enters the recurrence here (this layout; type io_dtype, or fp32
    int d_o_f32;                         //   if d_o_f32 is set)
    float *dweight;                      // [Hh, d], or NULL
    lasad_layout_t in, dout, grad;
    int io_dtype, grad_dtype;
    int B, Hh, d;
    int grid_w;
    int start_pos, n_tokens;
    int mode;
    float q_scale;
    const float *norm_w;                 // [Hh, d] or NULL (ones)
    float norm_eps;                      // < 0: no normalisation
    void *workspace;
};
hipError_t launch_backward_layer(const LayerBackwardArgs &a, bool use_mfma, hipStream_t s);
size_t backward_layer_workspace_bytes(int B, int Hh, int n_tokens, int d, int io_dtype, const lasad_layout_t &in);
size_t backward_gated_workspace_bytes(int64_t n_seq, int n_tokens, int d);
// extra workspace of lasad_backward_gated with carried states
size_t backward_gated_carried_extra_bytes(int64_t n_seq, int d);

hipError_t launch_decay_factors(const float *gamma, int Hh, int grid_w, int start_pos, int n,
                                int mode, float *lambda_out, int32_t *cum_out, hipStream_t s);
hipError_t launch_forward_generic(const ForwardArgs &a, hipStream_t s);
// d == 64, any storage type, scalar or vector decay: token-serial fp32 scan kernel.
hipError_t launch_forward_scan(const ForwardArgs &a, hipStream_t s);
// bf16 in, d == 64: MFMA chunked kernel.
hipError_t launch_forward_mfma(const ForwardArgs &a, hipStream_t s);
// bf16 in, d == 64, vector decay (lam given): MFMA chunked kernel.
hipError_t launch_forward_gated_mfma(const ForwardArgs &a, hipStream_t s);
// the same with eight wavefronts per sequence (whole sequences only, no segment plan)
hipError_t launch_forward_mfma_ws(const ForwardArgs &a, hipStream_t s);
// twelve wavefronts, doubled LDS buffers, one barrier per chunk: for workgroups that own a compute unit
hipError_t launch_forward_mfma_ws12(const ForwardArgs &a, hipStream_t s);
// n_pass whole-sequence passes (same shapes, types, gamma; fp32 or bf16 output alike) in ONE launch
hipError_t launch_forward_mfma_multi(const ForwardArgs &common, const MultiPass &m, hipStream_t s);
// the vector-decay kernel with twelve wavefronts per sequence (no fused norm)
hipError_t launch_forward_gated_ws(const ForwardArgs &a, hipStream_t s);
// device workspace the MFMA kernel wants for n_seq sequences of n_tokens tokens (0 = none)
size_t forward_mfma_workspace_bytes(int64_t n_seq, int n_tokens);
hipError_t launch_decode(const DecodeArgs &a, hipStream_t s);
// Backward of the scalar-decay forward: three runs of the forward kernels (MFMA kernel if
// use_mfma, else the generic / scan kernels) plus two small finishing kernels.
hipError_t launch_backward(const BackwardArgs &a, bool use_mfma, hipStream_t s);
hipError_t launch_zero_f32(float *p, int n, hipStream_t s);
hipError_t launch_copy_state(const float *src, float *dst, int64_t n, hipStream_t s);   // dst = src (zeros if src is NULL)
size_t backward_workspace_bytes(int64_t n_seq, int n_tokens, int d, int io_dtype);
// extra workspace of a backward call with carried states (transposed copies, the passes' final states, one sum per sequence)
size_t backward_carried_extra_bytes(int64_t n_seq, int d);

// ---- host helpers of the backward passes ---------------------------------------

// Start column for a pass that walks a call's n tokens backwards: with it, reversed step m >= 1
// meets the boundary test of original token n - m (the one whose decay the step applies); the
// mirrored and shifted boundary pattern of a raster grid is again "every W-th position".
inline int reversed_start(int start_pos, int n, int grid_w, int mode)
{
    const int64_t W = grid_w;
    int64_t s = 0;
    if (mode == LASAD_RESET_LAST_COL) s = -((int64_t)start_pos + n + 2);
    else if (mode == LASAD_RESET_FIRST_COL) s = -((int64_t)start_pos + n);
    s %= W;
    if (s < 0) s += W;
    return (int)s;
}

// address of the last of n tokens of a tensor (the base of a walk with a negative token stride)
inline const void *last_token(const void *p, const lasad_layout_t &l, int n, int elt)
{
    return p ? (const char *)p + (int64_t)(n - 1) * l.stride_n * elt : nullptr;
}

// ---- device helpers -----------------------------------------------------------

// Is 1-indexed raster position t one where the decay is switched off
// (Section 3.4 second equation / Algorithm 1 boundary branch)?
__host__ __device__ inline bool is_boundary(int t, int grid_w, int mode)
{
    if (mode == LASAD_RESET_LAST_COL) return (t % grid_w) == 0;
    if (mode == LASAD_RESET_FIRST_COL) return ((t - 1) % grid_w) == 0;
    return false;
}

// factor for an incoming state whose first decay is switched off (ForwardArgs::first_decay_off): the kernels of the
// separable form apply the first token's decay to everything that was there before it, so the state is pre-divided
__device__ inline float incoming_state_scale(const ForwardArgs &a, float gamma)
{
    if (a.first_decay_off && !is_boundary(a.start_pos + 1, a.grid_w, a.mode)) return 1.0f / gamma;
    return 1.0f;
}

// E(t): number of non-boundary positions among 1..t (t >= 0), closed form.
__host__ __device__ inline int cum_exp(int t, int grid_w, int mode)
{
    if (mode == LASAD_RESET_LAST_COL) return t - t / grid_w;
    if (mode == LASAD_RESET_FIRST_COL) return t - (t + grid_w - 1) / grid_w;
    return t;
}

// 1 / (1 + exp(-x)) and x / (1 + exp(-x)) in fp32 (hardware exp and reciprocal, ~1 ulp each;
// exp overflows to inf for very negative x and the reciprocal then returns 0, the right limit)
__device__ inline float sigmoid_f32(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
__device__ inline float silu_f32(float x) { return x * sigmoid_f32(x); }

__device__ inline float bf16_bits_to_float(uint16_t b)
{
    return __uint_as_float(((uint32_t)b) << 16);
}

// float -> bf16 bits, round to nearest even (NaN kept quiet).
__device__ inline uint16_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

}  // namespace lasad
