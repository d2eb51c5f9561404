// Recurrent decode step (Algorithm 1 loop body; Section 3.4 first equation):
//     S <- lambda S + k v^T,   o = q_scale * S^T q      for every (batch, head).
// 0.5 flop per byte: the kernel is a stream over the fp32 states (read once,
// written once, in place), so the design goal is HBM bandwidth.
//
// One 64-lane wavefront owns one d x d state.  A lane reads 16-byte pieces
// (4 value channels) so that every wave-wide load covers whole contiguous rows of
// S; up to 16 loads per lane (the whole state at d = 64) are issued back to back
// before any arithmetic to keep many bytes in flight.  Each lane keeps the partial q-weighted column sums of
// the rows it touched; lanes that share a column group are then combined with
// cross-lane shuffles (no LDS round trip for the reduction).
//
// The states are touched exactly once per step, so their loads and stores carry
// the non-temporal hint (measured: 28.6 us instead of 33.6 us per step on 5120
// states, the same as a plain read-modify-write stream over the same bytes), and
// a workgroup is a single wavefront so that every wave starts as early as possible.
#include "lasad_internal.h"

namespace lasad {

namespace {

constexpr int kWaves = 1;   // wavefronts (= states) per workgroup

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline float4 load_stream(const float4 *p)
{
    const f32x4 r = __builtin_nontemporal_load((const f32x4 *)p);
    return make_float4(r.x, r.y, r.z, r.w);
}

__device__ inline void store_stream(float4 *p, float4 x)
{
    const f32x4 r = {x.x, x.y, x.z, x.w};
    __builtin_nontemporal_store(r, (f32x4 *)p);
}

template <int IN_BF16>
__device__ inline float ld_in(const void *p, int64_t idx)
{
    if (IN_BF16) return bf16_bits_to_float(((const uint16_t *)p)[idx]);
    return ((const float *)p)[idx];
}

// GATED = 1: the decay is a vector over the key channels (row i of S is scaled by lambda[i],
// or by 1 at a row-boundary position) and the key is 1 - lambda unless a key is given
// (Section 3.4, Algorithm 1 as written).
template <int D, int IN_BF16, int OUT_BF16, int GATED>
__global__ void __launch_bounds__(kWaves * 64)
decode_kernel(DecodeArgs a, int n_states)
{
    constexpr int CG = D / 4;        // column groups (float4) per row
    constexpr int RPP = 64 / CG;     // rows covered by one wave-wide load
    constexpr int P = D / RPP;       // loads per lane for the whole state
    constexpr int PB = P < 16 ? P : 16;   // loads in flight per lane at a time
    __shared__ float sqk[kWaves][2 + GATED][D];

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bh = blockIdx.x * kWaves + wave;
    if (bh >= n_states) return;      // whole wave leaves together; no barrier below
    const int h = bh % a.Hh;
    const int cg = lane % CG, r0 = lane / CG;
    const int64_t vec = (int64_t)bh * D;
    int pos = a.pos;
    if (a.pos_rows) {                // continuous batching: every batch row at its own raster position
        pos = a.pos_rows[bh / a.Hh];
        if (pos < 0 || pos >= a.grid_n) {      // inactive row: state untouched, output row zero (whole wave)
            if (r0 == 0) {
                if (OUT_BF16) *(ushort4 *)((uint16_t *)a.o + vec + cg * 4) = make_ushort4(0, 0, 0, 0);
                else *(float4 *)((float *)a.o + vec + cg * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
            }
            return;
        }
    }
    const int t = pos + 1;
    const bool boundary = is_boundary(t, a.grid_w, a.mode);
    const float lam = (boundary || GATED) ? 1.0f : a.gamma[h];

    float4 *S = (float4 *)(a.state + (int64_t)bh * D * D);

    // Global loads in issue order: the small q, k, v vectors, then the first
    // batch of state pieces; only then are q and k parked in LDS (fp32,
    // wave-private region) so that every lane can read any row's q_i, k_i.
    constexpr int NQ = (D + 63) / 64;
    float qr[NQ], kr[NQ], lr[NQ];
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        const int c = lane + 64 * i;
        qr[i] = c < D ? ld_in<IN_BF16>(a.q, vec + c) : 0.f;
        if (GATED) {
            float l = c < D ? ld_in<IN_BF16>(a.lam, vec + c) : 1.f;
            if (a.fused_act) { l = sigmoid_f32(l); qr[i] = silu_f32(qr[i]); }     // Algorithm 1's activations
            kr[i] = a.k ? (c < D ? ld_in<IN_BF16>(a.k, vec + c) : 0.f) : 1.0f - l;   // key from the base decay
            lr[i] = boundary ? 1.0f : l;
        } else {
            kr[i] = c < D ? ld_in<IN_BF16>(a.k, vec + c) : 0.f;
            lr[i] = 1.0f;
        }
    }
    float4 vv;
    vv.x = ld_in<IN_BF16>(a.v, vec + cg * 4 + 0);
    vv.y = ld_in<IN_BF16>(a.v, vec + cg * 4 + 1);
    vv.z = ld_in<IN_BF16>(a.v, vec + cg * 4 + 2);
    vv.w = ld_in<IN_BF16>(a.v, vec + cg * 4 + 3);

    float4 s[PB];
#pragma unroll
    for (int p = 0; p < PB; ++p) s[p] = load_stream(&S[(r0 + p * RPP) * CG + cg]);

#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        const int c = lane + 64 * i;
        if (c < D) {
            sqk[wave][0][c] = qr[i];
            sqk[wave][1][c] = kr[i];
            if (GATED) sqk[wave][2][c] = lr[i];
        }
    }
    // wave-level ordering of the LDS writes above against the reads below
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int p0 = 0; p0 < P; p0 += PB) {
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            const int row = r0 + (p0 + p) * RPP;
            const float qi = sqk[wave][0][row], ki = sqk[wave][1][row];
            const float li = GATED ? sqk[wave][2][row] : lam;
            float4 x = s[p];
            x.x = fmaf(li, x.x, ki * vv.x);
            x.y = fmaf(li, x.y, ki * vv.y);
            x.z = fmaf(li, x.z, ki * vv.z);
            x.w = fmaf(li, x.w, ki * vv.w);
            store_stream(&S[row * CG + cg], x);
            acc.x = fmaf(qi, x.x, acc.x);
            acc.y = fmaf(qi, x.y, acc.y);
            acc.z = fmaf(qi, x.z, acc.z);
            acc.w = fmaf(qi, x.w, acc.w);
        }
        if (p0 + PB < P) {   // next batch of state pieces (d = 128 only)
#pragma unroll
            for (int p = 0; p < PB; ++p) s[p] = load_stream(&S[(r0 + (p0 + PB + p) * RPP) * CG + cg]);
        }
    }
    // combine the RPP lanes that share a column group (lane bits above log2(CG))
#pragma unroll
    for (int off = CG; off < 64; off <<= 1) {
        acc.x += __shfl_xor(acc.x, off, 64);
        acc.y += __shfl_xor(acc.y, off, 64);
        acc.z += __shfl_xor(acc.z, off, 64);
        acc.w += __shfl_xor(acc.w, off, 64);
    }
    float qs = a.q_scale;
    if (GATED && a.norm) {           // Norm(o): root mean square over the D channels (lanes 0 .. CG-1 hold them)
        float ss = (acc.x * acc.x + acc.y * acc.y) + (acc.z * acc.z + acc.w * acc.w);
#pragma unroll
        for (int off = CG / 2; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
        const float rstd = __builtin_amdgcn_rsqf(qs * qs * ss * (1.0f / D) + a.norm_eps);
        qs *= rstd;
        if (a.norm_w) {
            const float4 w4 = *(const float4 *)(a.norm_w + h * D + cg * 4);
            acc.x *= w4.x; acc.y *= w4.y; acc.z *= w4.z; acc.w *= w4.w;
        }
    }
    if (r0 == 0) {
        if (OUT_BF16) {
            uint16_t *o = (uint16_t *)a.o + vec + cg * 4;
            ushort4 pk;
            pk.x = float_to_bf16_bits(qs * acc.x);
            pk.y = float_to_bf16_bits(qs * acc.y);
            pk.z = float_to_bf16_bits(qs * acc.z);
            pk.w = float_to_bf16_bits(qs * acc.w);
            *(ushort4 *)o = pk;
        } else {
            float *o = (float *)a.o + vec + cg * 4;
            *(float4 *)o = make_float4(qs * acc.x, qs * acc.y, qs * acc.z, qs * acc.w);
        }
    }
}

template <int D>
hipError_t launch_d(const DecodeArgs &a, hipStream_t s)
{
    const int n_states = a.B * a.Hh;
    const dim3 grid((unsigned)((n_states + kWaves - 1) / kWaves)), block(kWaves * 64);
    const bool in16 = a.io_dtype == LASAD_BF16, out16 = a.out_dtype == LASAD_BF16;
    if (a.lam) {
        if (in16 && out16) hipLaunchKernelGGL((decode_kernel<D, 1, 1, 1>), grid, block, 0, s, a, n_states);
        else if (in16) hipLaunchKernelGGL((decode_kernel<D, 1, 0, 1>), grid, block, 0, s, a, n_states);
        else hipLaunchKernelGGL((decode_kernel<D, 0, 0, 1>), grid, block, 0, s, a, n_states);
    } else {
        if (in16 && out16) hipLaunchKernelGGL((decode_kernel<D, 1, 1, 0>), grid, block, 0, s, a, n_states);
        else if (in16) hipLaunchKernelGGL((decode_kernel<D, 1, 0, 0>), grid, block, 0, s, a, n_states);
        else hipLaunchKernelGGL((decode_kernel<D, 0, 0, 0>), grid, block, 0, s, a, n_states);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const DecodeArgs &a, hipStream_t s)
{
    switch (a.d) {
        case 32: return launch_d<32>(a, s);
        case 64: return launch_d<64>(a, s);
        case 128: return launch_d<128>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lasad
