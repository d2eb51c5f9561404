// Small helpers shared by the matrix-core kernels (gfx950): operand fragments of
// v_mfma_f32_32x32x16_bf16, the LDS transpose read, and the bf16 hi + lo split of a
// computed fp32 operand.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lasad {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((__vector_size__(4 * sizeof(short))));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4v __attribute__((ext_vector_type(4)));

// 16-byte global loads and stores.  NT: with the non-temporal hint, for rows that a call touches once
// (q, k, v in, o out): they stream through the caches without displacing what is reused.
template <bool NT>
__device__ inline uint4 gload16(const void *p)
{
    if (NT) {
        const u32x4 r = __builtin_nontemporal_load((const u32x4 *)p);
        return make_uint4(r.x, r.y, r.z, r.w);
    }
    return *(const uint4 *)p;
}
template <bool NT>
__device__ inline void gstore16(void *p, uint4 v)
{
    if (NT) {
        const u32x4 r = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(r, (u32x4 *)p);
    } else {
        *(uint4 *)p = v;
    }
}
template <bool NT>
__device__ inline void gstore16(float *p, float x, float y, float z, float w)
{
    if (NT) {
        const f32x4v r = {x, y, z, w};
        __builtin_nontemporal_store(r, (f32x4v *)p);
    } else {
        *(float4 *)p = make_float4(x, y, z, w);
    }
}

struct Frag {              // 8 bf16 = one lane's share of a 32x16 MFMA operand
    union { bf16x8 v; uint4 u; uint2 h[2]; };
};

__device__ inline uint32_t pack2(float lo, float hi)
{
    f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

__device__ inline uint2 tr_read(const uint16_t *p)
{
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
    return __builtin_bit_cast(uint2, r);
}

__device__ inline f32x16 mfma(const Frag &a, const Frag &b, f32x16 acc)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc, 0, 0, 0);
}

// Constants of the hi/lo split: the packed bf16 pairs (-1, 0) and (0, -1).  They are kept
// opaque to the compiler (in VGPRs) because, folded into an inline constant of
// v_dot2c_f32_bf16, -1.0 is encoded in the fp16 format and the product comes out wrong.
struct SplitConst {
    bf16x2 m10, m01;
    __device__ void init()
    {
        uint32_t a = 0x0000BF80u, b = 0xBF800000u;
        asm volatile("" : "+v"(a), "+v"(b));
        m10 = __builtin_bit_cast(bf16x2, a);
        m01 = __builtin_bit_cast(bf16x2, b);
    }
};

// split a pair of fp32 values into packed bf16 hi (round to nearest) and lo (the residual
// x - hi, exact in fp32, formed as x + (-1) * hi by one bf16 dot-product instruction each)
__device__ inline void split2(float x0, float x1, uint32_t &hi, uint32_t &lo, const SplitConst &sc)
{
    hi = pack2(x0, x1);
    const bf16x2 hv = __builtin_bit_cast(bf16x2, hi);
    const float l0 = __builtin_amdgcn_fdot2_f32_bf16(hv, sc.m10, x0, false);
    const float l1 = __builtin_amdgcn_fdot2_f32_bf16(hv, sc.m01, x1, false);
    lo = pack2(l0, l1);
}

}  // namespace lasad
