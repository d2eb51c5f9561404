// Decode step from a key / value cache instead of the d x d state, for the first positions of a
// sequence: unrolling the Section 3.4 recurrence from a zero state,
//     o_t = q_scale sum_{j<=t} gamma^(E(t) - E(j)) (q_t . k_j) v_j,    E = non-boundary positions so far,
// touches (t + 1) rows of k and v (2 d elements each) where the state form reads and writes
// d x d fp32 (Section 1 of the paper counts the same trade for softmax attention's cache): fewer
// bytes while t + 1 < 2 d^2 * 4 / (2 d * elt), i.e. the first 128 positions for d = 64 and bf16.
// A caller switches to the state form by building the state from the cache with one
// lasad_forward_chunked call (state_out) over the cached rows.
//
// One 256-thread workgroup per (batch, head).  Tokens go in tiles of 256: thread j forms the
// decayed score of token j against the query (its own k row, 16-byte loads), then thread
// (channel c, part p) adds score_j v_j[c] over the tokens j = p mod PARTS (v rows read by
// consecutive lanes); the parts are added in a fixed order.  The step's own k and v come from the
// call's arguments and are appended to the cache by the same launch.
#include "lasad_internal.h"

namespace lasad {

namespace {

constexpr int kCdThreads = 256;

template <int IN_BF16>
__device__ inline float cd_load(const void *p, int64_t i)
{
    return IN_BF16 ? bf16_bits_to_float(((const uint16_t *)p)[i]) : ((const float *)p)[i];
}

template <int IN_BF16, int OUT_BF16, int D>
__global__ void __launch_bounds__(kCdThreads)
decode_cached_kernel(CachedDecodeArgs a)
{
    constexpr int PARTS = kCdThreads / D;
    constexpr int VEC = IN_BF16 ? 8 : 4;                  // elements per 16-byte load
    __shared__ __attribute__((aligned(16))) float sQ[D];
    __shared__ float sS[kCdThreads];
    __shared__ float sRed[PARTS][D];
    const int bh = blockIdx.x, h = bh % a.Hh;
    const int tid = threadIdx.x;
    const int pos = a.pos;
    const int64_t tok_base = (int64_t)bh * D;                              // q, k, v, o: [B, Hh, d]
    const int64_t cache_base = (int64_t)bh * a.cache_tokens * D;          // caches: [B, Hh, T, d]
    const int elt = IN_BF16 ? 2 : 4;

    if (tid < D) sQ[tid] = cd_load<IN_BF16>(a.q, tok_base + tid);
    if (tid < 2 * D / VEC) {                                              // append this step's k and v rows
        const int which = tid / (D / VEC), piece = tid - which * (D / VEC);
        const char *src = (const char *)(which ? a.v : a.k) + (tok_base + piece * VEC) * elt;
        char *dst = (char *)(which ? a.v_cache : a.k_cache) + (cache_base + (int64_t)pos * D + piece * VEC) * elt;
        *(uint4 *)dst = *(const uint4 *)src;
    }
    const float lg = log2f(a.gamma[h]);
    const int e_now = cum_exp(pos + 1, a.grid_w, a.mode);
    __syncthreads();

    const int c = tid % D, part = tid / D;
    float acc = 0.f;
    for (int j0 = 0; j0 <= pos; j0 += kCdThreads) {
        {   // score of token j0 + tid
            const int j = j0 + tid;
            float s = 0.f;
            if (j <= pos) {
                const char *row = j == pos ? (const char *)a.k + tok_base * elt
                                           : (const char *)a.k_cache + (cache_base + (int64_t)j * D) * elt;
#pragma unroll
                for (int i = 0; i < D / VEC; ++i) {
                    const uint4 w = *(const uint4 *)(row + i * 16);
                    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
                    if (IN_BF16) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            s = fmaf(__uint_as_float(ww[e] << 16), sQ[i * 8 + 2 * e], s);
                            s = fmaf(__uint_as_float(ww[e] & 0xffff0000u), sQ[i * 8 + 2 * e + 1], s);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) s = fmaf(__uint_as_float(ww[e]), sQ[i * 4 + e], s);
                    }
                }
                const int de = e_now - cum_exp(j + 1, a.grid_w, a.mode);     // decays applied after token j
                s *= de == 0 ? 1.0f : __builtin_amdgcn_exp2f((float)de * lg);
            }
            sS[tid] = s;
        }
        __syncthreads();
        const int nj = min(kCdThreads, pos + 1 - j0);
        for (int jj = part; jj < nj; jj += PARTS) {
            const int j = j0 + jj;
            const float vj = j == pos ? cd_load<IN_BF16>(a.v, tok_base + c)
                                      : cd_load<IN_BF16>(a.v_cache, cache_base + (int64_t)j * D + c);
            acc = fmaf(sS[jj], vj, acc);
        }
        __syncthreads();
    }
    sRed[part][c] = acc;
    __syncthreads();
    if (tid < D) {
        float o = 0.f;
#pragma unroll
        for (int p = 0; p < PARTS; ++p) o += sRed[p][tid];
        o *= a.q_scale;
        if (OUT_BF16) ((uint16_t *)a.o)[tok_base + tid] = float_to_bf16_bits(o);
        else ((float *)a.o)[tok_base + tid] = o;
    }
}

template <int D>
void launch_d(const CachedDecodeArgs &a, hipStream_t s)
{
    const dim3 grid((unsigned)((int64_t)a.B * a.Hh)), block(kCdThreads);
    const bool in16 = a.io_dtype == LASAD_BF16, out16 = a.out_dtype == LASAD_BF16;
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
