// Kernel and launcher of the token-serial fp32 forward (see lasad_scan.h).
#include "lasad_scan.h"

namespace lasad {

namespace {

using namespace scan;

template <int IN_BF16, int OUT_BF16, int KIND, int NJ>
__global__ void __launch_bounds__(kThreads)
forward_scan_kernel(ForwardArgs a)
{
    constexpr int JS = kD / NJ;            // workgroups per sequence
    __shared__ __attribute__((aligned(16))) float lds[lds_floats<KIND>()];
    const int bh = blockIdx.x / JS;
    scan_sequence<IN_BF16, OUT_BF16, KIND, NJ>(a, bh, (blockIdx.x - bh * JS) * NJ, lds);
}

template <int IN_BF16, int OUT_BF16, int KIND>
void launch_nj(const ForwardArgs &a, hipStream_t s)
{
    const int64_t n_seq = (int64_t)a.B * a.Hh;
    // two workgroups per sequence while that still leaves workgroup slots free on 256 CUs
    if (n_seq <= 256 && !a.norm)     // (the output norm needs all 64 channels of a token in one workgroup)
        hipLaunchKernelGGL((forward_scan_kernel<IN_BF16, OUT_BF16, KIND, 32>), dim3((unsigned)(n_seq * 2)), dim3(kThreads), 0, s, a);
    else
        hipLaunchKernelGGL((forward_scan_kernel<IN_BF16, OUT_BF16, KIND, 64>), dim3((unsigned)n_seq), dim3(kThreads), 0, s, a);
}

template <int KIND>
void launch_kind(const ForwardArgs &a, hipStream_t s)
{
    const bool in16 = a.io_dtype == LASAD_BF16, out16 = a.out_dtype == LASAD_BF16;
    if (in16 && out16) launch_nj<1, 1, KIND>(a, s);
    else if (in16) launch_nj<1, 0, KIND>(a, s);
    else launch_nj<0, 0, KIND>(a, s);
}

}  // namespace

hipError_t launch_forward_scan(const ForwardArgs &a, hipStream_t s)
{
    if (a.d != kD || (int64_t)a.B * a.Hh * 2 > 0x7fffffff) return hipErrorInvalidValue;
    if (!a.lam) launch_kind<SCALAR>(a, s);
    else if (!a.k) launch_kind<TIED>(a, s);
    else launch_kind<OWNKEY>(a, s);
    return hipGetLastError();
}

}  // namespace lasad
