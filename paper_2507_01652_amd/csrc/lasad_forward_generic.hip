// Generic forward kernel: fp32 arithmetic on the vector ALUs, any supported head
// dim (32 / 64 / 128), fp32 or bf16 storage.  It is the path for fp32 inputs (whose
// 1e-5 tolerance rules out bf16 matrix-core operands) and for shapes the MFMA
// kernel does not take, and for the vector (data-dependent) decay of Section 3.4.
// One workgroup walks one (batch, head) sequence with the recurrence of
// Section 3.4 (see lasad_recurrence.h).  Head dim 64 goes to the faster scan kernel
// (lasad_forward_scan.hip) unless the environment sets LASAD_SCAN=0.
#include <stdlib.h>

#include "lasad_recurrence.h"

namespace lasad {

namespace {

template <int D, int IN_BF16, int OUT_BF16, int GATED>
__global__ void __launch_bounds__(kRecThreads)
forward_generic_kernel(ForwardArgs a)
{
    __shared__ float smem[recurrence_lds_floats<D, GATED>()];
    recurrence_sequence<D, IN_BF16, OUT_BF16, GATED>(a, blockIdx.x, smem);
}

template <int D>
hipError_t launch_d(const ForwardArgs &a, hipStream_t s)
{
    const dim3 grid((unsigned)(a.B * a.Hh)), block(kRecThreads);
    const bool in16 = a.io_dtype == LASAD_BF16, out16 = a.out_dtype == LASAD_BF16;
    if (a.lam) {
        if (in16 && out16) hipLaunchKernelGGL((forward_generic_kernel<D, 1, 1, 1>), grid, block, 0, s, a);
        else if (in16) hipLaunchKernelGGL((forward_generic_kernel<D, 1, 0, 1>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((forward_generic_kernel<D, 0, 0, 1>), grid, block, 0, s, a);
    } else {
        if (in16 && out16) hipLaunchKernelGGL((forward_generic_kernel<D, 1, 1, 0>), grid, block, 0, s, a);
        else if (in16) hipLaunchKernelGGL((forward_generic_kernel<D, 1, 0, 0>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((forward_generic_kernel<D, 0, 0, 0>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_forward_generic(const ForwardArgs &a, hipStream_t s)
{
    static const bool scan = [] { const char *e = getenv("LASAD_SCAN"); return !(e && e[0] == '0'); }();
    // the fused activations and the norm exist in the scan kernel only: such calls go there whatever the switch says
    const bool fused = a.fused_act || a.norm;
    if (fused && a.d != 64) return hipErrorInvalidValue;
    if (a.d == 64 && (scan || fused)) return launch_forward_scan(a, s);
    switch (a.d) {
        case 32: return launch_d<32>(a, s);
        case 64: return launch_d<64>(a, s);
        case 128: return launch_d<128>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace lasad
