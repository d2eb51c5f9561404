// Decay table of Spatial-Aware Decay (Section 3.4, second equation; Algorithm 1
// boundary branch): lambda[h, i] for positions start_pos+1 .. start_pos+n and the
// integer prefix E(t) (non-boundary positions among 1..t).  Pure index math plus a
// copy of gamma's bits; one thread per output element, coalesced stores.
#include "lasad_internal.h"

namespace lasad {

__global__ void __launch_bounds__(256)
decay_factors_kernel(const float *__restrict__ gamma, int Hh, int grid_w, int start_pos, int n,
                     int mode, float *__restrict__ lambda_out, int32_t *__restrict__ cum_out)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t n_lambda = lambda_out ? (int64_t)Hh * n : 0;
    if (idx < n_lambda) {
        const int h = (int)(idx / n);
        const int i = (int)(idx - (int64_t)h * n);
        const int t = start_pos + 1 + i;
        lambda_out[idx] = is_boundary(t, grid_w, mode) ? 1.0f : gamma[h];
    } else if (cum_out && idx - n_lambda <= n) {
        const int i = (int)(idx - n_lambda);
        cum_out[i] = cum_exp(start_pos + i, grid_w, mode);
    }
}

hipError_t launch_decay_factors(const float *gamma, int Hh, int grid_w, int start_pos, int n,
                                int mode, float *lambda_out, int32_t *cum_out, hipStream_t s)
{
    const int64_t total = (lambda_out ? (int64_t)Hh * n : 0) + (cum_out ? (int64_t)n + 1 : 0);
    if (total == 0) return hipSuccess;
    const int block = 256;
    const int64_t grid = (total + block - 1) / block;
    hipLaunchKernelGGL(decay_factors_kernel, dim3((unsigned)grid), dim3(block), 0, s,
                       gamma, Hh, grid_w, start_pos, n, mode, lambda_out, cum_out);
    return hipGetLastError();
}

}  // namespace lasad
