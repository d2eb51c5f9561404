// Twelve-wave variant of the chunked vector-decay forward (see lasad_forward_gated_mfma.hip for the
// algorithm, the operand preparation and the range rule) for the case that a sequence has a
// compute unit to itself (at most 256 sequences): three groups of four wavefronts on the same
// four SIMDs, every LDS buffer doubled, one barrier per chunk.
//
//   output waves (0-3):  scores K~ Q~^T, causal mask + split, P V, Q~ S, output tile            (chunk c)
//   state waves  (4-7):  state update K~^T V, row scaling by A_end, bf16 hi/lo copy of S^T      (chunk c -> c+1)
//   loader waves (8-11): global loads, running decay products, K~ and Q~ (split), tile writes   (chunk c+1),
//                        16-byte stores of the finished output tile                             (chunk c-1)
//
// A chunk whose decay leaves the range of the factorisation is seen by the loader waves one
// chunk ahead; the barrier carries the flag to every wave and the workgroup redoes its sequence
// with the token-serial fp32 routine (waves 0-3; the others leave).
// FUSED = 1 applies SiLU to q and the sigmoid to the gate while the chunk is prepared.
// NORM = 1 divides every output token by the root mean square of its 64 channels (times a weight):
// the two output waves that hold a token's channel halves leave their sums of squares in LDS
// before the chunk's barrier and keep the fp32 tile in registers; after the barrier, before they
// start the next chunk, they scale, round and write the tile, and the loader waves store it one
// chunk later than without the norm (one more barrier at the end of the sequence for the last tile).
#include "lasad_forward_gated_common.h"
#include "lasad_scan.h"

namespace lasad {

namespace {

using namespace gated;



}  // namespace
}  // namespace lasad

#include "lasad_gated_ws_body.h"

namespace lasad {

namespace {

using namespace gated;

template <int OUT_BF16, int OWNKEY, int FUSED, int NORM>
__global__ void __launch_bounds__(kWsThreads, 1)
forward_gated_ws_kernel(ForwardArgs a)
{
    constexpr int kScanFloats = scan::lds_floats<OWNKEY ? scan::OWNKEY : scan::TIED>();
    static_assert(2 * kSetHalfs * 2 >= kScanFloats * 4, "the fallback needs the LDS block");
    __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kSetHalfs];
    __shared__ __attribute__((aligned(16))) float sTot[2][D];  // A_end per key channel, by chunk parity
    __shared__ __attribute__((aligned(16))) int sTrip[2][4];   // range flag of each loader wave, by barrier parity
    __shared__ float sSS[NORM ? 2 * 2 * C : 1];                // sums of squares: chunk parity, channel half, token
    // (the out-of-line fallback takes the arguments by reference: it gets them where the launch put
    // them, in the kernel-argument segment -- a reference to the by-value parameter would make
    // every thread of every launch copy the struct to its stack first)
    const int bh = blockIdx.x;
    gated_ws_body<OUT_BF16, OWNKEY, FUSED, NORM, 0, 0, 0>(a, bh, smem, sTot, sTrip, sSS, [&](float *lds) {
        redo_sequence<OUT_BF16, OWNKEY>((const ForwardArgs *)__builtin_amdgcn_kernarg_segment_ptr(), bh, lds);
    });
}

}  // namespace


hipError_t launch_forward_gated_ws(const ForwardArgs &a, hipStream_t s)
{
    if (a.d != D || a.io_dtype != LASAD_BF16 || a.n_tokens < 1 || !a.lam) return hipErrorInvalidValue;
    if (a.fused_act && a.k) return hipErrorInvalidValue;
    const int64_t n_seq = (int64_t)a.B * a.Hh;
    if (n_seq > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)n_seq), block(kWsThreads);
    const bool out16 = a.out_dtype == LASAD_BF16;
#define LASAD_GWS_LAUNCH(K, F, N) do { \
        if (out16) hipLaunchKernelGGL((forward_gated_ws_kernel<1, K, F, N>), grid, block, 0, s, a); \
        else hipLaunchKernelGGL((forward_gated_ws_kernel<0, K, F, N>), grid, block, 0, s, a); } while (0)
    if (a.norm) {                      // (the norm comes with the fused activations only: the layer of Algorithm 1)
        if (!a.fused_act) return hipErrorInvalidValue;
        LASAD_GWS_LAUNCH(0, 1, 1);
    } else {
        if (a.fused_act) LASAD_GWS_LAUNCH(0, 1, 0);
        else if (a.k) LASAD_GWS_LAUNCH(1, 0, 0);
        else LASAD_GWS_LAUNCH(0, 0, 0);
    }
#undef LASAD_GWS_LAUNCH
    return hipGetLastError();
}

}  // namespace lasad
