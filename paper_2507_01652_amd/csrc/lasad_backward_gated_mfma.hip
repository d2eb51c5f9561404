// Chunked matrix-core passes of the vector-decay backward (bf16 inputs, head dim 64): the
// twelve-wave workgroup of lasad_gated_ws_body.h (output / state / loader waves, doubled LDS
// tiles, one barrier per chunk, the forward's operand preparation and range rule) for the two
// kinds of pass the gradients need (lasad_backward_gated.hip has the derivation):
//
// ROW pass (dv): the forward itself over the reversed sequence, query := the key of the token
//   (1 - lambda if tied), key := q, value := d_o, decay of step m := lambda of step m - 1.
//
// COL pass (dq; dk over the reversed sequence): with A_i the chunk-local running product of the
//   decay and Z~_j = z_j / A_j (z the key for dq, q for dk),
//       out_i = q_scale A_i (.) [ S x_i + sum_{j<=i} (x_i . y_j) Z~_j ],   S <- diag(A_end) (S + Z~^T Y)
//   (x, y: d_o and v for dq, v and d_o for dk).  The state and its update are those of the forward
//   (the state waves are unchanged); the output waves take the scores from the plain x and y
//   (one MFMA per step, no decay inside), contract them with Z~ (bf16 hi + lo on both sides: three
//   MFMAs) and the state with x over the VALUE index (S^T tiles read through the transposing LDS
//   load), and scale the fp32 tile by q_scale A_i, which the loader waves stage as "Q~ of a query
//   of ones".  x comes straight from global memory in operand layout, one chunk ahead.  Output fp32.
//
// A chunk that leaves the range of the factorisation sends the workgroup to the token-serial walk
// of the same pass (lasad_scan.h with operand roles).
#include "lasad_gated_ws_body.h"

namespace lasad {

namespace {

using namespace gated;

// The token-serial walk of a pass, out of line.  It is handed the arguments where the launch put
// them (the kernel-argument segment): references to the kernel's by-value parameter, or copies,
// would make every thread of every launch write them to its stack first.
template <int OUT_BF16, int COL>
__device__ __noinline__ void redo_roles(const ForwardArgs *a, const scan::ScanRoles *r, int bh, float *lds)
{
    if (COL) scan::scan_sequence<1, 0, scan::ROLES_COL, 64>(*a, bh, 0, lds, r);
    else scan::scan_sequence<1, OUT_BF16, scan::ROLES_ROW, 64>(*a, bh, 0, lds, r);
}

// One pass for sequence bh by the calling twelve-wave workgroup; ka, kr: the pass's arguments and
// operand roles in the kernel-argument segment (for the fallback).
template <int OUT_BF16, int OWNKEY, int FUSED, int SHIFT, int QMODE, int COL, int XLO = 0, int YLO = 0>
__device__ __forceinline__ void pass_body(const ForwardArgs &a, const ForwardArgs *ka, const scan::ScanRoles *kr, int bh,
                                          uint16_t *smem, float (*sTot)[D], int (*sTrip)[4])
{
    gated_ws_body<OUT_BF16, OWNKEY, FUSED, 0, SHIFT, QMODE, COL, XLO, YLO>(a, bh, smem, sTot, sTrip, nullptr, [&](float *lds) {
        redo_roles<OUT_BF16, COL>(ka, kr, bh, lds);
    });
}

struct PassSet {
    ForwardArgs a[3];              // dq, dv, dk: the pass's operands in the forward's fields
    scan::ScanRoles roles[3];      // the same passes for the token-serial walk (range fallback)
};

// The three passes of a call in one launch.  Workgroups come in groups of 8 sequences x 3 passes,
// a sequence's passes 8 workgroup ids apart: they start together on the same XCD (ids go round
// the 8 XCDs) and share what they both read through its L2 (dv and dk walk the same q, d_o and
// lambda rows in the same order).  TIED: the key is 1 - lambda.  FUSED (with TIED): the layer's
// backward: the q and lambda tensors hold Algorithm 1's pre-activation query and gate logits, and
// d_o comes as a bf16 pair hi + lo, both parts used in every pass (x of the dq pass, y of the dk pass, the value
// operand of the dv pass: one more MFMA per score or product step and per state term).  d_o is
// orthogonal to the recurrence output, which makes dq and dk small differences of larger terms
// early in a sequence; a single bf16 there costs up to 0.15 of the RMS in single elements, and in dv, which for
// the last tokens of a sequence is a multiple of a single d_o row, up to 0.02.
template <int OUT_BF16, int TIED, int FUSED = 0>
__global__ void __launch_bounds__(kWsThreads, 1)
backward_gated_passes_kernel(PassSet ps)
{
    constexpr int kScanFloats = scan::lds_floats<scan::ROLES_ROW>();
    static_assert(2 * kSetHalfs * 2 >= kScanFloats * 4, "the fallback needs the LDS block");
    __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kSetHalfs];
    __shared__ __attribute__((aligned(16))) float sTot[2][D];  // A_end per key channel, by chunk parity
    __shared__ __attribute__((aligned(16))) int sTrip[2][4];   // range flag of each loader wave, by barrier parity
    const int grp = blockIdx.x / 24, r = blockIdx.x - grp * 24;
    const int pass = r >> 3, bh = grp * 8 + (r & 7);
    if (bh >= ps.a[0].B * ps.a[0].Hh) return;                  // (the last group may be partly empty)
    const PassSet *kp = (const PassSet *)__builtin_amdgcn_kernarg_segment_ptr();
    if (pass == 0) pass_body<0, TIED ? 0 : 1, FUSED, 0, 1, 1, FUSED, 0>(ps.a[0], &kp->a[0], &kp->roles[0], bh, smem, sTot, sTrip);
    else if (pass == 1) pass_body<OUT_BF16, 1, FUSED, 1, TIED ? 2 : 0, 0, 0, FUSED>(ps.a[1], &kp->a[1], &kp->roles[1], bh, smem, sTot, sTrip);
    else pass_body<0, 1, FUSED, 1, 1, 1, 0, FUSED>(ps.a[2], &kp->a[2], &kp->roles[2], bh, smem, sTot, sTrip);
}

}  // namespace

// The three passes of the vector-decay backward with the matrix-core kernel, one launch.
// a[0..2], roles[0..2]: dq (column pass, forward order), dv (row pass, reversed; its query tensor
// is lambda itself when tied), dk (column pass, reversed), as lasad_backward_gated.hip sets them up.
hipError_t launch_backward_gated_passes(const ForwardArgs *a, const scan::ScanRoles *roles, bool tied, hipStream_t s)
{
    if (a[0].d != D || a[0].io_dtype != LASAD_BF16 || a[0].n_tokens < 1) return hipErrorInvalidValue;
    const int64_t n_seq = (int64_t)a[0].B * a[0].Hh;
    if ((n_seq + 7) / 8 * 24 > 0x7fffffff) return hipErrorInvalidValue;
    PassSet ps;
    for (int i = 0; i < 3; ++i) { ps.a[i] = a[i]; ps.roles[i] = roles[i]; }
    const dim3 grid((unsigned)((n_seq + 7) / 8 * 24)), block(kWsThreads);
    const bool out16 = a[1].out_dtype == LASAD_BF16;
    if (a[0].fused_act) {
        if (!tied || !a[0].q_lo || !a[1].v_lo || !a[2].v_lo) return hipErrorInvalidValue;
        if (out16) hipLaunchKernelGGL((backward_gated_passes_kernel<1, 1, 1>), grid, block, 0, s, ps);
        else hipLaunchKernelGGL((backward_gated_passes_kernel<0, 1, 1>), grid, block, 0, s, ps);
    } else if (tied) {
        if (out16) hipLaunchKernelGGL((backward_gated_passes_kernel<1, 1>), grid, block, 0, s, ps);
        else hipLaunchKernelGGL((backward_gated_passes_kernel<0, 1>), grid, block, 0, s, ps);
    } else {
        if (out16) hipLaunchKernelGGL((backward_gated_passes_kernel<1, 0>), grid, block, 0, s, ps);
        else hipLaunchKernelGGL((backward_gated_passes_kernel<0, 0>), grid, block, 0, s, ps);
    }
    return hipGetLastError();
}

}  // namespace lasad
