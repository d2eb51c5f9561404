/*
 * liblasad -- linear attention with Spatial-Aware Decay (SAD) for AMD MI355X (gfx950).
 *
 * C ABI of the hot path of "Autoregressive Image Generation with Linear
 * Complexity: A Spatial-Aware Decay Perspective" (LASAD): causal linear
 * attention over an H x W grid of image tokens flattened in raster order, with a
 * per-head base decay gamma_h that is switched off (factor 1) at row-boundary
 * positions, so that the decay between two tokens follows their true
 * (row, column) locations.
 *
 * Notation.  Grid H x W (the paper's h x w, Section 3.1), N = H*W, 1-indexed
 * raster position t = r*W + c + 1 for 0-indexed row r and column c.  Head dim d
 * (dk = dv = d; Section 3.4: s_t in R^{d x d}).  Per-head scalar base decay
 * gamma_h in [0, 1] (the constant-lambda case of Section 3.3).
 *
 *   lambda_t = 1        if t is a boundary position of the chosen rule,
 *            = gamma_h  otherwise                     (Section 3.4, 2nd equation;
 *                                                      Algorithm 1 boundary branch)
 *   s_t = lambda_t s_{t-1} + k_t v_t^T,   o_t^T = q_scale * q_t^T s_t
 *                                                     (Section 3.4, 1st equation)
 *
 * Conventions for every entry point
 *  - All data pointers are DEVICE pointers unless stated otherwise.  The caller
 *    owns every buffer; the library allocates no device memory and keeps no
 *    state between calls.
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *    the default stream).  No call synchronises; buffers must stay alive until
 *    the stream has run the work.
 *  - Return value: LASAD_OK or an error code.  Arguments are validated on the
 *    host before anything is launched; nothing is launched on error.  A
 *    human-readable reason is available from lasad_last_error().
 *  - gfx950 only.  There is no CPU path.
 *
 * Environment variables (test hooks, read once per process at the first call that needs them; none
 * changes a result beyond rounding, each forces a kernel the launcher would otherwise pick by size):
 *   LASAD_WS=0|8|12        scalar-decay forward, full pass: four-, eight- or twelve-wave workgroups
 *   LASAD_SPLIT=1|2        twelve-wave kernel: whole sequences | two workgroups per sequence
 *   LASAD_WS_MULTI=8|12    merged backward launch: eight- or twelve-wave workgroups
 *   LASAD_GATED_WS=0|1     vector-decay forward: four- or twelve-wave workgroups
 *   LASAD_GATED_BWD=walk   vector-decay backward: fp32 token-serial walks instead of the chunked passes
 *   LASAD_SCAN=0           fp32 head dim 64: the generic recurrence kernel instead of the scan kernel
 *   LASAD_FORCE_GENERIC=1  bf16 head dim 64: the fp32 kernels instead of the matrix-core kernels
 */
#ifndef LASAD_H
#define LASAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LASAD_OK = 0,
    LASAD_ERR_INVALID_ARG = 1,   /* null pointer, bad size, bad enum, misaligned pointer */
    LASAD_ERR_UNSUPPORTED = 2,   /* valid request the library has no kernel for */
    LASAD_ERR_WORKSPACE = 3,     /* workspace missing or smaller than the size query says */
    LASAD_ERR_HIP = 4            /* the HIP runtime refused the launch */
} lasad_status_t;

typedef enum { LASAD_F32 = 0, LASAD_BF16 = 1 } lasad_dtype_t;

/* Which positions get lambda_t = 1. */
typedef enum {
    LASAD_RESET_LAST_COL = 0,    /* the paper's rule: t mod W == 0, the last token of a row */
    LASAD_RESET_FIRST_COL = 1,   /* (t-1) mod W == 0, the first token of a row            */
    LASAD_RESET_NONE = 2         /* plain 1-D decay (Section 3.3), no boundary             */
} lasad_boundary_t;

/* Element strides of a [B, n_tokens, Hh, d] tensor; the stride of d is 1.
 * [B, N, Hh, d] contiguous: {N*Hh*d, Hh*d, d};  [B, Hh, N, d] contiguous: {Hh*N*d, d, N*d}. */
typedef struct {
    int64_t stride_b;
    int64_t stride_n;
    int64_t stride_h;
} lasad_layout_t;

/*
 * Decay table (Section 3.4, second equation; Algorithm 1 boundary branch).
 *   gamma      [n_heads] fp32, device.
 *   lambda_out [n_heads, n_tokens] fp32, device, or NULL: lambda_out[h, i] is the
 *              factor of position t = start_pos + 1 + i: the bits of gamma[h]
 *              copied unchanged, or exactly 1.0f.
 *   cum_exp_out [n_tokens + 1] int32, device, or NULL: cum_exp_out[i] =
 *              E(start_pos + i) where E(t) is the number of non-boundary positions
 *              among 1..t, so that prod_{s=j+1..i} lambda_s = gamma^(E(i) - E(j)).
 *   start_pos  tokens of the grid already consumed, 0 <= start_pos,
 *              start_pos + n_tokens <= grid_h * grid_w.  n_tokens may be 0.
 */
int lasad_decay_factors(const float *gamma, int n_heads, int grid_h, int grid_w,
                        int start_pos, int n_tokens, int boundary_mode,
                        float *lambda_out, int32_t *cum_exp_out, void *hip_stream);

/* Bytes of device workspace lasad_forward_chunked can use for these sizes (may be 0).  With
 * few, long sequences the bf16 d = 64 kernel cuts every sequence into segments that are
 * processed by different workgroups; the per-segment partial states live here. */
size_t lasad_forward_workspace_bytes(int B, int n_heads, int n_tokens, int d, int io_dtype);

/*
 * Chunked parallel forward (prefill / teacher-forced pass) over positions
 * start_pos+1 .. start_pos+n_tokens of every (batch, head) sequence.  Computes
 * exactly what the recurrence of Section 3.4 gives, chunk by chunk: inside a
 * chunk the decay-masked (Q K^T (.) D) V product, across chunks a d x d state.
 *
 *   q, k, v   [B, n_tokens, n_heads, d] with strides `qkv_layout`, type io_dtype.
 *   o         same logical shape with strides `o_layout`, type out_dtype; must not
 *             alias q, k or v.
 *   io_dtype  LASAD_F32 (then out_dtype must be LASAD_F32) or LASAD_BF16 (out_dtype
 *             LASAD_BF16 or LASAD_F32).  Accumulation is fp32 in every case.
 *   d         32, 64 or 128 (generic kernel); bf16 with d = 64 takes the MFMA kernel.
 *   gamma     [n_heads] fp32, each in [0, 1].  The matrix-core kernel factorises the in-chunk decay, which needs
 *             gamma > 0.5; a head with a smaller decay is walked token by token in fp32 inside the same launch
 *             (same results, about six times the time for that head's sequences).
 *   state_in  [B, n_heads, d, d] fp32, S[i][j] = sum_t (decay) k_t[i] v_t[j] (dv
 *             contiguous), the state after position start_pos; NULL means zeros.
 *   state_out [B, n_heads, d, d] fp32 or NULL; may equal state_in.
 *   workspace device scratch of at least lasad_forward_workspace_bytes(...) bytes, 16-byte
 *             aligned, contents irrelevant on entry and undefined on return; a smaller
 *             non-NULL workspace is LASAD_ERR_WORKSPACE.  NULL is allowed: the call then
 *             walks every sequence with one workgroup (same results up to rounding,
 *             slower when there are fewer sequences than the GPU has compute units).
 * Pointers must be aligned to 16 bytes and strides multiples of 8 elements for the
 * bf16 kernels (4 for fp32).  n_tokens may be 0 (then state_out = state_in).
 */
int lasad_forward_chunked(const void *q, const void *k, const void *v, void *o,
                          const lasad_layout_t *qkv_layout, const lasad_layout_t *o_layout,
                          int io_dtype, int out_dtype,
                          int B, int n_heads, int d, int grid_h, int grid_w,
                          int start_pos, int n_tokens,
                          const float *gamma, int boundary_mode, float q_scale,
                          const float *state_in, float *state_out,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * lasad_forward_chunked for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments and results as lasad_forward_chunked, without the workspace pair: the
 * per-segment partial states of the segment plan live in an array that is part of the loaded
 * library (lasad_forward_static_scratch_bytes() = 8 MiB per GPU, held until the process ends;
 * every size the segment plan can ask for fits, a larger request would be LASAD_ERR_WORKSPACE).
 * The call allocates nothing and synchronises nothing.  Every segment state that a call reads
 * is written earlier by the same call, so nothing is cleared between calls; but all calls on
 * one GPU share the one array: calls that may run at the same time on one GPU (different
 * streams, different threads) race on it and must use lasad_forward_chunked with workspaces of
 * their own.  Calls on one stream are ordered and safe.
 */
size_t lasad_forward_static_scratch_bytes(void);
int lasad_forward_chunked_static(const void *q, const void *k, const void *v, void *o,
                                 const lasad_layout_t *qkv_layout, const lasad_layout_t *o_layout,
                                 int io_dtype, int out_dtype,
                                 int B, int n_heads, int d, int grid_h, int grid_w,
                                 int start_pos, int n_tokens,
                                 const float *gamma, int boundary_mode, float q_scale,
                                 const float *state_in, float *state_out, void *hip_stream);

/*
 * Recurrent decode step (Algorithm 1 loop body; Section 3.4 first equation):
 * one token for every (batch, head):  S <- lambda S + k v^T,  o = q_scale * S^T q
 * with lambda = 1 if `pos` is a boundary position, else gamma[h].
 *   q, k, v   [B, n_heads, d] contiguous, type io_dtype; o same shape, out_dtype.
 *   pos       0-indexed raster index of THIS token (t = pos + 1), 0 <= pos < H*W.
 *   state     [B, n_heads, d, d] fp32, dv contiguous, updated IN PLACE.
 *   d         32, 64 or 128.
 */
int lasad_decode_step(const void *q, const void *k, const void *v, void *o,
                      int io_dtype, int out_dtype, int B, int n_heads, int d,
                      int grid_h, int grid_w, int pos,
                      const float *gamma, int boundary_mode, float q_scale,
                      float *state, void *hip_stream);

/*
 * The same decode step from a key / value cache instead of the d x d state, for the first
 * positions of a sequence that started from a zero state at position 0: the recurrence unrolled,
 *     o = q_scale sum_{j<=pos} lambda_{j+1} .. lambda_pos (q . k_j) v_j     (Section 3.4, first equation),
 * reads (pos + 1) rows of k and v where the state form moves the whole fp32 state (the memory
 * trade Section 1 describes for a growing cache), which is less traffic while pos + 1 < d for
 * fp32 rows (2 d for bf16: the first 128 positions at d = 64).  This step's k and v are appended to the caches (row pos) by the call.
 *   q, k, v          [B, n_heads, d] contiguous, io_dtype; o same shape, out_dtype.
 *   k_cache, v_cache [B, n_heads, cache_tokens, d] contiguous, io_dtype, owned by the caller; rows
 *                    0 .. pos-1 must hold the earlier steps' k and v; pos < cache_tokens.
 *   d                32, 64 or 128.
 * To continue with lasad_decode_step, build the state once with lasad_forward_chunked over the
 * cached rows (layout strides {n_heads*cache_tokens*d, d, cache_tokens*d}, state_out).
 */
int lasad_decode_step_cached(const void *q, const void *k, const void *v, void *o,
                             void *k_cache, void *v_cache, int cache_tokens,
                             int io_dtype, int out_dtype, int B, int n_heads, int d,
                             int grid_h, int grid_w, int pos,
                             const float *gamma, int boundary_mode, float q_scale,
                             void *hip_stream);

/*
 * lasad_decode_step_cached for the vector decay (Section 3.4 as written; Algorithm 1): the recurrence of
 * lasad_decode_step_gated unrolled from a zero state at position 0,
 *     o = q_scale sum_{j<=pos} [ sum_c q[c] (l_{j+1}[c] .. l_pos[c]) k_j[c] ] v_j,   l_s = 1 at a boundary position,
 * from caches of the gate rows and of v (and of k with an own key).  With the tied key (k, k_cache NULL:
 * k_j = 1 - lambda_j from the cached base gate) a cached token is two rows, as for the scalar decay, so the
 * form moves fewer bytes than the state for the same first positions.  This step's rows are appended (row pos).
 *   q, lam, k, v                 [B, n_heads, d] contiguous, io_dtype; o same shape, out_dtype.
 *   lam_cache, k_cache, v_cache  [B, n_heads, cache_tokens, d] contiguous, io_dtype, owned by the caller; rows
 *                                0 .. pos-1 must hold the earlier steps' rows; pos < cache_tokens.
 *   d                            32, 64 or 128.
 * To continue with lasad_decode_step_gated, build the state once with lasad_forward_gated over the cached rows
 * (state_out).
 */
int lasad_decode_step_gated_cached(const void *q, const void *lam, const void *k, const void *v, void *o,
                                   void *lam_cache, void *k_cache, void *v_cache, int cache_tokens,
                                   int io_dtype, int out_dtype, int B, int n_heads, int d,
                                   int grid_h, int grid_w, int pos, int boundary_mode, float q_scale,
                                   void *hip_stream);

/*
 * Vector, data-dependent decay: the recurrence exactly as Section 3.4 / Algorithm 1 write it.
 * Every token carries a decay vector lambda_t in [0, 1]^d over the key channels,
 *     s_t = diag(lambda_t^spatial) s_{t-1} + k_t v_t^T,   o_t^T = q_scale * q_t^T s_t,
 * lambda_t^spatial = 1 on every channel at a boundary position and lambda_t elsewhere.
 *   lam   [B, n_tokens, n_heads, d], same strides and type as q (the post-sigmoid gate).
 *   k     same shape, or NULL: then the key is tied to the base decay, k_t = 1 - lambda_t
 *         (Section 3.4 "base decay factor" equation; the key keeps the base lambda_t also
 *         at a boundary, Algorithm 1 sets it before the override).
 * Everything else as in lasad_forward_chunked.  bf16 storage with d = 64 runs a chunked
 * matrix-core kernel; fp32 storage and other head dims walk each sequence with the fp32
 * recurrence on the vector ALUs (fp32 state).  No workspace is needed.
 */
int lasad_forward_gated(const void *q, const void *lam, const void *k, const void *v, void *o,
                        const lasad_layout_t *in_layout, const lasad_layout_t *o_layout,
                        int io_dtype, int out_dtype,
                        int B, int n_heads, int d, int grid_h, int grid_w,
                        int start_pos, int n_tokens, int boundary_mode, float q_scale,
                        const float *state_in, float *state_out, void *hip_stream);

/*
 * Decode step of the vector-decay recurrence (Algorithm 1 loop body as written): one token for
 * every (batch, head): row i of S is scaled by lambda[i] (1 at a boundary position), then
 * S += k v^T with k = 1 - lambda when k is NULL, and o = q_scale * S^T q.
 *   q, lam, k (or NULL), v  [B, n_heads, d] contiguous; state [B, n_heads, d, d] fp32 in place.
 */
int lasad_decode_step_gated(const void *q, const void *lam, const void *k, const void *v, void *o,
                            int io_dtype, int out_dtype, int B, int n_heads, int d,
                            int grid_h, int grid_w, int pos, int boundary_mode, float q_scale,
                            float *state, void *hip_stream);

/*
 * The loop body of Algorithm 1 between its two Linear maps, fused around the vector-decay
 * recurrence (head dim 64 for the forward):
 *     q = SiLU(q_pre),  lambda = sigmoid(z),  k = 1 - lambda,  the recurrence of
 *     lasad_forward_gated / lasad_decode_step_gated,  o = Norm(o).
 * Norm is not specified further by the paper; it is taken as a root-mean-square normalisation
 * over the d channels of each head, o / sqrt(mean_c(o^2) + norm_eps), times norm_weight.
 *   q_pre, z      pre-activation query and gate, layout and type as q and lam of the gated calls.
 *   norm_weight   [n_heads, d] fp32 (device, 16-byte aligned), or NULL for ones.
 *   norm_eps      >= 0; a negative value switches the normalisation off (activations only).
 * The activations are evaluated in fp32 on load and nothing is rounded between the steps.
 * Everything else as in the gated calls.
 */
int lasad_forward_layer(const void *q_pre, const void *z, const void *v, void *o,
                        const lasad_layout_t *in_layout, const lasad_layout_t *o_layout,
                        int io_dtype, int out_dtype,
                        int B, int n_heads, int d, int grid_h, int grid_w,
                        int start_pos, int n_tokens, int boundary_mode, float q_scale,
                        const float *norm_weight, float norm_eps,
                        const float *state_in, float *state_out, void *hip_stream);
int lasad_decode_step_layer(const void *q_pre, const void *z, const void *v, void *o,
                            int io_dtype, int out_dtype, int B, int n_heads, int d,
                            int grid_h, int grid_w, int pos, int boundary_mode, float q_scale,
                            const float *norm_weight, float norm_eps,
                            float *state, void *hip_stream);

/*
 * Decode step with one raster position per batch row (continuous batching: the sequences of a
 * batch are at different points of their images, Section 3.1 raster order; each row's decay is
 * switched off by the boundary rule of Section 3.4 at ITS position).
 *   pos_rows  [B] int32 (device): 0-indexed raster position of the token each row consumes.  A
 *             row whose entry is outside 0 .. grid_h*grid_w-1 (say -1) is inactive: its states are
 *             left untouched and its output rows are zero.
 *   lam       vector decay [B, n_heads, d] (then gamma must be NULL, k may be NULL for the tied
 *             key), or NULL for the per-head scalar decay (then gamma [n_heads] and k are needed).
 * Everything else as in lasad_decode_step / lasad_decode_step_gated.
 */
int lasad_decode_step_rows(const void *q, const void *lam, const void *k, const void *v, void *o,
                           int io_dtype, int out_dtype, int B, int n_heads, int d,
                           int grid_h, int grid_w, const int32_t *pos_rows,
                           const float *gamma, int boundary_mode, float q_scale,
                           float *state, void *hip_stream);

/*
 * Backward pass of lasad_forward_chunked for a call that starts from a zero state and whose
 * final state is not used (a whole teacher-forced sequence, the training setting of Section 4.1):
 * given d_o = dL/do, the gradients of the Section 3.4 recurrence
 *     dq_i = q_scale sum_{j<=i} M[i][j] (d_o_i . v_j) k_j
 *     dk_j = q_scale sum_{i>=j} M[i][j] (d_o_i . v_j) q_i
 *     dv_j = q_scale sum_{i>=j} M[i][j] (q_i . k_j) d_o_i,      M[i][j] = prod_{s=j+1..i} lambda_s
 * and dgamma[h] = dL/dgamma_h, gamma_h being the decay of every non-boundary position of head h
 * (second equation of Section 3.4), summed over the batch.
 *   q, k, v, d_o   [B, n_tokens, n_heads, d] views sharing in_layout and io_dtype (device).
 *   dq, dk, dv     same logical shape, grad_layout, grad_dtype (fp32, or bf16 with bf16 inputs);
 *                  overwritten; must not alias the inputs or each other.
 *   dgamma         [n_heads] fp32, overwritten.  Needs gamma > 0 (it is formed from d/dlog gamma);
 *                  for gamma = 0 the entry is inf or NaN.
 *   workspace      device memory of at least lasad_backward_workspace_bytes(...) bytes, 256-byte
 *                  aligned, owned by the caller, free for reuse when the call's work on the stream
 *                  has finished.  Required (LASAD_ERR_WORKSPACE if NULL or too small).
 * Asynchronous on hip_stream; no allocation, no synchronisation.  Results are deterministic
 * (fixed summation order).
 */
size_t lasad_backward_workspace_bytes(int B, int n_heads, int n_tokens, int d, int io_dtype);
int lasad_backward_chunked(const void *q, const void *k, const void *v, const void *d_o,
                           void *dq, void *dk, void *dv, float *dgamma,
                           const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                           int io_dtype, int grad_dtype,
                           int B, int n_heads, int d, int grid_h, int grid_w,
                           int start_pos, int n_tokens,
                           const float *gamma, int boundary_mode, float q_scale,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * lasad_backward_chunked through carried states: the call covers tokens start_pos+1 .. start_pos+n_tokens of
 * sequences whose state before the first token is state_in, and the loss may also depend on the state after
 * the last token (the Section 3.4 recurrence differentiated with s_0 given; what one part of a sequence split
 * over several calls, or over several GPUs, hands to its neighbours).
 *   state_in     [B, n_heads, d, d] fp32 as in lasad_forward_chunked, or NULL (zeros).
 *   d_state_out  [B, n_heads, d, d] fp32: dL/d(final state of the forward call), or NULL (zeros).
 *   d_state_in   [B, n_heads, d, d] fp32, overwritten with dL/d(state_in), or NULL; must not alias the other two.
 * dq, dk, dv then include the terms through state_in and d_state_out, and dgamma includes the dependence of
 * the final state on the decay.  Two chained calls over a split sequence (the second call's d_state_in given
 * to the first as d_state_out) reproduce one call over the whole up to rounding.  With n_tokens = 0 dgamma is
 * zero and d_state_in = d_state_out.  Workspace: lasad_backward_carried_workspace_bytes(...) bytes.
 * Everything else as in lasad_backward_chunked.
 */
size_t lasad_backward_carried_workspace_bytes(int B, int n_heads, int n_tokens, int d, int io_dtype);
int lasad_backward_chunked_carried(const void *q, const void *k, const void *v, const void *d_o,
                                   const float *state_in, const float *d_state_out,
                                   void *dq, void *dk, void *dv, float *dgamma, float *d_state_in,
                                   const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                                   int io_dtype, int grad_dtype,
                                   int B, int n_heads, int d, int grid_h, int grid_w,
                                   int start_pos, int n_tokens,
                                   const float *gamma, int boundary_mode, float q_scale,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward pass of lasad_forward_gated (vector decay, Section 3.4 / Algorithm 1) for a call that
 * starts from a zero state and whose final state is not used: given d_o = dL/do, with
 * l_t = lambda_t^spatial (1 at a row boundary) and D[i][j][c] = prod_{s=j+1..i} l_s[c],
 *     dq_i[c] = q_scale sum_{j<=i} (d_o_i . v_j) k_j[c] D[i][j][c]
 *     dk_j[c] = q_scale sum_{i>=j} (d_o_i . v_j) q_i[c] D[i][j][c]
 *     dv_j    = q_scale sum_{i>=j} (sum_c q_i[c] k_j[c] D[i][j][c]) d_o_i
 * and dlam, the gradient for the lambda INPUT: through the decay where the position is not a
 * boundary (nothing at a boundary, where the applied decay is the constant 1, and nothing at the
 * first token, whose decay multiplies the zero state), and, with the tied key (k NULL,
 * k_t = 1 - lambda_t), through the key as well (- dk_t).
 *   q, lam, k, v, d_o   [B, n_tokens, n_heads, d] views sharing in_layout and io_dtype (device);
 *                       k NULL: tied key.  Head dim 32, 64 or 128 (64 with bf16 inputs: the matrix-core passes;
 *                       otherwise fp32 token-serial walks).
 *   dq, dlam, dk, dv    same logical shape, grad_layout, grad_dtype (fp32, or bf16 with bf16
 *                       inputs); overwritten; dk must be given exactly when k is; no aliasing.
 *   lambda must be > 0 wherever it is applied (dlam comes from d/dlog lambda; a zero decay gives
 *   inf or NaN there, and precision degrades like 1 / lambda for very small decays).
 *   workspace           device memory of at least lasad_backward_gated_workspace_bytes(...) bytes,
 *                       256-byte aligned, owned by the caller (LASAD_ERR_WORKSPACE if too small).
 * Asynchronous on hip_stream; no allocation, no synchronisation; deterministic.
 */
size_t lasad_backward_gated_workspace_bytes(int B, int n_heads, int n_tokens, int d);
int lasad_backward_gated(const void *q, const void *lam, const void *k, const void *v, const void *d_o,
                         void *dq, void *dlam, void *dk, void *dv,
                         const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                         int io_dtype, int grad_dtype,
                         int B, int n_heads, int d, int grid_h, int grid_w,
                         int start_pos, int n_tokens, int boundary_mode, float q_scale,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * lasad_backward_gated through carried states (see lasad_backward_chunked_carried): state_in is the state
 * before the call's first token, d_state_out = dL/d(final state), d_state_in receives dL/d(state_in) =
 * diag(l_1) g_1; each may be NULL.  dq, dlam, dk, dv include the terms through both states; in particular
 * the decay of the first token now has a gradient (it multiplies state_in), and every decay of the call
 * gains the products that end in the final state.  Workspace:
 * lasad_backward_gated_carried_workspace_bytes(...) bytes.  Everything else as in lasad_backward_gated.
 */
size_t lasad_backward_gated_carried_workspace_bytes(int B, int n_heads, int n_tokens, int d);
int lasad_backward_gated_carried(const void *q, const void *lam, const void *k, const void *v, const void *d_o,
                                 const float *state_in, const float *d_state_out,
                                 void *dq, void *dlam, void *dk, void *dv, float *d_state_in,
                                 const lasad_layout_t *in_layout, const lasad_layout_t *grad_layout,
                                 int io_dtype, int grad_dtype,
                                 int B, int n_heads, int d, int grid_h, int grid_w,
                                 int start_pos, int n_tokens, int boundary_mode, float q_scale,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward pass of lasad_forward_layer (Algorithm 1 between its two Linear maps; Norm as read
 * there: root mean square over the d channels of a head, times norm_weight) for a call that starts
 * from a zero state and whose final state is not used.  Given d_out = dL/d(layer output), the chain
 * rule runs through the normalisation (the recurrence output o is recomputed, not stored by the
 * forward), the recurrence (lasad_backward_gated with the tied key) and the two activations:
 *     dq_pre = dq * SiLU'(q_pre),   dz = dlam * lambda (1 - lambda),   dv,
 *     dweight[h][c] = sum over batch and tokens of d_out * o * rstd.
 *   q_pre, z, v     [B, n_tokens, n_heads, d] views sharing in_layout and io_dtype (device); head dim 64.
 *   d_out           same logical shape and type, its own dout_layout.
 *   dq_pre, dz, dv  same logical shape, grad_layout, grad_dtype (fp32, or bf16 with bf16 inputs);
 *                   overwritten; no aliasing.
 *   norm_weight     [n_heads, d] fp32 or NULL (ones); norm_eps < 0: no normalisation, as in the forward.
 *   dweight         [n_heads, d] fp32 (device), overwritten, or NULL.  Without norm_weight: the gradient at a
 *                   weight of ones; without a normalisation: zeros.
 *   workspace       device memory of at least lasad_backward_layer_workspace_bytes(...) bytes, 256-byte
 *                   aligned, owned by the caller (LASAD_ERR_WORKSPACE if too small).  It holds o in fp32,
 *                   the gradient that enters the recurrence (in the inputs' type, bf16 twice, and WITH THE
 *                   INPUTS' STRIDES, so its size follows the span of in_layout) and the recurrence's own
 *                   workspace.
 * The gate must not saturate to lambda = 0 where a decay is applied (see lasad_backward_gated).
 * Precision: the gradient that enters the recurrence is orthogonal to o, and where the state is
 * close to rank one (the first tokens of a sequence) dq and dz are small differences of larger
 * terms.  With bf16 inputs that gradient therefore crosses the workspace as a bf16 pair hi + lo,
 * both parts used where the cancellation happens; fp32 inputs keep it in fp32.
 * Asynchronous on hip_stream; no allocation, no synchronisation; deterministic.
 */
size_t lasad_backward_layer_workspace_bytes(int B, int n_heads, int n_tokens, int d, int io_dtype,
                                            const lasad_layout_t *in_layout);
int lasad_backward_layer(const void *q_pre, const void *z, const void *v, const void *d_out,
                         void *dq_pre, void *dz, void *dv, float *dweight,
                         const lasad_layout_t *in_layout, const lasad_layout_t *dout_layout,
                         const lasad_layout_t *grad_layout,
                         int io_dtype, int grad_dtype,
                         int B, int n_heads, int d, int grid_h, int grid_w,
                         int start_pos, int n_tokens, int boundary_mode, float q_scale,
                         const float *norm_weight, float norm_eps,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The first part of lasad_backward_layer alone: the gradient d_o = dL/do that leaves the
 * normalisation and enters the recurrence, and dweight.  With gw = d_out * norm_weight,
 *     d_o = rstd gw - o rstd^3 mean_c(gw o),   rstd = (mean_c(o^2) + norm_eps)^(-1/2),
 * o the recurrence output of Algorithm 1 for q_pre, z, v (recomputed here).  norm_eps >= 0.
 *   d_o   [B, n_tokens, n_heads, d], d_o_layout, type d_o_dtype (io_dtype, or LASAD_F32 also with bf16
 *         inputs: the value before its rounding to bf16); overwritten.
 * lasad_backward_layer computes this tensor by the same kernels and feeds it to the recurrence's
 * backward (with bf16 inputs together with what the rounding to bf16 left over, as a second
 * bf16 tensor); the latter alone is lasad_backward_layer with norm_eps < 0 and d_out := d_o.
 * Workspace and everything else as in lasad_backward_layer.
 */
int lasad_backward_layer_norm(const void *q_pre, const void *z, const void *v, const void *d_out,
                              void *d_o, float *dweight,
                              const lasad_layout_t *in_layout, const lasad_layout_t *dout_layout,
                              const lasad_layout_t *d_o_layout, int io_dtype, int d_o_dtype,
                              int B, int n_heads, int d, int grid_h, int grid_w,
                              int start_pos, int n_tokens, int boundary_mode, float q_scale,
                              const float *norm_weight, float norm_eps,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* Reason for the last non-OK status returned on this thread (static storage). */
const char *lasad_last_error(void);

/* Library version string, e.g. "lasad 0.1 gfx950". */
const char *lasad_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LASAD_H */
