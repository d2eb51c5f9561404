/*
 * LASAD CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 implementation of linear attention with Spatial-Aware
 * Decay (SAD) written directly from the paper's Section 3.4 recurrence and
 * Algorithm 1.  Only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it; it shares no code with the HIP library and the HIP library
 * never calls it.
 *
 * Reading used for the decay (one scalar base decay gamma_h per head, the
 * "constant lambda" case of Section 3.3, with the row-boundary rule of
 * Section 3.4 on top):
 *     lambda_t = 1        if t is a row-boundary position
 *              = gamma_h  otherwise,                 t = 1..N (1-indexed)
 * where the paper's rule (Section 3.4, second equation; Algorithm 1) makes
 * t a boundary when t mod w == 0 (the last token of a grid row).  Two other
 * rules are selectable for comparison: boundary at the first token of a row
 * ((t-1) mod w == 0) and no boundary at all (Section 3.3 plain decay).
 *
 * All tensors here are dense, fp64, in [B][Hh][n][d] order ("head-major");
 * states are [B][Hh][dk][dv] with dv contiguous: S[i][j] = sum_t k_t[i] v_t[j].
 *
 * Gradients (lasad_oracle_backward, lasad_oracle_dgamma, lasad_oracle_gated_backward)
 * differentiate the same recurrences step by step in reverse.
 *
 * Every function below is pinned by the CPU test-suite against values fixed by
 * the paper's equations (hand-worked recurrences, geometric-series closed
 * forms, the gamma = 1 reduction to plain causal linear attention of
 * Section 3.2, brute force); none is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_RESET_LAST_COL = 0, ORACLE_RESET_FIRST_COL = 1, ORACLE_RESET_NONE = 2 };

/* Section 3.4, second equation / Algorithm 1 "if (t mod w) = 0": is the
 * 1-indexed raster position t one where the decay is switched off? */
static int is_boundary(int64_t t, int grid_w, int mode)
{
    if (mode == ORACLE_RESET_LAST_COL)  return (t % grid_w) == 0;
    if (mode == ORACLE_RESET_FIRST_COL) return ((t - 1) % grid_w) == 0;
    return 0;
}

/*
 * Decay table (Section 3.4 second equation, Algorithm 1 boundary branch).
 *   lam_out[h*n + i]  = lambda of position t = start_pos + 1 + i for head h
 *                       (the fp32 gamma copied unchanged, or exactly 1.0f)
 *   cum_out[i]        = E(start_pos + i), i = 0..n, where E(t) counts the
 *                       positions s in 1..t that are NOT boundaries, so that
 *                       prod_{s=j+1..i} lambda_s = gamma^(E(i) - E(j)).
 * E is obtained by literally walking t = 1, 2, ... and counting.
 * Returns 0, or 1 on invalid arguments.
 */
int lasad_oracle_decay_factors(const float *gamma, int n_heads, int grid_h, int grid_w,
                               int start_pos, int n, int mode,
                               float *lam_out, int32_t *cum_out)
{
    if (!gamma || n_heads < 1 || grid_h < 1 || grid_w < 1 || start_pos < 0 || n < 0) return 1;
    if ((int64_t)start_pos + n > (int64_t)grid_h * grid_w) return 1;
    if (mode < 0 || mode > 2) return 1;
    if (lam_out) {
        for (int h = 0; h < n_heads; ++h)
            for (int i = 0; i < n; ++i) {
                int64_t t = (int64_t)start_pos + 1 + i;
                lam_out[(size_t)h * n + i] = is_boundary(t, grid_w, mode) ? 1.0f : gamma[h];
            }
    }
    if (cum_out) {
        int32_t e = 0;
        if (start_pos == 0) cum_out[0] = 0;
        for (int64_t t = 1; t <= (int64_t)start_pos + n; ++t) {
            if (!is_boundary(t, grid_w, mode)) e += 1;
            if (t >= start_pos) cum_out[t - start_pos] = e;
        }
    }
    return 0;
}

/*
 * Parallel ("full mask") form.  Unrolling s_t = lambda_t s_{t-1} + k_t v_t^T,
 * o_t^T = q_t^T s_t (Section 3.4 first equation) gives
 *     o_i = sum_{j<=i} M[i][j] (q_i . k_j) v_j,   M[i][j] = prod_{s=j+1..i} lambda_s
 * with M[i][i] = 1 (empty product) and M[i][j] = 0 for j > i.  The full n x n
 * M is materialised, then A = q_scale * Q K^T, P = A (.) M, O = P V.
 *
 * With a carried state S0 (the state after the tokens that precede this
 * call) the recurrence adds  (prod_{s=first..i} lambda_s) q_i^T S0  to o_i and
 *     S_out = (prod_{s=first..last} lambda_s) S0 + sum_j M[last][j] k_j v_j^T.
 *
 * lam is [Hh][n] (lambda of the n positions of this call), s0/s_out may be
 * NULL.  Returns 0, 1 on bad arguments, 2 when out of memory.
 */
int lasad_oracle_forward_fullmask(const double *q, const double *k, const double *v,
                                  const double *lam, double q_scale,
                                  const double *s0, double *o, double *s_out,
                                  int B, int n_heads, int n, int d)
{
    if (!q || !k || !v || !lam || !o || B < 1 || n_heads < 1 || n < 0 || d < 1) return 1;
    int status = 0;
    const int64_t n_seq = (int64_t)B * n_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < n_seq; ++bh) {
        const int h = (int)(bh % n_heads);
        const double *lm = lam + (size_t)h * n;
        const double *Q = q + (size_t)bh * n * d, *K = k + (size_t)bh * n * d;
        const double *V = v + (size_t)bh * n * d;
        double *O = o + (size_t)bh * n * d;
        double *M = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * (size_t)(n > 0 ? n : 1));
        double *p = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        double *pre = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        if (!M || !p || !pre) {
#pragma omp atomic write
            status = 2;
            free(M); free(p); free(pre);
            continue;
        }
        /* M[i][j] = lambda_{j+1} * ... * lambda_i, multiplied in increasing s. */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                double m;
                if (j > i) m = 0.0;
                else if (j == i) m = 1.0;
                else m = M[(size_t)(i - 1) * n + j] * lm[i];
                M[(size_t)i * n + j] = m;
            }
        /* pre[i] = lambda_first * ... * lambda_i : what multiplies S0 at step i. */
        for (int i = 0; i < n; ++i) pre[i] = (i == 0 ? 1.0 : pre[i - 1]) * lm[i];

        for (int i = 0; i < n; ++i) {
            for (int j = 0; j < n; ++j) {            /* row i of P = (q_scale Q K^T) (.) M */
                double a = 0.0;
                for (int c = 0; c < d; ++c) a += Q[(size_t)i * d + c] * K[(size_t)j * d + c];
                p[j] = (q_scale * a) * M[(size_t)i * n + j];
            }
            for (int c = 0; c < d; ++c) {            /* row i of O = P V */
                double acc = 0.0;
                for (int j = 0; j < n; ++j) acc += p[j] * V[(size_t)j * d + c];
                O[(size_t)i * d + c] = acc;
            }
            if (s0) {                                /* carried-state term */
                const double *S0 = s0 + (size_t)bh * d * d;
                for (int c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (int r = 0; r < d; ++r) acc += Q[(size_t)i * d + r] * S0[(size_t)r * d + c];
                    O[(size_t)i * d + c] += pre[i] * (q_scale * acc);
                }
            }
        }
        if (s_out) {
            double *S = s_out + (size_t)bh * d * d;
            for (int r = 0; r < d; ++r)
                for (int c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (int j = 0; j < n; ++j)
                        acc += M[(size_t)(n - 1) * n + j] * K[(size_t)j * d + r] * V[(size_t)j * d + c];
                    if (s0) acc += (n > 0 ? pre[n - 1] : 1.0) * s0[(size_t)bh * d * d + (size_t)r * d + c];
                    S[(size_t)r * d + c] = acc;
                }
        }
        free(M); free(p); free(pre);
    }
    return status;
}

/*
 * Sequential form: the loop of Algorithm 1 (recurrence lines only; the
 * projections, activations and Norm of the surrounding layer are outside this
 * path), state kept in fp64.  s_t = lambda_t s_{t-1} + k_t v_t^T, then
 * o_t^T = q_scale * q_t^T s_t (the state that already contains token t).
 * s0 NULL means s_0 = 0; s_out (may alias nothing else) receives s_n.
 */
int lasad_oracle_recurrent(const double *q, const double *k, const double *v,
                           const double *lam, double q_scale,
                           const double *s0, double *o, double *s_out,
                           int B, int n_heads, int n, int d)
{
    if (!q || !k || !v || !lam || !o || B < 1 || n_heads < 1 || n < 0 || d < 1) return 1;
    int status = 0;
    const int64_t n_seq = (int64_t)B * n_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < n_seq; ++bh) {
        const int h = (int)(bh % n_heads);
        double *S = (double *)malloc(sizeof(double) * (size_t)d * d);
        if (!S) {
#pragma omp atomic write
            status = 2;
            continue;
        }
        if (s0) memcpy(S, s0 + (size_t)bh * d * d, sizeof(double) * (size_t)d * d);
        else    memset(S, 0, sizeof(double) * (size_t)d * d);
        for (int t = 0; t < n; ++t) {
            const double l = lam[(size_t)h * n + t];
            const double *qt = q + ((size_t)bh * n + t) * d;
            const double *kt = k + ((size_t)bh * n + t) * d;
            const double *vt = v + ((size_t)bh * n + t) * d;
            double *ot = o + ((size_t)bh * n + t) * d;
            for (int r = 0; r < d; ++r)
                for (int c = 0; c < d; ++c)
                    S[(size_t)r * d + c] = l * S[(size_t)r * d + c] + kt[r] * vt[c];
            for (int c = 0; c < d; ++c) {
                double acc = 0.0;
                for (int r = 0; r < d; ++r) acc += qt[r] * S[(size_t)r * d + c];
                ot[c] = q_scale * acc;
            }
        }
        if (s_out) memcpy(s_out + (size_t)bh * d * d, S, sizeof(double) * (size_t)d * d);
        free(S);
    }
    return status;
}

/*
 * One decode step for every (batch, head): the body of Algorithm 1's loop for
 * a single position whose decay is lam_t[h].  state [B][Hh][d][d] is updated
 * in place; q, k, v, o are [B][Hh][d].
 */
int lasad_oracle_decode_step(const double *q, const double *k, const double *v,
                             const double *lam_t, double q_scale,
                             double *state, double *o, int B, int n_heads, int d)
{
    if (!q || !k || !v || !lam_t || !state || !o || B < 1 || n_heads < 1 || d < 1) return 1;
    const int64_t n_seq = (int64_t)B * n_heads;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < n_seq; ++bh) {
        const double l = lam_t[bh % n_heads];
        double *S = state + (size_t)bh * d * d;
        const double *qt = q + (size_t)bh * d, *kt = k + (size_t)bh * d, *vt = v + (size_t)bh * d;
        for (int r = 0; r < d; ++r)
            for (int c = 0; c < d; ++c)
                S[(size_t)r * d + c] = l * S[(size_t)r * d + c] + kt[r] * vt[c];
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int r = 0; r < d; ++r) acc += qt[r] * S[(size_t)r * d + c];
            o[(size_t)bh * d + c] = q_scale * acc;
        }
    }
    return 0;
}

/*
 * Brute force for tiny inputs: every (i, j) pair separately, the decay
 * product formed by its own loop over s = j+1..i, no table, no state.
 * Single sequence (one batch, one head): q, k, v, o are [n][d], lam is [n].
 */
int lasad_oracle_bruteforce(const double *q, const double *k, const double *v,
                            const double *lam, double q_scale, double *o, int n, int d)
{
    if (!q || !k || !v || !lam || !o || n < 0 || d < 1) return 1;
    for (int i = 0; i < n; ++i)
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int j = 0; j <= i; ++j) {
                double decay = 1.0;
                for (int s = j + 1; s <= i; ++s) decay *= lam[s];
                double dot = 0.0;
                for (int r = 0; r < d; ++r) dot += q[(size_t)i * d + r] * k[(size_t)j * d + r];
                acc += decay * (q_scale * dot) * v[(size_t)j * d + c];
            }
            o[(size_t)i * d + c] = acc;
        }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Vector, data-dependent decay: the recurrence exactly as Section 3.4 / Algorithm 1 state it.
 * Every token carries its own decay vector lambda_t in [0,1]^d over the key channels,
 *     s_t = diag(lambda_t^spatial) s_{t-1} + k_t v_t^T,   o_t^T = q_scale * q_t^T s_t,
 * with lambda_t^spatial = 1 (every channel) at a row-boundary position and lambda_t elsewhere,
 * and with the key tied to the decay, k_t = 1 - lambda_t (Section 3.4, "base decay factor"
 * equation; Algorithm 1 sets k before the boundary override, so k_t keeps the base lambda_t
 * also at a boundary).  When `k` is not NULL it is used instead of 1 - lambda (the gate of GLA
 * with an independent key, Section 4.5).
 * ------------------------------------------------------------------------------------------ */

/*
 * Sequential form (the loop of Algorithm 1), state in fp64.
 *   q, lam, k (or NULL), v, o : [B][Hh][n][d];  s0 / s_out : [B][Hh][d][d] or NULL.
 *   Positions are start_pos+1 .. start_pos+n of a grid of width grid_w under rule `mode`.
 */
int lasad_oracle_gated_recurrent(const double *q, const double *lam, const double *k, const double *v,
                                 double q_scale, const double *s0, double *o, double *s_out,
                                 int B, int n_heads, int n, int d, int grid_w, int start_pos, int mode)
{
    if (!q || !lam || !v || !o || B < 1 || n_heads < 1 || n < 0 || d < 1 || grid_w < 1 || start_pos < 0) return 1;
    if (mode < 0 || mode > 2) return 1;
    int status = 0;
    const int64_t n_seq = (int64_t)B * n_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < n_seq; ++bh) {
        double *S = (double *)malloc(sizeof(double) * (size_t)d * d);
        if (!S) {
#pragma omp atomic write
            status = 2;
            continue;
        }
        if (s0) memcpy(S, s0 + (size_t)bh * d * d, sizeof(double) * (size_t)d * d);
        else    memset(S, 0, sizeof(double) * (size_t)d * d);
        for (int t = 0; t < n; ++t) {
            const size_t off = ((size_t)bh * n + t) * d;
            const int boundary = is_boundary((int64_t)start_pos + 1 + t, grid_w, mode);
            for (int r = 0; r < d; ++r) {
                const double l = lam[off + r];
                const double kr = k ? k[off + r] : 1.0 - l;       /* key from the BASE decay */
                const double ls = boundary ? 1.0 : l;             /* spatial-aware decay     */
                for (int c = 0; c < d; ++c)
                    S[(size_t)r * d + c] = ls * S[(size_t)r * d + c] + kr * v[off + c];
            }
            for (int c = 0; c < d; ++c) {
                double acc = 0.0;
                for (int r = 0; r < d; ++r) acc += q[off + r] * S[(size_t)r * d + c];
                o[off + c] = q_scale * acc;
            }
        }
        if (s_out) memcpy(s_out + (size_t)bh * d * d, S, sizeof(double) * (size_t)d * d);
        free(S);
    }
    return status;
}

/*
 * Brute force for tiny inputs, one sequence: unrolling the recurrence channel by channel,
 *     o_i[c] = q_scale * sum_{j<=i} sum_r q_i[r] (prod_{s=j+1..i} lambda_s^spatial[r]) k_j[r] v_j[c],
 * every product formed by its own loop; no state.  q, lam, k (or NULL), v, o: [n][d].
 */
int lasad_oracle_gated_bruteforce(const double *q, const double *lam, const double *k, const double *v,
                                  double q_scale, double *o, int n, int d, int grid_w, int start_pos, int mode)
{
    if (!q || !lam || !v || !o || n < 0 || d < 1 || grid_w < 1 || mode < 0 || mode > 2) return 1;
    for (int i = 0; i < n; ++i)
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int j = 0; j <= i; ++j)
                for (int r = 0; r < d; ++r) {
                    double decay = 1.0;
                    for (int s = j + 1; s <= i; ++s)
                        decay *= is_boundary((int64_t)start_pos + 1 + s, grid_w, mode) ? 1.0 : lam[(size_t)s * d + r];
                    const double kr = k ? k[(size_t)j * d + r] : 1.0 - lam[(size_t)j * d + r];
                    acc += q[(size_t)i * d + r] * decay * kr * v[(size_t)j * d + c];
                }
            o[(size_t)i * d + c] = q_scale * acc;
        }
    return 0;
}

/* Threads the OpenMP loops above will use (reported by the benchmark). */
/*
 * Gradients of the sequential form (Section 3.4 recurrence) by differentiating it step by step in
 * reverse.  The call covers tokens 1..n of a sequence whose state before token 1 is s_0 (zero if
 * s0 is NULL) and whose loss may also depend on the state after token n: given d_o[t] = dL/do_t
 * and d_sn = dL/ds_n (zero if NULL), with
 *     s_t = lambda_t s_{t-1} + k_t v_t^T,        o_t = q_scale * s_t^T q_t,
 * the state gradient g_t = dL/ds_t obeys g_n = d_sn + q_scale q_n d_o_n^T,
 * g_t = q_scale q_t d_o_t^T + lambda_{t+1} g_{t+1}, and
 *     dq_t = q_scale * s_t d_o_t,   dk_t = g_t v_t,   dv_t = g_t^T k_t,   dlambda_t = <g_t, s_{t-1}>,
 *     d_s0 = lambda_1 g_1          (the gradient for the incoming state; not written if d_s0 is NULL).
 * The forward states s_0 .. s_n are kept (n+1 matrices per sequence).  lam is [Hh][n]; dq, dk, dv
 * are [B][Hh][n][d]; s0, d_sn, d_s0 are [B][Hh][d][d]; dlam is [B][Hh][n], the gradient with
 * respect to the decay applied at each token of each sequence (the caller sums it over whatever
 * positions share a parameter).
 */
int lasad_oracle_backward_carried(const double *q, const double *k, const double *v,
                                  const double *lam, double q_scale, const double *d_o,
                                  const double *s0, const double *d_sn,
                                  double *dq, double *dk, double *dv, double *dlam, double *d_s0,
                                  int B, int n_heads, int n, int d)
{
    if (!q || !k || !v || !lam || !d_o || !dq || !dk || !dv || !dlam || B < 1 || n_heads < 1 || n < 0 || d < 1)
        return 1;
    int status = 0;
    const int64_t n_seq = (int64_t)B * n_heads;
    const size_t dd = (size_t)d * d;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < n_seq; ++bh) {
        const int h = (int)(bh % n_heads);
        double *S = (double *)calloc((size_t)(n + 1) * dd, sizeof(double));   /* s_0 .. s_n */
        double *G = (double *)calloc(dd, sizeof(double));
        if (!S || !G) {
#pragma omp atomic write
            status = 2;
            free(S); free(G);
            continue;
        }
        if (s0) memcpy(S, s0 + (size_t)bh * dd, dd * sizeof(double));       /* s_0 */
        if (d_sn) memcpy(G, d_sn + (size_t)bh * dd, dd * sizeof(double));    /* dL/ds_n */
        for (int t = 0; t < n; ++t) {
            const double l = lam[(size_t)h * n + t];
            const double *kt = k + ((size_t)bh * n + t) * d;
            const double *vt = v + ((size_t)bh * n + t) * d;
            const double *Sp = S + (size_t)t * dd;
            double *Sn = S + (size_t)(t + 1) * dd;
            for (int r = 0; r < d; ++r)
                for (int c = 0; c < d; ++c)
                    Sn[(size_t)r * d + c] = l * Sp[(size_t)r * d + c] + kt[r] * vt[c];
        }
        for (int t = n - 1; t >= 0; --t) {
            const double l = lam[(size_t)h * n + t];
            const double *qt = q + ((size_t)bh * n + t) * d;
            const double *kt = k + ((size_t)bh * n + t) * d;
            const double *vt = v + ((size_t)bh * n + t) * d;
            const double *gt = d_o + ((size_t)bh * n + t) * d;
            const double *St = S + (size_t)(t + 1) * dd;      /* s_t (contains token t) */
            const double *Sp = S + (size_t)t * dd;            /* s_{t-1} */
            double *dqt = dq + ((size_t)bh * n + t) * d;
            double *dkt = dk + ((size_t)bh * n + t) * d;
            double *dvt = dv + ((size_t)bh * n + t) * d;
            for (int r = 0; r < d; ++r) {
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += St[(size_t)r * d + c] * gt[c];
                dqt[r] = q_scale * acc;
            }
            for (int r = 0; r < d; ++r)
                for (int c = 0; c < d; ++c)
                    G[(size_t)r * d + c] += q_scale * qt[r] * gt[c];
            for (int r = 0; r < d; ++r) {
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += G[(size_t)r * d + c] * vt[c];
                dkt[r] = acc;
            }
            for (int c = 0; c < d; ++c) {
                double acc = 0.0;
                for (int r = 0; r < d; ++r) acc += G[(size_t)r * d + c] * kt[r];
                dvt[c] = acc;
            }
            double dl = 0.0;
            for (size_t e = 0; e < dd; ++e) dl += G[e] * Sp[e];
            dlam[(size_t)bh * n + t] = dl;
            for (size_t e = 0; e < dd; ++e) G[e] *= l;
        }
        if (d_s0) memcpy(d_s0 + (size_t)bh * dd, G, dd * sizeof(double));    /* lambda_1 g_1 (d_sn itself if n = 0) */
        free(S); free(G);
    }
    return status;
}

/* The same from a zero state, final state unused. */
int lasad_oracle_backward(const double *q, const double *k, const double *v,
                          const double *lam, double q_scale, const double *d_o,
                          double *dq, double *dk, double *dv, double *dlam,
                          int B, int n_heads, int n, int d)
{
    return lasad_oracle_backward_carried(q, k, v, lam, q_scale, d_o, NULL, NULL, dq, dk, dv, dlam, NULL, B, n_heads, n, d);
}

/*
 * Gradient of the per-head base decay: gamma_h is the decay of every non-boundary position of
 * every sequence of head h (Section 3.4 second equation), so
 *     dgamma[h] = sum_b sum_{t not a boundary} dlam[b][h][t].
 * Positions are start_pos+1 .. start_pos+n (1-indexed raster positions).
 */
int lasad_oracle_dgamma(const double *dlam, int B, int n_heads, int n,
                        int grid_w, int start_pos, int mode, double *dgamma)
{
    if (!dlam || !dgamma || B < 1 || n_heads < 1 || n < 0 || grid_w < 1) return 1;
    for (int h = 0; h < n_heads; ++h) {
        double acc = 0.0;
        for (int b = 0; b < B; ++b)
            for (int t = 0; t < n; ++t)
                if (!is_boundary((int64_t)start_pos + t + 1, grid_w, mode))
                    acc += dlam[((size_t)b * n_heads + h) * n + t];
        dgamma[h] = acc;
    }
    return 0;
}

/*
 * Gradients of the vector-decay recurrence (Section 3.4 / Algorithm 1) by differentiating it step
 * by step in reverse, exactly as lasad_oracle_backward_carried does for one decay per token: the
 * state before the first token is s0 (zero if NULL), d_sn = dL/ds_n (zero if NULL) enters the state
 * gradient at the last token, and d_s0 = diag(l_1) g_1 is returned if d_s0 is not NULL.  With l_t = lambda_t^spatial (1 in every channel at a row boundary, lambda_t elsewhere),
 *     s_t = diag(l_t) s_{t-1} + k_t v_t^T,        o_t = q_scale * s_t^T q_t,
 * the state gradient g_t = dL/ds_t obeys g_t = q_scale q_t d_o_t^T + diag(l_{t+1}) g_{t+1}, and
 *     dq_t = q_scale * s_t d_o_t,   dk_t = g_t v_t,   dv_t = g_t^T k_t,
 *     dl_t[r] = sum_c g_t[r][c] s_{t-1}[r][c]      (gradient of the decay actually applied).
 * The gradient handed back for the input lambda_t is
 *     dlam_t[r] = (t a boundary ? 0 : dl_t[r])  -  (key tied: dk_t[r]),
 * because at a boundary the applied decay is the constant 1, and a tied key is k_t = 1 - lambda_t
 * (from the base decay, also at a boundary).  With an own key tensor, dk is returned as well
 * (dk must then be non-NULL); with the tied key, dk may be NULL.
 * All tensors [B][Hh][n][d]; the forward states s_0 .. s_n are kept (n+1 matrices per sequence).
 */
int lasad_oracle_gated_backward_carried(const double *q, const double *lam, const double *k, const double *v,
                                        double q_scale, const double *d_o, const double *s0, const double *d_sn,
                                        double *dq, double *dlam, double *dk, double *dv, double *d_s0,
                                        int B, int n_heads, int n, int d, int grid_w, int start_pos, int mode)
{
    if (!q || !lam || !v || !d_o || !dq || !dlam || !dv || (k && !dk)) return 1;
    if (B < 1 || n_heads < 1 || n < 0 || d < 1 || grid_w < 1 || start_pos < 0 || mode < 0 || mode > 2) return 1;
    int status = 0;
    const int64_t n_seq = (int64_t)B * n_heads;
    const size_t dd = (size_t)d * d;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < n_seq; ++bh) {
        double *S = (double *)calloc((size_t)(n + 1) * dd, sizeof(double));   /* s_0 .. s_n */
        double *G = (double *)calloc(dd, sizeof(double));
        double *kt = (double *)calloc((size_t)d, sizeof(double));
        double *dkt = (double *)calloc((size_t)d, sizeof(double));
        if (!S || !G || !kt || !dkt) {
#pragma omp atomic write
            status = 2;
            free(S); free(G); free(kt); free(dkt);
            continue;
        }
        if (s0) memcpy(S, s0 + (size_t)bh * dd, dd * sizeof(double));       /* s_0 */
        if (d_sn) memcpy(G, d_sn + (size_t)bh * dd, dd * sizeof(double));    /* dL/ds_n */
        for (int t = 0; t < n; ++t) {
            const size_t off = ((size_t)bh * n + t) * d;
            const int boundary = is_boundary((int64_t)start_pos + 1 + t, grid_w, mode);
            const double *Sp = S + (size_t)t * dd;
            double *Sn = S + (size_t)(t + 1) * dd;
            for (int r = 0; r < d; ++r) {
                const double l = lam[off + r];
                const double kr = k ? k[off + r] : 1.0 - l;
                const double ls = boundary ? 1.0 : l;
                for (int c = 0; c < d; ++c)
                    Sn[(size_t)r * d + c] = ls * Sp[(size_t)r * d + c] + kr * v[off + c];
            }
        }
        for (int t = n - 1; t >= 0; --t) {
            const size_t off = ((size_t)bh * n + t) * d;
            const int boundary = is_boundary((int64_t)start_pos + 1 + t, grid_w, mode);
            const double *St = S + (size_t)(t + 1) * dd;      /* s_t (contains token t) */
            const double *Sp = S + (size_t)t * dd;            /* s_{t-1} */
            for (int r = 0; r < d; ++r) kt[r] = k ? k[off + r] : 1.0 - lam[off + r];
            for (int r = 0; r < d; ++r) {
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += St[(size_t)r * d + c] * d_o[off + c];
                dq[off + r] = q_scale * acc;
            }
            for (int r = 0; r < d; ++r)
                for (int c = 0; c < d; ++c)
                    G[(size_t)r * d + c] += q_scale * q[off + r] * d_o[off + c];
            for (int r = 0; r < d; ++r) {
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += G[(size_t)r * d + c] * v[off + c];
                dkt[r] = acc;
            }
            for (int c = 0; c < d; ++c) {
                double acc = 0.0;
                for (int r = 0; r < d; ++r) acc += G[(size_t)r * d + c] * kt[r];
                dv[off + c] = acc;
            }
            for (int r = 0; r < d; ++r) {
                double dl = 0.0;
                for (int c = 0; c < d; ++c) dl += G[(size_t)r * d + c] * Sp[(size_t)r * d + c];
                if (boundary) dl = 0.0;                       /* the applied decay is the constant 1 */
                if (k) { dk[off + r] = dkt[r]; dlam[off + r] = dl; }
                else   { if (dk) dk[off + r] = dkt[r]; dlam[off + r] = dl - dkt[r]; }
            }
            for (int r = 0; r < d; ++r) {                     /* into g_{t-1}: times the decay applied at t */
                const double ls = boundary ? 1.0 : lam[off + r];
                for (int c = 0; c < d; ++c) G[(size_t)r * d + c] *= ls;
            }
        }
        if (d_s0) memcpy(d_s0 + (size_t)bh * dd, G, dd * sizeof(double));    /* diag(l_1) g_1 */
        free(S); free(G); free(kt); free(dkt);
    }
    return status;
}

/* The same from a zero state, final state unused. */
int lasad_oracle_gated_backward(const double *q, const double *lam, const double *k, const double *v,
                                double q_scale, const double *d_o,
                                double *dq, double *dlam, double *dk, double *dv,
                                int B, int n_heads, int n, int d, int grid_w, int start_pos, int mode)
{
    return lasad_oracle_gated_backward_carried(q, lam, k, v, q_scale, d_o, NULL, NULL, dq, dlam, dk, dv, NULL,
                                               B, n_heads, n, d, grid_w, start_pos, mode);
}

#ifdef _OPENMP
#include <omp.h>
int lasad_oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int lasad_oracle_num_threads(void) { return 1; }
#endif
