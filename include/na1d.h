/*
 * na1d.h -- C ABI of the MI355X (gfx950) 1D Neighborhood Attention entry points (same library
 * as na2d.h, whose dtype and status codes are reused).
 *
 * The operation of "Neighborhood Attention Transformer" (arXiv 2204.07143), Section 3.1,
 * Eq. 2-4, on a sequence of L tokens (the paper's package ships a 1D module next to the 2D one,
 * Appendix A, "Implementation notes"): every token attends to its k nearest tokens; at the two ends
 * the window is shifted, never shrunk, so each query keeps exactly k keys; a relative positional
 * bias B(i, j) is added to the logits (Eq. 2).  The split into entry points is the one of na2d.h.
 *
 * Conventions (as in na2d.h unless stated)
 * ----------------------------------------
 *  - All data pointers are DEVICE pointers owned by the caller, 16-byte aligned, contiguous,
 *    row-major.  The library never allocates, frees or synchronises; calls enqueue on `stream`
 *    (hipStream_t as void*, NULL = default stream).  Outputs are fully overwritten.
 *  - Layouts:  q, k, v, out, dout, dq, dk, dv : [B, heads, L, D]    (problem dtype)
 *              logits, p, dp, ds             : [B, heads, L, k]    (problem dtype)
 *              rpb                           : [heads, 2k-1]       (problem dtype)
 *              d_rpb                         : [heads, 2k-1]       (always fp32)
 *              lse                           : [B, heads, L]       (always fp32)
 *    Window slot a addresses key s(i) + a, s(i) = clamp(i - (k-1)/2, 0, L - k); the bias cell
 *    of (query i, key j) is rpb[head, j - i + k - 1].
 *  - Arithmetic: storage in the problem dtype (round-to-nearest-even on store); dot products,
 *    softmax and sums in fp32.
 *  - Supported: D = 32, odd k with 3 <= k <= 63 and k <= L (k = L is self attention).
 *  - Return value: NA2D_OK or a negative na2d_status; argument errors are detected on the host
 *    before any HIP call and nothing is enqueued then.  NA2D_ERR_TOO_SMALL: k > L.
 */
#ifndef NA1D_H_
#define NA1D_H_

#include "na2d.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t B, heads, L, D, k;
    int32_t dtype; /* na2d_dtype */
} na1d_problem;

/* Host only: NA2D_OK if every entry point below accepts the problem. */
int na1d_validate_problem(const na1d_problem *p);

/* Eq. 2: logits[n, a] = scale * <q_n, k_{s(n)+a}> + rpb[head, s(n)+a - n + k-1].  rpb may be NULL. */
int na1d_qk_rpb(const na1d_problem *p, const void *q, const void *k, const void *rpb, float scale, void *logits,
                void *stream);

/* Eq. 4: softmax over the k slots of every query.  `p_out` may alias `logits`. */
int na1d_softmax(const na1d_problem *p, const void *logits, void *p_out, void *stream);

/* Eq. 3-4: out[n, :] = sum_a p[n, a] * v[s(n)+a, :]. */
int na1d_av(const na1d_problem *p, const void *attn, const void *v, void *out, void *stream);

/* Eq. 2-4 in one kernel: no logits or weights in memory.  `lse` (nullable) receives the
 * log-sum-exp of every query's logits. */
int na1d_fused_fwd(const na1d_problem *p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                   void *out, float *lse, void *stream);

/* Gradients (the paper's list: q, k, b, a, v; Appendix A).  Same roles as in na2d.h. */
/* grad-a: dp[n, a] = <dout_n, v_{s(n)+a}> */
int na1d_av_bwd_p(const na1d_problem *p, const void *dout, const void *v, void *dp, void *stream);
/* grad-v: dv[j, :] = sum over the queries i that see j of p[i, j - s(i)] * dout[i, :] */
int na1d_av_bwd_v(const na1d_problem *p, const void *attn, const void *dout, void *dv, void *stream);
/* softmax backward: ds = p * (dp - <p, dp>) per query.  `ds` may alias `dp`. */
int na1d_softmax_bwd(const na1d_problem *p, const void *attn, const void *dp, void *ds, void *stream);
/* grad-q: dq[n, :] = scale * sum_a ds[n, a] * k[s(n)+a, :] */
int na1d_qk_bwd_q(const na1d_problem *p, const void *ds, const void *k, float scale, void *dq, void *stream);
/* grad-k: dk[j, :] = scale * sum over the queries i that see j of ds[i, j - s(i)] * q[i, :] */
int na1d_qk_bwd_k(const na1d_problem *p, const void *ds, const void *q, float scale, void *dk, void *stream);
/* grad-b: d_rpb[h, u] = sum over batch, queries and slots whose bias cell is u of ds.  Summed as
 * 64-bit fixed point (42 fraction bits), so the result does not depend on the order of the
 * additions (bitwise reproducible).  Range of that format: every ds is truncated to a multiple of
 * 2^-42 (gradients whose ds are all below that sum to 0; at |ds| ~ 1e-6 the relative error of a
 * term is 2e-7, that of fp32), and a ds with |ds| >= 2^21, or a non-finite one, counts as 0
 * instead of saturating or poisoning the sum.  `workspace` must hold
 * na1d_workspace_bytes(p) bytes; no initialisation needed. */
int na1d_qk_bwd_rpb(const na1d_problem *p, const void *ds, float *d_rpb, void *workspace, size_t workspace_bytes,
                    void *stream);
size_t na1d_workspace_bytes(const na1d_problem *p);

/* Whole backward without the k-wide tensors (the 1D counterpart of na2d_fused_bwd): dq, dk, dv and (if
 * d_rpb != NULL) d_rpb of out = NA(q, k, v, rpb) from q, k, v, rpb, dout and `lse`, the log-sum-exp that
 * na1d_fused_fwd stored for every query.  The attention weights are recomputed as
 * exp(scale <q, k> + bias - lse).  `rpb` may be NULL (no bias in the forward).  No output may alias an input
 * or another output.  d_rpb is summed in 64-bit fixed point as in na1d_qk_bwd_rpb (bitwise reproducible).
 * `workspace` must hold na1d_fused_bwd_workspace_bytes(p) bytes; no initialisation needed. */
int na1d_fused_bwd(const na1d_problem *p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                   const float *lse, const void *dout, void *dq, void *dk, void *dv, float *d_rpb, void *workspace,
                   size_t workspace_bytes, void *stream);
size_t na1d_fused_bwd_workspace_bytes(const na1d_problem *p);

#ifdef __cplusplus
}
#endif
#endif /* NA1D_H_ */
