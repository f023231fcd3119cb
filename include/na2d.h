/*
 * na2d.h -- C ABI of the MI355X (gfx950) 2D Neighborhood Attention library.
 *
 * The operation is the one defined in "Neighborhood Attention Transformer"
 * (arXiv 2204.07143), Section 3.1: every pixel attends to its k x k nearest pixels
 * (Eq. 2-4); at the borders the window is shifted, never shrunk, so each query keeps
 * exactly k*k keys (Section 1; Appendix figure "3x3 NA on a 7x7 map"); a relative
 * positional bias B(i, j) is added to the logits (Eq. 2).  The split into a logits
 * function and a weighted-sum function with a softmax in between follows the paper's
 * own package (Appendix A: C functions QK+RPB and AV, softmax applied between them;
 * gradients for q, k, b, a, v).
 *
 * Conventions common to every entry point
 * ---------------------------------------
 *  - All data pointers are DEVICE pointers owned by the caller (16-byte aligned,
 *    contiguous, row-major, last index fastest).  The only host pointers are the
 *    `const na2d_problem*` argument and the arguments of the na2d_host_* helpers.
 *  - The library never allocates, frees or synchronises.  Every call enqueues its
 *    kernels on `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 *    returns immediately.  Outputs are fully overwritten; nothing needs pre-zeroing.
 *  - Layouts:  q, k, v, out, dout, dq, dk, dv : [B, heads, H, W, D]      (problem dtype)
 *              logits, p, dp, ds             : [B, heads, H, W, k*k]    (problem dtype)
 *              rpb                           : [heads, 2k-1, 2k-1]      (problem dtype)
 *              d_rpb                         : [heads, 2k-1, 2k-1]      (always fp32)
 *              lse                           : [B, heads, H, W]         (always fp32)
 *    Window slot a*k + c addresses key (s(qy) + a, s(qx) + c), where
 *    s(i) = clamp(i - (k-1)/2, 0, L - k) is the first key coordinate seen by query
 *    coordinate i on an axis of length L (raster order over ascending key coordinates).
 *    The bias cell of (query i, key j) is rpb[head, jy - iy + k - 1, jx - ix + k - 1].
 *  - Arithmetic: storage in the problem dtype (round-to-nearest-even on store), all dot
 *    products, the softmax and all sums accumulated in fp32.  The bias is added to the fp32
 *    logit exactly as stored.  The fused 16-bit kernels (na2d_fused_fwd, na2d_fused_bwd) hold
 *    the table as fp16: an fp16 table is used bit for bit; a bf16 entry converts exactly while
 *    2^-14 <= |b| <= 65504, a larger one counts as +-65504 and a smaller one is rounded to a
 *    multiple of 2^-24.
 *  - Supported: odd k from 3 to 63 with k <= min(H, W); k = H = W is the self-attention limit
 *    (Section 3.1).  k in {3, 5, 7, 9, 11, 13}, the sizes the paper tunes for (Appendix A,
 *    "Tiled Neighborhood Attention"), run the tiled kernels described below; k >= 15 runs plain
 *    kernels with the window side as a run-time argument (every dtype, every head dim below;
 *    correct and deterministic, not tuned).  Head dims
 *    D in {16, 32, 64, 128}.  D = 32 (every NAT variant, Section 3.2) runs the matrix-core
 *    kernels in the 16-bit types; so do the weighted sums (av, grad-q, grad-v, grad-k) for
 *    D = 64 and 128, the logits, grad-a and the fused forward for D = 64 (for D = 128 the
 *    logits and grad-a with k <= 11, the fused forward with k <= 7), and all
 *    of these for D = 16 (a 16-channel head rides in the lower half of the 32-channel
 *    kernels); the softmax kernels and grad-b do not depend on D; the rest runs tiled
 *    plain-ALU kernels while their tiles fit the
 *    160 KB LDS (every k for D = 16 and for D = 64 in the 16-bit types, k <= 9 for D = 128 in
 *    the 16-bit types and for D = 64 in fp32, k = 3 for D = 128 in fp32) and the run-time-k
 *    kernels otherwise.
 *  - Inputs are expected to be finite.  The matrix-core kernels multiply values of
 *    neighbouring positions (up to a tile's query rectangle away) by zero weights instead of
 *    skipping them, so a NaN or an infinity in q, k, v, dout or a weight tensor can turn
 *    results of positions beyond its own neighbourhood into NaN.
 *  - Return value: NA2D_OK (0) or a negative na2d_status.  All argument errors are
 *    detected on the host before any HIP call; on error nothing is enqueued.
 */
#ifndef NA2D_H_
#define NA2D_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { NA2D_F32 = 0, NA2D_F16 = 1, NA2D_BF16 = 2 } na2d_dtype;

typedef enum {
    NA2D_OK = 0,
    NA2D_ERR_NULL = -1,        /* a required pointer is NULL */
    NA2D_ERR_DTYPE = -2,       /* dtype is not one of na2d_dtype */
    NA2D_ERR_KERNEL_SIZE = -3, /* k even, below 3 or above 63 */
    NA2D_ERR_TOO_SMALL = -4,   /* k > min(H, W): the neighbourhood is undefined */
    NA2D_ERR_HEAD_DIM = -5,    /* D not in {16, 32, 64, 128} */
    NA2D_ERR_SHAPE = -6,       /* non-positive extent, a tensor beyond 2^31-1 elements, or one (batch, head)
                                  plane of a tensor beyond 2^31-1 bytes */
    NA2D_ERR_ALIGN = -7,       /* a data pointer is not 16-byte aligned */
    NA2D_ERR_WORKSPACE = -8,   /* workspace missing or smaller than na2d_workspace_bytes() */
    NA2D_ERR_LAUNCH = -9,      /* hipGetLastError() reported a launch failure */
    NA2D_ERR_ALIAS = -10       /* an output aliases an input where that is not allowed */
} na2d_status;

typedef struct {
    int32_t B, heads, H, W, D, k;
    int32_t dtype; /* na2d_dtype */
} na2d_problem;

/* Which call a workspace size is asked for (na2d_workspace_bytes). */
typedef enum { NA2D_WS_QK_BWD_RPB = 0, NA2D_WS_BWD = 1, NA2D_WS_FUSED_BWD = 2 } na2d_ws_kind;

/* ---- forward ------------------------------------------------------------------ */

/*
 * Eq. 2: logits[n, a, c] = scale * <q_n, k_{rho(n; a, c)}> + B(n, rho(n; a, c)).
 * `rpb` may be NULL (no bias).  `scale` multiplies the fp32 dot product; the bias is
 * added unscaled (the paper's package folds the 1/sqrt(d) of Eq. 4 into q before its
 * QK+RPB call, so the bias is not divided by sqrt(d)).
 */
int na2d_qk_rpb(const na2d_problem *p, const void *q, const void *k, const void *rpb, float scale,
                void *logits, void *stream);

/* Eq. 4's softmax over the k*k axis (max-subtracted, fp32).  `p_out` may alias `logits`. */
int na2d_softmax(const na2d_problem *p, const void *logits, void *p_out, void *stream);

/* Eq. 3-4: out[n, :] = sum_{a, c} p[n, a, c] * v_{rho(n; a, c)}. */
int na2d_av(const na2d_problem *p, const void *attn, const void *v, void *out, void *stream);

/*
 * Eq. 2-4 in one kernel: the k*k logits and weights never leave the chip (the h*w*k^2
 * attention tensor is the memory term of the paper's complexity table, Section 3.3).
 * `rpb` may be NULL.  `lse` may be NULL; otherwise it receives the per-query
 * log-sum-exp of the logits.
 */
int na2d_fused_fwd(const na2d_problem *p, const void *q, const void *k, const void *v, const void *rpb,
                   float scale, void *out, float *lse, void *stream);

/* ---- backward (Appendix A: gradients for a, v, q, k and b) ------------------------ */

/* grad-a: dp[n, a, c] = <dout_n, v_{rho(n; a, c)}>. */
int na2d_av_bwd_p(const na2d_problem *p, const void *dout, const void *v, void *dp, void *stream);

/* grad-v: dv_j = sum over the queries n whose window holds j of attn[n, slot(n, j)] * dout_n.
 * Gathered over the inverse neighbourhood of j; no atomics, bitwise reproducible. */
int na2d_av_bwd_v(const na2d_problem *p, const void *attn, const void *dout, void *dv, void *stream);

/* Softmax backward: ds[n, :] = attn[n, :] * (dp[n, :] - <attn[n, :], dp[n, :]>).  `ds` may alias `dp`. */
int na2d_softmax_bwd(const na2d_problem *p, const void *attn, const void *dp, void *ds, void *stream);

/* grad-q: dq_n = scale * sum_{a, c} ds[n, a, c] * k_{rho(n; a, c)}. */
int na2d_qk_bwd_q(const na2d_problem *p, const void *ds, const void *k, float scale, void *dq, void *stream);

/* grad-k: dk_j = scale * sum over the queries n whose window holds j of ds[n, slot(n, j)] * q_n. */
int na2d_qk_bwd_k(const na2d_problem *p, const void *ds, const void *q, float scale, void *dk, void *stream);

/*
 * grad-b: d_rpb[h, u, v] = sum over batch, queries and slots whose bias cell is (u, v) of ds.
 * Two-level reduction in a fixed order (bitwise reproducible).  `workspace` must hold
 * na2d_workspace_bytes(p, NA2D_WS_QK_BWD_RPB) bytes; its contents need no initialisation.
 */
int na2d_qk_bwd_rpb(const na2d_problem *p, const void *ds, float *d_rpb, void *workspace, size_t workspace_bytes,
                    void *stream);

/*
 * na2d_qk_bwd_rpb for callers that cannot allocate device memory or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same order of
 * additions, same result bit for bit; the partial sums live in a device array of
 * NA2D_NOALLOC_SCRATCH_BYTES that is part of the library's code object (every GPU the library runs on
 * holds one copy from its first use until the process ends).  The call allocates and frees nothing; its
 * first use on a device looks up the array's address on that device.
 * A problem whose partials (na2d_workspace_bytes(p, NA2D_WS_QK_BWD_RPB) at most) do not fit the array is
 * refused with NA2D_ERR_WORKSPACE before any HIP call: 4 MiB hold, for example, 1024 workgroups'
 * partials at k = 13, or B * heads = 6000 planes at k = 7.
 * All calls on one GPU share the array: calls that may overlap in time (different streams, different
 * host threads) race on it and must be ordered by the caller.  Nothing needs clearing between calls.
 */
#define NA2D_NOALLOC_SCRATCH_BYTES (4u << 20)
int na2d_qk_bwd_rpb_noalloc(const na2d_problem *p, const void *ds, float *d_rpb, void *stream);

/*
 * Whole backward of out = NA(q, k, v, rpb): grad-a, grad-v, softmax backward, grad-q, grad-k
 * and (if d_rpb != NULL) grad-b.  For the 16-bit types with k <= 9 (D = 32 or 16), grad-a and the softmax
 * backward run as one kernel and dp is never stored (so ds is computed from the unrounded dp);
 * otherwise the six steps run one after the other exactly as the separate entry points do.
 * `attn` is the softmax output of the forward.  `workspace` must hold
 * na2d_workspace_bytes(p, NA2D_WS_BWD) bytes; on return it starts with the ds tensor
 * ([B, heads, H, W, k*k], problem dtype), followed by the grad-b partials.
 * No output (d_rpb included) may alias an input or another output.
 */
int na2d_bwd(const na2d_problem *p, const void *q, const void *k, const void *v, const void *attn,
             const void *dout, float scale, void *dq, void *dk, void *dv, float *d_rpb,
             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Whole backward without the k*k tensors (the step next to the fused forward; the paper has no fused
 * path and names NA as an implicit GEMM as future work, Appendix A): dq, dk, dv and (if d_rpb != NULL)
 * d_rpb of out = NA(q, k, v, rpb) from q, k, v, rpb, dout and `lse`, the log-sum-exp that
 * na2d_fused_fwd stored for every query.  The attention weights are recomputed per tile as
 * exp(scale <q, k> + bias - lse) and neither they nor dp / ds reach memory.  `rpb` may be NULL
 * (no bias in the forward).  No output may alias an input or another output.
 * For the 16-bit types with k <= 9 and D = 32 or 16 this runs two kernels: query patches (dq, the partial bias
 * gradients and delta_n = sum_j P[n, j] dP[n, j]) and key patches (dk, dv); na2d_fused_bwd_is_fused() tells.
 * There d_rpb is summed per workgroup with integer atomics in 64-bit fixed point, so it does not depend on
 * the order of the additions.  The fixed point has 32 fraction bits; a ds enters it with a relative error
 * below 2^-30 of the largest |ds| its query can have, or 2^-32 absolute, whichever is larger, and the sums
 * are exact while |ds| < 2^20: upstream gradients from about 1e-5 to 1e5 times unit scale keep d_rpb within
 * 1e-4 of its largest entry; beyond 2^20 the sums wrap.  A NaN ds counts as 0 there.
 * The weights are recomputed from the fp32 `lse`, whose spacing 2^-24 |lse| enters every weight as a relative
 * error (and d_rpb as the sum of those errors): logits, bias included, of a few hundred in magnitude at most
 * keep dq, dk, dv within the 16-bit bound and d_rpb within 1e-4 of its largest entry.
 * Every other case recomputes the attention weights into the workspace (one logits and one softmax launch)
 * and runs the unfused backward: it then costs more than na2d_bwd on stored weights, and its only gain is
 * that the caller need not keep them.  Both ways the results are bitwise reproducible.
 * `workspace` must hold na2d_workspace_bytes(p, NA2D_WS_FUSED_BWD) bytes; no initialisation needed.
 */
int na2d_fused_bwd(const na2d_problem *p, const void *q, const void *k, const void *v, const void *rpb,
                   float scale, const float *lse, const void *dout, void *dq, void *dk, void *dv, float *d_rpb,
                   void *workspace, size_t workspace_bytes, void *stream);

/* 1 if na2d_fused_bwd runs its two fused kernels for this problem, 0 if it recomputes the attention
 * weights and runs the unfused steps, a negative na2d_status for an invalid problem.  Host only. */
int na2d_fused_bwd_is_fused(const na2d_problem *p);

/* Bytes of device workspace the given call needs for this problem (0 on invalid problems). */
size_t na2d_workspace_bytes(const na2d_problem *p, int kind);

/* ---- neighbourhood indices (Section 3.1; "indices must match bit-exactly") --------- */

/*
 * Writes, for one H x W map, key_index[qy, qx, a*k+c] = ky*W + kx and
 * rpb_index[qy, qx, a*k+c] = (ky-qy+k-1)*(2k-1) + (kx-qx+k-1), both int32 [H, W, k*k],
 * using the same device index functions as the attention kernels.  Either may be NULL.
 */
int na2d_debug_indices(const na2d_problem *p, int32_t *key_index, int32_t *rpb_index, void *stream);

/* Host-side evaluation of the same index functions (HOST pointers; no GPU needed):
 * start[i] = s(i) and, for key coordinate j, the contiguous range [qs[j], qe[j]] of query
 * coordinates whose window holds j (the inverse neighbourhood).  Arrays have L entries; any may be NULL. */
int na2d_host_axis_tables(int32_t L, int32_t k, int32_t *start, int32_t *qs, int32_t *qe);

/* Validates a problem descriptor exactly as every entry point does (host only). */
int na2d_validate_problem(const na2d_problem *p);

const char *na2d_strerror(int status);
int na2d_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NA2D_H_ */
