// C ABI of the 2D Neighborhood Attention library: argument validation (host only, before any
// HIP call), dispatch to the kernel launchers, and the index-export helpers.
#include <stdint.h>

#include "na2d.h"
#include "na2d_common.hpp"
#include "na2d_kernels.hpp"
#include "na2d_valu_cfg.hpp"

namespace na2d {

static int validate(const na2d_problem *p) {
    if (!p) return NA2D_ERR_NULL;
    if (p->dtype != NA2D_F32 && p->dtype != NA2D_F16 && p->dtype != NA2D_BF16) return NA2D_ERR_DTYPE;
    if (p->B <= 0 || p->heads <= 0 || p->H <= 0 || p->W <= 0 || p->D <= 0 || p->k <= 0) return NA2D_ERR_SHAPE;
    const int k = p->k;
    if ((k & 1) == 0 || k < 3 || k > kMaxGenericK) return NA2D_ERR_KERNEL_SIZE;
    if (k > p->H || k > p->W) return NA2D_ERR_TOO_SMALL;
    if (p->D != 16 && p->D != 32 && p->D != 64 && p->D != 128) return NA2D_ERR_HEAD_DIM;
    // Index arithmetic inside the kernels is 64-bit for byte offsets, but element counts of a
    // tensor must fit int32 so that per-plane and per-row products cannot overflow.
    const int64_t nq = (int64_t)p->B * p->heads * p->H * p->W;
    const int64_t widest = k * k > p->D ? k * k : p->D;
    if (nq * widest > (int64_t)INT32_MAX) return NA2D_ERR_SHAPE;
    // ... and one (batch, head) plane of any tensor stays below 2^31 bytes: offsets inside a plane are 32-bit
    const int64_t elem = p->dtype == NA2D_F32 ? 4 : 2;
    if ((int64_t)p->H * p->W * widest * elem > (int64_t)INT32_MAX) return NA2D_ERR_SHAPE;
    return NA2D_OK;
}

static inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

static Problem to_problem(const na2d_problem *p) { return Problem{p->B, p->heads, p->H, p->W, p->k, p->dtype, p->D}; }

static int from_hip(hipError_t e) {
    if (e == hipSuccess) return NA2D_OK;
    (void)hipGetLastError();   // leave no stale error behind for the caller's next HIP call
    return NA2D_ERR_LAUNCH;
}

template <typename T, int K>
__global__ void indices_kernel(int32_t *key_index, int32_t *rpb_index, int H, int W) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    constexpr int KK = K * K, NB = 2 * K - 1;
    if (i >= H * W * KK) return;
    const int slot = i % KK, qlin = i / KK;
    const int qy = qlin / W, qx = qlin % W;
    const int a = slot / K, c = slot % K;
    const int ky = win_start(qy, H, K) + a, kx = win_start(qx, W, K) + c;
    if (key_index) key_index[i] = ky * W + kx;
    if (rpb_index) rpb_index[i] = (rpb_start(qy, H, K) + a) * NB + (rpb_start(qx, W, K) + c);
}

hipError_t launch_indices(const Problem &p, int32_t *key_index, int32_t *rpb_index, hipStream_t s) {
    if (untuned_window(p)) return launch_indices_generic(p, key_index, rpb_index, s);
    const int n = p.H * p.W * p.K * p.K;
    NA2D_DISPATCH_K(p.K, hipLaunchKernelGGL((indices_kernel<float, K>), dim3((n + 255) / 256), dim3(256), 0, s,
                                            key_index, rpb_index, p.H, p.W));
    return hipGetLastError();
}

}  // namespace na2d

using namespace na2d;

#define NA2D_CHECK_PROBLEM(p)             \
    do {                                  \
        int st_ = validate(p);            \
        if (st_ != NA2D_OK) return st_;   \
    } while (0)
#define NA2D_REQUIRE(ptr)                         \
    do {                                          \
        if (!(ptr)) return NA2D_ERR_NULL;         \
        if (misaligned(ptr)) return NA2D_ERR_ALIGN; \
    } while (0)
#define NA2D_OPTIONAL(ptr)                                 \
    do {                                                   \
        if ((ptr) && misaligned(ptr)) return NA2D_ERR_ALIGN; \
    } while (0)

extern "C" {

int na2d_validate_problem(const na2d_problem *p) { return validate(p); }

int na2d_qk_rpb(const na2d_problem *p, const void *q, const void *k, const void *rpb, float scale, void *logits,
                void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(q); NA2D_REQUIRE(k); NA2D_REQUIRE(logits); NA2D_OPTIONAL(rpb);
    if (logits == q || logits == k) return NA2D_ERR_ALIAS;
    return from_hip(launch_qk(to_problem(p), q, k, rpb, scale, logits, static_cast<hipStream_t>(stream)));
}

int na2d_softmax(const na2d_problem *p, const void *logits, void *p_out, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(logits); NA2D_REQUIRE(p_out);
    return from_hip(launch_softmax(to_problem(p), logits, p_out, static_cast<hipStream_t>(stream)));
}

int na2d_av(const na2d_problem *p, const void *attn, const void *v, void *out, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(attn); NA2D_REQUIRE(v); NA2D_REQUIRE(out);
    if (out == attn || out == v) return NA2D_ERR_ALIAS;
    return from_hip(launch_av(to_problem(p), attn, v, 1.0f, out, static_cast<hipStream_t>(stream)));
}

int na2d_fused_fwd(const na2d_problem *p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                   void *out, float *lse, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(q); NA2D_REQUIRE(k); NA2D_REQUIRE(v); NA2D_REQUIRE(out); NA2D_OPTIONAL(rpb); NA2D_OPTIONAL(lse);
    if (out == q || out == k || out == v) return NA2D_ERR_ALIAS;
    return from_hip(launch_fused_fwd(to_problem(p), q, k, v, rpb, scale, out, lse, static_cast<hipStream_t>(stream)));
}

int na2d_av_bwd_p(const na2d_problem *p, const void *dout, const void *v, void *dp, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(dout); NA2D_REQUIRE(v); NA2D_REQUIRE(dp);
    if (dp == dout || dp == v) return NA2D_ERR_ALIAS;
    return from_hip(launch_qk(to_problem(p), dout, v, nullptr, 1.0f, dp, static_cast<hipStream_t>(stream)));
}

int na2d_av_bwd_v(const na2d_problem *p, const void *attn, const void *dout, void *dv, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(attn); NA2D_REQUIRE(dout); NA2D_REQUIRE(dv);
    if (dv == attn || dv == dout) return NA2D_ERR_ALIAS;
    return from_hip(launch_inverse(to_problem(p), attn, dout, 1.0f, dv, static_cast<hipStream_t>(stream)));
}

int na2d_softmax_bwd(const na2d_problem *p, const void *attn, const void *dp, void *ds, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(attn); NA2D_REQUIRE(dp); NA2D_REQUIRE(ds);
    if (ds == attn) return NA2D_ERR_ALIAS;
    return from_hip(launch_softmax_bwd(to_problem(p), attn, dp, ds, static_cast<hipStream_t>(stream)));
}

int na2d_qk_bwd_q(const na2d_problem *p, const void *ds, const void *k, float scale, void *dq, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(ds); NA2D_REQUIRE(k); NA2D_REQUIRE(dq);
    if (dq == ds || dq == k) return NA2D_ERR_ALIAS;
    return from_hip(launch_av(to_problem(p), ds, k, scale, dq, static_cast<hipStream_t>(stream)));
}

int na2d_qk_bwd_k(const na2d_problem *p, const void *ds, const void *q, float scale, void *dk, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(ds); NA2D_REQUIRE(q); NA2D_REQUIRE(dk);
    if (dk == ds || dk == q) return NA2D_ERR_ALIAS;
    return from_hip(launch_inverse(to_problem(p), ds, q, scale, dk, static_cast<hipStream_t>(stream)));
}

size_t na2d_workspace_bytes(const na2d_problem *p, int kind) {
    if (validate(p) != NA2D_OK) return 0;
    const Problem pr = to_problem(p);
    const size_t rpb = (rpb_bwd_workspace_bytes(pr) + 255) & ~(size_t)255;
    if (kind == NA2D_WS_QK_BWD_RPB) return rpb;
    const size_t attn = (pr.queries() * p->k * p->k * pr.elem_bytes() + 255) & ~(size_t)255;
    if (kind == NA2D_WS_BWD) return attn + rpb;
    if (kind == NA2D_WS_FUSED_BWD) {
        if (!fused_bwd_supported(pr)) return attn + attn + rpb;
        const AvRpbSplit sp = fused_bwd_split(pr);
        const int nbc = 2 * pr.K - 1;
        const size_t partials = ((size_t)sp.npos * pr.heads * sp.splits * rpb_cell_stride(nbc * nbc) * sizeof(float) + 255) & ~(size_t)255;
        return 2 * ((pr.queries() * sizeof(float) + 255) & ~(size_t)255) + partials;   // delta, lse in the exp2 domain
    }
    return 0;
}

int na2d_qk_bwd_rpb(const na2d_problem *p, const void *ds, float *d_rpb, void *workspace, size_t workspace_bytes,
                    void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(ds); NA2D_REQUIRE(d_rpb);
    if (!workspace || misaligned(workspace) || workspace_bytes < na2d_workspace_bytes(p, NA2D_WS_QK_BWD_RPB))
        return NA2D_ERR_WORKSPACE;
    return from_hip(launch_rpb_bwd(to_problem(p), ds, d_rpb, workspace, static_cast<hipStream_t>(stream)));
}

int na2d_qk_bwd_rpb_noalloc(const na2d_problem *p, const void *ds, float *d_rpb, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(ds); NA2D_REQUIRE(d_rpb);
    if (rpb_bwd_partial_bytes(to_problem(p)) > (size_t)NA2D_NOALLOC_SCRATCH_BYTES) return NA2D_ERR_WORKSPACE;
    return from_hip(launch_rpb_bwd_noalloc(to_problem(p), ds, d_rpb, static_cast<hipStream_t>(stream)));
}

// The unfused backward on validated arguments: `ws` holds NA2D_WS_BWD bytes.
static int run_bwd(const Problem &pr, const void *q, const void *k, const void *v, const void *attn, const void *dout,
                   float scale, void *dq, void *dk, void *dv, float *d_rpb, char *ws, hipStream_t s) {
    void *dpds = ws;   // dp, overwritten in place by ds
    const size_t attn_bytes = (pr.queries() * pr.K * pr.K * pr.elem_bytes() + 255) & ~(size_t)255;
    void *rpb_ws = ws + attn_bytes;
    if (bwd_fused_supported(pr)) {   // grad-a and the softmax backward in one kernel: dp never reaches memory
        if (launch_bwd_fused(pr, attn, dout, v, dpds, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);
        if (launch_inverse(pr, attn, dout, 1.0f, dv, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);    // grad-v
    } else {
        if (launch_qk(pr, dout, v, nullptr, 1.0f, dpds, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);  // grad-a
        if (launch_inverse(pr, attn, dout, 1.0f, dv, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);    // grad-v
        if (launch_softmax_bwd(pr, attn, dpds, dpds, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);    // ds
    }
    if (d_rpb && av_rpb_supported(pr)) {   // grad-q also leaves the partial bias gradients: ds is read once less
        float *partial = static_cast<float *>(rpb_ws);
        if (launch_av_rpb(pr, dpds, k, scale, dq, partial, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);
        if (launch_rpb_final_av(pr, partial, d_rpb, av_rpb_split(pr), s) != hipSuccess) return from_hip(hipErrorLaunchFailure);
        if (launch_inverse(pr, dpds, q, scale, dk, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);      // grad-k
    } else {
        if (launch_av(pr, dpds, k, scale, dq, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);           // grad-q
        if (launch_inverse(pr, dpds, q, scale, dk, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);      // grad-k
        if (d_rpb && launch_rpb_bwd(pr, dpds, d_rpb, rpb_ws, s) != hipSuccess) return from_hip(hipErrorLaunchFailure); // grad-b
    }
    return NA2D_OK;
}

int na2d_bwd(const na2d_problem *p, const void *q, const void *k, const void *v, const void *attn, const void *dout,
             float scale, void *dq, void *dk, void *dv, float *d_rpb, void *workspace, size_t workspace_bytes,
             void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(q); NA2D_REQUIRE(k); NA2D_REQUIRE(v); NA2D_REQUIRE(attn); NA2D_REQUIRE(dout);
    NA2D_REQUIRE(dq); NA2D_REQUIRE(dk); NA2D_REQUIRE(dv); NA2D_OPTIONAL(d_rpb);
    if (!workspace || misaligned(workspace) || workspace_bytes < na2d_workspace_bytes(p, NA2D_WS_BWD))
        return NA2D_ERR_WORKSPACE;
    const void *ins[5] = {q, k, v, attn, dout};
    void *outs[4] = {dq, dk, dv, d_rpb};
    for (void *o : outs)
        for (const void *i : ins)
            if (o && o == i) return NA2D_ERR_ALIAS;
    if (dq == dk || dq == dv || dk == dv || d_rpb == dq || d_rpb == dk || d_rpb == dv) return NA2D_ERR_ALIAS;
    return run_bwd(to_problem(p), q, k, v, attn, dout, scale, dq, dk, dv, d_rpb, static_cast<char *>(workspace),
                   static_cast<hipStream_t>(stream));
}

int na2d_fused_bwd_is_fused(const na2d_problem *p) {
    NA2D_CHECK_PROBLEM(p);
    return fused_bwd_supported(to_problem(p)) ? 1 : 0;
}

// Workspace of the fused backward.  Two-kernel path: delta and log2(e) * lse, [B, heads, H, W] fp32 each, then one
// partial bias gradient per workgroup of the first kernel.  Otherwise: the recomputed attention weights, then the
// workspace of the unfused backward.
static size_t fused_bwd_delta_bytes(const Problem &pr) { return (pr.queries() * sizeof(float) + 255) & ~(size_t)255; }
static size_t fused_bwd_attn_bytes(const Problem &pr) { return (pr.queries() * pr.K * pr.K * pr.elem_bytes() + 255) & ~(size_t)255; }

int na2d_fused_bwd(const na2d_problem *p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                   const float *lse, const void *dout, void *dq, void *dk, void *dv, float *d_rpb, void *workspace,
                   size_t workspace_bytes, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    NA2D_REQUIRE(q); NA2D_REQUIRE(k); NA2D_REQUIRE(v); NA2D_OPTIONAL(rpb); NA2D_REQUIRE(lse); NA2D_REQUIRE(dout);
    NA2D_REQUIRE(dq); NA2D_REQUIRE(dk); NA2D_REQUIRE(dv); NA2D_OPTIONAL(d_rpb);
    if (!workspace || misaligned(workspace) || workspace_bytes < na2d_workspace_bytes(p, NA2D_WS_FUSED_BWD))
        return NA2D_ERR_WORKSPACE;
    const void *ins[6] = {q, k, v, rpb, lse, dout};
    void *outs[4] = {dq, dk, dv, d_rpb};
    for (void *o : outs)
        for (const void *i : ins)
            if (o && o == i) return NA2D_ERR_ALIAS;
    if (dq == dk || dq == dv || dk == dv || d_rpb == dq || d_rpb == dk || d_rpb == dv) return NA2D_ERR_ALIAS;
    const Problem pr = to_problem(p);
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    if (fused_bwd_supported(pr)) {
        float *delta = reinterpret_cast<float *>(ws);
        float *lse2 = reinterpret_cast<float *>(ws + fused_bwd_delta_bytes(pr));
        float *partial = d_rpb ? reinterpret_cast<float *>(ws + 2 * fused_bwd_delta_bytes(pr)) : nullptr;
        if (launch_fbwd_q(pr, q, k, v, rpb, scale, lse, dout, dq, delta, lse2, partial, s) != hipSuccess)
            return from_hip(hipErrorLaunchFailure);
        if (launch_fbwd_kv(pr, q, k, v, rpb, scale, lse2, delta, dout, dk, dv, s) != hipSuccess)
            return from_hip(hipErrorLaunchFailure);
        if (d_rpb && launch_rpb_final_av(pr, partial, d_rpb, fused_bwd_split(pr), s) != hipSuccess)
            return from_hip(hipErrorLaunchFailure);
        return NA2D_OK;
    }
    // the attention weights once more (logits, softmax in place), then the unfused steps
    void *attn = ws;
    if (launch_qk(pr, q, k, rpb, scale, attn, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);
    if (launch_softmax(pr, attn, attn, s) != hipSuccess) return from_hip(hipErrorLaunchFailure);
    return run_bwd(pr, q, k, v, attn, dout, scale, dq, dk, dv, d_rpb, ws + fused_bwd_attn_bytes(pr), s);
}

int na2d_debug_indices(const na2d_problem *p, int32_t *key_index, int32_t *rpb_index, void *stream) {
    NA2D_CHECK_PROBLEM(p);
    if (!key_index && !rpb_index) return NA2D_ERR_NULL;
    if ((int64_t)p->H * p->W * p->k * p->k > (int64_t)INT32_MAX) return NA2D_ERR_SHAPE;
    return from_hip(launch_indices(to_problem(p), key_index, rpb_index, static_cast<hipStream_t>(stream)));
}

int na2d_host_axis_tables(int32_t L, int32_t k, int32_t *start, int32_t *qs, int32_t *qe) {
    if (L <= 0) return NA2D_ERR_SHAPE;
    if ((k & 1) == 0 || k < 3 || k > kMaxGenericK) return NA2D_ERR_KERNEL_SIZE;
    if (k > L) return NA2D_ERR_TOO_SMALL;
    for (int i = 0; i < L; ++i) {
        if (start) start[i] = win_start(i, L, k);
        if (qs) qs[i] = inv_first(i, L, k);
        if (qe) qe[i] = inv_last(i, L, k);
    }
    return NA2D_OK;
}

const char *na2d_strerror(int status) {
    switch (status) {
        case NA2D_OK: return "ok";
        case NA2D_ERR_NULL: return "a required pointer is NULL";
        case NA2D_ERR_DTYPE: return "unknown dtype";
        case NA2D_ERR_KERNEL_SIZE: return "kernel size must be odd and between 3 and 63";
        case NA2D_ERR_TOO_SMALL: return "kernel size exceeds the feature map (k > min(H, W))";
        case NA2D_ERR_HEAD_DIM: return "head dim must be 16, 32, 64 or 128";
        case NA2D_ERR_SHAPE: return "non-positive extent or tensor too large";
        case NA2D_ERR_ALIGN: return "pointer is not 16-byte aligned";
        case NA2D_ERR_WORKSPACE: return "workspace missing, misaligned or too small (or the problem exceeds the built-in scratch array)";
        case NA2D_ERR_LAUNCH: return "HIP reported a launch failure";
        case NA2D_ERR_ALIAS: return "an output aliases an input";
        default: return "unknown status";
    }
}

int na2d_version(void) { return 100; }

}  // extern "C"
