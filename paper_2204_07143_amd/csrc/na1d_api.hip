// C ABI of the 1D Neighborhood Attention entry points: argument validation (host only, before any HIP
// call) and dispatch to the kernel launchers.
#include <stdint.h>

#include "na1d.h"
#include "na1d_kernels.hpp"

namespace na1d {

static int validate(const na1d_problem *p) {
    if (!p) return NA2D_ERR_NULL;
    if (p->dtype != NA2D_F32 && p->dtype != NA2D_F16 && p->dtype != NA2D_BF16) return NA2D_ERR_DTYPE;
    if (p->B <= 0 || p->heads <= 0 || p->L <= 0 || p->D <= 0 || p->k <= 0) return NA2D_ERR_SHAPE;
    if ((p->k & 1) == 0 || p->k < 3 || p->k > kMaxK) return NA2D_ERR_KERNEL_SIZE;
    if (p->k > p->L) return NA2D_ERR_TOO_SMALL;
    if (p->D != 32) return NA2D_ERR_HEAD_DIM;
    // element counts of every tensor fit int32 (byte offsets inside the kernels are 64-bit)
    const int64_t nq = (int64_t)p->B * p->heads * p->L;
    const int64_t widest = p->k > p->D ? p->k : p->D;
    if (nq * widest > (int64_t)INT32_MAX) return NA2D_ERR_SHAPE;
    // ... and one (batch, head) plane of any tensor stays below 2^31 bytes
    const int64_t elem = p->dtype == NA2D_F32 ? 4 : 2;
    if ((int64_t)p->L * widest * elem > (int64_t)INT32_MAX) return NA2D_ERR_SHAPE;
    return NA2D_OK;
}

static inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
static Problem to_problem(const na1d_problem *p) { return Problem{p->B, p->heads, p->L, p->k, p->dtype}; }
static int from_hip(hipError_t e) {
    if (e == hipSuccess) return NA2D_OK;
    (void)hipGetLastError();   // leave no stale error behind for the caller's next HIP call
    return NA2D_ERR_LAUNCH;
}

}  // namespace na1d

using namespace na1d;

#define NA1D_CHECK_PROBLEM(p)           \
    do {                                \
        int st_ = validate(p);          \
        if (st_ != NA2D_OK) return st_; \
    } while (0)
#define NA1D_REQUIRE(ptr)                           \
    do {                                            \
        if (!(ptr)) return NA2D_ERR_NULL;           \
        if (misaligned(ptr)) return NA2D_ERR_ALIGN; \
    } while (0)
#define NA1D_OPTIONAL(ptr)                                   \
    do {                                                     \
        if ((ptr) && misaligned(ptr)) return NA2D_ERR_ALIGN; \
    } while (0)

extern "C" {

int na1d_validate_problem(const na1d_problem *p) { return validate(p); }

int na1d_qk_rpb(const na1d_problem *p, const void *q, const void *k, const void *rpb, float scale, void *logits,
                void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(q); NA1D_REQUIRE(k); NA1D_REQUIRE(logits); NA1D_OPTIONAL(rpb);
    if (logits == q || logits == k) return NA2D_ERR_ALIAS;
    return from_hip(launch_qk(to_problem(p), q, k, rpb, scale, logits, static_cast<hipStream_t>(stream)));
}

int na1d_softmax(const na1d_problem *p, const void *logits, void *p_out, void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(logits); NA1D_REQUIRE(p_out);
    return from_hip(launch_softmax(to_problem(p), logits, p_out, static_cast<hipStream_t>(stream)));
}

int na1d_av(const na1d_problem *p, const void *attn, const void *v, void *out, void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(attn); NA1D_REQUIRE(v); NA1D_REQUIRE(out);
    if (out == attn || out == v) return NA2D_ERR_ALIAS;
    return from_hip(launch_av(to_problem(p), attn, v, 1.0f, out, static_cast<hipStream_t>(stream)));
}

int na1d_fused_fwd(const na1d_problem *p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                   void *out, float *lse, void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(q); NA1D_REQUIRE(k); NA1D_REQUIRE(v); NA1D_REQUIRE(out); NA1D_OPTIONAL(rpb); NA1D_OPTIONAL(lse);
    if (out == q || out == k || out == v) return NA2D_ERR_ALIAS;
    return from_hip(launch_fused_fwd(to_problem(p), q, k, v, rpb, scale, out, lse, static_cast<hipStream_t>(stream)));
}

int na1d_av_bwd_p(const na1d_problem *p, const void *dout, const void *v, void *dp, void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(dout); NA1D_REQUIRE(v); NA1D_REQUIRE(dp);
    if (dp == dout || dp == v) return NA2D_ERR_ALIAS;
    return from_hip(launch_qk(to_problem(p), dout, v, nullptr, 1.0f, dp, static_cast<hipStream_t>(stream)));
}

int na1d_av_bwd_v(const na1d_problem *p, const void *attn, const void *dout, void *dv, void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(attn); NA1D_REQUIRE(dout); NA1D_REQUIRE(dv);
    if (dv == attn || dv == dout) return NA2D_ERR_ALIAS;
    return from_hip(launch_inverse(to_problem(p), attn, dout, 1.0f, dv, static_cast<hipStream_t>(stream)));
}

int na1d_softmax_bwd(const na1d_problem *p, const void *attn, const void *dp, void *ds, void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(attn); NA1D_REQUIRE(dp); NA1D_REQUIRE(ds);
    if (ds == attn) return NA2D_ERR_ALIAS;
    return from_hip(launch_softmax_bwd(to_problem(p), attn, dp, ds, static_cast<hipStream_t>(stream)));
}

int na1d_qk_bwd_q(const na1d_problem *p, const void *ds, const void *k, float scale, void *dq, void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(ds); NA1D_REQUIRE(k); NA1D_REQUIRE(dq);
    if (dq == ds || dq == k) return NA2D_ERR_ALIAS;
    return from_hip(launch_av(to_problem(p), ds, k, scale, dq, static_cast<hipStream_t>(stream)));
}

int na1d_qk_bwd_k(const na1d_problem *p, const void *ds, const void *q, float scale, void *dk, void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(ds); NA1D_REQUIRE(q); NA1D_REQUIRE(dk);
    if (dk == ds || dk == q) return NA2D_ERR_ALIAS;
    return from_hip(launch_inverse(to_problem(p), ds, q, scale, dk, static_cast<hipStream_t>(stream)));
}

size_t na1d_workspace_bytes(const na1d_problem *p) {
    if (validate(p) != NA2D_OK) return 0;
    return rpb_workspace_bytes(to_problem(p));
}

int na1d_qk_bwd_rpb(const na1d_problem *p, const void *ds, float *d_rpb, void *workspace, size_t workspace_bytes,
                    void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(ds); NA1D_REQUIRE(d_rpb);
    if (!workspace || misaligned(workspace) || workspace_bytes < rpb_workspace_bytes(to_problem(p))) return NA2D_ERR_WORKSPACE;
    return from_hip(launch_rpb_grad(to_problem(p), ds, d_rpb, workspace, static_cast<hipStream_t>(stream)));
}

size_t na1d_fused_bwd_workspace_bytes(const na1d_problem *p) {
    if (validate(p) != NA2D_OK) return 0;
    return fused_bwd_workspace_bytes(to_problem(p));
}

int na1d_fused_bwd(const na1d_problem *p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                   const float *lse, const void *dout, void *dq, void *dk, void *dv, float *d_rpb, void *workspace,
                   size_t workspace_bytes, void *stream) {
    NA1D_CHECK_PROBLEM(p);
    NA1D_REQUIRE(q); NA1D_REQUIRE(k); NA1D_REQUIRE(v); NA1D_OPTIONAL(rpb); NA1D_REQUIRE(lse); NA1D_REQUIRE(dout);
    NA1D_REQUIRE(dq); NA1D_REQUIRE(dk); NA1D_REQUIRE(dv); NA1D_OPTIONAL(d_rpb);
    if (!workspace || misaligned(workspace) || workspace_bytes < fused_bwd_workspace_bytes(to_problem(p))) return NA2D_ERR_WORKSPACE;
    const void *ins[6] = {q, k, v, rpb, lse, dout};
    void *outs[4] = {dq, dk, dv, d_rpb};
    for (void *o : outs)
        for (const void *i : ins)
            if (o && o == i) return NA2D_ERR_ALIAS;
    if (dq == dk || dq == dv || dk == dv) return NA2D_ERR_ALIAS;
    return from_hip(launch_fused_bwd(to_problem(p), q, k, v, rpb, scale, lse, dout, dq, dk, dv, d_rpb, workspace,
                                     static_cast<hipStream_t>(stream)));
}

}  // extern "C"
