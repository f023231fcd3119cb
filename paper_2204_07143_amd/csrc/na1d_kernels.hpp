// Internal launch interface of the 1D Neighborhood Attention kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "na1d.h"

namespace na1d {

struct Problem {
    int B, heads, L, K, dtype;
    int planes() const { return B * heads; }
};

constexpr int kMaxK = 63;

// logits = scale * <x, y over the window> + bias     (QK+RPB; grad-a with x = dout, y = v, no bias)
hipError_t launch_qk(const Problem &p, const void *x, const void *y, const void *rpb, float scale, void *out, hipStream_t s);
// out = scale * sum over the window of w * y           (AV; grad-q with w = ds, y = k)
hipError_t launch_av(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s);
// out_j = scale * sum over the queries that see j of w[i, j - s(i)] * x_i   (grad-v, grad-k)
hipError_t launch_inverse(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s);
hipError_t launch_softmax(const Problem &p, const void *logits, void *out, hipStream_t s);
hipError_t launch_softmax_bwd(const Problem &p, const void *attn, const void *dp, void *ds, hipStream_t s);
hipError_t launch_fused_fwd(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                            void *out, float *lse, hipStream_t s);
size_t rpb_workspace_bytes(const Problem &p);
hipError_t launch_rpb_grad(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s);
// whole backward from q, k, v, rpb, dout and the forward's log-sum-exp (no k-wide tensor in memory)
size_t fused_bwd_workspace_bytes(const Problem &p);
hipError_t launch_fused_bwd(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                            const float *lse, const void *dout, void *dq, void *dk, void *dv, float *d_rpb, void *workspace,
                            hipStream_t s);

}  // namespace na1d
