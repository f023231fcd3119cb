// Internal launch interface between the C ABI layer and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lds_attr.hpp"
#include "na2d.h"

namespace na2d {

struct Problem {
    int B, heads, H, W, K, dtype;
    int D = 32;
    int planes() const { return B * heads; }
    size_t queries() const { return (size_t)B * heads * H * W; }
    int elem_bytes() const { return dtype == NA2D_F32 ? 4 : 2; }
};

// Window sides: 3..13 (odd) run the tuned kernels, 15..63 (odd) the run-time-K kernels of na2d_generic.hip.
constexpr int kMaxTunedK = 13, kMaxGenericK = 63;
bool generic_window(const Problem &p);   // neither the tuned window sides nor a plain-ALU tile that fits the LDS
bool untuned_window(const Problem &p);   // k beyond the tuned sides (what the kernels that do not depend on D ask)
hipError_t launch_qk_generic(const Problem &p, const void *x, const void *y, const void *rpb, float scale, void *logits,
                             hipStream_t s);
hipError_t launch_av_generic(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s);
hipError_t launch_inverse_generic(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s);
hipError_t launch_softmax_generic(const Problem &p, const void *in, void *out, hipStream_t s);
hipError_t launch_softmax_bwd_generic(const Problem &p, const void *attn, const void *dp, void *ds, hipStream_t s);
hipError_t launch_fused_generic(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                                void *out, float *lse, hipStream_t s);
size_t rpb_generic_workspace_bytes(const Problem &p);
hipError_t launch_rpb_generic(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s);
hipError_t launch_indices_generic(const Problem &p, int32_t *key_index, int32_t *rpb_index, hipStream_t s);

// logits = scale * <x, y_window> + bias   (QK+RPB, and grad-a with x = dout, y = v, no bias)
hipError_t launch_qk(const Problem &p, const void *x, const void *y, const void *rpb, float scale, void *logits,
                     hipStream_t s);
// the same contraction on the matrix cores (f16 / bf16 only)
hipError_t launch_qk_mfma(const Problem &p, const void *x, const void *y, const void *rpb, float scale, void *logits,
                          hipStream_t s);
// D = 32, and for k <= 7 also D = 64 (two 32-channel slices accumulated in the matrix cores)
bool qk_mfma_supported(const Problem &p);
// grad-a fused with the softmax backward (f16 / bf16, K <= 7): ds from attn, dout and v
bool bwd_fused_supported(const Problem &p);
hipError_t launch_bwd_fused(const Problem &p, const void *attn, const void *dout, const void *v, void *ds, hipStream_t s);
// out = scale * sum_window w * y          (AV, and grad-q with w = ds, y = k)
hipError_t launch_av(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s);
hipError_t launch_av_mfma(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s);
// the matrix-core kernel takes any multiple of 32 channels, one launch per 32-channel slice
bool av_mfma_supported(const Problem &p);
// out_j = scale * sum_{inverse neighbourhood} w[i, slot(i, j)] * x_i   (grad-v, grad-k)
hipError_t launch_inverse(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s);
bool inverse_ring_supported(const Problem &p);
hipError_t launch_inverse_ring(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s);
bool inverse_mfma_supported(const Problem &p);
// what the two kernels above do not take (K >= 11, very short axes): the query rectangle streamed through LDS two rows at a time
bool inverse_rows_supported(const Problem &p);
hipError_t launch_inverse_rows(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s);
hipError_t launch_inverse_mfma(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s);
hipError_t launch_softmax(const Problem &p, const void *logits, void *out, hipStream_t s);
hipError_t launch_softmax_bwd(const Problem &p, const void *attn, const void *dp, void *ds, hipStream_t s);
size_t rpb_bwd_workspace_bytes(const Problem &p);
hipError_t launch_rpb_bwd(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s);
// the same with the partials in the library's own device array (NA2D_NOALLOC_SCRATCH_BYTES); bytes it needs
size_t rpb_bwd_partial_bytes(const Problem &p);
hipError_t launch_rpb_bwd_noalloc(const Problem &p, const void *ds, float *d_rpb, hipStream_t s);
// grad-q that also leaves partial bias gradients (f16 / bf16, K <= 7): workgroup wg of the launch covers
// tile position wg % npos, head (wg / npos) % heads and batch range wg / (npos * heads) of `splits`
struct AvRpbSplit {
    int npos, splits;
};
// Partial bias gradients in a workspace: one row of rpb_cell_stride(cells) floats per workgroup of the kernel that
// leaves them (a whole number of 16-byte chunks; the floats past `cells` are never written and never used), the
// rows of a head next to each other: row (h * n + i) is partial i of head h, n partials per head.  The final
// reduction then walks a head's partials with a constant stride, four cells per lane and load.
__host__ __device__ constexpr int rpb_cell_stride(int cells) { return (cells + 3) & ~3; }
bool av_rpb_supported(const Problem &p);
AvRpbSplit av_rpb_split(const Problem &p);
hipError_t launch_av_rpb(const Problem &p, const void *w, const void *y, float scale, void *out, float *rpb_partial,
                         hipStream_t s);
hipError_t launch_rpb_final_av(const Problem &p, const float *partial, float *d_rpb, AvRpbSplit sp, hipStream_t s);
// fused backward (two kernels): query patches -> dq, delta, partial bias gradients; key patches -> dk, dv
bool fused_bwd_supported(const Problem &p);
AvRpbSplit fused_bwd_split(const Problem &p);
// (the first also leaves log2(e) * lse beside delta, which is what the second reads as `lse2`)
hipError_t launch_fbwd_q(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                         const float *lse, const void *dout, void *dq, float *delta, float *lse2, float *rpb_partial,
                         hipStream_t s);
hipError_t launch_fbwd_kv(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                          const float *lse2, const float *delta, const void *dout, void *dk, void *dv, hipStream_t s);
hipError_t launch_fused_fwd(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                            void *out, float *lse, hipStream_t s);
// D = 32, and for k <= 7 also D = 64 (two 32-channel slices)
bool fused_mfma_supported(const Problem &p);
hipError_t launch_fused_mfma(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                             void *out, float *lse, hipStream_t s);
hipError_t launch_indices(const Problem &p, int32_t *key_index, int32_t *rpb_index, hipStream_t s);

}  // namespace na2d

// Expands BODY once with `T` bound to the storage type and `K` to the window side.
#define NA2D_DISPATCH_K(kval, ...)                                   \
    switch (kval) {                                                  \
        case 3: { constexpr int K = 3; __VA_ARGS__; } break;         \
        case 5: { constexpr int K = 5; __VA_ARGS__; } break;         \
        case 7: { constexpr int K = 7; __VA_ARGS__; } break;         \
        case 9: { constexpr int K = 9; __VA_ARGS__; } break;         \
        case 11: { constexpr int K = 11; __VA_ARGS__; } break;       \
        case 13: { constexpr int K = 13; __VA_ARGS__; } break;       \
        default: return hipErrorInvalidValue;                        \
    }
// Head dims the plain-ALU kernels are built for (the matrix-core kernels serve D = 32 only).
#define NA2D_DISPATCH_D(dval, ...)                                    \
    switch (dval) {                                                   \
        case 16: { constexpr int D = 16; __VA_ARGS__; } break;        \
        case 32: { constexpr int D = 32; __VA_ARGS__; } break;        \
        case 64: { constexpr int D = 64; __VA_ARGS__; } break;        \
        case 128: { constexpr int D = 128; __VA_ARGS__; } break;      \
        default: return hipErrorInvalidValue;                         \
    }
#define NA2D_DISPATCH_T(dtval, ...)                                                  \
    switch (dtval) {                                                                 \
        case NA2D_F32: { using T = float; __VA_ARGS__; } break;                      \
        case NA2D_F16: { using T = ::na2d::f16_t; __VA_ARGS__; } break;              \
        case NA2D_BF16: { using T = ::na2d::bf16_t; __VA_ARGS__; } break;            \
        default: return hipErrorInvalidValue;                                        \
    }
