// Fused neighbourhood attention forward (arXiv 2204.07143, Eq. 2-4 in one kernel):
//   out_n = softmax_{a,c}( scale * <q_n, k_{rho(n;a,c)}> + B(n, rho(n;a,c)) ) . v_{rho(n;a,c)}
// The K*K logits and weights never reach HBM: the h*w*k^2 attention tensor is the memory
// term of the paper's complexity table (Section 3.3) and fusing removes its round trip.
//
// One workgroup per TY x 16 query tile; the key halo and the value halo of the tile are staged
// once in LDS.  Each thread owns one query and walks its window row by row with a running
// max / running sum (online softmax), rescaling its 32 fp32 accumulators once per window row.
#include "na2d_kernels.hpp"
#include "na2d_tile.hpp"
#include "na2d_valu_cfg.hpp"

namespace na2d {

template <typename T, int K, int TY, int D>
__global__ __launch_bounds__(kTileX *TY) void fused_fwd_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                                const T *__restrict__ v, const T *__restrict__ rpb,
                                                                float scale, T *__restrict__ out,
                                                                float *__restrict__ lse, int H, int W, int heads,
                                                                int tiles_x, int tiles_y, int ntiles) {
    using C = FusedCfg<T, K, TY, D>;
    constexpr int KBYTES = VecTraits<T, D>::kKeyBytes, STRIDE = VecTraits<T, D>::kKeyStride;
    extern __shared__ __align__(16) char lds[];
    char *khalo = lds;
    char *vhalo = lds + C::kHaloBytes;
    float *bias = reinterpret_cast<float *>(lds + 2 * C::kHaloBytes);

    const int t = xcd_contiguous_block(blockIdx.x, gridDim.x);
    if (t >= ntiles) return;
    const TileCoord tc = decode_tile(t, tiles_x, tiles_y);
    const int ty0 = tc.tiy * TY, tx0 = tc.tix * kTileX;
    const int tid = threadIdx.x;
    const int hy0 = win_start(ty0, H, K), hx0 = win_start(tx0, W, K);
    const size_t plane_q = (size_t)tc.plane * H * W;

    load_halo<T, C::HALO_H, C::HALO_W, C::kThreads, false, D>(reinterpret_cast<const char *>(k) + plane_q * KBYTES,
                                                    H, W, hy0, hx0, khalo, tid);
    load_halo<T, C::HALO_H, C::HALO_W, C::kThreads, false, D>(reinterpret_cast<const char *>(v) + plane_q * KBYTES,
                                                    H, W, hy0, hx0, vhalo, tid);
    {
        const int head = tc.plane % heads;
        for (int i = tid; i < C::NB * C::NB; i += C::kThreads)
            bias[i] = rpb ? to_f32(rpb[(size_t)head * C::NB * C::NB + i]) : 0.f;
    }
    workgroup_sync();

    const int lx = tid % kTileX, ly = tid / kTileX;
    const int qy = ty0 + ly, qx = tx0 + lx;
    if (qy < H && qx < W) {
        VecN<T, D> qv;
        load_vec32(qv, reinterpret_cast<const char *>(q) + (plane_q + (size_t)qy * W + qx) * KBYTES);
        const int sy = win_start(qy, H, K), sx = win_start(qx, W, K);
        const int py = sy - qy + (K - 1), px = sx - qx + (K - 1);
        const int hoff = ((sy - hy0) * C::HALO_W + (sx - hx0)) * STRIDE;
        const float *bbase = bias + py * C::NB + px;
        float acc[D];
#pragma unroll
        for (int d = 0; d < D; ++d) acc[d] = 0.f;
        float m = -INFINITY, l = 0.f;
#pragma unroll 1
        for (int a = 0; a < K; ++a) {
            float s[K];
            float rowmax = -INFINITY;
#pragma unroll
            for (int c = 0; c < K; ++c) {
                VecN<T, D> kv;
                lds_load_vec32(kv, khalo + hoff + (a * C::HALO_W + c) * STRIDE);
                s[c] = __builtin_fmaf(scale, dot32(qv, kv), bbase[a * C::NB + c]);
                rowmax = fmaxf(rowmax, s[c]);
            }
            const float mnew = fmaxf(m, rowmax);
            const float corr = __expf(m - mnew);   // exp(-inf) = 0 on the first row
            l *= corr;
#pragma unroll
            for (int d = 0; d < D; ++d) acc[d] *= corr;
#pragma unroll
            for (int c = 0; c < K; ++c) {
                const float e = __expf(s[c] - mnew);
                l += e;
                VecN<T, D> vv;
                lds_load_vec32(vv, vhalo + hoff + (a * C::HALO_W + c) * STRIDE);
                axpy32(acc, e, vv);
            }
            m = mnew;
        }
        const float inv = 1.0f / l;
#pragma unroll
        for (int d = 0; d < D; ++d) acc[d] *= inv;
        store_vec32<T>(reinterpret_cast<char *>(out) + (plane_q + (size_t)qy * W + qx) * KBYTES, acc);
        if (lse) lse[plane_q + (size_t)qy * W + qx] = m + __logf(l);
    }
}

template <typename T, int K, int D>
static hipError_t launch_fused_t(const Problem &p, const void *q, const void *k, const void *v, const void *rpb,
                                 float scale, void *out, float *lse, hipStream_t s) {
    if constexpr (!valu_fits<T, K, D>()) return hipErrorInvalidValue; else {
    constexpr int TY = tile_rows<FusedCfg, T, K, D>();
    using C = FusedCfg<T, K, TY, D>;
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + TY - 1) / TY;
    const int ntiles = tiles_x * tiles_y * p.planes();
    auto kern = fused_fwd_kernel<T, K, TY, D>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(ntiles)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(q), static_cast<const T *>(k), static_cast<const T *>(v),
                       static_cast<const T *>(rpb), scale, static_cast<T *>(out), lse, p.H, p.W, p.heads, tiles_x,
                       tiles_y, ntiles);
    return hipGetLastError();
    }
}

hipError_t launch_fused_fwd(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                            void *out, float *lse, hipStream_t s) {
    if (fused_mfma_supported(p)) return launch_fused_mfma(p, q, k, v, rpb, scale, out, lse, s);
    if (generic_window(p)) return launch_fused_generic(p, q, k, v, rpb, scale, out, lse, s);
    NA2D_DISPATCH_T(p.dtype, NA2D_DISPATCH_K(p.K, NA2D_DISPATCH_D(p.D, return (launch_fused_t<T, K, D>(p, q, k, v, rpb, scale, out, lse, s)))));
    return hipErrorInvalidValue;
}

}  // namespace na2d
