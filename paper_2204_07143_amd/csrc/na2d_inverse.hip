// Gradients that sum over queries, gathered through the inverse neighbourhood:
//   out_j = scale * sum over queries i whose window holds j of w[i, slot(i, j)] * x_i
// (grad-v with w = attention weights, x = dout; grad-k with w = ds, x = q;
// arXiv 2204.07143, Appendix A lists both among the package's gradient kernels).
//
// The queries that see key j form a contiguous rectangle [inv_first, inv_last] on each axis
// (K wide in the interior, up to K + (K-1)/2 next to a border), so each key gathers its own
// sum: no atomics, fixed summation order, bitwise reproducible.  One workgroup per TY x 16
// key tile; the x vectors of the tile's query rectangle are staged once in LDS.
#include "na2d_kernels.hpp"
#include "na2d_tile.hpp"
#include "na2d_valu_cfg.hpp"

namespace na2d {

template <typename T, int K, int TY, int D>
__global__ __launch_bounds__(kTileX *TY) void inverse_kernel(const T *__restrict__ w, const T *__restrict__ x,
                                                              float scale, T *__restrict__ out, int H, int W,
                                                              int tiles_x, int tiles_y, int ntiles) {
    using C = InvCfg<T, K, TY, D>;
    constexpr int KBYTES = VecTraits<T, D>::kKeyBytes, STRIDE = VecTraits<T, D>::kKeyStride;
    extern __shared__ __align__(16) char lds[];

    const int t = xcd_contiguous_block(blockIdx.x, gridDim.x);
    if (t >= ntiles) return;
    const TileCoord tc = decode_tile(t, tiles_x, tiles_y);
    const int ty0 = tc.tiy * TY, tx0 = tc.tix * kTileX;
    const int tid = threadIdx.x;
    const int ry0 = inv_first(ty0, H, K), rx0 = inv_first(tx0, W, K);
    const size_t plane_q = (size_t)tc.plane * H * W;
    const char *xplane = reinterpret_cast<const char *>(x) + plane_q * KBYTES;

    load_halo<T, C::RECT_H, C::RECT_W, C::kThreads, false, D>(xplane, H, W, ry0, rx0, lds, tid);
    workgroup_sync();

    const int lx = tid % kTileX, ly = tid / kTileX;
    const int jy = ty0 + ly, jx = tx0 + lx;
    if (jy < H && jx < W) {
        const int fy = inv_first(jy, H, K), ey = inv_last(jy, H, K);
        const int fx = inv_first(jx, W, K), ex = inv_last(jx, W, K);
        float acc[D];
#pragma unroll
        for (int d = 0; d < D; ++d) acc[d] = 0.f;
        for (int iy = fy; iy <= ey; ++iy) {
            const int a = jy - win_start(iy, H, K);
            const T *wrow = w + (plane_q + (size_t)iy * W) * C::KK + a * K;
            for (int ix = fx; ix <= ex; ++ix) {
                const int c = jx - win_start(ix, W, K);
                const float wt = to_f32(wrow[(size_t)ix * C::KK + c]);
                VecN<T, D> xv;
                const int ry = iy - ry0, rx = ix - rx0;
                if (ry < C::RECT_H && rx < C::RECT_W)
                    lds_load_vec32(xv, lds + (ry * C::RECT_W + rx) * STRIDE);
                else
                    load_vec32(xv, xplane + ((size_t)iy * W + ix) * KBYTES);
                axpy32(acc, wt, xv);
            }
        }
#pragma unroll
        for (int d = 0; d < D; ++d) acc[d] *= scale;
        store_vec32<T>(reinterpret_cast<char *>(out) + (plane_q + (size_t)jy * W + jx) * KBYTES, acc);
    }
}

template <typename T, int K, int D>
static hipError_t launch_inverse_t(const Problem &p, const void *w, const void *x, float scale, void *out,
                                   hipStream_t s) {
    if constexpr (!valu_fits<T, K, D>()) return hipErrorInvalidValue; else {
    constexpr int TY = tile_rows<InvCfg, T, K, D>();
    using C = InvCfg<T, K, TY, D>;
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + TY - 1) / TY;
    const int ntiles = tiles_x * tiles_y * p.planes();
    auto kern = inverse_kernel<T, K, TY, D>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(ntiles)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(w), static_cast<const T *>(x), scale, static_cast<T *>(out), p.H, p.W,
                       tiles_x, tiles_y, ntiles);
    return hipGetLastError();
    }
}

hipError_t launch_inverse(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s) {
    if (!untuned_window(p)) {
        if (inverse_ring_supported(p)) return launch_inverse_ring(p, w, x, scale, out, s);
        if (inverse_mfma_supported(p)) return launch_inverse_mfma(p, w, x, scale, out, s);
        if (inverse_rows_supported(p)) return launch_inverse_rows(p, w, x, scale, out, s);
    }
    if (generic_window(p)) return launch_inverse_generic(p, w, x, scale, out, s);
    NA2D_DISPATCH_T(p.dtype, NA2D_DISPATCH_K(p.K, NA2D_DISPATCH_D(p.D, return (launch_inverse_t<T, K, D>(p, w, x, scale, out, s)))));
    return hipErrorInvalidValue;
}

}  // namespace na2d
