// Neighbourhood weighted sum: out[n, :] = scale * sum_{a, c} w[n, a, c] * y_{rho(n; a, c)}
// (arXiv 2204.07143, Eq. 3-4: attention weights times neighbouring values; with w = ds,
// y = k and scale = 1/sqrt(d) it is grad-q of the backward pass, Appendix A).
//
// Same tiling as the logits kernel: the value halo of a TY x 16 query tile is staged once in
// LDS; the tile's weights (contiguous per tile row in global memory) are staged through LDS
// with 16-byte loads; each thread owns one query and accumulates its 32 outputs in fp32.
#include "na2d_kernels.hpp"
#include "na2d_tile.hpp"
#include "na2d_valu_cfg.hpp"

namespace na2d {

template <typename T, int K, int TY, int D>
__global__ __launch_bounds__(kTileX *TY) void av_kernel(const T *__restrict__ w, const T *__restrict__ y, float scale,
                                                         T *__restrict__ out, int H, int W, int tiles_x, int tiles_y,
                                                         int ntiles) {
    using C = AvCfg<T, K, TY, D>;
    constexpr int KBYTES = VecTraits<T, D>::kKeyBytes, STRIDE = VecTraits<T, D>::kKeyStride;
    extern __shared__ __align__(16) char lds[];
    char *halo = lds;
    char *rows = lds + C::kHaloBytes;

    const int t = xcd_contiguous_block(blockIdx.x, gridDim.x);
    if (t >= ntiles) return;
    const TileCoord tc = decode_tile(t, tiles_x, tiles_y);
    const int ty0 = tc.tiy * TY, tx0 = tc.tix * kTileX;
    const int tid = threadIdx.x;
    const int hy0 = win_start(ty0, H, K), hx0 = win_start(tx0, W, K);
    const size_t plane_q = (size_t)tc.plane * H * W;

    load_halo<T, C::HALO_H, C::HALO_W, C::kThreads, false, D>(reinterpret_cast<const char *>(y) + plane_q * KBYTES,
                                                    H, W, hy0, hx0, halo, tid);
    {
        const int wave = tid / kWave, lane = tid % kWave;
        constexpr int kWaves = (C::kThreads + kWave - 1) / kWave;
        const int nvalid = (W - tx0) < kTileX ? (W - tx0) : kTileX;
        for (int r = wave; r < TY; r += kWaves) {
            if (ty0 + r >= H) break;
            const size_t g0r = (plane_q + (size_t)(ty0 + r) * W + tx0) * C::KK * sizeof(T);
            stage_in<T, kTileX * C::KK * (int)sizeof(T), kWave>(reinterpret_cast<const char *>(w), g0r,
                                                                nvalid * C::KK * (int)sizeof(T), rows + r * C::kRowRegion, lane);
        }
    }
    workgroup_sync();

    const int lx = tid % kTileX, ly = tid / kTileX;
    const int qy = ty0 + ly, qx = tx0 + lx;
    if (qy < H && qx < W) {
        const size_t g0 = (plane_q + (size_t)qy * W + tx0) * C::KK * sizeof(T);
        const int sy = win_start(qy, H, K), sx = win_start(qx, W, K);
        const char *vbase = halo + ((sy - hy0) * C::HALO_W + (sx - hx0)) * STRIDE;
        const T *wrow = reinterpret_cast<const T *>(rows + ly * C::kRowRegion + (int)(g0 & 15)) + lx * C::KK;
        float acc[D];
#pragma unroll
        for (int d = 0; d < D; ++d) acc[d] = 0.f;
#pragma unroll 1
        for (int a = 0; a < K; ++a) {
#pragma unroll
            for (int c = 0; c < K; ++c) {
                VecN<T, D> vv;
                lds_load_vec32(vv, vbase + (a * C::HALO_W + c) * STRIDE);
                axpy32(acc, to_f32(wrow[a * K + c]), vv);
            }
        }
#pragma unroll
        for (int d = 0; d < D; ++d) acc[d] *= scale;
        store_vec32<T>(reinterpret_cast<char *>(out) + (plane_q + (size_t)qy * W + qx) * KBYTES, acc);
    }
}

template <typename T, int K, int D>
static hipError_t launch_av_t(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s) {
    if constexpr (!valu_fits<T, K, D>()) return hipErrorInvalidValue; else {
    constexpr int TY = tile_rows<AvCfg, T, K, D>();
    using C = AvCfg<T, K, TY, D>;
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + TY - 1) / TY;
    const int ntiles = tiles_x * tiles_y * p.planes();
    auto kern = av_kernel<T, K, TY, D>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(ntiles)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(w), static_cast<const T *>(y), scale, static_cast<T *>(out), p.H, p.W,
                       tiles_x, tiles_y, ntiles);
    return hipGetLastError();
    }
}

hipError_t launch_av(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s) {
    if (av_mfma_supported(p)) return launch_av_mfma(p, w, y, scale, out, s);
    if (generic_window(p)) return launch_av_generic(p, w, y, scale, out, s);
    NA2D_DISPATCH_T(p.dtype, NA2D_DISPATCH_K(p.K, NA2D_DISPATCH_D(p.D, return (launch_av_t<T, K, D>(p, w, y, scale, out, s)))));
    return hipErrorInvalidValue;
}

}  // namespace na2d
