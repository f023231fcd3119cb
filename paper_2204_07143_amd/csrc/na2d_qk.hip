// Neighbourhood logits: logits[n, a, c] = scale * <x_n, y_{rho(n; a, c)}> + bias
// (arXiv 2204.07143, Eq. 2: QK + relative positional bias; the same contraction with
// x = dout, y = v and no bias is grad-a of the backward pass, Appendix A).
//
// One workgroup per TY x 16 query tile: the (TY+K-1) x (16+K-1) key halo is staged once in
// LDS, each thread owns one query (held in registers in its storage type) and walks its
// K x K window with packed dot products (v_dot2 for f16/bf16), and the tile's logits are
// gathered in LDS so that they leave the chip as 16-byte coalesced stores (a query's K*K
// logits are not a multiple of 16 bytes, so stores are issued per contiguous tile row).
#include <stdlib.h>
#include <string.h>

#include "na2d_kernels.hpp"
#include "na2d_tile.hpp"
#include "na2d_valu_cfg.hpp"

namespace na2d {

template <typename T, int K, int TY, int D>
__global__ __launch_bounds__(kTileX *TY) void qk_kernel(const T *__restrict__ x, const T *__restrict__ y,
                                                         const T *__restrict__ rpb, float scale,
                                                         T *__restrict__ logits, int H, int W, int heads,
                                                         int tiles_x, int tiles_y, int ntiles) {
    using C = QkCfg<T, K, TY, D>;
    constexpr int KBYTES = VecTraits<T, D>::kKeyBytes, STRIDE = VecTraits<T, D>::kKeyStride;
    extern __shared__ __align__(16) char lds[];
    char *halo = lds;
    float *bias = reinterpret_cast<float *>(lds + C::kHaloBytes);
    char *rows = lds + C::kHaloBytes + C::kBiasBytes;

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
        const int head = tc.plane % heads;
        for (int i = tid; i < C::NB * C::NB; i += C::kThreads)
            bias[i] = rpb ? to_f32(rpb[(size_t)head * C::NB * C::NB + i]) : 0.f;
    }
    workgroup_sync();

    const int lx = tid % kTileX, ly = tid / kTileX;
    const int qy = ty0 + ly, qx = tx0 + lx;
    // Global byte offset of this tile row's run of logits; its low 4 bits are mirrored in LDS.
    const size_t g0 = (plane_q + (size_t)qy * W + tx0) * C::KK * sizeof(T);
    if (qy < H && qx < W) {
        VecN<T, D> qv;
        load_vec32(qv, reinterpret_cast<const char *>(x) + (plane_q + (size_t)qy * W + qx) * KBYTES);
        const int sy = win_start(qy, H, K), sx = win_start(qx, W, K);
        const int py = sy - qy + (K - 1), px = sx - qx + (K - 1);
        const char *kbase = halo + ((sy - hy0) * C::HALO_W + (sx - hx0)) * STRIDE;
        const float *bbase = bias + py * C::NB + px;
        T *orow = reinterpret_cast<T *>(rows + ly * C::kRowRegion + (int)(g0 & 15)) + lx * C::KK;
#pragma unroll 1
        for (int a = 0; a < K; ++a) {
#pragma unroll
            for (int c = 0; c < K; ++c) {
                VecN<T, D> kv;
                lds_load_vec32(kv, kbase + (a * C::HALO_W + c) * STRIDE);
                const float dot = dot32(qv, kv);
                orow[a * K + c] = from_f32<T>(__builtin_fmaf(scale, dot, bbase[a * C::NB + c]));
            }
        }
    }
    workgroup_sync();

    // Each wave streams out whole tile rows: one row's logits are contiguous in global memory.
    const int wave = tid / kWave, lane = tid % kWave;
    constexpr int kWaves = (C::kThreads + kWave - 1) / kWave;
    const int nvalid = (W - tx0) < kTileX ? (W - tx0) : kTileX;
    for (int r = wave; r < TY; r += kWaves) {
        if (ty0 + r >= H) break;
        const size_t g0r = (plane_q + (size_t)(ty0 + r) * W + tx0) * C::KK * sizeof(T);
        stage_out<T, kTileX * C::KK * (int)sizeof(T), kWave>(reinterpret_cast<char *>(logits), g0r,
                                                             nvalid * C::KK * (int)sizeof(T), rows + r * C::kRowRegion, lane);
    }
}

template <typename T, int K, int D>
static hipError_t launch_qk_t(const Problem &p, const void *x, const void *y, const void *rpb, float scale,
                              void *logits, hipStream_t s) {
    if constexpr (!valu_fits<T, K, D>()) return hipErrorInvalidValue; else {
    constexpr int TY = tile_rows<QkCfg, T, K, D>();
    using C = QkCfg<T, K, TY, D>;
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + TY - 1) / TY;
    const int ntiles = tiles_x * tiles_y * p.planes();
    auto kern = qk_kernel<T, K, TY, D>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(ntiles)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(x), static_cast<const T *>(y), static_cast<const T *>(rpb), scale,
                       static_cast<T *>(logits), p.H, p.W, p.heads, tiles_x, tiles_y, ntiles);
    return hipGetLastError();
    }
}

// do the LDS tiles of every plain-ALU kernel fit for this dtype, window and head dim?
bool head_dim_supported(int dtype, int K, int D) {
    if (K > kMaxTunedK) return false;
    auto probe = [&]() -> hipError_t {
        NA2D_DISPATCH_T(dtype, NA2D_DISPATCH_K(K, NA2D_DISPATCH_D(D, return (valu_fits<T, K, D>() ? hipSuccess : hipErrorInvalidValue))));
        return hipErrorInvalidValue;
    };
    return probe() == hipSuccess;
}

hipError_t launch_qk(const Problem &p, const void *x, const void *y, const void *rpb, float scale, void *logits,
                     hipStream_t s) {
    // matrix cores where they take the problem; else the tiled plain-ALU kernel while its tile fits the LDS; else the
    // kernels that stage nothing
    if (qk_mfma_supported(p)) return launch_qk_mfma(p, x, y, rpb, scale, logits, s);
    if (generic_window(p)) return launch_qk_generic(p, x, y, rpb, scale, logits, s);
    NA2D_DISPATCH_T(p.dtype, NA2D_DISPATCH_K(p.K, NA2D_DISPATCH_D(p.D, return (launch_qk_t<T, K, D>(p, x, y, rpb, scale, logits, s)))));
    return hipErrorInvalidValue;
}

}  // namespace na2d
