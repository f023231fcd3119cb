// LDS footprints and tile heights of the plain-ALU 2D kernels, shared by the kernels and by the argument
// validation of the C ABI (a head dim / kernel size pair is accepted only if every kernel's tile fits the
// 160 KB LDS of a compute unit at the smallest tile height).
#pragma once

#include "na2d_common.hpp"
#include "na2d_tile.hpp"

namespace na2d {

constexpr int kLdsLimit = 160 * 1024;

template <typename T, int K, int TY, int D = kHeadDim>
struct QkCfg {
    static constexpr int HALO_H = TY + K - 1, HALO_W = kTileX + K - 1;
    static constexpr int NB = 2 * K - 1;
    static constexpr int KK = K * K;
    static constexpr int kThreads = kTileX * TY;
    static constexpr int kHaloBytes = HALO_H * HALO_W * VecTraits<T, D>::kKeyStride;
    static constexpr int kBiasBytes = ((NB * NB * 4) + 15) & ~15;
    static constexpr int kRowRegion = mirror_bytes(kTileX * KK * (int)sizeof(T));
    static constexpr int kLdsBytes = kHaloBytes + kBiasBytes + TY * kRowRegion;
};

template <typename T, int K, int TY, int D = kHeadDim>
struct AvCfg {
    static constexpr int HALO_H = TY + K - 1, HALO_W = kTileX + K - 1;
    static constexpr int KK = K * K;
    static constexpr int kThreads = kTileX * TY;
    static constexpr int kHaloBytes = HALO_H * HALO_W * VecTraits<T, D>::kKeyStride;
    static constexpr int kRowRegion = mirror_bytes(kTileX * KK * (int)sizeof(T));
    static constexpr int kLdsBytes = kHaloBytes + TY * kRowRegion;
};

template <typename T, int K, int TY, int D = kHeadDim>
struct InvCfg {
    // Query rectangle of a tile: at most tile + (K-1) + (K-1)/2 on an axis unless the tile
    // touches both borders of a short axis; the rare remainder is read from global memory.
    static constexpr int RECT_H = TY + K - 1 + K / 2, RECT_W = kTileX + K - 1 + K / 2;
    static constexpr int KK = K * K;
    static constexpr int kThreads = kTileX * TY;
    static constexpr int kLdsBytes = RECT_H * RECT_W * VecTraits<T, D>::kKeyStride;
};

template <typename T, int K, int TY, int D = kHeadDim>
struct FusedCfg {
    static constexpr int HALO_H = TY + K - 1, HALO_W = kTileX + K - 1;
    static constexpr int NB = 2 * K - 1;
    static constexpr int kThreads = kTileX * TY;
    static constexpr int kHaloBytes = HALO_H * HALO_W * VecTraits<T, D>::kKeyStride;
    static constexpr int kBiasBytes = ((NB * NB * 4) + 15) & ~15;
    static constexpr int kLdsBytes = 2 * kHaloBytes + kBiasBytes;
};

// Tile height: the one that keeps the most waves resident on a compute unit (workgroups that fit the LDS x waves
// per workgroup, at most 32 waves), the taller tile on a tie (its halo is shared by more queries; measured faster).
template <template <typename, int, int, int> class Cfg, typename T, int K, int D>
constexpr int tile_rows() {
    int best = 4, best_waves = 0;
    const int lds[3] = {Cfg<T, K, 4, D>::kLdsBytes, Cfg<T, K, 8, D>::kLdsBytes, Cfg<T, K, 16, D>::kLdsBytes};
    for (int i = 0; i < 3; ++i) {
        const int ty = 4 << i, waves_per_wg = ty * kTileX / kWave;
        int wgs = lds[i] > 0 ? kLdsLimit / lds[i] : 0;
        int waves = wgs * waves_per_wg;
        waves = waves > 32 ? 32 : waves;
        if (waves >= best_waves && waves > 0) {
            best = ty;
            best_waves = waves;
        }
    }
    return best;
}
template <template <typename, int, int, int> class Cfg, typename T, int K, int D>
constexpr bool tile_fits() {
    return Cfg<T, K, tile_rows<Cfg, T, K, D>(), D>::kLdsBytes <= kLdsLimit;
}
// every plain-ALU kernel of the forward and the backward has a tile that fits
template <typename T, int K, int D>
constexpr bool valu_fits() {
    return tile_fits<QkCfg, T, K, D>() && tile_fits<AvCfg, T, K, D>() && tile_fits<InvCfg, T, K, D>() &&
           tile_fits<FusedCfg, T, K, D>();
}

// run-time form (false for window sides beyond the tuned ones)
bool head_dim_supported(int dtype, int K, int D);

}  // namespace na2d
