// Query-tile / key-halo machinery shared by the tiled kernels.
//
// A workgroup owns a TY x 16 tile of one (batch, head) plane.  Because neighbouring queries
// see almost the same keys, the union of the tile's windows -- a (TY+K-1) x (16+K-1) halo --
// is staged once in LDS (the tiling idea of arXiv 2204.07143, Appendix A "Tiled
// Neighborhood Attention": key tile side = query tile side + k - 1), and every thread then
// works out of LDS.  Tile sizes here are chosen for CDNA4's 160 KB LDS and 64-wide waves.
#pragma once

#include "na2d_common.hpp"

namespace na2d {

constexpr int kTileX = 16;
constexpr int kNumXcd = 8;

// Workgroups are handed to the 8 XCDs round-robin by launch index.  Remap so that each XCD
// (and its private L2) receives a contiguous range of tiles: neighbouring tiles share halo
// rows, so their re-reads then hit the same L2.
__device__ __forceinline__ int xcd_contiguous_block(int bid, int nblocks) {
    const int per = (nblocks + kNumXcd - 1) / kNumXcd;
    return (bid % kNumXcd) * per + bid / kNumXcd;
}
__host__ inline int xcd_padded_grid(int nblocks) { return ((nblocks + kNumXcd - 1) / kNumXcd) * kNumXcd; }

struct TileCoord {
    int plane, tiy, tix;   // plane index and tile indices along y and x
};

__device__ __forceinline__ TileCoord decode_tile(int t, int tiles_x, int tiles_y) {
    TileCoord c;
    c.tix = t % tiles_x;
    const int rest = t / tiles_x;
    c.tiy = rest % tiles_y;
    c.plane = rest / tiles_y;
    return c;
}

// Stage the keys (hy0 + ry, hx0 + rx), ry < ROWS, rx < COLS, of one plane into LDS with the
// padded per-key stride.  Positions outside the map are skipped (no window ever reads them).
template <typename T, int ROWS, int COLS>
__device__ __forceinline__ void load_halo(const char *plane_base, int H, int W, int hy0, int hx0, char *lds,
                                          int tid, int nthreads) {
    constexpr int CPK = Traits<T>::kKeyBytes / 16;
    constexpr int STRIDE = Traits<T>::kKeyStride;
    constexpr int TOTAL = ROWS * COLS * CPK;
    for (int i = tid; i < TOTAL; i += nthreads) {
        const int c = i % CPK;
        const int rx = (i / CPK) % COLS;
        const int ry = i / (CPK * COLS);
        const int y = hy0 + ry, x = hx0 + rx;
        if (y < H && x < W) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(plane_base + ((size_t)y * W + x) * Traits<T>::kKeyBytes + c * 16);
            *reinterpret_cast<u32x4 *>(lds + (ry * COLS + rx) * STRIDE + c * 16) = v;
        }
    }
}

template <typename T>
__device__ __forceinline__ void lds_load_vec32(Vec32<T> &v, const char *lds_key) {
    load_vec32(v, lds_key);
}

}  // namespace na2d
