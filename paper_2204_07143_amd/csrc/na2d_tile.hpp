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

// Stage the keys (oy + ry, ox + rx), ry < ROWS, rx < COLS, of one plane into LDS with the padded
// per-key stride.  The origin may be negative or the halo may reach beyond the map ("virtual"
// coordinates): positions outside the map are zero-filled when ZERO is set and skipped
// otherwise (no window ever reads them).  Loads are issued in batches of up to 4 per thread
// before the matching LDS stores, so a thread keeps its share of the halo in flight at once.
template <typename T, int ROWS, int COLS, int NTHREADS, bool ZERO = false, int D = kHeadDim>
__device__ __forceinline__ void load_halo(const char *plane_base, int H, int W, int oy, int ox, char *lds, int tid) {
    constexpr int KBYTES = VecTraits<T, D>::kKeyBytes;
    constexpr int CPK = KBYTES / 16;
    constexpr int STRIDE = VecTraits<T, D>::kKeyStride;
    constexpr int TOTAL = ROWS * COLS * CPK;
    constexpr int NITER = (TOTAL + NTHREADS - 1) / NTHREADS;
    constexpr int BATCH = 4;
    // The index arithmetic below depends only on the thread id; stop the compiler from hoisting it
    // out of a caller's tile loop, where it would pin dozens of registers for the whole kernel.
    asm volatile("" : "+v"(tid));
#pragma unroll
    for (int b0 = 0; b0 < NITER; b0 += BATCH) {
        u32x4 v[BATCH];
        int dst[BATCH];   // LDS byte offset, or -1 when nothing is to be stored
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            dst[u] = -1;
            v[u] = u32x4{0u, 0u, 0u, 0u};
            if (b0 + u < NITER) {
                const int i = tid + (b0 + u) * NTHREADS;
                const int c = i % CPK;
                const int rx = (i / CPK) % COLS;
                const int ry = i / (CPK * COLS);
                const int y = oy + ry, x = ox + rx;
                const bool in_tile = i < TOTAL;
                const bool in_map = y >= 0 && y < H && x >= 0 && x < W;
                if (in_tile && in_map)
                    v[u] = *reinterpret_cast<const u32x4 *>(plane_base + ((size_t)y * W + x) * KBYTES + c * 16);
                if (in_tile && (in_map || ZERO)) dst[u] = (ry * COLS + rx) * STRIDE + c * 16;
            }
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
            if (dst[u] >= 0) *reinterpret_cast<u32x4 *>(lds + dst[u]) = v[u];
    }
}

template <typename T, int D>
__device__ __forceinline__ void lds_load_vec32(VecN<T, D> &v, const char *lds_key) {
    load_vec32(v, lds_key);
}

// compile-time integer passed as a lambda argument
template <int V> struct IntC {
    static constexpr int value = V;
};

// Which 4 x 4 patch of its strip (the upper or the lower four rows of the 16 x 8 tile: wave / 4) a wave takes.
// Waves w and w + 4 share a SIMD; the rotation by two puts their patches on different halves of the tile, so a
// tile that is only half inside the map (at the right border, or a map narrower than nine positions) keeps one
// active wave on every SIMD instead of two on half of them.
__device__ inline int patch_of_wave(int wave) { return (wave + 2 * (wave >> 2)) & 3; }

// Work split of the position-stationary kernels: a unit is a (tile position, head) pair; the batch is
// cut into `splits` ranges so that about two workgroups per compute unit exist.
struct UnitSplit {
    int units, splits;
};
static inline UnitSplit unit_split(int tiles_x, int tiles_y, int heads, int nb) {
    UnitSplit u;
    u.units = tiles_x * tiles_y * heads;
    int s = (256 * 2) / u.units;
    s = s < 1 ? 1 : s;
    u.splits = s < nb ? s : nb;
    return u;
}
// First batch item of range `split` of `splits`.  Ranges differ by at most one item and the longer ones come
// first: the workgroups that are dispatched first carry the extra tile, not the ones that start last.
__host__ __device__ inline int range_begin(int split, int splits, int nb) { return (split * nb + splits - 1) / splits; }
// Which range the workgroups of (split, head) take: rotated per head, so that the longer ranges of different heads
// sit in different parts of the grid (different XCDs) instead of side by side.  All tile positions of one
// (split, head) keep the same range: they share halo rows and run together.
__device__ inline int batch_range_of(int split, int head, int heads, int splits) {
    return (split + (head * splits) / heads) % splits;
}

}  // namespace na2d
