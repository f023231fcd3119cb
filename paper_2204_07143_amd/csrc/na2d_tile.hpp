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

// The same staging split in two, for software pipelining across tiles: issue() starts the
// global loads of a thread's share of the halo into registers (positions outside the map become
// zeros), commit() writes them to LDS later.  A persistent workgroup issues the next tile's halo
// before it computes the current tile, so the memory latency is hidden behind the compute.
// Which halo positions a thread moves never changes, so their offsets are worked out once
// (init) and each tile only adds its origin and checks the map bounds.
// COLS columns are staged per halo row; PITCH >= COLS is the row pitch of the LDS image (the
// columns in between are never written by the stager).
template <typename T, int ROWS, int COLS, int NTHREADS, int PITCH = COLS>
struct HaloPrefetch {
    static constexpr int CPK = Traits<T>::kKeyBytes / 16;
    static constexpr int STRIDE = Traits<T>::kKeyStride;
    static constexpr int TOTAL = ROWS * COLS * CPK;
    static constexpr int NITER = (TOTAL + NTHREADS - 1) / NTHREADS;
    u32x4 v[NITER];
    int goff[NITER];   // byte offset from the halo's origin key in global memory
    int loff[NITER];   // byte offset in the LDS halo, -1 for the padding past the last chunk
    int pos[NITER];    // halo row | halo col << 16

    __device__ __forceinline__ void init(int W, int tid) {
#pragma unroll
        for (int it = 0; it < NITER; ++it) {
            const int i = tid + it * NTHREADS;
            const int c = i % CPK;
            const int rx = (i / CPK) % COLS;
            const int ry = i / (CPK * COLS);
            goff[it] = (ry * W + rx) * Traits<T>::kKeyBytes + c * 16;
            loff[it] = i < TOTAL ? (ry * PITCH + rx) * STRIDE + c * 16 : -1;
            pos[it] = ry | (rx << 16);
        }
    }
    // plane_base + origin_off addresses key (oy, ox); origin_off may be negative near a border.
    __device__ __forceinline__ void issue(const char *plane_base, int H, int W, int oy, int ox) {
        const int origin_off = (oy * W + ox) * Traits<T>::kKeyBytes;
#pragma unroll
        for (int it = 0; it < NITER; ++it) {
            const int y = oy + (pos[it] & 0xffff), x = ox + (pos[it] >> 16);
            v[it] = u32x4{0u, 0u, 0u, 0u};
            if (loff[it] >= 0 && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)W)
                v[it] = *reinterpret_cast<const u32x4 *>(plane_base + (origin_off + goff[it]));
        }
    }
    __device__ __forceinline__ void commit(char *lds) const {
#pragma unroll
        for (int it = 0; it < NITER; ++it)
            if (loff[it] >= 0) *reinterpret_cast<u32x4 *>(lds + loff[it]) = v[it];
    }
};

template <typename T, int D>
__device__ __forceinline__ void lds_load_vec32(VecN<T, D> &v, const char *lds_key) {
    load_vec32(v, lds_key);
}

// compile-time integer passed as a lambda argument
template <int V> struct IntC {
    static constexpr int value = V;
};

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

}  // namespace na2d
