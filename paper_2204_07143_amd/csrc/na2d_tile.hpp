// Query-tile / key-halo machinery shared by the tiled kernels.
//
// A workgroup owns a TY x 16 tile of one (batch, head) plane.  Because neighbouring queries
// see almost the same keys, the union of the tile's windows -- a (TY+K-1) x (16+K-1) halo --
// is staged once in LDS (the tiling idea of arXiv 2204.07143, Appendix A "Tiled
// Neighborhood Attention": key tile side = query tile side + k - 1), and every thread then
// works out of LDS.  Tile sizes here are chosen for CDNA4's 160 KB LDS and 64-wide waves.
#pragma once
#include <stdint.h>

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

// Division of a non-negative int by a divisor known at launch: the host works out a multiplier and a shift
// (m = ceil(2^(31+L) / d), L = ceil(log2 d)), the device needs a shift, a multiply-high and a shift, all on the
// scalar unit for uniform values.  Exact for every 0 <= n < 2^31 (Granlund & Montgomery, "Division by invariant
// integers using multiplication": n < 2^31 needs 31 + L fraction bits, and 2n keeps the product inside 64 bits).
// A workgroup decodes its place in the grid before it can issue its first load; the runtime divisions of that
// decode were two thirds of its scalar instructions.
struct FastDiv {
    uint32_t m, L;
};
static inline FastDiv make_fastdiv(int d) {
    FastDiv f;
    f.L = 0;
    while ((1ll << f.L) < (long long)d) ++f.L;
    f.m = (uint32_t)((((unsigned long long)1 << (31 + f.L)) + (unsigned long long)d - 1) / (unsigned long long)d);
    return f;
}
__device__ __forceinline__ int fdiv(int n, FastDiv f) { return (int)(__umulhi((uint32_t)n << 1, f.m) >> f.L); }

// What a workgroup of a position-stationary kernel needs to find its tile position, head and batch range.
struct GridDecode {
    FastDiv by_npos, by_heads, by_tiles_y, by_splits;
    int npos, range_base, range_rem;   // nb = splits * base + rem; batch range r starts at r * base + ceil(r * rem / splits)
};

// Work split of the position-stationary kernels: a unit is a (tile position, head) pair; the batch is
// cut into `splits` ranges so that about two workgroups per compute unit exist.
static inline GridDecode make_grid_decode(int tiles_x, int tiles_y, int heads, int nb, int splits) {
    GridDecode gd;
    gd.npos = tiles_x * tiles_y;
    gd.by_npos = make_fastdiv(gd.npos);
    gd.by_heads = make_fastdiv(heads);
    gd.by_tiles_y = make_fastdiv(tiles_y);
    gd.by_splits = make_fastdiv(splits);
    gd.range_base = nb / splits;
    gd.range_rem = nb % splits;
    return gd;
}
struct UnitSplit {
    int units, splits;
    GridDecode gd;
};
static inline UnitSplit unit_split(int tiles_x, int tiles_y, int heads, int nb) {
    UnitSplit u;
    u.units = tiles_x * tiles_y * heads;
    int s = (256 * 2) / u.units;
    s = s < 1 ? 1 : s;
    u.splits = s < nb ? s : nb;
    u.gd = make_grid_decode(tiles_x, tiles_y, heads, nb, u.splits);
    return u;
}
struct WorkItem {
    int pos, head, ty, tx, b_begin, b_end;   // tile row / column index; batch items [b_begin, b_end)
    int split;                               // which of the `splits` workgroups of this (position, head) pair
};
__device__ __forceinline__ WorkItem decode_work(int wg, int heads, int tiles_y, int splits, const GridDecode &gd) {
    WorkItem w;
    const int wq = fdiv(wg, gd.by_npos), split = fdiv(wq, gd.by_heads);
    w.pos = wg - wq * gd.npos;
    w.head = wq - split * heads;
    w.split = split;
    w.tx = fdiv(w.pos, gd.by_tiles_y);
    w.ty = w.pos - w.tx * tiles_y;
    // Ranges differ by at most one item; where only one is longer it comes first, so that a workgroup dispatched
    // early carries the extra tile.  Which range (split, head) takes is rotated per head, so that the longer ranges of different heads
    // sit in different parts of the grid (different XCDs) instead of side by side; all tile positions of one
    // (split, head) keep the same range: they share halo rows and run together.
    int r = split + fdiv(w.head * splits, gd.by_heads);   // < 2 splits
    r = r >= splits ? r - splits : r;
    // range r = [ceil(r nb / splits), ceil((r + 1) nb / splits)): the ranges that hold one item more are spread evenly
    w.b_begin = r * gd.range_base + fdiv(r * gd.range_rem + splits - 1, gd.by_splits);
    w.b_end = (r + 1) * gd.range_base + fdiv((r + 1) * gd.range_rem + splits - 1, gd.by_splits);
    return w;
}

}  // namespace na2d
