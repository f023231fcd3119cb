// Gradient of the relative positional bias (arXiv 2204.07143, Eq. 2's B(i, j); grad-b in
// the Appendix A kernel list):
//   d_rpb[h, u, v] = sum over batch, queries n and slots (a, c) with
//                    rpb_start(qy) + a = u and rpb_start(qx) + c = v of ds[n, a, c].
//
// Pure streaming of ds (HBM-bound), reduced in two levels in a fixed order, no atomics:
//   1. Each wave owns whole "segments" (up to 64 consecutive queries of one image row, fewer for long rows), which it
//      stages in its private LDS region with 16-byte loads.  Lanes are window slots, so one
//      query's K*K values land in K*K distinct table cells.  All queries of a segment share the
//      bias row offset; the interior run of a segment also shares the column offset and is
//      summed in registers with independent loads; the few border queries update the wave's
//      private (2K-1)^2 LDS table one query at a time.  The workgroup's wave tables are added
//      in wave order and written to the workspace as one partial per workgroup, the partials
//      of a head next to each other (rpb_cell_stride);
//   2. a second kernel adds the partials of each head, four cells per lane: 16 waves each sum
//      a strided subset in index order, then the 16 sub-sums are added in wave order.
#include "na2d_kernels.hpp"
#include "na2d_common.hpp"
#include "na2d_tile.hpp"

namespace na2d {

constexpr int kRpbWaves = 4;
// Queries per segment, at most: one wave's worth, fewer when K*K rows are long, so that a wave's staging region stays
// under 10 KB and four or more workgroups share a compute unit.  An image row is cut into the fewest segments
// that respect this, of equal length (rpb_split).
__host__ __device__ constexpr int rpb_seg_q(int kk, int elem_bytes) {
    const int q = (10 * 1024) / (kk * elem_bytes);
    return q > 64 ? 64 : q;
}
constexpr int kRpbFinalWaves = 16;

template <typename T, int K> struct RpbCfg {
    static constexpr int KK = K * K, NB = 2 * K - 1, CELLS = NB * NB;
    static constexpr int kSegQ = rpb_seg_q(KK, (int)sizeof(T));
    static constexpr int kRegion = mirror_bytes(kSegQ * KK * (int)sizeof(T));   // per wave, at most
    static constexpr int kTableBytes = ((CELLS * 4) + 15) & ~15;
    static constexpr int kLdsBytes = kRpbWaves * (kRegion + kTableBytes);        // at most
    static constexpr int kSlotsPerLane = (KK + kWave - 1) / kWave;
};

// Segments of one plane: rows x ceil(W / queries-per-segment).  Workgroups per plane are chosen so that the
// launch has on the order of a thousand workgroups (partials) whatever the batch size.
struct RpbSplit {
    int segs_per_row, segs_per_plane, groups_per_plane, segs_per_group;
    int seg_q;    // queries per segment (the last one of a row may be shorter)
    int region;   // bytes of a wave's staging region
};
static inline RpbSplit rpb_split(int planes, int H, int W, int K, int elem_bytes) {
    RpbSplit s;
    const int max_q = rpb_seg_q(K * K, elem_bytes);
    s.segs_per_row = (W + max_q - 1) / max_q;
    s.seg_q = (W + s.segs_per_row - 1) / s.segs_per_row;   // <= max_q
    s.region = mirror_bytes(s.seg_q * K * K * elem_bytes);
    s.segs_per_plane = H * s.segs_per_row;
    // about as many workgroups as the chip holds at once (LDS: four wave regions and tables each), 1024 at most
    const int nb = 2 * K - 1;
    const int lds = kRpbWaves * (s.region + ((nb * nb * 4 + 15) & ~15));
    const int per_cu = (160 * 1024) / lds < 4 ? ((160 * 1024) / lds < 1 ? 1 : (160 * 1024) / lds) : 4;
    int groups = (256 * per_cu + planes - 1) / planes;
    const int max_groups = (s.segs_per_plane + kRpbWaves - 1) / kRpbWaves;
    if (groups > max_groups) groups = max_groups;
    if (groups < 1) groups = 1;
    s.segs_per_group = (s.segs_per_plane + groups - 1) / groups;
    s.groups_per_plane = (s.segs_per_plane + s.segs_per_group - 1) / s.segs_per_group;
    return s;
}

template <typename T, int K>
__global__ __launch_bounds__(256) void rpb_partial_kernel(const T *__restrict__ ds, float *__restrict__ partial, int H,
                                                          int W, RpbSplit sp, int B, int heads) {
    using C = RpbCfg<T, K>;
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // (scalar: everything about a segment is wave-uniform)
    char *region = lds + wave * sp.region;
    float *tables = reinterpret_cast<float *>(lds + kRpbWaves * sp.region);
    float *mine = tables + wave * (C::kTableBytes / 4);
    const int plane = blockIdx.x / sp.groups_per_plane, group = blockIdx.x % sp.groups_per_plane;
    constexpr int R = K / 2;

    for (int i = lane; i < C::CELLS; i += kWave) mine[i] = 0.f;

    int cell_off[C::kSlotsPerLane];   // offset of this lane's slot inside the table, relative to (py, px)
    float acc_int[C::kSlotsPerLane];  // queries whose window is centred on both axes
#pragma unroll
    for (int s = 0; s < C::kSlotsPerLane; ++s) {
        const int slot = lane + s * kWave;
        cell_off[s] = (slot / K) * C::NB + (slot % K);
        acc_int[s] = 0.f;
    }

    const int seg_end = (group + 1) * sp.segs_per_group < sp.segs_per_plane ? (group + 1) * sp.segs_per_group
                                                                            : sp.segs_per_plane;
    for (int seg = group * sp.segs_per_group + wave; seg < seg_end; seg += kRpbWaves) {
        const int qy = seg / sp.segs_per_row;
        const int x0 = (seg - qy * sp.segs_per_row) * sp.seg_q;
        const int x1 = x0 + sp.seg_q < W ? x0 + sp.seg_q : W;
        const size_t g0 = (((size_t)plane * H + qy) * W + x0) * C::KK * sizeof(T);
        stage_in<T, C::kSegQ * C::KK * (int)sizeof(T), kWave>(reinterpret_cast<const char *>(ds), g0,
                                                              (x1 - x0) * C::KK * (int)sizeof(T), region, lane);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const T *tile = reinterpret_cast<const T *>(region + (int)(g0 & 15));
        const int py = rpb_start(qy, H, K);
        // interior run of this segment: queries whose column offset is the centred one
        const int xi0 = x0 > R ? x0 : R;
        const int xi1 = x1 < W - R ? x1 : W - R;
        float run[C::kSlotsPerLane];
#pragma unroll
        for (int s = 0; s < C::kSlotsPerLane; ++s) run[s] = 0.f;
        if (xi1 > xi0) {
#pragma unroll
            for (int s = 0; s < C::kSlotsPerLane; ++s) {
                const int slot = lane + s * kWave;
                if (slot < C::KK) {
                    const T *col = tile + (xi0 - x0) * C::KK + slot;
                    const int n = xi1 - xi0;
                    // eight queries per round: eight reads at immediate offsets from one address, eight sums
                    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    int i = 0;
                    for (; i + 8 <= n; i += 8) {
#pragma unroll
                        for (int u = 0; u < 8; ++u) a[u] += to_f32(col[(i + u) * C::KK]);
                    }
                    for (; i < n; ++i) a[0] += to_f32(col[i * C::KK]);
                    run[s] = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
                }
            }
        }
        if (py == R) {
#pragma unroll
            for (int s = 0; s < C::kSlotsPerLane; ++s) acc_int[s] += run[s];
        } else if (xi1 > xi0) {
#pragma unroll
            for (int s = 0; s < C::kSlotsPerLane; ++s) {
                const int slot = lane + s * kWave;
                if (slot < C::KK) mine[py * C::NB + R + cell_off[s]] += run[s];
            }
            __builtin_amdgcn_wave_barrier();
        }
        // border queries of the segment, one at a time (their cells overlap between queries)
        for (int x = x0; x < x1; ++x) {
            if (x >= xi0 && x < xi1) {
                x = xi1 - 1;
                continue;
            }
            const int base = py * C::NB + rpb_start(x, W, K);
#pragma unroll
            for (int s = 0; s < C::kSlotsPerLane; ++s) {
                const int slot = lane + s * kWave;
                if (slot < C::KK) mine[base + cell_off[s]] += to_f32(tile[(x - x0) * C::KK + slot]);
            }
            __builtin_amdgcn_wave_barrier();
        }
        __builtin_amdgcn_wave_barrier();   // region is reused by the next segment
    }
#pragma unroll
    for (int s = 0; s < C::kSlotsPerLane; ++s) {
        const int slot = lane + s * kWave;
        if (slot < C::KK) mine[R * C::NB + R + cell_off[s]] += acc_int[s];
    }
    workgroup_sync();
    // partial (b, group) of head h: row h * (B * groups) + b * groups + group
    const int b = plane / heads, h = plane - b * heads;
    float *row = partial + (size_t)((h * B + b) * sp.groups_per_plane + group) * rpb_cell_stride(C::CELLS);
    for (int i = tid; i < C::CELLS; i += 256) {
        float s = tables[i];
#pragma unroll
        for (int w = 1; w < kRpbWaves; ++w) s += tables[w * (C::kTableBytes / 4) + i];
        row[i] = s;
    }
}

// d_rpb[h, cell] = sum over i < n of partial[h * n + i][cell], rows of `stride` floats (rpb_cell_stride).
// One workgroup of 16 waves per head and block of 64 x 4 cells: a lane owns four neighbouring cells (one 16-byte
// load per partial, a wave reads a kilobyte of a row at once); wave w adds the partials whose index is w mod 16, in
// index order, sixteen loads in flight; the 16 sub-sums are then added in wave order.  No index arithmetic beyond
// one multiply per load: the rows of a head follow each other.
struct __attribute__((packed, aligned(4))) RpbQuad {
    f32x4 v;
};
__global__ __launch_bounds__(kRpbFinalWaves *kWave) void rpb_final_kernel(const float *__restrict__ partial,
                                                                           float *__restrict__ d_rpb, int n, int cells,
                                                                           int stride) {
    __shared__ f32x4 sub[kRpbFinalWaves][kWave];
    const int quad_blocks = (stride / 4 + kWave - 1) / kWave;
    const int h = blockIdx.x / quad_blocks;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int cell0 = ((blockIdx.x % quad_blocks) * kWave + lane) * 4;   // this lane's first cell
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    if (cell0 < stride) {
        const float *base = partial + (size_t)h * n * stride + cell0;
        constexpr int U = 16;   // loads in flight per lane; past the end they are skipped (adding 0 changes nothing)
        for (int i = wave; i < n; i += U * kRpbFinalWaves) {
            f32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int iu = i + u * kRpbFinalWaves;
                v[u] = iu < n ? reinterpret_cast<const RpbQuad *>(base + (size_t)iu * stride)->v : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < U; ++u) acc += v[u];
        }
    }
    sub[wave][lane] = acc;
    workgroup_sync();
    if (wave == 0 && cell0 < cells) {
        f32x4 s = sub[0][lane];
        for (int w = 1; w < kRpbFinalWaves; ++w) s += sub[w][lane];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (cell0 + c < cells) d_rpb[(size_t)h * cells + cell0 + c] = s[c];
    }
}

static hipError_t launch_rpb_final(const float *partial, float *d_rpb, int heads, int n, int cells, hipStream_t s) {
    const int stride = rpb_cell_stride(cells);
    hipLaunchKernelGGL(rpb_final_kernel, dim3(heads * ((stride / 4 + kWave - 1) / kWave)), dim3(kRpbFinalWaves * kWave), 0, s,
                       partial, d_rpb, n, cells, stride);
    return hipGetLastError();
}

// d_rpb from the partials that the grad-q kernel (or the fused backward's query-patch kernel) leaves: workgroup
// (position, head, split) of those kernels writes row head * (splits * npos) + split * npos + position.
hipError_t launch_rpb_final_av(const Problem &p, const float *partial, float *d_rpb, AvRpbSplit sp, hipStream_t s) {
    const int nb = 2 * p.K - 1;
    return launch_rpb_final(partial, d_rpb, p.heads, sp.npos * sp.splits, nb * nb, s);
}

size_t rpb_bwd_workspace_bytes(const Problem &p) {
    if (untuned_window(p)) return rpb_generic_workspace_bytes(p);
    const int nb = 2 * p.K - 1;
    const RpbSplit sp = rpb_split(p.planes(), p.H, p.W, p.K, p.elem_bytes());
    size_t bytes = (size_t)p.planes() * sp.groups_per_plane * rpb_cell_stride(nb * nb) * sizeof(float);
    if (av_rpb_supported(p)) {   // the composed backward keeps one partial per workgroup of the grad-q kernel
        const AvRpbSplit a = av_rpb_split(p);
        const size_t alt = (size_t)a.npos * p.heads * a.splits * rpb_cell_stride(nb * nb) * sizeof(float);
        bytes = bytes > alt ? bytes : alt;
    }
    return bytes;
}

template <typename T, int K>
static hipError_t launch_rpb_bwd_t(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s) {
    using C = RpbCfg<T, K>;
    const RpbSplit sp = rpb_split(p.planes(), p.H, p.W, K, (int)sizeof(T));
    auto kern = rpb_partial_kernel<T, K>;
    static_assert(C::kLdsBytes <= 160 * 1024, "segments do not fit the 160 KB LDS of a CDNA4 compute unit");
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    const int lds_bytes = kRpbWaves * (sp.region + C::kTableBytes);   // <= kLdsBytes: seg_q <= kSegQ
    hipLaunchKernelGGL(kern, dim3(p.planes() * sp.groups_per_plane), dim3(256), lds_bytes, s,
                       static_cast<const T *>(ds), static_cast<float *>(workspace), p.H, p.W, sp, p.B, p.heads);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_rpb_final(static_cast<const float *>(workspace), d_rpb, p.heads, p.B * sp.groups_per_plane, C::CELLS, s);
}

hipError_t launch_rpb_bwd(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s) {
    if (untuned_window(p)) return launch_rpb_generic(p, ds, d_rpb, workspace, s);
    NA2D_DISPATCH_T(p.dtype, NA2D_DISPATCH_K(p.K, return (launch_rpb_bwd_t<T, K>(p, ds, d_rpb, workspace, s))));
    return hipErrorInvalidValue;
}

// ---- the same call for callers that cannot allocate -------------------------------------------------
//
// The partials live in a device array that is part of the library's code object instead of a workspace
// the caller brings.  Every GPU the library runs on holds its own copy at its own address, from the
// first use until the process ends.  In host code the array's name is only a handle: its device address
// comes from hipGetSymbolAddress, asked once per device with that device current, and only that address
// is ever handed to a kernel.  The first kernel writes every partial it owns in full, so nothing needs
// clearing between calls; two calls that overlap on one GPU share the array and race.
static __device__ __align__(256) unsigned char scratch[NA2D_NOALLOC_SCRATCH_BYTES];

size_t rpb_bwd_partial_bytes(const Problem &p) {
    if (untuned_window(p)) return rpb_generic_workspace_bytes(p);
    const int nb = 2 * p.K - 1;
    const RpbSplit sp = rpb_split(p.planes(), p.H, p.W, p.K, p.elem_bytes());
    return (size_t)p.planes() * sp.groups_per_plane * rpb_cell_stride(nb * nb) * sizeof(float);
}

static hipError_t scratch_address(void **out) {
    constexpr int kMaxDev = 64;
    static std::atomic<void *> known[kMaxDev];   // zero-initialised; a device's slot is written once
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < kMaxDev;
    if (tracked) {
        if (void *ptr = known[dev].load(std::memory_order_acquire)) {
            *out = ptr;
            return hipSuccess;
        }
    }
    void *ptr = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    if (tracked) known[dev].store(ptr, std::memory_order_release);   // every thread would store the same address
    *out = ptr;
    return hipSuccess;
}

hipError_t launch_rpb_bwd_noalloc(const Problem &p, const void *ds, float *d_rpb, hipStream_t s) {
    if (rpb_bwd_partial_bytes(p) > sizeof(scratch)) return hipErrorInvalidValue;   // the C ABI layer has refused it already
    void *ptr = nullptr;
    if (hipError_t e = scratch_address(&ptr); e != hipSuccess) return e;
    return launch_rpb_bwd(p, ds, d_rpb, ptr, s);
}

}  // namespace na2d
