// Gradient of the relative positional bias (arXiv 2204.07143, Eq. 2's B(i, j); grad-b in
// the Appendix A kernel list):
//   d_rpb[h, u, v] = sum over batch, queries n and slots (a, c) with
//                    rpb_start(qy) + a = u and rpb_start(qx) + c = v of ds[n, a, c].
//
// Two-level reduction in a fixed order, no atomics:
//   1. a workgroup owns up to kRpbSub chunks of consecutive queries of one plane; their ds rows
//      are streamed through LDS with 16-byte loads; each wave walks its queries one at a time with
//      lanes = window slots, so a query's K*K values land in K*K distinct table cells.
//      Interior queries all map to the central K x K block and are accumulated in a register;
//      border queries update the wave's private (2K-1)^2 LDS table.  The four wave tables are
//      added in wave order and written to the workspace;
//   2. a second kernel adds the workgroup partials of each head in index order.
#include "na2d_kernels.hpp"
#include "na2d_common.hpp"

namespace na2d {

constexpr int kRpbSub = 4;       // chunks per workgroup
constexpr int kRpbWaves = 4;

// Queries staged at once: a multiple of the wave width, at most 256, sized so that one chunk
// of ds rows stays under 48 KB of LDS.
__host__ __device__ constexpr int rpb_chunk(int kk, int elem_bytes) {
    int q = (48 * 1024) / (kk * elem_bytes);
    q = (q / kWave) * kWave;
    return q < kWave ? kWave : (q > 256 ? 256 : q);
}

template <typename T, int K> struct RpbCfg {
    static constexpr int KK = K * K, NB = 2 * K - 1, CELLS = NB * NB;
    static constexpr int kChunk = rpb_chunk(KK, (int)sizeof(T));
    static constexpr int kQPerWave = kChunk / kRpbWaves;
    static constexpr int kRegion = mirror_bytes(kChunk * KK * (int)sizeof(T));
    static constexpr int kLdsBytes = kRegion + kRpbWaves * CELLS * 4;
    static constexpr int kSlotsPerLane = (KK + kWave - 1) / kWave;
};

static inline int rpb_groups_per_plane(int H, int W, int K, int elem_bytes) {
    const int per_group = rpb_chunk(K * K, elem_bytes) * kRpbSub;
    return (H * W + per_group - 1) / per_group;
}

template <typename T, int K>
__global__ __launch_bounds__(256) void rpb_partial_kernel(const T *__restrict__ ds, float *__restrict__ partial, int H,
                                                          int W, int groups_per_plane) {
    using C = RpbCfg<T, K>;
    extern __shared__ __align__(16) char lds[];
    float *tables = reinterpret_cast<float *>(lds + C::kRegion);
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int plane = blockIdx.x / groups_per_plane, group = blockIdx.x % groups_per_plane;
    const int HW = H * W;
    constexpr int R = K / 2;

    float *mine = tables + wave * C::CELLS;
    for (int i = lane; i < C::CELLS; i += kWave) mine[i] = 0.f;

    int cell_off[C::kSlotsPerLane];   // offset of this lane's slot inside the table, relative to (py, px)
    float acc[C::kSlotsPerLane];
#pragma unroll
    for (int s = 0; s < C::kSlotsPerLane; ++s) {
        const int slot = lane + s * kWave;
        cell_off[s] = (slot / K) * C::NB + (slot % K);
        acc[s] = 0.f;
    }

    for (int sub = 0; sub < kRpbSub; ++sub) {
        const int q0 = (group * kRpbSub + sub) * C::kChunk;
        if (q0 >= HW) break;
        const int nq = (HW - q0) < C::kChunk ? (HW - q0) : C::kChunk;
        const size_t g0 = ((size_t)plane * HW + q0) * C::KK * sizeof(T);
        __syncthreads();   // previous chunk fully consumed
        stage_in<T>(reinterpret_cast<const char *>(ds), g0, nq * C::KK * (int)sizeof(T), lds, tid, 256);
        __syncthreads();
        const T *tile = reinterpret_cast<const T *>(lds + (int)(g0 & 15));
        const int qend = (wave + 1) * C::kQPerWave < nq ? (wave + 1) * C::kQPerWave : nq;
        for (int qi = wave * C::kQPerWave; qi < qend; ++qi) {
            const int qlin = q0 + qi;
            const int qy = qlin / W, qx = qlin - qy * W;
            const int py = rpb_start(qy, H, K), px = rpb_start(qx, W, K);
            const bool interior = (py == R) && (px == R);
            const int base = py * C::NB + px;
#pragma unroll
            for (int s = 0; s < C::kSlotsPerLane; ++s) {
                const int slot = lane + s * kWave;
                if (slot < C::KK) {
                    const float val = to_f32(tile[qi * C::KK + slot]);
                    if (interior)
                        acc[s] += val;
                    else
                        mine[base + cell_off[s]] += val;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
#pragma unroll
    for (int s = 0; s < C::kSlotsPerLane; ++s) {
        const int slot = lane + s * kWave;
        if (slot < C::KK) mine[R * C::NB + R + cell_off[s]] += acc[s];
    }
    __syncthreads();
    for (int i = tid; i < C::CELLS; i += 256) {
        float s = tables[i];
#pragma unroll
        for (int w = 1; w < kRpbWaves; ++w) s += tables[w * C::CELLS + i];
        partial[(size_t)blockIdx.x * C::CELLS + i] = s;
    }
}

// d_rpb[h, cell] = sum over (batch, group) in index order of partial[(b * heads + h) * groups + group][cell]
__global__ __launch_bounds__(256) void rpb_final_kernel(const float *__restrict__ partial, float *__restrict__ d_rpb,
                                                        int B, int heads, int groups, int cells) {
    const int cell = blockIdx.x * 256 + threadIdx.x;
    const int h = blockIdx.y;
    if (cell >= cells) return;
    float lanes[4] = {0.f, 0.f, 0.f, 0.f};
    int it = 0;
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < groups; ++g, ++it)
            lanes[it & 3] += partial[((size_t)(b * heads + h) * groups + g) * cells + cell];
    d_rpb[(size_t)h * cells + cell] = (lanes[0] + lanes[1]) + (lanes[2] + lanes[3]);
}

size_t rpb_bwd_workspace_bytes(const Problem &p) {
    const int nb = 2 * p.K - 1;
    return (size_t)p.planes() * rpb_groups_per_plane(p.H, p.W, p.K, p.elem_bytes()) * nb * nb * sizeof(float);
}

template <typename T, int K>
static hipError_t launch_rpb_bwd_t(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s) {
    using C = RpbCfg<T, K>;
    const int groups = rpb_groups_per_plane(p.H, p.W, K, (int)sizeof(T));
    auto kern = rpb_partial_kernel<T, K>;
    static_assert(C::kLdsBytes <= 160 * 1024, "tile does not fit the 160 KB LDS of a CDNA4 compute unit");
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(p.planes() * groups), dim3(256), C::kLdsBytes, s, static_cast<const T *>(ds),
                       static_cast<float *>(workspace), p.H, p.W, groups);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rpb_final_kernel, dim3((C::CELLS + 255) / 256, p.heads), dim3(256), 0, s,
                       static_cast<const float *>(workspace), d_rpb, p.B, p.heads, groups, C::CELLS);
    return hipGetLastError();
}

hipError_t launch_rpb_bwd(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s) {
    NA2D_DISPATCH_T(p.dtype, NA2D_DISPATCH_K(p.K, return (launch_rpb_bwd_t<T, K>(p, ds, d_rpb, workspace, s))));
    return hipErrorInvalidValue;
}

}  // namespace na2d
