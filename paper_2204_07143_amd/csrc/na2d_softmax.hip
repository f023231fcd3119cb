// Softmax over the K*K axis and its backward (arXiv 2204.07143, Eq. 4; the paper applies
// the softmax between its two kernels, Appendix A).
//
// Pure streaming work: a workgroup moves a contiguous block of rows through LDS with 16-byte
// accesses (rows of K*K elements are not 16-byte multiples), a group of G lanes owns one row
// with E = ceil(K*K / G) elements per lane in registers, and the row max / sum are reduced
// with wavefront shuffles across the G lanes.
#include "na2d_kernels.hpp"
#include "na2d_common.hpp"

namespace na2d {

template <int K> struct RowSplit {
    static constexpr int KK = K * K;
    static constexpr int G = KK <= 12 ? 4 : (KK <= 88 ? 8 : 16);   // lanes per row
    static constexpr int E = (KK + G - 1) / G;                    // elements per lane
};

template <typename T, int K> struct SoftmaxCfg {
    static constexpr int KK = K * K;
    static constexpr int kThreads = 256;
    // Rows per workgroup: small blocks (one pass of the 256 threads over the rows, two for the shortest rows) give
    // many workgroups, which balances the chip and keeps loads, arithmetic and stores of different blocks
    // overlapped; 128-row blocks were 15-25 % slower.
    static constexpr int kRows = (KK * (int)sizeof(T) <= 60) ? 64 : kThreads / RowSplit<K>::G;
    static constexpr int kRegion = mirror_bytes(kRows * KK * (int)sizeof(T));
};

// Butterfly over the G lanes of a row group (G = 4, 8 or 16, groups aligned to G lanes), every lane ending with
// the group's result.  The exchanges are data-parallel-primitive moves inside the vector ALU (lane ^ 1 and
// lane ^ 2 as quad permutations, then the mirror of the half row and of the row, which bring the other half's
// partial result once both halves are uniform): no trip through the LDS pipe, which the row data already loads.
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
    const int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true);
    return __builtin_bit_cast(float, r);
}
constexpr int kDppXor1 = 0xB1;          // quad_perm [1, 0, 3, 2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2, 3, 0, 1]
constexpr int kDppHalfMirror = 0x141;   // lane i <-> 7 - i inside each group of 8
constexpr int kDppMirror = 0x140;       // lane i <-> 15 - i inside each row of 16
template <int G> __device__ __forceinline__ float group_max(float v) {
    static_assert(G == 4 || G == 8 || G == 16, "row groups");
    v = fmaxf(v, dpp_move<kDppXor1>(v));
    v = fmaxf(v, dpp_move<kDppXor2>(v));
    if constexpr (G >= 8) v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
    if constexpr (G >= 16) v = fmaxf(v, dpp_move<kDppMirror>(v));
    return v;
}
template <int G> __device__ __forceinline__ float group_sum(float v) {
    static_assert(G == 4 || G == 8 || G == 16, "row groups");
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    if constexpr (G >= 8) v += dpp_move<kDppHalfMirror>(v);
    if constexpr (G >= 16) v += dpp_move<kDppMirror>(v);
    return v;
}

template <typename T, int K>
__global__ __launch_bounds__(256) void softmax_kernel(const T *in, T *out, size_t nrows) {
    using C = SoftmaxCfg<T, K>;
    using S = RowSplit<K>;
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x;
    const size_t row0 = (size_t)blockIdx.x * C::kRows;
    const int rows = (int)((nrows - row0) < (size_t)C::kRows ? (nrows - row0) : (size_t)C::kRows);
    const size_t g0 = row0 * C::KK * sizeof(T);
    const int nbytes = rows * C::KK * (int)sizeof(T);
    stage_in<T, C::kRows * C::KK * (int)sizeof(T), C::kThreads>(reinterpret_cast<const char *>(in), g0, nbytes, lds, tid);
    workgroup_sync();
    T *tile = reinterpret_cast<T *>(lds + (int)(g0 & 15));
    const int sub = tid % S::G;
    for (int r = tid / S::G; r < rows; r += C::kThreads / S::G) {
        T *row = tile + r * C::KK;
        float v[S::E];
        float m = -INFINITY;
#pragma unroll
        for (int e = 0; e < S::E; ++e) {
            const int idx = sub * S::E + e;
            v[e] = idx < C::KK ? to_f32(row[idx]) : -INFINITY;
            m = fmaxf(m, v[e]);
        }
        m = group_max<S::G>(m);
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < S::E; ++e) {
            v[e] = __expf(v[e] - m);
            sum += v[e];
        }
        sum = group_sum<S::G>(sum);
        const float inv = 1.0f / sum;
#pragma unroll
        for (int e = 0; e < S::E; ++e) {
            const int idx = sub * S::E + e;
            if (idx < C::KK) row[idx] = from_f32<T>(v[e] * inv);
        }
    }
    workgroup_sync();
    stage_out<T, C::kRows * C::KK * (int)sizeof(T), C::kThreads>(reinterpret_cast<char *>(out), g0, nbytes, lds, tid);
}

template <typename T, int K>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const T *attn, const T *dp,
                                                          T *ds, size_t nrows) {
    using C = SoftmaxCfg<T, K>;
    using S = RowSplit<K>;
    extern __shared__ __align__(16) char lds[];
    char *reg_p = lds, *reg_g = lds + C::kRegion;
    const int tid = threadIdx.x;
    const size_t row0 = (size_t)blockIdx.x * C::kRows;
    const int rows = (int)((nrows - row0) < (size_t)C::kRows ? (nrows - row0) : (size_t)C::kRows);
    const size_t g0 = row0 * C::KK * sizeof(T);
    const int nbytes = rows * C::KK * (int)sizeof(T);
    {
        StageIn<T, C::kRows * C::KK * (int)sizeof(T), C::kThreads> sp, sg;
        sp.issue(reinterpret_cast<const char *>(attn), g0, nbytes, tid);
        sg.issue(reinterpret_cast<const char *>(dp), g0, nbytes, tid);
        sp.commit(reg_p, tid);
        sg.commit(reg_g, tid);
    }
    workgroup_sync();
    const T *tp = reinterpret_cast<const T *>(reg_p + (int)(g0 & 15));
    T *tg = reinterpret_cast<T *>(reg_g + (int)(g0 & 15));
    const int sub = tid % S::G;
    for (int r = tid / S::G; r < rows; r += C::kThreads / S::G) {
        const T *prow = tp + r * C::KK;
        T *grow = tg + r * C::KK;
        float pv[S::E], gv[S::E];
        float inner = 0.f;
#pragma unroll
        for (int e = 0; e < S::E; ++e) {
            const int idx = sub * S::E + e;
            pv[e] = idx < C::KK ? to_f32(prow[idx]) : 0.f;
            gv[e] = idx < C::KK ? to_f32(grow[idx]) : 0.f;
            inner = __builtin_fmaf(pv[e], gv[e], inner);
        }
        inner = group_sum<S::G>(inner);
#pragma unroll
        for (int e = 0; e < S::E; ++e) {
            const int idx = sub * S::E + e;
            if (idx < C::KK) grow[idx] = from_f32<T>(pv[e] * (gv[e] - inner));
        }
    }
    workgroup_sync();
    stage_out<T, C::kRows * C::KK * (int)sizeof(T), C::kThreads>(reinterpret_cast<char *>(ds), g0, nbytes, reg_g, tid);
}

template <typename T, int K>
static hipError_t launch_softmax_t(const Problem &p, const void *in, void *out, hipStream_t s) {
    using C = SoftmaxCfg<T, K>;
    const size_t nrows = p.queries();
    const unsigned grid = (unsigned)((nrows + C::kRows - 1) / C::kRows);
    auto kern = softmax_kernel<T, K>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kRegion, allowed); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::kThreads), C::kRegion, s, static_cast<const T *>(in),
                       static_cast<T *>(out), nrows);
    return hipGetLastError();
}

template <typename T, int K>
static hipError_t launch_softmax_bwd_t(const Problem &p, const void *attn, const void *dp, void *ds, hipStream_t s) {
    using C = SoftmaxCfg<T, K>;
    const size_t nrows = p.queries();
    const unsigned grid = (unsigned)((nrows + C::kRows - 1) / C::kRows);
    auto kern = softmax_bwd_kernel<T, K>;
    static_assert(2 * C::kRegion <= 160 * 1024, "rows do not fit the 160 KB LDS of a CDNA4 compute unit");
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, 2 * C::kRegion, allowed); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::kThreads), 2 * C::kRegion, s, static_cast<const T *>(attn),
                       static_cast<const T *>(dp), static_cast<T *>(ds), nrows);
    return hipGetLastError();
}

hipError_t launch_softmax(const Problem &p, const void *logits, void *out, hipStream_t s) {
    if (untuned_window(p)) return launch_softmax_generic(p, logits, out, s);
    NA2D_DISPATCH_T(p.dtype, NA2D_DISPATCH_K(p.K, return (launch_softmax_t<T, K>(p, logits, out, s))));
    return hipErrorInvalidValue;
}

hipError_t launch_softmax_bwd(const Problem &p, const void *attn, const void *dp, void *ds, hipStream_t s) {
    if (untuned_window(p)) return launch_softmax_bwd_generic(p, attn, dp, ds, s);
    NA2D_DISPATCH_T(p.dtype, NA2D_DISPATCH_K(p.K, return (launch_softmax_bwd_t<T, K>(p, attn, dp, ds, s))));
    return hipErrorInvalidValue;
}

}  // namespace na2d
