// 1D Neighborhood Attention kernels for gfx950 (arXiv 2204.07143, Section 3.1, Eq. 2-4 on a sequence;
// the gradients the paper lists for its package -- q, k, b, a, v -- Appendix A).
//
// Per query the 1D operator moves 2*D*e + k*e bytes for 2*k*D flops (3 flop/B at k = 7, f16): far below
// any arithmetic ridge of the chip, so these kernels are plain-ALU streaming kernels and the matrix
// cores are not used.  What matters is that every byte crosses HBM once and in 16-byte pieces:
//   * a workgroup owns TQ consecutive positions of one (batch, head) plane; the union of their windows
//     (TQ + k - 1 keys; TQ + 2(k-1) queries for the inverse neighbourhood) is staged in LDS once with
//     coalesced 16-byte loads, a padded per-key stride keeping the later 16-byte LDS reads conflict-free;
//   * the k-wide rows of logits / weights of a tile are one contiguous run in memory; it is mirrored in
//     LDS at its 16-byte phase, so it enters and leaves as aligned 16-byte chunks although a row (k
//     elements) is not a multiple of 16 bytes;
//   * one thread per position: the head vector (32 elements) lives in registers, dot products use the
//     packed dot instructions for the 16-bit types, all sums are fp32.
// k is a run-time argument (odd, <= 63); TQ is 256, or 128 for k > 31 so that the LDS images fit.
#include "na1d_kernels.hpp"
#include "lds_attr.hpp"
#include "na2d_common.hpp"
#include "na2d_kernels.hpp"   // the dtype dispatch macro

namespace na1d {

using namespace na2d;

// ---- staging helpers (run-time sizes) ------------------------------------------------------

// n 16-byte chunks: src(c) -> global address, dst(c) -> LDS address; four loads in flight per thread.
template <int NT, typename Src, typename Dst>
__device__ __forceinline__ void copy_chunks_in(int n, int tid, Src src, Dst dst) {
    for (int c0 = tid; c0 < n; c0 += 4 * NT) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (c0 + u * NT < n) v[u] = *reinterpret_cast<const u32x4 *>(src(c0 + u * NT));
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (c0 + u * NT < n) *reinterpret_cast<u32x4 *>(dst(c0 + u * NT)) = v[u];
    }
}

// `count` consecutive head vectors starting at `g` -> LDS with the padded stride.
template <typename T, int NT>
__device__ __forceinline__ void load_vectors(const char *g, int count, char *lds, int tid) {
    constexpr int CPK = Traits<T>::kKeyBytes / 16, STRIDE = Traits<T>::kKeyStride;
    copy_chunks_in<NT>(count * CPK, tid, [&](int c) { return g + (size_t)c * 16; },
                       [&](int c) { return lds + (c / CPK) * STRIDE + (c % CPK) * 16; });
}

// A run of nbytes at global byte offset g0 of gbase <-> its LDS mirror (same 16-byte phase): whole
// 16-byte chunks move as such, the ragged head and tail (under 16 bytes each) element by element.
template <typename T, int NT>
__device__ __forceinline__ void run_in(const char *gbase, size_t g0, int nbytes, char *region, int tid) {
    const RunSplit rs = split_run(g0, nbytes);
    const char *ga = gbase + (g0 - rs.mis);
    copy_chunks_in<NT>((rs.body_hi - rs.body_lo) >> 4, tid, [&](int c) { return ga + rs.body_lo + c * 16; },
                       [&](int c) { return region + rs.body_lo + c * 16; });
    const int head_end = rs.body_lo < rs.span ? rs.body_lo : rs.span;
    const int hb = rs.mis + tid * (int)sizeof(T);
    if (hb < head_end) *reinterpret_cast<T *>(region + hb) = *reinterpret_cast<const T *>(ga + hb);
    const int tb = rs.body_hi + (tid - 16) * (int)sizeof(T);
    if (tid >= 16 && rs.body_hi >= head_end && tb < rs.span)
        *reinterpret_cast<T *>(region + tb) = *reinterpret_cast<const T *>(ga + tb);
}

template <typename T, int NT>
__device__ __forceinline__ void run_out(char *gbase, size_t g0, int nbytes, const char *region, int tid) {
    const RunSplit rs = split_run(g0, nbytes);
    char *ga = gbase + (g0 - rs.mis);
    const int n = (rs.body_hi - rs.body_lo) >> 4;
    for (int c0 = tid; c0 < n; c0 += 4 * NT) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (c0 + u * NT < n) v[u] = *reinterpret_cast<const u32x4 *>(region + rs.body_lo + (c0 + u * NT) * 16);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (c0 + u * NT < n) *reinterpret_cast<u32x4 *>(ga + rs.body_lo + (c0 + u * NT) * 16) = v[u];
    }
    const int head_end = rs.body_lo < rs.span ? rs.body_lo : rs.span;
    const int hb = rs.mis + tid * (int)sizeof(T);
    if (hb < head_end) *reinterpret_cast<T *>(ga + hb) = *reinterpret_cast<const T *>(region + hb);
    const int tb = rs.body_hi + (tid - 16) * (int)sizeof(T);
    if (tid >= 16 && rs.body_hi >= head_end && tb < rs.span)
        *reinterpret_cast<T *>(ga + tb) = *reinterpret_cast<const T *>(region + tb);
}

// The head vectors a tile's threads hold (fp32, one per thread) -> memory as one contiguous run: each thread
// parks its vector in LDS (padded stride, the staging area of the inputs, which nobody reads any more after
// the barrier), then the run leaves in coalesced 16-byte chunks.  Called by every thread of the workgroup.
template <typename T, int NT>
__device__ __forceinline__ void store_tile(const float (&acc)[kHeadDim], bool live, char *stage, char *gdst, int n, int tid) {
    constexpr int CPK = Traits<T>::kKeyBytes / 16, STRIDE = Traits<T>::kKeyStride;
    workgroup_sync();
    if (live) store_vec32<T>(stage + tid * STRIDE, acc);
    workgroup_sync();
    const int nchunks = n * CPK;
    for (int c0 = tid; c0 < nchunks; c0 += 4 * NT) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * NT;
            if (c < nchunks) v[u] = *reinterpret_cast<const u32x4 *>(stage + (c / CPK) * STRIDE + (c % CPK) * 16);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * NT;
            if (c < nchunks) *reinterpret_cast<u32x4 *>(gdst + (size_t)c * 16) = v[u];
        }
    }
}

__host__ __device__ constexpr int align16(int n) { return (n + 15) & ~15; }

struct Tile {
    int plane, t0, n;   // plane, first position, positions in this tile
};
template <int TQ>
__device__ __forceinline__ Tile decode(int L, int tiles) {
    Tile t;
    t.plane = blockIdx.x / tiles;
    t.t0 = (blockIdx.x % tiles) * TQ;
    t.n = L - t.t0 < TQ ? L - t.t0 : TQ;
    return t;
}

// ---- logits / grad-a ------------------------------------------------------------------------

template <typename T, int TQ>
__host__ __device__ constexpr int qk_lds_bytes(int K) {
    return (TQ + K - 1) * Traits<T>::kKeyStride + align16((2 * K - 1) * 4) + mirror_bytes(TQ * K * (int)sizeof(T));
}

template <typename T, int TQ>
__global__ __launch_bounds__(TQ) void qk1d_kernel(const T *__restrict__ x, const T *__restrict__ y,
                                                  const T *__restrict__ rpb, float scale, T *__restrict__ out, int L,
                                                  int heads, int K, int tiles) {
    constexpr int KBYTES = Traits<T>::kKeyBytes, STRIDE = Traits<T>::kKeyStride;
    extern __shared__ __align__(16) char lds[];
    char *halo = lds;
    float *bias = reinterpret_cast<float *>(lds + (TQ + K - 1) * STRIDE);
    char *rows = reinterpret_cast<char *>(bias) + align16((2 * K - 1) * 4);
    const int tid = threadIdx.x;
    const Tile t = decode<TQ>(L, tiles);
    const int h0 = win_start(t.t0, L, K), h1 = win_start(t.t0 + t.n - 1, L, K) + K;   // keys [h0, h1), at most TQ + K - 1
    load_vectors<T, TQ>(reinterpret_cast<const char *>(y) + ((size_t)t.plane * L + h0) * KBYTES, h1 - h0, halo, tid);
    for (int i = tid; i < 2 * K - 1; i += TQ)
        bias[i] = rpb ? to_f32(rpb[(size_t)(t.plane % heads) * (2 * K - 1) + i]) : 0.f;
    workgroup_sync();
    const size_t g0 = ((size_t)t.plane * L + t.t0) * K * sizeof(T);   // the tile's run of logits
    if (tid < t.n) {
        const int i = t.t0 + tid;
        Vec32<T> xv;
        load_vec32(xv, reinterpret_cast<const char *>(x) + ((size_t)t.plane * L + i) * KBYTES);
        const int s = win_start(i, L, K);
        const char *kb = halo + (s - h0) * STRIDE;
        const float *bb = bias + (s - i + K - 1);
        T *orow = reinterpret_cast<T *>(rows + (int)(g0 & 15)) + tid * K;
        for (int a = 0; a < K; ++a) {
            Vec32<T> kv;
            load_vec32(kv, kb + a * STRIDE);
            orow[a] = from_f32<T>(__builtin_fmaf(scale, dot32(xv, kv), bb[a]));
        }
    }
    workgroup_sync();
    run_out<T, TQ>(reinterpret_cast<char *>(out), g0, t.n * K * (int)sizeof(T), rows, tid);
}

// ---- weighted sum / grad-q --------------------------------------------------------------------

template <typename T, int TQ>
__host__ __device__ constexpr int av_lds_bytes(int K) {
    return (TQ + K - 1) * Traits<T>::kKeyStride + mirror_bytes(TQ * K * (int)sizeof(T));
}

template <typename T, int TQ>
__global__ __launch_bounds__(TQ) void av1d_kernel(const T *__restrict__ w, const T *__restrict__ y, float scale,
                                                  T *__restrict__ out, int L, int K, int tiles) {
    constexpr int KBYTES = Traits<T>::kKeyBytes, STRIDE = Traits<T>::kKeyStride;
    extern __shared__ __align__(16) char lds[];
    char *halo = lds;
    char *rows = lds + (TQ + K - 1) * STRIDE;
    const int tid = threadIdx.x;
    const Tile t = decode<TQ>(L, tiles);
    const int h0 = win_start(t.t0, L, K), h1 = win_start(t.t0 + t.n - 1, L, K) + K;
    load_vectors<T, TQ>(reinterpret_cast<const char *>(y) + ((size_t)t.plane * L + h0) * KBYTES, h1 - h0, halo, tid);
    const size_t g0 = ((size_t)t.plane * L + t.t0) * K * sizeof(T);
    run_in<T, TQ>(reinterpret_cast<const char *>(w), g0, t.n * K * (int)sizeof(T), rows, tid);
    workgroup_sync();
    float acc[kHeadDim];
#pragma unroll
    for (int d = 0; d < kHeadDim; ++d) acc[d] = 0.f;
    if (tid < t.n) {
        const int i = t.t0 + tid;
        const int s = win_start(i, L, K);
        const char *yb = halo + (s - h0) * STRIDE;
        const T *wrow = reinterpret_cast<const T *>(rows + (int)(g0 & 15)) + tid * K;
        for (int a = 0; a < K; ++a) {
            Vec32<T> yv;
            load_vec32(yv, yb + a * STRIDE);
            axpy32(acc, to_f32(wrow[a]), yv);
        }
#pragma unroll
        for (int d = 0; d < kHeadDim; ++d) acc[d] *= scale;
    }
    store_tile<T, TQ>(acc, tid < t.n, halo, reinterpret_cast<char *>(out) + ((size_t)t.plane * L + t.t0) * KBYTES, t.n, tid);
}

// ---- grad-v / grad-k: gather over the inverse neighbourhood -------------------------------------

template <typename T, int TQ>
__host__ __device__ constexpr int inv_lds_bytes(int K) {
    return (TQ + 2 * (K - 1)) * Traits<T>::kKeyStride + mirror_bytes((TQ + 2 * (K - 1)) * K * (int)sizeof(T));
}

template <typename T, int TQ>
__global__ __launch_bounds__(TQ) void inverse1d_kernel(const T *__restrict__ w, const T *__restrict__ x, float scale,
                                                       T *__restrict__ out, int L, int K, int tiles) {
    constexpr int KBYTES = Traits<T>::kKeyBytes, STRIDE = Traits<T>::kKeyStride;
    extern __shared__ __align__(16) char lds[];
    char *halo = lds;
    char *rows = lds + (TQ + 2 * (K - 1)) * STRIDE;
    const int tid = threadIdx.x;
    const Tile t = decode<TQ>(L, tiles);
    // the queries that see any key of the tile: [i0, i1], at most TQ + 2 (K - 1) of them
    const int i0 = inv_first(t.t0, L, K), i1 = inv_last(t.t0 + t.n - 1, L, K);
    load_vectors<T, TQ>(reinterpret_cast<const char *>(x) + ((size_t)t.plane * L + i0) * KBYTES, i1 - i0 + 1, halo, tid);
    const size_t g0 = ((size_t)t.plane * L + i0) * K * sizeof(T);
    run_in<T, TQ>(reinterpret_cast<const char *>(w), g0, (i1 - i0 + 1) * K * (int)sizeof(T), rows, tid);
    workgroup_sync();
    float acc[kHeadDim];
#pragma unroll
    for (int d = 0; d < kHeadDim; ++d) acc[d] = 0.f;
    if (tid < t.n) {
        const int j = t.t0 + tid;
        const int qa = inv_first(j, L, K), qb = inv_last(j, L, K);
        const T *wbase = reinterpret_cast<const T *>(rows + (int)(g0 & 15));
        for (int i = qa; i <= qb; ++i) {
            const int a = j - win_start(i, L, K);   // slot of key j in query i's window
            Vec32<T> xv;
            load_vec32(xv, halo + (i - i0) * STRIDE);
            axpy32(acc, to_f32(wbase[(i - i0) * K + a]), xv);
        }
#pragma unroll
        for (int d = 0; d < kHeadDim; ++d) acc[d] *= scale;
    }
    store_tile<T, TQ>(acc, tid < t.n, halo, reinterpret_cast<char *>(out) + ((size_t)t.plane * L + t.t0) * KBYTES, t.n, tid);
}

// ---- softmax and its backward ----------------------------------------------------------------

template <typename T, int TQ>
__global__ __launch_bounds__(TQ) void softmax1d_kernel(const T *__restrict__ logits, T *__restrict__ out, int L, int K,
                                                       int tiles) {
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x;
    const Tile t = decode<TQ>(L, tiles);
    const size_t g0 = ((size_t)t.plane * L + t.t0) * K * sizeof(T);
    const int nbytes = t.n * K * (int)sizeof(T);
    run_in<T, TQ>(reinterpret_cast<const char *>(logits), g0, nbytes, lds, tid);
    workgroup_sync();
    if (tid < t.n) {
        T *row = reinterpret_cast<T *>(lds + (int)(g0 & 15)) + tid * K;
        constexpr float kLog2e = 1.4426950408889634f;
        float m = -INFINITY;
        for (int a = 0; a < K; ++a) m = fmaxf(m, to_f32(row[a]));
        float sum = 0.f;
        for (int a = 0; a < K; ++a) sum += __builtin_amdgcn_exp2f((to_f32(row[a]) - m) * kLog2e);
        const float inv = 1.0f / sum;
        for (int a = 0; a < K; ++a) row[a] = from_f32<T>(__builtin_amdgcn_exp2f((to_f32(row[a]) - m) * kLog2e) * inv);
    }
    workgroup_sync();
    run_out<T, TQ>(reinterpret_cast<char *>(out), g0, nbytes, lds, tid);
}

template <typename T, int TQ>
__global__ __launch_bounds__(TQ) void softmax_bwd1d_kernel(const T *__restrict__ attn, const T *__restrict__ dp,
                                                           T *__restrict__ ds, int L, int K, int tiles) {
    extern __shared__ __align__(16) char lds[];
    char *pa = lds, *pd = lds + mirror_bytes(TQ * K * (int)sizeof(T));
    const int tid = threadIdx.x;
    const Tile t = decode<TQ>(L, tiles);
    const size_t g0 = ((size_t)t.plane * L + t.t0) * K * sizeof(T);
    const int nbytes = t.n * K * (int)sizeof(T);
    run_in<T, TQ>(reinterpret_cast<const char *>(attn), g0, nbytes, pa, tid);
    run_in<T, TQ>(reinterpret_cast<const char *>(dp), g0, nbytes, pd, tid);
    workgroup_sync();
    if (tid < t.n) {
        const T *prow = reinterpret_cast<const T *>(pa + (int)(g0 & 15)) + tid * K;
        T *drow = reinterpret_cast<T *>(pd + (int)(g0 & 15)) + tid * K;
        float dot = 0.f;
        for (int a = 0; a < K; ++a) dot = __builtin_fmaf(to_f32(prow[a]), to_f32(drow[a]), dot);
        for (int a = 0; a < K; ++a) drow[a] = from_f32<T>(to_f32(prow[a]) * (to_f32(drow[a]) - dot));
    }
    workgroup_sync();
    run_out<T, TQ>(reinterpret_cast<char *>(ds), g0, nbytes, pd, tid);
}

// ---- fused forward ---------------------------------------------------------------------------

template <typename T, int TQ>
__host__ __device__ constexpr int fused_lds_bytes(int K) {
    return 2 * (TQ + K - 1) * Traits<T>::kKeyStride + align16((2 * K - 1) * 4);
}

template <typename T, int TQ>
__global__ __launch_bounds__(TQ) void fused1d_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                     const T *__restrict__ v, const T *__restrict__ rpb, float scale,
                                                     T *__restrict__ out, float *__restrict__ lse, int L, int heads, int K,
                                                     int tiles) {
    constexpr int KBYTES = Traits<T>::kKeyBytes, STRIDE = Traits<T>::kKeyStride;
    extern __shared__ __align__(16) char lds[];
    char *khalo = lds, *vhalo = lds + (TQ + K - 1) * STRIDE;
    float *bias = reinterpret_cast<float *>(lds + 2 * (TQ + K - 1) * STRIDE);
    const int tid = threadIdx.x;
    const Tile t = decode<TQ>(L, tiles);
    const int h0 = win_start(t.t0, L, K), h1 = win_start(t.t0 + t.n - 1, L, K) + K;
    const size_t hoff = ((size_t)t.plane * L + h0) * KBYTES;
    load_vectors<T, TQ>(reinterpret_cast<const char *>(k) + hoff, h1 - h0, khalo, tid);
    load_vectors<T, TQ>(reinterpret_cast<const char *>(v) + hoff, h1 - h0, vhalo, tid);
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    for (int i = tid; i < 2 * K - 1; i += TQ)
        bias[i] = rpb ? to_f32(rpb[(size_t)(t.plane % heads) * (2 * K - 1) + i]) * kLog2e : 0.f;
    workgroup_sync();
    float acc[kHeadDim];
#pragma unroll
    for (int d = 0; d < kHeadDim; ++d) acc[d] = 0.f;
    if (tid < t.n) {
        const int i = t.t0 + tid;
        Vec32<T> qv;
        load_vec32(qv, reinterpret_cast<const char *>(q) + ((size_t)t.plane * L + i) * KBYTES);
        const int s = win_start(i, L, K);
        const int off = (s - h0) * STRIDE;
        const float *bb = bias + (s - i + K - 1);
        const float scale2 = scale * kLog2e;
        // online softmax in the exp2 domain: running maximum m, running sum l, running weighted sum acc
        float m = -INFINITY, l = 0.f;
        for (int a = 0; a < K; ++a) {
            Vec32<T> kv, vv;
            load_vec32(kv, khalo + off + a * STRIDE);
            const float sv = __builtin_fmaf(scale2, dot32(qv, kv), bb[a]);
            const float mn = fmaxf(m, sv);
            const float c = __builtin_amdgcn_exp2f(m - mn);   // 0 on the first slot (m = -inf)
            const float pw = __builtin_amdgcn_exp2f(sv - mn);
            l = __builtin_fmaf(l, c, pw);
#pragma unroll
            for (int d = 0; d < kHeadDim; ++d) acc[d] *= c;
            load_vec32(vv, vhalo + off + a * STRIDE);
            axpy32(acc, pw, vv);
            m = mn;
        }
        const float inv = 1.0f / l;
#pragma unroll
        for (int d = 0; d < kHeadDim; ++d) acc[d] *= inv;
        if (lse) lse[(size_t)t.plane * L + i] = (m + __builtin_amdgcn_logf(l)) * kLn2;
    }
    store_tile<T, TQ>(acc, tid < t.n, khalo, reinterpret_cast<char *>(out) + ((size_t)t.plane * L + t.t0) * KBYTES, t.n, tid);
}

// ---- grad-b ------------------------------------------------------------------------------------
// d_rpb[h, u] = sum of ds over (batch, query, slot) with bias cell u.  Every ds becomes a 64-bit fixed-point
// integer (42 fraction bits; |ds| < 2^21) and all additions are integer additions, which commute: the
// result does not depend on which lane, wave or workgroup adds first.  Queries whose window is centred
// (all but (k-1)/2 at each end) send slot a to cell (k-1)/2 + a: those are summed across the wave first
// and one lane adds the wave's total to the workgroup's LDS table; the others add their own.  Per
// workgroup the table goes to the workspace as integers; a second kernel adds the workgroups' tables.

__device__ __forceinline__ long long to_fixed42(float x) {
    float y = x * 1024.f;
    if (!(__builtin_fabsf(y) < 2147483520.f)) y = 0.f;   // non-finite or out of range: counts as 0
    const float fl = __builtin_floorf(y);
    return (long long)(((unsigned long long)(uint32_t)(int)fl << 32) | (uint32_t)((y - fl) * 4294967296.f));
}

template <typename T, int TQ>
__host__ __device__ constexpr int rpb_lds_bytes(int K) {
    return mirror_bytes(TQ * K * (int)sizeof(T)) + (2 * K - 1) * 8;
}

template <typename T, int TQ>
__global__ __launch_bounds__(TQ) void rpb_partial1d_kernel(const T *__restrict__ ds, long long *__restrict__ partial, int L,
                                                           int K, int tiles) {
    extern __shared__ __align__(16) char lds[];
    const int NB = 2 * K - 1, R = K >> 1;
    unsigned long long *tbl = reinterpret_cast<unsigned long long *>(lds + mirror_bytes(TQ * K * (int)sizeof(T)));
    const int tid = threadIdx.x;
    const Tile t = decode<TQ>(L, tiles);
    const size_t g0 = ((size_t)t.plane * L + t.t0) * K * sizeof(T);
    run_in<T, TQ>(reinterpret_cast<const char *>(ds), g0, t.n * K * (int)sizeof(T), lds, tid);
    for (int i = tid; i < NB; i += TQ) tbl[i] = 0ull;
    workgroup_sync();
    const bool live = tid < t.n;
    const int i = t.t0 + tid;
    const int cell0 = live ? win_start(i, L, K) - i + K - 1 : R;
    const bool centred = cell0 == R;
    const T *row = reinterpret_cast<const T *>(lds + (int)(g0 & 15)) + tid * K;
    for (int a = 0; a < K; ++a) {
        const long long fx = live ? to_fixed42(to_f32(row[a])) : 0ll;
        long long tot = centred ? fx : 0ll;
#pragma unroll
        for (int sh = 1; sh < kWave; sh <<= 1) tot += __shfl_xor(tot, sh, kWave);
        if ((tid & (kWave - 1)) == 0)
            __hip_atomic_fetch_add(tbl + R + a, (unsigned long long)tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (live && !centred)
            __hip_atomic_fetch_add(tbl + cell0 + a, (unsigned long long)fx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    workgroup_sync();
    for (int u = tid; u < NB; u += TQ) partial[(size_t)blockIdx.x * NB + u] = (long long)tbl[u];
}

// one workgroup per (head, cell): adds the tables of every (batch, tile) of that head
constexpr int kFinalThreads = 256;
__global__ __launch_bounds__(kFinalThreads) void rpb_final1d_kernel(const long long *__restrict__ partial,
                                                                    float *__restrict__ d_rpb, int B, int heads, int tiles,
                                                                    int NB) {
    __shared__ long long wave_sum[kFinalThreads / kWave];
    const int h = blockIdx.x / NB, u = blockIdx.x % NB;
    const int total = B * tiles;
    long long sum = 0;
    for (int n0 = threadIdx.x; n0 < total; n0 += 4 * kFinalThreads) {
        long long v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + j * kFinalThreads;
            v[j] = n < total ? partial[(((size_t)(n / tiles) * heads + h) * tiles + n % tiles) * NB + u] : 0ll;
        }
        sum += (v[0] + v[1]) + (v[2] + v[3]);
    }
#pragma unroll
    for (int sh = 1; sh < kWave; sh <<= 1) sum += __shfl_xor(sum, sh, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) wave_sum[threadIdx.x / kWave] = sum;
    workgroup_sync();
    if (threadIdx.x == 0) {
        long long tot = 0;
        for (int w = 0; w < kFinalThreads / kWave; ++w) tot += wave_sum[w];
        d_rpb[(size_t)h * NB + u] = (float)((double)tot * (1.0 / 4398046511104.0));   // 2^-42
    }
}

// ---- fused backward ----------------------------------------------------------------------------
// dq, dk, dv and d_rpb from q, k, v, rpb, dout and the forward's log-sum-exp: the weights are recomputed as
// exp(scale <q, k> + bias - lse), so no k-wide tensor is read or written.  Two kernels, because dq sums over a
// query's window and dk / dv over a key's inverse neighbourhood:
//   * query side (one thread per query): a first sweep over the window sums delta = sum_a P_a dP_a
//     (dP_a = <dout, v_a>), a second one forms dS_a = P_a (dP_a - delta), accumulates dq += dS_a k_a and adds
//     dS_a to the bias-gradient table (64-bit fixed point, as in the unfused bias gradient).  Recomputing the two
//     dot products is cheaper than parking 2 k values per query (k is a run-time argument, up to 63);
//   * key side (one thread per key, k_j and v_j in registers): for every query i that sees key j,
//     P = exp(scale <q_i, k_j> + bias - lse_i), dP = <dout_i, v_j>, dS = P (dP - delta_i), dv += P dout_i,
//     dk += scale dS q_i, with q, dout, lse and delta of the tile's queries staged in LDS.

constexpr float kLog2eF = 1.4426950408889634f;

template <typename T, int TQ>
__host__ __device__ constexpr int fbwd_q_lds_bytes(int K) {
    return 2 * (TQ + K - 1) * Traits<T>::kKeyStride + align16((2 * K - 1) * 4) + (2 * K - 1) * 8;
}

template <typename T, int TQ>
__global__ __launch_bounds__(TQ) void fbwd1d_q_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                      const T *__restrict__ v, const T *__restrict__ rpb, float scale,
                                                      const float *__restrict__ lse, const T *__restrict__ dout,
                                                      T *__restrict__ dq, float *__restrict__ delta_out,
                                                      long long *__restrict__ partial, int L, int heads, int K, int tiles) {
    constexpr int KBYTES = Traits<T>::kKeyBytes, STRIDE = Traits<T>::kKeyStride;
    extern __shared__ __align__(16) char lds[];
    const int NB = 2 * K - 1, R = K >> 1;
    char *khalo = lds, *vhalo = lds + (TQ + K - 1) * STRIDE;
    float *bias = reinterpret_cast<float *>(lds + 2 * (TQ + K - 1) * STRIDE);
    unsigned long long *tbl = reinterpret_cast<unsigned long long *>(reinterpret_cast<char *>(bias) + align16(NB * 4));
    const int tid = threadIdx.x;
    const Tile t = decode<TQ>(L, tiles);
    const int h0 = win_start(t.t0, L, K), h1 = win_start(t.t0 + t.n - 1, L, K) + K;
    const size_t hoff = ((size_t)t.plane * L + h0) * KBYTES;
    load_vectors<T, TQ>(reinterpret_cast<const char *>(k) + hoff, h1 - h0, khalo, tid);
    load_vectors<T, TQ>(reinterpret_cast<const char *>(v) + hoff, h1 - h0, vhalo, tid);
    for (int i = tid; i < NB; i += TQ) {
        bias[i] = rpb ? to_f32(rpb[(size_t)(t.plane % heads) * NB + i]) * kLog2eF : 0.f;
        tbl[i] = 0ull;
    }
    workgroup_sync();
    const bool live = tid < t.n;
    const int i = t.t0 + (live ? tid : 0);
    const size_t qi = (size_t)t.plane * L + i;
    Vec32<T> qv, gv;
    load_vec32(qv, reinterpret_cast<const char *>(q) + qi * KBYTES);
    load_vec32(gv, reinterpret_cast<const char *>(dout) + qi * KBYTES);
    const float lse2 = lse[qi] * kLog2eF, scale2 = scale * kLog2eF;
    const int s = win_start(i, L, K);
    const int off = (s - h0) * STRIDE;
    const int cell0 = s - i + K - 1;
    const bool centred = cell0 == R;
    const float *bb = bias + cell0;
    // sweep 1: delta
    float delta = 0.f;
    for (int a = 0; a < K; ++a) {
        Vec32<T> kv, vv;
        load_vec32(kv, khalo + off + a * STRIDE);
        load_vec32(vv, vhalo + off + a * STRIDE);
        const float pw = __builtin_amdgcn_exp2f(__builtin_fmaf(scale2, dot32(qv, kv), bb[a]) - lse2);
        delta = __builtin_fmaf(pw, dot32(gv, vv), delta);
    }
    // sweep 2: dS, dq, bias gradient
    float acc[kHeadDim];
#pragma unroll
    for (int d = 0; d < kHeadDim; ++d) acc[d] = 0.f;
    for (int a = 0; a < K; ++a) {
        Vec32<T> kv, vv;
        load_vec32(kv, khalo + off + a * STRIDE);
        load_vec32(vv, vhalo + off + a * STRIDE);
        const float pw = __builtin_amdgcn_exp2f(__builtin_fmaf(scale2, dot32(qv, kv), bb[a]) - lse2);
        const float ds = live ? pw * (dot32(gv, vv) - delta) : 0.f;
        axpy32(acc, ds, kv);
        if (partial != nullptr) {   // the same for every thread
            const long long fx = to_fixed42(ds);
            long long tot = centred ? fx : 0ll;
#pragma unroll
            for (int sh = 1; sh < kWave; sh <<= 1) tot += __shfl_xor(tot, sh, kWave);
            if ((tid & (kWave - 1)) == 0)
                __hip_atomic_fetch_add(tbl + R + a, (unsigned long long)tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (live && !centred)
                __hip_atomic_fetch_add(tbl + cell0 + a, (unsigned long long)fx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
#pragma unroll
    for (int d = 0; d < kHeadDim; ++d) acc[d] *= scale;
    if (live) delta_out[qi] = delta;
    store_tile<T, TQ>(acc, live, khalo, reinterpret_cast<char *>(dq) + ((size_t)t.plane * L + t.t0) * KBYTES, t.n, tid);
    if (partial != nullptr)   // (store_tile's barriers have passed: every atomic of the workgroup is done)
        for (int u = tid; u < NB; u += TQ) partial[(size_t)blockIdx.x * NB + u] = (long long)tbl[u];
}

template <typename T, int TQ>
__host__ __device__ constexpr int fbwd_kv_lds_bytes(int K) {
    return 2 * (TQ + 2 * (K - 1)) * Traits<T>::kKeyStride + 2 * align16((TQ + 2 * (K - 1)) * 4) + align16((2 * K - 1) * 4);
}

template <typename T, int TQ>
__global__ __launch_bounds__(TQ) void fbwd1d_kv_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                       const T *__restrict__ v, const T *__restrict__ rpb, float scale,
                                                       const float *__restrict__ lse, const float *__restrict__ delta,
                                                       const T *__restrict__ dout, T *__restrict__ dk, T *__restrict__ dv,
                                                       int L, int heads, int K, int tiles) {
    constexpr int KBYTES = Traits<T>::kKeyBytes, STRIDE = Traits<T>::kKeyStride;
    extern __shared__ __align__(16) char lds[];
    const int NB = 2 * K - 1, NQ = TQ + 2 * (K - 1);
    char *qhalo = lds, *ghalo = lds + NQ * STRIDE;
    float *lse_s = reinterpret_cast<float *>(lds + 2 * NQ * STRIDE);
    float *delta_s = lse_s + align16(NQ * 4) / 4;
    float *bias = delta_s + align16(NQ * 4) / 4;
    const int tid = threadIdx.x;
    const Tile t = decode<TQ>(L, tiles);
    const int i0 = inv_first(t.t0, L, K), i1 = inv_last(t.t0 + t.n - 1, L, K);   // the queries that see the tile: at most NQ
    const size_t ioff = (size_t)t.plane * L + i0;
    load_vectors<T, TQ>(reinterpret_cast<const char *>(q) + ioff * KBYTES, i1 - i0 + 1, qhalo, tid);
    load_vectors<T, TQ>(reinterpret_cast<const char *>(dout) + ioff * KBYTES, i1 - i0 + 1, ghalo, tid);
    for (int u = tid; u <= i1 - i0; u += TQ) {
        lse_s[u] = lse[ioff + u] * kLog2eF;
        delta_s[u] = delta[ioff + u];
    }
    for (int u = tid; u < NB; u += TQ) bias[u] = rpb ? to_f32(rpb[(size_t)(t.plane % heads) * NB + u]) * kLog2eF : 0.f;
    workgroup_sync();
    const bool live = tid < t.n;
    const int j = t.t0 + (live ? tid : 0);
    const size_t kj = (size_t)t.plane * L + j;
    Vec32<T> kv, vv;
    load_vec32(kv, reinterpret_cast<const char *>(k) + kj * KBYTES);
    load_vec32(vv, reinterpret_cast<const char *>(v) + kj * KBYTES);
    const float scale2 = scale * kLog2eF;
    float dk_acc[kHeadDim], dv_acc[kHeadDim];
#pragma unroll
    for (int d = 0; d < kHeadDim; ++d) dk_acc[d] = dv_acc[d] = 0.f;
    if (live) {
        const int qa = inv_first(j, L, K), qb = inv_last(j, L, K);
        for (int i = qa; i <= qb; ++i) {
            Vec32<T> qv, gv;
            load_vec32(qv, qhalo + (i - i0) * STRIDE);
            load_vec32(gv, ghalo + (i - i0) * STRIDE);
            const float pw = __builtin_amdgcn_exp2f(__builtin_fmaf(scale2, dot32(qv, kv), bias[j - i + K - 1]) - lse_s[i - i0]);
            const float ds = pw * (dot32(gv, vv) - delta_s[i - i0]);
            axpy32(dv_acc, pw, gv);
            axpy32(dk_acc, ds, qv);
        }
#pragma unroll
        for (int d = 0; d < kHeadDim; ++d) dk_acc[d] *= scale;
    }
    char *gbase_k = reinterpret_cast<char *>(dk) + ((size_t)t.plane * L + t.t0) * KBYTES;
    char *gbase_v = reinterpret_cast<char *>(dv) + ((size_t)t.plane * L + t.t0) * KBYTES;
    store_tile<T, TQ>(dk_acc, live, qhalo, gbase_k, t.n, tid);
    store_tile<T, TQ>(dv_acc, live, ghalo, gbase_v, t.n, tid);
}

// ---- launchers ---------------------------------------------------------------------------------

// Dynamic LDS beyond 64 KB needs the attribute (allow_lds); it is set to the most the kernel can ask for.
using na2d::allow_lds;
template <int TQ> constexpr int max_k() { return TQ == 256 ? 31 : kMaxK; }

#define NA1D_DISPATCH(p, ...)                                                            \
    do {                                                                                 \
        if ((p).K <= 31) {                                                               \
            constexpr int TQ = 256;                                                      \
            NA2D_DISPATCH_T((p).dtype, __VA_ARGS__);                                     \
        } else {                                                                         \
            constexpr int TQ = 128;                                                      \
            NA2D_DISPATCH_T((p).dtype, __VA_ARGS__);                                     \
        }                                                                                \
    } while (0)

template <int TQ>
static int tiles_of(const Problem &p) { return (p.L + TQ - 1) / TQ; }

template <typename T, int TQ>
static hipError_t qk_t(const Problem &p, const void *x, const void *y, const void *rpb, float scale, void *out, hipStream_t s) {
    auto kern = qk1d_kernel<T, TQ>;
    static_assert(qk_lds_bytes<T, TQ>(max_k<TQ>()) <= 160 * 1024, "LDS");
    const int bytes = qk_lds_bytes<T, TQ>(p.K), tiles = tiles_of<TQ>(p);
    static na2d::LdsAllowed attr;
    if (hipError_t e = allow_lds(kern, qk_lds_bytes<T, TQ>(max_k<TQ>()), attr); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.planes() * tiles), dim3(TQ), bytes, s, static_cast<const T *>(x),
                       static_cast<const T *>(y), static_cast<const T *>(rpb), scale, static_cast<T *>(out), p.L, p.heads,
                       p.K, tiles);
    return hipGetLastError();
}
hipError_t launch_qk(const Problem &p, const void *x, const void *y, const void *rpb, float scale, void *out, hipStream_t s) {
    NA1D_DISPATCH(p, return (qk_t<T, TQ>(p, x, y, rpb, scale, out, s)));
    return hipErrorInvalidValue;
}

template <typename T, int TQ>
static hipError_t av_t(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s) {
    auto kern = av1d_kernel<T, TQ>;
    static_assert(av_lds_bytes<T, TQ>(max_k<TQ>()) <= 160 * 1024, "LDS");
    const int bytes = av_lds_bytes<T, TQ>(p.K), tiles = tiles_of<TQ>(p);
    static na2d::LdsAllowed attr;
    if (hipError_t e = allow_lds(kern, av_lds_bytes<T, TQ>(max_k<TQ>()), attr); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.planes() * tiles), dim3(TQ), bytes, s, static_cast<const T *>(w),
                       static_cast<const T *>(y), scale, static_cast<T *>(out), p.L, p.K, tiles);
    return hipGetLastError();
}
hipError_t launch_av(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s) {
    NA1D_DISPATCH(p, return (av_t<T, TQ>(p, w, y, scale, out, s)));
    return hipErrorInvalidValue;
}

template <typename T, int TQ>
static hipError_t inverse_t(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s) {
    auto kern = inverse1d_kernel<T, TQ>;
    static_assert(inv_lds_bytes<T, TQ>(max_k<TQ>()) <= 160 * 1024, "LDS");
    const int bytes = inv_lds_bytes<T, TQ>(p.K), tiles = tiles_of<TQ>(p);
    static na2d::LdsAllowed attr;
    if (hipError_t e = allow_lds(kern, inv_lds_bytes<T, TQ>(max_k<TQ>()), attr); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.planes() * tiles), dim3(TQ), bytes, s, static_cast<const T *>(w),
                       static_cast<const T *>(x), scale, static_cast<T *>(out), p.L, p.K, tiles);
    return hipGetLastError();
}
hipError_t launch_inverse(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s) {
    NA1D_DISPATCH(p, return (inverse_t<T, TQ>(p, w, x, scale, out, s)));
    return hipErrorInvalidValue;
}

template <typename T, int TQ>
static hipError_t softmax_t(const Problem &p, const void *logits, void *out, hipStream_t s) {
    auto kern = softmax1d_kernel<T, TQ>;
    const int bytes = mirror_bytes(TQ * p.K * (int)sizeof(T)), tiles = tiles_of<TQ>(p);
    static na2d::LdsAllowed attr;
    if (hipError_t e = allow_lds(kern, mirror_bytes(TQ * max_k<TQ>() * (int)sizeof(T)), attr); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.planes() * tiles), dim3(TQ), bytes, s, static_cast<const T *>(logits),
                       static_cast<T *>(out), p.L, p.K, tiles);
    return hipGetLastError();
}
hipError_t launch_softmax(const Problem &p, const void *logits, void *out, hipStream_t s) {
    NA1D_DISPATCH(p, return (softmax_t<T, TQ>(p, logits, out, s)));
    return hipErrorInvalidValue;
}

template <typename T, int TQ>
static hipError_t softmax_bwd_t(const Problem &p, const void *attn, const void *dp, void *ds, hipStream_t s) {
    auto kern = softmax_bwd1d_kernel<T, TQ>;
    const int bytes = 2 * mirror_bytes(TQ * p.K * (int)sizeof(T)), tiles = tiles_of<TQ>(p);
    static na2d::LdsAllowed attr;
    if (hipError_t e = allow_lds(kern, 2 * mirror_bytes(TQ * max_k<TQ>() * (int)sizeof(T)), attr); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.planes() * tiles), dim3(TQ), bytes, s, static_cast<const T *>(attn),
                       static_cast<const T *>(dp), static_cast<T *>(ds), p.L, p.K, tiles);
    return hipGetLastError();
}
hipError_t launch_softmax_bwd(const Problem &p, const void *attn, const void *dp, void *ds, hipStream_t s) {
    NA1D_DISPATCH(p, return (softmax_bwd_t<T, TQ>(p, attn, dp, ds, s)));
    return hipErrorInvalidValue;
}

template <typename T, int TQ>
static hipError_t fused_t(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                          void *out, float *lse, hipStream_t s) {
    auto kern = fused1d_kernel<T, TQ>;
    static_assert(fused_lds_bytes<T, TQ>(max_k<TQ>()) <= 160 * 1024, "LDS");
    const int bytes = fused_lds_bytes<T, TQ>(p.K), tiles = tiles_of<TQ>(p);
    static na2d::LdsAllowed attr;
    if (hipError_t e = allow_lds(kern, fused_lds_bytes<T, TQ>(max_k<TQ>()), attr); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(p.planes() * tiles), dim3(TQ), bytes, s, static_cast<const T *>(q),
                       static_cast<const T *>(k), static_cast<const T *>(v), static_cast<const T *>(rpb), scale,
                       static_cast<T *>(out), lse, p.L, p.heads, p.K, tiles);
    return hipGetLastError();
}
hipError_t launch_fused_fwd(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                            void *out, float *lse, hipStream_t s) {
    NA1D_DISPATCH(p, return (fused_t<T, TQ>(p, q, k, v, rpb, scale, out, lse, s)));
    return hipErrorInvalidValue;
}

static int rpb_tiles(const Problem &p) { return p.K <= 31 ? tiles_of<256>(p) : tiles_of<128>(p); }

size_t rpb_workspace_bytes(const Problem &p) {
    return (size_t)p.planes() * rpb_tiles(p) * (2 * p.K - 1) * sizeof(long long);
}

template <typename T, int TQ>
static hipError_t rpb_t(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s) {
    auto kern = rpb_partial1d_kernel<T, TQ>;
    const int bytes = rpb_lds_bytes<T, TQ>(p.K), tiles = tiles_of<TQ>(p);
    static na2d::LdsAllowed attr;
    if (hipError_t e = allow_lds(kern, rpb_lds_bytes<T, TQ>(max_k<TQ>()), attr); e != hipSuccess) return e;
    long long *partial = static_cast<long long *>(workspace);
    hipLaunchKernelGGL(kern, dim3(p.planes() * tiles), dim3(TQ), bytes, s, static_cast<const T *>(ds), partial, p.L, p.K, tiles);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    const int NB = 2 * p.K - 1;
    hipLaunchKernelGGL(rpb_final1d_kernel, dim3(p.heads * NB), dim3(kFinalThreads), 0, s, partial, d_rpb, p.B, p.heads, tiles, NB);
    return hipGetLastError();
}
hipError_t launch_rpb_grad(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s) {
    NA1D_DISPATCH(p, return (rpb_t<T, TQ>(p, ds, d_rpb, workspace, s)));
    return hipErrorInvalidValue;
}

size_t fused_bwd_workspace_bytes(const Problem &p) {
    const size_t delta_bytes = ((size_t)p.planes() * p.L * sizeof(float) + 255) & ~(size_t)255;
    return delta_bytes + rpb_workspace_bytes(p);
}

template <typename T, int TQ>
static hipError_t fused_bwd_t(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                              const float *lse, const void *dout, void *dq, void *dk, void *dv, float *d_rpb,
                              void *workspace, hipStream_t s) {
    const int tiles = tiles_of<TQ>(p), NB = 2 * p.K - 1;
    float *delta = static_cast<float *>(workspace);
    const size_t delta_bytes = ((size_t)p.planes() * p.L * sizeof(float) + 255) & ~(size_t)255;
    long long *partial = d_rpb ? reinterpret_cast<long long *>(static_cast<char *>(workspace) + delta_bytes) : nullptr;
    {
        auto kern = fbwd1d_q_kernel<T, TQ>;
        static_assert(fbwd_q_lds_bytes<T, TQ>(max_k<TQ>()) <= 160 * 1024, "LDS");
        static na2d::LdsAllowed attr;
        if (hipError_t e = allow_lds(kern, fbwd_q_lds_bytes<T, TQ>(max_k<TQ>()), attr); e != hipSuccess) return e;
        const int bytes = fbwd_q_lds_bytes<T, TQ>(p.K);
        hipLaunchKernelGGL(kern, dim3(p.planes() * tiles), dim3(TQ), bytes, s,
                           static_cast<const T *>(q), static_cast<const T *>(k), static_cast<const T *>(v),
                           static_cast<const T *>(rpb), scale, lse, static_cast<const T *>(dout), static_cast<T *>(dq), delta,
                           partial, p.L, p.heads, p.K, tiles);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    {
        auto kern = fbwd1d_kv_kernel<T, TQ>;
        static_assert(fbwd_kv_lds_bytes<T, TQ>(max_k<TQ>()) <= 160 * 1024, "LDS");
        static na2d::LdsAllowed attr;
        if (hipError_t e = allow_lds(kern, fbwd_kv_lds_bytes<T, TQ>(max_k<TQ>()), attr); e != hipSuccess) return e;
        const int bytes = fbwd_kv_lds_bytes<T, TQ>(p.K);
        hipLaunchKernelGGL(kern, dim3(p.planes() * tiles), dim3(TQ), bytes, s,
                           static_cast<const T *>(q), static_cast<const T *>(k), static_cast<const T *>(v),
                           static_cast<const T *>(rpb), scale, lse, delta, static_cast<const T *>(dout), static_cast<T *>(dk),
                           static_cast<T *>(dv), p.L, p.heads, p.K, tiles);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    if (d_rpb) {
        hipLaunchKernelGGL(rpb_final1d_kernel, dim3(p.heads * NB), dim3(kFinalThreads), 0, s, partial, d_rpb, p.B, p.heads, tiles, NB);
        return hipGetLastError();
    }
    return hipSuccess;
}
hipError_t launch_fused_bwd(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                            const float *lse, const void *dout, void *dq, void *dk, void *dv, float *d_rpb, void *workspace,
                            hipStream_t s) {
    NA1D_DISPATCH(p, return (fused_bwd_t<T, TQ>(p, q, k, v, rpb, scale, lse, dout, dq, dk, dv, d_rpb, workspace, s)));
    return hipErrorInvalidValue;
}

}  // namespace na1d
