// Shared device/host helpers of the gfx950 2D Neighborhood Attention kernels.
//
// Neighbourhood definition: arXiv 2204.07143, Section 3.1 (k nearest neighbours per axis,
// Eq. 2) and the Appendix figure "3x3 NA on a 7x7 map" (window shifted, not shrunk, at the
// borders).  Everything in this header is index arithmetic, storage-type conversion and
// LDS staging; the attention arithmetic lives in the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "na2d.h"

namespace na2d {

constexpr int kHeadDim = 32;       // D of every NAT variant (Section 3.2): the matrix-core kernels are built for it
// 16-channel heads on the 32-channel matrix-core kernels (16-bit types, small windows): a position's 32 bytes are
// copied into both halves of its 64-byte slot in LDS (chunk index & kHalfDimChunks).  Where the contraction runs
// over channels (logits, grad-a) the query operand of the lanes that hold channels 16..31 is zero, so the copy
// meets zeros; where channels are independent (weighted sums) the upper 16 results repeat the lower ones and only
// the lanes with channels 0..15 store.  Twice the matrix-core and LDS work the head needs, on pipelines that are
// bound by neither; the plain-ALU kernels this replaces were three to six times slower.
constexpr int kHalfDim = 16;
constexpr int kHalfDimChunks = 1;
constexpr int kWave = 64;          // CDNA wavefront width

// ---- neighbourhood index functions (one axis of length L, odd window K <= L) -----------

// First key coordinate seen by query coordinate i.
__host__ __device__ __forceinline__ int win_start(int i, int L, int K) {
    int s = i - (K >> 1);
    s = s < 0 ? 0 : s;
    int hi = L - K;
    return s > hi ? hi : s;
}

// Row/column of the bias table that window slot 0 of query coordinate i maps to:
// key - query + (K - 1) with key = win_start(i).
__host__ __device__ __forceinline__ int rpb_start(int i, int L, int K) {
    return win_start(i, L, K) - i + (K - 1);
}

// Inverse neighbourhood: the queries whose window holds key coordinate j form the contiguous
// range [inv_first(j), inv_last(j)].
__host__ __device__ __forceinline__ int inv_first(int j, int L, int K) {
    (void)L;
    return j <= K - 1 ? 0 : j - (K >> 1);
}
__host__ __device__ __forceinline__ int inv_last(int j, int L, int K) {
    return j >= L - K ? L - 1 : j + (K >> 1);
}

// ---- storage types -------------------------------------------------------------------

typedef _Float16 f16_t;
typedef __bf16 bf16_t;
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T> struct Traits;
template <> struct Traits<float> {
    static constexpr int kDtype = NA2D_F32;
    static constexpr int kKeyBytes = kHeadDim * 4;
    static constexpr int kKeyStride = kKeyBytes + 16;   // LDS stride of one key: 36 dwords, conflict-free for b128 reads
};
template <> struct Traits<f16_t> {
    static constexpr int kDtype = NA2D_F16;
    static constexpr int kKeyBytes = kHeadDim * 2;
    static constexpr int kKeyStride = kKeyBytes + 16;   // 20 dwords
};
template <> struct Traits<bf16_t> {
    static constexpr int kDtype = NA2D_BF16;
    static constexpr int kKeyBytes = kHeadDim * 2;
    static constexpr int kKeyStride = kKeyBytes + 16;
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(f16_t x) { return (float)x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }

template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ f16_t from_f32<f16_t>(float x) { return (f16_t)x; }   // round-to-nearest-even
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; } // round-to-nearest-even

// Byte size of a head vector of D elements and its padded LDS stride (+16 bytes: consecutive keys start
// 4 banks apart, so 16-byte LDS reads of neighbouring keys do not collide).
template <typename T, int D> struct VecTraits {
    static_assert(D % 8 == 0, "a head vector is a whole number of 16-byte chunks in every storage type");
    static constexpr int kKeyBytes = D * (int)sizeof(T);
    static constexpr int kKeyStride = kKeyBytes + 16;
};

// A head vector (D elements) held in registers in its storage type, as 32-bit words.
template <typename T, int D = kHeadDim> struct VecN {
    static constexpr int kChunks = VecTraits<T, D>::kKeyBytes / 16;
    static constexpr int kWords = VecTraits<T, D>::kKeyBytes / 4;
    uint32_t w[kWords];
};
template <typename T> using Vec32 = VecN<T, kHeadDim>;

template <typename T, int D>
__device__ __forceinline__ void load_vec32(VecN<T, D> &v, const void *p) {
    const u32x4 *s = reinterpret_cast<const u32x4 *>(p);
#pragma unroll
    for (int i = 0; i < VecN<T, D>::kChunks; ++i) {
        const u32x4 t = s[i];
        v.w[4 * i + 0] = t.x;
        v.w[4 * i + 1] = t.y;
        v.w[4 * i + 2] = t.z;
        v.w[4 * i + 3] = t.w;
    }
}

// fp32 dot product of two head vectors held in storage type.
template <int D>
__device__ __forceinline__ float dot32(const VecN<float, D> &a, const VecN<float, D> &b) {
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < D; ++i) acc = __builtin_fmaf(__uint_as_float(a.w[i]), __uint_as_float(b.w[i]), acc);
    return acc;
}
template <int D>
__device__ __forceinline__ float dot32(const VecN<f16_t, D> &a, const VecN<f16_t, D> &b) {
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < D / 2; ++i) {
        const uint32_t ua = a.w[i], ub = b.w[i];
        acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, ua), __builtin_bit_cast(f16x2, ub), acc, false);
    }
    return acc;
}
template <int D>
__device__ __forceinline__ float dot32(const VecN<bf16_t, D> &a, const VecN<bf16_t, D> &b) {
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < D / 2; ++i) {
        const uint32_t ua = a.w[i], ub = b.w[i];
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, ua), __builtin_bit_cast(bf16x2, ub), acc, false);
    }
    return acc;
}

// acc[0..D-1] += w * v  (fp32 accumulate, v in storage type).
template <int D>
__device__ __forceinline__ void axpy32(float (&acc)[D], float w, const VecN<float, D> &v) {
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] = __builtin_fmaf(w, __uint_as_float(v.w[i]), acc[i]);
}
template <int D>
__device__ __forceinline__ void axpy32(float (&acc)[D], float w, const VecN<f16_t, D> &v) {
#pragma unroll
    for (int i = 0; i < D / 2; ++i) {
        const uint32_t u = v.w[i];
        const f16_t lo = __builtin_bit_cast(f16_t, (uint16_t)(u & 0xffffu));
        const f16_t hi = __builtin_bit_cast(f16_t, (uint16_t)(u >> 16));
        acc[2 * i] = __builtin_fmaf(w, (float)lo, acc[2 * i]);
        acc[2 * i + 1] = __builtin_fmaf(w, (float)hi, acc[2 * i + 1]);
    }
}
template <int D>
__device__ __forceinline__ void axpy32(float (&acc)[D], float w, const VecN<bf16_t, D> &v) {
#pragma unroll
    for (int i = 0; i < D / 2; ++i) {
        const uint32_t u = v.w[i];
        acc[2 * i] = __builtin_fmaf(w, __uint_as_float(u << 16), acc[2 * i]);
        acc[2 * i + 1] = __builtin_fmaf(w, __uint_as_float(u & 0xffff0000u), acc[2 * i + 1]);
    }
}

// Store D fp32 values as one head vector in storage type (p is 16-byte aligned).
template <typename T, int D>
__device__ __forceinline__ void store_vec32(void *p, const float (&x)[D]) {
    if constexpr (sizeof(T) == 4) {
        f32x4 *d = reinterpret_cast<f32x4 *>(p);
#pragma unroll
        for (int i = 0; i < D / 4; ++i) d[i] = f32x4{x[i * 4], x[i * 4 + 1], x[i * 4 + 2], x[i * 4 + 3]};
    } else {
        u32x4 *d = reinterpret_cast<u32x4 *>(p);
        uint32_t w[D / 2];
#pragma unroll
        for (int i = 0; i < D / 2; ++i) {
            const T lo = from_f32<T>(x[2 * i]), hi = from_f32<T>(x[2 * i + 1]);
            w[i] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
        }
#pragma unroll
        for (int i = 0; i < D / 8; ++i) d[i] = u32x4{w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]};
    }
}

// ---- raw LDS addressing ----------------------------------------------------------------
// 32-bit LDS byte address of a __shared__ object, and the reverse: lets kernels keep tables of
// absolute LDS addresses in registers and store through them with plain ds_write instructions.
typedef __attribute__((address_space(3))) char lds_char_t;
__device__ __forceinline__ int lds_addr(const void *p) {
    return (int)(uintptr_t)(const lds_char_t *)p;
}
template <typename T>
__device__ __forceinline__ __attribute__((address_space(3))) T *lds_ptr(int addr) {
    return (__attribute__((address_space(3))) T *)(uintptr_t)(unsigned)addr;
}

// ---- streaming stores ---------------------------------------------------------------------------
// The head-dim results of the path (out, dq, dk, dv) are not read again by any of its kernels: their 16-byte
// stores carry the non-temporal hint, which keeps them from displacing what the kernels that follow will read
// (a plain device copy gains about 6 % from the hint on this chip; weighted sum 20.4 -> 18.1 us, grad-q
// 19.6 -> 17.2 us, grad-v / grad-k 24.5 -> 23.6 us at the benchmark shape).  The attention-shaped results
// (logits, weights, dp, ds) keep plain stores: the next kernel of the path reads them, out of the last-level
// cache when it follows at once; streaming them as well made each producer faster by itself (logits
// 24.2 -> 21.4 us) and the ten-call step slower.  (The logits kernel streams them all the same once the tensor
// has 48 MB or more: see its launcher.)  `p` may be aligned to the element only.
typedef u32x4 __attribute__((aligned(2))) u32x4_unaligned;
__device__ __forceinline__ void store16_stream(void *p, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_unaligned *>(p));
}

// ---- measurement build ------------------------------------------------------------------------
// Built with -DNA2D_PROBE_MEMORY_ONLY (a separate library for the benchmark, never the product), the tiled
// 16-bit contraction kernels keep every load and store of a launch and leave out the arithmetic between
// them (LDS gathers, matrix-core products, conversions): the time of such a launch is what the memory
// system takes for this access pattern, the bound the real kernel is held against.
#ifdef NA2D_PROBE_MEMORY_ONLY
constexpr bool kProbeMemoryOnly = true;
#else
constexpr bool kProbeMemoryOnly = false;
#endif

// ---- workgroup barrier -----------------------------------------------------------------------
// A workgroup barrier that orders LDS accesses across it.  __syncthreads() is a release fence, s_barrier
// and an acquire fence; the wait for the wave's outstanding LDS accesses that the release fence stands for
// is inserted by the compiler, and at the header of a loop whose back edge ends in LDS stores the compiler
// has left it out (seen in the generated code of the fused grad-a / softmax-backward kernel: the wave passed
// the barrier with its last stores still in flight and, once in a few million elements, another wave read
// the old contents).  The wait is therefore written out in front of every barrier of this library.
__device__ __forceinline__ void workgroup_sync() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();
}

// ---- alignment-preserving staging between global memory and LDS -------------------------
//
// A run of `nbytes` bytes starting at global byte offset g0 of `gbase` (gbase 16-byte
// aligned, g0 a multiple of sizeof(T)) is mirrored in an LDS region at offset (g0 & 15), so
// that 16-byte aligned global chunks map to 16-byte aligned LDS chunks.  Chunks that lie
// fully inside the run move as one 16-byte access; the ragged head and tail (fewer than 16
// bytes each) move element by element.  The region needs mirror_bytes(nbytes) bytes.
//
// All global loads of a stager are issued before the first LDS store, so a thread has its
// whole share of the run in flight at once instead of paying one memory latency per chunk.
// MAXBYTES bounds nbytes at compile time (it fixes the register footprint).

struct RunSplit {
    int mis, span, body_lo, body_hi;   // full 16-byte chunks cover [body_lo, body_hi)
};
__device__ __forceinline__ RunSplit split_run(size_t g0, int nbytes) {
    RunSplit r;
    r.mis = (int)(g0 & 15);
    r.span = r.mis + nbytes;
    r.body_lo = (r.mis + 15) & ~15;
    r.body_hi = r.span & ~15;
    if (r.body_hi < r.body_lo) r.body_hi = r.body_lo;   // no full chunk
    return r;
}

template <typename T, int MAXBYTES, int NTHREADS>
struct StageIn {
    static constexpr int kMaxChunks = (MAXBYTES + 15) / 16 + 1;
    static constexpr int NITER = (kMaxChunks + NTHREADS - 1) / NTHREADS;
    u32x4 v[NITER];
    RunSplit rs;
    const char *ga;

    __device__ __forceinline__ void issue(const char *gbase, size_t g0, int nbytes, int tid) {
        rs = split_run(g0, nbytes);
        ga = gbase + (g0 - rs.mis);
#pragma unroll
        for (int it = 0; it < NITER; ++it) {
            const int lo = rs.body_lo + ((tid + it * NTHREADS) << 4);
            if (lo < rs.body_hi) v[it] = *reinterpret_cast<const u32x4 *>(ga + lo);
        }
    }
    __device__ __forceinline__ void commit(char *region, int tid) const {
#pragma unroll
        for (int it = 0; it < NITER; ++it) {
            const int lo = rs.body_lo + ((tid + it * NTHREADS) << 4);
            if (lo < rs.body_hi) *reinterpret_cast<u32x4 *>(region + lo) = v[it];
        }
        // ragged head [mis, min(body_lo, span)) and tail [max(body_hi, body_lo) .. span): element-wise
        const int head_end = rs.body_lo < rs.span ? rs.body_lo : rs.span;
        const int hb = rs.mis + tid * (int)sizeof(T);
        if (hb < head_end) *reinterpret_cast<T *>(region + hb) = *reinterpret_cast<const T *>(ga + hb);
        const int tb = rs.body_hi + (tid - 16) * (int)sizeof(T);
        if (tid >= 16 && rs.body_hi >= head_end && tb < rs.span)
            *reinterpret_cast<T *>(region + tb) = *reinterpret_cast<const T *>(ga + tb);
    }
};

// One-shot form (issue + commit).
template <typename T, int MAXBYTES, int NTHREADS>
__device__ __forceinline__ void stage_in(const char *gbase, size_t g0, int nbytes, char *region, int tid) {
    StageIn<T, MAXBYTES, NTHREADS> st;
    st.issue(gbase, g0, nbytes, tid);
    st.commit(region, tid);
}

template <typename T, int MAXBYTES, int NTHREADS>
__device__ __forceinline__ void stage_out(char *gbase, size_t g0, int nbytes, const char *region, int tid) {
    constexpr int kMaxChunks = (MAXBYTES + 15) / 16 + 1;
    constexpr int NITER = (kMaxChunks + NTHREADS - 1) / NTHREADS;
    const RunSplit rs = split_run(g0, nbytes);
    char *ga = gbase + (g0 - rs.mis);
    u32x4 v[NITER];
#pragma unroll
    for (int it = 0; it < NITER; ++it) {
        const int lo = rs.body_lo + ((tid + it * NTHREADS) << 4);
        if (lo < rs.body_hi) v[it] = *reinterpret_cast<const u32x4 *>(region + lo);
    }
#pragma unroll
    for (int it = 0; it < NITER; ++it) {
        const int lo = rs.body_lo + ((tid + it * NTHREADS) << 4);
        if (lo < rs.body_hi) *reinterpret_cast<u32x4 *>(ga + lo) = v[it];
    }
    const int head_end = rs.body_lo < rs.span ? rs.body_lo : rs.span;
    const int hb = rs.mis + tid * (int)sizeof(T);
    if (hb < head_end) *reinterpret_cast<T *>(ga + hb) = *reinterpret_cast<const T *>(region + hb);
    const int tb = rs.body_hi + (tid - 16) * (int)sizeof(T);
    if (tid >= 16 && rs.body_hi >= head_end && tb < rs.span)
        *reinterpret_cast<T *>(ga + tb) = *reinterpret_cast<const T *>(region + tb);
}

// Bytes an LDS mirror region must have for a run of nbytes.
__host__ __device__ constexpr int mirror_bytes(int nbytes) { return (nbytes + 30 + 15) & ~15; }

// ---- host-side launch description ---------------------------------------------------

struct Geo {
    int B, heads, H, W;
    int planes;      // B * heads
};

}  // namespace na2d
