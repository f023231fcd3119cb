// Matrix-core building blocks of the tiled 16-bit kernels.
//
// A 4 x 4 patch of queries and the (4+K-1)^2 keys its windows can touch form a small dense
// contraction over the head dimension (16 queries x PW*PW keys x 32), masked afterwards by the
// window of each query (arXiv 2204.07143, Eq. 2; the paper names NA as an implicit GEMM as
// future work, Appendix A).  It is evaluated as S^T = K_block * Q^T with
// v_mfma_f32_16x16x32_{f16,bf16}: 16 keys per block as the M rows, the patch's 16 queries as
// the N columns, the whole head dimension as one K step.
//
// Lane layout of the 16x16x32 instruction (wave64), checked on hardware:
//   A operand: lane l holds row  m = l % 16, k-elements 8*(l/16) .. 8*(l/16)+7   (16 bytes)
//   B operand: lane l holds col  n = l % 16, k-elements 8*(l/16) .. 8*(l/16)+7   (16 bytes)
//   result   : lane l holds col  n = l % 16, rows 4*(l/16) + r, r = 0..3
// So lane (j = l%16, g = l/16) loads bytes [16g, 16g+16) of key (16*block + j) and of query j,
// and receives the dot products of query j with keys 16*block + 4g + r.
#pragma once

#include "na2d_common.hpp"

namespace na2d {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));

template <typename T> __device__ __forceinline__ f32x4 mfma_16x16x32(u32x4 a, u32x4 b, f32x4 c);
template <> __device__ __forceinline__ f32x4 mfma_16x16x32<f16_t>(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4 mfma_16x16x32<bf16_t>(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// The half-depth instruction (contraction over 16): lane l holds row / column l % 16 and the
// k-elements 4*(l/16) .. 4*(l/16)+3 of the A / B operand (8 bytes); the result layout is the same.
struct u32x2;
typedef short i16x4_t __attribute__((ext_vector_type(4)));
template <typename T> __device__ __forceinline__ f32x4 mfma_16x16x16(uint32_t a0, uint32_t a1, uint32_t b0, uint32_t b1, f32x4 c);
template <> __device__ __forceinline__ f32x4 mfma_16x16x16<f16_t>(uint32_t a0, uint32_t a1, uint32_t b0, uint32_t b1, f32x4 c) {
    const uint64_t a = (uint64_t)a0 | ((uint64_t)a1 << 32), b = (uint64_t)b0 | ((uint64_t)b1 << 32);
    return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a), __builtin_bit_cast(f16x4, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4 mfma_16x16x16<bf16_t>(uint32_t a0, uint32_t a1, uint32_t b0, uint32_t b1, f32x4 c) {
    const uint64_t a = (uint64_t)a0 | ((uint64_t)a1 << 32), b = (uint64_t)b0 | ((uint64_t)b1 << 32);
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(i16x4_t, a), __builtin_bit_cast(i16x4_t, b), c, 0, 0, 0);
}

// The fused kernels keep the bias B(i, j) of a (query, position) pair as fp16, two per register, beside the
// -inf that masks positions outside the window, and add it unscaled to the fp32 logit.  An fp16 table entry is
// kept bit for bit.  A bf16 entry (8 significant bits) converts exactly while it lies inside fp16's range:
// beyond +-65504 it counts as +-65504, and below 2^-14 in magnitude it is rounded to a multiple of 2^-24.
__device__ __forceinline__ f16_t bias_to_f16(f16_t x) { return x; }
__device__ __forceinline__ f16_t bias_to_f16(bf16_t x) {
    const float f = (float)x;
    return (f16_t)(f > 65504.f ? 65504.f : (f < -65504.f ? -65504.f : f));   // a NaN stays a NaN
}

// Geometry of a 4 x 4 query patch.  Patch-halo coordinates are "virtual": position (hy, hx)
// is key (oy + hy, ox + hx) whether or not that lies inside the map, with (oy, ox) =
// halo_origin() of the patch.  The windows of 4 consecutive queries span at most K + 3
// positions per axis, so a PW = K + 3 wide halo always holds them.
template <int K> struct Patch {
    static constexpr int R = K / 2;
    static constexpr int PW = 4 + K - 1;            // side of the patch halo
    static constexpr int NKEY = PW * PW;
    static constexpr int NBLK = (NKEY + 15) / 16;   // 16-key MFMA blocks
    static constexpr int NEL = NBLK * 4;            // result elements per lane
    // halo index -> (row, col): exact multiply-shift division for h < 1024
    static constexpr unsigned kMagic = (1u << 16) / PW + 1;
    __device__ static __forceinline__ int row_of(int h) { return (int)(((unsigned)h * kMagic) >> 16); }
};

// First (virtual, possibly negative) key coordinate of the halo that serves the n consecutive
// queries q0 .. q0+n-1 on an axis of length L.  It is q0 - R wherever that works: then the bias
// cell of (query, key) is the same function of their positions inside patch and halo for every
// patch.  Next to the far border the windows are pulled back to L - K and the halo follows;
// next to the near border (only for K > 7 with n = 4) the windows reach further right than
// q0 + n - 1 + R and the halo is pushed right by the excess.  The halo has n + K - 1 positions.
__host__ __device__ __forceinline__ int halo_origin(int q0, int n, int L, int K) {
    const int last = q0 + n - 1 < L - 1 ? q0 + n - 1 : L - 1;
    const int lo = win_start(last, L, K) - (n - 1);
    int o = q0 - (K >> 1);
    o = o < L - K ? o : L - K;
    return o > lo ? o : lo;
}

// ---- global memory -> LDS without registers, and transposing LDS reads --------------------
//
// gfx950 can load 16 bytes per lane from global memory straight into LDS: lane l of the wave
// writes [lds_base + 16 l, lds_base + 16 l + 16), lds_base being the same for the whole wave
// (inactive lanes write nothing).  The load is asynchronous and completes in vmcnt order.
// It is written as inline assembly, not through the compiler builtin: for the builtin the compiler
// assumes that every later LDS read may alias the data still in flight and puts a wait for all
// outstanding loads in front of the first LDS read that follows, which serialises a pipeline that
// loads stage n + 1 while stage n is read.  The kernels order these loads against their LDS reads
// themselves: wait_global_loads() and a workgroup barrier before a stage is read, a barrier after
// its last read before it is loaded again.  M0 holds the LDS base (one wait state before its use);
// it is taken through readfirstlane so that it sits in a scalar register whatever the caller passes,
// and the statements name M0 as clobbered: the compiler keeps values of its own there (the index of
// relative register moves, for one) and must not assume they survive.
__device__ __forceinline__ void global_to_lds_16(const void *g, int lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(__builtin_amdgcn_readfirstlane(lds_base)) : "memory", "m0");
}
// the same from a wave-uniform base pointer plus a 32-bit byte offset per lane
__device__ __forceinline__ void global_to_lds_16(const char *base, unsigned off, int lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(__builtin_amdgcn_readfirstlane(lds_base)) : "memory", "m0");
}
// four bytes per lane: lane l writes [lds_base + 4 l, lds_base + 4 l + 4)
__device__ __forceinline__ void global_to_lds_4(const char *base, unsigned off, int lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(__builtin_amdgcn_readfirstlane(lds_base)) : "memory", "m0");
}
// waits until every load of this wave, the direct-to-LDS ones included, has landed
__device__ __forceinline__ void wait_global_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// A ROWS x COLS rectangle of head-dim vectors of one plane, copied into LDS in its natural
// layout [row][col][channel] (64 bytes per position, no padding) by direct loads; the rows of
// work items (64 chunks each) are dealt round-robin to NWAVES waves.  Positions outside the
// map are replaced by the nearest one inside it: the kernels give them zero weight, or drop
// their results, so any finite value serves.
template <typename T, int ROWS, int COLS, int NWAVES>
struct HaloDma {
    static_assert(sizeof(T) == 2, "64-byte vectors");
    static constexpr int CPK = Traits<T>::kKeyBytes / 16;
    static constexpr int TOTAL = ROWS * COLS * CPK;
    static constexpr int NITEM = (TOTAL + kWave - 1) / kWave;
    static constexpr int PER_WAVE = (NITEM + NWAVES - 1) / NWAVES;
    static constexpr int kBytes = TOTAL * 16;
    int pos[PER_WAVE];   // row | col << 8 | chunk << 16 of this lane's chunk in item i, -1 past the end

    __device__ __forceinline__ void init(int wave, int lane) {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int q = (wave + i * NWAVES) * kWave + lane;
            const int pq = q / CPK, c = q % CPK;
            const int ry = pq / COLS, rx = pq % COLS;
            pos[i] = q < TOTAL ? (ry | (rx << 8) | (c << 16)) : -1;
        }
    }
    // Split form for loops that copy the same rectangle of many planes: the clamped byte offsets of
    // this lane's chunks inside a plane (-1: nothing), then one load per item from a plane's base.
    // `pitch`: bytes between consecutive positions in memory (more than 64 when the 32 channels copied are a
    // slice of a longer head vector).  `chunk_mask` 1 serves 16-channel heads (pitch 32): the two 16-byte
    // chunks of a position are copied twice, into the lower and the upper half of its 64-byte slot (see
    // kHalfDimChunks).
    __device__ __forceinline__ void offsets(int H, int W, int oy, int ox, int (&off)[PER_WAVE],
                                            int pitch = Traits<T>::kKeyBytes, int chunk_mask = 3) const {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            int y = oy + (pos[i] & 0xff), x = ox + ((pos[i] >> 8) & 0xff);
            y = y < 0 ? 0 : (y < H - 1 ? y : H - 1);
            x = x < 0 ? 0 : (x < W - 1 ? x : W - 1);
            off[i] = pos[i] >= 0 ? (y * W + x) * pitch + ((pos[i] >> 16) & chunk_mask) * 16 : -1;
        }
    }
    __device__ static __forceinline__ void issue_at(const char *plane_base, const int (&off)[PER_WAVE], int lds_base, int wave) {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i)
            if (off[i] >= 0) global_to_lds_16(plane_base, (unsigned)off[i], lds_base + (wave + i * NWAVES) * kWave * 16);
    }
    __device__ __forceinline__ void issue(const char *plane_base, int H, int W, int oy, int ox, int lds_base, int wave) const {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            if (pos[i] >= 0) {
                int y = oy + (pos[i] & 0xff), x = ox + ((pos[i] >> 8) & 0xff);
                y = y < 0 ? 0 : (y < H - 1 ? y : H - 1);
                x = x < 0 ? 0 : (x < W - 1 ? x : W - 1);
                global_to_lds_16(plane_base, (unsigned)((y * W + x) * Traits<T>::kKeyBytes + (pos[i] >> 16) * 16),
                                 lds_base + (wave + i * NWAVES) * kWave * 16);
            }
        }
    }
};

// Transposing 8-byte LDS read (ds_read_b64_tr_b16), checked on hardware: inside each group of 16
// lanes, lane i receives as element j (j = 0..3) the 16-bit element (i % 4) of the 8 bytes
// addressed by lane 4 j + i / 4 of the group.  With lane s of the group pointing at channels
// 4 (s % 4) .. + 3 of position P[s / 4], lane i gets channel i of the four positions P[0..3]:
// an MFMA operand whose contraction index runs over positions, read from the natural layout.
struct u32x2 {
    uint32_t x, y;
};
__device__ __forceinline__ u32x2 lds_read_tr16(int addr) {
    const i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(uintptr_t)(unsigned)addr);
    return __builtin_bit_cast(u32x2, v);
}

}  // namespace na2d
