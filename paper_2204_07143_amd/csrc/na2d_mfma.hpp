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

}  // namespace na2d
