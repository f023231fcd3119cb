// Fused neighbourhood attention forward on the matrix cores (f16 / bf16):
//   out_n = softmax_{a,c}( scale * <q_n, k_{rho(n;a,c)}> + B(n, rho(n;a,c)) ) . v_{rho(n;a,c)}
// (arXiv 2204.07143, Eq. 2-4 in one kernel; the k*k logits and weights never leave the chip).
//
// For one 4 x 4 patch of queries and the (K+3)^2 halo positions its windows can touch:
//   1. S^T = K_halo * Q^T    one 16x16x32 MFMA per block of 16 halo positions (keys in their natural
//                            layout in LDS, queries straight from global memory);
//   2. logits               one fma per result against a per-lane table that holds the bias of
//                            (query, position), as stored, and -inf where the position is outside
//                            the query's window;
//   3. softmax              row max and row sum in registers plus two cross-lane steps each
//                            (a query's positions are spread over 4 lanes), exp2 in fp32;
//   4. O^T = V_halo^T * P    the un-normalised weights, converted to the storage type, are already
//                            in the B-operand layout of the next MFMA; values through the
//                            transposing LDS read;
//   5. out = O / sum, lse    each lane owns 8 channels of its own query: no cross-lane traffic.
//
// Eight waves share a 16 x 8 query tile, one 4 x 4 patch each (four waves per SIMD).  A workgroup
// keeps one tile position and one head and walks a range of the batch, so the window mask, the bias
// table and every address are built once.  The key and the value halo of a tile reach LDS by direct
// loads in their natural layout, into one of two buffer pairs: the next tile's halos arrive while
// this tile is computed (one workgroup barrier per tile).  Keys are read as 16-byte A operands;
// values are read with the transposing LDS read, which hands each lane one channel of four halo
// positions, so the PV product contracts over positions without a transposed copy.  The halo
// positions are numbered h = hy * (K+3) + hx; MFMA pair m of the PV product contracts over the
// blocks 2m and 2m+1 of the logits, in the order the logits' MFMA left them in the lanes.
#include "na2d_kernels.hpp"
#include "na2d_mfma.hpp"
#include "na2d_tile.hpp"

namespace na2d {

// two floats -> one register of two storage-type values (round to nearest even; one packed
// conversion instruction on gfx950)
template <typename T> __device__ __forceinline__ uint32_t pack2(float a, float b) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef T tx2_t __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){a, b}, tx2_t));
}

// NS: 32-channel slices of the head vector (head dim 32 NS).  Every slice of the key and of the value halo is
// its own 64-byte-per-position image; the logits accumulate one MFMA per slice, the PV product runs per slice.
template <typename T, int K, int NS = 1>
struct FusedSmallCfg {
    using P = Patch<K>;
    static constexpr int STRIPS = 2;
    static constexpr int WAVES = 4 * STRIPS;
    static constexpr int TY = 4 * STRIPS;
    static constexpr int HALO_H = TY + K - 1, HALO_W = kTileX + K - 1;
    using Halo = HaloDma<T, HALO_H, HALO_W, WAVES>;
    static constexpr int NB = 2 * K - 1;
    static constexpr int NPAIR = (P::NBLK + 1) / 2;   // PV MFMAs per 16 channels
    static constexpr int NBLK2 = 2 * NPAIR;           // logits blocks, padded to whole pairs
    static constexpr int kThreads = kWave * WAVES;
    static constexpr int kHaloBytes = Halo::kBytes;             // one slice of one operand
    static constexpr int kStageBytes = 2 * NS * kHaloBytes;     // the key slices, then the value slices
    // Two buffer pairs (the next tile's halos arrive while this one is computed); one pair, loaded between tiles, where
    // two exceed the LDS of a compute unit (two slices, k >= 9)
    static constexpr bool kOneStage = 2 * kStageBytes > 160 * 1024;
    static constexpr int kLdsBytes = (kOneStage ? 1 : 2) * kStageBytes;
    static constexpr int kKeyBytesG = NS * Traits<T>::kKeyBytes;   // bytes per position in memory
    static constexpr int kWavesPerSimd = kLdsBytes <= 80 * 1024 ? 4 : 2;   // two workgroups, or one, per compute unit
};

template <typename T, int K, int NS>
__global__ __launch_bounds__(512, (FusedSmallCfg<T, K, NS>::kWavesPerSimd)) void fused_mfma_small_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                                  const T *__restrict__ v, const T *__restrict__ rpb,
                                                                  float scale, T *__restrict__ out, float *__restrict__ lse,
                                                                  int H, int W, int heads, int nb, int tiles_y, int units,
                                                                  int splits, GridDecode gd, int half_dim) {
    using C = FusedSmallCfg<T, K, NS>;
    using P = Patch<K>;
    static_assert(C::kThreads == 512, "launch bounds");
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int strip = wave >> 2, p = patch_of_wave(wave);
    const int j = lane & 15, g = lane >> 4, jy = j >> 2, jx = j & 3;
    const int lds0 = lds_addr(lds);

    const int wg = xcd_contiguous_block(blockIdx.x, gridDim.x);
    if (wg >= units * splits) return;
    // neighbouring workgroups take neighbouring tile positions of the same planes (the position index
    // runs fastest), so the positions whose halos overlap run at the same time on the same XCD and
    // the overlap is read from HBM once
    const WorkItem work = decode_work(wg, heads, tiles_y, splits, gd);
    const int head = work.head, ty0 = work.ty * C::TY, tx0 = work.tx * kTileX;
    const int b_begin = work.b_begin, b_end = work.b_end;
    if (b_begin >= b_end) return;

    const int hoy = halo_origin(ty0, C::TY, H, K), hox = halo_origin(tx0, kTileX, W, K);   // tile halo origin
    const int sy0 = ty0 + 4 * strip, px0 = tx0 + 4 * p;                                     // this wave's patch
    const bool active = sy0 < H && px0 < W;
    const int oy = halo_origin(sy0 < H ? sy0 : H - 1, 4, H, K), ox = halo_origin(px0 < W ? px0 : W - 1, 4, W, K);
    const int dy = oy - (sy0 - P::R), dx = ox - (px0 - P::R);   // 0 away from the borders
    const int qy = sy0 + jy, qx = px0 + jx;
    const bool q_ok = qy < H && qx < W;

    // the first tile's loads fly while the tables below are built
    typename C::Halo halo;
    halo.init(wave, lane);
    int hoff[C::Halo::PER_WAVE];
    // (half_dim: 16-channel heads, NS = 1; see kHalfDimChunks)
    const int pitch = half_dim ? C::kKeyBytesG / 2 : C::kKeyBytesG, chunk_mask = half_dim ? kHalfDimChunks : 3;
    halo.offsets(H, W, hoy, hox, hoff, pitch, chunk_mask);
    const int qlin = (qy < H - 1 ? qy : H - 1) * W + (qx < W - 1 ? qx : W - 1);   // this lane's query inside a plane
    const size_t plane_bytes = (size_t)H * W * pitch;
    u32x4 qnext[NS];
    auto issue = [&](int b, int par) {
        const size_t off = ((size_t)b * heads + head) * plane_bytes;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
            const size_t so = off + sl * Traits<T>::kKeyBytes;
            C::Halo::issue_at(reinterpret_cast<const char *>(k) + so, hoff, lds0 + par * C::kStageBytes + sl * C::kHaloBytes, wave);
            C::Halo::issue_at(reinterpret_cast<const char *>(v) + so, hoff,
                              lds0 + par * C::kStageBytes + (NS + sl) * C::kHaloBytes, wave);
            qnext[sl] = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(q) + so + (size_t)qlin * pitch + (g & chunk_mask) * 16);
        }
    };
    issue(b_begin, 0);

    // Operand addresses inside the first buffer pair.  Keys: halo position 16b + j, bytes [16g, 16g+16).
    // Values (transposing read): inside its group of 16 lanes, lane j points at four channels of halo
    // position 16b + 4g + j / 4 and receives the j-th channel of positions 16b + 4g .. + 3.  The channels
    // are dealt so that MFMA row m of half hf is channel 8 (m / 4) + 4 hf + m % 4: a lane then ends
    // up with the eight consecutive channels 8g .. 8g + 7 of its query, one 16-byte store.
    int koff[P::NBLK], vaddr[C::NBLK2];
#pragma unroll
    for (int b = 0; b < C::NBLK2; ++b) {
        int h = 16 * b + j;
        h = h < P::NKEY ? h : P::NKEY - 1;   // past the end: any real position (its weight is zero)
        int hy = P::row_of(h), hx = h - hy * P::PW;
        if (b < P::NBLK) koff[b] = lds0 + ((oy - hoy + hy) * C::HALO_W + (ox - hox) + hx) * Traits<T>::kKeyBytes + g * 16;
        h = 16 * b + 4 * g + (j >> 2);
        h = h < P::NKEY ? h : P::NKEY - 1;
        hy = P::row_of(h);
        hx = h - hy * P::PW;
        vaddr[b] = lds0 + NS * C::kHaloBytes + ((oy - hoy + hy) * C::HALO_W + (ox - hox) + hx) * Traits<T>::kKeyBytes + (j & 3) * 16;
    }
    // bias of (this lane's query, halo position), -inf outside the query's window; packed fp16 pairs
    // (half the registers; the fma below reads them as mixed-precision operands; see bias_to_f16)
    f16x2 biasm[P::NEL / 2];
    {
        const int wy = win_start(qy < H ? qy : H - 1, H, K) - oy, wx = win_start(qx < W ? qx : W - 1, W, K) - ox;
        // Built per group of four consecutive halo positions (e / 4): the positions of a group that lie
        // inside the query's window are in one halo row (a halo row holds K + 3 positions, the window K of
        // them), normally the row of the group's first position; when that one is already right of the
        // window, the group runs on into the next halo row and only that part can be inside.
        int bidx[P::NEL];   // cell of the bias table, -1 outside the window
#pragma unroll
        for (int G = 0; G < P::NBLK; ++G) {
            const int h0 = 16 * G + 4 * g;
            const int hy0 = P::row_of(h0), hx0 = h0 - hy0 * P::PW;
            const bool wrap = hx0 > wx + K - 1;
            const int hy = hy0 + (wrap ? 1 : 0), hxf = hx0 - (wrap ? P::PW : 0);   // halo row, column of the first position
            const int a = hy - wy;
            const int c0 = (q_ok && (unsigned)a < (unsigned)K) ? hxf - wx : 64;   // no row of the window: every column test fails
            const int cell0 = (hy - jy + P::R + dy) * C::NB + (hxf - jx + P::R + dx);   // inside the table wherever the window test holds
#pragma unroll
            for (int i = 0; i < 4; ++i) bidx[4 * G + i] = (unsigned)(c0 + i) < (unsigned)K ? cell0 + i : -1;
        }
        // all loads of the bias table in flight at once (one uniform branch on the table's presence)
        f16_t bias[P::NEL];
#pragma unroll
        for (int e = 0; e < P::NEL; ++e) bias[e] = (f16_t)0.f;
        if (rpb != nullptr) {
            const T *tbl = rpb + (size_t)head * C::NB * C::NB;
#pragma unroll
            for (int e = 0; e < P::NEL; ++e) bias[e] = bias_to_f16(tbl[bidx[e] < 0 ? 0 : bidx[e]]);
        }
#pragma unroll
        for (int e = 0; e < P::NEL; ++e) biasm[e >> 1][e & 1] = bidx[e] >= 0 ? bias[e] : (f16_t)-INFINITY;
    }

    auto compute = [&](auto par_c, const u32x4 (&qreg)[NS], int b) {
        constexpr int PAR = decltype(par_c)::value;
        if (!active) return;
        // 1-2. logits: fp32 dot product times scale, plus the bias as stored
        float s[4 * C::NBLK2];
#pragma unroll
        for (int bk = 0; bk < P::NBLK; ++bk) {
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sl = 0; sl < NS; ++sl) {
                const u32x4 a = *lds_ptr<u32x4>(koff[bk] + PAR * C::kStageBytes + sl * C::kHaloBytes);
                acc = mfma_16x16x32<T>(a, qreg[sl], acc);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
                s[4 * bk + r] = __builtin_fmaf(scale, acc[r], (float)biasm[(4 * bk + r) >> 1][(4 * bk + r) & 1]);
        }
        // 3. softmax over the query's window (spread over the 4 lanes j, j+16, j+32, j+48)
        float m = s[0];
#pragma unroll
        for (int e = 1; e < P::NEL; ++e) m = fmaxf(m, s[e]);
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        m = q_ok ? m : 0.f;   // lanes without a query: keep the arithmetic finite
        // exp(s - m) as exp2(log2(e) s - m2): the subtraction of the maximum and the change of base are one fma
        const float m2 = m * kLog2e;
        float l = 0.f;
#pragma unroll
        for (int e = 0; e < P::NEL; ++e) {
            s[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], kLog2e, -m2));
            l += s[e];
        }
#pragma unroll
        for (int e = P::NEL; e < 4 * C::NBLK2; ++e) s[e] = 0.f;   // padding block of the last pair
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        // 4. O^T = V^T * P
        f32x4 o[NS][2];
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) o[sl][0] = o[sl][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int pb = 0; pb < C::NPAIR; ++pb) {
            const u32x4 bop = u32x4{pack2<T>(s[8 * pb], s[8 * pb + 1]), pack2<T>(s[8 * pb + 2], s[8 * pb + 3]),
                                    pack2<T>(s[8 * pb + 4], s[8 * pb + 5]), pack2<T>(s[8 * pb + 6], s[8 * pb + 7])};
            // bf16 keeps 8 significant bits: a second operand carries the rounding remainder of the
            // weights so that the product sees them to 16 bits
            u32x4 bop_lo = u32x4{0u, 0u, 0u, 0u};
            if constexpr (sizeof(T) == 2 && Traits<T>::kDtype == NA2D_BF16) {
                float rem[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) rem[u] = s[8 * pb + u] - to_f32(from_f32<T>(s[8 * pb + u]));
                bop_lo = u32x4{pack2<T>(rem[0], rem[1]), pack2<T>(rem[2], rem[3]), pack2<T>(rem[4], rem[5]),
                               pack2<T>(rem[6], rem[7])};
            }
#pragma unroll
            for (int sl = 0; sl < NS; ++sl) {
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    const u32x2 lo = lds_read_tr16(vaddr[2 * pb] + PAR * C::kStageBytes + sl * C::kHaloBytes + hf * 8);
                    const u32x2 hi = lds_read_tr16(vaddr[2 * pb + 1] + PAR * C::kStageBytes + sl * C::kHaloBytes + hf * 8);
                    const u32x4 aop = u32x4{lo.x, lo.y, hi.x, hi.y};
                    o[sl][hf] = mfma_16x16x32<T>(aop, bop, o[sl][hf]);
                    if constexpr (sizeof(T) == 2 && Traits<T>::kDtype == NA2D_BF16)
                        o[sl][hf] = mfma_16x16x32<T>(aop, bop_lo, o[sl][hf]);
                }
            }
        }
        // 5. normalise and store this lane's 8 channels (8g .. 8g + 7) of its own query
        if (q_ok && (!half_dim || g < 2)) {
            const float inv = __builtin_amdgcn_rcpf(l);   // 1 ulp; the result is rounded to 11 or 8 bits
            const size_t plane = (size_t)b * heads + head;
            char *dst = reinterpret_cast<char *>(out) + plane * plane_bytes + (size_t)qlin * pitch + g * 16;
#pragma unroll
            for (int sl = 0; sl < NS; ++sl)   // channels 32 sl + 8g .. + 7
                store16_stream(dst + sl * Traits<T>::kKeyBytes,
                               u32x4{pack2<T>(o[sl][0][0] * inv, o[sl][0][1] * inv), pack2<T>(o[sl][0][2] * inv, o[sl][0][3] * inv),
                                     pack2<T>(o[sl][1][0] * inv, o[sl][1][1] * inv), pack2<T>(o[sl][1][2] * inv, o[sl][1][3] * inv)});
            if (lse != nullptr && g == 0) lse[plane * H * W + qlin] = (m2 + __builtin_amdgcn_logf(l)) * kLn2;
        }
    };

    int b = b_begin;
    auto step = [&](auto par_c) {
        constexpr int PAR = decltype(par_c)::value;
        wait_global_loads();   // this tile's halos and query chunk have landed
        workgroup_sync();       // ... for every wave, and nobody still reads the other buffer pair
        u32x4 qreg[NS];
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) qreg[sl] = (half_dim && g >= 2) ? u32x4{0u, 0u, 0u, 0u} : qnext[sl];
        if constexpr (C::kOneStage) {
            compute(par_c, qreg, b);
            if (b + 1 < b_end) {
                workgroup_sync();   // nobody still reads the halos
                issue(b + 1, 0);
            }
        } else {
            if (b + 1 < b_end) issue(b + 1, PAR ^ 1);
            compute(par_c, qreg, b);
        }
        ++b;
    };
    while (b < b_end) {
        step(IntC<0>{});
        if constexpr (!C::kOneStage) {
            if (b < b_end) step(IntC<1>{});
        }
    }
}

template <typename T, int K, int NS>
static hipError_t launch_fused_mfma_small_ns(const Problem &p, const void *q, const void *k, const void *v, const void *rpb,
                                             float scale, void *out, float *lse, hipStream_t s) {
    using C = FusedSmallCfg<T, K, NS>;
    static_assert(NS > 1 || K > 7 || C::kLdsBytes <= 80 * 1024, "two workgroups share the LDS of a compute unit");
    static_assert(C::kLdsBytes <= 160 * 1024, "LDS of a compute unit");
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    const UnitSplit us = unit_split(tiles_x, tiles_y, p.heads, p.B);
    auto kern = fused_mfma_small_kernel<T, K, NS>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(us.units * us.splits)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(q), static_cast<const T *>(k), static_cast<const T *>(v),
                       static_cast<const T *>(rpb), scale, static_cast<T *>(out), lse, p.H, p.W, p.heads, p.B, tiles_y,
                       us.units, us.splits, us.gd, p.D == kHalfDim ? 1 : 0);
    return hipGetLastError();
}

template <typename T, int K>
static hipError_t launch_fused_mfma_small_t(const Problem &p, const void *q, const void *k, const void *v, const void *rpb,
                                            float scale, void *out, float *lse, hipStream_t s) {
    if (p.D == 2 * kHeadDim) return launch_fused_mfma_small_ns<T, K, 2>(p, q, k, v, rpb, scale, out, lse, s);
    if constexpr (K <= 7) {
        if (p.D == 4 * kHeadDim) return launch_fused_mfma_small_ns<T, K, 4>(p, q, k, v, rpb, scale, out, lse, s);
    }
    return launch_fused_mfma_small_ns<T, K, 1>(p, q, k, v, rpb, scale, out, lse, s);
}

bool fused_mfma_supported(const Problem &p) {
    if (p.dtype == NA2D_F32 || p.K > kMaxTunedK) return false;
    // one, two or (while the key and value halos of four slices fit the LDS: k <= 7) four 32-channel slices
    return p.D == kHeadDim || p.D == kHalfDim || p.D == 2 * kHeadDim || (p.D == 4 * kHeadDim && p.K <= 7);
}

hipError_t launch_fused_mfma(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                             void *out, float *lse, hipStream_t s) {
    if (p.dtype == NA2D_F16) {
        using T = f16_t;
        NA2D_DISPATCH_K(p.K, return (launch_fused_mfma_small_t<T, K>(p, q, k, v, rpb, scale, out, lse, s)));
    } else if (p.dtype == NA2D_BF16) {
        using T = bf16_t;
        NA2D_DISPATCH_K(p.K, return (launch_fused_mfma_small_t<T, K>(p, q, k, v, rpb, scale, out, lse, s)));
    }
    return hipErrorInvalidValue;
}

}  // namespace na2d
