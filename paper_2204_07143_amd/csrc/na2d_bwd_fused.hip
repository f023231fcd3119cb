// Grad-a fused with the softmax backward on the matrix cores (f16 / bf16, K <= 9):
//   dp[n, a, c] = <dout_n, v_{rho(n; a, c)}>                         (grad-a)
//   ds[n, :]    = attn[n, :] * (dp[n, :] - <attn[n, :], dp[n, :]>)   (softmax backward)
// (arXiv 2204.07143, Eq. 3-4 differentiated; Appendix A lists the gradients).  dp never leaves the
// chip: ds is written once instead of dp being written, read back and overwritten.
//
// Same structure as the small-window logits kernel: eight waves share a 16 x 8 query tile, one 4 x 4
// patch each; a workgroup keeps one tile position and one head and walks a range of the batch; the
// value halo (natural layout) and the tile's eight attention row runs (mirrored at their 16-byte
// phase) are loaded straight into one of two LDS stages while the previous plane is computed.
//   1. dp^T = V_halo * dout^T          one MFMA per 16 halo positions (values read as 16-byte operands);
//   2. attn gathered from the row run  through a per-lane address table (the lane's private zero word
//                                      outside the query's window), in the layout the MFMA left dp in;
//   3. delta = <attn, dp>              28 fmas per lane + two cross-lane steps (a query is spread over 4 lanes);
//   4. ds = attn * (dp - delta)        written back in place of attn in the row run;
//   5. wave w streams row run w of ds to global memory with 16-byte stores while the next plane is
//      computed, then loads the run after next into the same place.
#include "na2d_kernels.hpp"
#include "na2d_mfma.hpp"
#include "na2d_tile.hpp"

namespace na2d {

template <typename T, int K>
struct BwdFusedCfg {
    using P = Patch<K>;
    static constexpr int STRIPS = 2;
    static constexpr int WAVES = 4 * STRIPS;
    static constexpr int TY = 4 * STRIPS;
    static constexpr int HALO_H = TY + K - 1, HALO_W = kTileX + K - 1;
    using Halo = HaloDma<T, HALO_H, HALO_W, WAVES>;
    static constexpr int KK = K * K;
    static constexpr int NPAIR = (P::NBLK + 1) / 2;
    static constexpr int NEL2 = 8 * NPAIR;
    static constexpr int kThreads = kWave * WAVES;
    static constexpr int kHaloBytes = Halo::kBytes;
    static constexpr int kRowBytes = kTileX * KK * (int)sizeof(T);
    static constexpr int kRowRegion = mirror_bytes(kRowBytes);
    static constexpr int kRowChunks = (kRowBytes + 15 + 15) / 16;
    static constexpr int kRowPasses = (kRowChunks + kWave - 1) / kWave;   // load instructions of one wave per row run
    static constexpr int kWBytes = TY * kRowRegion;
    // Large windows keep the gather addresses two per register, as 16-bit offsets without the row run's 16-byte
    // phase, which is added when they are used: a thread's private zero area is then 16 bytes, so that it reads
    // zero (and takes the dropped results) at any phase.
    static constexpr bool PACKED = K > 7;
    static constexpr int kZeroEach = PACKED ? 16 : 4;
    static constexpr int kZeroBytes = kThreads * kZeroEach;   // one private word (or four) per thread
    static constexpr int kStageBytes = kHaloBytes + kWBytes + kZeroBytes;
    // Two stages where two workgroups then still share a compute unit's LDS; one stage (k = 9), computed in, streamed
    // out and reloaded in turn while the other workgroup computes, where that is what makes them fit
    static constexpr bool kOneStage = 2 * kStageBytes > 80 * 1024;
    static constexpr int kLdsBytes = (kOneStage ? 1 : 2) * kStageBytes;
    static_assert(kStageBytes < 65536, "the second stage is reached through the 16-bit offset of the LDS accesses");
};

template <typename T, int K>
__global__ __launch_bounds__(512, 4) void bwd_fused_small_kernel(const T *__restrict__ attn, const T *__restrict__ dout,
                                                                 const T *__restrict__ v, T *__restrict__ ds, int H, int W,
                                                                 int heads, int nb, int tiles_y, int units, int splits, GridDecode gd,
                                                                 int half_dim) {
    using C = BwdFusedCfg<T, K>;
    using P = Patch<K>;
    static_assert(C::kThreads == 512, "launch bounds");
    constexpr int SZ = (int)sizeof(T);
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int strip = wave >> 2, p = patch_of_wave(wave);
    const int j = lane & 15, g = lane >> 4, jy = j >> 2, jx = j & 3;
    const int lds0 = lds_addr(lds);
    const int w0 = lds0 + C::kHaloBytes;          // attention / ds row runs (the value halo comes first)
    const int my_zero = w0 + C::kWBytes + tid * C::kZeroEach;

    const int wg = xcd_contiguous_block(blockIdx.x, gridDim.x);
    if (wg >= units * splits) return;
    const WorkItem work = decode_work(wg, heads, tiles_y, splits, gd);
    const int head = work.head, ty0 = work.ty * C::TY, tx0 = work.tx * kTileX;
    const int b_begin = work.b_begin, b_end = work.b_end;
    if (b_begin >= b_end) return;

    const int hoy = halo_origin(ty0, C::TY, H, K), hox = halo_origin(tx0, kTileX, W, K);   // tile halo origin
    const int sy0 = ty0 + 4 * strip, px0 = tx0 + 4 * p;                                     // this wave's patch
    const bool active = sy0 < H && px0 < W;
    const int oy = halo_origin(sy0 < H ? sy0 : H - 1, 4, H, K), ox = halo_origin(px0 < W ? px0 : W - 1, 4, W, K);
    const int qy = sy0 + jy, qx = px0 + jx;
    const bool q_ok = qy < H && qx < W;

    // loads of one plane: both halos, this wave's row run of the attention weights, this lane's dout chunk
    typename C::Halo halo;
    halo.init(wave, lane);
    int hoff[C::Halo::PER_WAVE];
    // (half_dim: 16-channel heads; see kHalfDimChunks)
    const int pitch = half_dim ? Traits<T>::kKeyBytes / 2 : Traits<T>::kKeyBytes, chunk_mask = half_dim ? kHalfDimChunks : 3;
    halo.offsets(H, W, hoy, hox, hoff, pitch, chunk_mask);
    const size_t plane_y = (size_t)H * W * pitch;   // bytes per plane of dout / v / k / dq
    const size_t plane_w = (size_t)H * W * C::KK * SZ;             // ... of attn / ds
    const int wrow = ty0 + wave;
    const int wrow_bytes = ((W - tx0) < kTileX ? (W - tx0) : kTileX) * C::KK * SZ;
    const size_t wrow_off = ((size_t)(wrow < H ? wrow : H - 1) * W + tx0) * C::KK * SZ;
    const int qlin = (qy < H - 1 ? qy : H - 1) * W + (qx < W - 1 ? qx : W - 1);
    auto issue = [&](int b, int par) {
        const size_t plane = (size_t)b * heads + head;
        C::Halo::issue_at(reinterpret_cast<const char *>(v) + plane * plane_y, hoff, lds0 + par * C::kStageBytes, wave);
        if (wrow < H) {
            const size_t g0 = plane * plane_w + wrow_off;
            const int mis = (int)(g0 & 15);
            const int nchunks = (mis + wrow_bytes + 15) >> 4;
            const char *src = reinterpret_cast<const char *>(attn) + (g0 - mis);
            const int region = w0 + par * C::kStageBytes + wave * C::kRowRegion;
            // only the last row run of the tensor can end inside a chunk that reaches past the tensor
            const bool at_end = b == nb - 1 && head == heads - 1 && wrow == H - 1 && tx0 + kTileX >= W;
            if (!at_end) {   // (wave-uniform) every chunk lies inside the tensor
#pragma unroll
                for (int it = 0; it < C::kRowPasses; ++it) {
                    const int c = lane + it * kWave;
                    if (c < nchunks) global_to_lds_16(src, (unsigned)(c * 16), region + it * kWave * 16);
                }
            } else {   // the chunk that would cross the tensor's end goes element by element
#pragma unroll 1
                for (int it = 0; it < C::kRowPasses; ++it) {
                    const int c = lane + it * kWave;
                    if (c < nchunks) {
                        if ((c + 1) * 16 <= mis + wrow_bytes) {
                            global_to_lds_16(src, (unsigned)(c * 16), region + it * kWave * 16);
                        } else {
                            for (int e = c * 16; e < mis + wrow_bytes; e += SZ)
                                *lds_ptr<T>(region + e) = *reinterpret_cast<const T *>(src + e);
                        }
                    }
                }
            }
        }
    };
    // this lane's 16 bytes of dout of its query (B operand); the next plane's are loaded as soon as the
    // MFMAs of the current plane have consumed the register
    auto load_dout = [&](int b) {
        const u32x4 d = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(dout) + ((size_t)b * heads + head) * plane_y +
                                                         qlin * pitch + (g & chunk_mask) * 16);
        return (half_dim && g >= 2) ? u32x4{0u, 0u, 0u, 0u} : d;
    };
    auto clear_zero = [&](int at) {
        if constexpr (C::PACKED) *lds_ptr<u32x4>(at) = u32x4{0u, 0u, 0u, 0u};
        else *lds_ptr<uint32_t>(at) = 0u;
    };
    clear_zero(my_zero);
    if constexpr (!C::kOneStage) clear_zero(my_zero + C::kStageBytes);
    issue(b_begin, 0);
    u32x4 dreg = load_dout(b_begin);

    // A operand: the values of halo position 16b + j, bytes [16g, 16g+16) (positions past the end of the
    // patch halo re-read its last one; their results are dropped).  Recomputed per plane from an opaque
    // copy of the lane index: seven more registers held across the loop would not fit.
    const int vbase = lds0 + ((oy - hoy) * C::HALO_W + (ox - hox)) * Traits<T>::kKeyBytes;
    // LDS address of this lane's query's weight for halo position 16 (e / 4) + 4g + e % 4: its slot in
    // the query's row run, the lane's private zero word where the position is outside the window.  The
    // addresses hold the 16-byte phase the run has in the first plane of the range.
    const size_t qrow_off = ((size_t)(qy < H ? qy : H - 1) * W + tx0) * C::KK * SZ;
    auto phase_of = [&](int b) { return (int)((((size_t)b * heads + head) * plane_w + qrow_off) & 15); };
    const int phase0 = phase_of(b_begin);
    int cur_phase = phase0;
    const bool phase_varies = (plane_w & 15) != 0;
    // Built per group of four consecutive halo positions (e / 4): the positions of a group that lie inside
    // the query's window are in one halo row (a halo row holds K + 3 positions, the window K of them),
    // normally the row of the group's first position; when that one is already right of the window, the
    // group runs on into the next halo row and only that part can be inside.
    int gaddr[C::PACKED ? P::NEL / 2 : P::NEL];
    static_assert(!C::PACKED || C::kWBytes + C::kZeroBytes <= 65536, "offsets from the first row run fit 16 bits");
    {
        const int wy = win_start(qy < H ? qy : H - 1, H, K) - oy, wx = win_start(qx < W ? qx : W - 1, W, K) - ox;
        const int lane_row = w0 + (4 * strip + jy) * C::kRowRegion + (C::PACKED ? 0 : phase0) + (4 * p + jx) * C::KK * SZ;
#pragma unroll
        for (int G = 0; G < P::NBLK; ++G) {
            const int h0 = 16 * G + 4 * g;
            const int hy0 = P::row_of(h0), hx0 = h0 - hy0 * P::PW;
            const bool wrap = hx0 > wx + K - 1;
            const int a = hy0 + (wrap ? 1 : 0) - wy;
            int c0 = hx0 - (wrap ? P::PW : 0) - wx;   // window column of the group's first position (may be negative)
            const int base = lane_row + (a * K + c0) * SZ;
            c0 = (q_ok && (unsigned)a < (unsigned)K) ? c0 : 64;   // no row of the window: every column test fails
            int ga[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) ga[i] = (unsigned)(c0 + i) < (unsigned)K ? base + i * SZ : my_zero;
            if constexpr (C::PACKED) {
                gaddr[2 * G] = (ga[0] - w0) | ((ga[1] - w0) << 16);
                gaddr[2 * G + 1] = (ga[2] - w0) | ((ga[3] - w0) << 16);
                __builtin_amdgcn_sched_barrier(0);   // one group's temporaries at a time
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) gaddr[4 * G + i] = ga[i];
            }
        }
    }
    // LDS address of the weight of result e in stage offset poff
    auto weight_addr = [&](int e, int poff) -> int {
        if constexpr (C::PACKED) {
            const uint32_t pk = (uint32_t)gaddr[e >> 1];
            return w0 + cur_phase + poff + (int)((e & 1) ? pk >> 16 : pk & 0xffffu);
        } else {
            return gaddr[e] + poff;
        }
    };
    auto compute = [&](auto par_c, int b) {
        constexpr int PAR = decltype(par_c)::value;
        constexpr int POFF = PAR * C::kStageBytes;
        if (!active) return;
        if constexpr (C::PACKED) {
            // the packed table stays packed: without this its unpacking is hoisted out of the loop over the planes
            // and takes a register per address
#pragma unroll
            for (int e = 0; e < P::NEL / 2; ++e) asm volatile("" : "+v"(gaddr[e]));
        }
        // 1. dp
        float dp[P::NEL];
        int lv = lane;
        asm volatile("" : "+v"(lv));
#pragma unroll
        for (int bk = 0; bk < P::NBLK; ++bk) {
            int h = 16 * bk + (lv & 15);
            h = h < P::NKEY ? h : P::NKEY - 1;
            const int hy = P::row_of(h), hx = h - hy * P::PW;
            const u32x4 a = *lds_ptr<u32x4>(vbase + (hy * C::HALO_W + hx) * Traits<T>::kKeyBytes + (lv >> 4) * 16 + POFF);
            const f32x4 acc = mfma_16x16x32<T>(a, dreg, f32x4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
            for (int r = 0; r < 4; ++r) dp[4 * bk + r] = acc[r];
        }
        if (b + 1 < b_end) dreg = load_dout(b + 1);
        // 2-3. attention weights (kept two per register, in the storage type) and delta
        uint32_t pw2[P::NEL / 2];
        auto half_of = [](uint32_t two, int which) {
            return to_f32(__builtin_bit_cast(T, (uint16_t)(which ? two >> 16 : two & 0xffffu)));
        };
        float delta = 0.f;
#pragma unroll
        for (int e = 0; e < P::NEL; e += 2) {
            pw2[e >> 1] = (uint32_t)*lds_ptr<uint16_t>(weight_addr(e, POFF)) | ((uint32_t)*lds_ptr<uint16_t>(weight_addr(e + 1, POFF)) << 16);
            delta = __builtin_fmaf(half_of(pw2[e >> 1], 0), dp[e], delta);
            delta = __builtin_fmaf(half_of(pw2[e >> 1], 1), dp[e + 1], delta);
            if constexpr (C::PACKED) {
                if ((e & 15) == 14) __builtin_amdgcn_sched_barrier(0);   // sixteen gathers in flight at a time
            }
        }
        delta += __shfl_xor(delta, 16);
        delta += __shfl_xor(delta, 32);
        // 4. ds, back into the row run (packed table: the addresses are unpacked again rather than kept since step 2)
        if constexpr (C::PACKED) {
#pragma unroll
            for (int e = 0; e < P::NEL / 2; ++e) asm volatile("" : "+v"(gaddr[e]));
        }
#pragma unroll
        for (int e = 0; e < P::NEL; e += 2) {
            typedef float f32x2_t __attribute__((ext_vector_type(2)));
            typedef T tx2_t __attribute__((ext_vector_type(2)));
            const tx2_t d2 = __builtin_convertvector(
                (f32x2_t){half_of(pw2[e >> 1], 0) * (dp[e] - delta), half_of(pw2[e >> 1], 1) * (dp[e + 1] - delta)}, tx2_t);
            *lds_ptr<T>(weight_addr(e, POFF)) = d2[0];
            *lds_ptr<T>(weight_addr(e + 1, POFF)) = d2[1];
        }
        clear_zero(my_zero + POFF);   // whatever the out-of-window results were, the area reads zero again
    };
    auto flush = [&](int b, int par) {
        if (wrow < H)
            stage_out<T, C::kRowBytes, kWave>(reinterpret_cast<char *>(ds), ((size_t)b * heads + head) * plane_w + wrow_off,
                                              wrow_bytes, lds + (w0 - lds0) + par * C::kStageBytes + wave * C::kRowRegion, lane);
    };

    int b = b_begin;
    auto step = [&](auto par_c) {
        constexpr int PAR = decltype(par_c)::value;
        wait_global_loads();   // this plane's halo, row runs and dout chunk have landed
        workgroup_sync();       // ... for every wave; the previous plane's ds row runs are complete
        if constexpr (!C::kOneStage) {
            if (b > b_begin) {
                flush(b - 1, PAR ^ 1);
                // this wave's run is flushed (its LDS reads have returned) before its next load may land there
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            if (b + 1 < b_end) issue(b + 1, PAR ^ 1);
        }
        if (phase_varies) {   // the table follows the phase of this plane's row run (in-window entries only)
            const int ph = phase_of(b), d = ph - cur_phase;
            cur_phase = ph;
            if constexpr (!C::PACKED) {
#pragma unroll
                for (int e = 0; e < P::NEL; ++e) gaddr[e] += gaddr[e] != my_zero ? d : 0;
            }
        }
        compute(par_c, b);
        if constexpr (C::kOneStage) {
            workgroup_sync();   // the ds row runs are complete, the halo is no longer read
            flush(b, 0);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (as above)
            if (b + 1 < b_end) issue(b + 1, 0);
        }
        ++b;
    };
    while (b < b_end) {
        step(IntC<0>{});
        if constexpr (!C::kOneStage) {
            if (b < b_end) step(IntC<1>{});
        }
    }
    if constexpr (!C::kOneStage) {
        workgroup_sync();
        flush(b_end - 1, (b_end - b_begin - 1) & 1);
    }
}

template <typename T, int K>
static hipError_t launch_bwd_fused_t(const Problem &p, const void *attn, const void *dout, const void *v, void *ds,
                                     hipStream_t s) {
    using C = BwdFusedCfg<T, K>;
    static_assert(C::kLdsBytes <= 80 * 1024, "two workgroups share the LDS of a compute unit");
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    const UnitSplit us = unit_split(tiles_x, tiles_y, p.heads, p.B);
    auto kern = bwd_fused_small_kernel<T, K>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(us.units * us.splits)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(attn), static_cast<const T *>(dout), static_cast<const T *>(v),
                       static_cast<T *>(ds), p.H, p.W, p.heads, p.B, tiles_y, us.units, us.splits, us.gd,
                       p.D == kHalfDim ? 1 : 0);
    return hipGetLastError();
}

bool bwd_fused_supported(const Problem &p) { return (p.D == kHeadDim || p.D == kHalfDim) && p.dtype != NA2D_F32 && p.K <= 9; }

hipError_t launch_bwd_fused(const Problem &p, const void *attn, const void *dout, const void *v, void *ds, hipStream_t s) {
#define NA2D_BWDF_K(TT)                                                                                   \
    switch (p.K) {                                                                                        \
        case 3: return launch_bwd_fused_t<TT, 3>(p, attn, dout, v, ds, s);                               \
        case 5: return launch_bwd_fused_t<TT, 5>(p, attn, dout, v, ds, s);                               \
        case 7: return launch_bwd_fused_t<TT, 7>(p, attn, dout, v, ds, s);                               \
        case 9: return launch_bwd_fused_t<TT, 9>(p, attn, dout, v, ds, s);                               \
        default: return hipErrorInvalidValue;                                                             \
    }
    if (p.dtype == NA2D_F16) { NA2D_BWDF_K(f16_t) }
    if (p.dtype == NA2D_BF16) { NA2D_BWDF_K(bf16_t) }
#undef NA2D_BWDF_K
    return hipErrorInvalidValue;
}

}  // namespace na2d
