// Neighbourhood weighted sum on the matrix cores (f16 / bf16):
//   out[n, :] = scale * sum_{a, c} w[n, a, c] * y_{rho(n; a, c)}
// (arXiv 2204.07143, Eq. 3-4; with w = ds, y = k it is grad-q, Appendix A).
//
// A 4 x 4 patch of queries against its halo is a dense contraction over the halo positions:
//   out^T[d, q] = sum_pos Y^T[d, pos] * P[pos, q].
//
// Eight waves share a 16 x 8 query tile, one 4 x 4 patch each.  A workgroup keeps one tile position
// and one head and walks a range of the batch: the per-lane gather addresses of the weights and
// the operand addresses of the values are built once.  Per tile the value halo (natural layout)
// and the tile's eight weight row runs (mirrored at their 16-byte phase) reach one of two LDS
// stages by direct loads while the previous tile is computed (large windows, k >= 9, keep one stage,
// loaded between tiles, so that two workgroups still share a compute unit's LDS).  Halo positions are numbered
// h = hy * (K+3) + hx; MFMA pair m contracts over the positions 32m .. 32m+31 in the lane order
//   lane group g, element e:  position 32m + 16 (e / 4) + 4g + e % 4.
//   A operand: channel j of those positions, two transposing LDS reads from the value halo;
//   B operand: the weights of query j at those positions, 2-byte gathers from its row run (zero
//              outside its window).
#include "na2d_kernels.hpp"
#include "na2d_mfma.hpp"
#include "na2d_tile.hpp"

namespace na2d {

template <typename T, int K>
struct AvSmallCfg {
    using P = Patch<K>;
    static constexpr int STRIPS = 2;
    static constexpr int WAVES = 4 * STRIPS;
    static constexpr int TY = 4 * STRIPS;
    static constexpr int HALO_H = TY + K - 1, HALO_W = kTileX + K - 1;
    using Halo = HaloDma<T, HALO_H, HALO_W, WAVES>;
    static constexpr int KK = K * K;
    static constexpr int NPAIR = (P::NBLK + 1) / 2;
    static constexpr int NEL2 = 8 * NPAIR;            // gathered weights per lane
    static constexpr int kThreads = kWave * WAVES;
    static constexpr int kHaloBytes = Halo::kBytes;
    static constexpr int kRowBytes = kTileX * KK * (int)sizeof(T);
    static constexpr int kRowRegion = mirror_bytes(kRowBytes);
    static constexpr int kRowChunks = (kRowBytes + 15 + 15) / 16;   // 16-byte chunks a run can touch
    static constexpr int kRowPasses = (kRowChunks + kWave - 1) / kWave;   // load instructions of one wave per row run
    static constexpr int kWBytes = TY * kRowRegion;
    static constexpr int kStageBytes = kHaloBytes + kWBytes + 16;   // + the zero word
    // Two stages (the next tile's loads arrive while this one is computed) where two workgroups then still share a
    // compute unit's LDS or one stage would not make them fit either; one stage, reloaded between tiles while the
    // workgroup that shares the compute unit computes, where that is what makes them fit (k = 9)
    static constexpr bool kOneStage = 2 * kStageBytes > 80 * 1024 && kStageBytes <= 80 * 1024;
    static constexpr int kLdsStages = (kOneStage ? 1 : 2) * kStageBytes;
    // per-wave bias-gradient tables (the grad-b variant exists for k <= 9 only)
    static constexpr int kRpbBytes = K <= 9 ? WAVES * (2 * K - 1) * (2 * K - 1) * 4 : 0;
    static constexpr int kLdsBytes = kLdsStages + kRpbBytes;
    static constexpr int kWavesPerSimd = kLdsBytes <= 80 * 1024 ? 4 : 2;   // two workgroups, or one, per compute unit
    static_assert(K > 7 || kStageBytes < 65536, "the second stage is reached through the 16-bit offset of the LDS reads");
    static_assert(kWBytes + 16 <= 65536, "offsets inside a stage's weight rows fit 16 bits");
};

// RPB: the kernel also sums the weights it gathers, per lane and halo position, over its planes; at
// the end the workgroup adds them up per cell of the (2K-1)^2 bias table in a fixed order and writes
// one partial bias gradient (with w = ds this is grad-b, arXiv 2204.07143 Appendix A; Eq. 2's B).
template <typename T, int K, bool RPB>
__global__ __launch_bounds__(512, (AvSmallCfg<T, K>::kWavesPerSimd)) void av_mfma_small_kernel(const T *__restrict__ w, const T *__restrict__ y, float scale,
                                                               T *__restrict__ out, float *__restrict__ rpb_partial, int H,
                                                               int W, int heads, int nb, int tiles_y, int units, int splits, GridDecode gd,
                                                               int pitch) {
    // `pitch`: bytes between consecutive positions of y and out.  The kernel works on 32 channels; a longer
    // head vector is served one 32-channel slice per launch (y and out then point at the slice).
    using C = AvSmallCfg<T, K>;
    using P = Patch<K>;
    static_assert(C::kThreads == 512, "launch bounds");
    constexpr int SZ = (int)sizeof(T);
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int strip = wave >> 2, p = patch_of_wave(wave);
    const int j = lane & 15, g = lane >> 4, jy = j >> 2, jx = j & 3;
    const int lds0 = lds_addr(lds);
    const int w0 = lds0 + C::kHaloBytes, zero_addr = w0 + C::kWBytes;

    const int wg = xcd_contiguous_block(blockIdx.x, gridDim.x);
    if (wg >= units * splits) return;
    // neighbouring workgroups take neighbouring tile positions of the same planes (the position index
    // runs fastest), so the positions whose halos overlap run at the same time on the same XCD and
    // the overlap is read from HBM once
    const WorkItem work = decode_work(wg, heads, tiles_y, splits, gd);
    const int head = work.head, ty0 = work.ty * C::TY, tx0 = work.tx * kTileX;
    const int b_begin = work.b_begin, b_end = work.b_end;
    if (b_begin >= b_end) return;

    // the zero words (one per stage) are never written by the loads
    if (tid < (C::kOneStage ? 4 : 8)) *lds_ptr<uint32_t>(zero_addr + (tid >> 2) * C::kStageBytes + (tid & 3) * 4) = 0u;

    const int hoy = halo_origin(ty0, C::TY, H, K), hox = halo_origin(tx0, kTileX, W, K);   // tile halo origin
    const int sy0 = ty0 + 4 * strip, px0 = tx0 + 4 * p;                                     // this wave's patch
    const bool active = sy0 < H && px0 < W;
    const int oy = halo_origin(sy0 < H ? sy0 : H - 1, 4, H, K), ox = halo_origin(px0 < W ? px0 : W - 1, 4, W, K);
    const int qy = sy0 + jy, qx = px0 + jx;
    const bool q_ok = qy < H && qx < W;

    // loads: value halo chunks of this lane; weight row run `wave` of the tile (two chunks per lane)
    typename C::Halo halo;
    halo.init(wave, lane);
    int hoff[C::Halo::PER_WAVE];
    const bool half_dim = pitch < Traits<T>::kKeyBytes;   // 16-channel heads: see kHalfDimChunks
    halo.offsets(H, W, hoy, hox, hoff, pitch, half_dim ? kHalfDimChunks : 3);
    const size_t plane_y = (size_t)H * W * pitch;                  // bytes per plane of y / out
    const size_t plane_w = (size_t)H * W * C::KK * SZ;             // ... of the weights
    const size_t w_bytes = plane_w * heads * nb;
    const int wrow = ty0 + wave;                                    // the row this wave loads
    const int wrow_bytes = ((W - tx0) < kTileX ? (W - tx0) : kTileX) * C::KK * SZ;
    const size_t wrow_off = ((size_t)(wrow < H ? wrow : H - 1) * W + tx0) * C::KK * SZ;
    auto issue = [&](int b, int par) {
        const size_t plane = (size_t)b * heads + head;
        C::Halo::issue_at(reinterpret_cast<const char *>(y) + plane * plane_y, hoff, lds0 + par * C::kStageBytes, wave);
        if (wrow < H) {
            const size_t g0 = plane * plane_w + wrow_off;
            const int mis = (int)(g0 & 15);
            const int nchunks = (mis + wrow_bytes + 15) >> 4;
            const char *src = reinterpret_cast<const char *>(w) + (g0 - mis);   // the same for the whole wave
            const size_t left = w_bytes - (g0 - mis);   // bytes up to the end of the tensor
            const int region = w0 + par * C::kStageBytes + wave * C::kRowRegion;
            if ((size_t)nchunks * 16 <= left) {   // (wave-uniform) every chunk lies inside the tensor
#pragma unroll
                for (int it = 0; it < C::kRowPasses; ++it) {
                    const int c = lane + it * kWave;
                    if (c < nchunks) global_to_lds_16(src, (unsigned)(c * 16), region + it * kWave * 16);
                }
            } else {   // the last row of the tensor: the chunk that would cross its end goes element by element
#pragma unroll 1
                for (int it = 0; it < C::kRowPasses; ++it) {
                    const int c = lane + it * kWave;
                    if (c < nchunks) {
                        if ((size_t)(c + 1) * 16 <= left) {
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
    issue(b_begin, 0);

    // Operand addresses inside the first stage.
    // Values (transposing read): inside its group of 16 lanes, lane j points at four channels of halo
    // position 16b + 4g + j / 4 and receives the j-th channel of positions 16b + 4g .. + 3.  The channels
    // are dealt so that MFMA row m of half hf is channel 8 (m / 4) + 4 hf + m % 4: a lane then ends
    // up with the eight consecutive channels 8g .. 8g + 7 of its query, one 16-byte store.
    // (one stage: the addresses two per register, as 16-bit offsets from the start of the stage, where a lane has
    // 128 registers)
    constexpr bool VPACKED = C::kOneStage;
    static_assert(!VPACKED || C::kHaloBytes <= 65536, "value addresses as 16-bit offsets");
    int vaddr[VPACKED ? (P::NBLK + 1) / 2 : P::NBLK];   // a padding block of the last pair re-reads the last real block (its weights are zero)
#pragma unroll
    for (int b = 0; b < P::NBLK; ++b) {
        int h = 16 * b + 4 * g + (j >> 2);
        h = h < P::NKEY ? h : P::NKEY - 1;   // past the end: any real position (its weight is zero)
        const int hy = P::row_of(h), hx = h - hy * P::PW;
        const int off = ((oy - hoy + hy) * C::HALO_W + (ox - hox) + hx) * Traits<T>::kKeyBytes + (j & 3) * 16;
        if constexpr (VPACKED) vaddr[b >> 1] = (b & 1) ? (vaddr[b >> 1] | (off << 16)) : off;
        else vaddr[b] = lds0 + off;
    }
    auto value_addr = [&](int b) -> int {
        // (a patch halo that is 16 positions wide: block b is its row b)
        if constexpr (VPACKED && P::PW == 16) return lds0 + (int)((uint32_t)vaddr[0] & 0xffffu) + b * C::HALO_W * Traits<T>::kKeyBytes;
        else if constexpr (VPACKED) return lds0 + (int)((b & 1) ? (uint32_t)vaddr[b >> 1] >> 16 : (uint32_t)vaddr[b >> 1] & 0xffffu);
        else return vaddr[b];
    };
    // Weights: LDS address of this lane's query's weight for halo position 16 (e / 4) + 4g + e % 4, the
    // zero word where the position is outside the query's window.  The addresses hold the 16-byte
    // phase the query's row run has in the first plane of the range; later planes add the difference.
    const size_t qrow_off = ((size_t)(qy < H ? qy : H - 1) * W + tx0) * C::KK * SZ;
    auto phase_of = [&](int b) { return (int)((((size_t)b * heads + head) * plane_w + qrow_off) & 15); };
    const int phase0 = phase_of(b_begin);
    int cur_phase = phase0;
    const bool phase_varies = (plane_w & 15) != 0;
    // Built per group of four consecutive halo positions (e / 4): the positions of a group that lie inside
    // the query's window are in one halo row (a halo row holds K + 3 positions, the window K of them),
    // normally the row of the group's first position; when that position is already right of the window,
    // the group runs on into the next halo row and only that part can be inside.
    // Large windows (up to 64 weights per lane) keep the addresses two per register, as 16-bit offsets from the
    // start of the stage's weight rows and without the phase, which is added when they are used: the entry of
    // a position outside the window is the zero area, sixteen zero bytes, so that it reads zero at any phase.
    constexpr bool PACKED = K > 7;
    int gaddr[PACKED ? P::NEL / 2 : P::NEL];   // the padding block of the last pair has no entries: its weights are zero
    {
        const int wy = win_start(qy < H ? qy : H - 1, H, K) - oy, wx = win_start(qx < W ? qx : W - 1, W, K) - ox;
        const int lane_row = w0 + (4 * strip + jy) * C::kRowRegion + (PACKED ? 0 : phase0) + (4 * p + jx) * C::KK * SZ;
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
            for (int i = 0; i < 4; ++i) ga[i] = (unsigned)(c0 + i) < (unsigned)K ? base + i * SZ : zero_addr;
            if constexpr (PACKED) {
                gaddr[2 * G] = (ga[0] - w0) | ((ga[1] - w0) << 16);
                gaddr[2 * G + 1] = (ga[2] - w0) | ((ga[3] - w0) << 16);
                __builtin_amdgcn_sched_barrier(0);   // one group's temporaries at a time
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) gaddr[4 * G + i] = ga[i];
            }
        }
    }
    const int qlin = (qy < H - 1 ? qy : H - 1) * W + (qx < W - 1 ? qx : W - 1);

    // RPB: wave w sums row run w of the weights per window slot (lane = slot).  All queries of the run
    // share the bias row offset; the queries away from the left and right border also share the column
    // offset and are summed in a register; the few border queries update the wave's private
    // (2K-1)^2 table in LDS one at a time.
    constexpr int NB = 2 * K - 1, CELLS = NB * NB;
    const int rtbl = lds0 + C::kLdsStages + wave * CELLS * 4;
    constexpr int SPL = (C::KK + kWave - 1) / kWave;   // window slots per lane (slot = lane + 64 s)
    float racc[SPL];
    int slot_cell[SPL];   // a slot's place inside the table, relative to (py, px)
#pragma unroll
    for (int sl = 0; sl < SPL; ++sl) {
        const int slot = lane + sl * kWave;
        racc[sl] = 0.f;
        slot_cell[sl] = (slot / K) * NB + (slot % K);
    }
    const int rpy = rpb_start(wrow < H ? wrow : H - 1, H, K);
    const int nvalid = (W - tx0) < kTileX ? (W - tx0) : kTileX;
    const int xi0 = (tx0 > P::R ? tx0 : P::R) - tx0;                                   // interior queries of the run:
    const int xi1 = ((tx0 + nvalid) < (W - P::R) ? (tx0 + nvalid) : (W - P::R)) - tx0;   // [xi0, xi1)
    if constexpr (RPB) {
        for (int i = tid; i < C::WAVES * CELLS; i += C::kThreads) *lds_ptr<float>(lds0 + C::kLdsStages + i * 4) = 0.f;
    }
    auto row_sums = [&](auto par_c, int b) {
        constexpr int PAR = decltype(par_c)::value;
        if (wrow >= H) return;
        const int run0 = w0 + PAR * C::kStageBytes + wave * C::kRowRegion +
                         (int)((((size_t)b * heads + head) * plane_w + wrow_off) & 15);
#pragma unroll
        for (int sl = 0; sl < SPL; ++sl) {
            const int slot = lane + sl * kWave;
            if (slot < C::KK) {
                const int run = run0 + slot * SZ;
                // all sixteen reads in flight at once (queries past the end of the run re-read its first one)
                float v[kTileX];
#pragma unroll
                for (int i = 0; i < kTileX; ++i) v[i] = to_f32(*lds_ptr<T>(run + (i < nvalid ? i : 0) * C::KK * SZ));
                float s0 = 0.f, s1 = 0.f;
#pragma unroll
                for (int i = 0; i < kTileX; i += 2) {
                    s0 += (i >= xi0 && i < xi1) ? v[i] : 0.f;
                    s1 += (i + 1 >= xi0 && i + 1 < xi1) ? v[i + 1] : 0.f;
                }
                racc[sl] += s0 + s1;
                if (xi0 > 0 || xi1 < nvalid) {   // border queries (the leftmost / rightmost tile of the map only)
#pragma unroll
                    for (int i = 0; i < kTileX; ++i) {
                        if (i < nvalid && !(i >= xi0 && i < xi1)) {
                            const int cell = rtbl + ((rpy * NB + rpb_start(tx0 + i, W, K)) + slot_cell[sl]) * 4;
                            *lds_ptr<float>(cell) += v[i];
                        }
                    }
                }
            }
        }
    };

    auto compute = [&](auto par_c, int b) {
        constexpr int PAR = decltype(par_c)::value;
        if (!active) return;
        f32x4 o[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
        // A pair of halo blocks needs eight gathered weights (the B operand) and four transposing reads of the
        // values (the A operands of the two channel halves).  The reads of pair pb + 1 are issued before pair pb is
        // multiplied, and the scheduling fences keep the compiler from sinking them back to their uses: a wave has
        // twelve reads in flight behind every pair of MFMAs instead of waiting for each pair's reads in turn.
        uint16_t wlo[2][4], whi[2][4];
        u32x2 xlo[2][2], xhi[2][2];
        if constexpr (C::kOneStage) {
            // the packed tables stay packed: without this their unpacking is hoisted out of the loop over the planes
            // and takes a register per address
#pragma unroll
            for (int e = 0; e < P::NEL / 2; ++e) asm volatile("" : "+v"(gaddr[e]));
#pragma unroll
            for (int e = 0; e < (P::NBLK + 1) / 2; ++e) asm volatile("" : "+v"(vaddr[e]));
        }
        auto fetch = [&](int pb, int st) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = 8 * pb + 2 * u;
                if (e >= P::NEL) {
                    wlo[st][u] = whi[st][u] = 0;
                    continue;
                }
                if constexpr (PACKED) {   // e is even: both addresses sit in one register
                    const uint32_t pk = (uint32_t)gaddr[e >> 1];
                    const int wbase = w0 + cur_phase + PAR * C::kStageBytes;
                    wlo[st][u] = *lds_ptr<uint16_t>(wbase + (int)(pk & 0xffffu));
                    whi[st][u] = *lds_ptr<uint16_t>(wbase + (int)(pk >> 16));
                } else {
                    wlo[st][u] = *lds_ptr<uint16_t>(gaddr[e] + PAR * C::kStageBytes);
                    whi[st][u] = *lds_ptr<uint16_t>(gaddr[e + 1] + PAR * C::kStageBytes);
                }
            }
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                xlo[st][hf] = lds_read_tr16(value_addr(2 * pb) + PAR * C::kStageBytes + hf * 8);
                xhi[st][hf] = lds_read_tr16(value_addr(2 * pb + 1 < P::NBLK ? 2 * pb + 1 : P::NBLK - 1) + PAR * C::kStageBytes + hf * 8);
            }
        };
        if (!kProbeMemoryOnly) {   // (measurement build: zeros are stored)
            fetch(0, 0);
#pragma unroll
            for (int pb = 0; pb < C::NPAIR; ++pb) {
                const int st = pb & 1;
                if (pb + 1 < C::NPAIR) fetch(pb + 1, st ^ 1);
                __builtin_amdgcn_sched_barrier(0);
                uint32_t wv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) wv[u] = (uint32_t)wlo[st][u] | ((uint32_t)whi[st][u] << 16);
                const u32x4 bop = u32x4{wv[0], wv[1], wv[2], wv[3]};
#pragma unroll
                for (int hf = 0; hf < 2; ++hf)
                    o[hf] = mfma_16x16x32<T>(u32x4{xlo[st][hf].x, xlo[st][hf].y, xhi[st][hf].x, xhi[st][hf].y}, bop, o[hf]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (q_ok && (!half_dim || g < 2)) {
            char *dst = reinterpret_cast<char *>(out) + ((size_t)b * heads + head) * plane_y + (size_t)qlin * pitch + g * 16;
            uint32_t ov[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                typedef float f32x2_t __attribute__((ext_vector_type(2)));
                typedef T tx2_t __attribute__((ext_vector_type(2)));
                const int hf = u >> 1, r = 2 * (u & 1);
                ov[u] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){o[hf][r] * scale, o[hf][r + 1] * scale}, tx2_t));
            }
            store16_stream(dst, u32x4{ov[0], ov[1], ov[2], ov[3]});   // channels 8g .. 8g + 7
        }
    };

    int b = b_begin;
    auto step = [&](auto par_c) {
        constexpr int PAR = decltype(par_c)::value;
        wait_global_loads();   // this tile's halo and weight rows have landed
        workgroup_sync();       // ... for every wave, and nobody still reads the other stage
        if constexpr (!C::kOneStage) {
            if (b + 1 < b_end) issue(b + 1, PAR ^ 1);
        }
        if (phase_varies) {   // the table follows the phase of this plane's row run (in-window entries only)
            const int ph = phase_of(b), d = ph - cur_phase;
            cur_phase = ph;
            if constexpr (!PACKED) {
#pragma unroll
                for (int e = 0; e < P::NEL; ++e) gaddr[e] += gaddr[e] != zero_addr ? d : 0;
            }
        }
        compute(par_c, b);
        if constexpr (RPB) row_sums(par_c, b);
        if constexpr (C::kOneStage) {
            if (b + 1 < b_end) {
                workgroup_sync();   // nobody still reads the stage
                issue(b + 1, 0);
            }
        }
        ++b;
    };
    while (b < b_end) {
        step(IntC<0>{});
        if constexpr (!C::kOneStage) {
            if (b < b_end) step(IntC<1>{});
        }
    }

    if constexpr (RPB) {
        // interior sums into the wave's table, then the eight tables are added in wave order
#pragma unroll
        for (int sl = 0; sl < SPL; ++sl)
            if (wrow < H && lane + sl * kWave < C::KK && xi1 > xi0) *lds_ptr<float>(rtbl + ((rpy * NB + P::R) + slot_cell[sl]) * 4) += racc[sl];
        workgroup_sync();
        for (int cell = tid; cell < CELLS; cell += C::kThreads) {
            float sum = *lds_ptr<float>(lds0 + C::kLdsStages + cell * 4);
#pragma unroll
            for (int wv_ = 1; wv_ < C::WAVES; ++wv_) sum += *lds_ptr<float>(lds0 + C::kLdsStages + (wv_ * CELLS + cell) * 4);
            // row of this workgroup's partial: the partials of a head follow each other (rpb_cell_stride)
            rpb_partial[(size_t)((head * splits + work.split) * gd.npos + work.pos) * rpb_cell_stride(CELLS) + cell] = sum;
        }
    }
}

template <typename T, int K, bool RPB = false>
static hipError_t launch_av_mfma_small_t(const Problem &p, const void *w, const void *y, float scale, void *out,
                                         hipStream_t s, float *rpb_partial = nullptr) {
    using C = AvSmallCfg<T, K>;
    static_assert(K > 7 || C::kLdsBytes <= 80 * 1024, "two workgroups share the LDS of a compute unit");
    static_assert(C::kLdsBytes <= 160 * 1024, "LDS of a compute unit");
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    const UnitSplit us = unit_split(tiles_x, tiles_y, p.heads, p.B);
    auto kern = av_mfma_small_kernel<T, K, RPB>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    // one launch per 32-channel slice of the head vector (the weights are read again by each)
    for (int sl = 0; sl < (p.D + kHeadDim - 1) / kHeadDim; ++sl) {   // (a 16-channel head is half a slice)
        hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(us.units * us.splits)), dim3(C::kThreads), C::kLdsBytes, s,
                           static_cast<const T *>(w), static_cast<const T *>(y) + sl * kHeadDim, scale,
                           static_cast<T *>(out) + sl * kHeadDim, rpb_partial, p.H, p.W, p.heads, p.B, tiles_y, us.units,
                           us.splits, us.gd, p.D * (int)sizeof(T));
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    return hipSuccess;
}

// grad-q together with partial bias gradients (one per workgroup, av_rpb_partials() of them)
bool av_rpb_supported(const Problem &p) { return (p.D == kHeadDim || p.D == kHalfDim) && p.dtype != NA2D_F32 && p.K <= 9; }
AvRpbSplit av_rpb_split(const Problem &p) {
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + 8 - 1) / 8;
    const UnitSplit us = unit_split(tiles_x, tiles_y, p.heads, p.B);
    AvRpbSplit r;
    r.npos = us.units / p.heads;
    r.splits = us.splits;
    return r;
}
hipError_t launch_av_rpb(const Problem &p, const void *w, const void *y, float scale, void *out, float *rpb_partial,
                         hipStream_t s) {
#define NA2D_AVR_K(TT)                                                                                        \
    switch (p.K) {                                                                                            \
        case 3: return launch_av_mfma_small_t<TT, 3, true>(p, w, y, scale, out, s, rpb_partial);              \
        case 5: return launch_av_mfma_small_t<TT, 5, true>(p, w, y, scale, out, s, rpb_partial);              \
        case 7: return launch_av_mfma_small_t<TT, 7, true>(p, w, y, scale, out, s, rpb_partial);              \
        case 9: return launch_av_mfma_small_t<TT, 9, true>(p, w, y, scale, out, s, rpb_partial);              \
        default: return hipErrorInvalidValue;                                                                 \
    }
    if (p.dtype == NA2D_F16) { NA2D_AVR_K(f16_t) }
    if (p.dtype == NA2D_BF16) { NA2D_AVR_K(bf16_t) }
#undef NA2D_AVR_K
    return hipErrorInvalidValue;
}

bool av_mfma_supported(const Problem &p) {
    // any multiple of 32 channels: one launch per 32-channel slice
    return p.dtype != NA2D_F32 && (p.D % kHeadDim == 0 || p.D == kHalfDim) && p.K <= kMaxTunedK;
}

hipError_t launch_av_mfma(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s) {
    if (p.dtype == NA2D_F16) {
        using T = f16_t;
        NA2D_DISPATCH_K(p.K, return (launch_av_mfma_small_t<T, K>(p, w, y, scale, out, s)));
    } else if (p.dtype == NA2D_BF16) {
        using T = bf16_t;
        NA2D_DISPATCH_K(p.K, return (launch_av_mfma_small_t<T, K>(p, w, y, scale, out, s)));
    }
    return hipErrorInvalidValue;
}

}  // namespace na2d
