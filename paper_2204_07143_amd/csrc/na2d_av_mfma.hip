// Neighbourhood weighted sum on the matrix cores (f16 / bf16):
//   out[n, :] = scale * sum_{a, c} w[n, a, c] * y_{rho(n; a, c)}
// (arXiv 2204.07143, Eq. 3-4; with w = ds, y = k it is grad-q, Appendix A).
//
// Same tiling as the matrix-core logits kernel: persistent workgroups walk 16 x (4*WAVES) query
// tiles, a wave owns a strip of four 4 x 4 query patches, and a patch against its halo is a
// dense contraction -- here over the halo positions:  out^T[d, q] = sum_pos Yt[d, pos] * P[pos, q].
//   A operand: the values, staged transposed in LDS as Yt[channel][halo position] (8-byte reads
//              of 4 consecutive positions; two 16-position blocks feed one 16x16x32 MFMA);
//   B operand: the patch's weights spread over the halo positions, gathered from the tile's
//              weight rows in LDS through a per-lane table of LDS addresses (positions outside a
//              query's window read a zero word).  The table depends only on the lane and on the
//              border shift of the window and is rebuilt only when that changes;
//   result   : lane (query j, group g) holds channels 16*half + 4g .. +3 of its own query, so the
//              scale and the 8-byte global stores need no cross-lane traffic.
// The next tile's values and weight rows are prefetched into registers while the current tile is
// computed.
#include "na2d_kernels.hpp"
#include "na2d_mfma.hpp"
#include "na2d_tile.hpp"

namespace na2d {

template <typename T, int K, int WAVES>
struct AvMfmaCfg {
    using P = PatchT<K>;
    static constexpr int TY = 4 * WAVES;
    static constexpr int HALO_H = 4 * (WAVES - 1) + P::ROWS;   // farthest strip offset + rows the enumeration touches
    static constexpr int HALO_W = 12 + P::PWP;                 // farthest patch offset + padded patch-halo width
    static constexpr int KK = K * K;
    static constexpr int kThreads = kWave * WAVES;
    using Halo = TransposedHalo<T, HALO_H, HALO_W, kThreads>;
    static constexpr int kRowBytes = kTileX * KK * (int)sizeof(T);
    static constexpr int kRowRegion = mirror_bytes(kRowBytes);
    static constexpr int kPatchStep = 4 * KK * (int)sizeof(T);
    static constexpr int kZeroBytes = (3 * kPatchStep + 16 + 15) & ~15;   // what out-of-window table entries read
    static constexpr int kWaveBytes = 4 * kRowRegion + kZeroBytes;
    static constexpr int kLdsBytes = Halo::kBytes + WAVES * kWaveBytes;
};

template <typename T, int K>
constexpr int av_mfma_waves() {
    return AvMfmaCfg<T, K, 4>::kLdsBytes <= 80 * 1024 ? 4 : 2;
}

struct AvTile {
    int ty0, tx0, plane, hoy, hox;
};

template <typename T, int K, int WAVES>
__global__ __launch_bounds__(kWave *WAVES, WAVES == 4 ? 2 : 1) void av_mfma_kernel(const T *__restrict__ w,
                                                                                    const T *__restrict__ y, float scale,
                                                                                    T *__restrict__ out, int H, int W,
                                                                                    int tiles_x, int tiles_y, int ntiles,
                                                                                    int tiles_per_wg) {
    using C = AvMfmaCfg<T, K, WAVES>;
    using P = PatchT<K>;
    using Halo = typename C::Halo;
    constexpr int SZ = (int)sizeof(T);
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int j = lane & 15, g = lane >> 4, jy = j >> 2, jx = j & 3;
    const int lds0 = lds_addr(lds);
    const int wreg_off = lds0 + Halo::kBytes + wave * C::kWaveBytes;
    char *wreg = lds + Halo::kBytes + wave * C::kWaveBytes;
    const int zero_addr = wreg_off + 4 * C::kRowRegion;
    for (int i = lane * 4; i < C::kZeroBytes; i += kWave * 4) *lds_ptr<uint32_t>(zero_addr + i) = 0u;

    // A-operand addresses of this lane (channel j of a half, positions 16b + 4g .. +3), relative
    // to the patch origin inside the tile halo
    int vtoff[P::NBLK];
#pragma unroll
    for (int b = 0; b < P::NBLK; ++b) {
        const int h0 = 16 * b + 4 * g;
        const int hy = P::row_of(h0), hx0 = h0 - hy * P::PWP;
        vtoff[b] = lds0 + j * Halo::DSTRIDE + (hy * C::HALO_W + hx0) * 2;
    }
    int gaddr[P::NEL];
#pragma unroll
    for (int e = 0; e < P::NEL; ++e) gaddr[e] = zero_addr;
    int cur_wy = -100000, cur_wx = -100000, cur_base = 0;

    const int wg = xcd_contiguous_block(blockIdx.x, gridDim.x);
    const int t_begin = wg * tiles_per_wg;
    const int t_end = (wg + 1) * tiles_per_wg < ntiles ? (wg + 1) * tiles_per_wg : ntiles;
    if (t_begin >= t_end) return;

    auto tile_of = [&](int t) {
        const TileCoord tc = decode_tile(t, tiles_x, tiles_y);
        AvTile q;
        q.ty0 = tc.tiy * C::TY;
        q.tx0 = tc.tix * kTileX;
        q.plane = tc.plane;
        q.hoy = halo_origin(q.ty0, C::TY, H, K);
        q.hox = halo_origin(q.tx0, kTileX, W, K);
        return q;
    };

    Halo halo;
    halo.init(W, tid, lds0);
    StageIn<T, C::kRowBytes, kWave> rows_in[4];
    auto prefetch = [&](const AvTile &tl) {
        const size_t plane_q = (size_t)tl.plane * H * W;
        halo.issue(reinterpret_cast<const char *>(y) + plane_q * Traits<T>::kKeyBytes, H, W, tl.hoy, tl.hox);
        const int nvalid = (W - tl.tx0) < kTileX ? (W - tl.tx0) : kTileX;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int qy = tl.ty0 + 4 * wave + r;
            const size_t g0r = (plane_q + (size_t)(qy < H ? qy : 0) * W + tl.tx0) * C::KK * SZ;
            rows_in[r].issue(reinterpret_cast<const char *>(w), g0r, qy < H ? nvalid * C::KK * SZ : 0, lane);
        }
    };

    AvTile cur = tile_of(t_begin);
    prefetch(cur);

    for (int t = t_begin; t < t_end; ++t) {
        const int ty0 = cur.ty0, tx0 = cur.tx0, hoy = cur.hoy, hox = cur.hox;
        const size_t plane_q = (size_t)cur.plane * H * W;
        __syncthreads();   // every wave is done with the previous tile's values
        halo.commit();
#pragma unroll
        for (int r = 0; r < 4; ++r) rows_in[r].commit(wreg + r * C::kRowRegion, lane);
        __syncthreads();
        if (t + 1 < t_end) {
            cur = tile_of(t + 1);
            prefetch(cur);
        }

        const int sy0 = ty0 + 4 * wave;
        if (sy0 >= H) continue;
        const int oy = halo_origin(sy0, 4, H, K);
        const int qy = sy0 + jy;
        const bool row_ok = qy < H;
        const size_t rowg0 = (plane_q + (size_t)qy * W + tx0) * C::KK * SZ;
        const int lanebase = wreg_off + jy * C::kRowRegion + (int)(rowg0 & 15) + jx * C::KK * SZ;
        const int wy = row_ok ? win_start(qy, H, K) - oy : 100000;

#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int px0 = tx0 + 4 * p;
            if (px0 < W) {
                const int ox = halo_origin(px0, 4, W, K);
                const int qx = px0 + jx;
                const bool q_ok = row_ok && qx < W;
                const int want_wy = q_ok ? wy : 100000;
                const int want_wx = q_ok ? win_start(qx, W, K) - ox : 100000;
                if (__any(want_wy != cur_wy || want_wx != cur_wx || lanebase != cur_base)) {
                    cur_wy = want_wy;
                    cur_wx = want_wx;
                    cur_base = lanebase;
                    int gv = g;
                    asm volatile("" : "+v"(gv));   // keep the index arithmetic inside this rare block
#pragma unroll
                    for (int e = 0; e < P::NEL; ++e) {
                        const int h = 16 * (e >> 2) + 4 * gv + (e & 3);
                        const int hy = P::row_of(h), hx = h - hy * P::PWP;
                        const int a = hy - want_wy, c = hx - want_wx;
                        const bool ok = (unsigned)a < (unsigned)K && (unsigned)c < (unsigned)K;
                        gaddr[e] = ok ? lanebase + (a * K + c) * SZ : zero_addr;
                    }
                }
                const int patch_off = ((oy - hoy) * C::HALO_W + (ox - hox)) * 2;
                const bool aligned = (patch_off & 7) == 0;
                f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
                for (int pb = 0; pb < P::NPAIR; ++pb) {
                    // weights of this lane's query at positions 16b + 4g + r of the two blocks
                    uint32_t wv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int e = 8 * pb + 2 * u;
                        const uint32_t lo = *lds_ptr<uint16_t>(gaddr[e] + p * C::kPatchStep);
                        const uint32_t hi = *lds_ptr<uint16_t>(gaddr[e + 1] + p * C::kPatchStep);
                        wv[u] = lo | (hi << 16);
                    }
                    const u32x4 bop = u32x4{wv[0], wv[1], wv[2], wv[3]};
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) {
                        const int a0 = vtoff[2 * pb] + patch_off + hf * 16 * Halo::DSTRIDE;
                        const int a1 = vtoff[2 * pb + 1] + patch_off + hf * 16 * Halo::DSTRIDE;
                        u32x4 aop;
                        if (aligned) {
                            const uint64_t lo = *lds_ptr<uint64_t>(a0);
                            const uint64_t hi = *lds_ptr<uint64_t>(a1);
                            aop = u32x4{(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
                        } else {
                            uint32_t q4[4];
#pragma unroll
                            for (int u = 0; u < 2; ++u) {
                                q4[u] = (uint32_t)*lds_ptr<uint16_t>(a0 + 4 * u) | ((uint32_t)*lds_ptr<uint16_t>(a0 + 4 * u + 2) << 16);
                                q4[2 + u] = (uint32_t)*lds_ptr<uint16_t>(a1 + 4 * u) | ((uint32_t)*lds_ptr<uint16_t>(a1 + 4 * u + 2) << 16);
                            }
                            aop = u32x4{q4[0], q4[1], q4[2], q4[3]};
                        }
                        acc[hf] = mfma_16x16x32<T>(aop, bop, acc[hf]);
                    }
                }
                if (q_ok) {
                    char *dst = reinterpret_cast<char *>(out) + (plane_q + (size_t)qy * W + qx) * Traits<T>::kKeyBytes + g * 8;
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) {
                        uint32_t o[2];
#pragma unroll
                        for (int u = 0; u < 2; ++u) {
                            const T lo = from_f32<T>(acc[hf][2 * u] * scale), hi = from_f32<T>(acc[hf][2 * u + 1] * scale);
                            o[u] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
                        }
                        *reinterpret_cast<uint64_t *>(dst + hf * 32) = (uint64_t)o[0] | ((uint64_t)o[1] << 32);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // the weight rows of this strip are consumed; the next commit may overwrite them
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- small windows (K <= 7): one patch per wave, operands loaded straight into LDS -----------
//
// Eight waves share a 16 x 8 query tile, one 4 x 4 patch each.  A workgroup keeps one tile position
// and one head and walks a range of the batch: the per-lane gather addresses of the weights and
// the operand addresses of the values are built once.  Per tile the value halo (natural layout)
// and the tile's eight weight row runs (mirrored at their 16-byte phase) reach one of two LDS
// stages by direct loads while the previous tile is computed.  Halo positions are numbered
// h = hy * (K+3) + hx; MFMA pair m contracts over the positions 32m .. 32m+31 in the lane order
//   lane group g, element e:  position 32m + 16 (e / 4) + 4g + e % 4.
//   A operand: channel j of those positions, two transposing LDS reads from the value halo;
//   B operand: the weights of query j at those positions, 2-byte gathers from its row run (zero
//              outside its window).
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
    static_assert(kRowChunks <= 2 * kWave, "a row run is loaded by two instructions of one wave");
    static constexpr int kWBytes = TY * kRowRegion;
    static constexpr int kStageBytes = kHaloBytes + kWBytes + 16;   // + the zero word
    static constexpr int kLdsStages = 2 * kStageBytes;
    static constexpr int kRpbBytes = WAVES * (2 * K - 1) * (2 * K - 1) * 4;   // per-wave bias-gradient tables (grad-b variant)
    static constexpr int kLdsBytes = kLdsStages + kRpbBytes;
    static_assert(kStageBytes < 65536, "the second stage is reached through the 16-bit offset of the LDS reads");
};

// RPB: the kernel also sums the weights it gathers, per lane and halo position, over its planes; at
// the end the workgroup adds them up per cell of the (2K-1)^2 bias table in a fixed order and writes
// one partial bias gradient (with w = ds this is grad-b, arXiv 2204.07143 Appendix A; Eq. 2's B).
template <typename T, int K, bool RPB>
__global__ __launch_bounds__(512, 4) void av_mfma_small_kernel(const T *__restrict__ w, const T *__restrict__ y, float scale,
                                                               T *__restrict__ out, float *__restrict__ rpb_partial, int H,
                                                               int W, int heads, int nb, int tiles_y, int units, int splits,
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
    const int strip = wave >> 2, p = wave & 3;
    const int j = lane & 15, g = lane >> 4, jy = j >> 2, jx = j & 3;
    const int lds0 = lds_addr(lds);
    const int w0 = lds0 + C::kHaloBytes, zero_addr = w0 + C::kWBytes;

    const int wg = xcd_contiguous_block(blockIdx.x, gridDim.x);
    if (wg >= units * splits) return;
    // neighbouring workgroups take neighbouring tile positions of the same planes (the position index
    // runs fastest), so the positions whose halos overlap run at the same time on the same XCD and
    // the overlap is read from HBM once
    const int npos = units / heads;
    const int pos = wg % npos, head = (wg / npos) % heads, split = wg / (npos * heads);
    const int ty0 = (pos % tiles_y) * C::TY, tx0 = (pos / tiles_y) * kTileX;
    const int b_begin = (split * nb) / splits, b_end = ((split + 1) * nb) / splits;
    if (b_begin >= b_end) return;

    // the zero words (one per stage) are never written by the loads
    if (tid < 8) *lds_ptr<uint32_t>(zero_addr + (tid >> 2) * C::kStageBytes + (tid & 3) * 4) = 0u;

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
    halo.offsets(H, W, hoy, hox, hoff, pitch);
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
            const char *src = reinterpret_cast<const char *>(w) + (g0 - mis);
            const size_t left = w_bytes - (g0 - mis);   // bytes up to the end of the tensor
            const int region = w0 + par * C::kStageBytes + wave * C::kRowRegion;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int c = lane + it * kWave;
                if (c < nchunks) {
                    if ((size_t)(c + 1) * 16 <= left) {
                        global_to_lds_16(src + c * 16, region + it * kWave * 16);
                    } else {   // the chunk that would cross the end of the tensor: element by element
                        for (int e = c * 16; e < mis + wrow_bytes; e += SZ)
                            *lds_ptr<T>(region + e) = *reinterpret_cast<const T *>(src + e);
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
    int vaddr[P::NBLK];   // a padding block of the last pair re-reads the last real block (its weights are zero)
#pragma unroll
    for (int b = 0; b < P::NBLK; ++b) {
        int h = 16 * b + 4 * g + (j >> 2);
        h = h < P::NKEY ? h : P::NKEY - 1;   // past the end: any real position (its weight is zero)
        const int hy = P::row_of(h), hx = h - hy * P::PW;
        vaddr[b] = lds0 + ((oy - hoy + hy) * C::HALO_W + (ox - hox) + hx) * Traits<T>::kKeyBytes + (j & 3) * 16;
    }
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
    int gaddr[P::NEL];   // the padding block of the last pair has no entries: its weights are zero
    {
        const int wy = win_start(qy < H ? qy : H - 1, H, K) - oy, wx = win_start(qx < W ? qx : W - 1, W, K) - ox;
        const int lane_row = w0 + (4 * strip + jy) * C::kRowRegion + phase0 + (4 * p + jx) * C::KK * SZ;
#pragma unroll
        for (int G = 0; G < P::NBLK; ++G) {
            const int h0 = 16 * G + 4 * g;
            const int hy0 = P::row_of(h0), hx0 = h0 - hy0 * P::PW;
            const bool wrap = hx0 > wx + K - 1;
            const int a = hy0 + (wrap ? 1 : 0) - wy;
            int c0 = hx0 - (wrap ? P::PW : 0) - wx;   // window column of the group's first position (may be negative)
            const int base = lane_row + (a * K + c0) * SZ;
            c0 = (q_ok && (unsigned)a < (unsigned)K) ? c0 : 64;   // no row of the window: every column test fails
#pragma unroll
            for (int i = 0; i < 4; ++i) gaddr[4 * G + i] = (unsigned)(c0 + i) < (unsigned)K ? base + i * SZ : zero_addr;
        }
    }
    const int qlin = (qy < H - 1 ? qy : H - 1) * W + (qx < W - 1 ? qx : W - 1);

    // RPB: wave w sums row run w of the weights per window slot (lane = slot).  All queries of the run
    // share the bias row offset; the queries away from the left and right border also share the column
    // offset and are summed in a register; the few border queries update the wave's private
    // (2K-1)^2 table in LDS one at a time.
    constexpr int NB = 2 * K - 1, CELLS = NB * NB;
    const int rtbl = lds0 + C::kLdsStages + wave * CELLS * 4;
    float racc = 0.f;
    const int rpy = rpb_start(wrow < H ? wrow : H - 1, H, K);
    const int nvalid = (W - tx0) < kTileX ? (W - tx0) : kTileX;
    const int xi0 = (tx0 > P::R ? tx0 : P::R) - tx0;                                   // interior queries of the run:
    const int xi1 = ((tx0 + nvalid) < (W - P::R) ? (tx0 + nvalid) : (W - P::R)) - tx0;   // [xi0, xi1)
    const int slot_cell = (lane / K) * NB + (lane % K);   // this lane's slot inside the table, relative to (py, px)
    if constexpr (RPB) {
        for (int i = tid; i < C::WAVES * CELLS; i += C::kThreads) *lds_ptr<float>(lds0 + C::kLdsStages + i * 4) = 0.f;
    }
    auto row_sums = [&](auto par_c, int b) {
        constexpr int PAR = decltype(par_c)::value;
        if (wrow >= H || lane >= C::KK) return;
        const int run = w0 + PAR * C::kStageBytes + wave * C::kRowRegion +
                        (int)((((size_t)b * heads + head) * plane_w + wrow_off) & 15) + lane * SZ;
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
        racc += s0 + s1;
        if (xi0 > 0 || xi1 < nvalid) {   // border queries (the leftmost / rightmost tile of the map only)
#pragma unroll
            for (int i = 0; i < kTileX; ++i) {
                if (i < nvalid && !(i >= xi0 && i < xi1)) {
                    const int cell = rtbl + ((rpy * NB + rpb_start(tx0 + i, W, K)) + slot_cell) * 4;
                    *lds_ptr<float>(cell) += v[i];
                }
            }
        }
    };

    auto compute = [&](auto par_c, int b) {
        constexpr int PAR = decltype(par_c)::value;
        if (!active) return;
        f32x4 o[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int pb = 0; pb < C::NPAIR; ++pb) {
            uint32_t wv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = 8 * pb + 2 * u;
                if (e >= P::NEL) {
                    wv[u] = 0u;
                    continue;
                }
                wv[u] = (uint32_t)*lds_ptr<uint16_t>(gaddr[e] + PAR * C::kStageBytes) |
                        ((uint32_t)*lds_ptr<uint16_t>(gaddr[e + 1] + PAR * C::kStageBytes) << 16);
            }
            const u32x4 bop = u32x4{wv[0], wv[1], wv[2], wv[3]};
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const u32x2 lo = lds_read_tr16(vaddr[2 * pb] + PAR * C::kStageBytes + hf * 8);
                const u32x2 hi = lds_read_tr16(vaddr[2 * pb + 1 < P::NBLK ? 2 * pb + 1 : P::NBLK - 1] + PAR * C::kStageBytes + hf * 8);
                o[hf] = mfma_16x16x32<T>(u32x4{lo.x, lo.y, hi.x, hi.y}, bop, o[hf]);
            }
        }
        if (q_ok) {
            char *dst = reinterpret_cast<char *>(out) + ((size_t)b * heads + head) * plane_y + (size_t)qlin * pitch + g * 16;
            uint32_t ov[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                typedef float f32x2_t __attribute__((ext_vector_type(2)));
                typedef T tx2_t __attribute__((ext_vector_type(2)));
                const int hf = u >> 1, r = 2 * (u & 1);
                ov[u] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){o[hf][r] * scale, o[hf][r + 1] * scale}, tx2_t));
            }
            *reinterpret_cast<u32x4 *>(dst) = u32x4{ov[0], ov[1], ov[2], ov[3]};   // channels 8g .. 8g + 7
        }
    };

    int b = b_begin;
    auto step = [&](auto par_c) {
        constexpr int PAR = decltype(par_c)::value;
        wait_global_loads();   // this tile's halo and weight rows have landed
        __syncthreads();       // ... for every wave, and nobody still reads the other stage
        if (b + 1 < b_end) issue(b + 1, PAR ^ 1);
        if (phase_varies) {   // the table follows the phase of this plane's row run (in-window entries only)
            const int ph = phase_of(b), d = ph - cur_phase;
            cur_phase = ph;
#pragma unroll
            for (int e = 0; e < P::NEL; ++e) gaddr[e] += gaddr[e] != zero_addr ? d : 0;
        }
        compute(par_c, b);
        if constexpr (RPB) row_sums(par_c, b);
        ++b;
    };
    while (b < b_end) {
        step(IntC<0>{});
        if (b < b_end) step(IntC<1>{});
    }

    if constexpr (RPB) {
        // interior sums into the wave's table, then the eight tables are added in wave order
        if (wrow < H && lane < C::KK && xi1 > xi0) *lds_ptr<float>(rtbl + ((rpy * NB + P::R) + slot_cell) * 4) += racc;
        __syncthreads();
        for (int cell = tid; cell < CELLS; cell += C::kThreads) {
            float sum = *lds_ptr<float>(lds0 + C::kLdsStages + cell * 4);
#pragma unroll
            for (int wv_ = 1; wv_ < C::WAVES; ++wv_) sum += *lds_ptr<float>(lds0 + C::kLdsStages + (wv_ * CELLS + cell) * 4);
            rpb_partial[(size_t)wg * CELLS + cell] = sum;
        }
    }
}

template <typename T, int K, bool RPB = false>
static hipError_t launch_av_mfma_small_t(const Problem &p, const void *w, const void *y, float scale, void *out,
                                         hipStream_t s, float *rpb_partial = nullptr) {
    using C = AvSmallCfg<T, K>;
    static_assert(C::kLdsBytes <= 80 * 1024, "two workgroups share the LDS of a compute unit");
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    const UnitSplit us = unit_split(tiles_x, tiles_y, p.heads, p.B);
    auto kern = av_mfma_small_kernel<T, K, RPB>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // one launch per 32-channel slice of the head vector (the weights are read again by each)
    for (int sl = 0; sl < p.D / kHeadDim; ++sl) {
        hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(us.units * us.splits)), dim3(C::kThreads), C::kLdsBytes, s,
                           static_cast<const T *>(w), static_cast<const T *>(y) + sl * kHeadDim, scale,
                           static_cast<T *>(out) + sl * kHeadDim, rpb_partial, p.H, p.W, p.heads, p.B, tiles_y, us.units,
                           us.splits, p.D * (int)sizeof(T));
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    return hipSuccess;
}

// grad-q together with partial bias gradients (one per workgroup, av_rpb_partials() of them)
bool av_rpb_supported(const Problem &p) { return p.D == kHeadDim && p.dtype != NA2D_F32 && p.K <= 7 && !force_valu(); }
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
        default: return hipErrorInvalidValue;                                                                 \
    }
    if (p.dtype == NA2D_F16) { NA2D_AVR_K(f16_t) }
    if (p.dtype == NA2D_BF16) { NA2D_AVR_K(bf16_t) }
#undef NA2D_AVR_K
    return hipErrorInvalidValue;
}

template <typename T, int K>
static hipError_t launch_av_mfma_t(const Problem &p, const void *w, const void *y, float scale, void *out,
                                   hipStream_t s) {
    constexpr int WAVES = av_mfma_waves<T, K>();
    using C = AvMfmaCfg<T, K, WAVES>;
    static_assert(C::kLdsBytes <= 160 * 1024, "tile does not fit the 160 KB LDS of a CDNA4 compute unit");
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    const int ntiles = tiles_x * tiles_y * p.planes();
    const int max_wgs = 256 * 2;
    const int tiles_per_wg = (ntiles + max_wgs - 1) / max_wgs;
    const int nwg = (ntiles + tiles_per_wg - 1) / tiles_per_wg;
    auto kern = av_mfma_kernel<T, K, WAVES>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(nwg)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(w), static_cast<const T *>(y), scale, static_cast<T *>(out), p.H, p.W,
                       tiles_x, tiles_y, ntiles, tiles_per_wg);
    return hipGetLastError();
}

bool av_mfma_supported(const Problem &p) {
    if (p.dtype == NA2D_F32 || force_valu()) return false;
    return p.D == kHeadDim || (p.D % kHeadDim == 0 && p.K <= 7);   // slices only in the small-window kernel
}

hipError_t launch_av_mfma(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s) {
    if (p.dtype == NA2D_F16) {
        using T = f16_t;
        if (p.K == 3) return launch_av_mfma_small_t<T, 3>(p, w, y, scale, out, s);
        if (p.K == 5) return launch_av_mfma_small_t<T, 5>(p, w, y, scale, out, s);
        if (p.K == 7) return launch_av_mfma_small_t<T, 7>(p, w, y, scale, out, s);
        NA2D_DISPATCH_K(p.K, return (launch_av_mfma_t<T, K>(p, w, y, scale, out, s)));
    } else if (p.dtype == NA2D_BF16) {
        using T = bf16_t;
        if (p.K == 3) return launch_av_mfma_small_t<T, 3>(p, w, y, scale, out, s);
        if (p.K == 5) return launch_av_mfma_small_t<T, 5>(p, w, y, scale, out, s);
        if (p.K == 7) return launch_av_mfma_small_t<T, 7>(p, w, y, scale, out, s);
        NA2D_DISPATCH_K(p.K, return (launch_av_mfma_t<T, K>(p, w, y, scale, out, s)));
    }
    return hipErrorInvalidValue;
}

}  // namespace na2d
