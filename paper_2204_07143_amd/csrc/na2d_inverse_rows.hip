// Gradients that sum over queries, on the matrix cores, where the query rectangle of a key tile does not fit the
// LDS images of the other two kernels (f16 / bf16): large windows (K >= 11), and maps with an axis so short that a
// tile is seen from both of its ends.  The rectangle is streamed through LDS two rows at a time.
//   out_j = scale * sum over queries i whose window holds j of w[i, slot(i, j)] * x_i
// (grad-v with w = attention weights, x = dout; grad-k with w = ds, x = q; arXiv 2204.07143, Appendix A).
//
// The arithmetic is that of the tile kernel in na2d_inverse_mfma.hip: a 16 x 8 key tile per workgroup, one 4 x 4
// key patch per wave; for a patch
//   out^T[d, key] = sum_pos x^T[d, pos] * Wg[pos, key]
// with x through the transposing LDS read and the weights w[query pos][slot of this lane's key] as 2-byte LDS
// gathers (zero word where query and key do not meet).  At K = 13 one weight row of the tile's query rectangle
// is 11 KB and the rectangle has up to 26 of them: it cannot sit in LDS as a whole.  So the rows pass through
// two small stages, a pair of rows at a time (a pair is the contraction depth of one MFMA: 2 rows x 16 columns),
// the next pair loading while the current one is multiplied; the accumulators of a patch stay in registers for
// the whole rectangle.  A patch is seen from up to K + (K-1)/2 + 3 <= 22 query columns: two column blocks of 16.
// The gather address is row term + column term: the column terms (which window column of query ix holds key
// column jx) are per-lane constants, the row terms (window row of query iy for key row jy) are two compares per
// row.  Rows that see no key of a wave's strip are skipped.  One workgroup barrier per pair of rows.
// A workgroup keeps one tile position and one head and walks a range of the batch; (plane, pair) steps form one
// pipeline, so the first pair of the next plane loads under the last pair of this one.
#include "na2d_kernels.hpp"
#include "na2d_mfma.hpp"
#include "na2d_tile.hpp"

namespace na2d {

// NP: key patches per wave, stacked eight key rows apart (the tile is 16 x 8 NP keys).  With two, a row of the
// query rectangle that passes through LDS serves sixteen key rows instead of eight: at K = 13 the rectangle of a
// tile has 8 NP + 18 rows, 3.25 per key row for NP = 1 and 2.1 for NP = 2, and that is what the kernel's time follows.
template <typename T, int K, int NP = 1>
struct InvRowsCfg {
    static constexpr int R = K / 2;
    static constexpr int PWI = K + R + 3;            // query columns (rows) that can see a 4 x 4 key patch
    static constexpr int NCB = (PWI + 15) / 16;      // 16-column MFMA blocks per row
    static constexpr int STRIPS = 2, WAVES = 4 * STRIPS, TY = 4 * STRIPS * NP;
    static constexpr int RW = kTileX + K - 1 + R;    // columns of a tile's query rectangle (next to one border at most)
    static constexpr int CH = 2;                     // rows per stage
    static constexpr int KK = K * K;
    static constexpr int kThreads = kWave * WAVES;
    static constexpr int KB = Traits<T>::kKeyBytes;
    static constexpr int kXRow = RW * KB;
    // + the reach of the last column block (it starts up to 12 columns into a row) past the last row of the stage
    static constexpr int kXSlack = (12 + 16 * NCB > RW ? 12 + 16 * NCB - RW : 0) * KB;
    static constexpr int kXStage = CH * kXRow + kXSlack;
    static constexpr int kXItems = (RW * (KB / 16) + kWave - 1) / kWave;      // 64-lane loads per x row
    static constexpr int kRowBytes = RW * KK * (int)sizeof(T);
    static constexpr int kRowRegion = mirror_bytes(kRowBytes);                // a weight row, mirrored at its 16-byte phase
    static constexpr int kWItems = (kRowRegion / 16 + kWave - 1) / kWave;     // 64-lane loads per weight row
    static constexpr int kWStage = CH * kRowRegion;
    static constexpr int kStageBytes = kXStage + kWStage + 16;                // + the zero word
    static constexpr int kLdsBytes = 2 * kStageBytes;
    static_assert(kLdsBytes <= 80 * 1024, "two workgroups share the LDS of a compute unit");
    static_assert(16 * NCB >= PWI, "column blocks cover the patch halo");
};

template <typename T, int K, int NP>
__global__ __launch_bounds__(512, 4) void inverse_rows_kernel(const T *__restrict__ w, const T *__restrict__ x, float scale,
                                                              T *__restrict__ out, int H, int W, int heads, int nb,
                                                              int tiles_y, int units, int splits, GridDecode gd, int pitch) {
    // `pitch`: bytes between consecutive positions of x and out (a longer head vector is served one 32-channel
    // slice per launch, x and out pointing at the slice)
    using C = InvRowsCfg<T, K, NP>;
    constexpr int SZ = (int)sizeof(T);
    constexpr int BIG = 1 << 24;   // invalid row / column terms push the sum past the zero word
    extern __shared__ __align__(16) char lds[];

    const int wg = xcd_contiguous_block(blockIdx.x, gridDim.x);
    if (wg >= units * splits) return;
    const WorkItem work = decode_work(wg, heads, tiles_y, splits, gd);
    const int head = work.head;
    const int b_begin = work.b_begin, b_end = work.b_end;
    if (b_begin >= b_end) return;

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int n = lane & 15, g = lane >> 4, ky = n >> 2, kx = n & 3;
    const int lds0 = lds_addr(lds);

    // Everything the loads do not write must hold finite numbers (it meets zero weights only); the zero words too.
    for (int i = tid * 16; i < C::kLdsBytes; i += C::kThreads * 16) *lds_ptr<u32x4>(lds0 + i) = u32x4{0u, 0u, 0u, 0u};

    const int ty0 = work.ty * C::TY, tx0 = work.tx * kTileX;
    const int ty1 = ty0 + C::TY - 1 < H - 1 ? ty0 + C::TY - 1 : H - 1;
    const int tx1 = tx0 + kTileX - 1 < W - 1 ? tx0 + kTileX - 1 : W - 1;
    const int ry0 = inv_first(ty0, H, K), ry1 = inv_last(ty1, H, K);
    const int rx0 = inv_first(tx0, W, K), rx1 = inv_last(tx1, W, K);
    const int nrows = ry1 - ry0 + 1, ncols = rx1 - rx0 + 1;   // ncols <= RW: checked by the host
    const int npairs = (nrows + 1) >> 1;
    const int row_pitch_bytes = W * C::KK * SZ;                // < 2^31: checked by the host
    const int pitch_phase = row_pitch_bytes & 15;
    const int wrow_bytes = ncols * C::KK * SZ;
    const size_t w_bytes = (size_t)nb * heads * H * W * C::KK * SZ;   // size of the weight tensor

    // this wave's patches (one column of the tile, NP of them eight key rows apart) and this lane's keys
    const int strip = wave >> 2, p = patch_of_wave(wave);
    const int px0 = tx0 + 4 * p;
    const int jx = px0 + kx;
    const int oqx = inv_first(px0 < W ? px0 : W - 1, W, K);   // first query column that sees the patches
    // per patch (all wave-uniform, worked out where they are used: nothing is held per patch but its accumulators)
    auto patch_row0 = [&](int np) { return ty0 + 4 * strip + 8 * np; };   // first key row of patch np
    const bool active = patch_row0(0) < H && px0 < W;   // the patches below the first one are inside the map only if it is

    // column terms: block cb, position 4g + r of it is query column oqx + 16 cb + 4g + r
    int colterm[C::NCB][4];
#pragma unroll
    for (int cb = 0; cb < C::NCB; ++cb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ix = oqx + 16 * cb + 4 * g + r;
            const int c = jx - win_start(ix < W ? ix : W - 1, W, K);
            colterm[cb][r] = (active && ix <= rx1 && jx < W && (unsigned)c < (unsigned)K) ? (ix - rx0) * C::KK * SZ + c * SZ : BIG;
        }
    }
    // lane-constant part of the A-operand address inside a stage's x rows (transposing read): inside its group of
    // 16, lane n points at four channels of position 4g + n / 4 of a block and receives the n-th channel of
    // positions 4g .. 4g + 3.  The channels are dealt so that MFMA row m of half hf is channel 8 (m / 4) + 4 hf +
    // m % 4: a lane ends up with the eight consecutive channels 8g .. 8g + 7 of its key, one 16-byte store.
    const int xa_lane = (oqx - rx0 + 4 * g + (n >> 2)) * C::KB + (n & 3) * 16;

    // loads: this lane's x chunks of a row, as byte offsets inside a query row (columns clamped into the map)
    const bool half_dim = pitch < C::KB;   // 16-channel heads: see kHalfDimChunks
    int xcol[C::kXItems];
#pragma unroll
    for (int j = 0; j < C::kXItems; ++j) {
        const int q = j * kWave + lane;
        int xx = rx0 + q / (C::KB / 16);
        xx = xx < W - 1 ? xx : W - 1;
        xcol[j] = q < C::RW * (C::KB / 16) ? xx * pitch + ((q % (C::KB / 16)) & (half_dim ? kHalfDimChunks : 3)) * 16 : -1;
    }
    // Which pairs of the rectangle's rows a patch takes part in (wave-uniform, fixed for the workgroup): pair pr
    // holds rows ry0 + 2 pr and + 1, and patch np is seen from the query rows [inv_first(first key row),
    // inv_last(last key row)].  An empty range for a patch below the map.
    int pair_lo[NP], pair_hi[NP];
#pragma unroll
    for (int np = 0; np < NP; ++np) {
        const int sy = patch_row0(np);
        const int sq0 = inv_first(sy < H ? sy : H - 1, H, K), sq1 = inv_last(sy + 3 < H - 1 ? sy + 3 : H - 1, H, K);
        pair_lo[np] = sy < H ? (sq0 - ry0) >> 1 : 1;
        pair_hi[np] = sy < H ? (sq1 - ry0) >> 1 : 0;
    }
    const int jy0 = ty0 + 4 * strip + ky;   // this lane's key row in patch 0; patch np: + 8 np

    // Loads pair `pr` of plane `b` into stage `par`.  Per row kWItems 64-lane loads of the weight row (mirrored at
    // its 16-byte phase) and kXItems of the x vectors; load j of a row is issued by wave j mod WAVES.  Everything
    // about a row is wave-uniform and 32 bits wide from the plane's base pointers on (a plane of either tensor is
    // shorter than 2 GB: checked by the host), so it runs on the scalar unit in a few instructions.
    constexpr int kRowItems = C::kWItems + C::kXItems;
    // (planes are walked by adding plane_stride_q to the first query of the plane: no 64-bit products of the batch
    // index in the step loop)
    const size_t plane_stride_q = (size_t)heads * H * W;
    auto uniform = [](const char *ptr) {   // (wave-uniform by construction; said again so that a base sits in scalar registers)
        const uint64_t v = (uint64_t)(uintptr_t)ptr;
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return reinterpret_cast<const char *>((uintptr_t)(((uint64_t)hi << 32) | lo));
    };
    auto issue = [&](size_t plane_q, int pr, int par) {
        const char *const xplane = reinterpret_cast<const char *>(x) + plane_q * pitch;
        const size_t wbase = (plane_q + rx0) * C::KK * SZ;   // first weight byte of query row 0 of the rectangle's columns
        const char *const wplane = reinterpret_cast<const char *>(w) + wbase;
        const size_t wleft = w_bytes - wbase;                 // bytes from wplane to the end of the weight tensor
        const int wphase = (int)(wbase & 15);
        const int stage = lds0 + par * C::kStageBytes;
#pragma unroll
        for (int rr = 0; rr < C::CH; ++rr) {
            const int iy = ry0 + 2 * pr + rr;
            if (iy > ry1) break;
            const int wo = iy * row_pitch_bytes;
            const int mis = (wphase + wo) & 15;
            const int nchunks = (mis + wrow_bytes + 15) >> 4;
            const char *src = uniform(wplane + (wo - mis));
            const bool whole = (size_t)(wo - mis) + (size_t)nchunks * 16 <= wleft;   // no chunk crosses the end of the tensor
            const int region = stage + C::kXStage + rr * C::kRowRegion;
            const char *xrow = uniform(xplane + iy * W * pitch);
#pragma unroll
            for (int t = 0; t < (kRowItems + C::WAVES - 1) / C::WAVES; ++t) {
                const int j = wave + t * C::WAVES;
                if (j < C::kWItems) {
                    const int c = j * kWave + lane;
                    if (c < nchunks) {
                        if (whole || (size_t)(wo - mis) + (size_t)(c + 1) * 16 <= wleft) {
                            global_to_lds_16(src, (unsigned)(c * 16), region + j * kWave * 16);
                        } else {   // the chunk that would cross the end of the tensor: element by element
                            for (int e = c * 16; e < mis + wrow_bytes; e += SZ)
                                *lds_ptr<T>(region + e) = *reinterpret_cast<const T *>(src + e);
                        }
                    }
                } else if (j < kRowItems) {
                    // (xcol is indexed by a compile-time constant after unrolling)
#pragma unroll
                    for (int q = 0; q < C::kXItems; ++q)
                        if (q == j - C::kWItems && xcol[q] >= 0)
                            global_to_lds_16(xrow, (unsigned)xcol[q], stage + rr * C::kXRow + q * kWave * 16);
                }
            }
        }
    };

    f32x4 acc[NP][2];
#pragma unroll
    for (int np = 0; np < NP; ++np) acc[np][0] = acc[np][1] = f32x4{0.f, 0.f, 0.f, 0.f};
    // One step: pair `pr` of plane `b`, staged in `par`.
    auto compute = [&](size_t plane_q, int pr, int par) {
        if (active) {
            const int stage = lds0 + par * C::kStageBytes;
            const int zero_addr = stage + C::kXStage + C::kWStage;
            // phase of the rectangle's first row (the low bits of its byte offset: 32-bit arithmetic will do)
            const int mis0 = (int)((((uint32_t)plane_q + (uint32_t)(ry0 * W + rx0)) * (uint32_t)(C::KK * SZ)) & 15u);
            const int iy0 = ry0 + 2 * pr;
            // the pair's two rows (wave-uniform): window start, whether the row exists, where its weights start
            int ws[2], rbase[2];
#pragma unroll
            for (int rr = 0; rr < 2; ++rr) {
                const int iy = iy0 + rr;
                ws[rr] = win_start(iy < H ? iy : H - 1, H, K);
                rbase[rr] = iy <= ry1 ? stage + C::kXStage + rr * C::kRowRegion + ((mis0 + (iy - ry0) * pitch_phase) & 15) : BIG;
            }
#pragma unroll
            for (int np = 0; np < NP; ++np) {
                if (pr < pair_lo[np] || pr > pair_hi[np]) continue;   // no row of the pair sees this patch's strip
                const int jyp = jy0 + 8 * np;   // this lane's key row
                // row terms of the pair's two rows for this lane's key row
                int rowterm[2];
#pragma unroll
                for (int rr = 0; rr < 2; ++rr) {
                    const int a = jyp - ws[rr];
                    rowterm[rr] = (jyp < H && (unsigned)a < (unsigned)K) ? rbase[rr] + a * K * SZ : BIG;
                }
                // all LDS reads of the patch's column blocks are issued before the first block is multiplied (the
                // scheduling fences keep the compiler from sinking them back to their uses, two at a time)
                uint16_t wlo[C::NCB][4], whi[C::NCB][4];
                u32x2 xlo[C::NCB][2], xhi[C::NCB][2];
#pragma unroll
                for (int cb = 0; cb < C::NCB; ++cb) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int rr = u >> 1, r0 = (u & 1) * 2;
                        int a_lo = rowterm[rr] + colterm[cb][r0], a_hi = rowterm[rr] + colterm[cb][r0 + 1];
                        a_lo = a_lo < zero_addr ? a_lo : zero_addr;
                        a_hi = a_hi < zero_addr ? a_hi : zero_addr;
                        wlo[cb][u] = *lds_ptr<uint16_t>(a_lo);
                        whi[cb][u] = *lds_ptr<uint16_t>(a_hi);
                    }
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) {
                        const int a0 = stage + xa_lane + cb * 16 * C::KB + hf * 8;
                        xlo[cb][hf] = lds_read_tr16(a0);
                        xhi[cb][hf] = lds_read_tr16(a0 + C::kXRow);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int cb = 0; cb < C::NCB; ++cb) {
                    uint32_t wv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) wv[u] = (uint32_t)wlo[cb][u] | ((uint32_t)whi[cb][u] << 16);
                    const u32x4 bop = u32x4{wv[0], wv[1], wv[2], wv[3]};
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf)
                        acc[np][hf] = mfma_16x16x32<T>(u32x4{xlo[cb][hf].x, xlo[cb][hf].y, xhi[cb][hf].x, xhi[cb][hf].y}, bop, acc[np][hf]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (pr == npairs - 1) {   // the rectangle is done: this lane's eight channels of its keys
#pragma unroll
                for (int np = 0; np < NP; ++np) {
                    const int jyp = jy0 + 8 * np;
                    if (jyp < H && jx < W && (!half_dim || g < 2)) {
                        char *dst = reinterpret_cast<char *>(out) + (plane_q + (size_t)jyp * W + jx) * pitch + g * 16;
                        uint32_t o[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const int hf = u >> 1, r = 2 * (u & 1);
                            const T lo = from_f32<T>(acc[np][hf][r] * scale), hi = from_f32<T>(acc[np][hf][r + 1] * scale);
                            o[u] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
                        }
                        store16_stream(dst, u32x4{o[0], o[1], o[2], o[3]});   // channels 8g .. 8g + 7
                    }
                    acc[np][0] = acc[np][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
    };

    workgroup_sync();   // the zero fill is done before the first loads land
    size_t plane_q = ((size_t)b_begin * heads + head) * H * W;   // first query of plane b
    issue(plane_q, 0, 0);
    int b = b_begin, pr = 0, par = 0;
    while (b < b_end) {
        wait_global_loads();   // this step's rows have landed
        workgroup_sync();       // ... for every wave, and nobody still reads the other stage
        // (the walk is wave-uniform; said again so that its arithmetic stays on the scalar unit)
        b = __builtin_amdgcn_readfirstlane(b);
        pr = __builtin_amdgcn_readfirstlane(pr);
        par = __builtin_amdgcn_readfirstlane(par);
        const bool last = pr + 1 == npairs;   // the last pair of a plane: the next plane's first pair loads under it
        const size_t next_q = last ? plane_q + plane_stride_q : plane_q;
        if (!last || b + 1 < b_end) issue(next_q, last ? 0 : pr + 1, par ^ 1);
        compute(plane_q, pr, par);
        plane_q = next_q;
        b += last ? 1 : 0;
        pr = last ? 0 : pr + 1;
        par ^= 1;
    }
}

template <typename T, int K, int NP>
static hipError_t launch_inverse_rows_np(const Problem &p, const void *w, const void *x, float scale, void *out,
                                         hipStream_t s) {
    using C = InvRowsCfg<T, K, NP>;
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    const UnitSplit us = unit_split(tiles_x, tiles_y, p.heads, p.B);
    auto kern = inverse_rows_kernel<T, K, NP>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    for (int sl = 0; sl < (p.D + kHeadDim - 1) / kHeadDim; ++sl) {   // one launch per 32-channel slice of the head vector (a 16-channel head is half a slice)
        hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(us.units * us.splits)), dim3(C::kThreads), C::kLdsBytes, s,
                           static_cast<const T *>(w), static_cast<const T *>(x) + sl * kHeadDim, scale,
                           static_cast<T *>(out) + sl * kHeadDim, p.H, p.W, p.heads, p.B, tiles_y, us.units, us.splits, us.gd,
                           p.D * (int)sizeof(T));
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Several patches per wave where the windows are large (the rectangle's K + R - 1 extra rows then weigh most) and
// the map has 8-row tiles to merge: grad-v / grad-k at B=64, 56 x 56, f16 take 153 / 120 / 96 us (K = 11) and
// 194 / 146 / 119 us (K = 13) with one / two / four patches per wave.
template <typename T, int K>
static hipError_t launch_inverse_rows_t(const Problem &p, const void *w, const void *x, float scale, void *out,
                                        hipStream_t s) {
    if constexpr (K >= 9) {   // (eight patches per wave, a whole column of a 56-row map, no longer fit 128 registers)
        if (p.H > 24) return launch_inverse_rows_np<T, K, 4>(p, w, x, scale, out, s);
        if (p.H > 8) return launch_inverse_rows_np<T, K, 2>(p, w, x, scale, out, s);
    }
    return launch_inverse_rows_np<T, K, 1>(p, w, x, scale, out, s);
}

// Every tile's query rectangle must be at most RW columns wide (rows are streamed, any number of them), and a
// patch must be seen from at most 16 NCB columns: both hold for every map with K <= min(H, W) (a tile next to both
// ends of a short axis has at most W <= 2K + 2 columns).  Checked anyway.
bool inverse_rows_supported(const Problem &p) {
    if ((p.D % kHeadDim != 0 && p.D != kHalfDim) || p.dtype == NA2D_F32) return false;
    const int K = p.K, RW = kTileX + K - 1 + K / 2, NCOL = 16 * ((K + K / 2 + 3 + 15) / 16);
    // offsets inside a plane of the weights and of x / out as 32-bit byte counts
    if ((int64_t)p.H * p.W * K * K * 4 >= (int64_t)1 << 31 || (int64_t)p.H * p.W * p.D * 4 >= (int64_t)1 << 31) return false;
    for (int tx0 = 0; tx0 < p.W; tx0 += kTileX) {
        const int tx1 = tx0 + kTileX - 1 < p.W - 1 ? tx0 + kTileX - 1 : p.W - 1;
        if (inv_last(tx1, p.W, K) - inv_first(tx0, p.W, K) + 1 > RW) return false;
        for (int px0 = tx0; px0 <= tx1; px0 += 4) {
            const int px1 = px0 + 3 < p.W - 1 ? px0 + 3 : p.W - 1;
            if (inv_last(px1, p.W, K) - inv_first(px0, p.W, K) + 1 > NCOL) return false;
        }
    }
    return true;
}

hipError_t launch_inverse_rows(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s) {
#define NA2D_INVW_K(TT)                                                               \
    switch (p.K) {                                                                    \
        case 3: return launch_inverse_rows_t<TT, 3>(p, w, x, scale, out, s);          \
        case 5: return launch_inverse_rows_t<TT, 5>(p, w, x, scale, out, s);          \
        case 7: return launch_inverse_rows_t<TT, 7>(p, w, x, scale, out, s);          \
        case 9: return launch_inverse_rows_t<TT, 9>(p, w, x, scale, out, s);          \
        case 11: return launch_inverse_rows_t<TT, 11>(p, w, x, scale, out, s);        \
        case 13: return launch_inverse_rows_t<TT, 13>(p, w, x, scale, out, s);        \
        default: return hipErrorInvalidValue;                                         \
    }
    if (p.dtype == NA2D_F16) { NA2D_INVW_K(f16_t) }
    if (p.dtype == NA2D_BF16) { NA2D_INVW_K(bf16_t) }
#undef NA2D_INVW_K
    return hipErrorInvalidValue;
}

}  // namespace na2d
