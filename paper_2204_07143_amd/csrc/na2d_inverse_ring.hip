// Gradients that sum over queries, on the matrix cores, walking down a column of key tiles (f16 / bf16,
// K <= 7):
//   out_j = scale * sum over queries i whose window holds j of w[i, slot(i, j)] * x_i
// (grad-v with w = attention weights, x = dout; grad-k with w = ds, x = q; arXiv 2204.07143, Appendix A).
//
// The arithmetic is that of the tile kernel in na2d_inverse_mfma.hip (4 x 4 key patches, one per wave, a
// block of 16 query positions per row of the query rectangle, weights gathered through row + column
// address terms, x through the transposing LDS read).  What differs is how the query rectangle reaches
// LDS.  A 16 x 8 key tile is seen from 8 + K-1 query rows, and vertically adjacent tiles share K-1 of them:
// a workgroup therefore owns one column of tiles of one plane and keeps the query rows (their weight rows
// and their x vectors) in a ring of 2*8 + K-1 row slots, slot = row mod ring size.  Per tile only the 8
// rows that are new are loaded (direct-to-LDS), and they are loaded while the previous tile is computed:
// 43 % fewer bytes through the L2-to-LDS path that bounds the tile kernel, overlapped with the gathers.
// Neighbouring workgroups take neighbouring columns of the same plane at the same time, so the query
// columns that adjacent columns of tiles share are fetched from HBM once.
#include "na2d_kernels.hpp"
#include "na2d_mfma.hpp"
#include "na2d_tile.hpp"

namespace na2d {

typedef int i32x2 __attribute__((ext_vector_type(2)));

template <typename T, int K>
struct InvRingCfg {
    static constexpr int R = K / 2;
    static constexpr int PWI = K + R + 3;          // query-halo side of a 4 x 4 key patch
    static constexpr int NBLK = PWI + (PWI & 1);   // halo rows, padded to whole pairs
    static constexpr int NPAIR = NBLK / 2;
    static constexpr int STRIPS = 2, WAVES = 4 * STRIPS, TY = 4 * STRIPS;
    static constexpr int RH = TY + K - 1;          // query rows that see a tile (tiles next to at most the near border)
    static constexpr int RW = kTileX + K - 1;      // ... and columns
    static constexpr int NR = RH + TY;             // ring slots: the rows of a tile and the new rows of the next one
    static constexpr int KK = K * K;
    static constexpr int kThreads = kWave * WAVES;
    static constexpr int KB = Traits<T>::kKeyBytes;
    static constexpr int kXRow = RW * KB;                         // x vectors of one query row, natural layout
    // + the reach of a 16-wide block (it starts up to 12 columns into a row) past the last slot
    static constexpr int kXBytes = NR * kXRow + (28 - RW) * KB;
    static constexpr int kXItems = (RW * (KB / 16) + kWave - 1) / kWave;   // 64-lane loads per x row
    static constexpr int kRowBytes = RW * KK * (int)sizeof(T);
    static constexpr int kRowRegion = mirror_bytes(kRowBytes);    // a weight row, mirrored at its 16-byte phase
    static constexpr int kWItems = (kRowRegion / 16 + kWave - 1) / kWave;   // 64-lane loads per weight row
    static constexpr int kWBytes = NR * kRowRegion;
    static constexpr int kColEntries = 4 * 4 * 4 * 4;             // [patch][g][kx][r]
    static constexpr int kRowEntries = STRIPS * 4 * 16;           // [strip][ky][b], b padded to 16: a lane reads its terms a pair at a time
    static_assert(NBLK <= 16, "sixteen row terms per lane");
    // two row-term tables: the next tile's is written while this tile's is read
    static constexpr int kLdsBytes = kXBytes + kWBytes + 16 + (kColEntries + 2 * kRowEntries) * 4;
    static_assert(kLdsBytes <= 80 * 1024, "two workgroups share the LDS of a compute unit");
    static constexpr int kMaxNew = RH;                            // rows loaded at once: the first tile's
    static constexpr int kRowsPerWave = (kMaxNew + WAVES - 1) / WAVES;
};

template <typename T, int K>
__global__ __launch_bounds__(512, 4) void inverse_ring_kernel(const T *__restrict__ w, const T *__restrict__ x, float scale,
                                                              T *__restrict__ out, int H, int W, int tiles_x, int tiles_y,
                                                              int nplanes, int nseg, FastDiv by_tiles_x, FastDiv by_nseg,
                                                              int pitch) {
    // `pitch`: bytes between consecutive positions of x and out (a longer head vector is served one 32-channel
    // slice per launch, x and out pointing at the slice)
    using C = InvRingCfg<T, K>;
    constexpr int SZ = (int)sizeof(T);
    constexpr int BIG = 1 << 24;   // invalid row / column terms push the sum past the zero word
    extern __shared__ __align__(16) char lds[];

    // workgroup -> (plane, segment of the column, column); the column index runs fastest.  A column is cut into
    // nseg segments of consecutive tiles when there are too few planes x columns to fill the chip.
    const int wg = xcd_contiguous_block(blockIdx.x, gridDim.x);
    if (wg >= nplanes * tiles_x * nseg) return;
    const int wq = fdiv(wg, by_tiles_x), tix = wg - wq * tiles_x, plane = fdiv(wq, by_nseg), seg = wq - plane * nseg;
    const int t_begin = fdiv(seg * tiles_y, by_nseg), t_end = fdiv((seg + 1) * tiles_y, by_nseg);
    if (t_begin >= t_end) return;

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int n = lane & 15, g = lane >> 4, ky = n >> 2, kx = n & 3;
    const int lds0 = lds_addr(lds);
    const int x0 = lds0;                               // x ring
    const int w0 = lds0 + C::kXBytes;                  // weight ring
    const int zero_addr = w0 + C::kWBytes;             // a zero word above every valid gather address
    const int tbl_col = zero_addr + 16, tbl_row = tbl_col + C::kColEntries * 4;

    // Everything the loads do not write must hold finite numbers (it meets zero weights only).
    for (int i = tid * 16; i < C::kLdsBytes; i += C::kThreads * 16) *lds_ptr<u32x4>(lds0 + i) = u32x4{0u, 0u, 0u, 0u};

    const int tx0 = tix * kTileX;
    const int tx1 = tx0 + kTileX - 1 < W - 1 ? tx0 + kTileX - 1 : W - 1;
    const int rx0 = inv_first(tx0, W, K), rx1 = inv_last(tx1, W, K);
    const int ncols = rx1 - rx0 + 1;   // <= RW: checked by the host
    const size_t plane_q = (size_t)plane * H * W;
    const size_t w_bytes = (size_t)nplanes * H * W * C::KK * SZ;   // size of the weight tensor
    const int row_pitch_bytes = W * C::KK * SZ;                    // < 2^31: checked by the host
    const size_t wbase = (plane_q + rx0) * C::KK * SZ;             // first weight byte of query row 0 of the rectangle's columns
    const int wrow_bytes = ncols * C::KK * SZ;

    // x loads of a row: this lane's chunks, as byte offsets inside a query row (columns clamped into the map)
    const bool half_dim = pitch < C::KB;   // 16-channel heads: see kHalfDimChunks
    int xcol[C::kXItems];
#pragma unroll
    for (int j = 0; j < C::kXItems; ++j) {
        const int q = j * kWave + lane;
        int xx = rx0 + q / (C::KB / 16);
        xx = xx < W - 1 ? xx : W - 1;
        xcol[j] = q < C::RW * (C::KB / 16) ? xx * pitch + ((q % (C::KB / 16)) & (half_dim ? kHalfDimChunks : 3)) * 16 : -1;
    }
    // Loads the query rows [r_begin, r_end) into their ring slots: row r_begin + wave, + WAVES, ... per wave.  All of a
    // row's address arithmetic is wave-uniform and 32 bits wide from the plane's base pointers on (a plane of either
    // tensor is shorter than 2 GB: checked by the host), so it runs on the scalar unit in a few instructions.
    const char *const xplane = reinterpret_cast<const char *>(x) + plane_q * pitch;
    const char *const wplane = reinterpret_cast<const char *>(w) + wbase;
    const size_t wleft = w_bytes - wbase;   // bytes from wplane to the end of the weight tensor
    const int wphase0 = (int)(wbase & 15);  // 16-byte phase of row iy: (wphase0 + iy * row_pitch_bytes) & 15
    auto load_rows = [&](int r_begin, int r_end) {
#pragma unroll
        for (int u = 0; u < C::kRowsPerWave; ++u) {
            const int iy = r_begin + wave + u * C::WAVES;
            if (iy >= r_end) break;
            const int slot = iy % C::NR;
            // x vectors
            const char *xrow = xplane + iy * W * pitch;
#pragma unroll
            for (int j = 0; j < C::kXItems; ++j)
                if (xcol[j] >= 0) global_to_lds_16(xrow, (unsigned)xcol[j], x0 + slot * C::kXRow + j * kWave * 16);
            // weight row, mirrored at its 16-byte phase: one 16-byte chunk per lane; the chunks at the two ends also
            // bring in bytes of the neighbouring rows, which nothing reads.  Only in a row whose last chunk would
            // cross the end of the tensor is that chunk copied element by element.
            const int wo = iy * row_pitch_bytes;
            const int mis = (wphase0 + wo) & 15;
            const int nchunks = (mis + wrow_bytes + 15) >> 4;
            const char *src = wplane + (wo - mis);   // (wplane - mis stays inside the allocation: mis <= the phase of wplane + wo)
            const int region = w0 + slot * C::kRowRegion;
            if ((size_t)(wo - mis) + (size_t)nchunks * 16 <= wleft) {
#pragma unroll
                for (int j = 0; j < C::kWItems; ++j) {
                    const int c = j * kWave + lane;
                    if (c < nchunks) global_to_lds_16(src, (unsigned)(c * 16), region + j * kWave * 16);
                }
            } else {
#pragma unroll
                for (int j = 0; j < C::kWItems; ++j) {
                    const int c = j * kWave + lane;
                    if (c < nchunks) {
                        if ((size_t)(wo - mis) + (size_t)(c + 1) * 16 <= wleft) {
                            global_to_lds_16(src, (unsigned)(c * 16), region + j * kWave * 16);
                        } else {
                            for (int e = c * 16; e < mis + wrow_bytes; e += SZ)
                                *lds_ptr<T>(region + e) = *reinterpret_cast<const T *>(src + e);
                        }
                    }
                }
            }
        }
    };

    // lane-constant part of the A-operand address (transposing read): inside its group of 16, lane n points at
    // four channels of position 4g + n / 4 of a block and receives the n-th channel of positions 4g .. 4g + 3.  The
    // channels are dealt so that MFMA row m of half hf is channel 8 (m / 4) + 4 hf + m % 4: a lane then ends up
    // with the eight consecutive channels 8g .. 8g + 7 of its key, one 16-byte store.
    const int strip = wave >> 2, p = patch_of_wave(wave);
    const int px0 = tx0 + 4 * p;
    const int oqx = inv_first(px0 < W ? px0 : W - 1, W, K);   // first query column that sees the patch
    const int xa_lane = x0 + (oqx - rx0 + 4 * g + (n >> 2)) * C::KB + (n & 3) * 16;
    const int jx = px0 + kx;
    const int pitch_phase = row_pitch_bytes & 15;   // phase of row iy: (wphase0 + iy * pitch_phase) & 15

    workgroup_sync();   // the zero fill is done
    // column terms: the same for every tile of the column
    for (int e = tid; e < C::kColEntries; e += C::kThreads) {
        const int r = e & 3, kxe = (e >> 2) & 3, ge = (e >> 4) & 3, pe = e >> 6;
        const int pp0 = tx0 + 4 * pe, jxe = pp0 + kxe;
        const int ix = inv_first(pp0 < W ? pp0 : W - 1, W, K) + 4 * ge + r;
        const int c = jxe - win_start(ix < W ? ix : W - 1, W, K);
        int term = BIG;
        if (pp0 < W && ix <= rx1 && jxe < W && (unsigned)c < (unsigned)K) term = (ix - rx0) * C::KK * SZ + c * SZ;
        *lds_ptr<int>(tbl_col + e * 4) = term;
    }
    // Row terms of tile t into table (t - t_begin) & 1, one entry per thread: the address of the weight that query
    // (iy, ix) gives key (jy, jx) is rowterm(iy, jy) + colterm(ix, jx); a pair that does not meet gets BIG.
    auto build_rowterms = [&](int t) {
        const int e = tid;
        if (e < C::kRowEntries) {
            const int ty0 = t * C::TY;
            const int ty1 = ty0 + C::TY - 1 < H - 1 ? ty0 + C::TY - 1 : H - 1;
            const int ry1 = inv_last(ty1, H, K);   // last query row of the tile's rectangle
            const int bb = e & 15, kye = (e >> 4) & 3, st = e >> 6;
            const int sy = ty0 + 4 * st, jyy = sy + kye;
            const int iy = inv_first(sy < H ? sy : H - 1, H, K) + bb;   // halo row bb of the strip
            const int a = jyy - win_start(iy < H ? iy : H - 1, H, K);
            int term = BIG;
            if (bb < C::PWI && iy <= ry1 && jyy < H && (unsigned)a < (unsigned)K)
                term = w0 + (iy % C::NR) * C::kRowRegion + ((wphase0 + iy * pitch_phase) & 15) + a * K * SZ;
            *lds_ptr<int>(tbl_row + (((t - t_begin) & 1) * C::kRowEntries + e) * 4) = term;
        }
    };
    // the rows and the row terms of the segment's first tile
    {
        const int ty0 = t_begin * C::TY;
        const int ty1 = ty0 + C::TY - 1 < H - 1 ? ty0 + C::TY - 1 : H - 1;
        load_rows(inv_first(ty0, H, K), inv_last(ty1, H, K) + 1);
    }
    build_rowterms(t_begin);
    wait_global_loads();
    workgroup_sync();
    int colterm[4];
    {
        const u32x4 ct = *lds_ptr<u32x4>(tbl_col + ((p * 4 + g) * 4 + kx) * 16);
        colterm[0] = (int)ct.x;
        colterm[1] = (int)ct.y;
        colterm[2] = (int)ct.z;
        colterm[3] = (int)ct.w;
    }

    for (int t = t_begin; t < t_end; ++t) {
        const int ty0 = t * C::TY;
        const int ty1 = ty0 + C::TY - 1 < H - 1 ? ty0 + C::TY - 1 : H - 1;
        const int ry1 = inv_last(ty1, H, K);   // last query row of this tile's rectangle (the first is inv_first(ty0))
        // the next tile's new rows go to the slots that the tile before this one has left, its row terms to the
        // table that tile read: both are ordered against their last readers by the barrier that ended that tile
        if (t + 1 < t_end) {
            const int ny1 = ty1 + C::TY < H - 1 ? ty1 + C::TY : H - 1;
            load_rows(ry1 + 1, inv_last(ny1, H, K) + 1);
            build_rowterms(t + 1);
        }

        const int sy0 = ty0 + 4 * strip;   // first key row of this wave's strip
        if (sy0 < H && px0 < W) {
            const int jy = sy0 + ky;
            const int oqy = inv_first(sy0, H, K);   // first query row of the strip's halo
            // this lane's row terms, halo row b at rt_at + 4 b: read a pair at a time, one pair ahead of its use
            const int rt_at = tbl_row + (((t - t_begin) & 1) * C::kRowEntries + (strip * 4 + ky) * 16) * 4;
            f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
            // Halo rows of the strip that some key row of it is seen from: oqy .. the last query row that sees the
            // strip's last key row.  They are taken in pairs (one MFMA is two rows deep); the pair loop is free of
            // branches, so that the gathers of one pair are in flight while the pair before it is multiplied, and
            // comes in three lengths of which a wave picks the shortest that covers its rows.
            const int sy1 = sy0 + 3 < H - 1 ? sy0 + 3 : H - 1;
            const int npairs = (inv_last(sy1, H, K) - oqy + 2) >> 1;   // <= NPAIR: the host has checked the map
            auto pairs = [&](auto npc) {
                constexpr int NP = decltype(npc)::value;
                // What a pair needs from LDS: eight gathered weights (the B operand: two halo rows x four columns
                // per lane) and four transposing reads of x (the A operands of the two channel halves).  The reads
                // of pair pb + 1 are issued before pair pb is multiplied, and the scheduling fences keep the
                // compiler from sinking them back to their uses: a wave has twelve reads in flight behind every
                // pair of MFMAs instead of waiting for each pair's reads in turn.
                uint16_t wlo[2][4], whi[2][4];
                u32x2 xlo[2][2], xhi[2][2];
                int slot = oqy % C::NR;   // ring slot of halo row 0; the following rows follow, wrapping
                i32x2 rt_next = *lds_ptr<i32x2>(rt_at);
                auto fetch = [&](int pb, int st) {
                    const int s_lo = slot, s_hi = slot + 1 < C::NR ? slot + 1 : 0;
                    slot = s_hi + 1 < C::NR ? s_hi + 1 : 0;
                    const int rowterm[2] = {rt_next.x, rt_next.y};
                    if (pb + 1 < NP) rt_next = *lds_ptr<i32x2>(rt_at + (pb + 1) * 8);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int bb = u >> 1;
                        const int r0 = (u & 1) * 2;
                        int a_lo = rowterm[bb] + colterm[r0], a_hi = rowterm[bb] + colterm[r0 + 1];
                        a_lo = a_lo < zero_addr ? a_lo : zero_addr;
                        a_hi = a_hi < zero_addr ? a_hi : zero_addr;
                        wlo[st][u] = *lds_ptr<uint16_t>(a_lo);
                        whi[st][u] = *lds_ptr<uint16_t>(a_hi);
                    }
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) {
                        xlo[st][hf] = lds_read_tr16(xa_lane + s_lo * C::kXRow + hf * 8);
                        xhi[st][hf] = lds_read_tr16(xa_lane + s_hi * C::kXRow + hf * 8);
                    }
                };
                fetch(0, 0);
#pragma unroll
                for (int pb = 0; pb < NP; ++pb) {
                    const int st = pb & 1;
                    if (pb + 1 < NP) fetch(pb + 1, st ^ 1);
                    __builtin_amdgcn_sched_barrier(0);
                    uint32_t wv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) wv[u] = (uint32_t)wlo[st][u] | ((uint32_t)whi[st][u] << 16);
                    const u32x4 bop = u32x4{wv[0], wv[1], wv[2], wv[3]};
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf)
                        acc[hf] = mfma_16x16x32<T>(u32x4{xlo[st][hf].x, xlo[st][hf].y, xhi[st][hf].x, xhi[st][hf].y}, bop, acc[hf]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            if (!kProbeMemoryOnly) {   // (measurement build: zeros are stored)
                if (npairs <= C::NPAIR - 2) pairs(IntC<(C::NPAIR > 2 ? C::NPAIR - 2 : 1)>{});
                else if (npairs == C::NPAIR - 1) pairs(IntC<C::NPAIR - 1>{});
                else pairs(IntC<C::NPAIR>{});
            }
            if (jy < H && jx < W && (!half_dim || g < 2)) {
                char *dst = reinterpret_cast<char *>(out) + (plane_q + (size_t)jy * W + jx) * pitch + g * 16;
                uint32_t o[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int hf = u >> 1, r = 2 * (u & 1);
                    const T lo = from_f32<T>(acc[hf][r] * scale), hi = from_f32<T>(acc[hf][r + 1] * scale);
                    o[u] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
                }
                store16_stream(dst, u32x4{o[0], o[1], o[2], o[3]});   // channels 8g .. 8g + 7
            }
        }
        wait_global_loads();   // the next tile's rows have landed
        workgroup_sync();       // ... for every wave; this tile's rows and row terms are no longer read
    }
}

template <typename T, int K>
static hipError_t launch_inverse_ring_t(const Problem &p, const void *w, const void *x, float scale, void *out,
                                        hipStream_t s) {
    using C = InvRingCfg<T, K>;
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    // segments per column: enough workgroups for the chip's 512 slots, at least two tiles each where possible
    int nseg = 512 / (p.planes() * tiles_x);
    nseg = nseg < 1 ? 1 : (nseg > (tiles_y + 1) / 2 ? (tiles_y + 1) / 2 : nseg);
    const int nwg = p.planes() * tiles_x * nseg;
    auto kern = inverse_ring_kernel<T, K>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    for (int sl = 0; sl < (p.D + kHeadDim - 1) / kHeadDim; ++sl) {   // one launch per 32-channel slice of the head vector (a 16-channel head is half a slice)
        hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(nwg)), dim3(C::kThreads), C::kLdsBytes, s, static_cast<const T *>(w),
                           static_cast<const T *>(x) + sl * kHeadDim, scale, static_cast<T *>(out) + sl * kHeadDim, p.H, p.W,
                           tiles_x, tiles_y, p.planes(), nseg, make_fastdiv(tiles_x), make_fastdiv(nseg),
                           p.D * (int)sizeof(T));
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    return hipSuccess;
}

// The ring holds 8 + K-1 rows per tile: every tile's query rectangle must fit that (and 16 + K-1 columns), which
// excludes maps with a tile next to the far border whose clamped queries reach further (the tile kernel takes those).
bool inverse_ring_supported(const Problem &p) {
    if ((p.D % kHeadDim != 0 && p.D != kHalfDim) || p.dtype == NA2D_F32 || p.K > 7) return false;
    const int K = p.K, TY = 8;
    // a 4 x 4 key patch seen from both clamped ends of an axis at once (axes of at most 2K + 2 positions) has
    // more than K + R + 3 query rows or columns: one MFMA block per row no longer covers it
    if ((p.H < p.W ? p.H : p.W) <= 2 * K + 2) return false;
    // row offsets inside a plane are 32-bit
    if ((size_t)p.H * p.W * K * K * p.elem_bytes() >= ((size_t)1 << 31) || (size_t)p.H * p.W * p.D * p.elem_bytes() >= ((size_t)1 << 31))
        return false;
    for (int ty0 = 0; ty0 < p.H; ty0 += TY) {
        const int ty1 = ty0 + TY - 1 < p.H - 1 ? ty0 + TY - 1 : p.H - 1;
        if (inv_last(ty1, p.H, K) - inv_first(ty0, p.H, K) + 1 > TY + K - 1) return false;
    }
    for (int tx0 = 0; tx0 < p.W; tx0 += kTileX) {
        const int tx1 = tx0 + kTileX - 1 < p.W - 1 ? tx0 + kTileX - 1 : p.W - 1;
        if (inv_last(tx1, p.W, K) - inv_first(tx0, p.W, K) + 1 > kTileX + K - 1) return false;
    }
    return true;
}

hipError_t launch_inverse_ring(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s) {
#define NA2D_INVR_K(TT)                                                               \
    switch (p.K) {                                                                    \
        case 3: return launch_inverse_ring_t<TT, 3>(p, w, x, scale, out, s);          \
        case 5: return launch_inverse_ring_t<TT, 5>(p, w, x, scale, out, s);          \
        case 7: return launch_inverse_ring_t<TT, 7>(p, w, x, scale, out, s);          \
        default: return hipErrorInvalidValue;                                         \
    }
    if (p.dtype == NA2D_F16) { NA2D_INVR_K(f16_t) }
    if (p.dtype == NA2D_BF16) { NA2D_INVR_K(bf16_t) }
#undef NA2D_INVR_K
    return hipErrorInvalidValue;
}

}  // namespace na2d
