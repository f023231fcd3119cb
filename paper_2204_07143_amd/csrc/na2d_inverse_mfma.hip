// Gradients that sum over queries, on the matrix cores (f16 / bf16, K <= 9), one key tile per step:
//   out_j = scale * sum over queries i whose window holds j of w[i, slot(i, j)] * x_i
// (grad-v with w = attention weights, x = dout; grad-k with w = ds, x = q; arXiv 2204.07143,
// Appendix A).  Gathered per key over its inverse neighbourhood: no atomics, fixed order.
//
// A workgroup owns a 16 x 8 key tile position and one head and walks a range of the batch (eight waves, one
// 4 x 4 key patch each).  The queries that see any key of the tile form a rectangle of at most
// (8 + K-1 + R) x (16 + K-1 + R) positions (R = (K-1)/2; the + R only matters next to the far border, where
// clamped queries reach further).  Per plane the rectangle's weight rows (mirrored at their 16-byte phase)
// and x vectors (natural layout) reach LDS by direct loads.  For one patch
//   out^T[d, key] = sum_pos x^T[d, pos] * Wg[pos, key]
// runs over the rows of the rectangle that see the patch, one row (16 positions) per MFMA block:
//   A operand: x through the transposing LDS read (4 consecutive query positions of one channel);
//   B operand: the weights w[query pos][slot of this lane's key], 2-byte LDS gathers whose
//              address is the sum of a per-lane row term (depends on the halo row and the lane's
//              key row) and a per-lane column term (depends on the 4 halo columns of the lane and
//              its key column); invalid combinations read a zero word.  Both kinds of terms are built
//              once per tile position into small LDS tables (one entry per thread);
//   halo rows that no key row of the strip is seen from are skipped (wave-uniform mask).
// Each lane ends up with 8 consecutive channels of its own key: scale, convert, one 16-byte global store.
// For K <= 7 on maps without far-border tiles the column-walking kernel (na2d_inverse_ring.hip) is used
// instead; this one serves K = 9 and the remaining maps.
#include "na2d_kernels.hpp"
#include "na2d_mfma.hpp"
#include "na2d_tile.hpp"

namespace na2d {

// COMPACT: LDS images sized for the rectangle of a tile away from the ragged end of the map,
// (TY + K-1) x (16 + K-1) positions; three workgroups then share a CU.  The launcher uses it when every
// tile of the map fits (always the case when H and W are multiples of the tile, e.g. 56 x 56).
// CHUNK: 0, or the rows of the rectangle that LDS holds at a time.  At K = 9 a whole rectangle (up to 20 rows of
// 28 positions: 129 KB) leaves room for one workgroup per compute unit, which then loads and multiplies in turn with
// nothing to overlap either with; in chunks of 8 or 10 rows two or three workgroups fit, and one computes while
// another loads.  A patch's accumulators stay in registers across the chunks of a plane.
template <typename T, int K, int STRIPS, int PPW, bool COMPACT, int CHUNK = 0>
struct InvMfmaCfg {
    static constexpr int R = K / 2;
    static constexpr int PWI = K + R + 3;          // query-halo side of a 4 x 4 key patch
    static_assert(PWI <= 16, "one MFMA block per query-halo row needs K + R + 3 <= 16");
    static constexpr int NBLK = PWI + (PWI & 1);   // halo rows, padded to whole pairs
    static constexpr int NPAIR = NBLK / 2;
    static_assert(PPW == 1 || PPW == 2 || PPW == 4, "a strip of four patches is split evenly over its waves");
    static constexpr int NWPS = 4 / PPW;              // waves per strip
    static constexpr int WAVES = STRIPS * NWPS;
    static constexpr int TY = 4 * STRIPS;
    static constexpr int RH = COMPACT ? TY + K - 1 : 4 * (STRIPS - 1) + NBLK;   // rows of the tile's query rectangle held in LDS
    static constexpr int RW = COMPACT ? kTileX + K - 1 : kTileX + K - 1 + R;  // columns that hold data
    static constexpr int LH = CHUNK ? CHUNK : RH;       // rows that LDS holds at a time
    static constexpr int NCH = (RH + LH - 1) / LH;      // chunks of a rectangle, at most
    // a pair of rows (one MFMA deep) must not straddle two chunks: chunks and the first row of every strip's halo
    // (multiples of 4 minus R, or 0) are even
    static_assert(CHUNK == 0 || (CHUNK % 2 == 0 && R % 2 == 0), "row pairs inside one chunk");
    static constexpr int KK = K * K;
    static constexpr int kThreads = kWave * WAVES;
    using XHalo = HaloDma<T, LH, RW, WAVES>;
    // the x rectangle in its natural layout, plus the positions an operand block can reach past it: a
    // 16-wide block that starts up to 12 columns into the row after the last one (they meet zero weights)
    static constexpr int kXBytes = XHalo::kBytes + 28 * Traits<T>::kKeyBytes;
    static constexpr int kRowBytes = RW * KK * (int)sizeof(T);
    static constexpr int kRowRegion = mirror_bytes(kRowBytes);
    static constexpr int kWBytes = LH * kRowRegion;
    // gather-address tables of the current tile: column terms [patch][g][kx][r], row terms [strip][b][ky]
    static constexpr int kColEntries = 4 * 4 * 4 * 4;
    static constexpr int kRowEntries = STRIPS * NBLK * 4;
    static constexpr int kTblBytes = (kColEntries + kRowEntries) * 4;
    static constexpr int kLdsBytes = kXBytes + kWBytes + 16 + kTblBytes;   // + the zero word
    // workgroups that share a CU (LDS is handed out in 512-byte units) and the waves per SIMD that gives
    static constexpr int kLdsAlloc = (kLdsBytes + 511) / 512 * 512;
    static constexpr int kWgCap = COMPACT && CHUNK == 0 ? 3 : 2;   // (three leave a lane 80 registers: not enough with chunk tables)
    static constexpr int kWgPerCu = (160 * 1024) / kLdsAlloc < kWgCap ? (160 * 1024) / kLdsAlloc : kWgCap;
    static_assert(kWgPerCu >= 1, "tile does not fit the 160 KB LDS of a CDNA4 compute unit");
    static constexpr int kWavesPerSimd = kWgPerCu * WAVES / 4;
    // chunk grid of the weight-row copy
    static constexpr int kRowChunks = kRowRegion / 16;
};

template <typename T, int K, int STRIPS, int PPW, bool COMPACT, int CHUNK>
__global__ __launch_bounds__(kWave *STRIPS *(4 / PPW), (InvMfmaCfg<T, K, STRIPS, PPW, COMPACT, CHUNK>::kWavesPerSimd)) void inverse_mfma_kernel(const T *__restrict__ w, const T *__restrict__ x,
                                                                       float scale, T *__restrict__ out, int H, int W,
                                                                       int heads, int nb, int tiles_y, int units, int splits, GridDecode gd,
                                                                       int pitch) {
    // `pitch`: bytes between consecutive positions of x and out (a longer head vector is served one 32-channel
    // slice per launch, x and out pointing at the slice)
    using C = InvMfmaCfg<T, K, STRIPS, PPW, COMPACT, CHUNK>;
    using XHalo = typename C::XHalo;
    constexpr int WAVES = C::WAVES;
    constexpr int SZ = (int)sizeof(T);
    constexpr int BIG = 1 << 24;   // invalid row / column terms push the sum past the zero word
    extern __shared__ __align__(16) char lds[];

    // A workgroup keeps one tile position and one head and walks a range of the batch: the tile's
    // geometry, the column terms and (while the 16-byte phase of the weight rows stays the same) the row
    // terms are worked out once.  Neighbouring workgroups take neighbouring positions (numbered down the
    // columns of the map) of the same planes at the same time, so the query rows and columns that
    // adjacent tiles share are fetched from memory once and found in the L2 cache by the others.
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
    const int w0 = lds0 + C::kXBytes;                 // weight rows
    const int zero_addr = w0 + C::kWBytes;            // a zero word above every valid gather address
    const int tbl_col = zero_addr + 16, tbl_row = tbl_col + C::kColEntries * 4;

    // Everything the stagers do not write must hold finite numbers (it meets zero weights only).
    for (int i = tid * 16; i < C::kLdsBytes; i += C::kThreads * 16) *lds_ptr<u32x4>(lds0 + i) = u32x4{0u, 0u, 0u, 0u};

    // lane-constant part of the A-operand address (transposing read): inside its group of 16, lane n
    // points at four channels of position 4g + n / 4 of a block and receives the n-th channel of positions
    // 4g .. 4g + 3.  The channels are dealt so that MFMA row m of half hf is channel 8 (m / 4) + 4 hf + m % 4:
    // a lane then ends up with the eight consecutive channels 8g .. 8g + 7 of its key, one 16-byte store.
    const int xa_lane = lds0 + (4 * g + (n >> 2)) * Traits<T>::kKeyBytes + (n & 3) * 16;

    const int ty0 = work.ty * C::TY, tx0 = work.tx * kTileX;
    const int ty1 = ty0 + C::TY - 1 < H - 1 ? ty0 + C::TY - 1 : H - 1;
    const int tx1 = tx0 + kTileX - 1 < W - 1 ? tx0 + kTileX - 1 : W - 1;
    const int ry0 = inv_first(ty0, H, K), ry1 = inv_last(ty1, H, K);
    const int rx0 = inv_first(tx0, W, K), rx1 = inv_last(tx1, W, K);
    const int nrows = ry1 - ry0 + 1, ncols = rx1 - rx0 + 1;   // <= RH, <= RW
    const int row_pitch_bytes = W * C::KK * SZ;                // < 2^31: checked by the host
    const int pitch_phase = row_pitch_bytes & 15;
    const int nbytes = ncols * C::KK * SZ;
    const size_t w_bytes = (size_t)nb * heads * H * W * C::KK * SZ;   // size of the weight tensor

    XHalo xhalo;
    xhalo.init(wave, lane);
    int xoff[C::NCH][XHalo::PER_WAVE];   // per chunk of rows (rows past the rectangle repeat the map's last row)
    const bool half_dim = pitch < Traits<T>::kKeyBytes;   // 16-channel heads: see kHalfDimChunks
#pragma unroll
    for (int c = 0; c < C::NCH; ++c) xhalo.offsets(H, W, ry0 + c * C::LH, rx0, xoff[c], pitch, half_dim ? kHalfDimChunks : 3);
    const int nch = CHUNK ? (nrows + C::LH - 1) / C::LH : 1;   // chunks of this tile's rectangle

    const int strip = wave / C::NWPS;
    const int sy0 = ty0 + 4 * strip;              // first key row of this wave's strip
    const int p0 = (wave % C::NWPS) * PPW;        // its first patch of the strip
    const int jy = sy0 + ky;
    const int oqy = inv_first(sy0 < H ? sy0 : H - 1, H, K);   // first query row of the strip's halo
    int rowterm[C::NBLK];
    int colterm[PPW][4];
    int xpatch[PPW];
#pragma unroll
    for (int p = 0; p < PPW; ++p) {
        const int px0 = tx0 + 4 * (p0 + p);
        const int oqx = inv_first(px0 < W ? px0 : W - 1, W, K);   // as in the column table
        xpatch[p] = ((oqy - ry0) * C::RW + (oqx - rx0)) * Traits<T>::kKeyBytes;
    }
    int mis_tables = -1;   // weight-row phase the tables in LDS were built for
    workgroup_sync();

    for (int b = b_begin; b < b_end; ++b) {
        const size_t plane_q = ((size_t)b * heads + head) * H * W;
        const size_t g0first = (plane_q + (size_t)ry0 * W + rx0) * C::KK * SZ;   // first byte of the first weight row
        const int mis0 = (int)(g0first & 15);   // 16-byte phase of row r: (mis0 + r * pitch_phase) & 15

        f32x4 acc[PPW][2];
#pragma unroll
        for (int p = 0; p < PPW; ++p) {
            acc[p][0] = f32x4{0.f, 0.f, 0.f, 0.f};
            acc[p][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll 1
        for (int c = 0; c < nch; ++c) {
        const int r_first = c * C::LH;                                                   // rectangle rows of this chunk:
        const int r_count = nrows - r_first < C::LH ? nrows - r_first : C::LH;           // [r_first, r_first + r_count)
        if (b > b_begin || c > 0) workgroup_sync();   // the previous LDS images are no longer read
        // Stage the rows.  Weight rows go from global memory straight into LDS (no registers): a
        // row is mirrored at its 16-byte phase, one 16-byte chunk per lane, 64 chunks per instruction;
        // the chunks at the two ends also bring in bytes of the neighbouring rows, which nothing reads.
        // Only the one chunk that would cross the end of the tensor is copied element by element.
        {
            constexpr int NI = (C::kRowChunks + kWave - 1) / kWave;   // instructions per row
            constexpr int PER_WAVE = (C::LH * NI + WAVES - 1) / WAVES;
            const char *wrow = reinterpret_cast<const char *>(w) + (g0first - mis0);   // 16-byte aligned
            const size_t left = w_bytes - (g0first - mis0);                             // bytes up to the tensor's end
            const int rem = left < (size_t)0x7fffffff ? (int)left : 0x7fffffff;
#pragma unroll
            for (int i = 0; i < PER_WAVE; ++i) {
                const int item = wave + i * WAVES;
                const int rl = item / NI, j = item - rl * NI;   // row inside the chunk
                if (rl < r_count) {
                    const int rel = mis0 + (r_first + rl) * row_pitch_bytes;   // row start, from wrow
                    const int nchunks = ((rel & 15) + nbytes + 15) >> 4;
                    const int cc = j * kWave + lane;
                    const int off = (rel & ~15) + cc * 16;
                    if (cc < nchunks && off + 16 <= rem)
                        global_to_lds_16(wrow + off, w0 + rl * C::kRowRegion + j * kWave * 16);
                }
            }
            const int rel_last = mis0 + (nrows - 1) * row_pitch_bytes;
            const int end_last = rel_last + nbytes;
            // the tensor ends inside the last chunk of the rectangle's last row
            if (((end_last + 15) & ~15) > rem && wave == 0 && nrows - 1 >= r_first && nrows - 1 < r_first + r_count) {
                const int off = (rem & ~15) + lane * SZ;
                if (lane < 16 / SZ && off < end_last)
                    *lds_ptr<T>(w0 + (nrows - 1 - r_first) * C::kRowRegion + (off - (rel_last & ~15))) = *reinterpret_cast<const T *>(wrow + off);
            }
        }
        // x vectors, natural layout
        {
            int xo[XHalo::PER_WAVE];   // this chunk's offsets (selected, not indexed: the tables stay in registers)
#pragma unroll
            for (int i = 0; i < XHalo::PER_WAVE; ++i) {
                xo[i] = xoff[0][i];
#pragma unroll
                for (int cc = 1; cc < C::NCH; ++cc) xo[i] = c == cc ? xoff[cc][i] : xo[i];
            }
            XHalo::issue_at(reinterpret_cast<const char *>(x) + plane_q * pitch, xo, lds0, wave);
        }

        // Gather-address tables, one entry per thread: the address of the weight that query (iy, ix)
        // gives key (jy, jx) is rowterm(iy, jy) + colterm(ix, jx); a pair that does not meet gets BIG.
        // (Row terms address the rectangle as if all of it were in LDS; a chunk subtracts its first row.)
        const bool rebuild = c == 0 && mis0 != mis_tables;   // same for the whole workgroup
        if (rebuild) {
            for (int e = tid; e < C::kColEntries + C::kRowEntries; e += C::kThreads) {
                int term = BIG;
                if (e < C::kColEntries) {
                    const int r = e & 3, kxe = (e >> 2) & 3, ge = (e >> 4) & 3, pe = e >> 6;
                    const int px0 = tx0 + 4 * pe, jx = px0 + kxe;
                    // halo columns start at the first query column that sees the patch; the 16-wide block
                    // reaches the last such column (at most K + R + 3 <= 13 of them)
                    const int ix = inv_first(px0 < W ? px0 : W - 1, W, K) + 4 * ge + r;
                    const int cw = jx - win_start(ix < W ? ix : W - 1, W, K);
                    if (px0 < W && ix <= rx1 && jx < W && (unsigned)cw < (unsigned)K) term = (ix - rx0) * C::KK * SZ + cw * SZ;
                } else {
                    const int l = e - C::kColEntries;
                    const int kye = l & 3, bb = (l >> 2) % C::NBLK, st = (l >> 2) / C::NBLK;
                    const int sy = ty0 + 4 * st, jyy = sy + kye;
                    const int iy = inv_first(sy < H ? sy : H - 1, H, K) + bb;   // halo row bb of the strip
                    const int a = jyy - win_start(iy < H ? iy : H - 1, H, K);
                    if (iy <= ry1 && jyy < H && (unsigned)a < (unsigned)K)   // (every bb < NBLK is a row the loop visits)
                        term = w0 + (iy - ry0) * C::kRowRegion + ((mis0 + (iy - ry0) * pitch_phase) & 15) + a * K * SZ;
                }
                *lds_ptr<int>(tbl_col + e * 4) = term;
            }
            mis_tables = mis0;
        }
        wait_global_loads();
        workgroup_sync();
        if (rebuild) {
#pragma unroll
            for (int bb = 0; bb < C::NBLK; ++bb) rowterm[bb] = *lds_ptr<int>(tbl_row + ((strip * C::NBLK + bb) * 4 + ky) * 4);
#pragma unroll
            for (int p = 0; p < PPW; ++p) {
                const u32x4 ct = *lds_ptr<u32x4>(tbl_col + (((p0 + p) * 4 + g) * 4 + kx) * 16);
                colterm[p][0] = (int)ct.x;
                colterm[p][1] = (int)ct.y;
                colterm[p][2] = (int)ct.z;
                colterm[p][3] = (int)ct.w;
            }
        }
        if (sy0 >= H) continue;

        const int wshift = r_first * C::kRowRegion;                       // what this chunk's LDS rows are short of
        const int xshift = r_first * C::RW * Traits<T>::kKeyBytes;        // ... the rectangle's, weights and x
        const int row_of_pair0 = oqy - ry0;                               // rectangle row of the strip's halo row 0
#pragma unroll
        for (int pb = 0; pb < C::NPAIR; ++pb) {
            // halo rows that no key row of the strip is seen from are skipped, and (CHUNK) those of other chunks
            const int rr = row_of_pair0 + 2 * pb;
            const bool here = CHUNK == 0 || (rr >= r_first && rr < r_first + C::LH);
            if (here && __any(rowterm[2 * pb] < BIG || rowterm[2 * pb + 1] < BIG)) {
#pragma unroll
                for (int p = 0; p < PPW; ++p) {
                    uint32_t wv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int bb = 2 * pb + (u >> 1);
                        const int r0 = (u & 1) * 2;
                        int a_lo = rowterm[bb] + colterm[p][r0] - wshift, a_hi = rowterm[bb] + colterm[p][r0 + 1] - wshift;
                        a_lo = a_lo < zero_addr ? a_lo : zero_addr;
                        a_hi = a_hi < zero_addr ? a_hi : zero_addr;
                        wv[u] = (uint32_t)*lds_ptr<uint16_t>(a_lo) | ((uint32_t)*lds_ptr<uint16_t>(a_hi) << 16);
                    }
                    const u32x4 bop = u32x4{wv[0], wv[1], wv[2], wv[3]};
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf) {
                        const int a0 = xa_lane + xpatch[p] - xshift + (2 * pb) * C::RW * Traits<T>::kKeyBytes + hf * 8;
                        const u32x2 lo = lds_read_tr16(a0);
                        const u32x2 hi = lds_read_tr16(a0 + C::RW * Traits<T>::kKeyBytes);
                        const u32x4 aop = u32x4{lo.x, lo.y, hi.x, hi.y};
                        acc[p][hf] = mfma_16x16x32<T>(aop, bop, acc[p][hf]);
                    }
                }
            }
        }
        }   // chunks
        if (sy0 >= H) continue;
#pragma unroll
        for (int p = 0; p < PPW; ++p) {
            const int jx = tx0 + 4 * (p0 + p) + kx;
            if (jy < H && jx < W && (!half_dim || g < 2)) {
                char *dst = reinterpret_cast<char *>(out) + (plane_q + (size_t)jy * W + jx) * pitch + g * 16;
                uint32_t o[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int hf = u >> 1, r = 2 * (u & 1);
                    const T lo = from_f32<T>(acc[p][hf][r] * scale), hi = from_f32<T>(acc[p][hf][r + 1] * scale);
                    o[u] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
                }
                store16_stream(dst, u32x4{o[0], o[1], o[2], o[3]});   // channels 8g .. 8g + 7
            }
        }
    }
}

template <typename T, int K, bool COMPACT, int CHUNK = 0>
static hipError_t launch_inverse_mfma_c(const Problem &p, const void *w, const void *x, float scale, void *out,
                                        hipStream_t s) {
    constexpr int STRIPS = 2, PPW = 1;
    using C = InvMfmaCfg<T, K, STRIPS, PPW, COMPACT, CHUNK>;
    constexpr int kWgPerCu = C::kWgPerCu;
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    // (tile position, head) units, the batch cut into ranges so that every workgroup slot of the chip is used
    const int units = tiles_x * tiles_y * p.heads;
    int splits = (256 * kWgPerCu) / units;
    splits = splits < 1 ? 1 : (splits < p.B ? splits : p.B);
    const int nwg = units * splits;
    const GridDecode gd = make_grid_decode(tiles_x, tiles_y, p.heads, p.B, splits);
    auto kern = inverse_mfma_kernel<T, K, STRIPS, PPW, COMPACT, CHUNK>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    for (int sl = 0; sl < (p.D + kHeadDim - 1) / kHeadDim; ++sl) {   // one launch per 32-channel slice of the head vector (a 16-channel head is half a slice)
        hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(nwg)), dim3(C::kThreads), C::kLdsBytes, s,
                           static_cast<const T *>(w), static_cast<const T *>(x) + sl * kHeadDim, scale,
                           static_cast<T *>(out) + sl * kHeadDim, p.H, p.W, p.heads, p.B, tiles_y, units, splits, gd,
                           p.D * (int)sizeof(T));
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Does the query rectangle of every 16 x 8 key tile fit rows x cols positions?
static bool rect_fits(const Problem &p, int rows, int cols) {
    const int K = p.K, TY = 8;
    for (int ty0 = 0; ty0 < p.H; ty0 += TY) {
        const int ty1 = ty0 + TY - 1 < p.H - 1 ? ty0 + TY - 1 : p.H - 1;
        if (inv_last(ty1, p.H, K) - inv_first(ty0, p.H, K) + 1 > rows) return false;
    }
    for (int tx0 = 0; tx0 < p.W; tx0 += kTileX) {
        const int tx1 = tx0 + kTileX - 1 < p.W - 1 ? tx0 + kTileX - 1 : p.W - 1;
        if (inv_last(tx1, p.W, K) - inv_first(tx0, p.W, K) + 1 > cols) return false;
    }
    return true;
}
static bool compact_fits(const Problem &p) { return rect_fits(p, 8 + p.K - 1, kTileX + p.K - 1); }

// Chunked variant: is the first halo row of every 4-row strip an even number of rows below the first row of its
// tile's rectangle (so that no pair of rows straddles two chunks)?  True for K = 9 on every map (the rows in
// question are 0 or multiples of 4 minus R = 4); checked all the same.
static bool chunk_pairs_aligned(const Problem &p) {
    for (int ty0 = 0; ty0 < p.H; ty0 += 8)
        for (int sy = ty0; sy < ty0 + 8 && sy < p.H; sy += 4)
            if ((inv_first(sy, p.H, p.K) - inv_first(ty0, p.H, p.K)) & 1) return false;
    return true;
}

template <typename T, int K>
static hipError_t launch_inverse_mfma_t(const Problem &p, const void *w, const void *x, float scale, void *out,
                                        hipStream_t s) {
    if (K == 9 && chunk_pairs_aligned(p)) {   // the rectangle in chunks of rows: two or three workgroups per compute unit instead of one
        if constexpr (K == 9)
            return compact_fits(p) ? launch_inverse_mfma_c<T, K, true, 8>(p, w, x, scale, out, s)
                                   : launch_inverse_mfma_c<T, K, false, 10>(p, w, x, scale, out, s);
    }
    return compact_fits(p) ? launch_inverse_mfma_c<T, K, true>(p, w, x, scale, out, s)
                           : launch_inverse_mfma_c<T, K, false>(p, w, x, scale, out, s);
}

// Is every 4-row strip of keys seen from at most NBLK query rows (the rows a wave walks from the strip's first
// query row on) and every 4-column patch from at most 16 query columns (one MFMA block)?  Always so away from
// short axes (K + R + 3 positions at most); on an axis of at most 2K + 2 positions a patch can be seen from both
// clamped ends at once, and then it depends on the length: 14 x 14 and 7 x 7 maps at K = 7 fit, 16 x 16 at K = 9
// does not.
static bool patch_halo_fits(const Problem &p) {
    const int K = p.K, PWI = K + K / 2 + 3, NBLK = PWI + (PWI & 1);
    for (int sy = 0; sy < p.H; sy += 4)
        if (inv_last(sy + 3 < p.H - 1 ? sy + 3 : p.H - 1, p.H, K) - inv_first(sy, p.H, K) + 1 > NBLK) return false;
    for (int px = 0; px < p.W; px += 4)
        if (inv_last(px + 3 < p.W - 1 ? px + 3 : p.W - 1, p.W, K) - inv_first(px, p.W, K) + 1 > 16) return false;
    return true;
}

// The kernel sizes its LDS images for key tiles whose query rectangle has at most (8 + K-1 + R) x (16 + K-1 + R)
// positions and walks NBLK query rows and 16 query columns per patch: maps where a tile or a patch is seen from
// more (some short axes) take the row-streaming kernel instead.
bool inverse_mfma_supported(const Problem &p) {
    const int R = p.K / 2;
    return (p.D % kHeadDim == 0 || p.D == kHalfDim) && p.dtype != NA2D_F32 && p.K <= 9 && patch_halo_fits(p) &&
           rect_fits(p, 8 + p.K - 1 + R, kTileX + p.K - 1 + R);
}

hipError_t launch_inverse_mfma(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s) {
#define NA2D_INV_K(TT)                                                                              \
    switch (p.K) {                                                                                  \
        case 3: return launch_inverse_mfma_t<TT, 3>(p, w, x, scale, out, s);                        \
        case 5: return launch_inverse_mfma_t<TT, 5>(p, w, x, scale, out, s);                        \
        case 7: return launch_inverse_mfma_t<TT, 7>(p, w, x, scale, out, s);                        \
        case 9: return launch_inverse_mfma_t<TT, 9>(p, w, x, scale, out, s);                        \
        default: return hipErrorInvalidValue;                                                       \
    }
    if (p.dtype == NA2D_F16) { NA2D_INV_K(f16_t) }
    if (p.dtype == NA2D_BF16) { NA2D_INV_K(bf16_t) }
#undef NA2D_INV_K
    return hipErrorInvalidValue;
}

}  // namespace na2d
