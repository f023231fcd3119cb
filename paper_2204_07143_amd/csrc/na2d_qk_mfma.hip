// Neighbourhood logits on the matrix cores (f16 / bf16):
//   logits[n, a, c] = scale * <x_n, y_{rho(n; a, c)}> + bias
// (arXiv 2204.07143, Eq. 2; with x = dout, y = v and no bias it is grad-a, Appendix A).
//
// Per 4 x 4 patch of queries: the queries are the B operand (one 16-byte global load per lane), each
// block of 16 positions of the patch halo is an A operand (one 16-byte LDS read per lane), one MFMA
// per block gives every lane 4 dot products of "its" query.  Which of them fall inside the query's
// window, and where they go in the k*k row, depends only on the lane and on how far the window is
// shifted at a border; that is kept as a per-lane table of LDS addresses (entries outside the
// window point at a dump word).  So the steady state per result is one fused multiply-add-convert
// (scale, bias) and one 2-byte LDS store.
//
// Eight waves share a 16 x 8 query tile, one 4 x 4 patch each, so a SIMD holds four waves whose
// LDS, matrix and conversion work overlap (two where the images of a second 32-channel slice fill the
// LDS: head dim 64).  The key halo reaches LDS by direct loads in its
// natural 64-byte-per-key layout (consecutive keys of an operand block are consecutive in LDS,
// so the 16-byte operand reads do not collide), into one of two buffers: the next tile's halo
// arrives while this tile is computed.  Results go to one of two staging images of the tile's
// eight row runs (phase-free: slot tables do not depend on where a run starts in memory); wave w
// streams row w of the previous tile to global memory while the current tile is computed.  One
// workgroup barrier per tile.  Large windows keep one staging image (k = 9) and one halo buffer as well
// (k = 11, 13) so that two workgroups still share a compute unit's LDS: a tile is then filled, and after a
// second barrier streamed out (and the next halo loaded), while the other workgroup computes.
#include "na2d_kernels.hpp"
#include "na2d_mfma.hpp"
#include "na2d_tile.hpp"

namespace na2d {

// NS: 32-channel slices of the head vector (head dim 32 NS).  Each slice of the halo is its own 64-byte-per-key
// image in LDS and one more MFMA into the same accumulators.
template <typename T, int K, int NS = 1>
struct QkSmallCfg {
    using P = Patch<K>;
    static constexpr int STRIPS = 2;
    static constexpr int WAVES = 4 * STRIPS;
    static constexpr int TY = 4 * STRIPS;
    static constexpr int HALO_H = TY + K - 1, HALO_W = kTileX + K - 1;
    using Halo = HaloDma<T, HALO_H, HALO_W, WAVES>;
    static constexpr int KK = K * K, NB = 2 * K - 1;
    static constexpr int kThreads = kWave * WAVES;
    static constexpr int kHaloBytes = Halo::kBytes;          // one slice
    static constexpr int kHaloAll = NS * kHaloBytes;         // one stage
    static constexpr int kKeyBytesG = NS * Traits<T>::kKeyBytes;   // bytes per position in memory
    static constexpr int kRowBytes = kTileX * KK * (int)sizeof(T);
    static constexpr int kRowPitch = (kRowBytes + 15) & ~15;
    static constexpr int kStageBytes = TY * kRowPitch;
    static constexpr int kDumpBytes = kThreads * 4;              // one word per thread for results outside its window
    static constexpr int kImage = kStageBytes + kDumpBytes;      // one staging image and the dump words
    // Two staging images where two workgroups then still share a compute unit's LDS (or where one image would not
    // make them fit either); one image, filled and streamed out in turn, where that is what makes them fit (k = 9)
    static constexpr bool kOneImage = 2 * kHaloAll + 2 * kImage > 80 * 1024 && 2 * kHaloAll + kImage <= 80 * 1024;
    // ... and one halo buffer too, loaded between tiles, where only that makes them fit (k = 11, 13)
    // (also where two buffers and two images exceed the LDS of a compute unit altogether: two slices, k >= 11)
    static constexpr bool kOneHalo = 2 * kHaloAll + kImage > 80 * 1024 && (kHaloAll + kImage <= 80 * 1024 || 2 * kHaloAll + 2 * kImage > 160 * 1024);
    static constexpr bool kOneBoth = kOneImage || kOneHalo;      // (one image either way)
    static constexpr int kParity = kOneBoth ? 0 : kImage;        // distance between the two staging images
    static constexpr int kHaloParity = kOneHalo ? 0 : kHaloAll;  // ... between the two halo buffers
    static constexpr int kLdsBytes = (kOneHalo ? 1 : 2) * kHaloAll + (kOneBoth ? 1 : 2) * kImage;
    static constexpr int kWavesPerSimd = kLdsBytes <= 80 * 1024 ? 4 : 2;   // two workgroups, or one, per compute unit
    static_assert(kImage < 65536, "the second staging image is reached through the 16-bit offset of the LDS store");
};


// One row run of the tile, LDS -> global.  The run starts on a 16-byte boundary in LDS but anywhere (a multiple
// of the element size) in global memory: it leaves as 16-byte stores to addresses that are aligned to the
// element only, which the chip's global memory path takes as they are (the compiler itself emits them for such
// pointers), and whose 64 lanes still cover one contiguous kilobyte.  Aligning the stores instead would put the
// misalignment on the LDS side, where a 16-byte read at a 2-byte phase costs eight reads.  The elements past
// the last whole chunk (ragged tiles only) go one by one.
// `stream`: the stores carry the non-temporal hint (see launch_qk_mfma_small_ns for when).
template <typename T, int PASSES>
__device__ __forceinline__ void flush_run(char *gbase, size_t g0, int nbytes, int lds_row, int lane, bool stream) {
    const int nbody = nbytes >> 4;
    char *ga = gbase + g0;
    struct __attribute__((packed, aligned(2))) Chunk {
        u32x4 v;
    };
#pragma unroll
    for (int it0 = 0; it0 < PASSES; it0 += 2) {   // two chunks per lane in flight
        u32x4 v[2];
#pragma unroll
        for (int it = it0; it < it0 + 2 && it < PASSES; ++it) {
            const int c = lane + it * kWave;
            if (c < nbody) v[it - it0] = *lds_ptr<u32x4>(lds_row + 16 * c);
        }
#pragma unroll
        for (int it = it0; it < it0 + 2 && it < PASSES; ++it) {
            const int c = lane + it * kWave;
            if (c < nbody) {
                if (stream) store16_stream(ga + 16 * c, v[it - it0]);
                else reinterpret_cast<Chunk *>(ga + 16 * c)->v = v[it - it0];
            }
        }
    }
    const int tb = 16 * nbody + lane * (int)sizeof(T);
    if (tb < nbytes) *reinterpret_cast<T *>(ga + tb) = *lds_ptr<T>(lds_row + tb);
}

template <typename T, int K, int NS, bool STREAM>
__global__ __launch_bounds__(512, (QkSmallCfg<T, K, NS>::kWavesPerSimd)) void qk_mfma_small_kernel(
    const T *__restrict__ x, const T *__restrict__ y, const T *__restrict__ rpb, float scale, T *__restrict__ logits, int H,
    int W, int heads, int nb, int tiles_y, int units, int splits, GridDecode gd, int half_dim) {
    // STREAM: the stores of the results carry the non-temporal hint (see launch_qk_mfma_small_ns for when)
    using C = QkSmallCfg<T, K, NS>;
    using P = Patch<K>;
    constexpr int kFlushPasses = (C::kRowBytes + kWave * 16 - 1) / (kWave * 16);   // 16-byte chunks per lane and row run
    static_assert(C::kThreads == 512, "launch bounds");
    constexpr int SZ = (int)sizeof(T);
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int strip = wave >> 2, p = patch_of_wave(wave);
    const int j = lane & 15, g = lane >> 4, jy = j >> 2, jx = j & 3;
    const int lds0 = lds_addr(lds);
    const int stage0 = lds0 + (C::kOneHalo ? 1 : 2) * C::kHaloAll;
    const int my_dump = stage0 + C::kStageBytes + tid * 4;

    // A workgroup keeps one tile position and one head and walks a range of the batch: everything
    // that depends on the position (halo geometry, window and bias tables, load offsets) is built once.
    // Neighbouring positions of a plane are handled by other workgroups at about the same time, so the
    // halo overlap is re-read from L2 while it is hot.
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

    // loads: the halo chunks of this lane and its 16 bytes of its query, as byte offsets inside a plane
    typename C::Halo halo;
    halo.init(wave, lane);
    int hoff[C::Halo::PER_WAVE];
    // (half_dim: 16-channel heads, NS = 1; see kHalfDimChunks)
    const int pitch = half_dim ? C::kKeyBytesG / 2 : C::kKeyBytesG, chunk_mask = half_dim ? kHalfDimChunks : 3;
    halo.offsets(H, W, hoy, hox, hoff, pitch, chunk_mask);
    const int qoff = ((qy < H - 1 ? qy : H - 1) * W + (qx < W - 1 ? qx : W - 1)) * pitch + (g & chunk_mask) * 16;
    const size_t plane_in = (size_t)H * W * pitch;          // bytes per plane of x / y
    const size_t plane_out = (size_t)H * W * C::KK * SZ;            // ... of the logits
    // stores: wave w streams row w of the tile
    const int frow = ty0 + wave;
    const int fbytes = ((W - tx0) < kTileX ? (W - tx0) : kTileX) * C::KK * SZ;
    const size_t foff = ((size_t)frow * W + tx0) * C::KK * SZ;

    u32x4 qnext[NS];
    auto issue = [&](int b, int par) {
        const size_t plane = (size_t)b * heads + head;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
            C::Halo::issue_at(reinterpret_cast<const char *>(y) + plane * plane_in + sl * Traits<T>::kKeyBytes, hoff,
                              lds0 + par * C::kHaloParity + sl * C::kHaloBytes, wave);
            // (read once: with the non-temporal hint where that gains, i.e. from k = 7 on while the stores are plain ones:
            // grad-a 23.0 -> 21.7 us at k = 7.  For smaller windows, for two slices and beside streaming stores it
            // loses: logits 14.7 -> 16.5 us at k = 5, 19.9 -> 27.7 us at D = 64, 39.4 -> 44.8 us at k = 11.)
            const u32x4 *qsrc = reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(x) + plane * plane_in + qoff +
                                                                sl * Traits<T>::kKeyBytes);
            if constexpr (K >= 7 && NS == 1 && !STREAM) qnext[sl] = __builtin_nontemporal_load(qsrc);
            else qnext[sl] = *qsrc;
        }
    };
    issue(b_begin, 0);   // the first tile's loads fly while the tables below are built

    // A operand: offsets of this lane's keys inside the tile halo (keys past the end of the patch halo
    // re-read its last one)
    // (a patch halo that is 16 positions wide, k = 13: block b is its row b, one address and a stride)
    constexpr bool KROWS = P::PW == 16;
    int koff[KROWS ? 1 : P::NBLK];
#pragma unroll
    for (int b = 0; b < (KROWS ? 1 : P::NBLK); ++b) {
        int h = 16 * b + j;
        h = h < P::NKEY ? h : P::NKEY - 1;
        const int hy = P::row_of(h), hx = h - hy * P::PW;
        koff[b] = lds0 + ((oy - hoy + hy) * C::HALO_W + (ox - hox) + hx) * Traits<T>::kKeyBytes + g * 16;
    }
    // Where this lane's results go: result e is the dot product of query j with patch-halo key
    // 16 (e / 4) + 4 g + e % 4.  Inside the query's window it is stored at its slot of the query's row
    // run in the staging image, outside it goes to the lane's dump word.  The bias of (query, key)
    // depends on key - query only (Eq. 2); it is kept two per register in the storage type.
    // Large windows (up to 64 results per lane) keep the store addresses two per register, as 16-bit offsets
    // from the first staging image; small windows keep them as absolute addresses, one per register.
    constexpr bool PACKED = K > 7;
    static_assert(C::kImage < 65536, "offsets inside a staging image fit 16 bits");
    uint32_t bias2[P::NEL / 2];
    int slotaddr[PACKED ? P::NEL / 2 : P::NEL];
    auto slot_of = [&](int e) -> int {
        if constexpr (PACKED) return stage0 + (int)((e & 1) ? (uint32_t)slotaddr[e >> 1] >> 16 : (uint32_t)slotaddr[e >> 1] & 0xffffu);
        else return slotaddr[e];
    };
    {
        const int wy = win_start(qy < H ? qy : H - 1, H, K) - oy, wx = win_start(qx < W ? qx : W - 1, W, K) - ox;
        const int lane_stage = stage0 + (4 * strip + jy) * C::kRowPitch + (4 * p + jx) * C::KK * SZ;
        // Built per group of four consecutive halo positions (e / 4): the positions of a group that lie
        // inside the query's window are in one halo row (a halo row holds K + 3 positions, the window K of
        // them), normally the row of the group's first position; when that one is already right of the
        // window, the group runs on into the next halo row and only that part can be inside.
        // Groups are handled four at a time: their sixteen loads of the bias table are in flight together (one
        // uniform branch on the table's presence per batch) without the indices of the whole patch halo being
        // alive at once (large windows have up to 64 results per lane).
        const uint16_t *tbl = rpb != nullptr ? reinterpret_cast<const uint16_t *>(rpb) + (size_t)head * C::NB * C::NB : nullptr;
#pragma unroll
        for (int G0 = 0; G0 < P::NBLK; G0 += 4) {
            int bidx[16];
#pragma unroll
            for (int G = G0; G < G0 + 4 && G < P::NBLK; ++G) {
                const int h0 = 16 * G + 4 * g;
                const int hy0 = P::row_of(h0), hx0 = h0 - hy0 * P::PW;
                const bool wrap = hx0 > wx + K - 1;
                const int hy = hy0 + (wrap ? 1 : 0), hxf = hx0 - (wrap ? P::PW : 0);   // halo row, column of the first position
                const int a = hy - wy;
                int c0 = hxf - wx;   // window column of the group's first position (may be negative)
                const int base = lane_stage + (a * K + c0) * SZ;
                c0 = (q_ok && (unsigned)a < (unsigned)K) ? c0 : 64;   // no row of the window: every column test fails
                int u = hy - jy + P::R + dy;
                u = u < 0 ? 0 : (u > C::NB - 1 ? C::NB - 1 : u);   // cells outside the table belong to keys
                const int v0 = hxf - jx + P::R + dx;               // outside every window: value unused
                int sa[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    sa[i] = (unsigned)(c0 + i) < (unsigned)K ? base + i * SZ : my_dump;
                    int v = v0 + i;
                    v = v < 0 ? 0 : (v > C::NB - 1 ? C::NB - 1 : v);
                    bidx[4 * (G - G0) + i] = u * C::NB + v;
                }
                if constexpr (PACKED) {
                    slotaddr[2 * G] = (sa[0] - stage0) | ((sa[1] - stage0) << 16);
                    slotaddr[2 * G + 1] = (sa[2] - stage0) | ((sa[3] - stage0) << 16);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) slotaddr[4 * G + i] = sa[i];
                }
            }
            uint32_t bits[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) bits[e] = 0u;
            if (tbl != nullptr) {
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (4 * G0 + e < P::NEL) bits[e] = tbl[bidx[e]];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (2 * G0 + e < P::NEL / 2) bias2[2 * G0 + e] = bits[2 * e] | (bits[2 * e + 1] << 16);
            if constexpr (K > 7) __builtin_amdgcn_sched_barrier(0);   // keep the batches apart: one batch of temporaries at a time
        }
    }

    auto flush = [&](int b, int par) {
        if (frow < H)
            flush_run<T, kFlushPasses>(reinterpret_cast<char *>(logits), ((size_t)b * heads + head) * plane_out + foff, fbytes,
                         stage0 + par * C::kParity + wave * C::kRowPitch, lane, STREAM);
    };
    auto compute = [&](auto par_c, const u32x4 (&qreg)[NS]) {
        constexpr int PAR = decltype(par_c)::value;
        if constexpr (kProbeMemoryOnly) {   // measurement build: the query chunks are still loaded, the staging images leave as they are
#pragma unroll
            for (int sl = 0; sl < NS; ++sl) asm volatile("" ::"v"(qreg[sl].x), "v"(qreg[sl].y), "v"(qreg[sl].z), "v"(qreg[sl].w));
            return;
        }
        if (!active) return;
        if constexpr (PACKED) {
            // the packed tables stay packed: without this their unpacking is hoisted out of the loop over the planes
            // and takes a register per entry
#pragma unroll
            for (int e = 0; e < P::NEL / 2; ++e) asm volatile("" : "+v"(slotaddr[e]), "+v"(bias2[e]));
        }
        // blocks in batches of eight: the MFMAs of a batch are issued back to back, then its 32 results are
        // stored; large windows (up to 16 blocks) never hold more than eight accumulators (five where two workgroups
        // per compute unit leave a lane 128 registers: k = 9)
        constexpr int BATCH = C::kOneBoth ? 5 : 8;
#pragma unroll
        for (int b0 = 0; b0 < P::NBLK; b0 += BATCH) {
            f32x4 acc[BATCH];
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int bk = b0 + u;
                if (bk >= P::NBLK) break;
                acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int sl = 0; sl < NS; ++sl) {
                    const int ka = KROWS ? koff[0] + bk * C::HALO_W * Traits<T>::kKeyBytes : koff[KROWS ? 0 : bk];
                    const u32x4 a = *lds_ptr<u32x4>(ka + PAR * C::kHaloParity + sl * C::kHaloBytes);
                    acc[u] = mfma_16x16x32<T>(a, qreg[sl], acc[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < 4 * BATCH; ++u) {
                const int e = 4 * b0 + u;
                if (e >= P::NEL) break;
                const uint16_t bb = (uint16_t)((e & 1) ? bias2[e >> 1] >> 16 : bias2[e >> 1] & 0xffffu);
                const float v = __builtin_fmaf(scale, acc[u >> 2][u & 3], to_f32(__builtin_bit_cast(T, bb)));
                *lds_ptr<T>(slot_of(e) + PAR * C::kParity) = from_f32<T>(v);
            }
        }
    };

    int b = b_begin;
    auto step = [&](auto par_c) {
        constexpr int PAR = decltype(par_c)::value;
        wait_global_loads();   // this tile's halo and query chunk have landed
        workgroup_sync();       // ... for every wave; the previous tile is fully staged, its halo no longer read
        u32x4 qreg[NS];
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) qreg[sl] = (half_dim && g >= 2) ? u32x4{0u, 0u, 0u, 0u} : qnext[sl];
        if constexpr (C::kOneHalo) {
            // one halo buffer, one image: compute, then the next tile's loads and this tile's results leave together
            compute(par_c, qreg);
            workgroup_sync();
            if (b + 1 < b_end) issue(b + 1, 0);
            flush(b, 0);
        } else if constexpr (C::kOneImage) {
            if (b + 1 < b_end) issue(b + 1, PAR ^ 1);
            // the one image: filled, then streamed out before the next tile's barrier lets anyone refill it (the
            // workgroup that shares the compute unit computes meanwhile)
            compute(par_c, qreg);
            workgroup_sync();
            flush(b, 0);
        } else {
            if (b + 1 < b_end) issue(b + 1, PAR ^ 1);
            if (b > b_begin) flush(b - 1, PAR ^ 1);
            compute(par_c, qreg);
        }
        ++b;
    };
    while (b < b_end) {
        step(IntC<0>{});
        if (b < b_end) step(IntC<1>{});
    }
    if constexpr (!C::kOneBoth) {
        workgroup_sync();
        flush(b_end - 1, (b_end - b_begin - 1) & 1);
    }
}

// D = 128: do one halo buffer of four slices and one staging image fit the 160 KB of a compute unit?
constexpr bool four_slices_fit(int K) {
    const int halo = (8 + K - 1) * (kTileX + K - 1) * 64, image = 8 * ((kTileX * K * K * 2 + 15) & ~15) + 512 * 4;
    return 4 * halo + image <= 160 * 1024;
}

template <typename T, int K, int NS>
static hipError_t launch_qk_mfma_small_ns(const Problem &p, const void *x, const void *y, const void *rpb, float scale,
                                          void *logits, hipStream_t s) {
    using C = QkSmallCfg<T, K, NS>;
    static_assert(NS > 1 || K > 7 || C::kLdsBytes <= 80 * 1024, "two workgroups share the LDS of a compute unit");
    static_assert(C::kLdsBytes <= 160 * 1024, "LDS of a compute unit");
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    const UnitSplit us = unit_split(tiles_x, tiles_y, p.heads, p.B);
    // The logits (or dp) are read by the next kernel of the path.  A small tensor is still in the last-level cache
    // then, so its stores are plain ones; from 48 MB on they carry the non-temporal hint, which keeps them from
    // competing with the halo re-reads of this kernel: at the benchmark shape (39 MB at k = 7) the hint makes this
    // kernel 2.6 us faster and the chain of calls 3 us slower, at k = 9, 11, 13 (65 to 136 MB) it makes the kernel
    // 3 to 12 us faster and the chain 2 to 4 us faster (measured with the two builds run in turn).
    const bool stream_out = (size_t)p.queries() * C::KK * sizeof(T) >= ((size_t)48 << 20);
    auto kern = stream_out ? qk_mfma_small_kernel<T, K, NS, true> : qk_mfma_small_kernel<T, K, NS, false>;
    static LdsAllowed allowed[2];
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed[stream_out]); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(us.units * us.splits)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(x), static_cast<const T *>(y), static_cast<const T *>(rpb), scale,
                       static_cast<T *>(logits), p.H, p.W, p.heads, p.B, tiles_y, us.units, us.splits, us.gd,
                       p.D == kHalfDim ? 1 : 0);
    return hipGetLastError();
}

template <typename T, int K>
static hipError_t launch_qk_mfma_small_t(const Problem &p, const void *x, const void *y, const void *rpb, float scale,
                                         void *logits, hipStream_t s) {
    if (p.D == 2 * kHeadDim) return launch_qk_mfma_small_ns<T, K, 2>(p, x, y, rpb, scale, logits, s);
    if constexpr (four_slices_fit(K)) {
        if (p.D == 4 * kHeadDim) return launch_qk_mfma_small_ns<T, K, 4>(p, x, y, rpb, scale, logits, s);
    }
    return launch_qk_mfma_small_ns<T, K, 1>(p, x, y, rpb, scale, logits, s);
}

bool qk_mfma_supported(const Problem &p) {
    if (p.dtype == NA2D_F32 || p.K > kMaxTunedK) return false;
    // one, two or (while one halo buffer and one staging image fit the LDS: k <= 11) four 32-channel slices
    return p.D == kHeadDim || p.D == kHalfDim || p.D == 2 * kHeadDim || (p.D == 4 * kHeadDim && four_slices_fit(p.K));
}

hipError_t launch_qk_mfma(const Problem &p, const void *x, const void *y, const void *rpb, float scale, void *logits,
                          hipStream_t s) {
    if (p.dtype == NA2D_F16) {
        using T = f16_t;
        NA2D_DISPATCH_K(p.K, return (launch_qk_mfma_small_t<T, K>(p, x, y, rpb, scale, logits, s)));
    } else if (p.dtype == NA2D_BF16) {
        using T = bf16_t;
        NA2D_DISPATCH_K(p.K, return (launch_qk_mfma_small_t<T, K>(p, x, y, rpb, scale, logits, s)));
    }
    return hipErrorInvalidValue;
}

}  // namespace na2d
