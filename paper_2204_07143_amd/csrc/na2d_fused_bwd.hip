// Fused neighbourhood attention backward on the matrix cores (f16 / bf16, K <= 9): the gradients
// of q, k, v and of the bias table from q, k, v, dout and the log-sum-exp of every query that the
// fused forward left behind; the k*k attention weights and their gradients never reach memory
// (arXiv 2204.07143: Eq. 2-4 differentiated; Appendix A lists the five gradients).
//
//   P[i, j]  = exp(scale <q_i, k_j> + B(i, j) - lse_i)           recomputed per tile
//   dP[i, j] = <dout_i, v_j>
//   delta_i  = sum_j P[i, j] dP[i, j]
//   dS[i, j] = P[i, j] (dP[i, j] - delta_i)
//   dq_i = scale sum_j dS[i, j] k_j      dB = sum over the queries of dS, per relative position
//   dk_j = scale sum_i dS[i, j] q_i      dv_j = sum_i P[i, j] dout_i
//
// Two kernels.  The first keeps 4 x 4 query patches (rows of P: dq, dB, and delta, which it leaves in
// the workspace for the second); the second keeps 4 x 4 key patches (columns of P: dk, dv).
#include "na2d_kernels.hpp"
#include "na2d_mfma.hpp"
#include "na2d_tile.hpp"

namespace na2d {

template <typename T> __device__ __forceinline__ uint32_t pack2_t(float a, float b) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef T tx2_t __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){a, b}, tx2_t));
}
// ---- part 1: query patches -> dq, delta, partial dB ------------------------------------------
//
// Same decomposition as the fused forward: eight waves share a 16 x 8 query tile, one 4 x 4 patch
// each; a workgroup keeps one tile position and one head and walks a range of the batch, so the
// window mask, the bias table and every address are built once; the key and the value halo of a
// tile reach one of two LDS buffer pairs by direct loads while the previous tile is computed.
// Two sweeps over the 16-position blocks of the patch halo.  Both evaluate
//   S^T = K_blk Q^T, dP^T = V_blk dout^T    (keys / values as 16-byte A operands, q / dout of the lane's
//                                            query as B operand)
// the first only to sum delta = sum P dP (a query's positions are spread over 4 lanes: two cross-lane
// steps), the second for
//   dS^T = P (dP - delta)                    in registers, already in the B-operand layout of
//   dq^T += K_blk^T dS^T                     the half-depth MFMA (keys through the transposing LDS read).
// Recomputing the two products is cheaper than keeping P and dP of the whole halo in registers.
// Every dS is also added to its cell of a (2K-1)^2 table in LDS (Eq. 2's B differentiated: the bias cell of a
// (query, position) pair depends on their offset only).  The tables are 64-bit fixed point with 32 fraction
// bits and the adds are integer atomics: on this chip an LDS integer add costs a few cycles per wave
// instruction where the floating-point add costs about 200, and integer addition does not depend on the
// order of the operands, so the bias gradient is bitwise reproducible although waves share tables.
// A dS is converted in two steps so that its precision follows its size: a lane bounds the dS of its query
// in a plane by B = max |dP| + |delta| (from the first sweep), takes sh = max(0, exponent(B) + 32 - 30), turns
// dS 2^(32 - sh) into a 32-bit integer (below 2^30 in magnitude, truncated: an error below 2^-30 B) and shifts
// it left by sh as a 64-bit integer.  Small gradients therefore keep an absolute resolution of 2^-32 (2.3e-10),
// large ones a relative one of 2^-30, and a workgroup's 64-bit sums (about 2^11 terms per cell) stay exact while
// |dS| < 2^20; beyond that they wrap.  A workgroup's tables, added up and converted to fp32 at the end, are
// one partial bias gradient.  (A NaN dS counts as 0.)
template <typename T, int K>
struct FbwdQCfg {
    using P = Patch<K>;
    static constexpr int STRIPS = 2;
    static constexpr int WAVES = 4 * STRIPS;
    static constexpr int TY = 4 * STRIPS;
    static constexpr int HALO_H = TY + K - 1, HALO_W = kTileX + K - 1;
    using Halo = HaloDma<T, HALO_H, HALO_W, WAVES>;
    static constexpr int NB = 2 * K - 1, CELLS = NB * NB;
    static constexpr int NPAIR = (P::NBLK + 1) / 2;
    static constexpr int NBLK2 = 2 * NPAIR;
    static constexpr int kThreads = kWave * WAVES;
    static constexpr int kHaloBytes = Halo::kBytes;
    static constexpr int kStageBytes = 2 * kHaloBytes;   // keys, then values
    // Two buffer pairs where two workgroups then still share a compute unit's LDS; one pair, reloaded between tiles
    // while the other workgroup computes, where that is what makes them fit (K = 9)
    static constexpr int kTblPad = 3;                    // cells in front of and behind a table (see the cell offsets)
    static constexpr int kTblBytes = (CELLS + 2 * kTblPad) * 8;
    static constexpr bool kOneStage = 2 * kStageBytes + kTblBytes > 80 * 1024;
    static constexpr int NSTAGE = kOneStage ? 1 : 2;
    // Bias-gradient tables behind the buffers, 64-bit fixed point (see above): as many as fit beside two
    // workgroups' buffers in a compute unit's 160 KB, at most one per wave
    static constexpr int kTblFit = (80 * 1024 - NSTAGE * kStageBytes) / kTblBytes;
    static constexpr int NTBL = kTblFit >= WAVES ? WAVES : (kTblFit >= 4 ? 4 : (kTblFit >= 2 ? 2 : 1));
    static_assert(kTblFit >= 1, "no room for a bias-gradient table");
    static constexpr int kFracBits = 32;   // fraction bits of the tables
    static constexpr int kLdsBytes = NSTAGE * kStageBytes + NTBL * kTblBytes;
};

template <typename T, int K, bool RPB>
__global__ __launch_bounds__(512, 4) void fbwd_q_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                        const T *__restrict__ v, const T *__restrict__ rpb, float scale,
                                                        const float *__restrict__ lse, const T *__restrict__ dout,
                                                        T *__restrict__ dq,
                                                        float *__restrict__ delta_out, float *__restrict__ lse2_out,
                                                        float *__restrict__ rpb_partial,
                                                        int H, int W, int heads, int nb, int tiles_y, int units, int splits, GridDecode gd,
                                                        int half_dim) {
    using C = FbwdQCfg<T, K>;
    using P = Patch<K>;
    static_assert(C::kThreads == 512, "launch bounds");
    constexpr float kLog2e = 1.4426950408889634f;
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

    const int hoy = halo_origin(ty0, C::TY, H, K), hox = halo_origin(tx0, kTileX, W, K);   // tile halo origin
    const int sy0 = ty0 + 4 * strip, px0 = tx0 + 4 * p;                                     // this wave's patch
    const bool active = sy0 < H && px0 < W;
    const int oy = halo_origin(sy0 < H ? sy0 : H - 1, 4, H, K), ox = halo_origin(px0 < W ? px0 : W - 1, 4, W, K);
    const int dy = oy - (sy0 - P::R), dx = ox - (px0 - P::R);   // 0 away from the borders
    const int qy = sy0 + jy, qx = px0 + jx;
    const bool q_ok = qy < H && qx < W;

    typename C::Halo halo;
    halo.init(wave, lane);
    int hoff[C::Halo::PER_WAVE];
    // (half_dim: 16-channel heads; see kHalfDimChunks)
    const int pitch = half_dim ? Traits<T>::kKeyBytes / 2 : Traits<T>::kKeyBytes, chunk_mask = half_dim ? kHalfDimChunks : 3;
    halo.offsets(H, W, hoy, hox, hoff, pitch, chunk_mask);
    const int qlin = (qy < H - 1 ? qy : H - 1) * W + (qx < W - 1 ? qx : W - 1);   // this lane's query inside a plane
    const size_t plane_bytes = (size_t)H * W * pitch;
    // per plane: both halos into LDS; this lane's 16 bytes (channels 8g .. 8g + 7) of q and dout of its query
    // and the query's log-sum-exp into registers
    u32x4 qnext, dnext;
    float lnext;
    auto issue = [&](int b, int par) {
        const size_t plane = (size_t)b * heads + head;
        const size_t off = plane * plane_bytes;
        C::Halo::issue_at(reinterpret_cast<const char *>(k) + off, hoff, lds0 + par * C::kStageBytes, wave);
        C::Halo::issue_at(reinterpret_cast<const char *>(v) + off, hoff, lds0 + par * C::kStageBytes + C::kHaloBytes, wave);
        const size_t qo = off + qlin * pitch + (g & chunk_mask) * 16;
        qnext = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(q) + qo);
        dnext = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(dout) + qo);
        lnext = lse[plane * H * W + qlin];
    };
    if (b_begin < b_end) issue(b_begin, 0);

    // Operand addresses inside the first buffer pair; those of the transposing reads are recomputed where they
    // are used, from an opaque copy of the lane index (eight more registers held across the loop cost more
    // than the arithmetic).
    // Keys / values as A operand rows: halo position 16b + j, bytes [16g, 16g+16).  Keys through the
    // transposing read: inside its group of 16 lanes, lane j points at four channels of halo position
    // 16b + 4g + j / 4 and receives the j-th channel of positions 16b + 4g .. + 3; the channels are dealt so
    // that MFMA row m of half hf is channel 8 (m / 4) + 4 hf + m % 4, which leaves a lane with the eight
    // consecutive channels 8g .. 8g + 7 of its query (one 16-byte store).
    const int kbase = lds0 + ((oy - hoy) * C::HALO_W + (ox - hox)) * Traits<T>::kKeyBytes;   // halo position 0 of the patch
    auto row_addr = [&](int lv, int b) {   // A operand row of block b
        int h = 16 * b + (lv & 15);
        h = h < P::NKEY ? h : P::NKEY - 1;   // past the end: any real position (its dS is zero)
        const int hy = P::row_of(h), hx = h - hy * P::PW;
        return kbase + (hy * C::HALO_W + hx) * Traits<T>::kKeyBytes + (lv >> 4) * 16;
    };
    int koff[P::NBLK];   // used twice per plane: kept
#pragma unroll
    for (int b = 0; b < P::NBLK; ++b) koff[b] = row_addr(lane, b);
    auto tr_addr = [&](int lv, int b) {   // transposing read of block b
        int h = 16 * b + 4 * (lv >> 4) + ((lv & 15) >> 2);
        h = h < P::NKEY ? h : P::NKEY - 1;
        const int hy = P::row_of(h), hx = h - hy * P::PW;
        return kbase + (hy * C::HALO_W + hx) * Traits<T>::kKeyBytes + (lv & 3) * 16;
    };
    // bias of (this lane's query, halo position), as stored (see bias_to_f16), -inf outside the query's window,
    // as packed fp16 pairs; cell[] is the position's cell in the bias table (-1 outside the window).  Built per
    // group of four consecutive halo positions: those of them inside the window are in one halo row (a halo row
    // holds K + 3 positions, the window K), normally the row of the first position; when that one is already
    // right of the window the group runs on into the next halo row and only that part can be inside.
    f16x2 biasm[P::NEL / 2];
    auto cell_group = [&](int lv, int G, int (&cell)[4]) {   // lv: the lane index (passed in so that the two uses share nothing)
        const int gg = lv >> 4, yy = (lv & 15) >> 2, xx = lv & 3;
        const int cy = sy0 + yy, cx = px0 + xx;
        const bool ok = cy < H && cx < W;
        const int wy = win_start(cy < H ? cy : H - 1, H, K) - oy, wx = win_start(cx < W ? cx : W - 1, W, K) - ox;
        const int h0 = 16 * G + 4 * gg;
        const int hy0 = P::row_of(h0), hx0 = h0 - hy0 * P::PW;
        const bool wrap = hx0 > wx + K - 1;
        const int hy = hy0 + (wrap ? 1 : 0), hxf = hx0 - (wrap ? P::PW : 0);
        const int a = hy - wy;
        const int c0 = (ok && (unsigned)a < (unsigned)K) ? hxf - wx : 64;   // no row of the window: every column test fails
        const int cell0 = (hy - yy + P::R + dy) * C::NB + (hxf - xx + P::R + dx);
#pragma unroll
        for (int i = 0; i < 4; ++i) cell[i] = (unsigned)(c0 + i) < (unsigned)K ? cell0 + i : -1;
    };
    // Where the results of block G are added: byte offset of the cell of result 4G inside a table; results 4G + 1 .. + 3
    // go to the three cells behind it (the cells of a group that lie inside the window are neighbours in one row of
    // the table).  Results outside the window are exactly 0 and adding them changes nothing, so they may go to any
    // cell: those of a group with a position inside the window simply land next to it, up to three cells in front of
    // or behind the table (kTblPad); a group with no position inside the window gets four cells that differ from lane
    // to lane, so that the adds of one instruction do not pile up on one address.
    int coff[RPB ? P::NBLK : 1];
    {
        const T *tbl = rpb != nullptr ? rpb + (size_t)head * C::CELLS : nullptr;
        constexpr int GB = K > 7 ? 2 : 4;   // groups per batch of bias loads (a batch of temporaries at a time)
#pragma unroll
        for (int G0 = 0; G0 < P::NBLK; G0 += GB) {
            int cell[4 * GB];
            f16_t bias[4 * GB];
#pragma unroll
            for (int u = 0; u < GB; ++u) {
                int c4[4] = {-1, -1, -1, -1};
                if (G0 + u < P::NBLK) cell_group(lane, G0 + u, c4);
#pragma unroll
                for (int i = 0; i < 4; ++i) cell[4 * u + i] = c4[i];
                if constexpr (RPB) {
                    if (G0 + u < P::NBLK) {
                        int first = -1;   // cell of result 4G, worked back from the first one inside the window
#pragma unroll
                        for (int i = 3; i >= 0; --i) first = c4[i] >= 0 ? c4[i] - i : first;
                        const bool any = (c4[0] & c4[1] & c4[2] & c4[3]) >= 0;
                        coff[G0 + u] = ((any ? first : lane % (C::CELLS - 3)) + C::kTblPad) * 8;
                    }
                }
            }
#pragma unroll
            for (int e = 0; e < 4 * GB; ++e) bias[e] = (f16_t)0.f;
            if (tbl != nullptr) {
#pragma unroll
                for (int e = 0; e < 4 * GB; ++e) bias[e] = bias_to_f16(tbl[cell[e] < 0 ? 0 : cell[e]]);
            }
#pragma unroll
            for (int e = 0; e < 4 * GB; ++e)
                if (4 * G0 + e < P::NEL) biasm[(4 * G0 + e) >> 1][e & 1] = cell[e] >= 0 ? bias[e] : (f16_t)-INFINITY;
            if constexpr (K > 7) __builtin_amdgcn_sched_barrier(0);
        }
    }
    const int tbl0 = lds0 + C::NSTAGE * C::kStageBytes;
    const int mytbl = tbl0 + (wave % C::NTBL) * C::kTblBytes;
    if constexpr (RPB) {
        for (int i = tid; i < C::NTBL * (C::kTblBytes / 8); i += C::kThreads) *lds_ptr<unsigned long long>(tbl0 + i * 8) = 0ull;
    }

    auto compute = [&](auto par_c, const u32x4 &qreg, const u32x4 &dreg, float lse2, int b) {
        constexpr int PAR = decltype(par_c)::value;
        if (!active) return;
        int lv = lane;
        asm volatile("" : "+v"(lv));
        // the packed table stays packed: without this the conversions to fp32 are hoisted out of the loop over
        // the planes and take 28 registers instead of 14
#pragma unroll
        for (int e = 0; e < P::NEL / 2; ++e) asm volatile("" : "+v"(biasm[e]));
        auto block = [&](int bk, f32x4 &sacc, f32x4 &pacc) {
            const int ra = koff[bk] + PAR * C::kStageBytes;
            const u32x4 ak = *lds_ptr<u32x4>(ra);
            const u32x4 av = *lds_ptr<u32x4>(ra + C::kHaloBytes);
            sacc = mfma_16x16x32<T>(ak, qreg, f32x4{0.f, 0.f, 0.f, 0.f});
            pacc = mfma_16x16x32<T>(av, dreg, f32x4{0.f, 0.f, 0.f, 0.f});
        };
        auto weight = [&](int e, float sv) {   // P of result e, 0 outside the window (bias -inf)
            return __builtin_amdgcn_exp2f(__builtin_fmaf(__builtin_fmaf(scale, sv, (float)biasm[e >> 1][e & 1]), kLog2e, -lse2));
        };
        // sweep 1: delta
        float delta = 0.f, dpmax = 0.f;
#pragma unroll
        for (int bk = 0; bk < P::NBLK; ++bk) {
            f32x4 sacc, pacc;
            block(bk, sacc, pacc);
#pragma unroll
            for (int r = 0; r < 4; ++r) delta = __builtin_fmaf(weight(4 * bk + r, sacc[r]), pacc[r], delta);
            if constexpr (RPB) dpmax = fmaxf(fmaxf(dpmax, fmaxf(fabsf(pacc[0]), fabsf(pacc[1]))), fmaxf(fabsf(pacc[2]), fabsf(pacc[3])));
            __builtin_amdgcn_sched_barrier(0);   // keeps the blocks from being evaluated all at once
        }
        delta += __shfl_xor(delta, 16);
        delta += __shfl_xor(delta, 32);
        // fixed-point conversion of this lane's dS in this plane: |dS| <= P |dP - delta| <= dpmax + |delta|
        float fx_scale = 0.f;
        int fx_shift = 0;
        if constexpr (RPB) {
            const int ex = __builtin_amdgcn_frexp_expf(dpmax + fabsf(delta));   // bound < 2^ex
            fx_shift = ex + C::kFracBits - 30;
            fx_shift = fx_shift < 0 ? 0 : (fx_shift > 32 ? 32 : fx_shift);
            fx_scale = __builtin_ldexpf(1.f, C::kFracBits - fx_shift);
        }
        // sweep 2: dS, dq (one block at a time: the half-depth MFMA takes the four positions a lane holds)
        f32x4 o[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int bk = 0; bk < P::NBLK; ++bk) {
            f32x4 sacc, pacc;
            block(bk, sacc, pacc);
            float dsv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int e = 4 * bk + r;
                dsv[r] = weight(e, sacc[r]) * (pacc[r] - delta);   // exactly 0 outside the window
                if constexpr (RPB) {
                    const long long fx = (long long)(int)(dsv[r] * fx_scale) << fx_shift;   // truncated, saturating; NaN -> 0
                    __hip_atomic_fetch_add(lds_ptr<unsigned long long>(mytbl + coff[bk] + 8 * r),
                                           (unsigned long long)fx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
            const uint32_t b0 = pack2_t<T>(dsv[0], dsv[1]), b1 = pack2_t<T>(dsv[2], dsv[3]);
            const int ta = tr_addr(lv, bk) + PAR * C::kStageBytes;
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const u32x2 a2 = lds_read_tr16(ta + hf * 8);
                o[hf] = mfma_16x16x16<T>(a2.x, a2.y, b0, b1, o[hf]);
                if constexpr (Traits<T>::kDtype == NA2D_BF16) {
                    // bf16 keeps 8 significant bits: a second operand carries the rounding remainder of dS so
                    // that the product sees it to 16 bits
                    const uint32_t l0 = pack2_t<T>(dsv[0] - to_f32(from_f32<T>(dsv[0])), dsv[1] - to_f32(from_f32<T>(dsv[1])));
                    const uint32_t l1 = pack2_t<T>(dsv[2] - to_f32(from_f32<T>(dsv[2])), dsv[3] - to_f32(from_f32<T>(dsv[3])));
                    o[hf] = mfma_16x16x16<T>(a2.x, a2.y, l0, l1, o[hf]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (q_ok) {
            const size_t plane = (size_t)b * heads + head;
            char *dst = reinterpret_cast<char *>(dq) + plane * plane_bytes + qlin * pitch + g * 16;
            if (!half_dim || g < 2)
                store16_stream(dst, u32x4{pack2_t<T>(o[0][0] * scale, o[0][1] * scale), pack2_t<T>(o[0][2] * scale, o[0][3] * scale),
                                          pack2_t<T>(o[1][0] * scale, o[1][1] * scale), pack2_t<T>(o[1][2] * scale, o[1][3] * scale)});
            if (g == 0) {   // for the key-patch kernel: delta, and the log-sum-exp in the exp2 domain
                delta_out[plane * H * W + qlin] = delta;
                lse2_out[plane * H * W + qlin] = lse2;
            }
        }
    };

    int b = b_begin;
    auto step = [&](auto par_c) {
        constexpr int PAR = decltype(par_c)::value;
        wait_global_loads();   // this tile's halos and the lane's query data have landed
        workgroup_sync();       // ... for every wave, and nobody still reads the other buffer pair
        const bool upper = half_dim && g >= 2;   // lanes whose channels a 16-channel head does not have
        const u32x4 qreg = upper ? u32x4{0u, 0u, 0u, 0u} : qnext, dreg = upper ? u32x4{0u, 0u, 0u, 0u} : dnext;
        const float lse2 = lnext * kLog2e;
        if constexpr (C::kOneStage) {
            compute(par_c, qreg, dreg, lse2, b);
            if (b + 1 < b_end) {
                workgroup_sync();   // nobody still reads the halos
                issue(b + 1, 0);
            }
        } else {
            if (b + 1 < b_end) issue(b + 1, PAR ^ 1);
            compute(par_c, qreg, dreg, lse2, b);
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
        // the tables added up (integers: any order), then to fp32: one partial bias gradient per workgroup
        workgroup_sync();
        for (int cell = tid; cell < C::CELLS; cell += C::kThreads) {
            long long sum = 0;
#pragma unroll
            for (int t = 0; t < C::NTBL; ++t) sum += (long long)*lds_ptr<unsigned long long>(tbl0 + t * C::kTblBytes + (cell + C::kTblPad) * 8);
            // row of this workgroup's partial: the partials of a head follow each other (rpb_cell_stride)
            rpb_partial[(size_t)((head * splits + work.split) * gd.npos + work.pos) * rpb_cell_stride(C::CELLS) + cell] =
                (float)((double)sum * (1.0 / 4294967296.0));   // 2^-32
        }
    }
}

template <typename T, int K>
static hipError_t launch_fbwd_q_t(const Problem &p, const void *q, const void *k, const void *v, const void *rpb,
                                  float scale, const float *lse, const void *dout, void *dq, float *delta, float *lse2,
                                  float *rpb_partial, hipStream_t s) {
    using C = FbwdQCfg<T, K>;
    static_assert(C::kLdsBytes <= 80 * 1024, "two workgroups share the LDS of a compute unit");
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    const UnitSplit us = unit_split(tiles_x, tiles_y, p.heads, p.B);
    const bool with_rpb = rpb_partial != nullptr;
    auto kern = with_rpb ? fbwd_q_kernel<T, K, true> : fbwd_q_kernel<T, K, false>;
    static LdsAllowed allowed[2];
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed[with_rpb]); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(us.units * us.splits)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(q), static_cast<const T *>(k), static_cast<const T *>(v),
                       static_cast<const T *>(rpb), scale, lse, static_cast<const T *>(dout), static_cast<T *>(dq), delta, lse2,
                       rpb_partial, p.H, p.W, p.heads, p.B, tiles_y, us.units, us.splits, us.gd, p.D == kHalfDim ? 1 : 0);
    return hipGetLastError();
}

// ---- part 2: key patches -> dk, dv -------------------------------------------------------------
//
// A workgroup owns a 16 x 8 key tile (eight waves, one 4 x 4 key patch each), keeps its position and head
// and walks a range of the batch.  The queries that see any key of the tile form a rectangle of at most
// (8 + K-1) x (16 + K-1) positions; per plane their q and dout vectors reach LDS by direct loads in the
// natural layout, their log-sum-exp and delta as fp32 rows.  Per row of the rectangle that sees the
// patch (a block of 16 consecutive query positions, the first one the leftmost query that sees the patch):
//   S = Q_blk K^T, dP = dout_blk V^T         (rows of q / dout as 16-byte A operands, the lane's key as B operand)
//   P = exp2(log2e S' - lse2), dS = P (dP - delta)   per result; a lane holds 4 consecutive positions of its key
//   dv^T += dout_blk^T P, dk^T += Q_blk^T dS the half-depth MFMA (q / dout through the transposing LDS read)
// The bias of (query, key) depends on their offset only; per block a lane needs four neighbouring cells
// of one table row.  The table is kept in LDS mirrored left to right and in four copies shifted by one
// element each, so that every such run of four starts on an 8-byte boundary in one of them.
// COMPACT: images sized for the rectangle of a tile away from the far border, (8 + K-1) x (16 + K-1) positions
// (three workgroups per compute unit); next to the far border the clamped queries reach R positions
// further, and a map with such tiles takes the larger images (two workgroups per compute unit).
template <typename T, int K, bool COMPACT>
struct FbwdKvCfg {
    static constexpr int R = K / 2;
    static constexpr int PWI = K + R + 3;   // query rows / columns that can see a 4 x 4 key patch
    static_assert(PWI <= 16, "one MFMA block per row of the query rectangle needs K + R + 3 <= 16");
    static constexpr int STRIPS = 2;
    static constexpr int WAVES = 4 * STRIPS;
    static constexpr int TY = 4 * STRIPS;
    // CHUNKED (K = 9): the images hold 16 rows of the rectangle at a time.  A rectangle of up to 20 rows (tiles next to
    // the far border) is taken in two chunks, its first 16 rows and its last 16 (the rows they share are used from the
    // first), so that two workgroups still share a compute unit; the accumulators stay in registers across them.
    static constexpr bool CHUNKED = K > 7;
    static_assert(!CHUNKED || !COMPACT, "the chunked images are always the wide ones");
    static constexpr int kRowsMax = TY + K - 1 + (COMPACT ? 0 : R);   // rows of a rectangle, at most
    static constexpr int RH = CHUNKED ? 16 : kRowsMax, RW = kTileX + K - 1 + (COMPACT ? 0 : R);   // the images
    static_assert(kRowsMax <= 32 && kRowsMax <= 2 * RH, "row flags; two chunks");
    static constexpr int NB = 2 * K - 1;
    static constexpr int kThreads = kWave * WAVES;
    using XHalo = HaloDma<T, RH, RW, WAVES>;
    // a block that starts up to 12 columns into the last row reaches 28 positions past the rectangle
    static constexpr int kXBytes = XHalo::kBytes + 28 * Traits<T>::kKeyBytes;
    static constexpr int SP = (RW + 3) & ~3;                       // row pitch of the fp32 images (>= RW, 16-byte rows)
    static_assert(SP >= RW && SP % 4 == 0, "fp32 rows");
    static constexpr int kSItems = (RH * SP + kWave - 1) / kWave;   // 64-lane loads per fp32 image
    static_assert(kSItems <= WAVES, "one fp32 load per wave and image");
    static_assert(!CHUNKED || kSItems * kWave <= RH * SP, "every word of a chunk's fp32 images is a row of the chunk");
    static constexpr int kSBytes = (kSItems * kWave + 32) * 4;      // + the reach of the last row's blocks
    static constexpr int BP = K > 7 ? 28 : 24;                      // row pitch (elements) of a bias copy (a multiple of 4)
    static_assert(NB + 3 + 3 + 3 < BP, "a shifted run of four stays inside its row");
    static constexpr int kBiasCopy = NB * BP * 2;
    static constexpr int kBiasBytes = 4 * kBiasCopy;
    static constexpr int kLdsBytes = 2 * kXBytes + 2 * kSBytes + kBiasBytes;
    static constexpr int kLdsAlloc = (kLdsBytes + 511) / 512 * 512;
    static constexpr int kWgPerCu = (160 * 1024) / kLdsAlloc < 3 ? (160 * 1024) / kLdsAlloc : 3;
    static_assert(kWgPerCu >= 2, "LDS");
    static constexpr int kWavesPerSimd = kWgPerCu * WAVES / 4;
};

template <typename T, int K, bool COMPACT>
__global__ __launch_bounds__(512, (FbwdKvCfg<T, K, COMPACT>::kWavesPerSimd)) void fbwd_kv_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v, const T *__restrict__ rpb, float scale,
    const float *__restrict__ lse2, const float *__restrict__ delta, const T *__restrict__ dout, T *__restrict__ dk,
    T *__restrict__ dv, int H, int W, int heads, int nb, int tiles_y, int units, int splits, GridDecode gd, int half_dim) {
    // lse2: the log-sum-exp of every query times log2(e), as the query-patch kernel left it beside delta
    using C = FbwdKvCfg<T, K, COMPACT>;
    using XHalo = typename C::XHalo;
    constexpr float kLog2e = 1.4426950408889634f;
    constexpr int KB = Traits<T>::kKeyBytes;
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
    const int q0 = lds0, d0 = lds0 + C::kXBytes;                           // q and dout of the rectangle
    const int l0 = d0 + C::kXBytes, e0 = l0 + C::kSBytes, bias0 = e0 + C::kSBytes;   // lse, delta, bias copies

    // everything the loads do not write must hold finite numbers (it only ever meets P = 0)
    for (int i = tid * 16; i < C::kLdsBytes - C::kBiasBytes; i += C::kThreads * 16) *lds_ptr<u32x4>(lds0 + i) = u32x4{0u, 0u, 0u, 0u};
    // bias copies: copy s holds B[u][v] (see bias_to_f16) at element u * BP + (NB-1 - v) + 3 + s, zeros elsewhere
    for (int i = tid; i < 4 * C::NB * C::BP; i += C::kThreads) {
        const int s = i / (C::NB * C::BP), rest = i - s * (C::NB * C::BP);
        const int u = rest / C::BP, col = rest - u * C::BP;
        const int vv = C::NB - 1 - (col - 3 - s);
        f16_t val = (f16_t)0.f;
        if (rpb != nullptr && (unsigned)vv < (unsigned)C::NB) val = bias_to_f16(rpb[((size_t)head * C::NB + u) * C::NB + vv]);
        *lds_ptr<f16_t>(bias0 + i * 2) = val;
    }

    const int ty0 = work.ty * C::TY, tx0 = work.tx * kTileX;
    const int tx1 = tx0 + kTileX - 1 < W - 1 ? tx0 + kTileX - 1 : W - 1;
    const int ty1 = ty0 + C::TY - 1 < H - 1 ? ty0 + C::TY - 1 : H - 1;
    const int ry0 = inv_first(ty0, H, K);   // the rectangle (fits kRowsMax x RW: checked by the host)
    const int rx0 = inv_first(tx0, W, K), rx1 = inv_last(tx1, W, K);
    const int nrows = inv_last(ty1, H, K) - ry0 + 1;
    const int nch = C::CHUNKED && nrows > C::RH ? 2 : 1;   // chunks of the rectangle
    const int org1 = nrows - C::RH;                        // first rectangle row of the second chunk

    // loads of one plane
    XHalo xhalo;
    xhalo.init(wave, lane);
    int xoff[XHalo::PER_WAVE];
    // (half_dim: 16-channel heads; see kHalfDimChunks)
    const int pitch = half_dim ? KB / 2 : KB, chunk_mask = half_dim ? kHalfDimChunks : 3;
    xhalo.offsets(H, W, ry0, rx0, xoff, pitch, chunk_mask);
    int soff;   // this lane's word of the fp32 images (waves 0 .. kSItems-1), clamped into the map
    {
        const int i = wave * kWave + lane;
        const int rr = i / C::SP, cc = i - rr * C::SP;
        int y = ry0 + rr, x = rx0 + cc;
        y = y < H - 1 ? y : H - 1;
        x = x < W - 1 ? x : W - 1;
        soff = (y * W + x) * 4;
    }

    const int strip = wave >> 2, p = patch_of_wave(wave);
    const int sy0 = ty0 + 4 * strip, px0 = tx0 + 4 * p;   // this wave's key patch
    const bool active = sy0 < H && px0 < W;
    const int jy = sy0 + ky, jx = px0 + kx;                // this lane's key
    const bool key_ok = jy < H && jx < W;
    const int oqy = inv_first(sy0 < H ? sy0 : H - 1, H, K), oqx = inv_first(px0 < W ? px0 : W - 1, W, K);
    const int sy3 = sy0 + 3 < H - 1 ? sy0 + 3 : H - 1;
    const int nblk = active ? inv_last(sy3, H, K) - oqy + 1 : 0;   // rows of the rectangle that see the patch (<= RH)
    const int row0 = oqy - ry0, col0 = oqx - rx0;
    // lane-constant address parts inside a rectangle row
    const int arow = (col0 + n) * KB + g * 16;                       // A operand row: position col0 + n, bytes [16g, 16g+16)
    const int atr = (col0 + 4 * g + (n >> 2)) * KB + (n & 3) * 16;   // transposing read (channels dealt as in part 1)
    const int sidx = (col0 + 4 * g) * 4;                             // fp32 images: positions col0 + 4g .. + 3
    // which of the lane's (position, key) pairs meet: the key must lie in the window of the query
    unsigned rowok = 0, colok = 0;
#pragma unroll
    for (int b = 0; b < C::kRowsMax; ++b) {
        const int iy = oqy + b;
        const bool ok = b < nblk && key_ok && (unsigned)(jy - win_start(iy < H ? iy : H - 1, H, K)) < (unsigned)K;
        rowok |= ok ? (1u << b) : 0u;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int ix = oqx + 4 * g + r;
        const bool ok = ix <= rx1 && key_ok && (unsigned)(jx - win_start(ix < W ? ix : W - 1, W, K)) < (unsigned)K;
        colok |= ok ? (1u << r) : 0u;
    }
    float colmask[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) colmask[r] = ((colok >> r) & 1u) ? 0.f : -INFINITY;
    // bias: row u = jy - iy + K-1 of the table, mirrored columns NB-1 - (jx - ix + K-1) = vm0 + r
    const int ub = jy - oqy + K - 1;
    int vm0 = C::NB - 1 - (jx - (oqx + 4 * g) + K - 1);
    vm0 = vm0 < -3 ? -3 : (vm0 > C::NB - 1 ? C::NB - 1 : vm0);   // outside the table only where nothing meets
    const int shift = (-(vm0 + 3)) & 3;
    const int cbase = bias0 + shift * C::kBiasCopy + (vm0 + 3 + shift) * 2;   // 8-byte aligned

    const size_t plane_px = (size_t)H * W;
    workgroup_sync();

    for (int b = b_begin; b < b_end; ++b) {
        const size_t plane = (size_t)b * heads + head;
        // the lane's key and value: bytes [16g, 16g+16) (B operands)
        const size_t koff = (plane * plane_px + (size_t)(jy < H ? jy : H - 1) * W + (jx < W ? jx : W - 1)) * pitch + (g & chunk_mask) * 16;
        const bool upper = half_dim && g >= 2;   // lanes whose channels a 16-channel head does not have
        const u32x4 kload = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(k) + koff);
        const u32x4 vload = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(v) + koff);
        const u32x4 kreg = upper ? u32x4{0u, 0u, 0u, 0u} : kload, vreg = upper ? u32x4{0u, 0u, 0u, 0u} : vload;
        f32x4 ak[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};   // dk^T, dv^T: channels 8g + 4 hf + r of the lane's key
        f32x4 av[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll 1
        for (int c = 0; c < nch; ++c) {
        if (b > b_begin || c > 0) workgroup_sync();   // the previous images are no longer read
        // rows of the rectangle in the images: [org, org + RH); the second chunk lies inside the map as a whole
        const int org = c ? org1 : 0;
        {
            int xo[XHalo::PER_WAVE];
#pragma unroll
            for (int i = 0; i < XHalo::PER_WAVE; ++i) xo[i] = xoff[i] >= 0 ? xoff[i] + org * W * pitch : -1;
            XHalo::issue_at(reinterpret_cast<const char *>(q) + plane * plane_px * pitch, xo, q0, wave);
            XHalo::issue_at(reinterpret_cast<const char *>(dout) + plane * plane_px * pitch, xo, d0, wave);
        }
        if (wave < C::kSItems) {
            global_to_lds_4(reinterpret_cast<const char *>(lse2) + plane * plane_px * 4, (unsigned)(soff + org * W * 4), l0 + wave * kWave * 4);
            global_to_lds_4(reinterpret_cast<const char *>(delta) + plane * plane_px * 4, (unsigned)(soff + org * W * 4), e0 + wave * kWave * 4);
        }
        wait_global_loads();
        workgroup_sync();
        if (!active) continue;

        // this chunk's part of the rows that see the patch: rectangle rows below RH in the first chunk, the others in
        // the second
        const int blk_lo = c ? (C::RH - row0 > 0 ? C::RH - row0 : 0) : 0;
        const int blk_hi = (nch == 2 && c == 0) ? (nblk < C::RH - row0 ? nblk : C::RH - row0) : nblk;
        for (int blk = blk_lo; blk < blk_hi; ++blk) {
            const int xr = (row0 + blk - org) * C::RW * KB;   // this row inside the q / dout images
            const int sr = (row0 + blk - org) * C::SP * 4;    // ... inside the fp32 images
            const u32x4 aq = *lds_ptr<u32x4>(q0 + xr + arow);
            const u32x4 ad = *lds_ptr<u32x4>(d0 + xr + arow);
            struct __attribute__((packed, aligned(4))) F4 {
                f32x4 v;
            };
            const f32x4 l4 = lds_ptr<F4>(l0 + sr + sidx)->v;
            const f32x4 e4 = lds_ptr<F4>(e0 + sr + sidx)->v;
            int u = ub - blk;
            u = u < 0 ? 0 : (u > C::NB - 1 ? C::NB - 1 : u);
            typedef uint32_t u32v2 __attribute__((ext_vector_type(2)));
            const u32v2 b4 = *lds_ptr<u32v2>(cbase + u * C::BP * 2);
            const f32x4 sacc = mfma_16x16x32<T>(aq, kreg, f32x4{0.f, 0.f, 0.f, 0.f});
            const f32x4 pacc = mfma_16x16x32<T>(ad, vreg, f32x4{0.f, 0.f, 0.f, 0.f});
            // the window test as an additive mask (0 inside, -inf outside: the weight becomes exactly 0), so that the
            // block stays free of branches
            const float rowmask = ((rowok >> blk) & 1u) ? 0.f : -INFINITY;
            float pw[4], ds[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t two = r < 2 ? b4.x : b4.y;
                const float bias = (float)__builtin_bit_cast(f16_t, (uint16_t)((r & 1) ? two >> 16 : two & 0xffffu));
                const float lg = __builtin_fmaf(scale, sacc[r], bias + (colmask[r] + rowmask));   // the logit, -inf outside the window
                pw[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(lg, kLog2e, -l4[r]));
                ds[r] = pw[r] * (pacc[r] - e4[r]);
            }
            const uint32_t p0 = pack2_t<T>(pw[0], pw[1]), p1 = pack2_t<T>(pw[2], pw[3]);
            const uint32_t s0 = pack2_t<T>(ds[0], ds[1]), s1 = pack2_t<T>(ds[2], ds[3]);
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const u32x2 td = lds_read_tr16(d0 + xr + atr + hf * 8);
                const u32x2 tq = lds_read_tr16(q0 + xr + atr + hf * 8);
                av[hf] = mfma_16x16x16<T>(td.x, td.y, p0, p1, av[hf]);
                ak[hf] = mfma_16x16x16<T>(tq.x, tq.y, s0, s1, ak[hf]);
                if constexpr (Traits<T>::kDtype == NA2D_BF16) {
                    // bf16 keeps 8 significant bits: second operands carry the rounding remainders of P and dS
                    auto rem = [](float x) { return x - to_f32(from_f32<T>(x)); };
                    av[hf] = mfma_16x16x16<T>(td.x, td.y, pack2_t<T>(rem(pw[0]), rem(pw[1])), pack2_t<T>(rem(pw[2]), rem(pw[3])), av[hf]);
                    ak[hf] = mfma_16x16x16<T>(tq.x, tq.y, pack2_t<T>(rem(ds[0]), rem(ds[1])), pack2_t<T>(rem(ds[2]), rem(ds[3])), ak[hf]);
                }
            }
        }
        }   // chunks
        if (key_ok && !upper) {
            const size_t o = (plane * plane_px + (size_t)jy * W + jx) * pitch + g * 16;
            store16_stream(reinterpret_cast<char *>(dk) + o,
                           u32x4{pack2_t<T>(ak[0][0] * scale, ak[0][1] * scale), pack2_t<T>(ak[0][2] * scale, ak[0][3] * scale),
                                 pack2_t<T>(ak[1][0] * scale, ak[1][1] * scale), pack2_t<T>(ak[1][2] * scale, ak[1][3] * scale)});
            store16_stream(reinterpret_cast<char *>(dv) + o,
                           u32x4{pack2_t<T>(av[0][0], av[0][1]), pack2_t<T>(av[0][2], av[0][3]), pack2_t<T>(av[1][0], av[1][1]),
                                 pack2_t<T>(av[1][2], av[1][3])});
        }
    }
}

// Does the query rectangle of every 16 x 8 key tile fit rows x cols positions?
static bool kv_rect_fits(const Problem &p, int rows, int cols) {
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

template <typename T, int K, bool COMPACT>
static hipError_t launch_fbwd_kv_c(const Problem &p, const void *q, const void *k, const void *v, const void *rpb,
                                   float scale, const float *lse, const float *delta, const void *dout, void *dk, void *dv,
                                   hipStream_t s) {
    using C = FbwdKvCfg<T, K, COMPACT>;
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + C::TY - 1) / C::TY;
    const int units = tiles_x * tiles_y * p.heads;
    int splits = (256 * C::kWgPerCu) / units;
    splits = splits < 1 ? 1 : (splits < p.B ? splits : p.B);
    auto kern = fbwd_kv_kernel<T, K, COMPACT>;
    static LdsAllowed allowed;
    if (hipError_t e = allow_lds(kern, C::kLdsBytes, allowed); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(xcd_padded_grid(units * splits)), dim3(C::kThreads), C::kLdsBytes, s,
                       static_cast<const T *>(q), static_cast<const T *>(k), static_cast<const T *>(v),
                       static_cast<const T *>(rpb), scale, lse, delta, static_cast<const T *>(dout), static_cast<T *>(dk),
                       static_cast<T *>(dv), p.H, p.W, p.heads, p.B, tiles_y, units, splits, make_grid_decode(tiles_x, tiles_y, p.heads, p.B, splits),
                       p.D == kHalfDim ? 1 : 0);
    return hipGetLastError();
}

template <typename T, int K>
static hipError_t launch_fbwd_kv_t(const Problem &p, const void *q, const void *k, const void *v, const void *rpb,
                                   float scale, const float *lse, const float *delta, const void *dout, void *dk, void *dv,
                                   hipStream_t s) {
    if constexpr (K > 7) {   // (chunked images: one size)
        return launch_fbwd_kv_c<T, K, false>(p, q, k, v, rpb, scale, lse, delta, dout, dk, dv, s);
    } else {
        return kv_rect_fits(p, 8 + K - 1, kTileX + K - 1)
                   ? launch_fbwd_kv_c<T, K, true>(p, q, k, v, rpb, scale, lse, delta, dout, dk, dv, s)
                   : launch_fbwd_kv_c<T, K, false>(p, q, k, v, rpb, scale, lse, delta, dout, dk, dv, s);
    }
}

hipError_t launch_fbwd_kv(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                          const float *lse, const float *delta, const void *dout, void *dk, void *dv, hipStream_t s) {
#define NA2D_FBKV_K(TT)                                                                                   \
    switch (p.K) {                                                                                        \
        case 3: return launch_fbwd_kv_t<TT, 3>(p, q, k, v, rpb, scale, lse, delta, dout, dk, dv, s);      \
        case 5: return launch_fbwd_kv_t<TT, 5>(p, q, k, v, rpb, scale, lse, delta, dout, dk, dv, s);      \
        case 7: return launch_fbwd_kv_t<TT, 7>(p, q, k, v, rpb, scale, lse, delta, dout, dk, dv, s);      \
        case 9: return launch_fbwd_kv_t<TT, 9>(p, q, k, v, rpb, scale, lse, delta, dout, dk, dv, s);      \
        default: return hipErrorInvalidValue;                                                             \
    }
    if (p.dtype == NA2D_F16) { NA2D_FBKV_K(f16_t) }
    if (p.dtype == NA2D_BF16) { NA2D_FBKV_K(bf16_t) }
#undef NA2D_FBKV_K
    return hipErrorInvalidValue;
}

// Is every 4-column key patch seen from at most 16 query columns (one MFMA block per rectangle row)?  Always so
// away from short axes (K + (K-1)/2 + 3 <= 16 columns); on an axis of at most 2K + 2 positions a patch can be seen
// from both clamped ends at once, and then it depends on the length.
static bool kv_patch_cols_fit(const Problem &p) {
    for (int px = 0; px < p.W; px += 4)
        if (inv_last(px + 3 < p.W - 1 ? px + 3 : p.W - 1, p.W, p.K) - inv_first(px, p.W, p.K) + 1 > 16) return false;
    return true;
}

// The second kernel sizes its images for key tiles that are next to at most one border per axis: a 16 x 8 tile
// whose query rectangle exceeds (8 + K-1 + R) x (16 + K-1 + R) positions (short axes, where a ragged tile is
// close to both borders) does not fit, and such maps take the unfused steps instead.
bool fused_bwd_supported(const Problem &p) {
    const int R = p.K / 2;
    return (p.D == kHeadDim || p.D == kHalfDim) && p.dtype != NA2D_F32 && p.K <= 9 && kv_patch_cols_fit(p) &&
           kv_rect_fits(p, 8 + p.K - 1 + R, kTileX + p.K - 1 + R);
}

AvRpbSplit fused_bwd_split(const Problem &p) {
    const int tiles_x = (p.W + kTileX - 1) / kTileX, tiles_y = (p.H + 7) / 8;
    const UnitSplit us = unit_split(tiles_x, tiles_y, p.heads, p.B);
    return AvRpbSplit{us.units / p.heads, us.splits};
}

hipError_t launch_fbwd_q(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                         const float *lse, const void *dout, void *dq, float *delta, float *lse2, float *rpb_partial,
                         hipStream_t s) {
#define NA2D_FBQ_K(TT)                                                                                             \
    switch (p.K) {                                                                                                 \
        case 3: return launch_fbwd_q_t<TT, 3>(p, q, k, v, rpb, scale, lse, dout, dq, delta, lse2, rpb_partial, s);       \
        case 5: return launch_fbwd_q_t<TT, 5>(p, q, k, v, rpb, scale, lse, dout, dq, delta, lse2, rpb_partial, s);       \
        case 7: return launch_fbwd_q_t<TT, 7>(p, q, k, v, rpb, scale, lse, dout, dq, delta, lse2, rpb_partial, s);       \
        case 9: return launch_fbwd_q_t<TT, 9>(p, q, k, v, rpb, scale, lse, dout, dq, delta, lse2, rpb_partial, s);       \
        default: return hipErrorInvalidValue;                                                                      \
    }
    if (p.dtype == NA2D_F16) { NA2D_FBQ_K(f16_t) }
    if (p.dtype == NA2D_BF16) { NA2D_FBQ_K(bf16_t) }
#undef NA2D_FBQ_K
    return hipErrorInvalidValue;
}

}  // namespace na2d
