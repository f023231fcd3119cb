// Neighbourhood attention for window sides beyond the tuned ones (odd K from 15 up to kMaxGenericK): the same
// operations as the tiled kernels (arXiv 2204.07143, Eq. 2-4 and the gradients of Appendix A) with the window
// side as a run-time argument.  The paper tunes its kernels for sides 3 to 13 and lets anything else take a
// plain path; so does this library.  Plain formulations, one thread per output element (one wave per row for
// the softmax, one wave per query for the fused forward), fp32 arithmetic, any of the three storage types and
// any head dim that is a whole number of 16-byte chunks.  Operands are read straight from global memory: at
// these sizes a query's window (225 positions and more) no longer fits the tiles the tuned kernels are built
// around, and the neighbouring threads of a wave read neighbouring keys, so the caches carry the reuse.
#include "na2d_kernels.hpp"
#include "na2d_common.hpp"
#include "na2d_valu_cfg.hpp"

namespace na2d {

namespace {

struct GShape {
    int B, heads, H, W, K, D;
};

// fp32 value of element i of a head vector / row stored as T
template <typename T> __device__ __forceinline__ float ld(const T *p, size_t i) { return to_f32(p[i]); }

// dot product of two head vectors (D elements, 16-byte aligned) in fp32
template <typename T>
__device__ __forceinline__ float dot_vec(const T *a, const T *b, int D) {
    constexpr int EPC = 16 / (int)sizeof(T);
    float acc = 0.f;
    for (int c = 0; c < D / EPC; ++c) {
        const u32x4 ua = reinterpret_cast<const u32x4 *>(a)[c], ub = reinterpret_cast<const u32x4 *>(b)[c];
        const uint32_t wa[4] = {ua.x, ua.y, ua.z, ua.w}, wb[4] = {ub.x, ub.y, ub.z, ub.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if constexpr (sizeof(T) == 4) {
                acc = __builtin_fmaf(__uint_as_float(wa[t]), __uint_as_float(wb[t]), acc);
            } else {
                acc = __builtin_fmaf(to_f32(__builtin_bit_cast(T, (uint16_t)(wa[t] & 0xffffu))),
                                     to_f32(__builtin_bit_cast(T, (uint16_t)(wb[t] & 0xffffu))), acc);
                acc = __builtin_fmaf(to_f32(__builtin_bit_cast(T, (uint16_t)(wa[t] >> 16))),
                                     to_f32(__builtin_bit_cast(T, (uint16_t)(wb[t] >> 16))), acc);
            }
        }
    }
    return acc;
}

// logits[n, a, c] = scale <x_n, y_key(n; a, c)> + bias: one thread per (query, slot)
template <typename T>
__global__ __launch_bounds__(256) void qk_generic_kernel(const T *__restrict__ x, const T *__restrict__ y,
                                                         const T *__restrict__ rpb, float scale, T *__restrict__ logits,
                                                         GShape g, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int KK = g.K * g.K, NB = 2 * g.K - 1;
    const size_t n = idx / KK;
    const int slot = (int)(idx - n * KK), a = slot / g.K, c = slot - a * g.K;
    const size_t plane = n / ((size_t)g.H * g.W);
    const int rest = (int)(n - plane * g.H * g.W), qy = rest / g.W, qx = rest - qy * g.W;
    const int ky = win_start(qy, g.H, g.K) + a, kx = win_start(qx, g.W, g.K) + c;
    const size_t key = (plane * g.H + ky) * g.W + kx;
    float v = scale * dot_vec(x + n * g.D, y + key * g.D, g.D);
    if (rpb != nullptr) {
        const int h = (int)(plane % g.heads);
        v += ld(rpb, ((size_t)h * NB + (ky - qy + g.K - 1)) * NB + (kx - qx + g.K - 1));
    }
    logits[idx] = from_f32<T>(v);
}

// out[n, d] = scale sum_slot w[n, slot] y_key(n; slot)[d]: one thread per (query, channel)
template <typename T>
__global__ __launch_bounds__(256) void av_generic_kernel(const T *__restrict__ w, const T *__restrict__ y, float scale,
                                                         T *__restrict__ out, GShape g, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int KK = g.K * g.K;
    const size_t n = idx / g.D;
    const int d = (int)(idx - n * g.D);
    const size_t plane = n / ((size_t)g.H * g.W);
    const int rest = (int)(n - plane * g.H * g.W), qy = rest / g.W, qx = rest - qy * g.W;
    const int sy = win_start(qy, g.H, g.K), sx = win_start(qx, g.W, g.K);
    const T *wr = w + n * KK;
    float acc = 0.f;
    for (int a = 0; a < g.K; ++a) {
        const T *yr = y + ((plane * g.H + sy + a) * g.W + sx) * g.D + d;
        for (int c = 0; c < g.K; ++c) acc = __builtin_fmaf(ld(wr, a * g.K + c), ld(yr, (size_t)c * g.D), acc);
    }
    out[idx] = from_f32<T>(scale * acc);
}

// out[j, d] = scale sum over the queries i that see key j of w[i, slot(i, j)] x_i[d]: one thread per (key, channel),
// the inverse neighbourhood walked in raster order (no atomics, one fixed order of additions)
template <typename T>
__global__ __launch_bounds__(256) void inverse_generic_kernel(const T *__restrict__ w, const T *__restrict__ x, float scale,
                                                              T *__restrict__ out, GShape g, size_t total) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int KK = g.K * g.K;
    const size_t j = idx / g.D;
    const int d = (int)(idx - j * g.D);
    const size_t plane = j / ((size_t)g.H * g.W);
    const int rest = (int)(j - plane * g.H * g.W), jy = rest / g.W, jx = rest - jy * g.W;
    const int y0 = inv_first(jy, g.H, g.K), y1 = inv_last(jy, g.H, g.K);
    const int x0 = inv_first(jx, g.W, g.K), x1 = inv_last(jx, g.W, g.K);
    float acc = 0.f;
    for (int iy = y0; iy <= y1; ++iy) {
        const int a = jy - win_start(iy, g.H, g.K);
        for (int ix = x0; ix <= x1; ++ix) {
            const int c = jx - win_start(ix, g.W, g.K);
            const size_t i = (plane * g.H + iy) * g.W + ix;
            acc = __builtin_fmaf(ld(w, i * KK + a * g.K + c), ld(x, i * g.D + d), acc);
        }
    }
    out[idx] = from_f32<T>(scale * acc);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// softmax of one row per wave (max-subtracted, fp32); out may alias in: a lane reads element i before it writes it
template <typename T>
__global__ __launch_bounds__(256) void softmax_generic_kernel(const T *in, T *out, int KK, size_t nrows) {
    const size_t row = (size_t)blockIdx.x * 4 + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    if (row >= nrows) return;
    const T *r = in + row * KK;
    float m = -INFINITY;
    for (int i = lane; i < KK; i += kWave) m = fmaxf(m, ld(r, i));
    m = wave_max(m);
    float l = 0.f;
    for (int i = lane; i < KK; i += kWave) l += __expf(ld(r, i) - m);
    l = wave_sum(l);
    const float inv = 1.f / l;
    T *o = out + row * KK;
    for (int i = lane; i < KK; i += kWave) o[i] = from_f32<T>(__expf(ld(r, i) - m) * inv);
}

// ds = attn * (dp - <attn, dp>), one row per wave; ds may alias dp
template <typename T>
__global__ __launch_bounds__(256) void softmax_bwd_generic_kernel(const T *attn, const T *dp, T *ds, int KK, size_t nrows) {
    const size_t row = (size_t)blockIdx.x * 4 + threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    if (row >= nrows) return;
    const T *pr = attn + row * KK, *dr = dp + row * KK;
    float dot = 0.f;
    for (int i = lane; i < KK; i += kWave) dot = __builtin_fmaf(ld(pr, i), ld(dr, i), dot);
    dot = wave_sum(dot);
    T *o = ds + row * KK;
    for (int i = lane; i < KK; i += kWave) o[i] = from_f32<T>(ld(pr, i) * (ld(dr, i) - dot));
}

// Fused forward, one wave per query: the logits of its K*K window go to the wave's LDS row (lanes over slots),
// max and sum by wave reductions, then the lanes turn to the channels and add up the weighted values.
template <typename T>
__global__ __launch_bounds__(256) void fused_generic_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                            const T *__restrict__ v, const T *__restrict__ rpb, float scale,
                                                            T *__restrict__ out, float *__restrict__ lse, GShape g, size_t nq) {
    extern __shared__ __align__(16) char lds[];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int KK = g.K * g.K, NB = 2 * g.K - 1;
    float *row = reinterpret_cast<float *>(lds) + (size_t)wave * KK;
    const size_t n = (size_t)blockIdx.x * 4 + wave;
    if (n >= nq) return;
    const size_t plane = n / ((size_t)g.H * g.W);
    const int rest = (int)(n - plane * g.H * g.W), qy = rest / g.W, qx = rest - qy * g.W;
    const int sy = win_start(qy, g.H, g.K), sx = win_start(qx, g.W, g.K);
    const int h = (int)(plane % g.heads);
    float m = -INFINITY;
    for (int slot = lane; slot < KK; slot += kWave) {
        const int a = slot / g.K, c = slot - a * g.K;
        const size_t key = (plane * g.H + sy + a) * g.W + sx + c;
        float s = scale * dot_vec(q + n * g.D, k + key * g.D, g.D);
        if (rpb != nullptr) s += ld(rpb, ((size_t)h * NB + (sy + a - qy + g.K - 1)) * NB + (sx + c - qx + g.K - 1));
        row[slot] = s;
        m = fmaxf(m, s);
    }
    m = wave_max(m);
    float l = 0.f;
    for (int slot = lane; slot < KK; slot += kWave) {
        const float p = __expf(row[slot] - m);
        row[slot] = p;
        l += p;
    }
    l = wave_sum(l);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const float inv = 1.f / l;
    for (int d = lane; d < g.D; d += kWave) {
        float acc = 0.f;
        for (int a = 0; a < g.K; ++a) {
            const T *vr = v + ((plane * g.H + sy + a) * g.W + sx) * g.D + d;
            for (int c = 0; c < g.K; ++c) acc = __builtin_fmaf(row[a * g.K + c], ld(vr, (size_t)c * g.D), acc);
        }
        out[n * g.D + d] = from_f32<T>(acc * inv);
    }
    if (lse != nullptr && lane == 0) lse[n] = m + __logf(l);
}

// Bias gradient, first level: one partial table per plane, one thread per cell (u, v), the queries whose window
// puts a slot on that cell walked in raster order.
template <typename T>
__global__ __launch_bounds__(256) void rpb_generic_partial_kernel(const T *__restrict__ ds, float *__restrict__ partial, GShape g) {
    const int NB = 2 * g.K - 1, cells = NB * NB, KK = g.K * g.K;
    const int cell_blocks = (cells + 255) / 256;
    const size_t plane = blockIdx.x / cell_blocks;
    const int cell = (int)(blockIdx.x - plane * cell_blocks) * 256 + threadIdx.x;
    if (cell >= cells) return;
    const int u = cell / NB, vv = cell - u * NB;
    float acc = 0.f;
    for (int qy = 0; qy < g.H; ++qy) {
        const int a = u - rpb_start(qy, g.H, g.K);
        if ((unsigned)a >= (unsigned)g.K) continue;
        for (int qx = 0; qx < g.W; ++qx) {
            const int c = vv - rpb_start(qx, g.W, g.K);
            if ((unsigned)c >= (unsigned)g.K) continue;
            acc += ld(ds, ((plane * g.H + qy) * g.W + qx) * KK + a * g.K + c);
        }
    }
    partial[plane * cells + cell] = acc;
}
// second level: the planes of a head in batch order
__global__ __launch_bounds__(256) void rpb_generic_final_kernel(const float *__restrict__ partial, float *__restrict__ d_rpb,
                                                                int B, int heads, int cells) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= heads * cells) return;
    const int h = i / cells, cell = i - h * cells;
    float acc = 0.f;
    for (int b = 0; b < B; ++b) acc += partial[((size_t)b * heads + h) * cells + cell];
    d_rpb[i] = acc;
}

__global__ __launch_bounds__(256) void indices_generic_kernel(int32_t *key_index, int32_t *rpb_index, int H, int W, int K) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int KK = K * K, NB = 2 * K - 1;
    if (i >= H * W * KK) return;
    const int slot = i % KK, qlin = i / KK;
    const int qy = qlin / W, qx = qlin % W;
    const int a = slot / K, c = slot % K;
    if (key_index) key_index[i] = (win_start(qy, H, K) + a) * W + win_start(qx, W, K) + c;
    if (rpb_index) rpb_index[i] = (rpb_start(qy, H, K) + a) * NB + (rpb_start(qx, W, K) + c);
}

GShape shape_of(const Problem &p) { return GShape{p.B, p.heads, p.H, p.W, p.K, p.D}; }
unsigned blocks_for(size_t total) { return (unsigned)((total + 255) / 256); }

}  // namespace

// Which problems take these kernels: window sides beyond the tuned ones, and the combinations of dtype, window and
// head dim whose plain-ALU tiles do not fit the LDS (fp32 with D >= 64 and a larger window, D = 128 in 16 bit with
// k >= 11): the kernels here stage nothing in LDS, so they take every head dim.
bool generic_window(const Problem &p) { return p.K > kMaxTunedK || !head_dim_supported(p.dtype, p.K, p.D); }
bool untuned_window(const Problem &p) { return p.K > kMaxTunedK; }

hipError_t launch_qk_generic(const Problem &p, const void *x, const void *y, const void *rpb, float scale, void *logits,
                             hipStream_t s) {
    const size_t total = p.queries() * p.K * p.K;
    NA2D_DISPATCH_T(p.dtype, hipLaunchKernelGGL((qk_generic_kernel<T>), dim3(blocks_for(total)), dim3(256), 0, s,
                                                static_cast<const T *>(x), static_cast<const T *>(y), static_cast<const T *>(rpb),
                                                scale, static_cast<T *>(logits), shape_of(p), total));
    return hipGetLastError();
}

hipError_t launch_av_generic(const Problem &p, const void *w, const void *y, float scale, void *out, hipStream_t s) {
    const size_t total = p.queries() * p.D;
    NA2D_DISPATCH_T(p.dtype, hipLaunchKernelGGL((av_generic_kernel<T>), dim3(blocks_for(total)), dim3(256), 0, s,
                                                static_cast<const T *>(w), static_cast<const T *>(y), scale, static_cast<T *>(out),
                                                shape_of(p), total));
    return hipGetLastError();
}

hipError_t launch_inverse_generic(const Problem &p, const void *w, const void *x, float scale, void *out, hipStream_t s) {
    const size_t total = p.queries() * p.D;
    NA2D_DISPATCH_T(p.dtype, hipLaunchKernelGGL((inverse_generic_kernel<T>), dim3(blocks_for(total)), dim3(256), 0, s,
                                                static_cast<const T *>(w), static_cast<const T *>(x), scale, static_cast<T *>(out),
                                                shape_of(p), total));
    return hipGetLastError();
}

hipError_t launch_softmax_generic(const Problem &p, const void *in, void *out, hipStream_t s) {
    const size_t rows = p.queries();
    NA2D_DISPATCH_T(p.dtype, hipLaunchKernelGGL((softmax_generic_kernel<T>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s,
                                                static_cast<const T *>(in), static_cast<T *>(out), p.K * p.K, rows));
    return hipGetLastError();
}

hipError_t launch_softmax_bwd_generic(const Problem &p, const void *attn, const void *dp, void *ds, hipStream_t s) {
    const size_t rows = p.queries();
    NA2D_DISPATCH_T(p.dtype, hipLaunchKernelGGL((softmax_bwd_generic_kernel<T>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s,
                                                static_cast<const T *>(attn), static_cast<const T *>(dp), static_cast<T *>(ds),
                                                p.K * p.K, rows));
    return hipGetLastError();
}

hipError_t launch_fused_generic(const Problem &p, const void *q, const void *k, const void *v, const void *rpb, float scale,
                                void *out, float *lse, hipStream_t s) {
    const size_t nq = p.queries();
    const int lds_bytes = 4 * p.K * p.K * (int)sizeof(float);   // at most 62 KB (K = 63): below the default limit
    NA2D_DISPATCH_T(p.dtype, hipLaunchKernelGGL((fused_generic_kernel<T>), dim3((unsigned)((nq + 3) / 4)), dim3(256), lds_bytes, s,
                                                static_cast<const T *>(q), static_cast<const T *>(k), static_cast<const T *>(v),
                                                static_cast<const T *>(rpb), scale, static_cast<T *>(out), lse, shape_of(p), nq));
    return hipGetLastError();
}

size_t rpb_generic_workspace_bytes(const Problem &p) {
    const int nb = 2 * p.K - 1;
    return (size_t)p.planes() * nb * nb * sizeof(float);
}

hipError_t launch_rpb_generic(const Problem &p, const void *ds, float *d_rpb, void *workspace, hipStream_t s) {
    const int nb = 2 * p.K - 1, cells = nb * nb;
    NA2D_DISPATCH_T(p.dtype, hipLaunchKernelGGL((rpb_generic_partial_kernel<T>), dim3((unsigned)(((cells + 255) / 256) * (size_t)p.planes())), dim3(256), 0, s,
                                                static_cast<const T *>(ds), static_cast<float *>(workspace), shape_of(p)));
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    hipLaunchKernelGGL(rpb_generic_final_kernel, dim3((p.heads * cells + 255) / 256), dim3(256), 0, s,
                       static_cast<const float *>(workspace), d_rpb, p.B, p.heads, cells);
    return hipGetLastError();
}

hipError_t launch_indices_generic(const Problem &p, int32_t *key_index, int32_t *rpb_index, hipStream_t s) {
    const int n = p.H * p.W * p.K * p.K;
    hipLaunchKernelGGL(indices_generic_kernel, dim3((n + 255) / 256), dim3(256), 0, s, key_index, rpb_index, p.H, p.W, p.K);
    return hipGetLastError();
}

}  // namespace na2d
