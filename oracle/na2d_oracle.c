/*
 * CPU oracle for 2D Neighborhood Attention (NA) -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct fp64 implementation of the operation defined in
 * "Neighborhood Attention Transformer" (arXiv 2204.07143), Section 3.1, Eq. 2-4:
 * every pixel attends to its k x k nearest pixels, the window being shifted (never
 * shrunk or zero-padded) at the borders (Section 1; Appendix, figure "3x3 NA on a
 * 7x7 map"), with a relative positional bias B(i, j) added to the logits (Eq. 2).
 *
 * It exists so that tests, the smoke check and the benchmark's CPU-baseline leg can
 * compare the GPU library against something independent.  It shares no code with the
 * HIP path, is never called by the product path, and is not tuned: one loop nest per
 * definition, double accumulation, no blocking, no fusion, no reordering.
 *
 * Parity pins (see tests/test_oracle_*.py): every function below is pinned by at
 * least one check that does not come from this file (dense self-attention at
 * k = H = W, brute-force nearest-k neighbourhoods, box-mean special case, closed-form
 * bias-gradient counts, finite differences, adjoint identities).  No function here is
 * "parity unpinned".
 *
 * Layouts (row-major, last index fastest):
 *   q, k, v, out, dq, dk, dv, dout : [B, heads, H, W, D]
 *   logits, p, dp, ds             : [B, heads, H, W, k*k]   (window slot = a*k + c,
 *                                   raster order over ascending key coordinates)
 *   rpb, d_rpb                    : [heads, 2k-1, 2k-1]
 *   lse                           : [B, heads, H, W]
 *
 * Readings of the paper taken here (the paper gives no index formula):
 *   - the "k nearest neighbours" of Eq. 2 are, per axis, the k positions closest to
 *     the query; with an odd k <= L that set is unique and is the contiguous range
 *     starting at clamp(i - (k-1)/2, 0, L - k); in 2D the neighbourhood is the product
 *     of the two per-axis ranges (the square window of the figures);
 *   - `k` is the window side, so a query has k*k neighbours;
 *   - logit = scale * (Q_i . K_j) + B(i, j): the bias is added unscaled, after the
 *     1/sqrt(d) scale of Eq. 4 has been applied to the dot product (the paper's
 *     software folds the scale into q before its QK+RPB call, Appendix A);
 *   - B(i, j) = rpb[head, (jy - iy) + k - 1, (jx - ix) + k - 1].
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- neighbourhood definition (Section 3.1; Appendix figure) -------------------- */

/* First key coordinate seen by query coordinate i on an axis of length L, window k. */
int na2d_oracle_window_start(int i, int L, int k)
{
    int r = (k - 1) / 2;
    int s = i - r;
    if (s < 0) s = 0;
    if (s > L - k) s = L - k;
    return s;
}

int na2d_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void na2d_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * Index tables for one H x W map: for query (qy, qx) and slot (a, c)
 *   key_index = ky * W + kx, rpb_index = (ky - qy + k - 1) * (2k - 1) + (kx - qx + k - 1).
 * Both are [H, W, k*k] int32.
 */
void na2d_oracle_indices(int H, int W, int k, int32_t *key_index, int32_t *rpb_index)
{
    int kk = k * k, nb = 2 * k - 1;
    for (int qy = 0; qy < H; ++qy)
        for (int qx = 0; qx < W; ++qx) {
            int sy = na2d_oracle_window_start(qy, H, k);
            int sx = na2d_oracle_window_start(qx, W, k);
            for (int a = 0; a < k; ++a)
                for (int c = 0; c < k; ++c) {
                    int ky = sy + a, kx = sx + c;
                    size_t o = ((size_t)qy * W + qx) * kk + a * k + c;
                    key_index[o] = ky * W + kx;
                    rpb_index[o] = (ky - qy + k - 1) * nb + (kx - qx + k - 1);
                }
        }
}

/* ---- forward (Eq. 2, 3, 4) ------------------------------------------------------ */

/* Eq. 2: logits[n, a, c] = scale * <q_n, k_{rho(n; a, c)}> + B(n, rho(n; a, c)). */
void na2d_oracle_qk_rpb(int B, int heads, int H, int W, int D, int k,
                        const double *q, const double *key, const double *rpb,
                        double scale, double *logits)
{
    int kk = k * k, nb = 2 * k - 1;
#pragma omp parallel for collapse(3) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < heads; ++h)
            for (int qy = 0; qy < H; ++qy) {
                size_t plane = ((size_t)b * heads + h) * H * W;
                for (int qx = 0; qx < W; ++qx) {
                    int sy = na2d_oracle_window_start(qy, H, k);
                    int sx = na2d_oracle_window_start(qx, W, k);
                    const double *qv = q + (plane + (size_t)qy * W + qx) * D;
                    double *lo = logits + (plane + (size_t)qy * W + qx) * kk;
                    for (int a = 0; a < k; ++a)
                        for (int c = 0; c < k; ++c) {
                            int ky = sy + a, kx = sx + c;
                            const double *kv = key + (plane + (size_t)ky * W + kx) * D;
                            double dot = 0.0;
                            for (int d = 0; d < D; ++d) dot += qv[d] * kv[d];
                            double bias = 0.0;
                            if (rpb)
                                bias = rpb[((size_t)h * nb + (ky - qy + k - 1)) * nb + (kx - qx + k - 1)];
                            lo[a * k + c] = scale * dot + bias;
                        }
                }
            }
}

/* Eq. 4's softmax over the k*k axis of `rows` rows; lse (nullable) gets log-sum-exp. */
void na2d_oracle_softmax(size_t rows, int kk, const double *logits, double *p, double *lse)
{
#pragma omp parallel for schedule(static)
    for (size_t n = 0; n < rows; ++n) {
        const double *x = logits + n * kk;
        double *y = p + n * kk;
        double m = x[0];
        for (int j = 1; j < kk; ++j) if (x[j] > m) m = x[j];
        double sum = 0.0;
        for (int j = 0; j < kk; ++j) sum += exp(x[j] - m);
        for (int j = 0; j < kk; ++j) y[j] = exp(x[j] - m) / sum;
        if (lse) lse[n] = m + log(sum);
    }
}

/* Eq. 3-4: out[n, :] = sum_{a, c} p[n, a, c] * v_{rho(n; a, c)}. */
void na2d_oracle_av(int B, int heads, int H, int W, int D, int k,
                    const double *p, const double *v, double *out)
{
    int kk = k * k;
#pragma omp parallel for collapse(3) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < heads; ++h)
            for (int qy = 0; qy < H; ++qy) {
                size_t plane = ((size_t)b * heads + h) * H * W;
                for (int qx = 0; qx < W; ++qx) {
                    int sy = na2d_oracle_window_start(qy, H, k);
                    int sx = na2d_oracle_window_start(qx, W, k);
                    const double *pr = p + (plane + (size_t)qy * W + qx) * kk;
                    double *o = out + (plane + (size_t)qy * W + qx) * D;
                    for (int d = 0; d < D; ++d) o[d] = 0.0;
                    for (int a = 0; a < k; ++a)
                        for (int c = 0; c < k; ++c) {
                            const double *vv = v + (plane + (size_t)(sy + a) * W + (sx + c)) * D;
                            double w = pr[a * k + c];
                            for (int d = 0; d < D; ++d) o[d] += w * vv[d];
                        }
                }
            }
}

/* Eq. 2-4 composed for every pixel; all intermediates stay in double. */
void na2d_oracle_fwd(int B, int heads, int H, int W, int D, int k,
                     const double *q, const double *key, const double *v, const double *rpb,
                     double scale, double *out, double *lse)
{
    size_t rows = (size_t)B * heads * H * W;
    int kk = k * k;
    double *logits = (double *)malloc(rows * kk * sizeof(double));
    double *p = (double *)malloc(rows * kk * sizeof(double));
    na2d_oracle_qk_rpb(B, heads, H, W, D, k, q, key, rpb, scale, logits);
    na2d_oracle_softmax(rows, kk, logits, p, lse);
    na2d_oracle_av(B, heads, H, W, D, k, p, v, out);
    free(logits);
    free(p);
}

/* ---- backward: the chain rule applied to Eq. 2-4 --------------------------------
 * The paper (Appendix A, "Naive CUDA kernels") lists which gradients exist -- for q,
 * k, b (bias), a (attention weights) and v -- not their formulas; these follow from
 * differentiating the forward definitions above.  Gradients that sum over queries
 * (dK, dV, d_rpb) are written as scatter-adds in query order.
 */

/* grad-a: dp[n, a, c] = <dout_n, v_{rho(n; a, c)}>  (derivative of Eq. 4 w.r.t. the weights). */
void na2d_oracle_av_bwd_p(int B, int heads, int H, int W, int D, int k,
                          const double *dout, const double *v, double *dp)
{
    na2d_oracle_qk_rpb(B, heads, H, W, D, k, dout, v, NULL, 1.0, dp);
}

/* grad-v: dv_j = sum over queries n that see j of p[n, slot(n, j)] * dout_n. */
void na2d_oracle_av_bwd_v(int B, int heads, int H, int W, int D, int k,
                          const double *p, const double *dout, double *dv)
{
    int kk = k * k;
    memset(dv, 0, (size_t)B * heads * H * W * D * sizeof(double));
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < heads; ++h) {
            size_t plane = ((size_t)b * heads + h) * H * W;
            for (int qy = 0; qy < H; ++qy)
                for (int qx = 0; qx < W; ++qx) {
                    int sy = na2d_oracle_window_start(qy, H, k);
                    int sx = na2d_oracle_window_start(qx, W, k);
                    const double *pr = p + (plane + (size_t)qy * W + qx) * kk;
                    const double *go = dout + (plane + (size_t)qy * W + qx) * D;
                    for (int a = 0; a < k; ++a)
                        for (int c = 0; c < k; ++c) {
                            double *g = dv + (plane + (size_t)(sy + a) * W + (sx + c)) * D;
                            double w = pr[a * k + c];
                            for (int d = 0; d < D; ++d) g[d] += w * go[d];
                        }
                }
        }
}

/* softmax backward: ds = p * (dp - <p, dp>) per row. */
void na2d_oracle_softmax_bwd(size_t rows, int kk, const double *p, const double *dp, double *ds)
{
#pragma omp parallel for schedule(static)
    for (size_t n = 0; n < rows; ++n) {
        const double *pr = p + n * kk, *g = dp + n * kk;
        double *o = ds + n * kk;
        double inner = 0.0;
        for (int j = 0; j < kk; ++j) inner += pr[j] * g[j];
        for (int j = 0; j < kk; ++j) o[j] = pr[j] * (g[j] - inner);
    }
}

/* grad-q: dq_n = scale * sum_{a, c} ds[n, a, c] * k_{rho(n; a, c)}. */
void na2d_oracle_qk_bwd_q(int B, int heads, int H, int W, int D, int k,
                          const double *ds, const double *key, double scale, double *dq)
{
    size_t n = (size_t)B * heads * H * W * D;
    na2d_oracle_av(B, heads, H, W, D, k, ds, key, dq);
    for (size_t i = 0; i < n; ++i) dq[i] *= scale;
}

/* grad-k: dk_j = scale * sum over queries n that see j of ds[n, slot(n, j)] * q_n. */
void na2d_oracle_qk_bwd_k(int B, int heads, int H, int W, int D, int k,
                          const double *ds, const double *q, double scale, double *dk)
{
    size_t n = (size_t)B * heads * H * W * D;
    na2d_oracle_av_bwd_v(B, heads, H, W, D, k, ds, q, dk);
    for (size_t i = 0; i < n; ++i) dk[i] *= scale;
}

/* grad-b: d_rpb[h, u, v] = sum over batch, queries and slots whose bias cell is (u, v) of ds. */
void na2d_oracle_qk_bwd_rpb(int B, int heads, int H, int W, int k,
                            const double *ds, double *d_rpb)
{
    int kk = k * k, nb = 2 * k - 1;
    memset(d_rpb, 0, (size_t)heads * nb * nb * sizeof(double));
#pragma omp parallel for schedule(static)
    for (int h = 0; h < heads; ++h)
        for (int b = 0; b < B; ++b) {
            size_t plane = ((size_t)b * heads + h) * H * W;
            for (int qy = 0; qy < H; ++qy)
                for (int qx = 0; qx < W; ++qx) {
                    int sy = na2d_oracle_window_start(qy, H, k);
                    int sx = na2d_oracle_window_start(qx, W, k);
                    const double *g = ds + (plane + (size_t)qy * W + qx) * kk;
                    for (int a = 0; a < k; ++a)
                        for (int c = 0; c < k; ++c) {
                            int u = (sy + a) - qy + k - 1, vv = (sx + c) - qx + k - 1;
                            d_rpb[((size_t)h * nb + u) * nb + vv] += g[a * k + c];
                        }
                }
        }
}

/*
 * Whole backward in double: recomputes the forward, then applies the six gradient
 * steps in order.  d_rpb may be NULL when rpb is NULL.
 */
void na2d_oracle_bwd(int B, int heads, int H, int W, int D, int k,
                     const double *q, const double *key, const double *v, const double *rpb,
                     double scale, const double *dout,
                     double *dq, double *dk, double *dv, double *d_rpb)
{
    size_t rows = (size_t)B * heads * H * W;
    int kk = k * k;
    double *logits = (double *)malloc(rows * kk * sizeof(double));
    double *p = (double *)malloc(rows * kk * sizeof(double));
    double *dp = (double *)malloc(rows * kk * sizeof(double));
    na2d_oracle_qk_rpb(B, heads, H, W, D, k, q, key, rpb, scale, logits);
    na2d_oracle_softmax(rows, kk, logits, p, NULL);
    na2d_oracle_av_bwd_p(B, heads, H, W, D, k, dout, v, dp);
    na2d_oracle_av_bwd_v(B, heads, H, W, D, k, p, dout, dv);
    na2d_oracle_softmax_bwd(rows, kk, p, dp, logits /* reuse as ds */);
    na2d_oracle_qk_bwd_q(B, heads, H, W, D, k, logits, key, scale, dq);
    na2d_oracle_qk_bwd_k(B, heads, H, W, D, k, logits, q, scale, dk);
    if (d_rpb) na2d_oracle_qk_bwd_rpb(B, heads, H, W, k, logits, d_rpb);
    free(logits);
    free(p);
    free(dp);
}
