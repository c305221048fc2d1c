/*
 * tbn_oracle.c -- plain CPU oracle for the tiled-bit layer (Tiled Bit Networks,
 * arXiv 2407.12075).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is slow on purpose, shares no code with the
 * HIP library, and must never be called from the product path: only tests,
 * the smoke check and the CPU-baseline leg of the benchmark may use it.
 *
 * Every function writes out one definition from the paper's Method section:
 *   - tile construction   : Eq. 1 (reshape), Eq. 2 (sum), Eq. 3 (threshold)
 *   - scalars             : Eq. 6 (one alpha), Eq. 7-8 (one alpha per tile)
 *   - dense weight        : Eq. 4 (replicate), Eq. 5 (reshape), then the
 *                           alpha multiplication described after Eq. 8
 *   - layer operation     : Y = X * B_hat^T, and the matching cross-correlation
 *   - Algorithm 1         : the running-index fully-connected forward pass
 *
 * Notation used here (the paper's letters in brackets):
 *   n  number of weights of the layer            [N]
 *   k  number of tile repeats = compression rate [p]
 *   p  tile length in bits, p = n / k            [q]
 *
 * Readings of places where the paper's text is ambiguous:
 *   - Eq. 1-2: the flattened weight (row-major, last index fastest) is viewed
 *     as k rows of p entries and summed over the k rows; position i of the sum
 *     collects exactly the weights that later share tile entry i in Eq. 4.
 *   - Eq. 4: the tile is repeated k times back to back (b[f] = t[f mod p]).
 *   - Eq. 7-8: alpha_r is the mean absolute value of the r-th contiguous
 *     segment of length p of the flattened tensor.
 *   - Eq. 3: s_i > 0 gives +1, everything else (zero, negative, NaN) gives -1.
 *   - sums for Eq. 2, 6, 8 are taken in double precision, terms in ascending
 *     flat index, and alpha is rounded once to float.
 *   - Algorithm 1 is read as: weight of flat position f = i*in + j is
 *     t[f mod p] * alpha[f div p]; the stray increment of alpha in the outer
 *     loop is ignored and the wrap happens when the next index would be p.
 *
 * Tile storage: 32-bit words, entry i in word i/32 at bit i%32 (LSB first),
 * bit 1 <-> +1, bit 0 <-> -1, unused high bits of the last word are zero.
 *
 * All pointers are host pointers.  Return value 0 = ok, nonzero = bad argument.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int tbn_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. 1-3 and Eq. 6 / Eq. 7-8.  a may be NULL (then w is used for alpha). */
int tbn_oracle_pack_tile(const float *w, const float *a, int64_t n, int32_t k,
                         int32_t n_alpha, uint32_t *tile_out, float *alpha_out)
{
    if (!w || !tile_out || !alpha_out) return 1;
    if (n <= 0 || k <= 0 || n % k != 0) return 2;
    if (n_alpha != 1 && n_alpha != k) return 2;
    const int64_t p = n / k;
    const int64_t words = (p + 31) / 32;
    for (int64_t wi = 0; wi < words; ++wi) tile_out[wi] = 0u;

    /* Eq. 2: s_i = sum over the k rows of the (k x p) view; Eq. 3: threshold */
    for (int64_t i = 0; i < p; ++i) {
        double s = 0.0;
        for (int32_t r = 0; r < k; ++r) s += (double)w[(int64_t)r * p + i];
        if (s > 0.0) tile_out[i >> 5] |= (1u << (i & 31));
    }

    const float *src = a ? a : w;
    if (n_alpha == 1) {
        /* Eq. 6: alpha = ||A||_1 / n */
        double l1 = 0.0;
        for (int64_t f = 0; f < n; ++f) l1 += fabs((double)src[f]);
        alpha_out[0] = (float)(l1 / (double)n);
    } else {
        /* Eq. 8: alpha_r = ||segment r||_1 / p */
        for (int32_t r = 0; r < k; ++r) {
            double l1 = 0.0;
            for (int64_t i = 0; i < p; ++i) l1 += fabs((double)src[(int64_t)r * p + i]);
            alpha_out[r] = (float)(l1 / (double)p);
        }
    }
    return 0;
}

/* Eq. 4-5 followed by the alpha scaling: w_hat[f] = alpha[f div p] * t[f mod p]. */
int tbn_oracle_materialise(const uint32_t *tile, const float *alpha, int32_t n_alpha,
                           int64_t n, int32_t k, double *w_hat)
{
    if (!tile || !alpha || !w_hat) return 1;
    if (n <= 0 || k <= 0 || n % k != 0) return 2;
    if (n_alpha != 1 && n_alpha != k) return 2;
    const int64_t p = n / k;
    for (int32_t r = 0; r < k; ++r) {
        const double scale = (double)alpha[n_alpha == 1 ? 0 : r];
        for (int64_t i = 0; i < p; ++i) {
            const int bit = (int)((tile[i >> 5] >> (i & 31)) & 1u);
            w_hat[(int64_t)r * p + i] = bit ? scale : -scale;
        }
    }
    return 0;
}

/* Fully-connected layer, no bias: y[m,o] = sum_j x[m,j] * w_hat[o,j]. */
int tbn_oracle_linear(const double *x, int64_t M, int64_t in, int64_t out,
                      const double *w_hat, double *y)
{
    if (!x || !w_hat || !y) return 1;
    if (M < 0 || in <= 0 || out <= 0) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t o = 0; o < out; ++o) {
            double acc = 0.0;
            for (int64_t j = 0; j < in; ++j) acc += x[m * in + j] * w_hat[o * in + j];
            y[m * out + o] = acc;
        }
    }
    return 0;
}

/* Selected outputs of the fully-connected layer: y_s[q] = y[rows[q], cols[q]]. */
int tbn_oracle_linear_at(const double *x, int64_t M, int64_t in, int64_t out,
                         const double *w_hat, const int64_t *rows, const int64_t *cols,
                         int64_t count, double *y_s)
{
    if (!x || !w_hat || !rows || !cols || !y_s) return 1;
    if (M <= 0 || in <= 0 || out <= 0 || count < 0) return 2;
    for (int64_t q = 0; q < count; ++q)
        if (rows[q] < 0 || rows[q] >= M || cols[q] < 0 || cols[q] >= out) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < count; ++q) {
        const double *xr = x + rows[q] * in;
        const double *wr = w_hat + cols[q] * in;
        double acc = 0.0;
        for (int64_t j = 0; j < in; ++j) acc += xr[j] * wr[j];
        y_s[q] = acc;
    }
    return 0;
}

/*
 * 2-D convolution layer as deep-learning frameworks define it (cross-correlation,
 * zero padding, no bias, dilation 1, one group); x is (N,C,H,W), w_hat is
 * (O,C,kh,kw), y is (N,O,Ho,Wo), all row-major.
 */
int tbn_oracle_conv2d(const double *x, int64_t N, int64_t C, int64_t H, int64_t W,
                      int64_t O, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                      int32_t ph, int32_t pw, const double *w_hat, double *y)
{
    if (!x || !w_hat || !y) return 1;
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || O <= 0 || kh <= 0 || kw <= 0 ||
        sh <= 0 || sw <= 0 || ph < 0 || pw < 0) return 2;
    if (H + 2 * ph < kh || W + 2 * pw < kw) return 2;
    const int64_t Ho = (H + 2 * ph - kh) / sh + 1;
    const int64_t Wo = (W + 2 * pw - kw) / sw + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < N; ++b) {
        for (int64_t o = 0; o < O; ++o) {
            for (int64_t yo = 0; yo < Ho; ++yo) {
                for (int64_t xo = 0; xo < Wo; ++xo) {
                    double acc = 0.0;
                    for (int64_t c = 0; c < C; ++c) {
                        for (int32_t dy = 0; dy < kh; ++dy) {
                            const int64_t yi = yo * sh + dy - ph;
                            if (yi < 0 || yi >= H) continue;
                            for (int32_t dx = 0; dx < kw; ++dx) {
                                const int64_t xi = xo * sw + dx - pw;
                                if (xi < 0 || xi >= W) continue;
                                acc += w_hat[((o * C + c) * kh + dy) * kw + dx] *
                                       x[((b * C + c) * H + yi) * W + xi];
                            }
                        }
                    }
                    y[((b * O + o) * Ho + yo) * Wo + xo] = acc;
                }
            }
        }
    }
    return 0;
}

/* Selected outputs of the convolution: idx[q] is a flat index into y (N,O,Ho,Wo). */
int tbn_oracle_conv2d_at(const double *x, int64_t N, int64_t C, int64_t H, int64_t W,
                         int64_t O, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                         int32_t ph, int32_t pw, const double *w_hat,
                         const int64_t *idx, int64_t count, double *y_s)
{
    if (!x || !w_hat || !idx || !y_s) return 1;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || O <= 0 || kh <= 0 || kw <= 0 ||
        sh <= 0 || sw <= 0 || ph < 0 || pw < 0 || count < 0) return 2;
    if (H + 2 * ph < kh || W + 2 * pw < kw) return 2;
    const int64_t Ho = (H + 2 * ph - kh) / sh + 1;
    const int64_t Wo = (W + 2 * pw - kw) / sw + 1;
    for (int64_t q = 0; q < count; ++q)
        if (idx[q] < 0 || idx[q] >= N * O * Ho * Wo) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < count; ++q) {
        int64_t r = idx[q];
        const int64_t xo = r % Wo; r /= Wo;
        const int64_t yo = r % Ho; r /= Ho;
        const int64_t o = r % O;
        const int64_t b = r / O;
        double acc = 0.0;
        for (int64_t c = 0; c < C; ++c)
            for (int32_t dy = 0; dy < kh; ++dy) {
                const int64_t yi = yo * sh + dy - ph;
                if (yi < 0 || yi >= H) continue;
                for (int32_t dx = 0; dx < kw; ++dx) {
                    const int64_t xi = xo * sw + dx - pw;
                    if (xi < 0 || xi >= W) continue;
                    acc += w_hat[((o * C + c) * kh + dy) * kw + dx] *
                           x[((b * C + c) * H + yi) * W + xi];
                }
            }
        y_s[q] = acc;
    }
    return 0;
}

/*
 * Algorithm 1 (fully-connected forward pass with tiling and many alphas) for a
 * batch of input vectors: a tile index and an alpha index run over the
 * flattened (out x in) weight without ever being reset at a row start; the
 * tile index returns to zero after entry p-1 and the alpha index then moves on.
 * relu != 0 applies the fused max(0, .) of the listing.
 */
int tbn_oracle_linear_alg1(const double *x, int64_t M, int64_t in, int64_t out,
                           const uint32_t *tile, int64_t p, const float *alpha,
                           int32_t n_alpha, int32_t relu, double *y)
{
    if (!x || !tile || !alpha || !y) return 1;
    if (M < 0 || in <= 0 || out <= 0 || p <= 0 || (in * out) % p != 0) return 2;
    if (n_alpha != 1 && (int64_t)n_alpha != (in * out) / p) return 2;
    for (int64_t m = 0; m < M; ++m) {
        int64_t ti = 0;
        int64_t ai = 0;
        for (int64_t i = 0; i < out; ++i) {
            double acc = 0.0;
            for (int64_t j = 0; j < in; ++j) {
                const double t = ((tile[ti >> 5] >> (ti & 31)) & 1u) ? 1.0 : -1.0;
                acc += t * x[m * in + j] * (double)alpha[ai];
                if (ti == p - 1) {
                    ti = 0;
                    if (n_alpha != 1) ++ai;
                } else {
                    ++ti;
                }
            }
            y[m * out + i] = (relu && acc < 0.0) ? 0.0 : acc;
        }
    }
    return 0;
}
