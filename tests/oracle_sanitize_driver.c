/*
 * Driver that runs every entry point of oracle/tbn_oracle.c under AddressSanitizer and
 * UndefinedBehaviorSanitizer (tests/test_oracle_sanitize.py compiles both files with
 * -fsanitize=address,undefined and runs the program).  Every buffer is a heap block of exactly the
 * documented size, so that an access one element outside shows up.  The checks themselves are pins:
 * the hand-worked example of tests/golden/hand_worked_pack.txt (Eq. 1-3, 6, 8 and the 2 x 4 layer built
 * from it), and on ragged shapes the agreement of the three independent ways the oracle computes a
 * layer output (dense product, sampled product, Algorithm 1's running index).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int tbn_oracle_pack_tile(const float *w, const float *a, int64_t n, int32_t k, int32_t n_alpha, uint32_t *tile_out,
                         float *alpha_out);
int tbn_oracle_materialise(const uint32_t *tile, const float *alpha, int32_t n_alpha, int64_t n, int32_t k, double *w_hat);
int tbn_oracle_linear(const double *x, int64_t M, int64_t in, int64_t out, const double *w_hat, double *y);
int tbn_oracle_linear_at(const double *x, int64_t M, int64_t in, int64_t out, const double *w_hat, const int64_t *rows,
                         const int64_t *cols, int64_t count, double *y_s);
int tbn_oracle_conv2d(const double *x, int64_t N, int64_t C, int64_t H, int64_t W, int64_t O, int32_t kh, int32_t kw,
                      int32_t sh, int32_t sw, int32_t ph, int32_t pw, const double *w_hat, double *y);
int tbn_oracle_conv2d_at(const double *x, int64_t N, int64_t C, int64_t H, int64_t W, int64_t O, int32_t kh, int32_t kw,
                         int32_t sh, int32_t sw, int32_t ph, int32_t pw, const double *w_hat, const int64_t *idx,
                         int64_t count, double *y_s);
int tbn_oracle_linear_alg1(const double *x, int64_t M, int64_t in, int64_t out, const uint32_t *tile, int64_t p,
                           const float *alpha, int32_t n_alpha, int32_t relu, double *y);

static int failures = 0;
#define CHECK(cond, ...)                              \
    do {                                              \
        if (!(cond)) {                                \
            ++failures;                               \
            fprintf(stderr, "FAIL line %d: ", __LINE__); \
            fprintf(stderr, __VA_ARGS__);             \
            fprintf(stderr, "\n");                    \
        }                                             \
    } while (0)

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double rnd(void)   /* uniform in (-1, 1), splitmix64 */
{
    uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    z ^= z >> 31;
    return (double)(z >> 11) / 4503599627370496.0 - 1.0;
}

static void *exact_alloc(size_t bytes) { return malloc(bytes ? bytes : 1); }

static void hand_worked(void)
{
    const float w_src[8] = {0.3f, -0.2f, 0.1f, -0.4f, -0.5f, 0.1f, -0.1f, 0.6f};
    float *w = exact_alloc(sizeof w_src);
    for (int i = 0; i < 8; ++i) w[i] = w_src[i];
    uint32_t *tile = exact_alloc(sizeof(uint32_t));
    float *a1 = exact_alloc(sizeof(float)), *a2 = exact_alloc(2 * sizeof(float));
    CHECK(tbn_oracle_pack_tile(w, NULL, 8, 2, 1, tile, a1) == 0, "pack, one alpha");
    CHECK(tile[0] == 8u, "tile word %u, want 8", tile[0]);
    CHECK(fabsf(a1[0] - 0.2875f) < 1e-7f, "alpha %g", a1[0]);
    CHECK(tbn_oracle_pack_tile(w, NULL, 8, 2, 2, tile, a2) == 0, "pack, alpha per tile");
    CHECK(tile[0] == 8u && fabsf(a2[0] - 0.25f) < 1e-7f && fabsf(a2[1] - 0.325f) < 1e-7f, "alphas %g %g", a2[0], a2[1]);
    double *w_hat = exact_alloc(8 * sizeof(double));
    CHECK(tbn_oracle_materialise(tile, a2, 2, 8, 2, w_hat) == 0, "materialise");
    double *x = exact_alloc(4 * sizeof(double)), *y = exact_alloc(2 * sizeof(double));
    for (int i = 0; i < 4; ++i) x[i] = i + 1;
    CHECK(tbn_oracle_linear(x, 1, 4, 2, w_hat, y) == 0, "linear");
    CHECK(fabs(y[0] + 0.5) < 1e-7 && fabs(y[1] + 0.65) < 1e-7, "y = %g %g, want -0.5 -0.65", y[0], y[1]);
    CHECK(tbn_oracle_linear_alg1(x, 1, 4, 2, tile, 4, a1, 1, 0, y) == 0, "alg1");
    CHECK(fabs(y[0] + 0.575) < 1e-7 && fabs(y[1] + 0.575) < 1e-7, "alg1 y = %g %g, want -0.575 twice", y[0], y[1]);
    free(w); free(tile); free(a1); free(a2); free(w_hat); free(x); free(y);
}

/* a fully-connected layer with a tile that ends inside rows and inside a word */
static void ragged_linear(int64_t M, int64_t in, int64_t out, int32_t k, int32_t n_alpha)
{
    const int64_t n = in * out, p = n / k;
    float *w = exact_alloc(n * sizeof(float));
    for (int64_t i = 0; i < n; ++i) w[i] = (float)rnd();
#ifdef PLANT_SHORT_TILE   /* shows that the sanitizer is active: the tile buffer lacks its last word */
    uint32_t *tile = exact_alloc(((p + 31) / 32 - 1) * sizeof(uint32_t));
#else
    uint32_t *tile = exact_alloc(((p + 31) / 32) * sizeof(uint32_t));
#endif
    float *alpha = exact_alloc(n_alpha * sizeof(float));
    CHECK(tbn_oracle_pack_tile(w, NULL, n, k, n_alpha, tile, alpha) == 0, "pack %ld x %ld k=%d", (long)in, (long)out, k);
    if (p % 32) CHECK((tile[p / 32] >> (p % 32)) == 0u, "unused high bits of the last word are set");
    double *w_hat = exact_alloc(n * sizeof(double));
    CHECK(tbn_oracle_materialise(tile, alpha, n_alpha, n, k, w_hat) == 0, "materialise");
    double *x = exact_alloc(M * in * sizeof(double));
    for (int64_t i = 0; i < M * in; ++i) x[i] = rnd();
    double *y = exact_alloc(M * out * sizeof(double)), *y1 = exact_alloc(M * out * sizeof(double));
    CHECK(tbn_oracle_linear(x, M, in, out, w_hat, y) == 0, "linear");
    CHECK(tbn_oracle_linear_alg1(x, M, in, out, tile, p, alpha, n_alpha, 0, y1) == 0, "alg1");
    double worst = 0;
    for (int64_t i = 0; i < M * out; ++i) worst = fmax(worst, fabs(y[i] - y1[i]));
    CHECK(worst < 1e-9, "dense product and Algorithm 1 differ by %g (%ld x %ld, k=%d)", worst, (long)in, (long)out, k);
    const int64_t count = M * out;
    int64_t *rows = exact_alloc(count * sizeof(int64_t)), *cols = exact_alloc(count * sizeof(int64_t));
    for (int64_t i = 0; i < count; ++i) { rows[i] = i / out; cols[i] = i % out; }
    if (M > 0) {   /* the sampled product takes no empty batch */
        CHECK(tbn_oracle_linear_at(x, M, in, out, w_hat, rows, cols, count, y1) == 0, "linear_at");
        worst = 0;
        for (int64_t i = 0; i < count; ++i) worst = fmax(worst, fabs(y[i] - y1[i]));
        CHECK(worst < 1e-12, "dense and sampled product differ by %g", worst);
    }
    free(w); free(tile); free(alpha); free(w_hat); free(x); free(y); free(y1); free(rows); free(cols);
}

static void ragged_conv(int64_t N, int64_t C, int64_t H, int64_t W, int64_t O, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                        int32_t ph, int32_t pw, int32_t k)
{
    const int64_t n = O * C * kh * kw, p = n / k;
    float *w = exact_alloc(n * sizeof(float));
    for (int64_t i = 0; i < n; ++i) w[i] = (float)rnd();
    uint32_t *tile = exact_alloc(((p + 31) / 32) * sizeof(uint32_t));
    float *alpha = exact_alloc(k * sizeof(float));
    CHECK(tbn_oracle_pack_tile(w, NULL, n, k, k, tile, alpha) == 0, "pack conv");
    double *w_hat = exact_alloc(n * sizeof(double));
    CHECK(tbn_oracle_materialise(tile, alpha, k, n, k, w_hat) == 0, "materialise conv");
    double *x = exact_alloc(N * C * H * W * sizeof(double));
    for (int64_t i = 0; i < N * C * H * W; ++i) x[i] = rnd();
    const int64_t Ho = (H + 2 * ph - kh) / sh + 1, Wo = (W + 2 * pw - kw) / sw + 1;
    const int64_t total = N * O * Ho * Wo;
    double *y = exact_alloc(total * sizeof(double)), *y1 = exact_alloc(total * sizeof(double));
    CHECK(tbn_oracle_conv2d(x, N, C, H, W, O, kh, kw, sh, sw, ph, pw, w_hat, y) == 0, "conv2d");
    int64_t *idx = exact_alloc(total * sizeof(int64_t));
    for (int64_t i = 0; i < total; ++i) idx[i] = i;
    CHECK(tbn_oracle_conv2d_at(x, N, C, H, W, O, kh, kw, sh, sw, ph, pw, w_hat, idx, total, y1) == 0, "conv2d_at");
    double worst = 0;
    for (int64_t i = 0; i < total; ++i) worst = fmax(worst, fabs(y[i] - y1[i]));
    CHECK(worst < 1e-12, "dense and sampled convolution differ by %g", worst);
    free(w); free(tile); free(alpha); free(w_hat); free(x); free(y); free(y1); free(idx);
}

int main(void)
{
    hand_worked();
    ragged_linear(3, 10, 6, 4, 4);     /* p = 15: tile ends inside rows and inside the only word */
    ragged_linear(5, 33, 7, 3, 3);     /* p = 77: three words, the last with 13 bits */
    ragged_linear(2, 64, 4, 1, 1);     /* k = 1 */
    ragged_linear(1, 40, 16, 16, 1);   /* p = in, one alpha */
    ragged_linear(0, 8, 8, 2, 2);      /* empty batch */
    ragged_conv(2, 3, 7, 5, 4, 3, 3, 1, 1, 1, 1, 4);
    ragged_conv(1, 2, 9, 8, 6, 3, 2, 2, 3, 0, 1, 3);
    ragged_conv(1, 4, 5, 5, 2, 1, 1, 1, 1, 0, 0, 2);
    if (failures) {
        fprintf(stderr, "%d checks failed\n", failures);
        return 1;
    }
    printf("oracle sanitize driver: ok\n");
    return 0;
}
