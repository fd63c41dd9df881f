/* Runs every function of the CPU oracle on small inputs with exactly sized heap buffers, for a build under
 * -fsanitize=address,undefined (tests/test_sanitizers.py): an out-of-bounds access, a signed overflow or a
 * misaligned access in the oracle aborts the run.  Checks only cheap invariants; the values are pinned elsewhere. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t oracle_keep_count(int64_t numel, double gamma);
int oracle_compress(const void *x, int64_t numel, int dtype, int64_t k, void *vals, int32_t *idx);
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
uint32_t oracle_random_key(int64_t i, uint64_t seed);
int oracle_compress_random(const void *x, int64_t numel, int dtype, int64_t k, uint64_t seed, void *vals, int32_t *idx);
int oracle_rows_from_pairs(const int32_t *idx, int64_t k, int64_t rows, int64_t row_len, uint16_t *col, int32_t *rowptr);
int oracle_pairs_from_rows(const uint16_t *col, const int32_t *rowptr, int64_t rows, int64_t row_len, int32_t *idx);
int oracle_mask_from_pairs(const int32_t *idx, int64_t k, int64_t numel, int64_t block, uint32_t *mask, int32_t *blockptr);
int64_t oracle_pairs_from_mask(const uint32_t *mask, const int32_t *blockptr, int64_t numel, int64_t block, int32_t *idx);
void oracle_widen(const void *src, int64_t n, int dtype, double *dst);
int oracle_densify(const void *vals, const int32_t *idx, int64_t k, int dtype, int64_t numel, double *xhat);
void oracle_dw_fc(const double *xhat, const double *dY, int64_t ntok, int64_t cin, int64_t cout, int64_t j0, int64_t j1, double *dW);
void oracle_dw_conv(const double *xhat, const double *dY, int64_t N, int64_t C, int64_t H, int64_t W, int64_t cout,
                    int64_t OH, int64_t OW, int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                    int64_t dh, int64_t dw, int64_t j0, int64_t j1, double *dW);

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed line %d: %s\n", __LINE__, #c); exit(3); } } while (0)

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s >> 8; }

static void *exact(size_t bytes) { void *p = malloc(bytes ? bytes : 1); CHECK(p); return p; }

static void selection(int dtype, int64_t n, double gamma, uint32_t seed)
{
    const size_t es = dtype == 0 ? 4 : 2;
    unsigned char *x = exact((size_t)n * es);
    for (int64_t i = 0; i < n; ++i) {
        if (dtype == 0) { float f = (float)((int)(lcg(&seed) % 2001) - 1000) / 37.0f; memcpy(x + i * 4, &f, 4); }
        else { uint16_t b = (uint16_t)(lcg(&seed) & 0xBFFFu); memcpy(x + i * 2, &b, 2); }
    }
    const int64_t k = oracle_keep_count(n, gamma);
    CHECK(k >= 0 && k <= n);
    unsigned char *vals = exact((size_t)k * es);
    int32_t *idx = exact((size_t)k * 4);
    CHECK(oracle_compress(x, n, dtype, k, vals, idx) == 0);
    for (int64_t j = 0; j < k; ++j) {
        CHECK(idx[j] >= 0 && idx[j] < n && (j == 0 || idx[j] > idx[j - 1]));
        CHECK(memcmp(vals + j * es, x + (size_t)idx[j] * es, es) == 0);
    }
    double *xh = exact((size_t)n * 8);
    CHECK(oracle_densify(vals, idx, k, dtype, n, xh) == 0);
    double *w = exact((size_t)n * 8);
    oracle_widen(x, n, dtype, w);
    int32_t *ridx = exact((size_t)k * 4);
    CHECK(oracle_compress_random(x, n, dtype, k, 0x123456789ABCDEFull + seed, vals, ridx) == 0);
    for (int64_t j = 1; j < k; ++j) CHECK(ridx[j] > ridx[j - 1]);
    /* the cheaper index forms and back, on the min-k indices */
    for (int64_t row_len = 1; row_len <= n; row_len = row_len * 3 + 1) {
        if (n % row_len) continue;
        const int64_t rows = n / row_len;
        if (row_len > 65536) break;
        uint16_t *col = exact((size_t)k * 2);
        int32_t *rowptr = exact((size_t)(rows + 1) * 4), *back = exact((size_t)k * 4);
        CHECK(oracle_rows_from_pairs(idx, k, rows, row_len, col, rowptr) == 0);
        CHECK(rowptr[0] == 0 && rowptr[rows] == k);
        CHECK(oracle_pairs_from_rows(col, rowptr, rows, row_len, back) == 0);
        CHECK(memcmp(back, idx, (size_t)k * 4) == 0);
        free(col); free(rowptr); free(back);
    }
    for (int64_t block = 32; block <= 1024; block *= 4) {
        uint32_t *mask = exact((size_t)((n + 31) / 32) * 4);
        int32_t *bp = exact((size_t)((n + block - 1) / block + 1) * 4), *back = exact((size_t)n * 4);
        CHECK(oracle_mask_from_pairs(idx, k, n, block, mask, bp) == 0);
        CHECK(oracle_pairs_from_mask(mask, bp, n, block, back) == k);
        CHECK(memcmp(back, idx, (size_t)k * 4) == 0);
        free(mask); free(bp); free(back);
    }
    free(x); free(vals); free(idx); free(xh); free(w); free(ridx);
}

static void gradients(void)
{
    uint32_t seed = 7;
    /* FC: 13 tokens, 5 -> 3 */
    const int64_t nt = 13, ci = 5, co = 3;
    double *xh = exact(nt * ci * 8), *dy = exact(nt * co * 8), *dw = exact(co * ci * 8);
    for (int64_t i = 0; i < nt * ci; ++i) xh[i] = (double)(lcg(&seed) % 7) - 3;
    for (int64_t i = 0; i < nt * co; ++i) dy[i] = (double)(lcg(&seed) % 5) - 2;
    memset(dw, 0, co * ci * 8);
    oracle_dw_fc(xh, dy, nt, ci, co, 0, co, dw);
    oracle_dw_fc(xh, dy, nt, ci, co, 1, 2, dw);          /* a row range */
    free(xh); free(dy); free(dw);
    /* conv: geometries with padding wider than the window, stride, dilation, single pixels */
    const int64_t geo[][8] = { {3,3,1,1,1,1,1,1}, {1,1,1,1,0,0,1,1}, {3,2,2,1,4,0,2,3}, {5,5,3,2,2,1,1,1}, {2,2,1,1,3,3,1,1} };
    for (unsigned g = 0; g < sizeof geo / sizeof geo[0]; ++g) {
        const int64_t N = 2, C = 3, H = 7, W = 6, J = 2;
        const int64_t kh = geo[g][0], kw = geo[g][1], sh = geo[g][2], sw = geo[g][3], ph = geo[g][4], pw = geo[g][5],
                      dh = geo[g][6], dwd = geo[g][7];
        const int64_t eh = H + 2 * ph - dh * (kh - 1) - 1, ew = W + 2 * pw - dwd * (kw - 1) - 1;
        if (eh < 0 || ew < 0) continue;
        const int64_t OH = eh / sh + 1, OW = ew / sw + 1;
        double *x = exact(N * C * H * W * 8), *gy = exact(N * J * OH * OW * 8), *out = exact(J * C * kh * kw * 8);
        for (int64_t i = 0; i < N * C * H * W; ++i) x[i] = (double)(lcg(&seed) % 9) - 4;
        for (int64_t i = 0; i < N * J * OH * OW; ++i) gy[i] = (double)(lcg(&seed) % 3) - 1;
        memset(out, 0, J * C * kh * kw * 8);
        oracle_dw_conv(x, gy, N, C, H, W, J, OH, OW, kh, kw, sh, sw, ph, pw, dh, dwd, 0, J, out);
        free(x); free(gy); free(out);
    }
}

int main(void)
{
    CHECK(oracle_keep_count(16384, 0.9) == 1638 && oracle_keep_count(100, 0.9) == 10);
    CHECK(oracle_keep_count(-1, 0.5) == -1 && oracle_keep_count(10, 1.5) == -1);
    const int64_t sizes[] = {1, 2, 7, 8, 9, 63, 64, 65, 1000, 4096, 4097};
    const double gammas[] = {0.0, 0.3, 0.5, 0.9, 0.999, 1.0};
    for (unsigned s = 0; s < sizeof sizes / sizeof sizes[0]; ++s)
        for (unsigned g = 0; g < sizeof gammas / sizeof gammas[0]; ++g)
            for (int dtype = 0; dtype < 2; ++dtype) selection(dtype, sizes[s], gammas[g], 11u * (s + 1) + g);
    uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6}, out[4];
    oracle_philox4x32_10(ctr, key, out);
    (void)oracle_random_key(2147483646LL, 0xFFFFFFFFFFFFFFFFull);
    gradients();
    puts("oracle under sanitizers: OK");
    return 0;
}
