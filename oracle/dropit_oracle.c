/*
 * CPU oracle for the DropIT hot path (arXiv 2202.13808).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * statement of what the GPU library must compute.  It is compiled with gcc,
 * shares no code, header, table or helper with the HIP path, and is called
 * only from the tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * What it states (paper passages in brackets):
 *   - keep count        k = floor((1-gamma)*numel)        [Sec. 4.1, a share of 1-gamma is kept;
 *                                                          Sec. 3.3 Min-K; Table 4]
 *   - min-k dropping    D(a) = {a_Xr, Xr}: keep the k elements of largest
 *                       absolute magnitude, with their indices
 *                                                         [Sec. 3.2; Sec. 3.3 Min-K; Sec. 4.1]
 *   - random dropping   D(a) with X_r a uniformly random k-subset            [Sec. 3.3 Random Elements]
 *   - row form of X_r   the retained indices re-encoded as 16-bit positions within
 *                       rows plus row offsets (lossless; the index cost the paper
 *                       discusses)                          [Sec. 4.3, memory of indices; App. on choosing gamma]
 *   - recover           R(a^): dense tensor, dropped positions zero
 *                                                         [Sec. 3.2; Fig. 1 caption]
 *   - FC weight grad    g[j][c] = sum_n dz[n][j] * a^[n][c]
 *                                                         [Sec. 3.2, Eq. fc_backward_elem_save]
 *   - conv weight grad  g[j][c][u][v] = sum_{n,y,x} dz[n][j][y][x] * a^[n][c][y'][x']
 *                                                         [Sec. 3.2, Eq. conv_backward_elem]
 *
 * Readings where the paper is silent (each one is listed in the design notes):
 *   ties at the threshold -> lowest flat index wins; output in ascending flat
 *   index; |x| order is the unsigned order of the bit pattern with the sign
 *   bit cleared (so -0 == +0, denormals ordered exactly, NaN above inf);
 *   int32 0-based row-major flat indices [App. A.7]; conv is a
 *   cross-correlation with 0-based y' = y*stride - pad + u*dil and zero
 *   padding.  Random dropping keeps exactly k elements (the same k as min-k):
 *   element i draws the 32-bit word (i mod 4) of Philox4x32-10 (Salmon et al.,
 *   "Parallel random numbers: as easy as 1, 2, 3", SC'11) at counter
 *   (floor(i/4), 0, 0, 0) under key (seed mod 2^32, seed div 2^32); the k
 *   elements with the largest draw, shifted right by one bit, are kept, equal
 *   draws going to the lowest index.
 *
 * All floating-point accumulation is fp64, in the summation order the
 * formulas are written in.  No blocking, fusion or reordering.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* ---- keep count ------------------------------------------------------- */
/* k = floor((1-gamma)*numel), evaluated as numel - ceil(gamma*numel) in IEEE
 * double so that gamma=0.9, numel=100 gives 10 (1.0-0.9 is not 0.1 in
 * binary).  Returns -1 for gamma outside [0,1], NaN, or numel < 0. */
int64_t oracle_keep_count(int64_t numel, double gamma)
{
    if (numel < 0 || !(gamma >= 0.0) || !(gamma <= 1.0)) return -1;
    double dropped = ceil(gamma * (double)numel);
    int64_t k = numel - (int64_t)dropped;
    if (k < 0) k = 0;
    if (k > numel) k = numel;
    return k;
}

/* ---- magnitude key ---------------------------------------------------- */
static uint32_t key_of(const void *x, int64_t i, int dtype)
{
    if (dtype == ORACLE_F32) {
        uint32_t b;
        memcpy(&b, (const char *)x + 4 * i, 4);
        return b & 0x7FFFFFFFu;
    } else {
        uint16_t b;
        memcpy(&b, (const char *)x + 2 * i, 2);
        return (uint32_t)(b & 0x7FFFu);
    }
}

typedef struct { uint32_t key; int32_t idx; } pair_t;

/* larger key first; equal keys: lower index first */
static int cmp_key_desc_idx_asc(const void *pa, const void *pb)
{
    const pair_t *a = (const pair_t *)pa, *b = (const pair_t *)pb;
    if (a->key != b->key) return (a->key > b->key) ? -1 : 1;
    if (a->idx != b->idx) return (a->idx < b->idx) ? -1 : 1;
    return 0;
}

static int cmp_i32_asc(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/* ---- D(a): min-k drop by full sort ------------------------------------ */
/* Sort every (key, index) pair by (key descending, index ascending), keep the
 * first k, put those k back into ascending index order, copy their original
 * bit patterns.  Returns 0, or -1 on bad arguments / out of memory. */
int oracle_compress(const void *x, int64_t numel, int dtype, int64_t k,
                    void *vals, int32_t *idx)
{
    if (numel < 0 || numel > 2147483647LL || k < 0 || k > numel) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
    if (k == 0) return 0;
    pair_t *p = (pair_t *)malloc((size_t)numel * sizeof(pair_t));
    if (!p) return -1;
    for (int64_t i = 0; i < numel; ++i) {
        p[i].key = key_of(x, i, dtype);
        p[i].idx = (int32_t)i;
    }
    qsort(p, (size_t)numel, sizeof(pair_t), cmp_key_desc_idx_asc);
    for (int64_t j = 0; j < k; ++j) idx[j] = p[j].idx;
    free(p);
    qsort(idx, (size_t)k, sizeof(int32_t), cmp_i32_asc);
    size_t es = (dtype == ORACLE_F32) ? 4 : 2;
    for (int64_t j = 0; j < k; ++j)
        memcpy((char *)vals + es * (size_t)j, (const char *)x + es * (size_t)idx[j], es);
    return 0;
}

/* ---- random dropping -------------------------------------------------- */
/* Philox4x32 with 10 rounds as published (Salmon, Moraes, Dror, Shaw, SC'11):
 * each round multiplies counter words 0 and 2 by two fixed odd constants, and
 * the new counter is (hi(p1)^c1^k0, lo(p1), hi(p0)^c3^k1, lo(p0)); the key
 * advances by the two Weyl constants before every round but the first. */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 31-bit selection key of element i under `seed`. */
uint32_t oracle_random_key(int64_t i, uint64_t seed)
{
    uint32_t ctr[4] = { (uint32_t)(i >> 2), 0u, 0u, 0u };
    uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    return out[i & 3] >> 1;
}

/* D(a) with random X_r: the same full sort as oracle_compress, on the drawn
 * keys instead of the magnitudes.  Returns 0, or -1 on bad arguments. */
int oracle_compress_random(const void *x, int64_t numel, int dtype, int64_t k, uint64_t seed,
                           void *vals, int32_t *idx)
{
    if (numel < 0 || numel > 2147483647LL || k < 0 || k > numel) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
    if (k == 0) return 0;
    pair_t *p = (pair_t *)malloc((size_t)numel * sizeof(pair_t));
    if (!p) return -1;
    for (int64_t i = 0; i < numel; ++i) {
        p[i].key = oracle_random_key(i, seed);
        p[i].idx = (int32_t)i;
    }
    qsort(p, (size_t)numel, sizeof(pair_t), cmp_key_desc_idx_asc);
    for (int64_t j = 0; j < k; ++j) idx[j] = p[j].idx;
    free(p);
    qsort(idx, (size_t)k, sizeof(int32_t), cmp_i32_asc);
    size_t es = (dtype == ORACLE_F32) ? 4 : 2;
    for (int64_t j = 0; j < k; ++j)
        memcpy((char *)vals + es * (size_t)j, (const char *)x + es * (size_t)idx[j], es);
    return 0;
}

/* ---- row form of the retained index set ------------------------------- */
/* The tensor is read as `rows` rows of `row_len` consecutive elements (its last
 * dimension).  col[j] = idx[j] mod row_len; rowptr[r] = number of retained
 * indices below r*row_len, r = 0..rows, so row r owns pairs rowptr[r] ..
 * rowptr[r+1]-1.  Needs row_len <= 65536.  Returns 0, or -1 on bad arguments
 * (including an index outside the tensor or out of order). */
int oracle_rows_from_pairs(const int32_t *idx, int64_t k, int64_t rows, int64_t row_len,
                           uint16_t *col, int32_t *rowptr)
{
    if (k < 0 || rows < 1 || row_len < 1 || row_len > 65536) return -1;
    for (int64_t r = 0; r <= rows; ++r) rowptr[r] = 0;
    for (int64_t j = 0; j < k; ++j) {
        int64_t i = idx[j];
        if (i < 0 || i >= rows * row_len) return -1;
        if (j > 0 && idx[j - 1] >= idx[j]) return -1;
        int64_t r = i / row_len;
        col[j] = (uint16_t)(i - r * row_len);
        rowptr[r + 1] += 1;                     /* count per row ... */
    }
    for (int64_t r = 0; r < rows; ++r) rowptr[r + 1] += rowptr[r];   /* ... then running sum */
    return 0;
}

/* Inverse: idx[j] = r*row_len + col[j] for every j in row r. */
int oracle_pairs_from_rows(const uint16_t *col, const int32_t *rowptr, int64_t rows, int64_t row_len,
                           int32_t *idx)
{
    if (rows < 1 || row_len < 1 || row_len > 65536 || rowptr[0] != 0) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        if (rowptr[r + 1] < rowptr[r]) return -1;
        for (int64_t j = rowptr[r]; j < rowptr[r + 1]; ++j) {
            if (col[j] >= row_len) return -1;
            idx[j] = (int32_t)(r * row_len + col[j]);
        }
    }
    return 0;
}

/* ---- bit-mask form of the retained index set --------------------------- */
/* One bit per element of the tensor (bit i%32 of word i/32 set iff element i is
 * retained; the bits past numel in the last word are 0), plus, for every block of
 * `block` consecutive elements (a multiple of 32), the number of retained elements
 * before it: blockptr[b], b = 0..ceil(numel/block).  numel/8 bytes of mask against
 * 4 bytes per retained int32 index: smaller whenever more than 1/32 of the tensor
 * is kept (Sec. 4.3 counts the index bytes as part of the method's memory; the
 * appendix on choosing gamma prices an int32 index at one fp32 activation).
 * Returns 0, or -1 on bad arguments (an index outside the tensor or out of order). */
int oracle_mask_from_pairs(const int32_t *idx, int64_t k, int64_t numel, int64_t block,
                           uint32_t *mask, int32_t *blockptr)
{
    if (k < 0 || numel < 1 || block < 32 || block % 32 != 0) return -1;
    const int64_t words = (numel + 31) / 32, blocks = (numel + block - 1) / block;
    for (int64_t w = 0; w < words; ++w) mask[w] = 0;
    for (int64_t b = 0; b <= blocks; ++b) blockptr[b] = 0;
    for (int64_t j = 0; j < k; ++j) {
        int64_t i = idx[j];
        if (i < 0 || i >= numel) return -1;
        if (j > 0 && idx[j - 1] >= idx[j]) return -1;
        mask[i / 32] |= (uint32_t)1 << (i % 32);
        blockptr[i / block + 1] += 1;           /* count per block ... */
    }
    for (int64_t b = 0; b < blocks; ++b) blockptr[b + 1] += blockptr[b];   /* ... then running sum */
    return 0;
}

/* Inverse: the ascending flat indices of the set bits.  Returns their number, or -1 if
 * blockptr does not match the mask. */
int64_t oracle_pairs_from_mask(const uint32_t *mask, const int32_t *blockptr, int64_t numel, int64_t block,
                               int32_t *idx)
{
    if (numel < 1 || block < 32 || block % 32 != 0) return -1;
    int64_t j = 0;
    for (int64_t i = 0; i < numel; ++i) {
        if (i % block == 0 && blockptr[i / block] != j) return -1;
        if ((mask[i / 32] >> (i % 32)) & 1u) idx[j++] = (int32_t)i;
    }
    if (blockptr[(numel + block - 1) / block] != j) return -1;
    return j;
}

/* ---- exact widening to double ----------------------------------------- */
static double widen(const void *v, int64_t i, int dtype)
{
    uint32_t b;
    if (dtype == ORACLE_F32) {
        memcpy(&b, (const char *)v + 4 * i, 4);
    } else {
        uint16_t h;
        memcpy(&h, (const char *)v + 2 * i, 2);
        b = (uint32_t)h << 16;               /* bf16 is the top half of an fp32 */
    }
    float f;
    memcpy(&f, &b, 4);
    return (double)f;
}

/* Widen a raw fp32 / bf16 buffer to fp64 (exact). */
void oracle_widen(const void *src, int64_t n, int dtype, double *dst)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = widen(src, i, dtype);
}

/* ---- R(a^): zero-fill recover ----------------------------------------- */
int oracle_densify(const void *vals, const int32_t *idx, int64_t k, int dtype,
                   int64_t numel, double *xhat)
{
    for (int64_t i = 0; i < numel; ++i) xhat[i] = 0.0;
    for (int64_t j = 0; j < k; ++j) {
        if (idx[j] < 0 || (int64_t)idx[j] >= numel) return -1;
        xhat[idx[j]] = widen(vals, j, dtype);
    }
    return 0;
}

/* ---- FC weight gradient ------------------------------------------------ */
/* dW[j][c] = sum_{n=0}^{ntok-1} dY[n][j] * xhat[n][c]   for j in [j0, j1).
 * xhat [ntok][cin], dY [ntok][cout], dW [cout][cin] (rows outside [j0,j1)
 * are left untouched).  One accumulator per output, n ascending. */
void oracle_dw_fc(const double *xhat, const double *dY, int64_t ntok,
                  int64_t cin, int64_t cout, int64_t j0, int64_t j1, double *dW)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = j0; j < j1; ++j) {
        for (int64_t c = 0; c < cin; ++c) {
            double acc = 0.0;
            for (int64_t n = 0; n < ntok; ++n)
                acc += dY[n * cout + j] * xhat[n * cin + c];
            dW[j * cin + c] = acc;
        }
    }
}

/* ---- conv weight gradient ---------------------------------------------- */
/* dW[j][c][u][v] = sum_n sum_oy sum_ox dY[n][j][oy][ox] * xhat[n][c][iy][ix],
 * iy = oy*sh - ph + u*dh, ix = ox*sw - pw + v*dw, terms with (iy,ix) outside
 * the input are zero.  xhat NCHW [N][C][H][W], dY [N][cout][OH][OW],
 * dW [cout][C][kh][kw]; computed for j in [j0, j1). */
void oracle_dw_conv(const double *xhat, const double *dY,
                    int64_t N, int64_t C, int64_t H, int64_t W,
                    int64_t cout, int64_t OH, int64_t OW,
                    int64_t kh, int64_t kw, int64_t sh, int64_t sw,
                    int64_t ph, int64_t pw, int64_t dh, int64_t dw,
                    int64_t j0, int64_t j1, double *dW)
{
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t j = j0; j < j1; ++j) {
        for (int64_t c = 0; c < C; ++c) {
            for (int64_t u = 0; u < kh; ++u) {
                for (int64_t v = 0; v < kw; ++v) {
                    double acc = 0.0;
                    for (int64_t n = 0; n < N; ++n) {
                        for (int64_t oy = 0; oy < OH; ++oy) {
                            int64_t iy = oy * sh - ph + u * dh;
                            if (iy < 0 || iy >= H) continue;
                            for (int64_t ox = 0; ox < OW; ++ox) {
                                int64_t ix = ox * sw - pw + v * dw;
                                if (ix < 0 || ix >= W) continue;
                                acc += dY[((n * cout + j) * OH + oy) * OW + ox] *
                                       xhat[((n * C + c) * H + iy) * W + ix];
                            }
                        }
                    }
                    dW[((j * C + c) * kh + u) * kw + v] = acc;
                }
            }
        }
    }
}

/* number of OpenMP threads the dW loops will use (for the benchmark report) */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
