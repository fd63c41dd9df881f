// Internal interfaces between the weight-gradient host entry point and its kernels.
#pragma once

#include <algorithm>

#include "common.hpp"

namespace dropit {

struct FcProblem {
    int64_t ntok, cin, cout, k;
};

struct FcDensePlan {
    int nkb, nb_count, mb_count, splits, pitch, rows_per_wg;
    bool narrow;                               // the 128-row tile configuration (layers with few output channels)
    int64_t ntok_pad;                          // rows of the dense operand: the tokens rounded up to whole token blocks
    size_t dense_bytes, partial_bytes;
    // the in-LDS form keeps no dense operand: the pairs regrouped by tile (a word each), the table of tile starts
    // and the table of token-block starts take its place at the front of the workspace
    bool fused;
    size_t packed_bytes, table_bytes, kbptr_bytes;
    size_t operand_bytes() const { return fused ? packed_bytes + table_bytes + kbptr_bytes : dense_bytes; }
    size_t total() const { return operand_bytes() + partial_bytes; }
};

// bf16 fully-connected weight gradient: recover R(a^) densely, then a direct-to-LDS GEMM (wgrad_fc_dense.hip)
bool fc_dense_supported(const FcProblem &p);
FcDensePlan fc_dense_plan(const FcProblem &p, bool fused = false);
dropit_status fc_dense_run(const FcProblem &p, const FcDensePlan &plan, const void *vals, const int32_t *idx,
                           const void *dY, float *dW, char *ws, hipStream_t stream);

// the same product with the recover step inside it: the zero-filled tensor exists only as LDS tiles (plan.fused)
bool fc_fused_supported(const FcProblem &p);
dropit_status fc_fused_run(const FcProblem &p, const FcDensePlan &plan, const void *vals, const int32_t *idx,
                           const void *dY, float *dW, char *ws, hipStream_t stream);

// the same from the row form of the cache (col = position in the row, rowptr = pairs before each row)
dropit_status fc_dense_run_rows(const FcProblem &p, const FcDensePlan &plan, const void *vals, const uint16_t *col,
                                const int32_t *rowptr, const void *dY, float *dW, char *ws, hipStream_t stream);

// ... and from the bit-mask form (mask bit per element, blockptr = pairs before each block of DROPIT_MASK_BLOCK);
// only when fc_dense_mask_native(p): c_in % 8 == 0
bool fc_dense_mask_native(const FcProblem &p);
dropit_status fc_dense_run_mask(const FcProblem &p, const FcDensePlan &plan, const void *vals, const uint32_t *mask,
                                const int32_t *blockptr, const void *dY, float *dW, char *ws, hipStream_t stream);

// the GEMM and the K-slice sum alone, on operands that are already dense: dY [ntok][cout], dense [plan.ntok_pad][plan.pitch]
// (rows past ntok zero); `partial` holds plan.partial_bytes
dropit_status fc_dense_gemm(const FcProblem &p, const FcDensePlan &plan, const void *dY, const uint16_t *dense,
                            float *partial, float *dW, hipStream_t stream);

// Row starts of the index-sorted pairs: row_ptr[r] = number of pairs whose flat index lies before row r
// of `row_len` consecutive elements, r = 0..R (row_ptr[R] = k).  One pass over idx: every pair is compared
// with its predecessor and fills the row starts that fall between them; the entry j == k closes the table.
// A thread takes four consecutive pairs (one 16-byte load when idx is 16-byte aligned) and divides each
// index once.  Indices are below 2^31: 32-bit unsigned division (a 64-bit one is several times the instructions).
template <bool VEC>
static __global__ void __launch_bounds__(256)
row_starts_kernel(const int32_t *__restrict__ idx, int64_t k, uint32_t row_len, int64_t R, uint32_t *__restrict__ row_ptr)
{
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    const int64_t stride = int64_t(gridDim.x) * blockDim.x * 4;
    for (int64_t j0 = (int64_t(blockIdx.x) * blockDim.x + threadIdx.x) * 4; j0 <= k; j0 += stride) {
        int64_t before = (j0 == 0) ? -1 : min<int64_t>(uint32_t(idx[j0 - 1]) / row_len, R);
        int32_t v[4];
        if (VEC && j0 + 4 <= k) {
            const i32x4 q = *reinterpret_cast<const i32x4 *>(idx + j0);
            v[0] = q[0]; v[1] = q[1]; v[2] = q[2]; v[3] = q[3];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = j0 + e < k ? idx[j0 + e] : 0;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t j = j0 + e;
            if (j > k) break;
            const int64_t here = (j == k) ? R : min<int64_t>(uint32_t(v[e]) / row_len, R);
            for (int64_t r = before + 1; r <= here; ++r) row_ptr[r] = uint32_t(j);
            before = here;
        }
    }
}

inline void launch_row_starts(const int32_t *idx, int64_t k, uint32_t row_len, int64_t R, uint32_t *row_ptr,
                              hipStream_t stream)
{
    const int blocks = int(std::min<int64_t>((k / 4 + 1 + 255) / 256, 4096));
    if (aligned(idx, 16))
        row_starts_kernel<true><<<blocks, 256, 0, stream>>>(idx, k, row_len, R, row_ptr);
    else
        row_starts_kernel<false><<<blocks, 256, 0, stream>>>(idx, k, row_len, R, row_ptr);
}

struct ConvProblem {
    int64_t N, C, H, W, J, k;
};

struct ConvPlan {
    int cb_count, jb_count, bands, rb, pitch_c;
    int wp;                                    // row width the kernel works with: W rounded up to whole groups of 8
    int imgs_per_wg, img_groups;               // a workgroup accumulates over this many images; ceil(N / imgs_per_wg) groups
    size_t lds_bytes, rowptr_bytes, partial_bytes;
    size_t dypad_bytes;                        // zero-padded copy of dY when wp != W, else 0
    size_t total() const { return rowptr_bytes + partial_bytes + dypad_bytes; }
};

// bf16 3x3/s1/p1 convolution weight gradient on the matrix cores (wgrad_conv_mfma.hip)
bool conv_mfma_supported(const ConvProblem &p);
ConvPlan conv_mfma_plan(const ConvProblem &p);
dropit_status conv_mfma_run(const ConvProblem &p, const ConvPlan &plan, const void *vals, const int32_t *idx,
                            const void *dY, float *dW, char *ws, hipStream_t stream);

// The same gradient as one GEMM over explicit im2col rows, for small planes with many channels
// (wgrad_conv_gemm.hip)
struct ConvGemmPlan {
    FcProblem fp;                              // tokens = N*H*W output positions, c_in = 9*C taps, c_out = J
    FcDensePlan gemm;
    int cb, cblocks;                           // input channels per im2col workgroup
    size_t lds_bytes, dyt_bytes;
    size_t total() const { return gemm.dense_bytes + gemm.partial_bytes + dyt_bytes; }
};
bool conv_gemm_supported(const ConvProblem &p);
bool conv_gemm_preferred(const ConvProblem &p);
ConvGemmPlan conv_gemm_plan(const ConvProblem &p);
dropit_status conv_gemm_run(const ConvProblem &p, const ConvGemmPlan &plan, const void *vals, const int32_t *idx,
                            const void *dY, float *dW, char *ws, hipStream_t stream);

// Any geometry, NCHW or NHWC, bf16: zero-filled im2col rows written from the pairs + the FC GEMM
// (wgrad_conv_im2col.hip)
struct ConvGeneral {
    int64_t N, C, H, W, OH, OW, J, k;
    dropit_conv2d g;
    bool nhwc;
};
struct ConvIm2colPlan {
    FcProblem fp;                              // tokens = N*OH*OW, c_in = C*kh*kw, c_out = J
    FcDensePlan gemm;
    size_t dyt_bytes;                          // token-major copy of dY (NCHW only)
    bool tiled;                                // im2col rows assembled in LDS tiles (else zero fill + scatter)
    int nblocks, blk, bands, rb, rowlen;       // tiled form: column blocks, their width, row bands, rows per band, tile row length
    size_t lds_bytes, rowptr_bytes;
    size_t total() const { return gemm.dense_bytes + gemm.partial_bytes + dyt_bytes + rowptr_bytes; }
};
bool conv_im2col_supported(const ConvGeneral &p);
ConvIm2colPlan conv_im2col_plan(const ConvGeneral &p);
dropit_status conv_im2col_run(const ConvGeneral &p, const ConvIm2colPlan &plan, const void *vals, const int32_t *idx,
                              const void *dY, float *dW, char *ws, hipStream_t stream);

}  // namespace dropit
