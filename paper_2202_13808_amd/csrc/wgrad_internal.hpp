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
    size_t dense_bytes, partial_bytes;
    size_t total() const { return dense_bytes + partial_bytes; }
};

// bf16 fully-connected weight gradient: recover R(a^) densely, then a direct-to-LDS GEMM (wgrad_fc_dense.hip)
bool fc_dense_supported(const FcProblem &p);
FcDensePlan fc_dense_plan(const FcProblem &p);
dropit_status fc_dense_run(const FcProblem &p, const FcDensePlan &plan, const void *vals, const int32_t *idx,
                           const void *dY, float *dW, char *ws, hipStream_t stream);

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

}  // namespace dropit
