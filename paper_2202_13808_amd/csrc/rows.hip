// Row form of the retained index set: 16-bit positions within rows + row offsets.
//
// The paper counts the indices as the method's own memory cost (Sec. 4.3: index memory next to the
// saved activations; appendix on choosing gamma: an int32 index is as wide as an fp32 activation,
// hence gamma > 50 %).  With bf16 activations an int32 index is twice as wide as the value it
// locates.  Reading the tensor as rows of its last dimension (<= 65536 long), a retained element
// needs only its 16-bit position in the row, and each row one 32-bit offset into the pair arrays:
// 2k + 4(rows + 1) bytes instead of 4k.  The encoding is lossless; the selection itself and the
// weight-gradient kernels are the ones behind dropit_compress / dropit_weight_grad.
#include <algorithm>

#include "common.hpp"
#include "wgrad_internal.hpp"

namespace dropit {
namespace {

// One pass over the ascending flat indices: position in the row for every pair, and for every row
// the number of pairs before it.  Pair j writes the offsets of the rows that start between its
// predecessor and itself; j == k closes the table.
__global__ void __launch_bounds__(256)
rows_from_idx_kernel(const int32_t *__restrict__ idx, int64_t k, int64_t row_len, int64_t rows,
                     uint16_t *__restrict__ col, int32_t *__restrict__ rowptr)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t j = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; j <= k; j += stride) {
        // indices are below 2^31 and row_len <= 65536: 32-bit unsigned division
        const uint32_t len = static_cast<uint32_t>(row_len);
        const int64_t before = (j == 0) ? -1 : min<int64_t>(static_cast<uint32_t>(idx[j - 1]) / len, rows);
        int64_t here = rows;
        if (j < k) {
            const uint32_t flat = static_cast<uint32_t>(idx[j]);
            const uint32_t row = flat / len;
            here = min<int64_t>(row, rows);
            col[j] = static_cast<uint16_t>(flat - row * len);
        }
        for (int64_t r = before + 1; r <= here; ++r) rowptr[r] = static_cast<int32_t>(j);
    }
}

// Inverse: one wavefront per row writes the flat indices of that row's pairs.
__global__ void __launch_bounds__(256)
idx_from_rows_kernel(const uint16_t *__restrict__ col, const int32_t *__restrict__ rowptr, int64_t rows,
                     int64_t row_len, int64_t k, int32_t *__restrict__ idx)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t waves = static_cast<int64_t>(gridDim.x) * (blockDim.x / WAVE);
    for (int64_t r = static_cast<int64_t>(blockIdx.x) * (blockDim.x / WAVE) + threadIdx.x / WAVE; r < rows;
         r += waves) {
        // a malformed table must not make the kernel write outside idx[0, k)
        const int64_t first = max<int64_t>(rowptr[r], 0), last = min<int64_t>(rowptr[r + 1], k);
        for (int64_t j = first + lane; j < last; j += WAVE)
            idx[j] = static_cast<int32_t>(r * row_len + col[j]);
    }
}

struct RowShape {
    int64_t numel, row_len, rows;
};

// rows are the last dimension; it must fit a 16-bit position
bool row_shape(const int64_t *shape, int ndim, RowShape &rs)
{
    rs.numel = checked_numel(shape, ndim);
    if (rs.numel < 1) return false;
    rs.row_len = shape[ndim - 1];
    if (rs.row_len > 65536) return false;
    rs.rows = rs.numel / rs.row_len;
    return true;
}

unsigned grid_for(int64_t threads_needed)
{
    return static_cast<unsigned>(std::min<int64_t>(std::max<int64_t>((threads_needed + 255) / 256, 1), 256 * 16));
}

}  // namespace
}  // namespace dropit

using namespace dropit;

extern "C" size_t dropit_compress_rows_workspace_bytes(int64_t numel, int64_t k, dropit_dtype dt)
{
    const size_t select_bytes = dropit_compress_workspace_bytes(numel, dt);
    if (select_bytes == 0 || k < 0 || k > numel) return 0;
    return round_up(select_bytes, 256) + round_up(static_cast<size_t>(k) * 4 + 4, 256);
}

extern "C" dropit_status dropit_compress_rows(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                                              double gamma, void *vals, uint16_t *col, int32_t *rowptr,
                                              void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (dt != DROPIT_F32 && dt != DROPIT_BF16) return DROPIT_EINVAL;
    RowShape rs;
    if (!row_shape(shape, ndim, rs)) return DROPIT_EINVAL;
    const int64_t k = dropit_keep_count(rs.numel, gamma);
    if (k < 0) return DROPIT_EINVAL;
    if (rowptr == nullptr || !aligned(rowptr, 4)) return DROPIT_EINVAL;
    if (k > 0 && (col == nullptr || !aligned(col, 2))) return DROPIT_EINVAL;
    if (workspace == nullptr || !aligned(workspace, 256)) return DROPIT_EINVAL;
    if (workspace_bytes < dropit_compress_rows_workspace_bytes(rs.numel, k, dt)) return DROPIT_EWORKSPACE;
    const size_t select_bytes = round_up(dropit_compress_workspace_bytes(rs.numel, dt), 256);
    int32_t *idx = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + select_bytes);
    const dropit_status st = dropit_compress(x, shape, ndim, dt, gamma, vals, idx, workspace, select_bytes, hip_stream);
    if (st != DROPIT_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    rows_from_idx_kernel<<<grid_for(k + 1), 256, 0, stream>>>(idx, k, rs.row_len, rs.rows, col, rowptr);
    trace_mark(stream);
    return launch_status();
}

extern "C" size_t dropit_weight_grad_rows_workspace_bytes(const int64_t *x_shape, int ndim, dropit_dtype dt,
                                                          int64_t k, int64_t c_out, const dropit_conv2d *conv)
{
    RowShape rs;
    if (!row_shape(x_shape, ndim, rs) || k < 0 || k > rs.numel) return 0;
    const size_t inner = dropit_weight_grad_workspace_bytes(x_shape, ndim, dt, k, c_out, conv);
    if (inner == 0) return 0;
    return round_up(inner, 256) + round_up(static_cast<size_t>(k) * 4 + 4, 256);
}

extern "C" dropit_status dropit_weight_grad_rows(const void *vals, const uint16_t *col, const int32_t *rowptr,
                                                 int64_t k, const int64_t *x_shape, int ndim, dropit_dtype dt,
                                                 const void *dY, int64_t c_out, const dropit_conv2d *conv,
                                                 float *dW, void *workspace, size_t workspace_bytes,
                                                 void *hip_stream)
{
    RowShape rs;
    if (!row_shape(x_shape, ndim, rs) || k < 0 || k > rs.numel) return DROPIT_EINVAL;
    if (k > 0 && (col == nullptr || rowptr == nullptr || !aligned(col, 2) || !aligned(rowptr, 4)))
        return DROPIT_EINVAL;
    if (workspace == nullptr || !aligned(workspace, 256)) return DROPIT_EINVAL;
    const size_t inner = dropit_weight_grad_workspace_bytes(x_shape, ndim, dt, k, c_out, conv);
    if (inner == 0) return DROPIT_EINVAL;
    if (workspace_bytes < dropit_weight_grad_rows_workspace_bytes(x_shape, ndim, dt, k, c_out, conv))
        return DROPIT_EWORKSPACE;
    int32_t *idx = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + round_up(inner, 256));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // A bf16 fully-connected layer on the matrix cores recovers straight from the row form: its rows are
    // the rows of the recovered matrix.  (Everything else expands the flat indices first.)
    if (conv == nullptr && dt == DROPIT_BF16 && k > 0 && c_out >= 1) {
        const FcProblem fp = {rs.rows, rs.row_len, c_out, k};
        if (fc_dense_supported(fp) && dropit_weight_grad_path(x_shape, ndim, dt, k, c_out, conv) == DROPIT_PATH_FC_MFMA) {
            if (vals == nullptr || !aligned(vals, 2)) return DROPIT_EINVAL;
            if (dY == nullptr || dW == nullptr || !aligned(dY, 16) || !aligned(dW, 16)) return DROPIT_EINVAL;
            const FcDensePlan plan = fc_dense_plan(fp);
            if (plan.total() > inner) return DROPIT_EWORKSPACE;
            return fc_dense_run_rows(fp, plan, vals, col, rowptr, dY, dW, static_cast<char *>(workspace), stream);
        }
    }
    if (k > 0) {
        trace_mark(stream);
        const int64_t waves_needed = std::min<int64_t>(rs.rows, 256 * 16 * 4);
        idx_from_rows_kernel<<<grid_for(waves_needed * WAVE), 256, 0, stream>>>(col, rowptr, rs.rows, rs.row_len, k, idx);
        if (launch_status() != DROPIT_OK) return DROPIT_EHIP;
    }
    return dropit_weight_grad(vals, k > 0 ? idx : nullptr, k, x_shape, ndim, dt, dY, c_out, conv, dW, workspace,
                              inner, hip_stream);
}
