// Bit-mask form of the retained index set: one bit per element + block offsets.
//
// The paper counts the indices as the method's own memory cost (Sec. 4.3: index memory next to the
// saved activations; appendix on choosing gamma: an int32 index is as wide as an fp32 activation).
// A mask of numel/8 bytes locates the retained elements of a tensor whatever their number: smaller
// than 4-byte indices whenever more than 1/32 of the tensor is kept (gamma < 0.97), and than the
// 16-bit row form whenever more than 1/16 is.  For every block of 1024 elements the table
// blockptr[] gives the number of retained elements before it, so that any block can be expanded
// on its own: pair j of block b is the j-th set bit of its 32 mask words, at vals[blockptr[b] + j].
// The encoding is lossless; the selection itself and the weight-gradient kernels are the ones
// behind dropit_compress / dropit_weight_grad.
#include <algorithm>

#include "common.hpp"
#include "wgrad_internal.hpp"

namespace dropit {
namespace {

constexpr int MASK_BLOCK = DROPIT_MASK_BLOCK;       // elements per block offset
constexpr int BLOCK_WORDS = MASK_BLOCK / 32;
static_assert(BLOCK_WORDS % 2 == 0, "a wavefront expands two mask words per step");

__global__ void __launch_bounds__(256) mask_zero_kernel(uint32_t *__restrict__ mask, int64_t words)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < words; i += stride) mask[i] = 0u;
}

// One pass over the ascending flat indices, a wavefront per 64 consecutive pairs.  The pairs of one
// mask word are neighbours, so an OR-scan over the lanes that stops at word boundaries leaves, in
// the last lane of every run, the bits this wavefront holds for that word; that lane adds them to
// the word (atomically: a word's pairs can straddle two wavefronts).  Pair j also writes the offsets
// of the blocks that start between its predecessor and itself; j == k closes the table.
__global__ void __launch_bounds__(256)
mask_from_idx_kernel(const int32_t *__restrict__ idx, int64_t k, int64_t numel, int64_t blocks,
                     uint32_t *__restrict__ mask, int32_t *__restrict__ blockptr)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    // whole wavefronts take part in every iteration (the scan below talks across lanes)
    for (int64_t j0 = static_cast<int64_t>(blockIdx.x) * blockDim.x + (threadIdx.x - lane); j0 <= k; j0 += stride) {
        const int64_t j = j0 + lane;
        const bool pair = j < k;
        const uint32_t flat = pair ? static_cast<uint32_t>(idx[j]) : 0xffffffffu;
        if (j <= k) {
            const int64_t before = (j == 0) ? -1 : min<int64_t>(static_cast<uint32_t>(idx[j - 1]) / MASK_BLOCK, blocks);
            const int64_t here = pair ? min<int64_t>(flat / MASK_BLOCK, blocks) : blocks;
            for (int64_t b = before + 1; b <= here; ++b) blockptr[b] = static_cast<int32_t>(j);
        }
        const uint32_t w = flat >> 5;                                   // 0x7ffffff for the lanes past the last pair
        uint32_t bits = pair && static_cast<int64_t>(flat) < numel ? 1u << (flat & 31) : 0u;
#pragma unroll
        for (int o = 1; o < WAVE; o <<= 1) {
            const uint32_t up_bits = __shfl_up(bits, o, WAVE), up_w = __shfl_up(w, o, WAVE);
            if (lane >= o && up_w == w) bits |= up_bits;
        }
        const uint32_t next_w = __shfl_down(w, 1, WAVE);
        if (bits != 0u && (lane == WAVE - 1 || next_w != w)) atomicOr(&mask[w], bits);
    }
}

// Inverse, a lane per element: 64 elements (two mask words) per wavefront step; a retained element's
// place among the pairs is the block's offset plus the set bits before it, and neighbouring retained
// elements write neighbouring indices.
__global__ void __launch_bounds__(256)
idx_from_mask_kernel(const uint32_t *__restrict__ mask, const int32_t *__restrict__ blockptr, int64_t numel,
                     int64_t blocks, int64_t k, int32_t *__restrict__ idx)
{
    const int lane = threadIdx.x & (WAVE - 1);
    const int64_t words = (numel + 31) / 32;
    const int64_t wave_id = static_cast<int64_t>(blockIdx.x) * (blockDim.x / WAVE) + threadIdx.x / WAVE;
    const int64_t waves = static_cast<int64_t>(gridDim.x) * (blockDim.x / WAVE);
    for (int64_t b = wave_id; b < blocks; b += waves) {
        int64_t base = blockptr[b];
#pragma unroll 4
        for (int s = 0; s < BLOCK_WORDS / 2; ++s) {
            const int64_t w0 = b * BLOCK_WORDS + 2 * s;
            const uint32_t lo = w0 < words ? mask[w0] : 0u, hi = w0 + 1 < words ? mask[w0 + 1] : 0u;
            const uint64_t both = (static_cast<uint64_t>(hi) << 32) | lo;
            const uint64_t below = both & ((uint64_t(1) << lane) - 1);
            const int64_t j = base + __popcll(below);
            // a malformed table must not write outside idx[0, k)
            if ((both >> lane) & 1u && j >= 0 && j < k) idx[j] = static_cast<int32_t>(w0 * 32 + lane);
            base += __popcll(both);
        }
    }
}

int64_t mask_words(int64_t numel) { return (numel + 31) / 32; }
int64_t mask_blocks(int64_t numel) { return (numel + MASK_BLOCK - 1) / MASK_BLOCK; }

unsigned grid_for(int64_t threads_needed)
{
    return static_cast<unsigned>(std::min<int64_t>(std::max<int64_t>((threads_needed + 255) / 256, 1), 256 * 16));
}

}  // namespace
}  // namespace dropit

using namespace dropit;

extern "C" size_t dropit_compress_mask_workspace_bytes(int64_t numel, int64_t k, dropit_dtype dt)
{
    const size_t select_bytes = dropit_compress_workspace_bytes(numel, dt);
    if (select_bytes == 0 || k < 0 || k > numel) return 0;
    return round_up(select_bytes, 256) + round_up(static_cast<size_t>(k) * 4 + 4, 256);
}

extern "C" dropit_status dropit_compress_mask(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                                              double gamma, void *vals, uint32_t *mask, int32_t *blockptr,
                                              void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (dt != DROPIT_F32 && dt != DROPIT_BF16) return DROPIT_EINVAL;
    const int64_t numel = checked_numel(shape, ndim);
    if (numel < 1) return DROPIT_EINVAL;
    const int64_t k = dropit_keep_count(numel, gamma);
    if (k < 0) return DROPIT_EINVAL;
    if (mask == nullptr || blockptr == nullptr || !aligned(mask, 4) || !aligned(blockptr, 4)) return DROPIT_EINVAL;
    if (workspace == nullptr || !aligned(workspace, 256)) return DROPIT_EINVAL;
    if (workspace_bytes < dropit_compress_mask_workspace_bytes(numel, k, dt)) return DROPIT_EWORKSPACE;
    const size_t select_bytes = round_up(dropit_compress_workspace_bytes(numel, dt), 256);
    int32_t *idx = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + select_bytes);
    const dropit_status st = dropit_compress(x, shape, ndim, dt, gamma, vals, idx, workspace, select_bytes, hip_stream);
    if (st != DROPIT_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    mask_zero_kernel<<<grid_for(mask_words(numel)), 256, 0, stream>>>(mask, mask_words(numel));
    mask_from_idx_kernel<<<grid_for(k + 1), 256, 0, stream>>>(idx, k, numel, mask_blocks(numel), mask, blockptr);
    trace_mark(stream);
    return launch_status();
}

extern "C" size_t dropit_weight_grad_mask_workspace_bytes(const int64_t *x_shape, int ndim, dropit_dtype dt,
                                                          int64_t k, int64_t c_out, const dropit_conv2d *conv)
{
    const size_t inner = dropit_weight_grad_workspace_bytes(x_shape, ndim, dt, k, c_out, conv);
    if (inner == 0) return 0;
    return round_up(inner, 256) + round_up(static_cast<size_t>(k) * 4 + 4, 256);
}

extern "C" dropit_status dropit_weight_grad_mask(const void *vals, const uint32_t *mask, const int32_t *blockptr,
                                                 int64_t k, const int64_t *x_shape, int ndim, dropit_dtype dt,
                                                 const void *dY, int64_t c_out, const dropit_conv2d *conv,
                                                 float *dW, void *workspace, size_t workspace_bytes,
                                                 void *hip_stream)
{
    const int64_t numel = checked_numel(x_shape, ndim);
    if (numel < 1 || k < 0 || k > numel) return DROPIT_EINVAL;
    if (mask == nullptr || blockptr == nullptr || !aligned(mask, 4) || !aligned(blockptr, 4)) return DROPIT_EINVAL;
    if (workspace == nullptr || !aligned(workspace, 256)) return DROPIT_EINVAL;
    const size_t inner = dropit_weight_grad_workspace_bytes(x_shape, ndim, dt, k, c_out, conv);
    if (inner == 0) return DROPIT_EINVAL;
    if (workspace_bytes < dropit_weight_grad_mask_workspace_bytes(x_shape, ndim, dt, k, c_out, conv))
        return DROPIT_EWORKSPACE;
    int32_t *idx = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + round_up(inner, 256));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // A bf16 fully-connected layer on the matrix cores recovers straight from the mask (c_in % 8 == 0: the
    // recovered matrix has the tensor's own layout).  Everything else expands the flat indices first.
    if (conv == nullptr && dt == DROPIT_BF16 && k > 0 && c_out >= 1) {
        const int64_t cin = x_shape[ndim - 1];
        const FcProblem fp = {numel / cin, cin, c_out, k};
        if (fc_dense_mask_native(fp) && dropit_weight_grad_path(x_shape, ndim, dt, k, c_out, conv) == DROPIT_PATH_FC_MFMA) {
            if (vals == nullptr || !aligned(vals, 2)) return DROPIT_EINVAL;
            if (dY == nullptr || dW == nullptr || !aligned(dY, 16) || !aligned(dW, 16)) return DROPIT_EINVAL;
            const FcDensePlan plan = fc_dense_plan(fp);
            if (plan.total() > inner) return DROPIT_EWORKSPACE;
            return fc_dense_run_mask(fp, plan, vals, mask, blockptr, dY, dW, static_cast<char *>(workspace), stream);
        }
    }
    if (k > 0) {
        trace_mark(stream);
        const int64_t blocks = mask_blocks(numel);
        idx_from_mask_kernel<<<grid_for(blocks * WAVE), 256, 0, stream>>>(mask, blockptr, numel, blocks, k, idx);
        if (launch_status() != DROPIT_OK) return DROPIT_EHIP;
    }
    return dropit_weight_grad(vals, k > 0 ? idx : nullptr, k, x_shape, ndim, dt, dY, c_out, conv, dW, workspace,
                              inner, hip_stream);
}
