// 3x3 / stride 1 / pad 1 convolution weight gradient as ONE dense GEMM over explicit im2col rows.
//
// Sec. 3.2 (convolution weight gradient): dW[j][c][u][v] = sum over images and output positions of
// dY[n][j][oy][ox] * R(a^)[n][c][oy + u - 1][ox + v - 1].  Read as a matrix product this is
// dW[j][(c, u, v)] = sum_t dYt[t][j] * B[t][(c, u, v)] with one "token" t per output position
// (n, oy, ox) and B the im2col rows of the recovered input: exactly the fully-connected form
// dY^T * x^ of the same section, with 9 * C input features.
//
// For small planes with many channels (the last stages of a ResNet: 14x14x256, 7x7x512) B is
// small (tens of MB) and the product has hundreds of output tiles, so it runs on the
// fully-connected GEMM kernel, where the row-band kernel of wgrad_conv_mfma.hip
// spends most of its time staging a few hundred positions per workgroup.  Large planes with few
// channels are the opposite case (B would be nine times the activation) and stay there.
//
// One small kernel prepares both operands: B is assembled from the (value, index) pairs in LDS
// tiles (one image x a block of channels: its pairs are one contiguous run of the sorted arrays)
// and written once in full lines, no separate zero fill; other workgroups of the same launch transpose
// dY from [N][J][H][W] to token-major [N*H*W][J].  The result lands in dW's own layout [J][C][3][3].
#include "wgrad_internal.hpp"
#include "dev_hooks.hpp"

namespace dropit {
namespace {

constexpr int IM2COL_THREADS = 256;
constexpr int IM2COL_WINDOW = 32;             // window entries per thread (see for_pairs_in_range)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int DYT_JB = 64;                    // output channels per transposing workgroup

// dY [N][J][HW] -> dYt [N * HW][J]: workgroup (n, block of 64 output channels) moves a contiguous
// 64 x HW slab through LDS.  J % 8 == 0, so the slab starts on a 16-byte boundary and is whole
// 16-byte vectors: each thread's loads are independent vector loads, all issued before the first
// LDS store; the stores leave as pairs of neighbouring channels.
__device__ inline void dy_to_tokens(const uint16_t *__restrict__ dY, int J, int HW, int unit, int jblocks,
                                    uint16_t *__restrict__ dYt, uint16_t *slab /* [64][HW | 1] */)
{
    const int n = unit / jblocks, j0 = (unit % jblocks) * DYT_JB;
    const int jw = min(DYT_JB, J - j0);                                   // a multiple of 8
    const int ld = HW | 1;                                                // odd pitch: the transposed reads spread over the banks
    const u32x4 *src = reinterpret_cast<const u32x4 *>(dY + (int64_t(n) * J + j0) * HW);
    const int vecs = jw * HW / 8;
    constexpr int BATCH = 4;
    for (int i0 = threadIdx.x; i0 < vecs; i0 += BATCH * IM2COL_THREADS) {
        u32x4 v[BATCH];
#pragma unroll
        for (int q = 0; q < BATCH; ++q)
            if (i0 + q * IM2COL_THREADS < vecs) v[q] = src[i0 + q * IM2COL_THREADS];
#pragma unroll
        for (int q = 0; q < BATCH; ++q) {
            const int i = i0 + q * IM2COL_THREADS;
            if (i >= vecs) continue;
            int jj = (i * 8) / HW, t = i * 8 - jj * HW;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                slab[jj * ld + t] = uint16_t(v[q][e >> 1] >> ((e & 1) * 16));
                if (++t == HW) {
                    t = 0;
                    ++jj;
                }
            }
        }
    }
    __syncthreads();
    uint32_t *dst = reinterpret_cast<uint32_t *>(dYt + int64_t(n) * HW * J + j0);     // j0 and J are even
    for (int i = threadIdx.x; i < HW * (DYT_JB / 2); i += IM2COL_THREADS) {
        const int t = i / (DYT_JB / 2), jj = (i % (DYT_JB / 2)) * 2;
        if (jj < jw) dst[(int64_t(t) * J + jj) / 2] = uint32_t(slab[jj * ld + t]) | (uint32_t(slab[(jj + 1) * ld + t]) << 16);
    }
}

// Both operands of the GEMM in one launch.  Workgroup (n, channel block), the first N * cblocks: the
// im2col columns [9 * c0, 9 * (c0 + cw)) of the H * W token rows of image n.  The next pad_wgs
// workgroups zero the pad rows [ntok, ntok_pad) of B; the last N * jblocks transpose dY.
__global__ void __launch_bounds__(IM2COL_THREADS)
conv_im2col_kernel(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx, int64_t k, int N, int C,
                   int H, int W, int cb, int cblocks, int pitch, int64_t ntok, int64_t ntok_pad, int pad_wgs,
                   int64_t margin, uint16_t *__restrict__ B, const uint16_t *__restrict__ dY, int J, int jblocks,
                   uint16_t *__restrict__ dYt)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t tile[];      // [H * W][cw * 9], or the dY slab
    const int tid = threadIdx.x;
    const int units = N * cblocks;
    if (int(blockIdx.x) >= units + pad_wgs) {
        dy_to_tokens(dY, J, H * W, int(blockIdx.x) - units - pad_wgs, jblocks, dYt, tile);
        return;
    }
    if (int(blockIdx.x) >= units) {
        // pad rows: 16-byte zero stores, shared among the extra workgroups
        const int64_t chunks = (ntok_pad - ntok) * pitch / 8;
        u32x4 *dst = reinterpret_cast<u32x4 *>(B + ntok * pitch);
        const int64_t stride = int64_t(pad_wgs) * IM2COL_THREADS;
        for (int64_t i = int64_t(blockIdx.x - units) * IM2COL_THREADS + tid; i < chunks; i += stride)
            dst[i] = u32x4{0u, 0u, 0u, 0u};
        return;
    }
    const int n = blockIdx.x / cblocks, c0 = (blockIdx.x % cblocks) * cb;
    const int cw = min(cb, C - c0);
    const int HW = H * W, row = cw * 9;                                   // row: 16-bit elements per token in the tile
    const int64_t lo = (int64_t(n) * C + c0) * HW, hi = lo + int64_t(cw) * HW;

    u32x4 *tile16 = reinterpret_cast<u32x4 *>(tile);
    const int chunks = HW * row / 8;                                      // cw % 8 == 0

    // element (c, ih, iw) is the (u, v) tap of output position (ih + 1 - u, iw + 1 - v)
    auto place = [&](int32_t flat, uint32_t v16) {
        const uint32_t rel = uint32_t(int64_t(flat) - lo);
        if (rel >= uint32_t(cw * HW)) return;                             // another workgroup's pair
        const uint32_t c = rel / uint32_t(HW), rem = rel - c * uint32_t(HW);
        const int ih = int(rem / uint32_t(W)), iw = int(rem - uint32_t(ih) * uint32_t(W));
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int oy = ih + 1 - u;
            if (oy < 0 || oy >= H) continue;
#pragma unroll
            for (int v = 0; v < 3; ++v) {
                const int ox = iw + 1 - v;
                if (ox < 0 || ox >= W) continue;
                tile[(oy * W + ox) * row + int(c) * 9 + u * 3 + v] = uint16_t(v16);
            }
        }
    };
    // the pairs of [lo, hi): one round of loads around their interpolated position, else a search
    for_pairs_in_range<IM2COL_THREADS, IM2COL_WINDOW>(vals, idx, k, int64_t(N) * C * HW, lo, hi, margin, place, [&] {
        for (int i = tid; i < chunks; i += IM2COL_THREADS) tile16[i] = u32x4{0u, 0u, 0u, 0u};
    });
    __syncthreads();

    // a token's segment is row * 2 bytes (a multiple of 144) at a 16-byte aligned column offset
    const int per_row = row / 8;
    for (int i = tid; i < chunks; i += IM2COL_THREADS) {
        const int t = i / per_row, w = i - t * per_row;
        u32x4 *dst = reinterpret_cast<u32x4 *>(B + (int64_t(n) * HW + t) * pitch + int64_t(c0) * 9);
        dst[w] = tile16[i];
    }
}

}  // namespace

ConvGemmPlan conv_gemm_plan(const ConvProblem &p)
{
    ConvGemmPlan plan;
    plan.fp = FcProblem{p.N * p.H * p.W, 9 * p.C, p.J, p.k};
    plan.gemm = fc_dense_plan(plan.fp);
    const int64_t HW = p.H * p.W;
    // channel block: a multiple of 8, its tile within the LDS budget where that leaves at least 8 channels
    int64_t budget = 32 * 1024;                // several workgroups per compute unit (measured: 16-24 KB and 64+ KB slower)
    budget = dev_env("DROPIT_IM2COL_LDS", budget);
    int64_t cb = budget / (HW * 18) / 8 * 8;
    // ... but token segments of at least 16 channels (288 bytes) while the tile stays within 64 KB:
    // with 8 (144 bytes, 2.25 lines) the writes of B were 3 us slower on 14x14 planes
    if (cb < 16 && HW * 16 * 18 <= 64 * 1024) cb = 16;
    cb = std::max<int64_t>(8, std::min<int64_t>(cb, 64));
    cb = std::min<int64_t>(cb, p.C);
    plan.cb = int(cb);
    plan.cblocks = int((p.C + cb - 1) / cb);
    plan.lds_bytes = size_t(HW) * cb * 18;
    plan.dyt_bytes = round_up(size_t(plan.fp.ntok) * p.J * 2, 256);
    return plan;
}

bool conv_gemm_supported(const ConvProblem &p)
{
    if (p.C % 8 != 0 || p.J % 8 != 0 || p.H < 1 || p.W < 1) return false;
    const int64_t HW = p.H * p.W;
    if (HW > 256 || p.N * HW >= (int64_t(1) << 31) / (9 * p.C)) return false;
    if (p.N * p.C > INT32_MAX / 2) return false;
    return fc_dense_supported(FcProblem{p.N * HW, 9 * p.C, p.J, p.k});
}

// Taken for small planes with many channels, where the im2col rows are small and the product is
// large enough to be worth three more dispatches: measured against the row-band kernel on
// ResNet-50's 3x3 layers at batch 64 (56x56x64 and 28x28x128 stay there; 14x14x256 and 7x7x512
// come here).
bool conv_gemm_preferred(const ConvProblem &p)
{
    if (!conv_gemm_supported(p)) return false;
    const ConvGemmPlan plan = conv_gemm_plan(p);
    return p.H * p.W <= 200 && p.C >= 128 &&
           int64_t(plan.gemm.nb_count) * plan.gemm.mb_count * plan.gemm.nkb >= 256;
}

dropit_status conv_gemm_run(const ConvProblem &p, const ConvGemmPlan &plan, const void *vals, const int32_t *idx,
                            const void *dY, float *dW, char *ws, hipStream_t stream)
{
    uint16_t *B = reinterpret_cast<uint16_t *>(ws);
    float *partial = reinterpret_cast<float *>(ws + plan.gemm.dense_bytes);
    uint16_t *dYt = reinterpret_cast<uint16_t *>(ws + plan.gemm.dense_bytes + plan.gemm.partial_bytes);
    const int64_t ntok_pad = plan.gemm.ntok_pad;          // B is padded to whole token blocks of the GEMM with zero rows
    if (ntok_pad < plan.fp.ntok || size_t(ntok_pad) * plan.gemm.pitch * 2 > plan.gemm.dense_bytes) return DROPIT_EINVAL;
    const int HW = int(p.H * p.W);

    static std::atomic<uint64_t> attr_set{0};
    if (!once_per_device(attr_set, [] {
            return hipFuncSetAttribute(reinterpret_cast<const void *>(conv_im2col_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024) == hipSuccess;
        }))
        return DROPIT_EHIP;

    trace_mark(stream);
    const int units = int(p.N) * plan.cblocks;
    const int64_t pad_chunks = (ntok_pad - plan.fp.ntok) * plan.gemm.pitch / 8;
    const int pad_wgs = int(std::min<int64_t>((pad_chunks + IM2COL_THREADS - 1) / IM2COL_THREADS, 64));
    const int jblocks = int((p.J + DYT_JB - 1) / DYT_JB);
    // half-width of the pair window: 4 standard deviations of an evenly spread selection plus a little
    const int64_t margin = 2 * static_cast<int64_t>(__builtin_sqrt(static_cast<double>(p.k))) + 256;
    const size_t lds = std::max(plan.lds_bytes, size_t(DYT_JB) * (HW | 1) * 2);
    conv_im2col_kernel<<<units + pad_wgs + int(p.N) * jblocks, IM2COL_THREADS, lds, stream>>>(
        static_cast<const uint16_t *>(vals), idx, p.k, int(p.N), int(p.C), int(p.H), int(p.W), plan.cb, plan.cblocks,
        plan.gemm.pitch, plan.fp.ntok, ntok_pad, pad_wgs, margin, B, static_cast<const uint16_t *>(dY), int(p.J), jblocks, dYt);
    trace_mark(stream);
    if (launch_status() != DROPIT_OK) return DROPIT_EHIP;
    return fc_dense_gemm(plan.fp, plan.gemm, dYt, B, partial, dW, stream);
}

}  // namespace dropit
