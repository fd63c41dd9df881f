// Weight gradient from the sparsified cache (Sec. 3.2): recover R(a^) (zeros at
// dropped positions) and take the ordinary dense weight gradient,
//   FC   : dW[j][c]       = sum_n dY[n][j] * R(a^)[n][c]            (Eq. fc_backward_elem_save)
//   conv : dW[j][c][u][v] = sum_{n,oy,ox} dY[n][j][oy][ox] * R(a^)[n][c][oy+u-1][ox+v-1]
//                                                                   (Eq. conv_backward_elem, 3x3/s1/p1)
//
// This file holds the host entry points and the generic fp32-FMA kernels
// (exact fp32 products, fixed summation order).  They serve fp32 inputs and
// any bf16 shape the MFMA kernels do not cover.
#include "common.hpp"
#include "wgrad_internal.hpp"
#include "dev_hooks.hpp"
#include <cstdlib>

namespace dropit {
namespace {

__device__ inline float to_f32(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }
__device__ inline float to_f32(uint32_t b) { return __uint_as_float(b); }

// ---- recover R(a^) into a dense buffer of the input type ------------------
__global__ void __launch_bounds__(256) zero_kernel(uint4 *p, size_t n16)
{
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (size_t i = blockIdx.x * size_t(blockDim.x) + threadIdx.x; i < n16; i += size_t(gridDim.x) * blockDim.x)
        p[i] = z;
}

__global__ void __launch_bounds__(256) zero_f32_kernel(float *p, int64_t n)
{
    for (int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; i < n; i += int64_t(gridDim.x) * blockDim.x)
        p[i] = 0.f;
}

template <typename RAW>
__global__ void __launch_bounds__(256) scatter_kernel(const RAW *__restrict__ vals, const int32_t *__restrict__ idx,
                                                      int64_t k, int64_t numel, RAW *__restrict__ dense)
{
    for (int64_t j = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; j < k; j += int64_t(gridDim.x) * blockDim.x) {
        const int64_t i = idx[j];
        if (i >= 0 && i < numel) dense[i] = vals[j];   // an out-of-range index is ignored, never written
    }
}

// ---- FC: 64x64 output tile per workgroup, 4x4 per thread, fp32 FMA --------
constexpr int FT = 64;      // tile edge
constexpr int FK = 64;      // tokens per step

// The next step's operands are fetched into registers while the current step multiplies, so a short
// problem (a few steps) does not pay one memory round trip per step.  Every output element still adds
// its terms in ascending token order: the result does not depend on FK.
template <typename RAW>
__global__ void __launch_bounds__(256)
fc_fma_kernel(const RAW *__restrict__ xhat, const RAW *__restrict__ dY, int64_t ntok, int cin, int cout,
              float *__restrict__ dW)
{
    __shared__ float sA[FK][FT + 4];   // dY tile  [token][j]
    __shared__ float sB[FK][FT + 4];   // x^ tile  [token][c]
    constexpr int PER = FK * FT / 256; // elements of each tile a thread moves
    const int tid = threadIdx.x;
    const int j0 = blockIdx.y * FT, c0 = blockIdx.x * FT;
    const int tj = (tid / 16) * 4, tc = (tid % 16) * 4;
    float acc[4][4] = {};
    float na[PER], nb[PER];
    auto fetch = [&](int64_t n0) {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int e = tid + u * 256, r = e / FT, q = e % FT;
            const int64_t n = n0 + r;
            na[u] = (n < ntok && j0 + q < cout) ? to_f32(dY[n * cout + j0 + q]) : 0.f;
            nb[u] = (n < ntok && c0 + q < cin) ? to_f32(xhat[n * cin + c0 + q]) : 0.f;
        }
    };
    fetch(0);
    for (int64_t n0 = 0; n0 < ntok; n0 += FK) {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int e = tid + u * 256, r = e / FT, q = e % FT;
            sA[r][q] = na[u];
            sB[r][q] = nb[u];
        }
        __syncthreads();
        if (n0 + FK < ntok) fetch(n0 + FK);
#pragma unroll 16
        for (int r = 0; r < FK; ++r) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sA[r][tj + i]; b[i] = sB[r][tc + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[i][q] = __builtin_fmaf(a[i], b[q], acc[i][q]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (j0 + tj + i < cout && c0 + tc + q < cin)
                dW[int64_t(j0 + tj + i) * cin + c0 + tc + q] = acc[i][q];
}

// ---- FC, small layers: recover and multiply in ONE launch --------------------------------------------
// A layer whose whole input fits the LDS of a compute unit (numel <= SMALL_NUMEL fp32 values) is bound by
// launches, not by work: the zero fill, the scatter and the product as three kernels cost three dispatch
// slots for a few microseconds of arithmetic.  Here every workgroup rebuilds the whole R(a^) in its own LDS
// (zero fill, then one store per pair: the k pairs are a few thousand), fetches its SMALL_JB columns of dY,
// and multiplies: thread (j, c-group) adds its terms in ascending token order with true fp32 multiply-adds
// (bf16 inputs are widened exactly), the same order and arithmetic as fc_fma_kernel.
constexpr int SMALL_NUMEL = 16384;         // elements of x: 64 KB of fp32 in LDS
constexpr int SMALL_TOKENS = 1024;         // tokens: the dY slice is SMALL_TOKENS x SMALL_JB fp32 = 64 KB
constexpr int SMALL_JB = 16;               // rows of dW per workgroup

template <typename RAW>
__global__ void __launch_bounds__(256)
fc_small_kernel(const RAW *__restrict__ vals, const int32_t *__restrict__ idx, int k, const RAW *__restrict__ dY,
                int ntok, int cin, int cout, float *__restrict__ dW)
{
    extern __shared__ __attribute__((aligned(16))) float small_lds[];
    float *xs = small_lds;                                 // R(a^)  [ntok][cin]
    float *gs = small_lds + ntok * cin;                    // dY     [ntok][SMALL_JB], columns j0 ..
    const int tid = threadIdx.x;
    const int j0 = blockIdx.x * SMALL_JB;
    const int numel = ntok * cin;                          // a multiple of 4 (cin is)
    float4 *xs4 = reinterpret_cast<float4 *>(xs);
    for (int i = tid; i < numel / 4; i += 256) xs4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int e = tid; e < ntok * SMALL_JB; e += 256) {
        const int n = e / SMALL_JB, j = j0 + e % SMALL_JB;
        gs[e] = j < cout ? to_f32(dY[int64_t(n) * cout + j]) : 0.f;
    }
    __syncthreads();
    for (int q = tid; q < k; q += 256) {
        const int i = idx[q];
        if (i >= 0 && i < numel) xs[i] = to_f32(vals[q]);  // an out-of-range index is ignored, never written
    }
    __syncthreads();
    const int j = tid / 16;                                // 16 rows of dW x 16 groups of 4 columns per pass
    for (int c0 = (tid % 16) * 4; c0 < cin; c0 += 64) {
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        for (int n = 0; n < ntok; ++n) {
            const float g = gs[n * SMALL_JB + j];
            const float4 b = *reinterpret_cast<const float4 *>(xs + n * cin + c0);
            acc[0] = __builtin_fmaf(g, b.x, acc[0]);
            acc[1] = __builtin_fmaf(g, b.y, acc[1]);
            acc[2] = __builtin_fmaf(g, b.z, acc[2]);
            acc[3] = __builtin_fmaf(g, b.w, acc[3]);
        }
        if (j0 + j < cout)
            *reinterpret_cast<float4 *>(dW + int64_t(j0 + j) * cin + c0) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    }
}

// ---- conv 3x3 / stride 1 / pad 1: one workgroup per (j, c), fixed-order reduce
template <typename RAW>
__global__ void __launch_bounds__(256)
conv3x3_fma_kernel(const RAW *__restrict__ xhat, const RAW *__restrict__ dY, int N, int C, int H, int W, int cout,
                   float *__restrict__ dW)
{
    __shared__ float red[256][9];
    const int j = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
    float acc[9] = {};
    const int plane = H * W;
    for (int n = 0; n < N; ++n) {
        const RAW *xp = xhat + (int64_t(n) * C + c) * plane;
        const RAW *gp = dY + (int64_t(n) * cout + j) * plane;
        for (int p = tid; p < plane; p += 256) {
            const int oy = p / W, ox = p % W;
            const float g = to_f32(gp[p]);
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const int iy = oy + u - 1;
#pragma unroll
                for (int v = 0; v < 3; ++v) {
                    const int ix = ox + v - 1;
                    if (iy >= 0 && iy < H && ix >= 0 && ix < W)
                        acc[u * 3 + v] = __builtin_fmaf(g, to_f32(xp[iy * W + ix]), acc[u * 3 + v]);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 9; ++i) red[tid][i] = acc[i];
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s)
#pragma unroll
            for (int i = 0; i < 9; ++i) red[tid][i] += red[tid + s][i];
        __syncthreads();
    }
    if (tid < 9) dW[(int64_t(j) * C + c) * 9 + tid] = red[0][tid];
}

// ---- any other convolution geometry: one workgroup per (j, c), taps in chunks of 16 ----
// Each thread walks the output positions (n, oy, ox) with a fixed stride and keeps 16 tap sums;
// the workgroup adds them up in a fixed tree, so the result is reproducible.  Slow (the data is
// walked once per 16 taps) but exact, for the geometries the matrix-core kernel does not take.
constexpr int TAP_CHUNK = 16;
// Element strides of the two layouts: x and dY as (image, channel, row, column), dW as (filter, channel, tap).
struct ConvStrides {
    int64_t xn, xc, xh, xw, yn, yc, yh, yw, wj, wc, wt;
};

template <typename RAW>
__global__ void __launch_bounds__(256)
conv_general_fma_kernel(const RAW *__restrict__ xhat, const RAW *__restrict__ dY, int N, int C, int H, int W, int cout,
                        int OH, int OW, int kh, int kw, int sh, int sw, int ph, int pw, int dh, int dw,
                        ConvStrides st, float *__restrict__ dW)
{
    __shared__ float red[256][TAP_CHUNK + 1];
    const int j = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
    const int taps = kh * kw;
    const int64_t oplane = int64_t(OH) * OW;
    const int64_t positions = int64_t(N) * oplane;
    for (int t0 = 0; t0 < taps; t0 += TAP_CHUNK) {
        float acc[TAP_CHUNK];
#pragma unroll
        for (int q = 0; q < TAP_CHUNK; ++q) acc[q] = 0.f;
        for (int64_t p = tid; p < positions; p += 256) {
            const int n = int(p / oplane);
            const int r = int(p - int64_t(n) * oplane);
            const int oy = r / OW, ox = r - oy * OW;
            const float g = to_f32(dY[n * st.yn + j * st.yc + oy * st.yh + ox * st.yw]);
            const RAW *xp = xhat + n * st.xn + c * st.xc;
#pragma unroll
            for (int q = 0; q < TAP_CHUNK; ++q) {
                const int tap = t0 + q;                         // uniform
                if (tap < taps) {
                    const int u = tap / kw, v = tap - u * kw;
                    const int64_t iy = int64_t(oy) * sh - ph + int64_t(u) * dh, ix = int64_t(ox) * sw - pw + int64_t(v) * dw;
                    if (iy >= 0 && iy < H && ix >= 0 && ix < W)
                        acc[q] = __builtin_fmaf(g, to_f32(xp[iy * st.xh + ix * st.xw]), acc[q]);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < TAP_CHUNK; ++q) red[tid][q] = acc[q];
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s)
#pragma unroll
                for (int q = 0; q < TAP_CHUNK; ++q) red[tid][q] += red[tid + s][q];
            __syncthreads();
        }
        if (tid < TAP_CHUNK && t0 + tid < taps) dW[j * st.wj + c * st.wc + (t0 + tid) * st.wt] = red[0][tid];
        __syncthreads();
    }
}

struct Problem {
    bool conv;
    int64_t numel, ntok, cin, cout;
    int64_t N, C, H, W, OH, OW;
    dropit_conv2d g;
    bool is_3x3_s1_p1;
    bool nhwc;                                   // x [N][H][W][C], dY [N][OH][OW][J], dW [J][kh][kw][C]
};

// Validates shape arguments; returns DROPIT_OK and fills `p`.
dropit_status describe(const int64_t *x_shape, int ndim, dropit_dtype dt, int64_t c_out,
                       const dropit_conv2d *conv, Problem &p, bool nhwc = false)
{
    p.nhwc = nhwc;
    if (dt != DROPIT_F32 && dt != DROPIT_BF16) return DROPIT_EINVAL;
    p.numel = checked_numel(x_shape, ndim);
    if (p.numel < 1 || c_out < 1 || c_out > INT32_MAX) return DROPIT_EINVAL;
    p.cout = c_out;
    p.conv = conv != nullptr;
    p.is_3x3_s1_p1 = false;
    p.g = dropit_conv2d{};
    p.N = p.C = p.H = p.W = p.OH = p.OW = 0;
    if (!p.conv) {
        p.cin = x_shape[ndim - 1];
        p.ntok = p.numel / p.cin;
        if (p.ntok * c_out > int64_t(1) << 40) return DROPIT_EINVAL;
        return DROPIT_OK;
    }
    if (ndim != 4) return DROPIT_EINVAL;
    if (conv->kh < 1 || conv->kw < 1 || conv->stride_h < 1 || conv->stride_w < 1 || conv->pad_h < 0 ||
        conv->pad_w < 0 || conv->dil_h < 1 || conv->dil_w < 1)
        return DROPIT_EINVAL;
    p.g = *conv;
    p.is_3x3_s1_p1 = conv->kh == 3 && conv->kw == 3 && conv->stride_h == 1 && conv->stride_w == 1 && conv->pad_h == 1 &&
                     conv->pad_w == 1 && conv->dil_h == 1 && conv->dil_w == 1;
    p.N = x_shape[0];
    if (nhwc) {
        p.H = x_shape[1]; p.W = x_shape[2]; p.C = x_shape[3];
    } else {
        p.C = x_shape[1]; p.H = x_shape[2]; p.W = x_shape[3];
    }
    constexpr int64_t GEOM_MAX = 65535;              // keeps every index expression far inside 64 bits
    if (conv->kh > 1024 || conv->kw > 1024 || conv->pad_h > GEOM_MAX || conv->pad_w > GEOM_MAX ||
        conv->stride_h > GEOM_MAX || conv->stride_w > GEOM_MAX || conv->dil_h > GEOM_MAX || conv->dil_w > GEOM_MAX)
        return DROPIT_EINVAL;
    const int64_t eh = p.H + 2 * conv->pad_h - conv->dil_h * (conv->kh - 1) - 1;   // output extent: floor(e / stride) + 1
    const int64_t ew = p.W + 2 * conv->pad_w - conv->dil_w * (conv->kw - 1) - 1;
    if (eh < 0 || ew < 0) return DROPIT_EINVAL;                                    // the window does not fit the padded input
    p.OH = eh / conv->stride_h + 1;
    p.OW = ew / conv->stride_w + 1;
    if (p.N * c_out * p.OH * p.OW > INT32_MAX * int64_t(16)) return DROPIT_EINVAL;
    if (c_out * p.C * conv->kh * conv->kw > INT32_MAX) return DROPIT_EINVAL;
    // A channels-last 1x1 / stride 1 / unpadded convolution IS a fully-connected layer over the N*H*W
    // positions: x [N*H*W][C], dY [N*H*W][J], dW [J][1][1][C] = [J][C].  It takes the FC kernels.
    if (nhwc && conv->kh == 1 && conv->kw == 1 && conv->stride_h == 1 && conv->stride_w == 1 && conv->pad_h == 0 &&
        conv->pad_w == 0) {
        p.conv = false;
        p.cin = p.C;
        p.ntok = p.numel / p.C;
    }
    return DROPIT_OK;
}

size_t dense_bytes(const Problem &p, dropit_dtype dt)
{
    return round_up(size_t(p.numel) * (dt == DROPIT_F32 ? 4 : 2), 256);
}

template <typename RAW>
dropit_status run_generic(const Problem &p, const void *vals, const int32_t *idx, int64_t k, const void *dY,
                          float *dW, char *ws, size_t dense_sz, hipStream_t stream)
{
    RAW *dense = reinterpret_cast<RAW *>(ws);
    trace_mark(stream);
    zero_kernel<<<1024, 256, 0, stream>>>(reinterpret_cast<uint4 *>(dense), dense_sz / 16);
    if (k > 0) {
        const int blocks = static_cast<int>(std::min<int64_t>((k + 255) / 256, 4096));
        scatter_kernel<RAW><<<blocks, 256, 0, stream>>>(static_cast<const RAW *>(vals), idx, k, p.numel, dense);
    }
    trace_mark(stream);
    if (!p.conv) {
        const dim3 grid((p.cin + FT - 1) / FT, (p.cout + FT - 1) / FT);
        fc_fma_kernel<RAW><<<grid, 256, 0, stream>>>(dense, static_cast<const RAW *>(dY), p.ntok, int(p.cin),
                                                      int(p.cout), dW);
    } else {
        const dim3 grid(p.C, p.cout);
        const int64_t taps = p.g.kh * p.g.kw;
        const ConvStrides st = p.nhwc
            ? ConvStrides{p.H * p.W * p.C, 1, p.W * p.C, p.C, p.OH * p.OW * p.cout, 1, p.OW * p.cout, p.cout, taps * p.C, 1, p.C}
            : ConvStrides{p.C * p.H * p.W, p.H * p.W, p.W, 1, p.cout * p.OH * p.OW, p.OH * p.OW, p.OW, 1, p.C * taps, taps, 1};
        if (p.is_3x3_s1_p1 && !p.nhwc)
            conv3x3_fma_kernel<RAW><<<grid, 256, 0, stream>>>(dense, static_cast<const RAW *>(dY), int(p.N), int(p.C),
                                                               int(p.H), int(p.W), int(p.cout), dW);
        else
            conv_general_fma_kernel<RAW><<<grid, 256, 0, stream>>>(
                dense, static_cast<const RAW *>(dY), int(p.N), int(p.C), int(p.H), int(p.W), int(p.cout), int(p.OH),
                int(p.OW), int(p.g.kh), int(p.g.kw), int(p.g.stride_h), int(p.g.stride_w), int(p.g.pad_h),
                int(p.g.pad_w), int(p.g.dil_h), int(p.g.dil_w), st, dW);
    }
    trace_mark(stream);
    return launch_status();
}

}  // namespace
}  // namespace dropit

using namespace dropit;

static bool use_fc_dense(const FcProblem &fp) { return fc_dense_supported(fp); }

static ConvGeneral general_of(const Problem &p, int64_t k)
{
    return ConvGeneral{p.N, p.C, p.H, p.W, p.OH, p.OW, p.cout, k, p.g, p.nhwc};
}

// Which kernels serve this problem.
static bool fc_small(const Problem &p)
{
    return !p.conv && p.numel <= SMALL_NUMEL && p.ntok <= SMALL_TOKENS && p.cin % 4 == 0 && p.cout <= 4096;
}

// 0: recover into a dense operand in the workspace, then the product; 1: recover inside the product where that
// form exists (see dropit_set_fc_recover).  Per host thread.
static int &fc_recover_form()
{
    static thread_local int form = 0;
    return form;
}

static dropit_wgrad_path choose_path(const Problem &p, dropit_dtype dt, int64_t k)
{
    if (fc_small(p)) return DROPIT_PATH_FC_SMALL;
    if (dt != DROPIT_BF16) return DROPIT_PATH_FMA;
    if (!p.conv) {
        const FcProblem fp = {p.ntok, p.cin, p.cout, k};
        if (!use_fc_dense(fp)) return DROPIT_PATH_FMA;
        return fc_recover_form() == 1 && k >= 1 && fc_fused_supported(fp) ? DROPIT_PATH_FC_FUSED : DROPIT_PATH_FC_MFMA;
    }
    if (p.is_3x3_s1_p1 && !p.nhwc) {
        const ConvProblem cp = {p.N, p.C, p.H, p.W, p.cout, k};
        bool gemm = conv_gemm_preferred(cp);
        if (const long forced = dev_env("DROPIT_CONV_GEMM", -1); forced >= 0) gemm = forced == 1 && conv_gemm_supported(cp);
        if (gemm) return DROPIT_PATH_CONV_GEMM;
        if (conv_mfma_supported(cp)) return DROPIT_PATH_CONV_BANDS;
    }
    return conv_im2col_supported(general_of(p, k)) ? DROPIT_PATH_CONV_IM2COL : DROPIT_PATH_FMA;
}

// Workspace need of the path dropit_weight_grad will take for this problem.
static size_t workspace_need(const Problem &p, dropit_dtype dt, int64_t k)
{
    const ConvProblem cp = {p.N, p.C, p.H, p.W, p.cout, k};
    switch (choose_path(p, dt, k)) {
    case DROPIT_PATH_FC_MFMA: return fc_dense_plan(FcProblem{p.ntok, p.cin, p.cout, k}).total();
    case DROPIT_PATH_FC_FUSED: return fc_dense_plan(FcProblem{p.ntok, p.cin, p.cout, k}, true).total();
    case DROPIT_PATH_CONV_GEMM: return conv_gemm_plan(cp).total();
    case DROPIT_PATH_CONV_BANDS: return conv_mfma_plan(cp).total();
    case DROPIT_PATH_CONV_IM2COL: return conv_im2col_plan(general_of(p, k)).total();
    case DROPIT_PATH_FC_SMALL: return 256;           // nothing is kept outside LDS; a token size so that callers' buffers exist
    default: return dense_bytes(p, dt);
    }
}

static dropit_status run(const Problem &p, const void *vals, const int32_t *idx, int64_t k, dropit_dtype dt,
                         const void *dY, float *dW, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (k < 0 || k > p.numel) return DROPIT_EINVAL;
    if (k > 0 && (vals == nullptr || idx == nullptr)) return DROPIT_EINVAL;
    if (k > 0 && (!aligned(vals, dt == DROPIT_F32 ? 4 : 2) || !aligned(idx, 4))) return DROPIT_EINVAL;
    if (dY == nullptr || dW == nullptr || !aligned(dY, 16) || !aligned(dW, 16)) return DROPIT_EINVAL;
    if (workspace == nullptr || !aligned(workspace, 256)) return DROPIT_EINVAL;
    const size_t need = workspace_need(p, dt, k);
    if (workspace_bytes < need) return DROPIT_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    if (k == 0) {                                  // everything was dropped: R(a^) = 0, so dW = 0
        const int64_t n = p.conv ? p.cout * p.C * p.g.kh * p.g.kw : p.cout * p.cin;
        zero_f32_kernel<<<int(std::min<int64_t>((n + 255) / 256, 2048)), 256, 0, stream>>>(dW, n);
        return launch_status();
    }
    const ConvProblem cp = {p.N, p.C, p.H, p.W, p.cout, k};
    switch (choose_path(p, dt, k)) {
    case DROPIT_PATH_FC_MFMA: {
        const FcProblem fp = {p.ntok, p.cin, p.cout, k};
        return fc_dense_run(fp, fc_dense_plan(fp), vals, idx, dY, dW, ws, stream);
    }
    case DROPIT_PATH_FC_FUSED: {
        const FcProblem fp = {p.ntok, p.cin, p.cout, k};
        return fc_fused_run(fp, fc_dense_plan(fp, true), vals, idx, dY, dW, ws, stream);
    }
    case DROPIT_PATH_CONV_GEMM: return conv_gemm_run(cp, conv_gemm_plan(cp), vals, idx, dY, dW, ws, stream);
    case DROPIT_PATH_CONV_BANDS: return conv_mfma_run(cp, conv_mfma_plan(cp), vals, idx, dY, dW, ws, stream);
    case DROPIT_PATH_CONV_IM2COL: {
        const ConvGeneral cg = general_of(p, k);
        return conv_im2col_run(cg, conv_im2col_plan(cg), vals, idx, dY, dW, ws, stream);
    }
    case DROPIT_PATH_FC_SMALL: {
        const size_t lds = size_t(p.numel + p.ntok * SMALL_JB) * sizeof(float);
        const unsigned grid = unsigned((p.cout + SMALL_JB - 1) / SMALL_JB);
        trace_mark(stream);
        if (dt == DROPIT_BF16) {
            static std::atomic<uint64_t> set_up{0};
            if (!once_per_device(set_up, [] {
                    return hipFuncSetAttribute(reinterpret_cast<const void *>(fc_small_kernel<uint16_t>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               int((SMALL_NUMEL + SMALL_TOKENS * SMALL_JB) * sizeof(float))) == hipSuccess;
                }))
                return DROPIT_EHIP;
            fc_small_kernel<uint16_t><<<grid, 256, lds, stream>>>(static_cast<const uint16_t *>(vals), idx, int(k),
                                                                  static_cast<const uint16_t *>(dY), int(p.ntok),
                                                                  int(p.cin), int(p.cout), dW);
        } else {
            static std::atomic<uint64_t> set_up{0};
            if (!once_per_device(set_up, [] {
                    return hipFuncSetAttribute(reinterpret_cast<const void *>(fc_small_kernel<uint32_t>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               int((SMALL_NUMEL + SMALL_TOKENS * SMALL_JB) * sizeof(float))) == hipSuccess;
                }))
                return DROPIT_EHIP;
            fc_small_kernel<uint32_t><<<grid, 256, lds, stream>>>(static_cast<const uint32_t *>(vals), idx, int(k),
                                                                  static_cast<const uint32_t *>(dY), int(p.ntok),
                                                                  int(p.cin), int(p.cout), dW);
        }
        trace_mark(stream);
        return launch_status();
    }
    default: break;
    }
    if (dt == DROPIT_BF16) return run_generic<uint16_t>(p, vals, idx, k, dY, dW, ws, need, stream);
    return run_generic<uint32_t>(p, vals, idx, k, dY, dW, ws, need, stream);
}

extern "C" dropit_status dropit_set_fc_recover(int form)
{
    if (form != 0 && form != 1) return DROPIT_EINVAL;
    fc_recover_form() = form;
    return DROPIT_OK;
}

extern "C" dropit_wgrad_path dropit_weight_grad_path(const int64_t *x_shape, int ndim, dropit_dtype dt, int64_t k,
                                                     int64_t c_out, const dropit_conv2d *conv)
{
    Problem p;
    if (describe(x_shape, ndim, dt, c_out, conv, p) != DROPIT_OK) return DROPIT_PATH_NONE;
    if (k < 0 || k > p.numel) return DROPIT_PATH_NONE;
    return choose_path(p, dt, k);
}

extern "C" size_t dropit_weight_grad_workspace_bytes(const int64_t *x_shape, int ndim, dropit_dtype dt,
                                                     int64_t k, int64_t c_out, const dropit_conv2d *conv)
{
    Problem p;
    if (describe(x_shape, ndim, dt, c_out, conv, p) != DROPIT_OK) return 0;
    if (k < 0 || k > p.numel) return 0;
    return workspace_need(p, dt, k);
}

extern "C" dropit_status dropit_weight_grad(const void *vals, const int32_t *idx, int64_t k,
                                            const int64_t *x_shape, int ndim, dropit_dtype dt, const void *dY,
                                            int64_t c_out, const dropit_conv2d *conv, float *dW, void *workspace,
                                            size_t workspace_bytes, void *hip_stream)
{
    Problem p;
    const dropit_status st = describe(x_shape, ndim, dt, c_out, conv, p);
    if (st != DROPIT_OK) return st;
    return run(p, vals, idx, k, dt, dY, dW, workspace, workspace_bytes, hip_stream);
}

// ---- channels-last convolutions ------------------------------------------------
extern "C" dropit_wgrad_path dropit_weight_grad_nhwc_path(const int64_t *x_shape, dropit_dtype dt, int64_t k,
                                                          int64_t c_out, const dropit_conv2d *conv)
{
    Problem p;
    if (conv == nullptr || describe(x_shape, 4, dt, c_out, conv, p, true) != DROPIT_OK) return DROPIT_PATH_NONE;
    if (k < 0 || k > p.numel) return DROPIT_PATH_NONE;
    return choose_path(p, dt, k);
}

extern "C" size_t dropit_weight_grad_nhwc_workspace_bytes(const int64_t *x_shape, dropit_dtype dt, int64_t k,
                                                          int64_t c_out, const dropit_conv2d *conv)
{
    Problem p;
    if (conv == nullptr || describe(x_shape, 4, dt, c_out, conv, p, true) != DROPIT_OK) return 0;
    if (k < 0 || k > p.numel) return 0;
    return workspace_need(p, dt, k);
}

extern "C" dropit_status dropit_weight_grad_nhwc(const void *vals, const int32_t *idx, int64_t k,
                                                 const int64_t *x_shape, dropit_dtype dt, const void *dY,
                                                 int64_t c_out, const dropit_conv2d *conv, float *dW,
                                                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (conv == nullptr) return DROPIT_EINVAL;
    Problem p;
    const dropit_status st = describe(x_shape, 4, dt, c_out, conv, p, true);
    if (st != DROPIT_OK) return st;
    return run(p, vals, idx, k, dt, dY, dW, workspace, workspace_bytes, hip_stream);
}
