// 3x3 / stride 1 / pad 1 convolution weight gradient from the sparsified input on
// the gfx950 matrix cores (Sec. 3.2, Eq. conv_backward_elem; recover step R(.) fused):
//   dW[j][c][u][v] = sum_{n,oy,ox} dY[n][j][oy][ox] * R(a^)[n][c][oy+u-1][ox+v-1]
//
// Implicit im2col: for each of the 9 taps this is a GEMM with M = c_out (j),
// N = c_in (c) and K = (n, oy, ox).  No im2col matrix and no dense recovered
// tensor ever exists in HBM:
//   A (dY)  : NCHW keeps ox contiguous, which is exactly the 8-consecutive-K
//             operand layout of v_mfma_f32_32x32x16_bf16, so fragments are loaded
//             straight from global memory (16 bytes per lane), one per K step,
//             shared by all 9 taps.
//   B (a^)  : a prep kernel re-buckets the sorted (value, index) pairs by
//             (image, input row, channel block).  The GEMM workgroup owns one image
//             and a band of output rows, zero-fills LDS rows [channel][8 | W | 8]
//             (zero pads left and right = the horizontal padding; rows outside the
//             image stay zero = the vertical padding) and scatters its pairs with one
//             16-bit store each.  A fragment for tap (u, v) is row oy+u-1 read at
//             ox+v-1: one aligned 16-byte read plus its two neighbouring dwords,
//             funnel-shifted by one element in registers for v = 0 and v = 2.
// One K step = 8 consecutive ox of TWO adjacent output rows (the two K-halves of the
// MFMA), so any even or odd H works and W only has to be a multiple of 8.
// Each workgroup keeps all 9 x 64 x 64 partial sums in registers and writes them
// once; a second kernel adds the per-workgroup partials in fixed order, so dW is
// bit-reproducible.
#include "common.hpp"
#include "wgrad_internal.hpp"

namespace dropit {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int CT = 256;            // threads per GEMM workgroup (4 wavefronts: 2 j-halves x 2 c-halves)
constexpr int BJ = 64, BC = 64;    // output-channel / input-channel block of a workgroup
constexpr int PREP_T = 1024;

__device__ inline int64_t block_lower_bound_1024(const int32_t *__restrict__ idx, int64_t n, int64_t target)
{
    int64_t lo = 0, hi = n;
    while (hi > lo) {
        const int64_t span = hi - lo;
        const int64_t step = (span + PREP_T - 1) / PREP_T;
        const int64_t pos = lo + int64_t(threadIdx.x) * step;
        const int pred = (pos < hi) && (int64_t(idx[pos]) < target);
        const int c = __syncthreads_count(pred);
        if (c == 0) {
            hi = lo;
        } else {
            const int64_t nlo = lo + int64_t(c - 1) * step + 1;
            const int64_t nhi = min(lo + int64_t(c) * step, hi);
            lo = nlo;
            hi = nhi;
        }
    }
    return lo;
}

// Prep: one workgroup per image.  Buckets the image's pairs by (input row h, channel
// block) and packs each as  value << 16 | local channel << 7 | w.  Order inside a bucket
// is arbitrary (each pair has its own LDS slot), so it cannot affect dW.
__global__ void __launch_bounds__(PREP_T)
conv_bucket_kernel(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx, int64_t k, int C, int H,
                   int W, int cb_count, uint32_t *__restrict__ packed, uint32_t *__restrict__ row_ptr)
{
    extern __shared__ uint32_t s_cnt[];                 // [2 * nbuckets + 1]
    __shared__ uint32_t s_wave[PREP_T / WAVE];
    const int tid = threadIdx.x;
    const int n = blockIdx.x;
    const int nbuckets = H * cb_count;
    uint32_t *s_fill = s_cnt + nbuckets + 1;
    const int64_t plane = int64_t(H) * W;
    const int64_t img_first = int64_t(n) * C * plane;
    const int64_t img_elems = int64_t(C) * plane;
    const int64_t lo = block_lower_bound_1024(idx, k, img_first);
    const int64_t hi = block_lower_bound_1024(idx, k, img_first + img_elems);
    for (int i = tid; i < 2 * nbuckets + 1; i += PREP_T) s_cnt[i] = 0;
    __syncthreads();
    for (int64_t j = lo + tid; j < hi; j += PREP_T) {
        const int64_t r = int64_t(idx[j]) - img_first;
        if (r >= 0 && r < img_elems) {
            const uint32_t c = uint32_t(r) / uint32_t(plane);
            const uint32_t h = (uint32_t(r) - c * uint32_t(plane)) / uint32_t(W);
            atomicAdd(&s_cnt[h * cb_count + c / BC], 1u);
        }
    }
    __syncthreads();
    uint32_t carry = 0;
    for (int base = 0; base < nbuckets; base += PREP_T) {
        const int b = base + tid;
        const uint32_t c = (b < nbuckets) ? s_cnt[b] : 0u;
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<PREP_T>(c, s_wave, total);
        if (b < nbuckets) s_cnt[b] = carry + ex;
        carry += total;
        __syncthreads();
    }
    if (tid == 0) s_cnt[nbuckets] = carry;
    __syncthreads();
    uint32_t *rp = row_ptr + int64_t(n) * (nbuckets + 1);
    for (int b = tid; b <= nbuckets; b += PREP_T) rp[b] = uint32_t(lo) + s_cnt[b];
    for (int64_t j = lo + tid; j < hi; j += PREP_T) {
        const int64_t r = int64_t(idx[j]) - img_first;
        if (r >= 0 && r < img_elems) {
            const uint32_t c = uint32_t(r) / uint32_t(plane);
            const uint32_t rem = uint32_t(r) - c * uint32_t(plane);
            const uint32_t h = rem / uint32_t(W);
            const uint32_t w = rem - h * uint32_t(W);
            const uint32_t b = h * cb_count + c / BC;
            const uint32_t slot = atomicAdd(&s_fill[b], 1u);
            packed[lo + s_cnt[b] + slot] = (uint32_t(vals[j]) << 16) | ((c % BC) << 7) | w;
        }
    }
}

// GEMM: workgroup = (image n, band of RB output rows, 64 x 64 block of (j, c)).
__global__ void __launch_bounds__(CT)
conv3x3_mfma_kernel(const uint16_t *__restrict__ dY, const uint32_t *__restrict__ packed,
                    const uint32_t *__restrict__ row_ptr, int C, int H, int W, int J, int RB, int bands,
                    int cb_count, int jb_count, int pitch_c /*bytes per (row, channel)*/,
                    float *__restrict__ partial /*[N*bands][9][J][C]*/)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wj = wave >> 1, wc = wave & 1;
    int v = blockIdx.x;
    const int cb = v % cb_count; v /= cb_count;
    const int jb = v % jb_count; v /= jb_count;
    const int band = v % bands;
    const int n = v / bands;
    const int r0 = band * RB;
    const int rows = min(RB, H - r0);                  // output rows of this band
    const int slots = rows + 2;                        // input rows r0-1 .. r0+rows
    const int slot_bytes = BC * pitch_c;

    // ---- recover R(a^) for this band into LDS: zero fill, then scatter ------------
    {
        const int n16 = slots * slot_bytes / 16;
        for (int i = tid; i < n16; i += CT) reinterpret_cast<u32x4 *>(lds)[i] = u32x4{0, 0, 0, 0};
    }
    __syncthreads();
    const uint32_t *rp = row_ptr + int64_t(n) * (H * cb_count + 1);
    for (int s = 0; s < slots; ++s) {
        const int ih = r0 - 1 + s;
        if (ih < 0 || ih >= H) continue;               // vertical zero padding
        const uint32_t lo = rp[ih * cb_count + cb], hi = rp[ih * cb_count + cb + 1];
        char *row = lds + s * slot_bytes + 16;
        for (uint32_t j = lo + tid; j < hi; j += CT) {
            const uint32_t p = packed[j];
            *reinterpret_cast<uint16_t *>(row + ((p >> 7) & 0x3Fu) * pitch_c + (p & 0x7Fu) * 2) = uint16_t(p >> 16);
        }
    }
    __syncthreads();

    // ---- multiply ---------------------------------------------------------------
    f32x16 acc[9];
#pragma unroll
    for (int i = 0; i < 9; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

    const int kg = lane >> 5;                          // K-half: which row of the pair
    const int j = jb * BJ + wj * 32 + (lane & 31);
    const int cl = wc * 32 + (lane & 31);
    const int groups = W / 8;
    const int jc = min(j, J - 1);
    for (int pr = 0; pr < rows; pr += 2) {
        const int oy_l = pr + kg;                      // row inside the band
        const bool a_ok = (j < J) && (oy_l < rows);
        const int oy = r0 + min(oy_l, rows - 1);
        const uint16_t *arow = dY + ((int64_t(n) * J + jc) * H + oy) * W;
        // slot of input row oy-1 (tap u = 0); a K-half past the band reads valid rows and multiplies by zero
        const char *brow = lds + min(oy_l, rows - 1) * slot_bytes + cl * pitch_c + 16;
        for (int t = 0; t < groups; ++t) {
            u32x4 a4 = *reinterpret_cast<const u32x4 *>(arow + t * 8);
            if (!a_ok) a4 = u32x4{0, 0, 0, 0};
            const bf16x8 a = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const char *p = brow + u * slot_bytes + t * 16;
                const u32x4 ctr = *reinterpret_cast<const u32x4 *>(p);
                const uint32_t left = *reinterpret_cast<const uint32_t *>(p - 4);
                const uint32_t right = *reinterpret_cast<const uint32_t *>(p + 16);
                const uint32_t f0 = __builtin_amdgcn_alignbyte(ctr[0], left, 2);
                const uint32_t f1 = __builtin_amdgcn_alignbyte(ctr[1], ctr[0], 2);
                const uint32_t f2 = __builtin_amdgcn_alignbyte(ctr[2], ctr[1], 2);
                const uint32_t f3 = __builtin_amdgcn_alignbyte(ctr[3], ctr[2], 2);
                const uint32_t f4 = __builtin_amdgcn_alignbyte(right, ctr[3], 2);
                const bf16x8 b0 = __builtin_bit_cast(bf16x8, (u32x4{f0, f1, f2, f3}));   // ox - 1
                const bf16x8 b1 = __builtin_bit_cast(bf16x8, ctr);                        // ox
                const bf16x8 b2 = __builtin_bit_cast(bf16x8, (u32x4{f1, f2, f3, f4}));   // ox + 1
                acc[u * 3 + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b0, acc[u * 3 + 0], 0, 0, 0);
                acc[u * 3 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b1, acc[u * 3 + 1], 0, 0, 0);
                acc[u * 3 + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b2, acc[u * 3 + 2], 0, 0, 0);
            }
        }
    }

    // ---- partial sums: [workgroup][tap][j][c] ------------------------------------
    float *dst = partial + (int64_t(n) * bands + band) * 9 * int64_t(J) * C;
#pragma unroll
    for (int s = 0; s < 9; ++s)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int jj = jb * BJ + wj * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
            const int cc = cb * BC + wc * 32 + (lane & 31);
            if (jj < J && cc < C) dst[(int64_t(s) * J + jj) * C + cc] = acc[s][e];
        }
}

// dW[j][c][tap] = sum over workgroups (ascending) of partial[p][tap][j][c]
__global__ void __launch_bounds__(256)
conv_reduce_kernel(const float *__restrict__ partial, int parts, int J, int C, float *__restrict__ dW)
{
    const int64_t jc = int64_t(J) * C;
    const int64_t total = jc * 9;
    for (int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; i < total; i += int64_t(gridDim.x) * blockDim.x) {
        float s = 0.f;
        for (int p = 0; p < parts; ++p) s += partial[int64_t(p) * total + i];
        const int64_t tap = i / jc, rem = i - tap * jc;             // i = (tap, j, c)
        dW[rem * 9 + tap] = s;
    }
}

}  // namespace

bool conv_mfma_supported(const ConvProblem &p)
{
    if (p.W % 8 != 0 || p.W > 120 || p.H < 1) return false;
    const ConvPlan plan = conv_mfma_plan(p);
    return plan.lds_bytes <= 160 * 1024 && int64_t(p.H) * plan.cb_count <= 8192 &&
           int64_t(p.N) * plan.bands * plan.cb_count * plan.jb_count <= INT32_MAX;
}

ConvPlan conv_mfma_plan(const ConvProblem &p)
{
    ConvPlan plan;
    plan.cb_count = int((p.C + BC - 1) / BC);
    plan.jb_count = int((p.J + BJ - 1) / BJ);
    plan.pitch_c = int(p.W + 16) * 2;
    if ((plan.pitch_c / 16) % 2 == 0) plan.pitch_c += 16;            // odd multiple of 16: conflict-free row reads
    // bands: enough workgroups for the 256 compute units, bounded by the LDS a band's rows need
    const int64_t per_band_wgs = p.N * plan.cb_count * plan.jb_count;
    int bands = int((256 + per_band_wgs - 1) / per_band_wgs);
    if (bands < 1) bands = 1;
    if (bands > p.H) bands = int(p.H);
    int rb = int((p.H + bands - 1) / bands);
    rb = (rb + 1) / 2 * 2;                                            // whole row pairs
    const int max_rb = (150 * 1024 / (BC * plan.pitch_c) - 2) / 2 * 2;
    if (rb > max_rb) rb = max_rb;
    if (rb < 2) rb = 2;
    plan.rb = rb;
    plan.bands = int((p.H + rb - 1) / rb);
    plan.lds_bytes = size_t(rb + 2) * BC * plan.pitch_c;
    plan.packed_bytes = round_up(size_t(p.k > 0 ? p.k : 1) * 4, 256);
    plan.rowptr_bytes = round_up(size_t(p.N) * (p.H * plan.cb_count + 1) * 4, 256);
    plan.partial_bytes = round_up(size_t(p.N) * plan.bands * 9 * p.J * p.C * 4, 256);
    return plan;
}

dropit_status conv_mfma_run(const ConvProblem &p, const ConvPlan &plan, const void *vals, const int32_t *idx,
                            const void *dY, float *dW, char *ws, hipStream_t stream)
{
    uint32_t *packed = reinterpret_cast<uint32_t *>(ws);
    uint32_t *row_ptr = reinterpret_cast<uint32_t *>(ws + plan.packed_bytes);
    float *partial = reinterpret_cast<float *>(ws + plan.packed_bytes + plan.rowptr_bytes);

    trace_mark(stream);
    const size_t bucket_lds = size_t(2 * p.H * plan.cb_count + 1) * 4;
    conv_bucket_kernel<<<int(p.N), PREP_T, bucket_lds, stream>>>(static_cast<const uint16_t *>(vals), idx, p.k,
                                                                 int(p.C), int(p.H), int(p.W), plan.cb_count, packed,
                                                                 row_ptr);
    trace_mark(stream);
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(conv3x3_mfma_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return DROPIT_EHIP;
        attr_set = true;
    }
    const int grid = int(p.N) * plan.bands * plan.jb_count * plan.cb_count;
    conv3x3_mfma_kernel<<<grid, CT, plan.lds_bytes, stream>>>(static_cast<const uint16_t *>(dY), packed, row_ptr,
                                                              int(p.C), int(p.H), int(p.W), int(p.J), plan.rb,
                                                              plan.bands, plan.cb_count, plan.jb_count, plan.pitch_c,
                                                              partial);
    trace_mark(stream);
    const int64_t total = p.J * p.C * 9;
    const int blocks = int(std::min<int64_t>((total + 255) / 256, 2048));
    conv_reduce_kernel<<<blocks, 256, 0, stream>>>(partial, int(p.N) * plan.bands, int(p.J), int(p.C), dW);
    trace_mark(stream);
    return launch_status();
}

}  // namespace dropit
