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
//   B (a^)  : the index-sorted (value, index) pairs of an NCHW tensor already are a CSR
//             matrix over its (image, channel, row) rows; a prep kernel only marks where
//             each row starts.  The GEMM workgroup owns one image and a band of output
//             rows, zero-fills LDS rows [channel][8 | W | 8] (zero pads left and right =
//             the horizontal padding; rows outside the image stay zero = the vertical
//             padding) and scatters the pairs of its 64 channels (one contiguous run of
//             the arrays per channel) with one 16-bit store each.  A fragment for tap (u, v) is row oy+u-1 read at
//             ox+v-1: one aligned 16-byte read plus its two neighbouring dwords,
//             funnel-shifted by one element in registers for v = 0 and v = 2.
// One K step = 8 consecutive ox of TWO adjacent output rows (the two K-halves of the
// MFMA), so any even or odd H works; a W that is not a multiple of 8 goes through a zero-padded copy of dY.
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

constexpr int CT = 512;            // threads per GEMM workgroup: 2 K-groups x (2 j-halves x 2 c-halves) wavefronts
constexpr int BJ = 64, BC = 64;    // output-channel / input-channel block of a workgroup

// Prep (row_starts_kernel): row_ptr[r] = number of pairs whose flat index lies before row r, for every
// row r = (n * C + c) * H + h of W elements (row_ptr[R] = k).

// GEMM: workgroup = (image n, band of RB output rows, 64 x 64 block of (j, c)).
// AG = column groups (of 8) multiplied per step; the host picks the instantiation that wastes the
// fewest padded groups for the row width at hand.
template <int AG, bool MULTI>
__global__ void __launch_bounds__(CT)
conv3x3_mfma_kernel(const uint16_t *__restrict__ dY, const uint16_t *__restrict__ vals,
                    const int32_t *__restrict__ idx, int64_t k, const uint32_t *__restrict__ row_ptr, int C, int H,
                    int W, int Wp /*row width of dY as passed: W rounded up to a multiple of 8*/, int J, int RB, int bands,
                    int cb_count, int jb_count, int pitch_c /*bytes per (row, channel)*/, int N, int imgs_per_wg,
                    float *__restrict__ partial /*[image groups * bands][9][J][C]*/)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave >> 2;                          // K-group: takes every other step of the band
    const int wj = (wave >> 1) & 1, wc = wave & 1;
    int v = blockIdx.x;
    const int cb = v % cb_count; v /= cb_count;
    const int jb = v % jb_count; v /= jb_count;
    const int band = v % bands;
    const int ng = v / bands;                          // image group: images ng * imgs_per_wg ...
    const int n_begin = ng * imgs_per_wg, n_end = min(n_begin + imgs_per_wg, N);
    const int r0 = band * RB;
    const int rows = min(RB, H - r0);                  // output rows of this band
    const int slots = rows + 2;                        // input rows r0-1 .. r0+rows
    const int slot_bytes = BC * pitch_c;

    // With several images per workgroup (MULTI) the accumulators live across the images; with one they
    // start after the scatter, which leaves the scatter the registers to keep two batches of loads in flight.
    f32x16 acc[9];
    if constexpr (MULTI) {
#pragma unroll
        for (int i = 0; i < 9; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    }

    for (int n = n_begin; n < (MULTI ? n_end : n_begin + 1); ++n) {
    if (n != n_begin) __syncthreads();             // the previous image's rows have been read by every wavefront
    // ---- recover R(a^) for this band into LDS: zero fill, then scatter ------------
    // Pairs of this band: for each of the 64 channels one contiguous run [first, last) of the arrays
    // (input rows ih_lo .. ih_hi of that channel).  The runs are laid end to end (prefix sums of
    // their lengths in LDS) and the threads stride over that flat range, so every thread has
    // work and the loads of a run are coalesced.  The run bounds are fetched before the zero fill,
    // which hides their latency.
    __shared__ uint32_t s_first[BC], s_last[BC];
    const int ih_lo = max(r0 - 1, 0), ih_hi = min(r0 + rows, H - 1);
    uint32_t first = 0, last = 0;
    if (tid < BC && cb * BC + tid < C) {
        const int64_t row0 = (int64_t(n) * C + cb * BC + tid) * H;
        first = row_ptr[row0 + ih_lo];
        last = row_ptr[row0 + ih_hi + 1];
    }
    {
        const int n16 = slots * slot_bytes / 16;
        for (int i = tid; i < n16; i += CT) reinterpret_cast<u32x4 *>(lds)[i] = u32x4{0, 0, 0, 0};
    }
    if (tid < BC) {
        first = min<uint32_t>(first, uint32_t(k));      // clamped: a malformed index array may
        last = min<uint32_t>(last, uint32_t(k));        // leave row starts unwritten
        s_first[tid] = first;
        s_last[tid] = max(last, first);
    }
    __syncthreads();
    // Each wavefront takes 8 of the 64 channels, SC at a time: the runs of SC channels are walked
    // together so that SC x 2 loads per lane are in flight, and everything per channel (run bounds,
    // plane offset, LDS row base) is wave-uniform scalar work.  Row and column of a pair come from
    // its offset in the channel plane by a multiply-high with ceil(2^32 / W), exact here because
    // the offset is far below 2^32 / W, and checked anyway.
    constexpr int SC = 8;
    const uint32_t w_magic = uint32_t(((1ull << 32) + uint32_t(W) - 1) / uint32_t(W));
    const uint32_t plane = uint32_t(H) * uint32_t(W);
    for (int c0 = wave * (BC / 8); c0 < (wave + 1) * (BC / 8); c0 += SC) {
        uint32_t lo[SC], hi[SC], longest = 0;
#pragma unroll
        for (int q = 0; q < SC; ++q) {
            lo[q] = __builtin_amdgcn_readfirstlane(s_first[c0 + q]);
            hi[q] = __builtin_amdgcn_readfirstlane(s_last[c0 + q]);
            longest = max(longest, hi[q] - lo[q]);
        }
        // the loads of the next 64 positions are issued before the current ones are stored: one memory
        // round trip per channel batch instead of one per 64 positions
        int flat[SC], flat_next[SC];
        uint32_t val[SC], val_next[SC];     // full registers: 16-bit destinations get packed in pairs and their loads serialised
        auto fetch_pairs = [&](uint32_t off, int (&f)[SC], uint32_t (&v)[SC]) {
#pragma unroll
            for (int q = 0; q < SC; ++q) {
                const uint32_t at = min(lo[q] + off, uint32_t(k) - 1);   // unconditional, clamped (k > 0)
                f[q] = idx[at];
                v[q] = vals[at];
            }
        };
        // (not with several images per workgroup: their accumulators leave no registers for a second batch)
        if (!MULTI && lane < longest) fetch_pairs(lane, flat, val);
        for (uint32_t off = lane; off < longest; off += WAVE) {
            const bool more = !MULTI && off + WAVE < longest;
            if (MULTI) fetch_pairs(off, flat, val);
            if (more) fetch_pairs(off + WAVE, flat_next, val_next);
#pragma unroll
            for (int q = 0; q < SC; ++q) {
                if (lo[q] + off >= hi[q]) continue;
                const int64_t base = (int64_t(n) * C + cb * BC + c0 + q) * int64_t(plane);   // scalar
                const int64_t rel64 = int64_t(flat[q]) - base;                              // offset inside the channel plane
                if (rel64 < 0 || rel64 >= int64_t(plane)) continue;   // never for a sorted, in-range index array
                const uint32_t rel = uint32_t(rel64);
                uint32_t ih = __umulhi(rel, w_magic);
                if (ih * uint32_t(W) > rel) --ih;
                const uint32_t w = rel - ih * uint32_t(W);
                if (int(ih) >= ih_lo && int(ih) <= ih_hi && w < uint32_t(W))
                    *reinterpret_cast<uint16_t *>(lds + (int(ih) - (r0 - 1)) * slot_bytes + 16 + (c0 + q) * pitch_c + w * 2) = uint16_t(val[q]);
            }
            if (more) {
#pragma unroll
                for (int q = 0; q < SC; ++q) {
                    flat[q] = flat_next[q];
                    val[q] = val_next[q];
                }
            }
        }
    }
    __syncthreads();

    // ---- multiply ---------------------------------------------------------------
    if constexpr (!MULTI) {
#pragma unroll
        for (int i = 0; i < 9; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    }
    const int kg = lane >> 5;                          // K-half: which row of the pair
    const int j = jb * BJ + wj * 32 + (lane & 31);
    const int cl_b = wc * 32 + (lane & 31);            // this lane's input channel inside the block
    const int groups = Wp / 8;
    const int jc = min(j, J - 1);
    // The dY fragments come straight from global memory; they are fetched one chunk (a row pair x
    // AG groups of 8 columns) ahead of the chunk being multiplied, all loads of a chunk in flight
    // at once, so their latency hides behind a chunk's worth of MFMAs.  A chunk's body is
    // branch-free (groups past the row get a zero dY fragment and a clamped LDS address), so
    // the compiler can run its LDS reads ahead of the MFMAs across the whole chunk.
    const int chunks = (groups + AG - 1) / AG;          // per row pair
    const int n_steps = ((rows + 1) / 2) * chunks;
    auto fetch = [&](u32x4 (&a)[AG], int step) {
        const int pr = (step / chunks) * 2, t0 = (step % chunks) * AG;
        const int oy_l = pr + kg;                      // row inside the band
        const bool a_ok = (j < J) && (oy_l < rows);
        const int oy = r0 + min(oy_l, rows - 1);
        const uint16_t *arow = dY + ((int64_t(n) * J + jc) * H + oy) * Wp;
#pragma unroll
        for (int g = 0; g < AG; ++g) {
            const u32x4 v4 = *reinterpret_cast<const u32x4 *>(arow + min(t0 + g, groups - 1) * 8);   // clamped, unconditional
            a[g] = (a_ok && t0 + g < groups) ? v4 : u32x4{0, 0, 0, 0};
        }
    };
    // the two K-groups of wavefronts take alternate steps; their sums meet in LDS at the end
    u32x4 cur[AG], nxt[AG];
    fetch(cur, min(wk, n_steps - 1));
    for (int step = wk; step < n_steps; step += 2) {
        fetch(nxt, min(step + 2, n_steps - 1));
        const int pr = (step / chunks) * 2, t0 = (step % chunks) * AG;
        const int oy_l = pr + kg;
        // slot of input row oy-1 (tap u = 0); a K-half past the band reads valid rows and multiplies by zero
        const char *brow = lds + min(oy_l, rows - 1) * slot_bytes + cl_b * pitch_c + 16;
#pragma unroll
        for (int g = 0; g < AG; ++g) {
            const int t = min(t0 + g, groups - 1);     // past the row: any valid address, the dY fragment is zero
            const bf16x8 a = __builtin_bit_cast(bf16x8, cur[g]);
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
#pragma unroll
        for (int g = 0; g < AG; ++g) cur[g] = nxt[g];
    }

    }   // images of the group

    // ---- the two K-groups meet: group 1 parks its sums in LDS (the rows are no longer needed: 4 wavefronts x
    // 9 tiles x 4 KB = exactly the 144 KB the accumulators take), group 0 adds them and writes -----------
    __syncthreads();                                   // every wavefront is done reading the rows
    float *park = reinterpret_cast<float *>(lds) + (wave & 3) * (9 * 16 * WAVE);
    if (wk == 1) {
#pragma unroll
        for (int s = 0; s < 9; ++s)
#pragma unroll
            for (int e = 0; e < 16; ++e) park[(s * 16 + e) * WAVE + lane] = acc[s][e];
    }
    __syncthreads();
    if (wk == 0) {
        // partial sums: [workgroup][tap][j][c]
        float *dst = partial + (int64_t(ng) * bands + band) * 9 * int64_t(J) * C;
#pragma unroll
        for (int s = 0; s < 9; ++s)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int jj = jb * BJ + wj * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                const int cc = cb * BC + wc * 32 + (lane & 31);
                if (jj < J && cc < C) dst[(int64_t(s) * J + jj) * C + cc] = acc[s][e] + park[(s * 16 + e) * WAVE + lane];
            }
    }
}

// Rows of a width that is not a multiple of 8 (28, 14, 7 in the later stages of a ResNet): dY is copied
// once into rows of Wp = W rounded up, zero beyond W, so that the kernel's 16-byte fragment loads stay
// aligned; the added columns multiply zeros (the LDS rows of the recovered input are zero there too).
// One thread per group of 8 output columns.
__global__ void __launch_bounds__(256)
conv_pad_rows_kernel(const uint16_t *__restrict__ dY, int64_t rows, int W, int Wp, uint16_t *__restrict__ out)
{
    const int gpr = Wp / 8;                             // groups per row
    const int64_t total = rows * gpr;
    for (int64_t g = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; g < total; g += int64_t(gridDim.x) * blockDim.x) {
        const int64_t r = g / gpr;
        const int w0 = int(g - r * gpr) * 8;
        uint32_t e[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) e[i] = (w0 + i < W) ? uint32_t(dY[r * W + w0 + i]) : 0u;
        *reinterpret_cast<u32x4 *>(out + r * Wp + w0) =
            u32x4{e[0] | e[1] << 16, e[2] | e[3] << 16, e[4] | e[5] << 16, e[6] | e[7] << 16};
    }
}

// dW[j][c][tap] = sum over the GEMM workgroups' partials partial[p][tap][j][c], in a fixed order:
// a workgroup takes 64 consecutive (tap, j, c) outputs; each of its (up to 16) wavefronts adds its share
// of the parts in ascending order (enough loads in flight to cover the memory latency), then the
// first wavefront adds the wavefronts' sums in ascending order.
// VEC = 4 (taken when J * C is a multiple of 4): a thread sums four consecutive outputs with 16-byte loads.
constexpr int RED_GROUPS = 16;
template <int VEC>
__global__ void __launch_bounds__(64 * RED_GROUPS)
conv_reduce_kernel(const float *__restrict__ partial, int parts, int J, int C, float *__restrict__ dW)
{
    typedef float vec_t __attribute__((ext_vector_type(VEC == 1 ? 2 : VEC)));   // (a 1-vector is not indexable: lane 0 of a pair)
    __shared__ vec_t s_sum[RED_GROUPS][64];
    const int groups = blockDim.x / 64;                 // wavefronts of this launch (a power of two up to 16)
    const int64_t jc = int64_t(J) * C;
    const int64_t total = jc * 9;
    const int o = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int64_t i = (int64_t(blockIdx.x) * 64 + o) * VEC;              // first of this thread's outputs
    vec_t s = 0.f;
    if (i < total) {
        const int per = (parts + groups - 1) / groups;
        const int p0 = grp * per, p1 = min(p0 + per, parts);
#pragma unroll 8
        for (int p = p0; p < p1; ++p) {
            if constexpr (VEC == 1) s[0] += partial[int64_t(p) * total + i];
            else s += *reinterpret_cast<const vec_t *>(partial + int64_t(p) * total + i);
        }
    }
    s_sum[grp][o] = s;
    __syncthreads();
    if (grp == 0 && i < total) {
        vec_t t = s_sum[0][o];
        for (int g = 1; g < groups; ++g) t += s_sum[g][o];
        const int64_t tap = i / jc, rem = i - tap * jc;                 // i = (tap, j, c); the VEC outputs share tap and j
#pragma unroll
        for (int e = 0; e < VEC; ++e) dW[(rem + e) * 9 + tap] = t[e];
    }
}

}  // namespace

bool conv_mfma_supported(const ConvProblem &p)
{
    if (p.W < 2 || p.W > 120 || p.H < 1) return false;     // (the scatter divides by W with a 32-bit reciprocal: W >= 2)
    const ConvPlan plan = conv_mfma_plan(p);
    return plan.lds_bytes <= 150 * 1024 && p.N * p.C * p.H < INT32_MAX &&
           int64_t(plan.img_groups) * plan.bands * plan.cb_count * plan.jb_count <= INT32_MAX;
}

ConvPlan conv_mfma_plan(const ConvProblem &p)
{
    ConvPlan plan;
    plan.cb_count = int((p.C + BC - 1) / BC);
    plan.jb_count = int((p.J + BJ - 1) / BJ);
    plan.wp = int((p.W + 7) / 8 * 8);
    plan.pitch_c = (plan.wp + 16) * 2;
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
    // the rows of a band, and afterwards the parked accumulators of one K-group (4 x 9 x 16 x 64 floats)
    plan.lds_bytes = std::max(size_t(rb + 2) * BC * plan.pitch_c, size_t(4) * 9 * 16 * WAVE * 4);
    plan.rowptr_bytes = round_up(size_t(p.N * p.C * p.H + 1) * 4, 256);
    // A workgroup accumulates over several images when there are more (image, band, block) units than
    // compute units: the partial sums it writes are a whole 9 x 64 x 64 tile however much it summed.
    const int64_t units = p.N * plan.bands * plan.cb_count * plan.jb_count;
    plan.imgs_per_wg = int(std::min<int64_t>(std::max<int64_t>(units / 256, 1), p.N));
    plan.img_groups = int((p.N + plan.imgs_per_wg - 1) / plan.imgs_per_wg);
    plan.partial_bytes = round_up(size_t(plan.img_groups) * plan.bands * 9 * p.J * p.C * 4, 256);
    plan.dypad_bytes = plan.wp != p.W ? round_up(size_t(p.N) * p.J * p.H * plan.wp * 2, 256) : 0;
    return plan;
}

dropit_status conv_mfma_run(const ConvProblem &p, const ConvPlan &plan, const void *vals, const int32_t *idx,
                            const void *dY, float *dW, char *ws, hipStream_t stream)
{
    uint32_t *row_ptr = reinterpret_cast<uint32_t *>(ws);
    float *partial = reinterpret_cast<float *>(ws + plan.rowptr_bytes);

    trace_mark(stream);
    const int64_t R = p.N * p.C * p.H;
    launch_row_starts(idx, p.k, uint32_t(p.W), R, row_ptr, stream);
    trace_mark(stream);
    const uint16_t *dy_rows = static_cast<const uint16_t *>(dY);
    if (plan.wp != p.W) {
        uint16_t *padded = reinterpret_cast<uint16_t *>(ws + plan.rowptr_bytes + plan.partial_bytes);
        const int64_t rows = p.N * p.J * p.H;
        const int blocks = int(std::min<int64_t>((rows * (plan.wp / 8) + 255) / 256, 8192));
        conv_pad_rows_kernel<<<blocks, 256, 0, stream>>>(dy_rows, rows, int(p.W), plan.wp, padded);
        dy_rows = padded;
        trace_mark(stream);
    }
    // groups of 8 columns per row: take the chunk width (8, 7, 6 or 5) that pads the row least
    const int groups = plan.wp / 8;
    int ag = 8, padded = (groups + 7) / 8 * 8;
    for (int cand = 7; cand >= 5; --cand) {
        const int pc = (groups + cand - 1) / cand * cand;
        if (pc < padded) {
            ag = cand;
            padded = pc;
        }
    }
    const int grid = plan.img_groups * plan.bands * plan.jb_count * plan.cb_count;
    auto launch = [&](auto kernel) -> dropit_status {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                150 * 1024) != hipSuccess)
            return DROPIT_EHIP;
        kernel<<<grid, CT, plan.lds_bytes, stream>>>(dy_rows, static_cast<const uint16_t *>(vals),
                                                     idx, p.k, row_ptr, int(p.C), int(p.H), int(p.W), plan.wp, int(p.J), plan.rb,
                                                     plan.bands, plan.cb_count, plan.jb_count, plan.pitch_c, int(p.N),
                                                     plan.imgs_per_wg, partial);
        return DROPIT_OK;
    };
    dropit_status st = DROPIT_OK;
    const bool multi = plan.imgs_per_wg > 1;
    switch (ag) {
    case 5: st = multi ? launch(conv3x3_mfma_kernel<5, true>) : launch(conv3x3_mfma_kernel<5, false>); break;
    case 6: st = multi ? launch(conv3x3_mfma_kernel<6, true>) : launch(conv3x3_mfma_kernel<6, false>); break;
    case 7: st = multi ? launch(conv3x3_mfma_kernel<7, true>) : launch(conv3x3_mfma_kernel<7, false>); break;
    default: st = multi ? launch(conv3x3_mfma_kernel<8, true>) : launch(conv3x3_mfma_kernel<8, false>); break;
    }
    if (st != DROPIT_OK) return st;
    trace_mark(stream);
    const int64_t total = p.J * p.C * 9;
    // wavefronts per 64 (x4) outputs: enough that a thread has about four loads in flight, at most 16
    const int parts = plan.img_groups * plan.bands;
    int red_groups = 1;
    while (red_groups * 8 <= parts && red_groups < RED_GROUPS) red_groups *= 2;
    if ((p.J * p.C) % 4 == 0)
        conv_reduce_kernel<4><<<int((total / 4 + 63) / 64), 64 * red_groups, 0, stream>>>(partial, parts, int(p.J), int(p.C), dW);
    else
        conv_reduce_kernel<1><<<int((total + 63) / 64), 64 * red_groups, 0, stream>>>(partial, parts, int(p.J), int(p.C), dW);
    trace_mark(stream);
    return launch_status();
}

}  // namespace dropit
