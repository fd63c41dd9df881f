// Convolution weight gradient of ANY 2-d geometry (kernel extent, stride, padding, dilation) and
// either memory layout as one dense GEMM over explicit im2col rows, bf16 on the matrix cores.
//
// Sec. 3.2 (convolution weight gradient):
//   dW[j][c][u][v] = sum_{n,oy,ox} dY[n][j][oy][ox] * R(a^)[n][c][oy*sh - ph + u*dh][ox*sw - pw + v*dw].
// With one "token" t per output position (n, oy, ox) this is dW[j][col] = sum_t dYt[t][j] * B[t][col],
// the fully-connected form of the same section, where row t of B holds the kh*kw*C input elements
// under the window of t (zero where the window hangs over the padding or the element was dropped).
//
//   NCHW: x [N][C][H][W], dY [N][J][OH][OW];  col = (c*kh + u)*kw + v   ->  dW [J][C][kh][kw]
//   NHWC: x [N][H][W][C], dY [N][OH][OW][J];  col = (u*kw + v)*C + c    ->  dW [J][kh][kw][C]
//
// B is written straight from the (value, index) pairs: a retained element lands in every
// (token, tap) whose window covers it, at most ceil(kh/sh) * ceil(kw/sw) places.  Normally B is
// assembled in LDS tiles and written once in full lines (im2col_tiled_kernel); where no aligned
// tiling exists it is zero-filled and scattered into (im2col_scatter_kernel).
// In NHWC dY is token-major already; in NCHW a tiled transposition makes it so.  The 3x3 / stride 1
// / pad 1 NCHW case has kernels of its own (wgrad_conv_mfma.hip, wgrad_conv_gemm.hip) that never
// materialise the nine-fold B; this path serves everything else: 1x1, strided, dilated, large-window
// (patch embedding) convolutions, and channels-last tensors.
#include "wgrad_internal.hpp"
#include "dev_hooks.hpp"
#include <cstdlib>

namespace dropit {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256) fill_zero16_kernel(u32x4 *__restrict__ p, int64_t chunks)
{
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < chunks; i += stride) p[i] = u32x4{0u, 0u, 0u, 0u};
}

struct Geometry {
    int C, H, W, OH, OW, kh, kw, sh, sw, ph, pw, dh, dw;
};

// One thread per pair.  Input row ih is under tap row u of output row oy iff oy*sh - ph + u*dh == ih.
template <bool NHWC>
__global__ void __launch_bounds__(256)
im2col_scatter_kernel(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx, int64_t k, int64_t numel,
                      Geometry g, int pitch, uint16_t *__restrict__ B)
{
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t j = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; j < k; j += stride) {
        const uint32_t flat = uint32_t(idx[j]);
        if (int64_t(flat) >= numel) continue;                   // a malformed index must not write outside B
        const uint32_t val = vals[j];
        uint32_t n, c, ih, iw;
        if (NHWC) {
            uint32_t t = flat / uint32_t(g.C);
            c = flat - t * uint32_t(g.C);
            const uint32_t t2 = t / uint32_t(g.W);
            iw = t - t2 * uint32_t(g.W);
            n = t2 / uint32_t(g.H);
            ih = t2 - n * uint32_t(g.H);
        } else {
            uint32_t t = flat / uint32_t(g.W);
            iw = flat - t * uint32_t(g.W);
            const uint32_t t2 = t / uint32_t(g.H);
            ih = t - t2 * uint32_t(g.H);
            n = t2 / uint32_t(g.C);
            c = t2 - n * uint32_t(g.C);
        }
        for (int u = 0; u < g.kh; ++u) {
            const int num_y = int(ih) + g.ph - u * g.dh;
            if (num_y < 0) break;                               // larger u only lowers it further
            const int oy = num_y / g.sh;
            if (oy * g.sh != num_y || oy >= g.OH) continue;
            for (int v = 0; v < g.kw; ++v) {
                const int num_x = int(iw) + g.pw - v * g.dw;
                if (num_x < 0) break;
                const int ox = num_x / g.sw;
                if (ox * g.sw != num_x || ox >= g.OW) continue;
                const int64_t t = (int64_t(n) * g.OH + oy) * g.OW + ox;
                const int col = NHWC ? (u * g.kw + v) * g.C + int(c) : (int(c) * g.kh + u) * g.kw + v;
                B[t * pitch + col] = uint16_t(val);
            }
        }
    }
}

// The im2col rows assembled in LDS tiles and written once, in full lines, with no zero-fill pass.
// Workgroup = (image n, column block, band of RB output rows).  A column block is a block of input
// channels in NCHW (columns (c, u, v)) and a block of taps in NHWC (columns (u, v, c)), so that its
// columns are one contiguous, 16-byte aligned segment of every token's row.  The input rows under
// the band are contiguous in the index-sorted pair arrays (per channel in NCHW, all channels at once
// in NHWC); row_ptr says where they start.  Every retained element is placed into the (token, tap)
// cells of the tile whose window covers it; the output rows it can belong to follow from its input
// row without trying every tap:  oy * sh = ih + ph - u * dh  for some tap row u in [0, kh).
#ifndef DROPIT_IM2COL_BATCH
#define DROPIT_IM2COL_BATCH 8
#endif
struct TileShape {
    int nblocks, blk, bands, rb, rowlen;      // column blocks, their width (channels or taps), bands, rows per band, tile row length
    int tmin;                                 // NCHW: at least this many threads share a channel's run (a power of two)
};

template <bool NHWC>
__global__ void __launch_bounds__(256)
im2col_tiled_kernel(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx,
                    const uint32_t *__restrict__ row_ptr, int N, Geometry g, TileShape ts, int pitch, int64_t ntok,
                    int64_t ntok_pad, int pad_wgs, uint16_t *__restrict__ B)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t tile[];      // [rb * OW][rowlen]
    const int tid = threadIdx.x;
    const int64_t units = int64_t(N) * ts.nblocks * ts.bands;
    if (int64_t(blockIdx.x) >= units) {                                    // zero rows after the last token
        const int64_t chunks = (ntok_pad - ntok) * pitch / 8;
        u32x4 *dst = reinterpret_cast<u32x4 *>(B + ntok * pitch);
        for (int64_t i = (int64_t(blockIdx.x) - units) * 256 + tid; i < chunks; i += int64_t(pad_wgs) * 256)
            dst[i] = u32x4{0u, 0u, 0u, 0u};
        return;
    }
    const int band = blockIdx.x % ts.bands;
    const int blk = (blockIdx.x / ts.bands) % ts.nblocks;
    const int n = int(blockIdx.x / (int64_t(ts.bands) * ts.nblocks));
    const int oy0 = band * ts.rb, rb = min(ts.rb, g.OH - oy0);
    const int taps = g.kh * g.kw;
    const int b0 = blk * ts.blk;                                           // first channel (NCHW) or tap (NHWC) of the block
    const int bw = min(ts.blk, (NHWC ? taps : g.C) - b0);
    const int rowlen = ts.rowlen;
    const int chunks = rb * g.OW * (rowlen / 8);
    u32x4 *tile16 = reinterpret_cast<u32x4 *>(tile);
    for (int i = tid; i < chunks; i += 256) tile16[i] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    // input rows under the band
    const int ih_lo = max(0, oy0 * g.sh - g.ph);
    const int ih_hi = min(g.H - 1, (oy0 + rb - 1) * g.sh - g.ph + (g.kh - 1) * g.dh);

    // place the element at (c, ih, iw) into every cell of the tile it belongs to
    auto place = [&](int c, int ih, int iw, uint32_t v16) {
        const int y_top = ih + g.ph, x_top = iw + g.pw;                    // oy * sh + u * dh, ox * sw + v * dw
        const int y_bot = max(y_top - (g.kh - 1) * g.dh, 0), x_bot = max(x_top - (g.kw - 1) * g.dw, 0);
        const int oy_hi = min(g.sh == 1 ? y_top : int(uint32_t(y_top) / uint32_t(g.sh)), oy0 + rb - 1);
        const int oy_lo = max(g.sh == 1 ? y_bot : int((uint32_t(y_bot) + uint32_t(g.sh) - 1) / uint32_t(g.sh)), oy0);
        const int ox_hi = min(g.sw == 1 ? x_top : int(uint32_t(x_top) / uint32_t(g.sw)), g.OW - 1);
        const int ox_lo = g.sw == 1 ? x_bot : int((uint32_t(x_bot) + uint32_t(g.sw) - 1) / uint32_t(g.sw));
        for (int oy = oy_lo; oy <= oy_hi; ++oy) {
            const int ny = y_top - oy * g.sh;
            int u = ny;
            if (g.dh != 1) {
                u = int(uint32_t(ny) / uint32_t(g.dh));
                if (u * g.dh != ny) continue;
            }
            for (int ox = ox_lo; ox <= ox_hi; ++ox) {
                const int nx = x_top - ox * g.sw;
                int v = nx;
                if (g.dw != 1) {
                    v = int(uint32_t(nx) / uint32_t(g.dw));
                    if (v * g.dw != nx) continue;
                }
                const int tap = u * g.kw + v;
                int col;
                if (NHWC) {
                    if (tap < b0 || tap >= b0 + bw) continue;
                    col = (tap - b0) * g.C + c;
                } else {
                    col = (c - b0) * taps + tap;
                }
                tile[((oy - oy0) * g.OW + ox) * rowlen + col] = uint16_t(v16);
            }
        }
    };
    // pairs [j0, j1) of one run, `step` threads sharing it starting at `first`: a batch of loads in flight per thread
    auto walk = [&](uint32_t j0, uint32_t j1, int first, int step, auto &&decode) {
        constexpr int BATCH = DROPIT_IM2COL_BATCH;
        for (uint32_t j = j0 + first; j < j1; j += BATCH * step) {
            uint32_t pi[BATCH], pv[BATCH];
#pragma unroll
            for (int q = 0; q < BATCH; ++q)
                if (j + q * step < j1) {
                    pi[q] = uint32_t(idx[j + q * step]);
                    pv[q] = vals[j + q * step];
                }
#pragma unroll
            for (int q = 0; q < BATCH; ++q)
                if (j + q * step < j1) decode(pi[q], pv[q]);
        }
    };
    if (NHWC && ts.nblocks > 1) {
        // Blocks of taps: a tap (u, v) takes, for output row oy, exactly the input row oy*sh - ph + u*dh,
        // which is one run of the pairs (all its columns and channels).  The (tap, output row) runs of the
        // tile are dealt to groups of threads, so all of them are read at the same time and no workgroup
        // reads rows its taps do not use.
        const int nruns = bw * rb;
        int rpow = 1;
        while (rpow < nruns && rpow < 256) rpow <<= 1;
        const int T = 256 / rpow;
        const int grp = tid / T, sub = tid - grp * T;
        const uint32_t row_elems = uint32_t(g.W * g.C);
        for (int r = grp; r < nruns; r += 256 / T) {
            const int tapi = r / rb, oyi = r - tapi * rb;
            const int tap = b0 + tapi, u = tap / g.kw, v = tap - u * g.kw;
            const int ih = (oy0 + oyi) * g.sh - g.ph + u * g.dh;
            if (ih < 0 || ih >= g.H) continue;
            const int64_t r0 = int64_t(n) * g.H + ih;
            const uint32_t base = uint32_t(r0) * row_elems;
            uint16_t *out_row = tile + oyi * g.OW * rowlen + tapi * g.C;
            walk(row_ptr[r0], row_ptr[r0 + 1], sub, T, [&](uint32_t flat, uint32_t v16) {
                const uint32_t rel = flat - base;
                if (rel >= row_elems) return;                              // unsorted input must not write outside the tile
                const uint32_t iw = rel / uint32_t(g.C), c = rel - iw * uint32_t(g.C);
                const int nx = int(iw) + g.pw - v * g.dw;
                if (nx < 0) return;
                const int ox = g.sw == 1 ? nx : int(uint32_t(nx) / uint32_t(g.sw));
                if (ox * g.sw != nx || ox >= g.OW) return;
                out_row[ox * rowlen + int(c)] = uint16_t(v16);
            });
        }
    } else if (ih_lo <= ih_hi) {
        if (NHWC) {
            const int64_t r0 = int64_t(n) * g.H + ih_lo;
            const uint32_t base = uint32_t(r0) * uint32_t(g.W * g.C);      // flat index of (n, ih_lo, 0, 0)
            const uint32_t span = uint32_t(ih_hi - ih_lo + 1) * uint32_t(g.W * g.C);
            walk(row_ptr[r0], row_ptr[r0 + (ih_hi - ih_lo + 1)], tid, 256, [&](uint32_t flat, uint32_t v16) {
                const uint32_t rel = flat - base;
                if (rel >= span) return;                                   // unsorted input must not write outside the tile
                const uint32_t t = rel / uint32_t(g.C), c = rel - t * uint32_t(g.C);
                const uint32_t ihr = t / uint32_t(g.W), iw = t - ihr * uint32_t(g.W);
                place(int(c), ih_lo + int(ihr), int(iw), v16);
            });
        } else {
            // Each channel's pairs are a run of their own.  The 256 threads are dealt to the channels of the
            // block in groups of T = 256 / (channels rounded up to a power of two), between ts.tmin and a
            // wavefront: a few channels with long runs get a wavefront each and are all read at the same
            // time; many channels with short runs are taken 256 / tmin at a time.
            int cpow = 1;
            while (cpow < bw && cpow < 256) cpow <<= 1;
            const int T = min(64, max(256 / cpow, ts.tmin));
            const int grp = tid / T, sub = tid - grp * T;
            for (int c = b0 + grp; c < b0 + bw; c += 256 / T) {
                const int64_t r0 = (int64_t(n) * g.C + c) * g.H + ih_lo;
                const uint32_t base = uint32_t(r0) * uint32_t(g.W);
                const uint32_t span = uint32_t(ih_hi - ih_lo + 1) * uint32_t(g.W);
                walk(row_ptr[r0], row_ptr[r0 + (ih_hi - ih_lo + 1)], sub, T, [&](uint32_t flat, uint32_t v16) {
                    const uint32_t rel = flat - base;
                    if (rel >= span) return;
                    const uint32_t ihr = rel / uint32_t(g.W), iw = rel - ihr * uint32_t(g.W);
                    place(c, ih_lo + int(ihr), int(iw), v16);
                });
            }
        }
    }
    __syncthreads();
    // a token's segment: the block's columns (the whole padded row when there is one block), whole 16-byte
    // units at a 16-byte aligned column; a ragged last block writes only its own columns
    const int seg = ts.nblocks == 1 ? rowlen : bw * (NHWC ? g.C : taps);
    const int per_row = seg / 8, tile_row = rowlen / 8;
    const int64_t tok0 = (int64_t(n) * g.OH + oy0) * g.OW;
    const int col0 = NHWC ? b0 * g.C : b0 * taps;
    for (int i = tid; i < rb * g.OW * per_row; i += 256) {
        const int t = i / per_row, w = i - t * per_row;
        reinterpret_cast<u32x4 *>(B + (tok0 + t) * pitch + col0)[w] = tile16[t * tile_row + w];
    }
}

// dY [N][J][P] -> dYt [N * P][J]  (P = OH * OW): workgroup (n, 64 output channels, 256 positions)
// through an LDS slab; loads run along the positions, stores along the channels.  PAIRS (P even):
// a lane loads two positions (4 bytes) and stores four channels (8 bytes); the slab pitch of 129
// words keeps both the 4-byte stores aligned and the transposed reads off each other's banks.
// (A variant with 16-byte loads and stores needs a pitch that is a multiple of 8 and was 40 % slower
// for the bank conflicts.)  Otherwise 2-byte loads and channel-pair stores.
constexpr int TJ = 64, TP = 256;
template <bool PAIRS>
__global__ void __launch_bounds__(256)
dy_tokens_tiled_kernel(const uint16_t *__restrict__ dY, int J, int64_t P, int jblocks, int pblocks,
                       uint16_t *__restrict__ dYt)
{
    constexpr int PITCH = PAIRS ? TP + 2 : TP + 1;
    __shared__ __attribute__((aligned(4))) uint16_t slab[TJ][PITCH];
    const int tid = threadIdx.x;
    const int pb = blockIdx.x % pblocks;
    const int jb = (blockIdx.x / pblocks) % jblocks;
    const int64_t n = blockIdx.x / (int64_t(pblocks) * jblocks);
    const int j0 = jb * TJ, jw = min(TJ, J - j0);                 // jw is a multiple of 8
    const int64_t p0 = int64_t(pb) * TP;
    const int pw = int(min<int64_t>(TP, P - p0));                 // even when PAIRS
    constexpr int BATCH = 8;
    if (PAIRS) {
        // 128 lanes cover the 256 positions of a channel; the two halves of the workgroup take alternate channels
        const int half = tid >> 7, pp = (tid & 127) * 2;
        for (int jj0 = half; jj0 < jw; jj0 += 2 * BATCH) {
            uint32_t v[BATCH];
#pragma unroll
            for (int q = 0; q < BATCH; ++q)
                if (jj0 + 2 * q < jw && pp < pw)
                    v[q] = *reinterpret_cast<const uint32_t *>(dY + (n * J + j0 + jj0 + 2 * q) * P + p0 + pp);
#pragma unroll
            for (int q = 0; q < BATCH; ++q)
                if (jj0 + 2 * q < jw && pp < pw) *reinterpret_cast<uint32_t *>(&slab[jj0 + 2 * q][pp]) = v[q];
        }
        __syncthreads();
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        for (int i = tid; i < TP * (TJ / 4); i += 256) {
            const int t = i / (TJ / 4), jj = (i % (TJ / 4)) * 4;
            if (t < pw && jj < jw) {
                const u32x2 o = {uint32_t(slab[jj][t]) | (uint32_t(slab[jj + 1][t]) << 16),
                                 uint32_t(slab[jj + 2][t]) | (uint32_t(slab[jj + 3][t]) << 16)};
                *reinterpret_cast<u32x2 *>(dYt + ((n * P + p0 + t) * J + j0 + jj)) = o;
            }
        }
    } else {
        // thread tid reads position tid of every channel: eight loads in flight, each in a full register
        for (int jj0 = 0; jj0 < jw; jj0 += BATCH) {
            uint32_t v[BATCH];
#pragma unroll
            for (int q = 0; q < BATCH; ++q)
                if (jj0 + q < jw && tid < pw) v[q] = dY[(n * J + j0 + jj0 + q) * P + p0 + tid];
#pragma unroll
            for (int q = 0; q < BATCH; ++q)
                if (jj0 + q < jw && tid < pw) slab[jj0 + q][tid] = uint16_t(v[q]);
        }
        __syncthreads();
        uint32_t *dst = reinterpret_cast<uint32_t *>(dYt);       // J is even: a channel pair is one aligned word
        for (int i = tid; i < TP * (TJ / 2); i += 256) {
            const int t = i / (TJ / 2), jj = (i % (TJ / 2)) * 2;
            if (t < pw && jj < jw)
                dst[((n * P + p0 + t) * J + j0 + jj) / 2] = uint32_t(slab[jj][t]) | (uint32_t(slab[jj + 1][t]) << 16);
        }
    }
}

}  // namespace

ConvIm2colPlan conv_im2col_plan(const ConvGeneral &p)
{
    ConvIm2colPlan plan;
    plan.fp = FcProblem{p.N * p.OH * p.OW, p.C * p.g.kh * p.g.kw, p.J, p.k};
    plan.gemm = fc_dense_plan(plan.fp);
    plan.dyt_bytes = p.nhwc ? 0 : round_up(size_t(plan.fp.ntok) * p.J * 2, 256);

    // Tiled form: column blocks whose segment of a token's row is whole 16-byte units.  With C % 8 == 0
    // a block is as narrow as keeps the segment at 256 bytes or more (blocks of channels in NCHW, of taps
    // in NHWC): the narrower the block, the more output rows fit a tile, and the longer the runs of pairs
    // a workgroup reads per channel (1x1 over 256 channels: 131 us with one block, 85 with two).
    // Otherwise one block holds the whole padded row, if a row of tokens fits the LDS at all.
    const int64_t taps = p.g.kh * p.g.kw;
    int64_t budget = 32 * 1024;                // several workgroups per compute unit hide each other's load rounds (64 KB: 10-15 % slower)
    const int64_t hard = 150 * 1024;
    budget = dev_env("DROPIT_IM2COL_LDS", budget);
    const int64_t units_total = p.nhwc ? taps : p.C;          // what a block is a range of
    const int64_t per_unit = p.nhwc ? p.C : taps;             // columns per unit
    plan.tiled = false;
    plan.rowptr_bytes = 0;
    int64_t blk = units_total, rowlen = plan.gemm.pitch;
    if (p.C % 8 == 0) {
        blk = (128 + per_unit - 1) / per_unit;                // 128 elements = 256 bytes
        if (!p.nhwc) blk = (blk + 7) / 8 * 8;                 // channel blocks: multiples of 8 keep c0 * taps aligned for odd tap counts
        while (blk > (p.nhwc ? 1 : 8) && p.OW * blk * per_unit * 2 > budget) blk -= p.nhwc ? 1 : 8;
        blk = std::min(blk, units_total);
        if (blk < units_total) rowlen = blk * per_unit;
    }
    if (p.OW * rowlen * 2 > hard || rowlen % 8 != 0) return plan;
    const int64_t nblocks = (units_total + blk - 1) / blk;
    if (nblocks > 1 && (blk * per_unit) % 8 != 0) return plan;
    // rows per band: fill the budget, but leave at least ~512 workgroups when the problem has them
    int64_t rb = std::max<int64_t>(1, budget / (p.OW * rowlen * 2));
    rb = std::min(rb, std::max<int64_t>(1, p.N * nblocks * p.OH / 512));
    rb = std::min(rb, p.OH);
    const int64_t bands = (p.OH + rb - 1) / rb;
    const int64_t rows = p.nhwc ? p.N * p.H : p.N * p.C * p.H;
    if (p.N * nblocks * bands + 64 > INT32_MAX || rows + 1 > INT32_MAX) return plan;
    if (p.nhwc && p.W * p.C > INT32_MAX) return plan;
    plan.tiled = true;
    plan.nblocks = int(nblocks);
    plan.blk = int(blk);
    plan.bands = int(bands);
    plan.rb = int(rb);
    plan.rowlen = int(rowlen);
    plan.lds_bytes = size_t(rb) * p.OW * rowlen * 2;
    plan.rowptr_bytes = round_up(size_t(rows + 1) * 4, 256);
    return plan;
}

bool conv_im2col_supported(const ConvGeneral &p)
{
    if (p.J % 8 != 0 || p.N < 1 || p.C < 1 || p.OH < 1 || p.OW < 1) return false;
    const int64_t taps = p.g.kh * p.g.kw;
    if (taps > 32768 || p.C * taps > 32768) return false;
    const int64_t ntok = p.N * p.OH * p.OW;
    if (ntok > INT32_MAX) return false;
    if (!fc_dense_supported(FcProblem{ntok, p.C * taps, p.J, p.k})) return false;
    // the im2col rows live in the workspace: at most 1 GiB of them
    const ConvIm2colPlan plan = conv_im2col_plan(p);
    return plan.gemm.dense_bytes <= (size_t(1) << 30);
}

dropit_status conv_im2col_run(const ConvGeneral &p, const ConvIm2colPlan &plan, const void *vals, const int32_t *idx,
                              const void *dY, float *dW, char *ws, hipStream_t stream)
{
    uint16_t *B = reinterpret_cast<uint16_t *>(ws);
    float *partial = reinterpret_cast<float *>(ws + plan.gemm.dense_bytes);
    uint16_t *dYt = reinterpret_cast<uint16_t *>(ws + plan.gemm.dense_bytes + plan.gemm.partial_bytes);
    if (size_t(plan.gemm.ntok_pad) * plan.gemm.pitch * 2 > plan.gemm.dense_bytes) return DROPIT_EINVAL;
    const int64_t numel = p.N * p.C * p.H * p.W;
    const Geometry g = {int(p.C), int(p.H), int(p.W), int(p.OH), int(p.OW), int(p.g.kh), int(p.g.kw),
                        int(p.g.stride_h), int(p.g.stride_w), int(p.g.pad_h), int(p.g.pad_w), int(p.g.dil_h),
                        int(p.g.dil_w)};

    trace_mark(stream);
    if (plan.tiled) {
        uint32_t *row_ptr = reinterpret_cast<uint32_t *>(ws + plan.gemm.dense_bytes + plan.gemm.partial_bytes + plan.dyt_bytes);
        const int64_t rows = p.nhwc ? p.N * p.H : p.N * p.C * p.H;
        const uint32_t row_len = uint32_t(p.nhwc ? p.W * p.C : p.W);
        launch_row_starts(idx, p.k, row_len, rows, row_ptr, stream);
        static std::atomic<uint64_t> attr_set{0};
        if (!once_per_device(attr_set, [] {
                return hipFuncSetAttribute(reinterpret_cast<const void *>(im2col_tiled_kernel<true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024) == hipSuccess &&
                       hipFuncSetAttribute(reinterpret_cast<const void *>(im2col_tiled_kernel<false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024) == hipSuccess;
            }))
            return DROPIT_EHIP;
        // at least 8 threads per channel run: neighbouring lanes then read neighbouring pairs (with one or two
        // threads per run every lane of a load asks for a line of its own: 1x1 over 256 channels 144 -> 126 us)
        int tmin = 8;
        tmin = int(dev_env("DROPIT_IM2COL_TMIN", tmin));
        const TileShape ts = {plan.nblocks, plan.blk, plan.bands, plan.rb, plan.rowlen, tmin};
        const int64_t pad_chunks = (plan.gemm.ntok_pad - plan.fp.ntok) * plan.gemm.pitch / 8;
        const int pad_wgs = int(std::min<int64_t>((pad_chunks + 255) / 256, 64));
        const int grid = int(p.N * plan.nblocks * plan.bands) + pad_wgs;
        if (p.nhwc)
            im2col_tiled_kernel<true><<<grid, 256, plan.lds_bytes, stream>>>(
                static_cast<const uint16_t *>(vals), idx, row_ptr, int(p.N), g, ts, plan.gemm.pitch, plan.fp.ntok,
                plan.gemm.ntok_pad, pad_wgs, B);
        else
            im2col_tiled_kernel<false><<<grid, 256, plan.lds_bytes, stream>>>(
                static_cast<const uint16_t *>(vals), idx, row_ptr, int(p.N), g, ts, plan.gemm.pitch, plan.fp.ntok,
                plan.gemm.ntok_pad, pad_wgs, B);
    } else {
        const int64_t chunks = int64_t(plan.gemm.dense_bytes / 16);
        fill_zero16_kernel<<<int(std::min<int64_t>((chunks + 255) / 256, 8192)), 256, 0, stream>>>(
            reinterpret_cast<u32x4 *>(B), chunks);
        const int blocks = int(std::min<int64_t>((p.k + 255) / 256, 16384));
        if (p.nhwc)
            im2col_scatter_kernel<true><<<blocks, 256, 0, stream>>>(static_cast<const uint16_t *>(vals), idx, p.k, numel,
                                                                    g, plan.gemm.pitch, B);
        else
            im2col_scatter_kernel<false><<<blocks, 256, 0, stream>>>(static_cast<const uint16_t *>(vals), idx, p.k, numel,
                                                                     g, plan.gemm.pitch, B);
    }
    const void *tokens = dY;
    if (!p.nhwc) {
        const int64_t P = p.OH * p.OW;
        const int jblocks = int((p.J + TJ - 1) / TJ);
        const int64_t pblocks = (P + TP - 1) / TP;
        const int64_t grid = p.N * jblocks * pblocks;
        if (grid > INT32_MAX) return DROPIT_EINVAL;
        if (P % 2 == 0)
            dy_tokens_tiled_kernel<true><<<int(grid), 256, 0, stream>>>(static_cast<const uint16_t *>(dY), int(p.J), P,
                                                                        jblocks, int(pblocks), dYt);
        else
            dy_tokens_tiled_kernel<false><<<int(grid), 256, 0, stream>>>(static_cast<const uint16_t *>(dY), int(p.J), P,
                                                                         jblocks, int(pblocks), dYt);
        tokens = dYt;
    }
    trace_mark(stream);
    if (launch_status() != DROPIT_OK) return DROPIT_EHIP;
    return fc_dense_gemm(plan.fp, plan.gemm, tokens, B, partial, dW, stream);
}

}  // namespace dropit
