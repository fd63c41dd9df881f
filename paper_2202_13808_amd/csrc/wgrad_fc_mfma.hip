// FC weight gradient dW = dY^T * R(a^) on the gfx950 matrix cores
// (Sec. 3.2, Eq. fc_backward_elem_save; the recover step R(.) of Sec. 3.2 is
// fused: the zero-filled tensor only ever exists as LDS tiles).
//
// GEMM view: M = c_out (columns of dY), N = c_in (columns of a^), reduction
// K = tokens.  Both operands are stored with K as the slow axis, so
//   A (dY)  : global -> registers -> LDS [k][m] (row pitch = 64 bytes mod 256),
//             fragments via the LDS transpose read (ds_read_b64_tr_b16)
//   B (a^)  : a prep kernel re-buckets the sorted (value, index) pairs by
//             (token block, column block) and packs each as
//             [bf16 value | LDS byte offset]; the GEMM zero-fills an LDS tile
//             [n][k] and scatters one 16-bit store per pair, fragments via
//             ds_read_b128.
// Products are exact (bf16 x bf16 in fp32), accumulation is fp32 in a fixed
// order (K ascending inside a split, splits summed in ascending order by a
// separate kernel), so dW is bit-reproducible.
#include "common.hpp"
#include "wgrad_internal.hpp"

namespace dropit {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int THREADS = 256;

// ---------------------------------------------------------------------------
// Cooperative lower_bound over a sorted int32 array: number of elements < target.
// All THREADS threads of the block must call it (contains barriers).
__device__ inline int64_t block_lower_bound(const int32_t *__restrict__ idx, int64_t n, int64_t target)
{
    int64_t lo = 0, hi = n;
    while (hi > lo) {
        const int64_t span = hi - lo;
        const int64_t step = (span + THREADS - 1) / THREADS;
        const int64_t pos = lo + int64_t(threadIdx.x) * step;
        const int pred = (pos < hi) && (int64_t(idx[pos]) < target);
        const int c = __syncthreads_count(pred);   // probes are monotone: the first c are true
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

// ---------------------------------------------------------------------------
// Prep: one workgroup per token block.  Re-buckets that block's pairs by column
// block and packs them for the GEMM's LDS scatter.  The order of pairs inside a
// bucket is arbitrary (each targets a distinct LDS slot), so it cannot affect dW.
template <int BK, int BN, int PITCH_B /*bytes*/>
__global__ void __launch_bounds__(THREADS)
fc_bucket_kernel(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx, int64_t k, int64_t ntok,
                 int n_cols, int nb_count, uint32_t *__restrict__ packed, uint32_t *__restrict__ tile_ptr)
{
    extern __shared__ uint32_t s_cnt[];               // [2 * nb_count + 1]: counts / bases, then fill cursors
    uint32_t *s_fill = s_cnt + nb_count + 1;
    __shared__ uint32_t s_wave[THREADS / WAVE];
    const int tid = threadIdx.x;
    const int64_t kb = blockIdx.x;
    const int64_t seg_first = kb * BK * int64_t(n_cols);               // first flat index of the block
    const int64_t seg_elems = min<int64_t>(BK, ntok - kb * BK) * n_cols;
    const int64_t lo = block_lower_bound(idx, k, seg_first);
    const int64_t hi = block_lower_bound(idx, k, seg_first + seg_elems);
    for (int i = tid; i < 2 * nb_count + 1; i += THREADS) s_cnt[i] = 0;
    __syncthreads();
    for (int64_t j = lo + tid; j < hi; j += THREADS) {
        const int64_t r = int64_t(idx[j]) - seg_first;
        if (r >= 0 && r < seg_elems) {
            const uint32_t col = uint32_t(r) % uint32_t(n_cols);
            atomicAdd(&s_cnt[col / BN], 1u);
        }
    }
    __syncthreads();
    // exclusive scan of the bucket counts (nb_count <= 2*THREADS handled per pass of THREADS)
    uint32_t carry = 0;
    for (int base = 0; base < nb_count; base += THREADS) {
        const int b = base + tid;
        const uint32_t c = (b < nb_count) ? s_cnt[b] : 0u;
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<THREADS>(c, s_wave, total);
        if (b < nb_count) s_cnt[b] = carry + ex;
        carry += total;
        __syncthreads();
    }
    if (tid == 0) s_cnt[nb_count] = carry;
    __syncthreads();
    uint32_t *tp = tile_ptr + kb * (nb_count + 1);
    for (int b = tid; b <= nb_count; b += THREADS) tp[b] = uint32_t(lo) + s_cnt[b];
    for (int64_t j = lo + tid; j < hi; j += THREADS) {
        const int64_t r = int64_t(idx[j]) - seg_first;
        if (r >= 0 && r < seg_elems) {
            const uint32_t kl = uint32_t(r) / uint32_t(n_cols);
            const uint32_t col = uint32_t(r) - kl * uint32_t(n_cols);
            const uint32_t nb = col / BN;
            const uint32_t nl = col - nb * BN;
            const uint32_t slot = atomicAdd(&s_fill[nb], 1u);
            packed[lo + s_cnt[nb] + slot] = (uint32_t(vals[j]) << 16) | (nl * PITCH_B + kl * 2);
        }
    }
}

// ---------------------------------------------------------------------------
// GEMM: one workgroup = one BM x BN tile of dW over a contiguous range of token
// blocks (split `blockIdx.z` of `splits`).  4 wavefronts in a 2x2 grid, each
// (BM/2) x (BN/2) built from 32x32x16 bf16 MFMAs.
template <int BM, int BN, int BK>
struct FcTile {
    static constexpr int PITCH_A = (BM + 32) * 2;          // bytes; == 64 mod 256 for BM = 128/256
    static constexpr int PITCH_B = BK * 2 + 16;            // bytes; odd multiple of 16
    static constexpr int A_BYTES = BK * PITCH_A;
    static constexpr int B_BYTES = BN * PITCH_B;
    static constexpr int LDS_BYTES = 2 * A_BYTES + 3 * B_BYTES;
    static constexpr int WM = BM / 2, WN = BN / 2;
    static constexpr int FM = WM / 32, FN = WN / 32;
    static constexpr int A_VECS = BK * (BM / 8) / THREADS; // 16-byte global loads per thread per step
    static constexpr int B_VEC16 = B_BYTES / 16;
    static constexpr int B_ZERO = (B_VEC16 + THREADS - 1) / THREADS;  // 16-byte zero stores per thread per step
    static constexpr int ENT = 4;                          // packed pairs prefetched per thread per step
    static_assert(BK * (BM / 8) % THREADS == 0, "A tile must divide over the block");
};

template <int BM, int BN, int BK>
__global__ void __launch_bounds__(THREADS)
fc_mfma_kernel(const uint16_t *__restrict__ dY, const uint32_t *__restrict__ packed,
               const uint32_t *__restrict__ tile_ptr, int64_t ntok, int M, int N, int nb_count,
               int nkb, int splits, float *__restrict__ out /* dW or partials [splits][M][N] */)
{
    using T = FcTile<BM, BN, BK>;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char *ldsA = lds;                         // [2][BK][PITCH_A]
    char *ldsB = lds + 2 * T::A_BYTES;        // [3][BN][PITCH_B]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int nb = blockIdx.x, mb = blockIdx.y, split = blockIdx.z;
    const int m0 = mb * BM;

    // token blocks of this split: an even partition of [0, nkb)
    const int kb_begin = int(int64_t(nkb) * split / splits);
    const int kb_end = int(int64_t(nkb) * (split + 1) / splits);
    const int steps = kb_end - kb_begin;

    f32x16 acc[T::FM][T::FN];
#pragma unroll
    for (int i = 0; i < T::FM; ++i)
#pragma unroll
        for (int j = 0; j < T::FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // per-thread A load geometry: vector v covers row (v / (BM/8)), columns 8*(v % (BM/8))
    uint4 a_reg[T::A_VECS];
    uint32_t e_reg[T::ENT];
    uint32_t e_lo = 0, e_hi = 0;              // packed range of the prefetched step

    auto load_step = [&](int kb) {
        const int64_t tok0 = int64_t(kb) * BK;
#pragma unroll
        for (int i = 0; i < T::A_VECS; ++i) {
            const int v = tid + i * THREADS;
            const int row = v / (BM / 8), cv = v % (BM / 8);
            const int64_t tok = tok0 + row;
            const int m = m0 + cv * 8;
            uint4 q = make_uint4(0, 0, 0, 0);
            if (tok < ntok && m < M) q = *reinterpret_cast<const uint4 *>(dY + tok * M + m);
            a_reg[i] = q;
        }
        e_lo = tile_ptr[int64_t(kb) * (nb_count + 1) + nb];
        e_hi = tile_ptr[int64_t(kb) * (nb_count + 1) + nb + 1];
#pragma unroll
        for (int i = 0; i < T::ENT; ++i) {
            const uint32_t j = e_lo + tid + i * THREADS;
            e_reg[i] = (j < e_hi) ? packed[j] : 0xFFFFFFFFu;
        }
    };
    auto store_step = [&](int abuf, int bbuf) {
        char *a = ldsA + abuf * T::A_BYTES;
#pragma unroll
        for (int i = 0; i < T::A_VECS; ++i) {
            const int v = tid + i * THREADS;
            const int row = v / (BM / 8), cv = v % (BM / 8);
            *reinterpret_cast<uint4 *>(a + row * T::PITCH_A + cv * 16) = a_reg[i];
        }
        char *b = ldsB + bbuf * T::B_BYTES;
#pragma unroll
        for (int i = 0; i < T::ENT; ++i) {
            const uint32_t p = e_reg[i];
            if (p != 0xFFFFFFFFu) *reinterpret_cast<uint16_t *>(b + (p & 0xFFFFu)) = uint16_t(p >> 16);
        }
        // pairs beyond the prefetch depth (dense tiles): fetched and scattered in place
        for (uint32_t j = e_lo + tid + T::ENT * THREADS; j < e_hi; j += THREADS) {
            const uint32_t p = packed[j];
            *reinterpret_cast<uint16_t *>(b + (p & 0xFFFFu)) = uint16_t(p >> 16);
        }
    };
    auto zero_b = [&](int bbuf) {
        char *b = ldsB + bbuf * T::B_BYTES;
#pragma unroll
        for (int i = 0; i < T::B_ZERO; ++i)
            if (tid + i * THREADS < T::B_VEC16)
                *reinterpret_cast<uint4 *>(b + (tid + i * THREADS) * 16) = make_uint4(0, 0, 0, 0);
    };
    auto compute = [&](int abuf, int bbuf) {
        const char *a = ldsA + abuf * T::A_BYTES;
        const char *b = ldsB + bbuf * T::B_BYTES;
        const int g = lane >> 4, p16 = lane & 15;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[T::FM], bfv[T::FN];
#pragma unroll
            for (int i = 0; i < T::FM; ++i) {
                const int krow = kk * 16 + (g >> 1) * 8 + (p16 >> 2);
                const int mcol = wm * T::WM + i * 32 + (g & 1) * 16 + (p16 & 3) * 4;
                const char *p = a + krow * T::PITCH_A + mcol * 2;
                const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
                const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * T::PITCH_A));
                const s16x8 full = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
                af[i] = __builtin_bit_cast(bf16x8, full);
            }
#pragma unroll
            for (int j = 0; j < T::FN; ++j) {
                const int ncol = wn * T::WN + j * 32 + (lane & 31);
                const char *p = b + ncol * T::PITCH_B + (kk * 16 + (lane >> 5) * 8) * 2;
                bfv[j] = *reinterpret_cast<const bf16x8 *>(p);
            }
#pragma unroll
            for (int i = 0; i < T::FM; ++i)
#pragma unroll
                for (int j = 0; j < T::FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfv[j], acc[i][j], 0, 0, 0);
        }
    };

    if (steps > 0) {
        zero_b(0);
        zero_b(1);
        load_step(kb_begin);
        __syncthreads();
        store_step(0, 0);
        if (steps > 1) load_step(kb_begin + 1);
        __syncthreads();
        for (int s = 0; s < steps; ++s) {
            if (s + 1 < steps) store_step((s + 1) & 1, (s + 1) % 3);
            if (s + 2 < steps) load_step(kb_begin + s + 2);
            zero_b((s + 2) % 3);
            compute(s & 1, s % 3);
            __syncthreads();
        }
    }

    // epilogue: acc[i][j][e] is row 8*(e/4) + 4*(lane/32) + e%4, column lane%32 of its 32x32 block
    float *dst = out + int64_t(split) * M * N;
#pragma unroll
    for (int i = 0; i < T::FM; ++i)
#pragma unroll
        for (int j = 0; j < T::FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * T::WM + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                const int n = nb * BN + wn * T::WN + j * 32 + (lane & 31);
                if (m < M && n < N) dst[int64_t(m) * N + n] = acc[i][j][e];
            }
}

// Sums the split-K partials in ascending split order: dW = ((p0 + p1) + p2) + ...
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float4 *__restrict__ partial, int64_t n4, int splits, float4 *__restrict__ dW)
{
    for (int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; i < n4; i += int64_t(gridDim.x) * blockDim.x) {
        float4 s = partial[i];
        for (int p = 1; p < splits; ++p) {
            const float4 v = partial[int64_t(p) * n4 + i];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        dW[i] = s;
    }
}

constexpr int BM = 128, BN = 128, BK = 32;
using Tile = FcTile<BM, BN, BK>;

}  // namespace

bool fc_mfma_supported(const FcProblem &p)
{
    // 16-byte dY vectors need c_out % 8 == 0; packed offsets and counters are 32-bit
    return p.cout % 8 == 0 && p.cin >= 1 && (p.cin + BN - 1) / BN <= 2 * THREADS && p.cout * p.cin % 4 == 0;
}

FcPlan fc_mfma_plan(const FcProblem &p)
{
    FcPlan plan;
    plan.nkb = int((p.ntok + BK - 1) / BK);
    plan.nb_count = int((p.cin + BN - 1) / BN);
    plan.mb_count = int((p.cout + BM - 1) / BM);
    const int tiles = plan.nb_count * plan.mb_count;
    int splits = (2 * 256 + tiles - 1) / tiles;        // about two workgroups per compute unit
    if (splits > plan.nkb) splits = plan.nkb;
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    plan.splits = splits;
    plan.packed_bytes = round_up(size_t(p.k > 0 ? p.k : 1) * 4, 256);
    plan.tileptr_bytes = round_up(size_t(plan.nkb) * (plan.nb_count + 1) * 4, 256);
    plan.partial_bytes = splits > 1 ? round_up(size_t(splits) * p.cout * p.cin * 4, 256) : 0;
    return plan;
}

dropit_status fc_mfma_run(const FcProblem &p, const FcPlan &plan, const void *vals, const int32_t *idx,
                          const void *dY, float *dW, char *ws, hipStream_t stream)
{
    uint32_t *packed = reinterpret_cast<uint32_t *>(ws);
    uint32_t *tile_ptr = reinterpret_cast<uint32_t *>(ws + plan.packed_bytes);
    float *partial = reinterpret_cast<float *>(ws + plan.packed_bytes + plan.tileptr_bytes);

    trace_mark(stream);
    const size_t bucket_lds = size_t(2 * plan.nb_count + 1) * 4;
    fc_bucket_kernel<BK, BN, Tile::PITCH_B><<<plan.nkb, THREADS, bucket_lds, stream>>>(
        static_cast<const uint16_t *>(vals), idx, p.k, p.ntok, int(p.cin), plan.nb_count, packed, tile_ptr);

    trace_mark(stream);
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(fc_mfma_kernel<BM, BN, BK>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, Tile::LDS_BYTES) != hipSuccess)
            return DROPIT_EHIP;
        attr_set = true;
    }
    const dim3 grid(plan.nb_count, plan.mb_count, plan.splits);
    float *out = plan.splits > 1 ? partial : dW;
    fc_mfma_kernel<BM, BN, BK><<<grid, THREADS, Tile::LDS_BYTES, stream>>>(
        static_cast<const uint16_t *>(dY), packed, tile_ptr, p.ntok, int(p.cout), int(p.cin), plan.nb_count,
        plan.nkb, plan.splits, out);

    trace_mark(stream);
    if (plan.splits > 1) {
        const int64_t n4 = p.cout * p.cin / 4;
        const int blocks = int(std::min<int64_t>((n4 + 255) / 256, 2048));
        splitk_reduce_kernel<<<blocks, 256, 0, stream>>>(reinterpret_cast<const float4 *>(partial), n4, plan.splits,
                                                         reinterpret_cast<float4 *>(dW));
    }
    trace_mark(stream);
    return launch_status();
}

}  // namespace dropit
