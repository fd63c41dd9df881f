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
#include <cstdlib>

#ifndef DROPIT_ABLATE
#define DROPIT_ABLATE 0          // development only: bit mask of pipeline parts to leave out (wrong results)
#endif

namespace dropit {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int THREADS = 1024;     // prep (bucket) kernel workgroup size
constexpr int PREP_CACHE = 12;    // pairs per thread the prep kernel keeps in registers between its two phases

// ---------------------------------------------------------------------------
// Cooperative lower_bound over a sorted int32 array for two targets at once
// (number of elements < t0 and < t1): THREADS-ary search, both targets share the
// rounds, so ~3 rounds of one load each for a million elements.
// All THREADS threads of the block must call it (contains barriers).
__device__ inline void block_lower_bound2(const int32_t *__restrict__ idx, int64_t n, int64_t t0, int64_t t1,
                                          int64_t &r0, int64_t &r1)
{
    int64_t lo[2] = {0, 0}, hi[2] = {n, n};
    const int64_t target[2] = {t0, t1};
    while (hi[0] > lo[0] || hi[1] > lo[1]) {
        int pred[2];
        int64_t step[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int64_t span = hi[q] - lo[q];
            step[q] = (span + THREADS - 1) / THREADS;
            const int64_t pos = lo[q] + int64_t(threadIdx.x) * step[q];
            pred[q] = (pos < hi[q]) && (int64_t(idx[pos]) < target[q]);
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int c = __syncthreads_count(pred[q]);   // probes are monotone: the first c are true
            if (hi[q] > lo[q]) {
                if (c == 0) {
                    hi[q] = lo[q];
                } else {
                    const int64_t nlo = lo[q] + int64_t(c - 1) * step[q] + 1;
                    const int64_t nhi = min(lo[q] + int64_t(c) * step[q], hi[q]);
                    lo[q] = nlo;
                    hi[q] = nhi;
                }
            }
        }
    }
    r0 = lo[0];
    r1 = lo[1];
}

// ---------------------------------------------------------------------------
// Prep: one workgroup per token block.  Re-buckets that block's pairs by column
// block and packs them for the GEMM's LDS scatter.  The order of pairs inside a
// bucket is arbitrary (each targets a distinct LDS slot), so it cannot affect dW.
// A returning LDS atomic hands every pair its slot inside its bucket while the
// buckets are being counted, and the packed words wait in registers for the bucket
// bases, so the block's pairs are read once.
template <int BK, int BN, int PITCH_B /*bytes*/>
__global__ void __launch_bounds__(THREADS)
fc_bucket_kernel(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx, int64_t k, int64_t ntok,
                 int n_cols, int nb_count, uint32_t *__restrict__ packed, uint32_t *__restrict__ tile_ptr)
{
    extern __shared__ uint32_t s_cnt[];               // [nb_count + 1]: counts, then exclusive bases
    __shared__ uint32_t s_wave[THREADS / WAVE];
    const int tid = threadIdx.x;
    const int64_t kb = blockIdx.x;
    const int64_t seg_first = kb * BK * int64_t(n_cols);               // first flat index of the block
    const int64_t seg_elems = min<int64_t>(BK, ntok - kb * BK) * n_cols;
    int64_t lo, hi;
    block_lower_bound2(idx, k, seg_first, seg_first + seg_elems, lo, hi);
    for (int i = tid; i <= nb_count; i += THREADS) s_cnt[i] = 0;
    __syncthreads();

    // phase 1: count, and remember (packed word, bucket, slot in bucket) per pair
    uint32_t word[PREP_CACHE], where[PREP_CACHE];     // where = bucket << 16 | slot
    auto classify = [&](int64_t j, uint32_t &w, uint32_t &nb) -> bool {
        const int64_t r = int64_t(idx[j]) - seg_first;
        if (r < 0 || r >= seg_elems) return false;    // never for a sorted, in-range index array
        const uint32_t kl = uint32_t(r) / uint32_t(n_cols);
        const uint32_t col = uint32_t(r) - kl * uint32_t(n_cols);
        nb = col / BN;
        w = (uint32_t(vals[j]) << 16) | ((col - nb * BN) * PITCH_B + kl * 2);
        return true;
    };
#pragma unroll
    for (int i = 0; i < PREP_CACHE; ++i) {
        const int64_t j = lo + tid + int64_t(i) * THREADS;
        where[i] = 0xFFFFFFFFu;
        word[i] = 0;
        uint32_t nb;
        if (j < hi && classify(j, word[i], nb)) where[i] = (nb << 16) | atomicAdd(&s_cnt[nb], 1u);
    }
    const int64_t j_rest = lo + int64_t(PREP_CACHE) * THREADS;         // pairs beyond the register cache (dense blocks)
    uint32_t *s_fill = s_cnt + nb_count + 1;                           // [nb_count] cursors of the uncached tail
    if (j_rest < hi) {                                                 // uniform
        __syncthreads();                                               // cached pairs own slots [0, cached count)
        for (int i = tid; i < nb_count; i += THREADS) s_fill[i] = s_cnt[i];
        __syncthreads();
        for (int64_t j = j_rest + tid; j < hi; j += THREADS) {
            uint32_t w, nb;
            if (classify(j, w, nb)) atomicAdd(&s_cnt[nb], 1u);
        }
    }
    __syncthreads();
    // exclusive scan of the bucket counts
    uint32_t carry = 0;
    for (int base = 0; base < nb_count; base += THREADS) {
        const int b = base + tid;
        const uint32_t c = (b < nb_count) ? s_cnt[b] : 0u;
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<THREADS>(c, s_wave, total);
        __syncthreads();
        if (b < nb_count) s_cnt[b] = carry + ex;
        carry += total;
    }
    if (tid == 0) s_cnt[nb_count] = carry;
    __syncthreads();
    uint32_t *tp = tile_ptr + kb * (nb_count + 1);
    for (int b = tid; b <= nb_count; b += THREADS) tp[b] = uint32_t(lo) + s_cnt[b];
    // phase 2: place
#pragma unroll
    for (int i = 0; i < PREP_CACHE; ++i)
        if (where[i] != 0xFFFFFFFFu) packed[lo + s_cnt[where[i] >> 16] + (where[i] & 0xFFFFu)] = word[i];
    if (j_rest < hi) {
        // the uncached tail takes the slots after the cached pairs of its bucket
        for (int64_t j = j_rest + tid; j < hi; j += THREADS) {
            uint32_t w, nb;
            if (classify(j, w, nb)) packed[lo + s_cnt[nb] + atomicAdd(&s_fill[nb], 1u)] = w;
        }
    }
}

// ---------------------------------------------------------------------------
// GEMM: one workgroup = one BM x BN tile of dW over a contiguous range of token
// blocks (one of `splits` K-slices).  WAVES_M x WAVES_N wavefronts, each a
// (BM/WAVES_M) x (BN/WAVES_N) sub-tile built from 32x32x16 bf16 MFMAs.
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int WPE_, int STAGES_, int PROD_ = 0>
struct FcCfg {
    // PROD = 0: every wavefront both moves data and multiplies.  PROD > 0: that many extra wavefronts do all
    // the data movement (global loads, LDS stores, scatter, clear) while the WAVES_M x WAVES_N others only
    // read LDS and issue MFMAs, so a step's memory waits never sit in front of its matrix work.
    static constexpr int PROD = PROD_;
    static constexpr int CONS_WAVES = WAVES_M_ * WAVES_N_;
    static constexpr int STAGES = STAGES_;                 // register stages = global-load prefetch depth (even)
    static_assert(STAGES_ >= 2 && STAGES_ % 2 == 0, "prefetch depth must be even");
    static constexpr int WPE = WPE_;                       // wavefronts per SIMD the register budget must allow
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
    static constexpr int NTHREADS = WAVE * (WAVES_M * WAVES_N + PROD);
    static constexpr int MOVERS = PROD ? WAVE * PROD : NTHREADS;   // threads that move data
    static constexpr int PITCH_A = (BM + 32) * 2;          // bytes; rows 64 bytes apart mod 256: conflict-free transpose reads
    static constexpr int PITCH_B = BK * 2 + 16;            // bytes; odd multiple of 16: conflict-free 16-byte row reads
    static constexpr int A_BYTES = BK * PITCH_A;
    static constexpr int B_BYTES = (BN * PITCH_B + MOVERS * 16 - 1) / (MOVERS * 16) * (MOVERS * 16);  // whole 16-byte stores per thread
    static constexpr int LDS_BYTES = 2 * A_BYTES + 3 * B_BYTES;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int FM = WM / 32, FN = WN / 32;
    static constexpr int A_VECS = BK * (BM / 8) / MOVERS; // 16-byte global loads per thread per step
    static constexpr int B_ZERO = B_BYTES / 16 / MOVERS;
    static constexpr int ENT = (BK * BN / 4 / MOVERS) < 2 ? 2 : (BK * BN / 4 / MOVERS);  // prefetch depth: 25% density
    static_assert(BK * (BM / 8) % MOVERS == 0, "A tile must divide over the block");
    static_assert(BN * PITCH_B < 65536, "packed LDS offsets are 16-bit");
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0, "MFMA 32x32x16 tiling");
};

template <typename C>
__global__ void __launch_bounds__(C::NTHREADS) __attribute__((amdgpu_waves_per_eu(C::WPE, C::WPE)))
fc_mfma_kernel(const uint16_t *__restrict__ dY, const uint32_t *__restrict__ packed,
               const uint32_t *__restrict__ tile_ptr, int64_t n_pairs, int64_t ntok, int M, int N, int nb_count,
               int mb_count, int nkb, int splits, float *__restrict__ out /* dW or partials [splits][M][N] */)
{
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, NT = C::MOVERS;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char *ldsA = lds;                         // [2][BK][PITCH_A]
    char *ldsB = lds + 2 * C::A_BYTES;        // [3][BN][PITCH_B]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool is_mover = C::PROD == 0 || wave >= C::CONS_WAVES;
    const bool is_consumer = C::PROD == 0 || wave < C::CONS_WAVES;
    const int tid = C::PROD ? int(threadIdx.x) - WAVE * C::CONS_WAVES : int(threadIdx.x);   // index among the movers
    const int wm = (wave % C::CONS_WAVES) / C::WAVES_N, wn = wave % C::WAVES_N;

    // Workgroups are dealt to the 8 XCDs round-robin by launch order.  Re-number so
    // that the workgroups sharing one XCD's L2 are consecutive tiles: same rows of
    // dY (mb), neighbouring column blocks (nb).
    const int total = nb_count * mb_count * splits;
    const int per_xcd = gridDim.x / 8;
    const int v = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    if (v >= total) return;
    const int nb = v % nb_count;
    const int mb = (v / nb_count) % mb_count;
    const int split = v / (nb_count * mb_count);
    const int m0 = mb * BM;

    // token blocks of this split: an even partition of [0, nkb)
    const int kb_begin = int(int64_t(nkb) * split / splits);
    const int kb_end = int(int64_t(nkb) * (split + 1) / splits);
    const int steps = kb_end - kb_begin;

    constexpr int TP_CAP = 512;                // token blocks whose pair ranges are kept in LDS
    __shared__ uint2 s_tp[TP_CAP];
    for (int i = threadIdx.x; i < min(steps, TP_CAP); i += C::NTHREADS) {
        const uint32_t *tp = tile_ptr + int64_t(kb_begin + i) * (nb_count + 1) + nb;
        s_tp[i] = make_uint2(tp[0], tp[1]);
    }
    __syncthreads();

    f32x16 acc[C::FM][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // One pipeline stage held in registers: the dY vectors and packed pairs of one token block.
    struct Stage {
        u32x4 a[C::A_VECS];
        uint32_t e[C::ENT];
        uint32_t lo, hi;                      // packed range of the step
    };
    constexpr int R = C::STAGES;
    Stage st[R];
    if (DROPIT_ABLATE & (1 | 16 | 32)) {      // keep the registers defined when loads are left out
        for (int r = 0; r < R; ++r) {
            st[r].lo = st[r].hi = 0;
            for (int i = 0; i < C::A_VECS; ++i) st[r].a[i] = u32x4{0, 0, 0, 0};
            for (int i = 0; i < C::ENT; ++i) st[r].e[i] = 0;
        }
    }

    // Branch-free on purpose: every load is issued unconditionally from a valid address, so
    // the compiler can count exactly how many newer loads may stay in flight when an older
    // stage is consumed.  Rows past the last token re-read the last token (their a^ rows are
    // zero, so they add nothing), columns past M re-read valid columns (those outputs are never
    // stored), pair slots past the end of the tile's range read into the slack the packed buffer
    // ends with (ignored at scatter time).
    // Addresses are a per-step scalar base plus a per-thread 32-bit offset computed once, so a
    // step issues its loads without any vector address arithmetic.
    uint32_t a_off[C::A_VECS], a_off_tail[C::A_VECS];   // byte offsets inside a token block
    const int kb_tail = int((ntok - 1) / BK);           // the (possibly partial) last token block
    const int rows_tail = int(ntok - int64_t(kb_tail) * BK);
#pragma unroll
    for (int i = 0; i < C::A_VECS; ++i) {
        const int vv = tid + i * NT;
        const int row = vv / (BM / 8), cv = vv % (BM / 8);
        const int m = min(m0 + cv * 8, M - 8);
        a_off[i] = uint32_t(row * M + m) * 2u;
        a_off_tail[i] = uint32_t(min(row, rows_tail - 1) * M + m) * 2u;
    }
    auto load_step = [&](Stage &st, int kb) {
        if (DROPIT_ABLATE & 1) return;
        const char *abase = reinterpret_cast<const char *>(dY) + int64_t(kb) * BK * M * 2;
        const bool tail = kb == kb_tail;
        if (!(DROPIT_ABLATE & 16)) {
#pragma unroll
            for (int i = 0; i < C::A_VECS; ++i)
                st.a[i] = *reinterpret_cast<const u32x4 *>(abase + (tail ? a_off_tail[i] : a_off[i]));
        }
        if (DROPIT_ABLATE & 32) return;
        // pair range of this (token block, column block): read from the LDS copy made in the
        // prologue -- a load from global memory here would put its full latency into every step
        const int rel = kb - kb_begin;
        if (rel < TP_CAP) {
            const uint2 r2 = s_tp[rel];
            st.lo = r2.x;
            st.hi = r2.y;
        } else {
            st.lo = tile_ptr[int64_t(kb) * (nb_count + 1) + nb];
            st.hi = tile_ptr[int64_t(kb) * (nb_count + 1) + nb + 1];
        }
        const uint32_t *pbase = packed + st.lo;
#pragma unroll
        for (int i = 0; i < C::ENT; ++i) st.e[i] = pbase[uint32_t(tid + i * NT)];
    };
    // What was scattered into a B buffer, kept until the buffer is cleared again.
    struct Dirty {
        uint32_t off[C::ENT];                 // LDS byte offsets (low 16 bits used)
        uint32_t lo, hi;
    };
    Dirty dirty[2];                           // by parity of the step
    dirty[0].lo = dirty[0].hi = dirty[1].lo = dirty[1].hi = 0;
#pragma unroll
    for (int i = 0; i < C::ENT; ++i) dirty[0].off[i] = dirty[1].off[i] = 0;

    uint32_t keep_alive = 0;                  // development only (ablation): keeps otherwise dead loads alive
    auto store_step = [&](const Stage &st, Dirty &d, int abuf, int bbuf) {
        if (DROPIT_ABLATE & 2) return;
        char *a = ldsA + abuf * C::A_BYTES;
#pragma unroll
        for (int i = 0; i < C::A_VECS; ++i) {
            const int vv = tid + i * NT;
            const int row = vv / (BM / 8), cv = vv % (BM / 8);
            *reinterpret_cast<u32x4 *>(a + row * C::PITCH_A + cv * 16) = st.a[i];
        }
        char *b = ldsB + bbuf * C::B_BYTES;
        // A masked LDS store costs a wavefront ~30 cycles even with no lane enabled, so whole
        // slots past the end of the range are skipped with a scalar branch.
        const uint32_t count = st.hi - st.lo;
#pragma unroll
        for (int i = 0; i < C::ENT; ++i) {
            const uint32_t p = st.e[i];
            d.off[i] = p;
            if (DROPIT_ABLATE & 64) {
                keep_alive ^= p;
            } else if (uint32_t(i * NT) < count) {
                if (uint32_t(tid + i * NT) < count) *reinterpret_cast<uint16_t *>(b + (p & 0xFFFFu)) = uint16_t(p >> 16);
            }
        }
        d.lo = st.lo;
        d.hi = st.hi;
        // pairs beyond the prefetch depth (dense tiles): fetched and scattered in place
        if (st.hi - st.lo > uint32_t(C::ENT * NT)) {
            for (uint32_t j = st.lo + tid + C::ENT * NT; j < st.hi; j += NT) {
                const uint32_t p = packed[j];
                *reinterpret_cast<uint16_t *>(b + (p & 0xFFFFu)) = uint16_t(p >> 16);
            }
        }
    };
    // Clears exactly the slots store_step filled (about a tenth of the tile) instead of
    // re-zeroing the whole buffer.
    auto clear_step = [&](const Dirty &d, int bbuf) {
        if (DROPIT_ABLATE & 4) return;
        char *b = ldsB + bbuf * C::B_BYTES;
        const uint32_t count = d.hi - d.lo;
#pragma unroll
        for (int i = 0; i < C::ENT; ++i)
            if (uint32_t(i * NT) < count) {
                if (uint32_t(tid + i * NT) < count) *reinterpret_cast<uint16_t *>(b + (d.off[i] & 0xFFFFu)) = uint16_t(0);
            }
        if (d.hi - d.lo > uint32_t(C::ENT * NT)) {
            for (uint32_t j = d.lo + tid + C::ENT * NT; j < d.hi; j += NT)
                *reinterpret_cast<uint16_t *>(b + (packed[j] & 0xFFFFu)) = uint16_t(0);
        }
    };
    auto zero_b = [&](int bbuf) {
        char *b = ldsB + bbuf * C::B_BYTES;
#pragma unroll
        for (int i = 0; i < C::B_ZERO; ++i)
            *reinterpret_cast<uint4 *>(b + (tid + i * NT) * 16) = make_uint4(0, 0, 0, 0);
    };
    auto compute = [&](int abuf, int bbuf) {
        if (DROPIT_ABLATE & 8) return;
        const char *a = ldsA + abuf * C::A_BYTES;
        const char *b = ldsB + bbuf * C::B_BYTES;
        const int g = lane >> 4, p16 = lane & 15;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[C::FM], bfv[C::FN];
#pragma unroll
            for (int i = 0; i < C::FM; ++i) {
                const int krow = kk * 16 + (g >> 1) * 8 + (p16 >> 2);
                const int mcol = wm * C::WM + i * 32 + (g & 1) * 16 + (p16 & 3) * 4;
                const char *p = a + krow * C::PITCH_A + mcol * 2;
                const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
                const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * C::PITCH_A));
                const s16x8 full = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
                af[i] = __builtin_bit_cast(bf16x8, full);
            }
#pragma unroll
            for (int j = 0; j < C::FN; ++j) {
                const int ncol = wn * C::WN + j * 32 + (lane & 31);
                const char *p = b + ncol * C::PITCH_B + (kk * 16 + (lane >> 5) * 8) * 2;
                bfv[j] = *reinterpret_cast<const bf16x8 *>(p);
            }
#pragma unroll
            for (int i = 0; i < C::FM; ++i)
#pragma unroll
                for (int j = 0; j < C::FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfv[j], acc[i][j], 0, 0, 0);
        }
    };

        // Software pipeline with R register stages: the block of token step t lives in stage
    // t % R from its global load until its LDS store, R - 1 steps later.  Iteration s:
    //   clear what step s-1 scattered (B buffer (s+2)%3), store step s+1 (registers -> A
    //   buffer (s+1)%2, B buffer (s+1)%3), reload that stage with step s+1+R, multiply
    //   step s, barrier.
    // The B buffer being read, the one being filled and the one being cleared are always
    // different; register stage indices are compile-time (the loop is unrolled R times),
    // LDS buffer indices are scalars.
#ifdef DROPIT_PHASE_CLOCK          // development only: where does a mover wavefront's step go
    unsigned long long pc_t[5] = {0, 0, 0, 0, 0}, pc_sum[4] = {0, 0, 0, 0};
#define PHASE_CLOCK(i)                                                        \
    do {                                                                      \
        pc_t[i] = wall_clock64();                                             \
        if ((i) > 0) pc_sum[(i) - 1] += pc_t[i] - pc_t[(i) - 1];              \
    } while (0)
#else
#define PHASE_CLOCK(i) do { } while (0)
#endif
    if (steps > 0) {
        // Loads and stores past the last block are clamped to it instead of branched
        // around: the loop body stays straight-line, so every wait counts exactly the
        // newer loads it may leave in flight.  The duplicates land in LDS buffers that
        // are never multiplied.
        const int kb_last = kb_end - 1;
        const int rounds = (steps + R - 1) / R * R;       // every wavefront passes 2 + rounds barriers
        if (C::PROD == 0) {
            zero_b(0);
            zero_b(1);
            zero_b(2);
#pragma unroll
            for (int r = 0; r < R; ++r) load_step(st[r], min(kb_begin + r, kb_last));
            __syncthreads();
            store_step(st[0], dirty[0], 0, 0);
            load_step(st[0], min(kb_begin + R, kb_last));
            __syncthreads();
            for (int s0 = 0; s0 < rounds; s0 += R) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int s = s0 + r;
                    clear_step(dirty[(r + 1) & 1], (s + 2) % 3);          // step s-1 (nothing on the first pass)
                    store_step(st[(r + 1) % R], dirty[(r + 1) & 1], (s + 1) & 1, (s + 1) % 3);
                    load_step(st[(r + 1) % R], min(kb_begin + s + 1 + R, kb_last));
                    if (s < steps) compute(s & 1, s % 3);
                    __syncthreads();
                }
            }
        } else if (is_mover) {
            // data-movement wavefronts: same schedule without the multiply (separate loop, so that
            // their registers and the accumulators of the other wavefronts are never live together)
            zero_b(0);
            zero_b(1);
            zero_b(2);
#pragma unroll
            for (int r = 0; r < R; ++r) load_step(st[r], min(kb_begin + r, kb_last));
            __syncthreads();
            store_step(st[0], dirty[0], 0, 0);
            load_step(st[0], min(kb_begin + R, kb_last));
            __syncthreads();
            for (int s0 = 0; s0 < rounds; s0 += R) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int s = s0 + r;
                    PHASE_CLOCK(0);
                    clear_step(dirty[(r + 1) & 1], (s + 2) % 3);
                    PHASE_CLOCK(1);
                    store_step(st[(r + 1) % R], dirty[(r + 1) & 1], (s + 1) & 1, (s + 1) % 3);
                    PHASE_CLOCK(2);
                    load_step(st[(r + 1) % R], min(kb_begin + s + 1 + R, kb_last));
                    PHASE_CLOCK(3);
                    __syncthreads();
                    PHASE_CLOCK(4);
                }
            }
        } else {
            // matrix wavefronts: LDS reads and MFMAs only
            __syncthreads();
            __syncthreads();
            for (int s = 0; s < rounds; ++s) {
                if (s < steps) compute(s & 1, s % 3);
                __syncthreads();
            }
        }
    }

#ifdef DROPIT_PHASE_CLOCK
    if (v == total / 2 && tid == 0 && is_mover) {
        float *o = out + int64_t(splits) * M * N;      // scratch past the partials (the test over-allocates)
        for (int i = 0; i < 4; ++i) o[i] = float(pc_sum[i]);
        o[4] = float(steps);
    }
#endif
    if ((DROPIT_ABLATE & 64) && keep_alive == 0x12345678u) out[0] = 1.f;
    // epilogue: acc[i][j][e] is row 8*(e/4) + 4*(lane/32) + e%4, column lane%32 of its 32x32 block
    if (!is_consumer) return;
    float *dst = out + int64_t(split) * M * N;
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * C::WM + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                const int n = nb * BN + wn * C::WN + j * 32 + (lane & 31);
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

#ifndef DROPIT_FC_CFG
#define DROPIT_FC_CFG 256, 256, 32, 2, 4, 3, 2, 4
#endif
using Cfg = FcCfg<DROPIT_FC_CFG>;

int tuned_splits(int tiles, int nkb)
{
    // one workgroup (8 matrix + 4 data-movement wavefronts) per compute unit: as many K-slices
    // as fill the 256 compute units without starting a second round
    int splits = 256 / tiles;
#ifdef DROPIT_TUNING
    if (const char *e = getenv("DROPIT_FC_SPLITS")) splits = atoi(e);
#endif
    if (splits > nkb) splits = nkb;
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    return splits;
}

}  // namespace

bool fc_mfma_supported(const FcProblem &p)
{
    // 16-byte dY vectors need c_out % 8 == 0; packed offsets and counters are 32-bit
    return p.cout % 8 == 0 && p.cin >= 1 && (p.cin + Cfg::BN - 1) / Cfg::BN <= 2 * THREADS;
}

FcPlan fc_mfma_plan(const FcProblem &p)
{
    FcPlan plan;
    plan.nkb = int((p.ntok + Cfg::BK - 1) / Cfg::BK);
    plan.nb_count = int((p.cin + Cfg::BN - 1) / Cfg::BN);
    plan.mb_count = int((p.cout + Cfg::BM - 1) / Cfg::BM);
    plan.splits = tuned_splits(plan.nb_count * plan.mb_count, plan.nkb);
    // slack: a step may read up to ENT * NTHREADS pair slots past the end of its range
    plan.packed_bytes = round_up(size_t(p.k > 0 ? p.k : 1) * 4 + size_t(Cfg::ENT) * Cfg::MOVERS * 4, 256);
    plan.tileptr_bytes = round_up(size_t(plan.nkb) * (plan.nb_count + 1) * 4, 256);
    plan.partial_bytes = plan.splits > 1 ? round_up(size_t(plan.splits) * p.cout * p.cin * 4, 256) : 0;
    return plan;
}

dropit_status fc_mfma_run(const FcProblem &p, const FcPlan &plan, const void *vals, const int32_t *idx,
                          const void *dY, float *dW, char *ws, hipStream_t stream)
{
    uint32_t *packed = reinterpret_cast<uint32_t *>(ws);
    uint32_t *tile_ptr = reinterpret_cast<uint32_t *>(ws + plan.packed_bytes);
    float *partial = reinterpret_cast<float *>(ws + plan.packed_bytes + plan.tileptr_bytes);

    trace_mark(stream);
    const size_t bucket_lds = size_t(2 * plan.nb_count + 2) * 4;
    fc_bucket_kernel<Cfg::BK, Cfg::BN, Cfg::PITCH_B><<<plan.nkb, THREADS, bucket_lds, stream>>>(
        static_cast<const uint16_t *>(vals), idx, p.k, p.ntok, int(p.cin), plan.nb_count, packed, tile_ptr);

    trace_mark(stream);
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(fc_mfma_kernel<Cfg>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES) != hipSuccess)
            return DROPIT_EHIP;
        attr_set = true;
    }
    const int total = plan.nb_count * plan.mb_count * plan.splits;
    const int grid = (total + 7) / 8 * 8;
    float *out = plan.splits > 1 ? partial : dW;
    fc_mfma_kernel<Cfg><<<grid, Cfg::NTHREADS, Cfg::LDS_BYTES, stream>>>(
        static_cast<const uint16_t *>(dY), packed, tile_ptr, p.k, p.ntok, int(p.cout), int(p.cin), plan.nb_count,
        plan.mb_count, plan.nkb, plan.splits, out);

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
