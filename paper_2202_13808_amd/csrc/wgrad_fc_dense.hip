// FC weight gradient dW = dY^T * R(a^) on the gfx950 matrix cores
// (Sec. 3.2: recover R(a^), then the ordinary backward of Eq. fc_backward_elem_save).
//
//   1. recover : one pass over the (value, index) pairs rebuilds R(a^) as a dense
//                bf16 matrix [tokens padded to BK][c_in padded to 8] in the workspace.
//                It is transient (one layer at a time), as in the method itself.
//   2. GEMM    : M = c_out (columns of dY), N = c_in (columns of R(a^)), reduction over
//                tokens.  Both operands have the token axis slow, so both tiles are
//                [k][m] row blocks.  They go from global memory straight into LDS
//                (16-byte direct loads, no registers in between), STAGES deep, and the
//                MFMA fragments come out through the LDS transpose read
//                (ds_read_b64_tr_b16).  A direct load writes 64 lanes x 16 bytes to
//                consecutive LDS bytes, so rows cannot be padded; bank conflicts of the
//                transpose reads are avoided by an XOR swizzle instead: the 64-byte unit
//                u of row r is kept at unit u ^ (r & 3).  The swizzle costs nothing at run
//                time: on the way in it only permutes which global address a lane asks
//                for, on the way out it is folded into per-lane constants.
//   3. reduce  : split-K partials are summed in ascending split order.
// Products are exact (bf16 x bf16 in fp32), accumulation is fp32 in a fixed order,
// so dW is bit-reproducible.
#include "common.hpp"
#include "wgrad_internal.hpp"
#include "dev_hooks.hpp"
#include <cstdlib>
#include <type_traits>

namespace dropit {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

#define DROPIT_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define DROPIT_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

#ifndef DROPIT_RECOVER_CFG
#define DROPIT_RECOVER_CFG 256, 16384
#endif
constexpr int recover_cfg[2] = {DROPIT_RECOVER_CFG};
constexpr int RECOVER_THREADS = recover_cfg[0];
// Dense elements one recover workgroup builds in LDS.  Small tiles keep many workgroups resident
// per compute unit, which hides the latency of each one's search; rows wider than that get the
// large tile (64 KB of LDS), rows wider than the large tile take the generic path.
constexpr int RECOVER_ELEMS = recover_cfg[1];
constexpr int RECOVER_ELEMS_MAX = 32768;

// ---------------------------------------------------------------------------
// Recover R(a^): workgroup b owns rows [b * rows_per_wg, ...) of the padded dense
// matrix.  Its pairs are one contiguous run of the index-sorted arrays (found by
// search), so the rows are assembled in LDS (zero fill, one 16-bit store per pair)
// and leave as full 16-byte stores: every byte of the dense matrix is written exactly
// once, no separate zero-fill pass.
// The pairs come through for_pairs_in_range: a window around the interpolated positions of the
// rows' first and last flat index, one round of loads, with the exact search as the fallback.
constexpr int RECOVER_WINDOW = 28;                    // window entries per thread, at most

// (The host uses fc_recover_stream_kernel instead when the window would be several times the pairs a
// workgroup needs.)
__global__ void __launch_bounds__(RECOVER_THREADS)
fc_recover_kernel(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx, int64_t k, int64_t ntok,
                  int64_t ntok_pad, int cin, int pitch, int rows_per_wg, int64_t margin, uint16_t *__restrict__ dense)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t tile[];   // [rows_per_wg][pitch]
    const int tid = threadIdx.x;
    const int64_t r0 = int64_t(blockIdx.x) * rows_per_wg;
    const int64_t r1 = min(r0 + rows_per_wg, ntok_pad);
    const int rows = int(r1 - r0);
    const int chunks = rows * (pitch / 8);                            // 16-byte units
    u32x4 *tile16 = reinterpret_cast<u32x4 *>(tile);
    const int64_t first = min(r0, ntok) * cin, last = min(r1, ntok) * cin;   // flat index range of these rows
    const uint32_t span = uint32_t(last - first);
    const int64_t numel = ntok * cin;
    auto place = [&](int32_t flat, uint32_t v) {
        const uint32_t rel = uint32_t(int64_t(flat) - first);
        if (rel >= span) return;                                      // not one of this workgroup's rows
        uint32_t pos = rel;
        if (pitch != cin) {
            const uint32_t row = rel / uint32_t(cin);
            pos = row * uint32_t(pitch) + (rel - row * uint32_t(cin));
        }
        tile[pos] = static_cast<uint16_t>(v);
    };

    for_pairs_in_range<RECOVER_THREADS, RECOVER_WINDOW>(vals, idx, k, numel, first, last, margin, place, [&] {
        for (int i = tid; i < chunks; i += RECOVER_THREADS) tile16[i] = u32x4{0, 0, 0, 0};
    });
    __syncthreads();
    u32x4 *out16 = reinterpret_cast<u32x4 *>(dense + r0 * pitch);
    for (int i = tid; i < chunks; i += RECOVER_THREADS) out16[i] = tile16[i];
}

// Recover from the row form of the cache (16-bit positions within rows + row offsets): the offsets say
// where a workgroup's rows start among the pairs, so there is nothing to guess or search, and a pair's
// place in its row is its 16-bit position as it stands.  Which row a pair belongs to follows from the
// offsets of the workgroup's rows, kept in LDS behind the tile.
__global__ void __launch_bounds__(RECOVER_THREADS)
fc_recover_rows_kernel(const uint16_t *__restrict__ vals, const uint16_t *__restrict__ col,
                       const int32_t *__restrict__ rowptr, int64_t k, int64_t ntok, int64_t ntok_pad, int cin,
                       int pitch, int rows_per_wg, uint16_t *__restrict__ dense)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t tile[];   // [rows_per_wg][pitch], then rows_per_wg + 1 offsets
    const int tid = threadIdx.x;
    const int64_t r0 = int64_t(blockIdx.x) * rows_per_wg;
    const int64_t r1 = min(r0 + rows_per_wg, ntok_pad);
    const int rows = int(r1 - r0);
    const int chunks = rows * (pitch / 8);                            // 16-byte units
    u32x4 *tile16 = reinterpret_cast<u32x4 *>(tile);
    int32_t *starts = reinterpret_cast<int32_t *>(tile + size_t(rows_per_wg) * pitch);
    const int64_t q0 = min(r0, ntok);
    const int real = int(min(r1, ntok) - q0);                         // rows that exist in the tensor (the rest is padding)
    for (int i = tid; i <= real; i += RECOVER_THREADS)
        starts[i] = int32_t(min<int64_t>(max<int64_t>(rowptr[q0 + i], 0), k));   // a malformed table must not read outside the pairs
    for (int i = tid; i < chunks; i += RECOVER_THREADS) tile16[i] = u32x4{0, 0, 0, 0};
    __syncthreads();
    if (real > 0) {
        const int64_t jb = starts[0], je = starts[real];
        constexpr int BATCH = 8;
        for (int64_t j0 = jb + tid; j0 < je; j0 += int64_t(BATCH) * RECOVER_THREADS) {
            uint32_t pc[BATCH], pv[BATCH];                            // full registers: 16-bit destinations get packed in pairs
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int64_t j = j0 + int64_t(u) * RECOVER_THREADS;
                if (j < je) {
                    pc[u] = col[j];
                    pv[u] = vals[j];
                }
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int64_t j = j0 + int64_t(u) * RECOVER_THREADS;
                if (j >= je) continue;
                int lo = 0, hi = real - 1;                            // the last row i with starts[i] <= j
                while (lo < hi) {
                    const int mid = (lo + hi + 1) >> 1;
                    if (int64_t(starts[mid]) <= j) lo = mid; else hi = mid - 1;
                }
                if (pc[u] < uint32_t(cin)) tile[size_t(lo) * pitch + pc[u]] = static_cast<uint16_t>(pv[u]);
            }
        }
    }
    __syncthreads();
    u32x4 *out16 = reinterpret_cast<u32x4 *>(dense + r0 * pitch);
    for (int i = tid; i < chunks; i += RECOVER_THREADS) out16[i] = tile16[i];
}

// Recover from the bit-mask form of the cache (one bit per element + the number of retained elements
// before every block of 1024): pure streaming.  A thread takes 8 consecutive elements, i.e. one byte of
// the mask; the retained ones among them are the next popcount(byte) values after the block's offset
// plus the bits set before the byte within the block (a prefix sum over the block's 128 threads).
// Needs pitch == c_in (c_in % 8 == 0): the recovered matrix then has the tensor's own flat layout.
__global__ void __launch_bounds__(256)
fc_recover_mask_kernel(const uint16_t *__restrict__ vals, const uint32_t *__restrict__ mask,
                       const int32_t *__restrict__ blockptr, int64_t k, int64_t numel, int64_t dense_elems,
                       uint16_t *__restrict__ dense)
{
    static_assert(DROPIT_MASK_BLOCK == 1024, "a block is the 8 x 128 elements of half a workgroup");
    __shared__ uint32_t first_wave_total[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t e0 = (int64_t(blockIdx.x) * 256 + tid) * 8;
    const int64_t block = e0 / DROPIT_MASK_BLOCK;
    const uint32_t byte = e0 < numel ? (mask[e0 >> 5] >> (e0 & 31)) & 0xFFu : 0u;
    const uint32_t c = __builtin_popcount(byte);
    const uint32_t inc = wave_inclusive_scan(c);
    if ((wave & 1) == 0 && lane == 63) first_wave_total[wave >> 1] = inc;
    __syncthreads();
    const uint32_t before = inc - c + ((wave & 1) ? first_wave_total[wave >> 1] : 0u);
    if (e0 >= dense_elems) return;
    const int64_t base = (e0 < numel ? int64_t(blockptr[block]) : 0) + before;
    uint32_t v[8];                                                    // full registers: 16-bit destinations get packed in pairs
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (uint32_t(i) < c && base + i >= 0 && base + i < k) ? vals[base + i] : 0u;
    uint32_t out[8];
    int taken = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const bool set = (byte >> e) & 1u;
        uint32_t val = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) val = (set && taken == i) ? v[i] : val;
        out[e] = val;
        taken += set ? 1 : 0;
    }
    const u32x4 o = {out[0] | (out[1] << 16), out[2] | (out[3] << 16), out[4] | (out[5] << 16), out[6] | (out[7] << 16)};
    *reinterpret_cast<u32x4 *>(dense + e0) = o;
}

// Recover for large k: the error of the interpolated guess grows with sqrt(k) (and with the ties at
// the threshold, which are all kept at the low-index end of the tensor), the pairs of a tile do not, so
// a window per tile would be mostly overlap -- and an exact search per tile costs ~500 scattered probes
// of the index array (measured: 15 of 33 us on a 38 M-element tensor).  Here a workgroup takes several
// consecutive tiles, searches once for the start of its first one, and then walks the pair arrays
// forward: a tile's pairs follow the previous tile's.  A tile is done when a batch of pairs ends with
// an index beyond it.
__global__ void __launch_bounds__(RECOVER_THREADS)
fc_recover_stream_kernel(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx, int64_t k, int64_t ntok,
                         int64_t ntok_pad, int cin, int pitch, int rows_per_tile, int tiles_per_wg,
                         uint16_t *__restrict__ dense)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t tile[];   // [rows_per_tile][pitch]
    constexpr int NWAVES = RECOVER_THREADS / WAVE;
    constexpr int BATCH = 8;
    __shared__ uint32_t wave_taken[2][NWAVES];
    const int tid = threadIdx.x;
    u32x4 *tile16 = reinterpret_cast<u32x4 *>(tile);
    const int64_t tiles = (ntok_pad + rows_per_tile - 1) / rows_per_tile;
    const int64_t t_begin = int64_t(blockIdx.x) * tiles_per_wg, t_end = min(t_begin + tiles_per_wg, tiles);

    int64_t pos, unused;
    {
        const int64_t start = min(t_begin * rows_per_tile, ntok) * cin;
        block_lower_bound2<RECOVER_THREADS>(idx, start, start, 0, k, 0, k, pos, unused);
    }
    int32_t pi[BATCH];
    uint32_t pv[BATCH];             // a full register each (16-bit destinations get packed and the loads serialised)
    auto load_batch = [&]() {       // the pairs at pos, pos + 1, ... : BATCH per thread, all loads in flight together
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const int64_t j = pos + int64_t(u) * RECOVER_THREADS + tid;
            if (j < k) {
                pi[u] = idx[j];
                pv[u] = vals[j];
            }
        }
    };
    load_batch();
    uint32_t parity = 0;
    for (int64_t t = t_begin; t < t_end; ++t) {
        const int64_t r0 = t * rows_per_tile, r1 = min(r0 + rows_per_tile, ntok_pad);
        const int chunks = int(r1 - r0) * (pitch / 8);                // 16-byte units
        const int64_t first = min(r0, ntok) * cin, last = min(r1, ntok) * cin;
        const uint32_t span = uint32_t(last - first);
        for (int i = tid; i < chunks; i += RECOVER_THREADS) tile16[i] = u32x4{0, 0, 0, 0};
        __syncthreads();
        for (;;) {
            uint32_t mine = 0;
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int64_t j = pos + int64_t(u) * RECOVER_THREADS + tid;
                if (j < k && int64_t(pi[u]) < last) {
                    ++mine;
                    const uint32_t rel = uint32_t(int64_t(pi[u]) - first);
                    if (rel < span) {                                 // always, for a sorted index array
                        uint32_t at = rel;
                        if (pitch != cin) {
                            const uint32_t row = rel / uint32_t(cin);
                            at = row * uint32_t(pitch) + (rel - row * uint32_t(cin));
                        }
                        tile[at] = static_cast<uint16_t>(pv[u]);
                    }
                }
            }
            mine = wave_sum(mine);
            if ((tid & (WAVE - 1)) == 0) wave_taken[parity][tid / WAVE] = mine;
            __syncthreads();                                           // also: this batch's scatter is complete
            uint32_t taken = 0;
#pragma unroll
            for (int w = 0; w < NWAVES; ++w) taken += wave_taken[parity][w];
            parity ^= 1u;
            const int64_t loaded = min<int64_t>(int64_t(BATCH) * RECOVER_THREADS, k - pos);
            pos += taken;
            // The next pairs are fetched right away: more of this tile if the batch lay wholly inside
            // it, else the start of the next tile, whose loads then overlap this tile's write-out.
            const bool more = int64_t(taken) == loaded && pos < k;
            if (more || t + 1 < t_end) load_batch();
            if (!more) break;
        }
        u32x4 *out16 = reinterpret_cast<u32x4 *>(dense + r0 * pitch);
        for (int i = tid; i < chunks; i += RECOVER_THREADS) out16[i] = tile16[i];
        __syncthreads();                                               // tile read before the next one is zeroed
    }
}

// ---------------------------------------------------------------------------
// GEMM: one workgroup = one BM x BN tile of dW over a contiguous range of token
// blocks (one of `splits` K-slices).  WAVES_M x WAVES_N wavefronts, each a
// (BM/WAVES_M) x (BN/WAVES_N) sub-tile built from 32x32x16 bf16 MFMAs.
template <int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int STAGES_, int WPE_, int EARLY_>
struct GemmCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, STAGES = STAGES_;
    // WPE: wavefronts per SIMD the register budget must allow (2 = one workgroup of 8 per compute unit, 4 = two).
    // EARLY: the first fragments of a token block are read during the previous block, so the matrix pipe never
    // waits for LDS after a barrier; costs one more stage of load latency cover.  Without it the reads follow
    // the barrier, which a second resident workgroup can hide.
    static constexpr int WPE = WPE_;
    static constexpr bool EARLY = EARLY_ != 0;
    static constexpr int NWAVES = WAVES_M * WAVES_N;
    static constexpr int WGS_PER_CU = WPE * 4 / NWAVES;
    static constexpr int NTHREADS = WAVE * NWAVES;
    static constexpr int ROW_A = BM * 2, ROW_B = BN * 2;            // bytes per LDS row (one token)
    static constexpr int A_BYTES = BK * ROW_A, B_BYTES = BK * ROW_B;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    static constexpr int A_LOADS = A_BYTES / 1024 / NWAVES;          // 1 KB direct loads per wavefront per step
    static constexpr int B_LOADS = B_BYTES / 1024 / NWAVES;
    static constexpr int LOADS = A_LOADS + B_LOADS;
    static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    static constexpr int FM = WM / 32, FN = WN / 32;
    static_assert(STAGES >= 2, "at least double buffering");
    static_assert(A_BYTES % (1024 * NWAVES) == 0 && B_BYTES % (1024 * NWAVES) == 0, "tiles must divide over the wavefronts");
    static_assert(ROW_A % 256 == 0 && ROW_B % 256 == 0, "the swizzle permutes the four 64-byte units of a 256-byte group");
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0, "MFMA 32x32x16 tiling");
    static_assert(WGS_PER_CU >= 1 && LDS_BYTES * WGS_PER_CU <= 160 * 1024, "LDS of one compute unit");
};

template <int N>
__device__ inline void wait_loads()          // until at most N of this wavefront's global loads are in flight
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int N>
__device__ inline void lgkm_wait()           // until at most N of this wavefront's LDS reads are in flight
{
    static_assert(N >= 0 && N <= 15, "4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}

__device__ inline void workgroup_barrier()
{
    asm volatile("s_barrier" ::: "memory");
}

// LDS transpose read: lane i of each 16-lane group receives column i of the 4 x 16 block of
// 16-bit elements whose lane p supplied row p / 4, columns 4 * (p % 4)..+3.  Result valid after lgkm_wait.
template <int OFFSET>
__device__ inline s16x4 tr_read(uint32_t lds_addr)
{
    static_assert(OFFSET >= 0 && OFFSET < 65536, "16-bit immediate");
    s16x4 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(lds_addr), "n"(OFFSET) : "memory");
    return r;
}

template <int I, int N, typename F>
__device__ inline void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// FUSED: the recover step R(a^) happens inside the product.  The B operand is not a dense matrix in memory:
// a prep kernel (fc_bucket_kernel) has put the pairs of every (token block, column block) tile next to each
// other as words  value << 16 | byte offset in the tile's LDS rows.  At step s the workgroup
//   - fetches the words of tile s + 4 straight into an LDS staging slot (direct loads, counted with the A loads),
//   - zero-fills the LDS rows of tile s + 3,
//   - places the words of tile s + 2 (one 16-bit LDS store each, at the swizzled address a direct load of the
//     dense operand would have filled),
// each a workgroup barrier of the main loop behind the one before it, and all of it issued behind the second
// half of a sub-step's MFMAs.  The zero-filled tensor exists only as these rows.
constexpr int FUSE_STAGE_WORDS = 1024;            // words of a tile staged per step (more than that: a slow path)
constexpr int FUSE_SLOTS = 4;                     // staging slots: tile t uses slot t % 4 (tiles s + 2 .. s + 4 are in flight at step s)
constexpr int FUSE_LDS_BYTES = FUSE_SLOTS * FUSE_STAGE_WORDS * 4 + 512 * 4;     // + a spare word per thread

template <typename C, bool FUSED, bool PP = false>
__global__ void __launch_bounds__(C::NTHREADS) __attribute__((amdgpu_waves_per_eu(C::WPE, C::WPE)))
fc_dense_kernel(const uint16_t *__restrict__ dY, const uint16_t *__restrict__ xd, int64_t ntok, int M, int N,
                int pitch, int nb_count, int mb_count, int nkb, int splits,
                float *__restrict__ out /* dW or partials [splits][M][N] */,
                const uint32_t *__restrict__ packed /* FUSED: the tiles' words */,
                const uint32_t *__restrict__ tile_ptr /* FUSED: [(nkb + 6) * nb_count + 1] first word of each tile, then slack */,
                uint32_t kpairs)
{
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK;
    static_assert(!FUSED || (C::NTHREADS == 512 && BN == 256 && BK == 32 && C::EARLY && C::STAGES == 4),
                  "the fused form is laid out for 512 threads, 32 x 256 B tiles, four stages, early reads");
    constexpr int PK_LOADS = FUSED ? FUSE_STAGE_WORDS / C::NTHREADS : 0;      // staging loads (64 words each) per wavefront per step
    constexpr int STEP_LOADS = FUSED ? C::A_LOADS + PK_LOADS : C::LOADS;      // global loads a wavefront issues per step
    extern __shared__ __attribute__((aligned(1024))) char lds[];     // [STAGES][A tile | B tile]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;

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
    const int m0 = mb * BM, n0 = nb * BN;

    // token blocks of this K-slice: an even partition of [0, nkb)
    const int kb_begin = int(int64_t(nkb) * split / splits);
    const int kb_end = int(int64_t(nkb) * (split + 1) / splits);
    const int steps = kb_end - kb_begin;

    f32x16 acc[C::FM][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // ---- global -> LDS -----------------------------------------------------------
    // Direct load q of a tile fills LDS bytes [q * 1024, (q + 1) * 1024): lane L lands at
    // byte o = q * 1024 + L * 16, i.e. row r = o / ROW, byte b' = o % ROW of that row, and
    // therefore asks for byte b = b' ^ ((r & 3) << 6) of global row r (the swizzle).
    // Every load is issued unconditionally from a valid address, so waits can count loads:
    // columns past M (or the padded c_in) re-read valid columns (those outputs are never
    // stored); rows past the last token re-read the last token (the matching rows of the
    // padded R(a^) are zero, so they add nothing that the last token does not add already).
    const int kb_tail = int((ntok - 1) / BK);           // the (possibly partial) last token block
    const int rows_tail = int(ntok - int64_t(kb_tail) * BK);
    uint32_t a_off[C::A_LOADS], a_off_tail[C::A_LOADS], b_off[C::B_LOADS];   // byte offsets inside a token block
#pragma unroll
    for (int i = 0; i < C::A_LOADS; ++i) {
        const int o = (wave * C::A_LOADS + i) * 1024 + lane * 16;
        const int r = o / C::ROW_A;
        const int b = (o % C::ROW_A) ^ ((r & 3) << 6);
        const int m = min(m0 + b / 2, M - 8);
        a_off[i] = uint32_t(r * M + m) * 2u;
        a_off_tail[i] = uint32_t(min(r, rows_tail - 1) * M + m) * 2u;
    }
#pragma unroll
    for (int i = 0; i < C::B_LOADS; ++i) {
        const int o = (wave * C::B_LOADS + i) * 1024 + lane * 16;
        const int r = o / C::ROW_B;
        const int b = (o % C::ROW_B) ^ ((r & 3) << 6);
        const int n = min(n0 + b / 2, pitch - 8);
        b_off[i] = FUSED ? 0u : uint32_t(r * pitch + n) * 2u;
    }
    // FUSED: first word of the tile whose words are being staged this step (tile s + 4), and the staging slot
    char *stg = lds + C::LDS_BYTES;                    // [FUSE_SLOTS][FUSE_STAGE_WORDS] words behind the stages
    uint32_t dma_start = 0;
    int dma_slot = 0;
    uint32_t pk_off[FUSE_STAGE_WORDS / C::NTHREADS];   // byte offset of this lane's word in staging load i
#pragma unroll
    for (int i = 0; i < FUSE_STAGE_WORDS / C::NTHREADS; ++i) pk_off[i] = uint32_t(i * C::NTHREADS + wave * 64 + lane) * 4u;
    // load number q (0 .. LOADS-1) of a step: the A loads first, then the B loads
    auto issue_load = [&](auto q_, int stage, int kb) {
        constexpr int q = decltype(q_)::value;
        if constexpr (q < C::A_LOADS) {
            const char *abase = reinterpret_cast<const char *>(dY) + int64_t(kb) * BK * M * 2;
            char *sa = lds + stage * C::STAGE_BYTES + wave * (C::A_LOADS * 1024);
            __builtin_amdgcn_global_load_lds(DROPIT_GPTR(abase + (kb == kb_tail ? a_off_tail[q] : a_off[q])),
                                             DROPIT_LPTR(sa + q * 1024), 16, 0, 0);
        } else if constexpr (FUSED) {
            // staging load i of the step: words [i * 512 + wave * 64, + 64) of the tile, one per lane (a direct
            // 4-byte load lands at the wave-uniform LDS base + lane * 4); unconditional: past the tile's words it
            // brings the next tiles', which are not placed
            constexpr int i = q - C::A_LOADS;
            const char *src = reinterpret_cast<const char *>(packed + dma_start);     // wavefront-uniform; the words are
            __builtin_amdgcn_global_load_lds(DROPIT_GPTR(src + pk_off[i]),            // followed by a slot's worth of slack
                                             DROPIT_LPTR(stg + dma_slot * (FUSE_STAGE_WORDS * 4) + (i * C::NTHREADS + wave * 64) * 4),
                                             4, 0, 0);
        } else {
            constexpr int i = q - C::A_LOADS;
            const char *bbase = reinterpret_cast<const char *>(xd) + int64_t(kb) * BK * pitch * 2;
            char *sb = lds + stage * C::STAGE_BYTES + C::A_BYTES + wave * (C::B_LOADS * 1024);
            __builtin_amdgcn_global_load_lds(DROPIT_GPTR(bbase + b_off[i]), DROPIT_LPTR(sb + i * 1024), 16, 0, 0);
        }
    };
    auto issue_loads = [&](int stage, int kb) {
        static_for<0, STEP_LOADS>([&](auto q_) { issue_load(q_, stage, kb); });
    };
    // ---- FUSED: the B tile of a step is zero-filled and the staged words placed, by hand-written LDS accesses
    // (the compiler would put vmcnt(0) in front of LDS accesses it knows about, see below) ----
    const uint32_t lds_base0 = uint32_t(size_t(DROPIT_LPTR(lds)));
    u32x4 zero4 = {0u, 0u, 0u, 0u};                    // kept in registers for the whole loop
    if constexpr (FUSED) asm volatile("" : "+v"(zero4));
    auto zero_b_half = [&](int stage, int half) {      // 16 KB: 2 x 16 bytes per thread
        const uint32_t a = lds_base0 + stage * C::STAGE_BYTES + C::A_BYTES + half * (C::NTHREADS * 16) + threadIdx.x * 16;
        asm volatile("ds_write_b128 %0, %1" ::"v"(a), "v"(zero4) : "memory");
    };
    auto zero_b = [&](int stage) {
        zero_b_half(stage, 0);
        zero_b_half(stage, 1);
    };
    uint32_t staged_w[FUSE_STAGE_WORDS / C::NTHREADS];             // this thread's words of the tile being placed
    auto read_staged = [&](int slot) {
        const uint32_t a = lds_base0 + C::LDS_BYTES + slot * (FUSE_STAGE_WORDS * 4) + threadIdx.x * 4;
#pragma unroll
        for (int i = 0; i < FUSE_STAGE_WORDS / C::NTHREADS; ++i)
            asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(staged_w[i]) : "v"(a), "n"(i * C::NTHREADS * 4) : "memory");
    };
    // a word is  value << 16 | byte offset in the tile's LDS rows  (row * 512 + 2 * swizzled column: 14 bits); the
    // store takes the value from the upper half of the register
    auto place_word = [&](uint32_t w, uint32_t b_base) {
        const uint32_t a = b_base + (w & 0x3fffu);
        asm volatile("ds_write_b16_d16_hi %0, %1" ::"v"(a), "v"(w) : "memory");
    };
    // staged word i of this thread, or -- past the tile's count -- a store to a spare location of the thread's own
    const uint32_t spare = lds_base0 + C::LDS_BYTES + FUSE_SLOTS * FUSE_STAGE_WORDS * 4 + threadIdx.x * 4;
    auto place_staged_one = [&](auto i_, int stage, uint32_t count) {
        constexpr int i = decltype(i_)::value;
        const uint32_t b_base = lds_base0 + stage * C::STAGE_BYTES + C::A_BYTES;
        asm volatile("" : "+v"(staged_w[i]));
        const bool valid = uint32_t(i * C::NTHREADS) + threadIdx.x < count;
        const uint32_t a = valid ? b_base + (staged_w[i] & 0x3fffu) : spare;
        asm volatile("ds_write_b16_d16_hi %0, %1" ::"v"(a), "v"(staged_w[i]) : "memory");
    };
    auto place_staged = [&](int stage, uint32_t count) {          // after the lgkm wait that follows read_staged
        static_for<0, FUSE_STAGE_WORDS / C::NTHREADS>([&](auto i_) { place_staged_one(i_, stage, count); });
    };
    // a tile of more words than the staging slot holds (values that bunch up): the rest straight from memory
    auto place_overflow = [&](int stage, uint32_t start, uint32_t count) {
        const uint32_t b_base = lds_base0 + stage * C::STAGE_BYTES + C::A_BYTES;
        for (uint32_t w = FUSE_STAGE_WORDS + threadIdx.x; w < count; w += C::NTHREADS) {
            const uint32_t word = packed[min(start + w, kpairs - 1)];
            place_word(word, b_base);
        }
    };
    // (the FUSED instantiation alone uses these)
    (void)zero_b; (void)read_staged; (void)place_staged; (void)place_overflow; (void)stg; (void)place_staged_one;

    // ---- LDS -> MFMA fragments -----------------------------------------------------
    // A 32x32x16 operand wants, in lane l, row (l % 32) and k = 8 * (l / 32) + 0..7.  One
    // transpose read hands lane i of a 16-lane group column i of a 4(k) x 16(m) block whose
    // lane p supplied row p / 4, columns 4 * (p % 4)..+3; two of them (k and k + 4) make an
    // operand.  The token row of a lane is 4-aligned plus p / 4, so its swizzle term is the
    // per-lane constant (p / 4) << 6.
    const int g = lane >> 4, p16 = lane & 15;
    const int krow = (g >> 1) * 8 + (p16 >> 2);
    const int sw = (p16 >> 2) << 6;
    uint32_t a_frag[C::FM], b_frag[C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
        a_frag[i] = krow * C::ROW_A + (((wm * C::WM + i * 32 + (g & 1) * 16 + (p16 & 3) * 4) * 2) ^ sw);
#pragma unroll
    for (int j = 0; j < C::FN; ++j)
        b_frag[j] = C::A_BYTES + krow * C::ROW_B + (((wn * C::WN + j * 32 + (g & 1) * 16 + (p16 & 3) * 4) * 2) ^ sw);

    // The fragment reads, the waits and the barrier are written as asm on purpose.  The compiler
    // cannot tell which direct load fills which LDS bytes, so it would drain every load in flight
    // (vmcnt(0)) in front of each LDS read and barrier it knows about, which serialises the pipeline.
    // Here the dependency is kept by hand: wait_loads<>() + barrier before a stage is read, and
    // lgkm_wait<>() before the registers of a batch of reads are used (the empty "+v" asm statements
    // tie the MFMA operands to that wait).
    constexpr int KK = BK / 16;                        // 16-token sub-steps (one MFMA depth) per token block
    constexpr int NM = C::FM * C::FN;                  // MFMAs per sub-step
    constexpr int SET_READS = 2 * (C::FM + C::FN);     // LDS reads per sub-step
    constexpr int READS_PER_MFMA = (SET_READS + NM / 2 - 1) / (NM / 2);   // all reads go out with the first half
    static_assert(KK % 2 == 0, "fragment sets alternate per sub-step and must line up across token blocks");
    static_assert(NM >= 2, "the reads of a sub-step go out with the first half of the previous one's MFMAs");
    const uint32_t lds_base = lds_base0;
    s16x4 fa[2][C::FM][2], fb[2][C::FN][2];            // two fragment sets: one multiplying, one being read
    // read number r (0 .. SET_READS-1) of sub-step kk of the stage at `stage_base`, into fragment set `set`
    auto issue_read = [&](auto set_, auto kk_, auto r_, uint32_t stage_base) {
        constexpr int set = decltype(set_)::value, kk = decltype(kk_)::value, r = decltype(r_)::value;
        if constexpr (r < 2 * C::FM) {
            constexpr int i = r / 2, h = r % 2;
            fa[set][i][h] = tr_read<(kk * 16 + h * 4) * C::ROW_A>(stage_base + a_frag[i]);
        } else {
            constexpr int j = (r - 2 * C::FM) / 2, h = r % 2;
            fb[set][j][h] = tr_read<(kk * 16 + h * 4) * C::ROW_B>(stage_base + b_frag[j]);
        }
    };
    // One sub-step: the MFMAs of fragment set `set`, with the LDS reads of the next sub-step (into
    // the other set) issued between the first half of them, and this sub-step's share of the step's
    // global loads spread evenly between all of them.  A wavefront issues in order, and the two
    // wavefronts of a SIMD run in lockstep between barriers, so anything not tucked between MFMAs
    // would leave the matrix pipe idle in both at once; and a burst of loads would wait for the
    // address unit, which all eight wavefronts feed at the same time.
    static_assert(STEP_LOADS <= KK * NM, "at most one global load rides behind each MFMA");
    // FUSED, per step s (fz_*: set at the top of the step): sub-step 0 zero-fills the B rows of tile s + 3 and reads
    // this thread's staged words of tile s + 2; sub-step 1 places them.
    int fz_zero_stage = 0, fz_place_stage = 0, fz_place_t = 0, fz_decode_t = 0;
    uint32_t fz_place_count = 0, fz_raw_lo = 0, fz_raw_hi = 0, fz_next_start = 0, fz_next_count = 0;
    const int steps_f = steps;
    // table entry of the slice's tile t: fz_table[t * nb_count] (first word) and the entry after it (end); the table
    // is followed by six token blocks' worth of slack, so entries of tiles past the slice can be fetched (and ignored)
    const uint32_t *fz_table = FUSED ? tile_ptr + (int64_t(kb_begin) * nb_count + nb) : nullptr;
    auto tile_decode = [&](int t, uint32_t raw_lo, uint32_t raw_hi, uint32_t &start, uint32_t &count) {
        start = min(raw_lo, kpairs);
        const uint32_t end = min(raw_hi, kpairs);
        count = t < steps_f ? min(end - start, uint32_t(BK * BN)) : 0u;   // (a tile has at most BK * BN words whatever the table says)
    };
    (void)tile_decode;                                 // (used by the FUSED instantiation only)
    auto substep = [&](auto kk_, auto next_kk_, auto read_next_, uint32_t next_base, int load_stage, int load_kb) {
        constexpr int kk = decltype(kk_)::value, set = kk % 2;
        constexpr bool read_next = decltype(read_next_)::value;
        lgkm_wait<0>();                                // the reads of this set were issued one sub-step ago
        if constexpr (FUSED && kk == 1) {
            tile_decode(fz_decode_t, fz_raw_lo, fz_raw_hi, fz_next_start, fz_next_count);   // (fetched at the top of the step)
            if (fz_place_count > uint32_t(FUSE_STAGE_WORDS))
                place_overflow(fz_place_stage, min(fz_table[int64_t(fz_place_t) * nb_count], kpairs), fz_place_count);
        }
        bf16x8 af[C::FM], bfv[C::FN];
#pragma unroll
        for (int i = 0; i < C::FM; ++i) {
            asm volatile("" : "+v"(fa[set][i][0]), "+v"(fa[set][i][1]));
            af[i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(fa[set][i][0], fa[set][i][1], 0, 1, 2, 3, 4, 5, 6, 7));
        }
#pragma unroll
        for (int j = 0; j < C::FN; ++j) {
            asm volatile("" : "+v"(fb[set][j][0]), "+v"(fb[set][j][1]));
            bfv[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(fb[set][j][0], fb[set][j][1], 0, 1, 2, 3, 4, 5, 6, 7));
        }
        static_for<0, NM>([&](auto m_) {
            constexpr int m = decltype(m_)::value, i = m / C::FN, j = m % C::FN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfv[j], acc[i][j], 0, 0, 0);
            static_for<m * READS_PER_MFMA, (m + 1) * READS_PER_MFMA>([&](auto r_) {
                if constexpr (read_next && decltype(r_)::value < SET_READS)
                    issue_read(std::integral_constant<int, 1 - set>{}, next_kk_, r_, next_base);
            });
            // FUSED: the second half of the MFMAs, which has no reads behind it, carries the zero fill and the staged
            // reads (sub-step 0) and the placement (sub-step 1)
            if constexpr (FUSED && kk == 0) {
                if constexpr (m == NM / 2 || m == NM / 2 + 1) zero_b_half(fz_zero_stage, m - NM / 2);
                if constexpr (m == NM / 2 + 2) read_staged(fz_place_stage);      // (tile t is staged in slot t % 4 = its stage)
            }
            if constexpr (FUSED && kk == 1 && m >= NM / 2 && m < NM / 2 + FUSE_STAGE_WORDS / C::NTHREADS)
                place_staged_one(std::integral_constant<int, m - NM / 2>{}, fz_place_stage, fz_place_count);
            constexpr int g = kk * NM + m;             // MFMA number within the step
            static_for<0, STEP_LOADS>([&](auto q_) {   // load q rides behind MFMA (q + 1) * MFMAs / LOADS - 1
                constexpr int q = decltype(q_)::value;
                if constexpr (g == (q + 1) * KK * NM / STEP_LOADS - 1) issue_load(q_, load_stage, load_kb);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // ---- pipeline --------------------------------------------------------------------
    // Token block t of the split lives in stage t % STAGES; its loads are issued D = STAGES - 1
    // steps ahead.  LDS reads run one sub-step ahead of the MFMAs.
    // EARLY: the fragments of (step s + 1, sub-step 0) are read during step s, so a stage must be
    // complete one step before it is multiplied.  Iteration s: wait until this wavefront's loads
    // of step s + 1 have landed (the D - 2 newer steps may stay in flight), barrier (now
    // everybody's have, and everybody is done reading step s - 1), then the sub-steps, which
    // between them also refill the stage step s - 1 used with step s + D.
    // Otherwise: wait for step s itself (D - 1 newer steps in flight), barrier, read sub-step 0,
    // then the sub-steps; the exposed read is for a second resident workgroup to hide.
    // Loads past the last block are clamped to it instead of branched around, so the in-flight
    // count is the same in every iteration; they land in stages that are never multiplied.
    if constexpr (PP) {
        // Alternating wavefronts.  The two wavefronts of a SIMD (w and w + 4: a workgroup's wavefronts are dealt to the
        // four SIMDs in turn) never want the same unit: while one multiplies a token block (its 16 MFMAs back to back,
        // nothing between them), the other reads the fragments of its next block from LDS and issues its share of the
        // global loads; a workgroup barrier ends every phase and the roles swap.  The second group enters the
        // sequence one barrier late, which is all it takes to put it a phase behind the first, and leaves out the
        // last barrier in exchange, so both groups execute the same number of barriers.
        //   phase        2s      2s+1    2s+2           (s: token block; M = read its fragments + issue loads, C = multiply)
        //   waves 0-3    M(s)    C(s)    M(s+1)
        //   waves 4-7    C(s-1)  M(s)    C(s)
        // The stage of block s is read in phases 2s and 2s+1; every M ends with the wait for its own reads, so after
        // the barrier of phase 2s+1 nobody reads it any more.  The loads of block s + 3 go out in M(s) (phases 2s and
        // 2s+1), into the stage block s - 1 left in phase 2s - 1.  At the end of M(s) a wavefront also waits until at
        // most the loads it issued in M(s - 1) and M(s) are in flight: block s + 1 (loaded in M(s - 2)) is then
        // complete in every wavefront before phase 2s + 2 reads it.
        // Measured against the loop below (same tile, both wavefronts of a SIMD in lockstep, reads and loads tucked
        // between the MFMAs): 5 - 7 % less time per launch.  Variants that were slower than this one: a phase per
        // 16-token sub-step (twice the barriers); the second sub-step's reads, or the loads, inside or at either
        // end of the multiplying phase (anything a multiplying wavefront issues besides MFMAs delays them); no wait
        // for the reads before the barrier; one barrier per block with the groups half a block apart.
        static_assert(!FUSED && C::STAGES >= 4 && BK == 32 && C::NWAVES == 8 && C::LOADS == 4, "laid out for the wide tile");
        constexpr int D = C::STAGES - 1;               // blocks a load runs ahead of the block being read
        if (steps > 0) {
            const int kb_last = kb_end - 1;
            const bool late = wave >= C::NWAVES / 2;
#pragma unroll
            for (int d = 0; d < D; ++d) issue_loads(d, min(kb_begin + d, kb_last));
            wait_loads<(D - 1) * C::LOADS>();          // block 0 is there; the loop's own waits cover the others
            workgroup_barrier();
            if (late) workgroup_barrier();
            int stage = 0, fill = D;
            for (int s = 0; s < steps; ++s) {
                const uint32_t cur_base = lds_base + stage * C::STAGE_BYTES;
                const int load_kb = min(kb_begin + s + D, kb_last);
                // M: the fragments of both sub-steps of the block, this wavefront's four loads between them (a load
                // takes tens of cycles to issue: behind the reads that time is covered by their latency, in front
                // of them or next to the MFMAs it is not)
                static_for<0, 2>([&](auto kk_) {
                    constexpr int kk = decltype(kk_)::value;
                    static_for<0, SET_READS>([&](auto r_) { issue_read(kk_, kk_, r_, cur_base); });
                    issue_load(std::integral_constant<int, 2 * kk>{}, fill, load_kb);
                    issue_load(std::integral_constant<int, 2 * kk + 1>{}, fill, load_kb);
                });
                lgkm_wait<0>();
                wait_loads<(D - 1) * C::LOADS>();
                __builtin_amdgcn_sched_barrier(0);
                workgroup_barrier();
                __builtin_amdgcn_sched_barrier(0);
                // C: the block's MFMAs, back to back, nothing between them
                static_for<0, 2>([&](auto kk_) {
                    constexpr int kk = decltype(kk_)::value;
                    bf16x8 af[C::FM], bfv[C::FN];
#pragma unroll
                    for (int i = 0; i < C::FM; ++i) {
                        asm volatile("" : "+v"(fa[kk][i][0]), "+v"(fa[kk][i][1]));
                        af[i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(fa[kk][i][0], fa[kk][i][1], 0, 1, 2, 3, 4, 5, 6, 7));
                    }
#pragma unroll
                    for (int j = 0; j < C::FN; ++j) {
                        asm volatile("" : "+v"(fb[kk][j][0]), "+v"(fb[kk][j][1]));
                        bfv[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(fb[kk][j][0], fb[kk][j][1], 0, 1, 2, 3, 4, 5, 6, 7));
                    }
                    static_for<0, NM>([&](auto m_) {
                        constexpr int m = decltype(m_)::value, i = m / C::FN, j = m % C::FN;
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfv[j], acc[i][j], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    });
                });
                if (!(late && s + 1 == steps)) workgroup_barrier();
                __builtin_amdgcn_sched_barrier(0);
                stage = stage + 1 == C::STAGES ? 0 : stage + 1;
                fill = fill + 1 == C::STAGES ? 0 : fill + 1;
            }
            wait_loads<0>();
            lgkm_wait<0>();
        }
    } else
    if (steps > 0) {
        constexpr int D = C::STAGES - 1;
        constexpr int AHEAD = C::EARLY ? 1 : 0;        // how many steps before its own a stage must be complete
        static_assert(D >= 1 + AHEAD, "stages: one being multiplied, one per step of load latency, one more if read early");
        const int kb_last = kb_end - 1;
        // FUSED: counts of the tiles s + 2 .. s + 4 (placed two steps after they are staged) and where tile s + 4 starts
        uint32_t c2 = 0, c3 = 0, c4 = 0, st4 = 0;
        const uint32_t *fz_tp = fz_table;
        if constexpr (FUSED) {
            // before the first step: tiles 0 .. 3 staged, stages 0 .. 2 zero-filled, tiles 0 and 1 placed -- the table
            // entries, the A tiles of the first three steps and the staged words are all requested before the first wait
            uint32_t lo[5], hi[5], st[5], ct[5];
#pragma unroll
            for (int t = 0; t < 5; ++t) {
                lo[t] = fz_table[int64_t(t) * nb_count];
                hi[t] = fz_table[int64_t(t) * nb_count + 1];
            }
#pragma unroll
            for (int d = 0; d < D; ++d)
                static_for<0, C::A_LOADS>([&](auto q_) { issue_load(q_, d, min(kb_begin + d, kb_last)); });
#pragma unroll
            for (int t = 0; t < 5; ++t) tile_decode(t, lo[t], hi[t], st[t], ct[t]);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                dma_start = st[t];
                dma_slot = t;
                static_for<C::A_LOADS, STEP_LOADS>([&](auto q_) { issue_load(q_, 0, 0); });
            }
            zero_b(0);
            zero_b(1);
            zero_b(2);
            wait_loads<0>();
            lgkm_wait<0>();
            workgroup_barrier();
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                read_staged(t);
                lgkm_wait<0>();
                place_staged(t, ct[t]);
                if (ct[t] > uint32_t(FUSE_STAGE_WORDS)) place_overflow(t, st[t], ct[t]);
            }
            lgkm_wait<0>();
            c2 = ct[2];
            c3 = ct[3];
            c4 = ct[4];
            st4 = st[4];
            fz_tp = fz_table + int64_t(4) * nb_count;
        } else {
#pragma unroll
            for (int d = 0; d < D; ++d) issue_loads(d, min(kb_begin + d, kb_last));
        }
        if constexpr (C::EARLY) {
            if constexpr (FUSED) wait_loads<0>();
            else wait_loads<(D - 1) * C::LOADS>();
            workgroup_barrier();
            static_for<0, SET_READS>([&](auto r_) {
                issue_read(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, r_, lds_base);
            });
        }
        int stage = 0, fill = D;                       // s % STAGES and (s + D) % STAGES
        static_assert(!FUSED || (FUSE_SLOTS == 4 && C::STAGES == 4), "tile t is staged in slot t % 4, which is also its stage");
        for (int s = 0; s < steps; ++s) {
            const int next = stage + 1 == C::STAGES ? 0 : stage + 1;
            wait_loads<(D - 1 - AHEAD) * STEP_LOADS>();
            if constexpr (FUSED) lgkm_wait<0>();           // this wavefront's zero fill and placed words are in LDS
            workgroup_barrier();
            if constexpr (FUSED) {
                fz_tp += nb_count;                         // tile s + 5: decoded during the step, staged in the next one
                fz_raw_lo = fz_tp[0];
                fz_raw_hi = fz_tp[1];
                fz_decode_t = s + 5;
                fz_zero_stage = (stage + 3) % C::STAGES;
                fz_place_stage = (stage + 2) % C::STAGES;
                fz_place_t = s + 2;
                fz_place_count = c2;
                dma_start = st4;
                dma_slot = stage;
            }
            const uint32_t cur_base = lds_base + stage * C::STAGE_BYTES;
            const uint32_t next_base = lds_base + next * C::STAGE_BYTES;
            const int load_kb = min(kb_begin + s + D, kb_last);
            if constexpr (!C::EARLY)
                static_for<0, SET_READS>([&](auto r_) {
                    issue_read(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, r_, cur_base);
                });
            static_for<0, KK>([&](auto kk_) {
                constexpr int kk = decltype(kk_)::value;
                if constexpr (kk + 1 < KK)
                    substep(kk_, std::integral_constant<int, kk + 1>{}, std::true_type{}, cur_base, fill, load_kb);
                else
                    substep(kk_, std::integral_constant<int, 0>{}, std::integral_constant<bool, C::EARLY>{}, next_base,
                            fill, load_kb);
            });
            stage = next;
            fill = fill + 1 == C::STAGES ? 0 : fill + 1;
            if constexpr (FUSED) {
                c2 = c3;
                c3 = c4;
                c4 = fz_next_count;
                st4 = fz_next_start;
            }
        }
        wait_loads<0>();                               // nothing may still be writing LDS
        lgkm_wait<0>();                                // or registers when the wavefront goes on
    }

    // epilogue: acc[i][j][e] is row 8*(e/4) + 4*(lane/32) + e%4, column lane%32 of its 32x32 block.
    if (splits == 1) {                                  // straight into dW, row-major
#pragma unroll
        for (int i = 0; i < C::FM; ++i)
#pragma unroll
            for (int j = 0; j < C::FN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = m0 + wm * C::WM + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
                    const int n = n0 + wn * C::WN + j * 32 + (lane & 31);
                    if (m < M && n < N) out[int64_t(m) * N + n] = acc[i][j][e];
                }
    } else {
        // A K-slice's partial tile is written in the accumulator's own order instead: [i][j][e/4]
        // [thread] x 4 floats, so every store is 16 bytes per lane and 1 KB contiguous per wavefront.
        // The seven-fold partial traffic then moves in full lines, and the one pass that adds the
        // slices (splitk_sum_kernel) does the transposition into row-major dW.
        f32x4 *dst = reinterpret_cast<f32x4 *>(out) +
                     (int64_t(split) * (nb_count * mb_count) + (mb * nb_count + nb)) * (BM * BN / 4) + threadIdx.x;
#pragma unroll
        for (int i = 0; i < C::FM; ++i)
#pragma unroll
            for (int j = 0; j < C::FN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 v4 = {acc[i][j][q * 4], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
                    dst[((i * C::FN + j) * 4 + q) * C::NTHREADS] = v4;
                }
    }
}

// Sums the split-K partials in ascending split order, dW = ((p0 + p1) + p2) + ..., and moves
// them from the accumulator order the GEMM wrote (see its epilogue) to row-major dW.
// One thread per 4 accumulator floats: rows m .. m+3 of one column.
template <typename C>
__global__ void __launch_bounds__(256)
splitk_sum_kernel(const f32x4 *__restrict__ partial, int splits, int M, int N, int nb_count, int mb_count,
                  float *__restrict__ dW)
{
    constexpr int TILE4 = C::BM * C::BN / 4;            // float4 groups per tile
    const int64_t tiles = int64_t(nb_count) * mb_count;
    const int64_t total = tiles * TILE4;
    for (int64_t g = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; g < total; g += int64_t(gridDim.x) * blockDim.x) {
        // eight slices at a time: all their loads are issued before the first add
        f32x4 s = partial[g];
        for (int p0 = 1; p0 < splits; p0 += 8) {
            f32x4 part[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (p0 + u < splits) part[u] = partial[(p0 + u) * total + g];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (p0 + u < splits) s += part[u];
        }
        const int tile = int(g / TILE4), r = int(g % TILE4);
        const int tid = r % C::NTHREADS, slot = r / C::NTHREADS;   // slot = (i * FN + j) * 4 + q
        const int q = slot & 3, j = (slot >> 2) % C::FN, i = (slot >> 2) / C::FN;
        const int lane = tid & 63, wave = tid >> 6;
        const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
        const int mb = tile / nb_count, nb = tile % nb_count;
        const int m = mb * C::BM + wm * C::WM + i * 32 + q * 8 + (lane >> 5) * 4;
        const int n = nb * C::BN + wn * C::WN + j * 32 + (lane & 31);
        if (n < N) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (m + e < M) dW[int64_t(m + e) * N + n] = s[e];
        }
    }
}

// The same sum for many slices of few tiles (a result of one or two tiles is cut into up to 256 slices, one
// per compute unit): 16 threads share an output group, thread p of them adds the slices p, p + 16, ... in
// ascending order, and the 16 sums are added in ascending p through LDS -- a fixed order again, with 16
// times the loads in flight (one thread per group took 20 us for 256 slices of a single tile).
template <typename C>
__global__ void __launch_bounds__(256)
splitk_sum_wide_kernel(const f32x4 *__restrict__ partial, int splits, int M, int N, int nb_count, int mb_count,
                       float *__restrict__ dW)
{
    constexpr int PARTS = 16, GPB = 16;                // slice lanes per group, groups per workgroup
    constexpr int TILE4 = C::BM * C::BN / 4;
    __shared__ f32x4 red[PARTS][GPB];
    const int64_t total = int64_t(nb_count) * mb_count * TILE4;
    const int part = threadIdx.x / GPB, gi = threadIdx.x % GPB;
    const int64_t g = int64_t(blockIdx.x) * GPB + gi;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (g < total) {
        for (int p0 = part; p0 < splits; p0 += 4 * PARTS) {
            f32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (p0 + u * PARTS < splits) v[u] = partial[(p0 + u * PARTS) * total + g];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (p0 + u * PARTS < splits) s += v[u];
        }
    }
    red[part][gi] = s;
    __syncthreads();
    if (part != 0 || g >= total) return;
#pragma unroll
    for (int q = 1; q < PARTS; ++q) s += red[q][gi];
    const int tile = int(g / TILE4), r = int(g % TILE4);
    const int tid = r % C::NTHREADS, slot = r / C::NTHREADS;   // slot = (i * FN + j) * 4 + q
    const int q = slot & 3, j = (slot >> 2) % C::FN, i = (slot >> 2) / C::FN;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
    const int mb = tile / nb_count, nb = tile % nb_count;
    const int m = mb * C::BM + wm * C::WM + i * 32 + q * 8 + (lane >> 5) * 4;
    const int n = nb * C::BN + wn * C::WN + j * 32 + (lane & 31);
    if (n < N) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (m + e < M) dW[int64_t(m + e) * N + n] = s[e];
    }
}

// Prep of the in-LDS form: the pairs of token block kb (pairs [kb_ptr[kb], kb_ptr[kb + 1]), in index order, that
// is by row and then by column) are regrouped by column block of 256 as the words the product consumes, and the
// table of where each (token block, column block) tile starts is written.  In index order the pairs of one
// (row, column block) are a run; the regrouping moves whole runs: run (r, b) goes behind the runs (r' < r, b) of
// its column block, which go behind all of the column blocks before b.  Run starts are found like row starts
// (every pair is compared with its predecessor), so no counter is contended and the order of the words is fixed.
// One workgroup per token block.
constexpr int BUCKET_THREADS = 512;
constexpr int BUCKET_MAX_NB = RECOVER_ELEMS_MAX / 256;
__global__ void __launch_bounds__(BUCKET_THREADS)
fc_bucket_kernel(const uint16_t *__restrict__ vals, const int32_t *__restrict__ idx, int64_t k, uint32_t cin,
                 int nb_count, int nkb, const uint32_t *__restrict__ kb_ptr, uint32_t *__restrict__ packed,
                 uint32_t *__restrict__ tile_ptr)
{
    extern __shared__ uint32_t bucket_lds[];
    const int runs = 32 * nb_count;
    uint32_t *run_in = bucket_lds;                     // [runs + 1] first pair of run (r, b), key r * nb_count + b
    uint32_t *run_out = bucket_lds + runs + 1;         // [runs]     where its first word goes
    uint32_t *total = run_out + runs;                  // [nb_count] pairs of the column block, then its first word
    const int kb = blockIdx.x;
    const uint32_t lo = kb_ptr[kb], hi = kb_ptr[kb + 1];
    const uint32_t first = uint32_t(kb) * 32u * cin;      // flat index of the block's first element (below 2^31)
    const float inv = 1.0f / float(cin);
    // row and column of an element of the block: rel < 32 * cin, so the quotient estimate is off by one at most
    auto split = [&](uint32_t rel, uint32_t &r, uint32_t &col) {
        r = min(uint32_t(float(rel) * inv), 31u);
        int32_t c = int32_t(rel - r * cin);
        if (c < 0) { r -= 1; c += int32_t(cin); }
        if (c >= int32_t(cin)) { r += 1; c -= int32_t(cin); }
        r &= 31u;
        col = uint32_t(c);
    };
    auto key_of = [&](uint32_t flat) {
        uint32_t r, col;
        split(flat - first, r, col);
        return int(r) * nb_count + int(min(col >> 8, uint32_t(nb_count - 1)));
    };
    constexpr int U = 4;                               // pairs per thread in flight: all their loads go out first
    for (uint32_t j0 = lo + threadIdx.x; j0 <= hi; j0 += U * BUCKET_THREADS) {
        uint32_t cur[U], prev[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t j = j0 + u * BUCKET_THREADS;
            cur[u] = j < hi ? uint32_t(idx[j]) : first;
            prev[u] = j > lo && j <= hi ? uint32_t(idx[j - 1]) : first;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t j = j0 + u * BUCKET_THREADS;
            if (j > hi) break;
            const int before = j == lo ? -1 : key_of(prev[u]);
            const int here = j == hi ? runs : key_of(cur[u]);
            for (int q = before + 1; q <= here; ++q) run_in[q] = j;
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < nb_count; b += BUCKET_THREADS) {
        uint32_t acc = 0;
        for (int r = 0; r < 32; ++r) {
            run_out[r * nb_count + b] = acc;
            acc += run_in[r * nb_count + b + 1] - run_in[r * nb_count + b];
        }
        total[b] = acc;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = lo;
        for (int b = 0; b < nb_count; ++b) {
            const uint32_t n = total[b];
            total[b] = run;
            tile_ptr[int64_t(kb) * nb_count + b] = run;
            run += n;
        }
        if (kb == nkb - 1) tile_ptr[int64_t(nkb) * nb_count] = uint32_t(k);
    }
    __syncthreads();
    for (uint32_t j0 = lo + threadIdx.x; j0 < hi; j0 += U * BUCKET_THREADS) {
        uint32_t cur[U], val[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t j = j0 + u * BUCKET_THREADS;
            cur[u] = j < hi ? uint32_t(idx[j]) : first;
            val[u] = j < hi ? uint32_t(vals[j]) : 0u;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t j = j0 + u * BUCKET_THREADS;
            if (j >= hi) break;
            uint32_t r, col;
            split(cur[u] - first, r, col);
            const int b = int(min(col >> 8, uint32_t(nb_count - 1)));
            const int key = int(r) * nb_count + b;
            const uint32_t at = min(max(total[b] + run_out[key] + (j - run_in[key]), lo), hi - 1);   // (inside the block whatever idx holds)
            packed[at] = val[u] << 16 | (r << 8 | ((col & 255u) ^ ((r & 3u) << 5))) << 1;
        }
    }
}

#ifndef DROPIT_GEMM_CFG
#define DROPIT_GEMM_CFG 256, 256, 32, 4, 2, 4, 2, 1
#endif
// For layers with at most 128 output channels: half the rows, wavefronts 2 x 4 of 64 x 64 each.  A 128-row
// tile multiplies at ~0.7 of the wide tile's rate per flop (more LDS bytes per flop), but the wide one
// would spend half its rows or more on padding there.
#ifndef DROPIT_GEMM_CFG_NARROW
#define DROPIT_GEMM_CFG_NARROW 128, 256, 32, 2, 4, 4, 2, 1
#endif
using Cfg = GemmCfg<DROPIT_GEMM_CFG>;
using CfgFused = GemmCfg<256, 256, 32, 4, 2, 4, 2, 1>;          // the in-LDS recover form is laid out for four stages
using CfgNarrow = GemmCfg<DROPIT_GEMM_CFG_NARROW>;
static_assert(Cfg::BK == CfgNarrow::BK && Cfg::BN == CfgNarrow::BN, "the recovered operand is laid out once for both");
static_assert(Cfg::BM == CfgFused::BM && Cfg::BN == CfgFused::BN && Cfg::BK == CfgFused::BK, "one plan serves both forms");

template <typename C>
int tuned_splits(int tiles, int nkb)
{
    // as many K-slices as fill the 256 compute units (one or two resident workgroups each)
    // without starting a second round -- but a slice of at least ~20 token blocks: every slice
    // writes a whole partial tile however little it summed, and below that depth the partial
    // traffic costs more than the idle compute units (measured on 3136 and 12544 tokens:
    // the best slice count was the one with 19.6 blocks per slice both times)
    int splits = std::min(256 * C::WGS_PER_CU / tiles, std::max(1, (nkb + 10) / 20));
    splits = int(dev_env("DROPIT_FC_SPLITS", splits));
    if (splits > nkb) splits = nkb;
    if (splits < 1) splits = 1;
    if (splits > 256) splits = 256;      // one slice per compute unit when the whole result is a single tile
    return splits;
}

bool use_narrow(const FcProblem &p)
{
    if (const long forced = dev_env("DROPIT_GEMM_NARROW", -1); forced >= 0) return forced == 1;
    return p.cout <= CfgNarrow::BM;
}

template <typename C>
void plan_tiles(const FcProblem &p, FcDensePlan &plan)
{
    plan.nb_count = int((p.cin + C::BN - 1) / C::BN);
    plan.mb_count = int((p.cout + C::BM - 1) / C::BM);
    plan.splits = tuned_splits<C>(plan.nb_count * plan.mb_count, plan.nkb);
    // K-slice partials are whole tiles (ragged edge tiles included) in accumulator order
    plan.partial_bytes = plan.splits > 1 ? size_t(plan.splits) * plan.nb_count * plan.mb_count * C::BM * C::BN * 4 : 0;
}

}  // namespace

bool fc_dense_supported(const FcProblem &p)
{
    // 16-byte dY vectors need c_out % 8 == 0; per-lane byte offsets inside a token block are 32-bit;
    // a recover workgroup holds at least one padded row in LDS
    const int64_t pitch = (p.cin + 7) / 8 * 8;
    return p.cout % 8 == 0 && p.cout >= 8 && p.cin >= 1 && pitch <= RECOVER_ELEMS_MAX &&
           p.cout * Cfg::BK * 2 < (int64_t(1) << 31);
}

bool fc_fused_supported(const FcProblem &p)
{
    // the wide tile only; the column blocks of a token block are counted in LDS; pair positions are 32-bit
    return fc_dense_supported(p) && !use_narrow(p) && (p.cin + Cfg::BN - 1) / Cfg::BN <= BUCKET_MAX_NB &&
           p.k < (int64_t(1) << 31);
}

FcDensePlan fc_dense_plan(const FcProblem &p, bool fused)
{
    FcDensePlan plan;
    plan.nkb = int((p.ntok + Cfg::BK - 1) / Cfg::BK);
    plan.narrow = use_narrow(p);
    if (plan.narrow)
        plan_tiles<CfgNarrow>(p, plan);
    else
        plan_tiles<Cfg>(p, plan);
    plan.pitch = int((p.cin + 7) / 8 * 8);
    plan.rows_per_wg = std::max(1, (plan.pitch <= RECOVER_ELEMS ? RECOVER_ELEMS : RECOVER_ELEMS_MAX) / plan.pitch);
    plan.ntok_pad = int64_t(plan.nkb) * Cfg::BK;
    plan.dense_bytes = round_up(size_t(plan.ntok_pad) * plan.pitch * 2, 256);
    plan.fused = fused;
    // (the product fetches a staging slot's worth of words from any tile start, and table entries up to six token
    // blocks past its slice: both arrays carry that much slack)
    plan.packed_bytes = round_up((size_t(std::max<int64_t>(p.k, 1)) + FUSE_STAGE_WORDS) * 4, 256);
    plan.table_bytes = round_up(((size_t(plan.nkb) + 6) * plan.nb_count + 1) * 4, 256);
    plan.kbptr_bytes = round_up((size_t(plan.nkb) + 1) * 4, 256);
    return plan;
}

static bool fc_dense_attributes()
{
    static std::atomic<uint64_t> attr_set{0};
    return once_per_device(attr_set, [] {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(fc_recover_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                   RECOVER_ELEMS_MAX * 2) == hipSuccess &&
               hipFuncSetAttribute(reinterpret_cast<const void *>(fc_recover_stream_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                   RECOVER_ELEMS_MAX * 2) == hipSuccess &&
               hipFuncSetAttribute(reinterpret_cast<const void *>(fc_recover_rows_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                   RECOVER_ELEMS_MAX * 2 + (RECOVER_ELEMS_MAX / 8 + 1) * 4) == hipSuccess &&
               hipFuncSetAttribute(reinterpret_cast<const void *>(fc_dense_kernel<Cfg, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES) == hipSuccess &&
               hipFuncSetAttribute(reinterpret_cast<const void *>(fc_dense_kernel<Cfg, false, true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES) == hipSuccess &&
               hipFuncSetAttribute(reinterpret_cast<const void *>(fc_dense_kernel<CfgFused, true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, CfgFused::LDS_BYTES + FUSE_LDS_BYTES) == hipSuccess &&
               hipFuncSetAttribute(reinterpret_cast<const void *>(fc_dense_kernel<CfgNarrow, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, CfgNarrow::LDS_BYTES) == hipSuccess;
    });
}

template <typename C, bool FUSED = false, bool PP = false>
static dropit_status launch_gemm(const FcProblem &p, const FcDensePlan &plan, const void *dY, const uint16_t *dense,
                                 float *partial, float *dW, hipStream_t stream, const uint32_t *packed = nullptr,
                                 const uint32_t *tile_ptr = nullptr)
{
    const int total = plan.nb_count * plan.mb_count * plan.splits;
    const int grid = (total + 7) / 8 * 8;
    float *out = plan.splits > 1 ? partial : dW;
    fc_dense_kernel<C, FUSED, PP><<<grid, C::NTHREADS, C::LDS_BYTES + (FUSED ? FUSE_LDS_BYTES : 0), stream>>>(
        static_cast<const uint16_t *>(dY), dense, p.ntok, int(p.cout), int(p.cin), plan.pitch, plan.nb_count,
        plan.mb_count, plan.nkb, plan.splits, out, packed, tile_ptr, uint32_t(std::max<int64_t>(p.k, 1)));

    trace_mark(stream);
    if (plan.splits > 1) {
        const int64_t groups = int64_t(plan.nb_count) * plan.mb_count * (C::BM * C::BN / 4);
        if (plan.splits > 16) {
            splitk_sum_wide_kernel<C><<<int((groups + 15) / 16), 256, 0, stream>>>(
                reinterpret_cast<const f32x4 *>(partial), plan.splits, int(p.cout), int(p.cin), plan.nb_count,
                plan.mb_count, dW);
        } else {
            const int blocks = int(std::min<int64_t>((groups + 255) / 256, 1 << 20));   // one group per thread
            splitk_sum_kernel<C><<<blocks, 256, 0, stream>>>(reinterpret_cast<const f32x4 *>(partial), plan.splits,
                                                             int(p.cout), int(p.cin), plan.nb_count, plan.mb_count, dW);
        }
    }
    trace_mark(stream);
    return launch_status();
}

dropit_status fc_dense_gemm(const FcProblem &p, const FcDensePlan &plan, const void *dY, const uint16_t *dense,
                            float *partial, float *dW, hipStream_t stream)
{
    if (!fc_dense_attributes()) return DROPIT_EHIP;
    if (plan.narrow) return launch_gemm<CfgNarrow>(p, plan, dY, dense, partial, dW, stream);
    if (dev_env("DROPIT_GEMM_LOCKSTEP", 0)) return launch_gemm<Cfg>(p, plan, dY, dense, partial, dW, stream);
    return launch_gemm<Cfg, false, true>(p, plan, dY, dense, partial, dW, stream);
}

dropit_status fc_dense_run(const FcProblem &p, const FcDensePlan &plan, const void *vals, const int32_t *idx,
                           const void *dY, float *dW, char *ws, hipStream_t stream)
{
    uint16_t *dense = reinterpret_cast<uint16_t *>(ws);
    float *partial = reinterpret_cast<float *>(ws + plan.dense_bytes);
    const int64_t ntok_pad = plan.ntok_pad;
    if (!fc_dense_attributes() || plan.fused) return DROPIT_EHIP;

    trace_mark(stream);
    const int recover_grid = int((ntok_pad + plan.rows_per_wg - 1) / plan.rows_per_wg);
    const size_t recover_lds = size_t(plan.rows_per_wg) * plan.pitch * 2;
    // half-width of the window of pairs a recover workgroup loads around its interpolated positions:
    // 4 standard deviations of an evenly spread selection (sqrt(k)/2 at worst) plus a little
    const int64_t margin = 2 * static_cast<int64_t>(__builtin_sqrt(static_cast<double>(p.k))) + 256;
    const double pairs_per_wg = static_cast<double>(p.k) * plan.rows_per_wg / static_cast<double>(std::max<int64_t>(p.ntok, 1));
    bool windowed = pairs_per_wg + 2.0 * margin <= double(RECOVER_WINDOW) * RECOVER_THREADS;
    if (dev_env("DROPIT_RECOVER_STREAM", 0)) windowed = false;
    if (windowed) {
        fc_recover_kernel<<<recover_grid, RECOVER_THREADS, recover_lds, stream>>>(
            static_cast<const uint16_t *>(vals), idx, p.k, p.ntok, ntok_pad, int(p.cin), plan.pitch, plan.rows_per_wg,
            margin, dense);
    } else {
        // several consecutive tiles per workgroup, about two workgroups per compute unit (measured best of 1, 2, 4, 8)
        const int tiles_per_wg = std::max(1, (recover_grid + 511) / 512);
        const int grid = (recover_grid + tiles_per_wg - 1) / tiles_per_wg;
        fc_recover_stream_kernel<<<grid, RECOVER_THREADS, recover_lds, stream>>>(
            static_cast<const uint16_t *>(vals), idx, p.k, p.ntok, ntok_pad, int(p.cin), plan.pitch, plan.rows_per_wg,
            tiles_per_wg, dense);
    }

    trace_mark(stream);
    return fc_dense_gemm(p, plan, dY, dense, partial, dW, stream);
}

dropit_status fc_fused_run(const FcProblem &p, const FcDensePlan &plan, const void *vals, const int32_t *idx,
                           const void *dY, float *dW, char *ws, hipStream_t stream)
{
    if (!fc_dense_attributes() || !plan.fused || plan.narrow || p.k < 1) return DROPIT_EHIP;
    uint32_t *packed = reinterpret_cast<uint32_t *>(ws);
    uint32_t *tile_ptr = reinterpret_cast<uint32_t *>(ws + plan.packed_bytes);
    uint32_t *kb_ptr = reinterpret_cast<uint32_t *>(ws + plan.packed_bytes + plan.table_bytes);
    float *partial = reinterpret_cast<float *>(ws + plan.operand_bytes());
    trace_mark(stream);
    launch_row_starts(idx, p.k, uint32_t(Cfg::BK * p.cin), plan.nkb, kb_ptr, stream);
    trace_mark(stream);
    const size_t lds = (size_t(2) * Cfg::BK * plan.nb_count + 1 + plan.nb_count) * 4;
    fc_bucket_kernel<<<plan.nkb, BUCKET_THREADS, lds, stream>>>(static_cast<const uint16_t *>(vals), idx, p.k,
                                                                uint32_t(p.cin), plan.nb_count, plan.nkb, kb_ptr, packed,
                                                                tile_ptr);
    trace_mark(stream);
    return launch_gemm<CfgFused, true>(p, plan, dY, nullptr, partial, dW, stream, packed, tile_ptr);
}

bool fc_dense_mask_native(const FcProblem &p) { return fc_dense_supported(p) && p.cin % 8 == 0; }

dropit_status fc_dense_run_mask(const FcProblem &p, const FcDensePlan &plan, const void *vals, const uint32_t *mask,
                                const int32_t *blockptr, const void *dY, float *dW, char *ws, hipStream_t stream)
{
    uint16_t *dense = reinterpret_cast<uint16_t *>(ws);
    float *partial = reinterpret_cast<float *>(ws + plan.dense_bytes);
    if (!fc_dense_attributes() || plan.pitch != p.cin) return DROPIT_EHIP;
    trace_mark(stream);
    const int64_t dense_elems = plan.ntok_pad * plan.pitch;          // a multiple of 8
    fc_recover_mask_kernel<<<int((dense_elems + 2047) / 2048), 256, 0, stream>>>(
        static_cast<const uint16_t *>(vals), mask, blockptr, p.k, p.ntok * p.cin, dense_elems, dense);
    trace_mark(stream);
    return fc_dense_gemm(p, plan, dY, dense, partial, dW, stream);
}

dropit_status fc_dense_run_rows(const FcProblem &p, const FcDensePlan &plan, const void *vals, const uint16_t *col,
                                const int32_t *rowptr, const void *dY, float *dW, char *ws, hipStream_t stream)
{
    uint16_t *dense = reinterpret_cast<uint16_t *>(ws);
    float *partial = reinterpret_cast<float *>(ws + plan.dense_bytes);
    if (!fc_dense_attributes()) return DROPIT_EHIP;
    trace_mark(stream);
    const int grid = int((plan.ntok_pad + plan.rows_per_wg - 1) / plan.rows_per_wg);
    const size_t lds = size_t(plan.rows_per_wg) * plan.pitch * 2 + size_t(plan.rows_per_wg + 1) * 4;
    fc_recover_rows_kernel<<<grid, RECOVER_THREADS, lds, stream>>>(
        static_cast<const uint16_t *>(vals), col, rowptr, p.k, p.ntok, plan.ntok_pad, int(p.cin), plan.pitch,
        plan.rows_per_wg, dense);
    trace_mark(stream);
    return fc_dense_gemm(p, plan, dY, dense, partial, dW, stream);
}

}  // namespace dropit
