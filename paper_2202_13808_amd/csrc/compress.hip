// Min-k dropping D(a) = {a_Xr, Xr} (Sec. 3.2; Sec. 3.3, min-k strategy; Sec. 4.1)
// as a bandwidth-bound radix select + ordered stream compaction for gfx950.
//
// The magnitude key of an element is its bit pattern with the sign cleared
// (15 bits for bf16, 31 for fp32); unsigned key order == |x| order.
//
// The steps, whichever way they are launched:
//   hist pass : MSB-first digit histogram of the keys that match the digits
//               resolved so far (LDS histogram per workgroup, merged with
//               global atomics), then the digit holding the k-th key is resolved
//   count pass: resolves the last (4/5-bit) digit; every workgroup owns one
//               contiguous chunk of x and records, per chunk, how many keys
//               are above the resolved prefix and a small histogram of the
//               matching ones.  From these follow the threshold key t, the tie
//               budget m = k - #{key > t}, and the exclusive per-chunk offsets
//               of {key > t} and {key == t}.
//   compact   : each workgroup writes the (value, index) pairs of its chunk in
//               ascending index order; of the keys equal to t only the first m
//               by flat index are kept.
// bf16: 11 + 4 bits (one hist pass); fp32: 13 + 13 + 5 bits (two hist passes).
//
// Default: ONE persistent kernel (select_fused_kernel) does all of it with grid
// barriers between the steps, the chunk parked in LDS, and a serial redo path
// should the barriers ever give up.  For large 16-bit tensors it predicts the
// first digit from a sample of the tensor and lets the count pass, which is
// exact, confirm the prediction (see "sampled first digit" below); the bytes
// it writes are the same either way.  Alternative: the steps as separate kernels
// (init, hist, count, compact) with a last-workgroup-to-arrive ticket instead of
// barriers.  Nothing here synchronises with the host; counts are integer, so the
// result does not depend on the order in which workgroups run.
#include "common.hpp"
#include "dev_hooks.hpp"
#include <atomic>
#include <cstdlib>
#include <random>
#include <type_traits>

namespace dropit {
namespace {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_MAX_CHUNKS = 512;
constexpr int SEL_UNROLL = 4;
constexpr int MAX_HIST_BITS = 13;
constexpr int MAX_LAST_BINS = 48;       // rows of the per-chunk table: up to three 16-key bins of a sampled bracket, else 2^LAST_BITS

struct SelState {
    uint32_t prefix;     // key digits resolved so far (key >> remaining bits)
    uint32_t k_rem;      // elements still to take among the keys matching prefix
    uint32_t t;          // threshold key (valid after the count pass)
    uint32_t m;          // how many keys equal to t are kept (lowest flat index first)
    uint32_t ticket[4];  // arrival counters, one per pass
    uint32_t barrier;    // arrivals at the fused kernel's grid barriers (monotone within a call)
    uint32_t error;      // hint: some workgroup ran out of patience at a grid barrier (the others stop waiting)
    uint32_t exited;     // fused kernel: low 16 bits = workgroups done, high 16 bits = how many of them gave up
    uint32_t path;       // fused kernel, for the tests: 0 exact digit histograms, 1 sampled bracket confirmed, 2 sampled bracket missed (exact retry)
    unsigned long long ready;    // == the call's generation number once workgroup 0 has cleared the words above and the histograms;
                                 // the last workgroup to leave puts 0 back (no generation is 0), so a launch replayed with
                                 // the same number (a captured graph) waits for its own workgroup 0 again
    uint32_t redo;       // fused kernel, for callers and tests: 1 if the grid barriers gave up and the last workgroup redid the selection alone
    uint32_t staged;     // fused kernel, for the tests: how many workgroups compacted from candidates staged in LDS (one read of x)
    uint32_t pad[48];
};
static_assert(sizeof(SelState) == 256, "state block is 256 bytes");

// Workspace carving (in bytes from the 256-byte aligned base).
struct SelWorkspace {
    static constexpr size_t state_off = 0;
    static constexpr size_t hist0_off = state_off + sizeof(SelState);
    static constexpr size_t hist1_off = hist0_off + sizeof(uint32_t) * (1u << MAX_HIST_BITS);
    static constexpr size_t table_off = hist1_off + sizeof(uint32_t) * (1u << MAX_HIST_BITS);
    static constexpr size_t offgt_off = table_off + sizeof(uint32_t) * (MAX_LAST_BINS + 1) * SEL_MAX_CHUNKS;
    static constexpr size_t offeq_off = offgt_off + sizeof(uint32_t) * SEL_MAX_CHUNKS;
    static constexpr size_t xbar_off = offeq_off + sizeof(uint32_t) * SEL_MAX_CHUNKS;   // 8 arrival counters, 256 B apart
    static constexpr size_t bytes = xbar_off + 8 * 256;
    static constexpr size_t zero_bytes = table_off;   // state + both histograms are cleared per call
};

template <typename RAW> struct KeyTraits;
template <> struct KeyTraits<uint16_t> {
    static constexpr int VEC = 8;
    static constexpr uint32_t MASK = 0x7FFFu;
};
template <> struct KeyTraits<uint32_t> {
    static constexpr int VEC = 4;
    static constexpr uint32_t MASK = 0x7FFFFFFFu;
};

// Calls f(raw_bits, e) for the VEC elements of one 16-byte vector, e ascending.
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;   // plain register vector (no class wrapper)

template <typename V, typename F> __device__ inline void for_each_raw(uint16_t, const V &q, F f)
{
    f(q.x & 0xFFFFu, 0); f(q.x >> 16, 1); f(q.y & 0xFFFFu, 2); f(q.y >> 16, 3);
    f(q.z & 0xFFFFu, 4); f(q.z >> 16, 5); f(q.w & 0xFFFFu, 6); f(q.w >> 16, 7);
}
template <typename V, typename F> __device__ inline void for_each_raw(uint32_t, const V &q, F f)
{
    f(q.x, 0); f(q.y, 1); f(q.z, 2); f(q.w, 3);
}

__global__ void __launch_bounds__(256) init_kernel(uint32_t *ws, uint32_t nwords, uint32_t k)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += gridDim.x * blockDim.x)
        ws[i] = (i == offsetof(SelState, k_rem) / 4) ? k : 0u;
}

// Ticket: true in every thread of exactly one workgroup, the last to arrive.
// The fences make every earlier workgroup's global writes visible to the
// ordinary loads the last workgroup issues afterwards.
__device__ inline bool last_block_to_arrive(uint32_t *ticket)
{
    __shared__ uint32_t s_last;
    __syncthreads();                       // the whole workgroup's global writes are issued
    if (threadIdx.x == 0) {
        __threadfence();                   // release them (one fence per workgroup: it is device-wide)
        const uint32_t t = atomicAdd(ticket, 1u);
        const bool last = t == gridDim.x - 1;
        if (last) __threadfence();         // acquire every other workgroup's writes
        s_last = last ? 1u : 0u;
    }
    __syncthreads();
    return s_last != 0;
}

// One workgroup: find the digit d with  #{digit > d} < k_rem <= #{digit >= d}
// in hist[0..NB), then fold it into the state.
template <int NB, int BITS>
__device__ inline void resolve_digit(const uint32_t *hist, SelState *st, uint32_t *scan /*[SEL_THREADS]*/)
{
    constexpr int PER = (NB + SEL_THREADS - 1) / SEL_THREADS;
    const int tid = threadIdx.x;
    const int lo = tid * PER;
    uint32_t c[PER];
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        c[i] = (lo + i < NB) ? hist[lo + i] : 0u;
        mine += c[i];
    }
    // inclusive suffix sum over threads: scan[tid] = sum of `mine` for threads >= tid
    scan[tid] = mine;
    __syncthreads();
    for (int o = 1; o < SEL_THREADS; o <<= 1) {
        const uint32_t add = (tid + o < SEL_THREADS) ? scan[tid + o] : 0u;
        __syncthreads();
        scan[tid] += add;
        __syncthreads();
    }
    const uint32_t k_rem = st->k_rem;
    const uint32_t prefix = st->prefix;
    uint32_t above = scan[tid] - mine;     // keys with a digit in a higher thread's range
    __syncthreads();                       // every thread has read the state before it changes
    if (above < k_rem && k_rem <= above + mine) {
#pragma unroll
        for (int i = PER - 1; i >= 0; --i) {
            if (above + c[i] >= k_rem) {
                st->prefix = (prefix << BITS) | static_cast<uint32_t>(lo + i);
                st->k_rem = k_rem - above;
                break;
            }
            above += c[i];
        }
    }
}

// Digit histogram of the keys whose higher digits equal the resolved prefix.
// x is walked as `nvf` full 16-byte vectors split into contiguous chunks of
// `vpc` vectors (one per workgroup); the last workgroup also takes the
// numel % VEC ragged elements.  The inner loop is branch-free: a key that does
// not match, or whose digit is 0 (exact zeros are common after ReLU), is
// counted in a per-lane spill slot instead of a shared bin.
template <typename RAW, int SHIFT, int BITS, bool FIRST>
__global__ void __launch_bounds__(SEL_THREADS)
hist_kernel(const RAW *__restrict__ x, int64_t numel, int64_t nvf, int64_t vpc, SelState *st,
            uint32_t *ghist, int pass)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    constexpr uint32_t MASK = KeyTraits<RAW>::MASK;
    constexpr int NB = 1 << BITS;
    __shared__ uint32_t lh[NB + 2 * WAVE];
    __shared__ uint32_t scan[SEL_THREADS];
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    for (int i = tid; i < NB + 2 * WAVE; i += SEL_THREADS) lh[i] = 0;
    const uint32_t prefix = FIRST ? 0u : st->prefix;
    __syncthreads();

    const uint32_t zslot = NB + lane, dslot = NB + WAVE + lane;
    auto count = [&](uint32_t raw, int) {
        const uint32_t key = raw & MASK;
        const uint32_t d = (key >> SHIFT) & (NB - 1);
        uint32_t a = d ? d : zslot;
        if (!FIRST) a = ((key >> (SHIFT + BITS)) == prefix) ? a : dslot;
        atomicAdd(&lh[a], 1u);
    };
    const uint4 *xv = reinterpret_cast<const uint4 *>(x);
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * vpc;
    const int64_t v1 = min(v0 + vpc, nvf);
    int64_t vb = v0;
    for (; vb + SEL_THREADS * SEL_UNROLL <= v1; vb += SEL_THREADS * SEL_UNROLL) {
        uint4 q[SEL_UNROLL];
#pragma unroll
        for (int u = 0; u < SEL_UNROLL; ++u) q[u] = xv[vb + u * SEL_THREADS + tid];
#pragma unroll
        for (int u = 0; u < SEL_UNROLL; ++u) for_each_raw(RAW(0), q[u], count);
    }
    for (int64_t v = vb + tid; v < v1; v += SEL_THREADS) for_each_raw(RAW(0), xv[v], count);
    if (blockIdx.x == gridDim.x - 1 && tid == 0)
        for (int64_t i = nvf * VEC; i < numel; ++i) count(x[i], 0);
    __syncthreads();
    if (tid < WAVE) {                      // fold the digit-0 spill slots into bin 0
        const uint32_t z = wave_sum(lh[NB + tid]);
        if (tid == 0) lh[0] += z;
    }
    __syncthreads();
    for (int i = tid; i < NB; i += SEL_THREADS) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&ghist[i], c);
    }
    if (!last_block_to_arrive(&st->ticket[pass])) return;
    resolve_digit<NB, BITS>(ghist, st, scan);
}

// Last digit + per-chunk bookkeeping for the ordered compaction.
template <typename RAW, int LAST_BITS>
__global__ void __launch_bounds__(SEL_THREADS)
count_kernel(const RAW *__restrict__ x, int64_t numel, int64_t nvf, int64_t vpc, SelState *st,
             uint32_t *table /*[LB+1][G]*/, uint32_t *off_gt, uint32_t *off_eq, int pass)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    constexpr uint32_t MASK = KeyTraits<RAW>::MASK;
    constexpr int LB = 1 << LAST_BITS;
    constexpr int NW = SEL_THREADS / WAVE;
    __shared__ uint32_t lh[LB + 1 + WAVE];
    __shared__ uint32_t s_digit;
    __shared__ uint32_t wave_tot2[2 * NW];
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int G = gridDim.x;
    for (int i = tid; i < LB + 1 + WAVE; i += SEL_THREADS) lh[i] = 0;
    const uint32_t prefix = st->prefix;    // == (threshold key) >> LAST_BITS
    __syncthreads();

    const uint32_t dslot = LB + 1 + lane;
    uint32_t above = 0;
    auto count = [&](uint32_t raw, int) {
        const uint32_t key = raw & MASK;
        const uint32_t hi = key >> LAST_BITS;
        above += (hi > prefix) ? 1u : 0u;
        atomicAdd(&lh[(hi == prefix) ? (key & (LB - 1)) : dslot], 1u);
    };
    const uint4 *xv = reinterpret_cast<const uint4 *>(x);
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * vpc;
    const int64_t v1 = min(v0 + vpc, nvf);
    int64_t vb = v0;
    for (; vb + SEL_THREADS * SEL_UNROLL <= v1; vb += SEL_THREADS * SEL_UNROLL) {
        uint4 q[SEL_UNROLL];
#pragma unroll
        for (int u = 0; u < SEL_UNROLL; ++u) q[u] = xv[vb + u * SEL_THREADS + tid];
#pragma unroll
        for (int u = 0; u < SEL_UNROLL; ++u) for_each_raw(RAW(0), q[u], count);
    }
    for (int64_t v = vb + tid; v < v1; v += SEL_THREADS) for_each_raw(RAW(0), xv[v], count);
    if (blockIdx.x == gridDim.x - 1 && tid == 0)
        for (int64_t i = nvf * VEC; i < numel; ++i) count(x[i], 0);
    above = wave_sum(above);
    if (lane == 0 && above) atomicAdd(&lh[LB], above);
    __syncthreads();
    if (tid <= LB) table[tid * G + blockIdx.x] = lh[tid];
    if (!last_block_to_arrive(&st->ticket[pass])) return;

    // ---- last workgroup: resolve the final digit, then per-chunk offsets ----
    // totals per bin: each wavefront sums whole rows of table[b][0..G)
    for (int b = tid / WAVE; b < LB; b += NW) {
        uint32_t s = 0;
        for (int c = lane; c < G; c += WAVE) s += table[b * G + c];
        s = wave_sum(s);
        if (lane == 0) lh[b] = s;
    }
    __syncthreads();
    if (tid == 0) {
        const uint32_t k_rem = st->k_rem;
        uint32_t acc = 0;
        int d = 0;
        for (int b = LB - 1; b >= 0; --b) {
            if (acc + lh[b] >= k_rem) { d = b; break; }
            acc += lh[b];
        }
        st->t = (prefix << LAST_BITS) | static_cast<uint32_t>(d);
        st->m = k_rem - acc;
        s_digit = static_cast<uint32_t>(d);
    }
    __syncthreads();
    const int d = static_cast<int>(s_digit);
    // exclusive scan over chunks of (#{key > t}, #{key == t}); consecutive chunks per thread
    constexpr int CPT = (SEL_MAX_CHUNKS + SEL_THREADS - 1) / SEL_THREADS;
    uint32_t gt[CPT], eq[CPT];
    uint32_t mine_gt = 0, mine_eq = 0;
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = tid * CPT + i;
        gt[i] = eq[i] = 0;
        if (c < G) {
            uint32_t g = table[LB * G + c];
#pragma unroll
            for (int b = 0; b < LB; ++b) {
                const uint32_t n = table[b * G + c];
                g += (b > d) ? n : 0u;
                eq[i] = (b == d) ? n : eq[i];
            }
            gt[i] = g;
        }
        mine_gt += gt[i];
        mine_eq += eq[i];
    }
    uint32_t run_gt, run_eq, total_gt, total_eq;
    block_exclusive_scan2<SEL_THREADS>(mine_gt, mine_eq, wave_tot2, run_gt, run_eq, total_gt, total_eq);
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = tid * CPT + i;
        if (c < G) {
            off_gt[c] = run_gt;
            off_eq[c] = run_eq;
        }
        run_gt += gt[i];
        run_eq += eq[i];
    }
}

// Ordered compaction of one chunk per workgroup.
template <typename RAW>
__global__ void __launch_bounds__(SEL_THREADS)
compact_kernel(const RAW *__restrict__ x, int64_t numel, int64_t nvf, int64_t vpc,
               const SelState *__restrict__ st, const uint32_t *__restrict__ off_gt,
               const uint32_t *__restrict__ off_eq, RAW *__restrict__ vals, int32_t *__restrict__ idx)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    constexpr uint32_t MASK = KeyTraits<RAW>::MASK;
    __shared__ uint32_t wave_tot[SEL_THREADS / WAVE];
    const int tid = threadIdx.x;
    const uint32_t t = st->t;
    const uint32_t m = st->m;
    uint32_t run_gt = off_gt[blockIdx.x];  // #{key > t} before this tile
    uint32_t run_eq = off_eq[blockIdx.x];  // #{key == t} before this tile
    const uint4 *xv = reinterpret_cast<const uint4 *>(x);
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * vpc;
    const int64_t v1 = min(v0 + vpc, nvf);
    for (int64_t vb = v0; vb < v1; vb += SEL_THREADS) {
        const int64_t v = vb + tid;
        const bool live = v < v1;
        uint4 q = make_uint4(0, 0, 0, 0);
        if (live) q = xv[v];
        uint32_t cnt = 0;                  // low 16 bits: #gt, high 16 bits: #eq (tile <= 8192 elements)
        for_each_raw(RAW(0), q, [&](uint32_t raw, int) {
            const uint32_t key = raw & MASK;
            cnt += (key > t ? 1u : 0u) + (key == t ? 0x10000u : 0u);
        });
        if (!live) cnt = 0;
        uint32_t total;
        const uint32_t excl = block_exclusive_scan<SEL_THREADS>(cnt, wave_tot, total);
        uint32_t my_gt = run_gt + (excl & 0xFFFFu);
        uint32_t my_eq = run_eq + (excl >> 16);
        const int64_t base = v * VEC;
        if (live && cnt) {
            for_each_raw(RAW(0), q, [&](uint32_t raw, int e) {
                const uint32_t key = raw & MASK;
                if (key > t) {
                    const uint32_t pos = my_gt + min(my_eq, m);
                    vals[pos] = static_cast<RAW>(raw);
                    idx[pos] = static_cast<int32_t>(base + e);
                    ++my_gt;
                } else if (key == t) {
                    if (my_eq < m) {
                        const uint32_t pos = my_gt + my_eq;
                        vals[pos] = static_cast<RAW>(raw);
                        idx[pos] = static_cast<int32_t>(base + e);
                    }
                    ++my_eq;
                }
            });
        }
        run_gt += total & 0xFFFFu;
        run_eq += total >> 16;
    }
    // ragged tail (numel % VEC elements) after the last full vector
    if (blockIdx.x == gridDim.x - 1 && tid == 0) {
        for (int64_t i = nvf * VEC; i < numel; ++i) {
            const RAW raw = x[i];
            const uint32_t key = raw & MASK;
            if (key > t) {
                const uint32_t pos = run_gt + min(run_eq, m);
                vals[pos] = raw;
                idx[pos] = static_cast<int32_t>(i);
                ++run_gt;
            } else if (key == t) {
                if (run_eq < m) {
                    const uint32_t pos = run_gt + run_eq;
                    vals[pos] = raw;
                    idx[pos] = static_cast<int32_t>(i);
                }
                ++run_eq;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Fused path: the whole select + compaction as ONE persistent kernel with one
// workgroup per compute unit.  Each workgroup parks the first FUSED_RES x 16 KB of its
// chunk in LDS across all phases (the whole chunk for tensors up to ~25 MB; anything
// beyond is re-read, mostly from the Infinity Cache), and the phases are separated by
// grid barriers instead of kernel boundaries.  Loops over the parked vectors are rolled
// on purpose: unrolling them 8x made the kernel 48 KB of code and instruction-fetch bound.  Every workgroup resolves the digits itself
// from the merged histogram, so the select state lives in registers.
//
// The kernel is an ordinary launch (a cooperative launch costs ~14 us of queue switching before and
// after the kernel on this runtime): the host only checks that the grid fits the device all at once.
// Should the workgroups nevertheless not all become resident (a device shared with other persistent
// kernels), the bounded grid barriers give up, every workgroup leaves, and the last one to leave
// redoes the whole selection on its own (select_serial): slow, but the result is always complete.
//
// Everything workgroups exchange (histogram, per-chunk table, barrier counter) is
// accessed ONLY with device-scope atomics, which are coherent by themselves, so no
// device-wide fence is needed: on this 8-XCD part such a fence writes back and
// invalidates a whole L2 and was measured at 5-8 us per grid barrier.  The ordering
// rests on what the hardware does, not on the language's memory model: a wave's exchanged
// stores and atomics are complete (s_waitcnt at the __syncthreads() in front of the
// arrival) before thread 0 issues the arrival atomic, and nothing exchanged is ever read
// through a non-coherent cache line.  The form the model itself guarantees -- acq_rel on the
// group counter, release on the top counter, an acquire fence after the wait, all at agent
// scope -- was measured beside it: 3.4-4.8 us more per call on every benchmark tensor (one
// barrier per call), for the L2 write-back and invalidate it implies; the relaxed form stays.
constexpr int FUSED_RES = 6;             // 16-byte vectors per thread parked in LDS
// Patience in polls (~0.25 us each); every wave exits even if it runs out.  A resident grid meets at a barrier within
// microseconds (a millisecond for the largest tensors), so the barriers give up after ~15 ms: a grid that is not
// resident all at once then costs those milliseconds plus the serial redo, not a second.  Waiting for workgroup 0's
// clearing pass is another matter: it is dispatched first and needs a few microseconds, and a workgroup that stops
// waiting for it leaves the exit count short (nobody then puts `ready` back to 0), so that wait is long.
constexpr uint32_t SPIN_LIMIT = 1u << 16;
constexpr uint32_t READY_SPIN_LIMIT = 1u << 26;

__device__ inline uint32_t dev_load(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void dev_store(uint32_t *p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline unsigned long long dev_load64(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void dev_store64(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// All workgroups of the grid meet here (`round` = 1, 2, ... counts the barriers of the call).
// Arrival is two-level: a workgroup bumps the counter of its group (launch order modulo 8, counters
// 256 bytes apart), the last of a group bumps the top counter, everybody polls the top counter;
// 256 atomics on ONE word take ~10 ns each, one after the other.
// The grid is sized so that every workgroup is resident at once, but nothing enforces that the
// device is not shared, so the wait is bounded: returns false (in every thread of the workgroup)
// if the others did not all arrive within `spin_limit` polls or if some workgroup already gave
// up.  The caller then skips to the kernel's exit protocol.
// __syncthreads() makes every wave wait for its own outstanding atomics first.
__device__ inline bool grid_barrier(SelState *st, uint32_t *xbar, uint32_t round, uint32_t spin_limit, uint32_t *ok_slot)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t G = gridDim.x, group = blockIdx.x & 7u;
        const uint32_t groups = G < 8u ? G : 8u, members = (G - group + 7u) / 8u;
        const uint32_t before = __hip_atomic_fetch_add(&xbar[group * 64], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (before + 1 == round * members)
            __hip_atomic_fetch_add(&st->barrier, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t spins = 0, ok = 1;
        while (dev_load(&st->barrier) < round * groups) {
            if (++spins > spin_limit || ((spins & 31u) == 0 && dev_load(&st->error) != 0)) {
                dev_store(&st->error, 1u);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(8);        // ~0.2 us between polls: 256 pollers on one word compete with the arrivals
        }
        *ok_slot = ok;
    }
    __syncthreads();
    return *ok_slot != 0;
}

// Finds the digit d with #{digit > d} < k_rem <= #{digit >= d} in the merged histogram
// and folds it into the workgroup's copy of the select state.  Thread t owns the bins
// of reversed rank t, so an ordinary exclusive prefix scan counts the keys above it.
template <int NB, int BITS>
__device__ inline void resolve_digit_local(const uint32_t *hist, uint32_t &prefix, uint32_t &k_rem,
                                           uint32_t *wave_tot, uint32_t *bcast /*[2]*/)
{
    constexpr int PER = (NB + SEL_THREADS - 1) / SEL_THREADS;
    const int tid = threadIdx.x;
    const int hi_bin = NB - 1 - tid * PER;           // this thread's highest bin; it owns hi_bin, hi_bin-1, ...
    uint32_t c[PER];
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        c[i] = (hi_bin - i >= 0) ? dev_load(hist + hi_bin - i) : 0u;
        mine += c[i];
    }
    uint32_t total;
    uint32_t above = block_exclusive_scan<SEL_THREADS>(mine, wave_tot, total);
    if (above < k_rem && k_rem <= above + mine) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            if (above + c[i] >= k_rem) {
                bcast[0] = (prefix << BITS) | static_cast<uint32_t>(hi_bin - i);
                bcast[1] = k_rem - above;
                break;
            }
            above += c[i];
        }
    }
    __syncthreads();
    prefix = bcast[0];
    k_rem = bcast[1];
    __syncthreads();
}

// ---- sampled first digit (16-bit element types) ---------------------------------------------------
// The first digit's histogram needs one LDS atomic per element, which is what bounds that pass (the
// LDS atomic unit of a compute unit takes ~16 cycles per wavefront instruction whatever it adds), then
// a merge with global atomics, a grid barrier, and a read-back of the merged histogram.  The bin that
// holds the k-th largest key can be predicted from a sample instead, and without any exchange: EVERY
// workgroup reads the same 512 pieces of 64 bytes (one per equal stretch of the tensor, at a hashed
// position inside it -- many small pieces, so that values that come in runs, like the tokens of an
// activation, do not fool it; served by the L2 caches after the first reader), histograms them in its own LDS and
// derives the same bracket of up to three adjacent bins around the sample's quantile, wide enough for
// 5 standard deviations of the sampling error.  The bracket is only a prediction: the pass over all
// elements that follows counts exactly how many keys lie above the bracket and how many on each key
// inside it, so a bracket that does not contain the k-th largest key is detected, and the selection
// then runs with the exact histogram.  The result is the same in every case; only the time differs.
constexpr int SAMPLE_VECTORS_PER_THREAD = 2;          // x 1024 threads x 8 elements = 16 384 sampled elements
constexpr int64_t SAMPLE_MIN_NUMEL = int64_t(1) << 21; // below this the exact histogram is cheap
constexpr int BRACKET_MAX_BINS = 3;

constexpr int SAMPLE_PIECE = 4;                       // vectors per sampled piece (64 bytes: four lanes share a cache line)

// First vector of sample piece i of n: stretch i of the tensor, hashed offset inside it (whole pieces).
__device__ inline int64_t sample_piece(int i, int n, int64_t nvf)
{
    const int64_t seg = (nvf / SAMPLE_PIECE) / n;                     // pieces per stretch
    const uint32_t h = (static_cast<uint32_t>(i) + 1u) * 0x9E3779B1u;
    return (int64_t(i) * seg + static_cast<int64_t>((h >> 8) % static_cast<uint32_t>(seg))) * SAMPLE_PIECE;
}

// From the sample's histogram (in LDS): the bins that hold the sample ranks r - margin and r + margin,
// r = the sample's share of k.  Returns false (in every thread) if there is no usable bracket (a
// quantile too close to either end of the sample, more than BRACKET_MAX_BINS bins).
template <int NB>
__device__ inline bool sample_bracket(const uint32_t *hist, uint32_t k, int64_t numel, uint32_t *wave_tot,
                                      uint32_t *bcast /*[3]*/, uint32_t &b_lo, uint32_t &b_hi)
{
    constexpr int PER = (NB + SEL_THREADS - 1) / SEL_THREADS;
    const int tid = threadIdx.x;
    const int hi_bin = NB - 1 - tid * PER;           // as in resolve_digit_local: descending bins, ascending ranks
    uint32_t c[PER];
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        c[i] = (hi_bin - i >= 0) ? hist[hi_bin - i] : 0u;
        mine += c[i];
    }
    uint32_t total;
    const uint32_t above = block_exclusive_scan<SEL_THREADS>(mine, wave_tot, total);
    const float frac = static_cast<float>(k) / static_cast<float>(numel);
    const float r = frac * static_cast<float>(total);
    const float margin = 5.0f * __builtin_sqrtf(fmaxf(r * (1.0f - frac), 1.0f)) + 8.0f;
    const float lo_f = r - margin, hi_f = r + margin;
    const bool usable = lo_f >= 1.0f && hi_f <= static_cast<float>(total) - 1.0f;
    if (tid == 0) bcast[2] = usable ? 1u : 0u;
    if (usable) {
        const uint32_t rank[2] = {static_cast<uint32_t>(lo_f), static_cast<uint32_t>(hi_f) + 1u};   // higher bin first
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            if (above < rank[q] && rank[q] <= above + mine) {
                uint32_t a = above;
#pragma unroll
                for (int i = 0; i < PER; ++i) {
                    if (a + c[i] >= rank[q]) {
                        bcast[q] = static_cast<uint32_t>(hi_bin - i);
                        break;
                    }
                    a += c[i];
                }
            }
        }
    }
    __syncthreads();
    b_hi = bcast[0];
    b_lo = bcast[1];
    const bool ok = bcast[2] != 0 && b_hi >= b_lo && b_hi - b_lo < static_cast<uint32_t>(BRACKET_MAX_BINS);
    __syncthreads();
    return ok;
}

// ---- one read of x: candidates staged in LDS (16-bit element types, sampled bracket) ----------------
// With the bracket [key_lo, key_lo + nf) known BEFORE the pass over the chunk, everything that can still
// be kept is known too: the elements with key >= key_lo, a share of (1 - gamma) plus the bracket's width
// (11-15 % at gamma = 0.9).  The pass therefore stages them in LDS, in flat-index order, as one word each
// (value << 16 | position), and both the exact counts and the compaction then walk the staged words
// instead of reading x again -- x is read from memory exactly once, whatever the tensor size.
// Each wavefront owns a contiguous 1/16 of the chunk and a staging segment of its own, so the pass needs
// no workgroup barrier: a wavefront loads ST_U x 64 vectors (coalesced), turns them through a private
// LDS buffer so that every lane holds ST_U CONSECUTIVE vectors (flat order = lane order: one wavefront
// scan of the per-lane candidate counts gives every candidate its slot), and copies the candidates out
// of that buffer.  The buffer is padded by 16 bytes per 128 so that both the coalesced writes and the
// 32-byte-per-lane reads are free of bank conflicts.
// A chunk with more candidates than a segment holds (values that bunch up along the tensor; tensors
// beyond ~110 MB) takes the two-read form below for that workgroup; the bytes written are the same.
constexpr int ST_U = 2;                                    // vectors per lane per block
constexpr int ST_BLKV = ST_U * WAVE;                       // vectors per block (1024 16-bit elements)
constexpr int ST_EPL = ST_U * 8;                           // elements per lane per block
constexpr int ST_TRANS_BYTES = ST_BLKV * 16 + (ST_BLKV / 8) * 16;
constexpr int ST_LH_OFF = (SEL_THREADS / WAVE) * ST_TRANS_BYTES;
constexpr int ST_STAGE_OFF = ST_LH_OFF + 256;
constexpr size_t FUSED_SMEM_BYTES = 156 * 1024;            // of the 160 KB of a compute unit; the rest is static
constexpr int ST_SEGCAP = int((FUSED_SMEM_BYTES - ST_STAGE_OFF) / 4 / (SEL_THREADS / WAVE));   // staged words per wavefront
static_assert(ST_STAGE_OFF + 4 * ((1 << 11) + 2 * WAVE) <= int(FUSED_SMEM_BYTES), "the exact retry's histogram fits behind ST_LH_OFF");
static_assert(ST_STAGE_OFF % 16 == 0 && ST_SEGCAP % 4 == 0, "staged words are read four at a time");

// bit b of the result: element b of the ST_EPL consecutive 16-bit elements in r[] has key >= key_lo.
// Per 32-bit word: one AND clears both signs, one unsigned compare per half (the upper half against
// key_lo << 16: the lower half cannot change the outcome), and an add-with-carry shifts each outcome
// into the mask; the elements are taken last to first so that element 0 ends in bit 0.
__device__ inline uint32_t candidate_mask(const u32x4 (&r)[ST_U], uint32_t key_lo)
{
    uint32_t mask = 0, k;
    const uint32_t lo = key_lo, hi = key_lo << 16;
#pragma unroll
    for (int u = ST_U - 1; u >= 0; --u)
#pragma unroll
        for (int w = 3; w >= 0; --w) {
            const uint32_t word = r[u][w];
            asm("v_and_b32 %1, 0x7fff7fff, %2\n\t"
                "v_cmp_le_u32 vcc, %4, %1\n\t"
                "v_addc_co_u32 %0, vcc, %0, %0, vcc\n\t"
                "v_cmp_le_u16 vcc, %3, %1\n\t"
                "v_addc_co_u32 %0, vcc, %0, %0, vcc"
                : "+v"(mask), "=&v"(k)
                : "v"(word), "s"(lo), "s"(hi)
                : "vcc");
        }
    return mask;
}

// The parallel selection.  Returns (the same in every thread) SEL_DONE, or SEL_GAVE_UP if a grid
// barrier ran out of patience, or SEL_NEVER_READY if the exchange area was never published; in the
// last two cases the outputs are incomplete (whatever was written is correct, nothing is out of bounds).
enum SelOutcome { SEL_DONE = 0, SEL_GAVE_UP = 1, SEL_NEVER_READY = 2 };

template <typename RAW>
__device__ inline SelOutcome select_fused_body(const RAW *__restrict__ x, int64_t numel, int64_t nvf, int64_t vpc, uint32_t k,
                                         SelState *st, uint32_t *hist0, uint32_t *hist1, uint32_t *table,
                                         RAW *__restrict__ vals, int32_t *__restrict__ idx, uint32_t spin_limit,
                                         unsigned long long gen)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    constexpr uint32_t MASK = KeyTraits<RAW>::MASK;
    constexpr bool F32 = sizeof(RAW) == 4;
    constexpr int BITS1 = F32 ? 13 : 11, SHIFT1 = F32 ? 18 : 4;   // first digit
    constexpr int BITS2 = 13, SHIFT2 = 5;                         // second digit (fp32 only)
    constexpr int LAST_BITS = F32 ? 5 : 4;
    constexpr int LB = 1 << LAST_BITS;
    constexpr int NW = SEL_THREADS / WAVE;
    constexpr int TILE = SEL_THREADS * VEC;                       // elements per compaction tile
    // The histogram and the compaction staging buffers share storage: never live together.
    extern __shared__ __attribute__((aligned(16))) u32x4 dyn_smem[];
    u32x4 *res = dyn_smem;                                            // [FUSED_RES][SEL_THREADS]
    uint32_t *smem = reinterpret_cast<uint32_t *>(dyn_smem + FUSED_RES * SEL_THREADS);
    int32_t *stage_idx = reinterpret_cast<int32_t *>(smem);
    RAW *stage_val = reinterpret_cast<RAW *>(smem + TILE);
    __shared__ uint32_t bcast[4];
    __shared__ uint32_t wave_tot[NW];
    __shared__ uint32_t wave_tot2[2 * NW];
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const int G = gridDim.x;
    const bool last_chunk = blockIdx.x == gridDim.x - 1;
    const u32x4 *xv = reinterpret_cast<const u32x4 *>(x);
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * vpc;
    const int64_t v1 = min(v0 + vpc, nvf);

    // development builds only: phase time stamps of one workgroup into the state block's spare words
    [[maybe_unused]] unsigned long long *stamps = reinterpret_cast<unsigned long long *>(st->pad + 6);
#define STAMP(i) DROPIT_DEV_STAMP(stamps, i, tid == 0 && blockIdx.x == gridDim.x / 2)
    STAMP(0);

    const bool sampling = !F32 && numel >= SAMPLE_MIN_NUMEL;       // uniform over the grid
    // The threshold lies in the key range [key_lo, key_lo + nf): predicted from the sample here (16-bit
    // types, large tensors), else (or if the prediction fails) exactly known after the digit histograms.
    uint32_t key_lo = 0, nf = LB;
    bool predicted = false;

    // ---- the staged form's geometry: wavefront `wave` owns vectors [wv0, wv1) of the chunk --------------
    const int wave = __builtin_amdgcn_readfirstlane(tid / WAVE);
    const int64_t vpw = ((vpc + NW - 1) / NW + 7) / 8 * 8;          // wavefront ranges start on 128-byte lines
    const int64_t wv0 = min(v0 + int64_t(wave) * vpw, v1), wv1 = min(wv0 + vpw, v1);
    const int nblk = static_cast<int>((wv1 - wv0 + ST_BLKV - 1) / ST_BLKV);
    // uniform over the grid: a position within a wavefront's range must fit the 16 bits of a staged word
    bool staged = !F32 && sampling && vpw * VEC <= 65536;
    char *dyn_bytes = reinterpret_cast<char *>(dyn_smem);
    uint32_t *lh = staged ? reinterpret_cast<uint32_t *>(dyn_bytes + ST_LH_OFF) : smem;
    uint32_t *seg = reinterpret_cast<uint32_t *>(dyn_bytes + ST_STAGE_OFF) + wave * ST_SEGCAP;
    __shared__ uint32_t wcount[NW];                                  // staged words per wavefront
    __shared__ uint32_t whist[F32 ? 1 : NW][MAX_LAST_BINS + 1];      // per wavefront: staged keys on each key of the range, and above it
    __shared__ uint32_t overflow;                                    // some wavefront's segment was too small
    u32x4 qa[ST_U], qb[ST_U];                                        // two blocks of the wavefront's range in flight
    auto issue_block = [&](u32x4 (&q)[ST_U], int blk) {
#pragma unroll
        for (int u = 0; u < ST_U; ++u)
            q[u] = xv[min(wv0 + int64_t(blk) * ST_BLKV + u * WAVE + lane, nvf - 1)];
    };

    // ---- park the head of the chunk in LDS (each thread only ever reads its own slots) --
    int nres = 0;
    auto park = [&]() {
        nres = static_cast<int>(min<int64_t>(FUSED_RES, (max<int64_t>(v1 - v0, 0) + SEL_THREADS - 1) / SEL_THREADS));
        if (nvf > 0) {
            u32x4 q[FUSED_RES];
#pragma unroll
            for (int i = 0; i < FUSED_RES; ++i)     // unconditional, clamped: all loads in flight at once
                q[i] = xv[min(v0 + int64_t(i) * SEL_THREADS + tid, nvf - 1)];
#pragma unroll
            for (int i = 0; i < FUSED_RES; ++i) res[i * SEL_THREADS + tid] = q[i];
        }
    };
    {
        u32x4 q[FUSED_RES];
        u32x4 sq[SAMPLE_VECTORS_PER_THREAD];
        if (staged) {
            if (nblk > 0) issue_block(qa, 0);
            if (nblk > 1) issue_block(qb, 1);
        } else if (nvf > 0) {
            nres = static_cast<int>(min<int64_t>(FUSED_RES, (max<int64_t>(v1 - v0, 0) + SEL_THREADS - 1) / SEL_THREADS));
#pragma unroll
            for (int i = 0; i < FUSED_RES; ++i)     // unconditional, clamped: all loads in flight at once
                q[i] = xv[min(v0 + int64_t(i) * SEL_THREADS + tid, nvf - 1)];
        }
        if (sampling) {
#pragma unroll
            for (int j = 0; j < SAMPLE_VECTORS_PER_THREAD; ++j)
                sq[j] = xv[sample_piece((j * SEL_THREADS + tid) / SAMPLE_PIECE,
                                        SAMPLE_VECTORS_PER_THREAD * SEL_THREADS / SAMPLE_PIECE, nvf) + tid % SAMPLE_PIECE];
        }
        // Workgroup 0 clears what the workgroups exchange through (histograms, barrier counters) while its
        // loads are in flight, then publishes this call's generation number; the others look for it before
        // their first global atomic.  No separate clearing kernel, and a workspace with arbitrary contents
        // is fine: a stale word equals the generation (a per-process random number plus a call count)
        // with probability 2^-64.  Device-scope atomic stores, like everything else that is exchanged.
        if (blockIdx.x == 0) {
            // only the bins this element type uses: bf16 one 2048-bin pass, fp32 two 8192-bin passes (hist1 follows hist0)
            constexpr int CLEAR_WORDS = F32 ? 2 * (1 << MAX_HIST_BITS) : (1 << BITS1);
            for (int i = tid; i < CLEAR_WORDS; i += SEL_THREADS) dev_store(hist0 + i, 0u);
            if (tid == 0) {
                dev_store(&st->barrier, 0u);
                dev_store(&st->error, 0u);
                dev_store(&st->exited, 0u);
                dev_store(&st->redo, 0u);
                dev_store(&st->staged, 0u);
            }
            if (tid < 8)
                dev_store(reinterpret_cast<uint32_t *>(reinterpret_cast<char *>(st) + SelWorkspace::xbar_off) + tid * 64, 0u);
            __syncthreads();                    // every wave has waited for its stores
            if (tid == 0) dev_store64(&st->ready, gen);
        }
        if (!staged && nvf > 0) {
#pragma unroll
            for (int i = 0; i < FUSED_RES; ++i) res[i * SEL_THREADS + tid] = q[i];
        }
        STAMP(8);
        if (sampling) {
            constexpr int NB = 1 << BITS1;
            // the sample's histogram: where the digit histograms live, which in the staged form lies behind
            // the transposition buffers and reaches into the (still empty) staging segments
            for (int i = tid; i < NB + WAVE; i += SEL_THREADS) lh[i] = 0;
            __syncthreads();
#pragma unroll
            for (int j = 0; j < SAMPLE_VECTORS_PER_THREAD; ++j)
                for_each_raw(RAW(0), sq[j], [&](uint32_t raw, int) {
                    const uint32_t dgt = ((raw & MASK) >> SHIFT1) & (NB - 1);
                    atomicAdd(&lh[dgt ? dgt : NB + lane], 1u);          // exact zeros go to per-lane slots
                });
            __syncthreads();
            STAMP(9);
            if (tid < WAVE) {
                const uint32_t z = wave_sum(lh[NB + tid]);
                if (tid == 0) lh[0] += z;
            }
            __syncthreads();
            uint32_t b_lo, b_hi;
            predicted = sample_bracket<NB>(lh, k, numel, wave_tot, bcast, b_lo, b_hi);
            if (predicted) {
                key_lo = b_lo << SHIFT1;                                // a first-digit bin is 2^SHIFT1 = 2^LAST_BITS keys
                nf = (b_hi - b_lo + 1) << SHIFT1;
            }
        }
        if (staged && !predicted) {     // no usable bracket (uniform over the grid): the exact form, with the head parked after all
            staged = false;
            lh = smem;
            park();
        }
    }
    const int64_t v_stream = v0 + int64_t(nres) * SEL_THREADS;        // first vector that is not parked
    // visits the chunk: fv(vector) for every full 16-byte vector, ft(raw bits) for the ragged tail's elements
    auto for_chunk_v = [&](auto fv, auto ft) {
        for (int i = 0; i < nres; ++i) {
            const int64_t v = v0 + int64_t(i) * SEL_THREADS + tid;
            if (v < v1) fv(res[i * SEL_THREADS + tid]);
        }
        int64_t vb = v_stream;
        for (; vb + SEL_THREADS * SEL_UNROLL <= v1; vb += SEL_THREADS * SEL_UNROLL) {
            u32x4 q[SEL_UNROLL];
#pragma unroll
            for (int u = 0; u < SEL_UNROLL; ++u) q[u] = xv[vb + u * SEL_THREADS + tid];
#pragma unroll
            for (int u = 0; u < SEL_UNROLL; ++u) fv(q[u]);
        }
        for (int64_t v = vb + tid; v < v1; v += SEL_THREADS) fv(xv[v]);
        if (last_chunk && tid == 0)
            for (int64_t i = nvf * VEC; i < numel; ++i) ft(x[i]);
    };
    // visits every element of the chunk: f(raw bits)
    auto for_chunk = [&](auto f) {
        for_chunk_v([&](const u32x4 &q) { for_each_raw(RAW(0), q, [&](uint32_t raw, int) { f(raw); }); }, f);
    };

    uint32_t prefix = 0, k_rem = k;
    uint32_t barriers = 0;
    uint32_t *xbar = reinterpret_cast<uint32_t *>(reinterpret_cast<char *>(st) + SelWorkspace::xbar_off);

    // ---- digit histograms ---------------------------------------------------------
    __shared__ uint32_t verdict;
    __shared__ uint32_t offs[2];
    __shared__ uint32_t lp[MAX_LAST_BINS + 1];
    // Waits until workgroup 0 has published this call's generation number: the exchange area is then
    // cleared.  False (in every thread) if that never happens.
    bool ready_seen = false;
    auto wait_ready = [&]() -> bool {
        if (ready_seen) return true;
        if (tid == 0) {
            uint32_t spins = 0, ok = 1;
            while (dev_load64(&st->ready) != gen) {
                if (++spins > READY_SPIN_LIMIT) {      // workgroup 0 never ran: not this workgroup's patience setting
                    ok = 0;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            bcast[3] = ok;
        }
        __syncthreads();
        ready_seen = bcast[3] != 0;
        return ready_seen;
    };
    // One digit's histogram of the chunk, merged into ghist; ends with a grid barrier, after which
    // ghist holds the whole tensor's histogram.
    auto hist_pass = [&](auto shift_c, auto bits_c, auto first_c, uint32_t *ghist) -> SelOutcome {
        constexpr int SHIFT = decltype(shift_c)::value, BITS = decltype(bits_c)::value;
        constexpr bool FIRST = decltype(first_c)::value;
        constexpr int NB = 1 << BITS;
        for (int i = tid; i < NB + 2 * WAVE; i += SEL_THREADS) lh[i] = 0;
        __syncthreads();
        const uint32_t zslot = NB + lane, dslot = NB + WAVE + lane;
        auto add = [&](uint32_t raw) {
            const uint32_t key = raw & MASK;
            const uint32_t d = (key >> SHIFT) & (NB - 1);
            uint32_t a = d ? d : zslot;
            if (!FIRST) a = ((key >> (SHIFT + BITS)) == prefix) ? a : dslot;
            atomicAdd(&lh[a], 1u);
        };
        for_chunk(add);
        __syncthreads();
        if (tid < WAVE) {
            const uint32_t z = wave_sum(lh[NB + tid]);
            if (tid == 0) lh[0] += z;
        }
        __syncthreads();
        if (!wait_ready()) return SEL_NEVER_READY;      // the exchange area must have been cleared for this call
        for (int i = tid; i < NB; i += SEL_THREADS) {
            const uint32_t c = lh[i];
            if (c) atomicAdd(&ghist[i], c);
        }
        if (!grid_barrier(st, xbar, ++barriers, spin_limit, &bcast[3])) return SEL_GAVE_UP;
        return SEL_DONE;
    };

    bool missed = false;
    bool use_staged = false;     // this workgroup's candidates are all staged in LDS (uniform over the workgroup)
    STAMP(1);
    uint32_t t = 0, m = 0;
    for (;;) {
        if (!predicted) {
            // exact digits
            prefix = 0;
            k_rem = k;
            if (const SelOutcome o = hist_pass(std::integral_constant<int, SHIFT1>{}, std::integral_constant<int, BITS1>{},
                                               std::true_type{}, hist0))
                return o;
            resolve_digit_local<(1 << BITS1), BITS1>(hist0, prefix, k_rem, wave_tot, bcast);
            if constexpr (F32) {
                if (const SelOutcome o = hist_pass(std::integral_constant<int, SHIFT2>{}, std::integral_constant<int, BITS2>{},
                                                   std::false_type{}, hist1))
                    return o;
                resolve_digit_local<(1 << BITS2), BITS2>(hist1, prefix, k_rem, wave_tot, bcast);
            }
            key_lo = prefix << LAST_BITS;
            nf = LB;
            STAMP(2);
        }

        // ---- exact counts over the range and above it, per chunk ----------------------
        for (int i = tid; i <= static_cast<int>(nf); i += SEL_THREADS) lh[i] = 0;
        if (tid == 0) overflow = 0;
        __syncthreads();
        bool counted = false;
        if constexpr (!F32) {
            if (staged && predicted) {
                // One pass over the wavefront's range: candidates (key >= key_lo) staged in flat-index order.
                const uint32_t key_lo_s = __builtin_amdgcn_readfirstlane(key_lo);
                char *tb = dyn_bytes + wave * ST_TRANS_BYTES;                   // this wavefront's transposition buffer
                char *mine = tb + lane * (ST_U * 16) + ((lane * ST_U) >> 3) * 16;   // this lane's ST_U consecutive vectors in it
                uint32_t n_w = 0;
                bool full = false;
                auto process = [&](u32x4 (&q)[ST_U], int blk) {
#pragma unroll
                    for (int u = 0; u < ST_U; ++u) {
                        const int vi = u * WAVE + lane;                        // as loaded: lane after lane
                        *reinterpret_cast<u32x4 *>(tb + vi * 16 + (vi >> 3) * 16) = q[u];
                    }
                    if (blk + 2 < nblk) issue_block(q, blk + 2);               // the registers are free again
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");     // a wavefront's LDS accesses execute in order
                    u32x4 r[ST_U];
#pragma unroll
                    for (int u = 0; u < ST_U; ++u) r[u] = *reinterpret_cast<const u32x4 *>(mine + u * 16);
                    uint32_t mask = candidate_mask(r, key_lo_s);
                    // whole vectors past the end of the wavefront's range are not there
                    const int64_t left = (wv1 - wv0 - int64_t(blk) * ST_BLKV) - int64_t(lane) * ST_U;
                    if (left < ST_U) mask &= left <= 0 ? 0u : (1u << (static_cast<int>(left) * VEC)) - 1u;
                    const uint32_t cnt = __builtin_popcount(mask);
                    const uint32_t incl = wave_inclusive_scan(cnt);
                    const uint32_t total = uint32_t(__builtin_amdgcn_readlane(int(incl), WAVE - 1));
                    if (n_w + total > uint32_t(ST_SEGCAP)) {
                        full = true;
                        return;
                    }
                    uint32_t slot = n_w + incl - cnt;
                    const uint32_t pos0 = static_cast<uint32_t>(blk) * (ST_BLKV * VEC) + lane * ST_EPL;
                    while (mask) {
                        const int b = __builtin_ctz(mask);
                        mask &= mask - 1;
                        const uint32_t raw = *reinterpret_cast<const uint16_t *>(mine + 2 * b);
                        seg[slot++] = (raw << 16) | (pos0 + b);
                    }
                    n_w += total;
                };
                for (int blk = 0; blk < nblk && !full; blk += 2) {
                    process(qa, blk);
                    if (blk + 1 < nblk && !full) process(qb, blk + 1);
                }
                if (lane == 0) {
                    wcount[wave] = n_w;
                    if (full) overflow = 1u;
                }
                __syncthreads();
                STAMP(3);
                if (overflow == 0) {
                    // Exact counts from the staged words, per wavefront (whist[wave]: one counter per key of the
                    // range, the last one for the keys above it); four words per lane and read, the segment's
                    // capacity is a multiple of four.
                    const uint32_t key_end = key_lo + nf;
                    uint32_t *wh = whist[wave];
                    if (lane <= static_cast<int>(nf)) wh[lane] = 0;
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    uint32_t above = 0;
                    for (uint32_t q0 = 0; q0 < n_w; q0 += 4 * WAVE) {
                        const uint32_t q = q0 + lane * 4;
                        if (q < n_w) {
                            const u32x4 w4 = *reinterpret_cast<const u32x4 *>(seg + q);
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const uint32_t key = (w4[j] >> 16) & MASK;
                                const bool there = q + j < n_w;
                                above += (there && key >= key_end) ? 1u : 0u;
                                const uint32_t rel = key - key_lo;
                                if (there && rel < nf) atomicAdd(&wh[rel], 1u);
                            }
                        }
                    }
                    above = wave_sum(above);
                    if (lane == 0) atomicAdd(&wh[nf], above);
                    __syncthreads();
                    if (tid <= static_cast<int>(nf)) {        // the workgroup's row of the table: the wavefronts' counts added up
                        uint32_t sum = 0;
#pragma unroll
                        for (int w2 = 0; w2 < NW; ++w2) sum += whist[w2][tid];
                        lh[tid] = sum;
                    }
                    if (last_chunk) {                          // the tensor's ragged end belongs to the chunk, but to no wavefront's range
                        __syncthreads();
                        if (tid == 0)
                            for (int64_t i = nvf * VEC; i < numel; ++i) {
                                const uint32_t key = x[i] & MASK;
                                if (key >= key_end) lh[nf] += 1u;
                                else if (key - key_lo < nf) lh[key - key_lo] += 1u;
                            }
                    }
                    use_staged = true;
                    counted = true;
                }
            }
        }
        if (!counted) {
            // Few keys fall into the range, so unlike the digit histograms this pass branches: a
            // wavefront with no such key among its lanes skips the LDS atomic altogether (an LDS
            // atomic costs its issue cycles whatever the number of active lanes).
            uint32_t above = 0;
            const uint32_t key_end = key_lo + nf;
            auto one = [&](uint32_t raw) {
                const uint32_t key = raw & MASK;
                above += (key >= key_end) ? 1u : 0u;
                const uint32_t rel = key - key_lo;             // wraps to a huge value below the range
                if (rel < nf) atomicAdd(&lh[rel], 1u);
            };
            if constexpr (F32) {
                for_chunk(one);
            } else {
                // Two 15-bit keys per 32-bit word are classified together: adding 0x8000 - E to a key sets
                // its bit 15 iff key >= E, and neither half can carry into the other (E <= 0x8000).
                const uint32_t c_end = (0x8000u - key_end) * 0x00010001u;
                const uint32_t c_lo = (0x8000u - key_lo) * 0x00010001u;
                for_chunk_v(
                    [&](const u32x4 &q) {
                        uint32_t kw[4], in_range[4], any = 0;
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            kw[w] = q[w] & 0x7FFF7FFFu;
                            const uint32_t ge_end = kw[w] + c_end, ge_lo = kw[w] + c_lo;
                            above += __builtin_popcount(ge_end & 0x80008000u);
                            in_range[w] = (ge_lo ^ ge_end) & 0x80008000u;     // >= key_lo and not >= key_end
                            any |= in_range[w];
                        }
                        if (any) {
#pragma unroll
                            for (int w = 0; w < 4; ++w) {
                                if (in_range[w] & 0x8000u) atomicAdd(&lh[(kw[w] & 0xFFFFu) - key_lo], 1u);
                                if (in_range[w] & 0x80000000u) atomicAdd(&lh[(kw[w] >> 16) - key_lo], 1u);
                            }
                        }
                    },
                    one);
            }
            above = wave_sum(above);
            if (lane == 0 && above) atomicAdd(&lh[nf], above);
        }
        __syncthreads();
        if (!wait_ready()) return SEL_NEVER_READY;      // (already seen, unless the range was predicted)
        if (tid <= static_cast<int>(nf)) dev_store(&table[tid * G + blockIdx.x], lh[tid]);
        STAMP(4);
        if (!grid_barrier(st, xbar, ++barriers, spin_limit, &bcast[3])) return SEL_GAVE_UP;
        STAMP(5);

        // Per row of the table (a key of the range; the last row = the keys above the range): the total
        // over all chunks and the part in the chunks before this one, one wavefront per row.
        {
            // every wavefront takes up to ROWS rows (wave, wave + NW, ...); all their loads are issued together
            constexpr int ROWS = (MAX_LAST_BINS + 1 + NW - 1) / NW;
            constexpr int COLS = SEL_MAX_CHUNKS / WAVE;
            const int wave = tid / WAVE;
            uint32_t v[ROWS][COLS];
#pragma unroll
            for (int r = 0; r < ROWS; ++r)
#pragma unroll
                for (int j = 0; j < COLS; ++j) {
                    const int row = wave + r * NW, c = lane + j * WAVE;
                    v[r][j] = (row <= static_cast<int>(nf) && c < G) ? dev_load(&table[row * G + c]) : 0u;
                }
#pragma unroll
            for (int r = 0; r < ROWS; ++r) {
                const int row = wave + r * NW;
                if (row > static_cast<int>(nf)) break;         // uniform over the wavefront
                uint32_t s = 0, sp = 0;
#pragma unroll
                for (int j = 0; j < COLS; ++j) {
                    s += v[r][j];
                    sp += (lane + j * WAVE < static_cast<int>(blockIdx.x)) ? v[r][j] : 0u;
                }
                s = wave_sum(s);
                sp = wave_sum(sp);
                if (lane == 0) {
                    lh[row] = s;
                    lp[row] = sp;
                }
            }
        }
        __syncthreads();
        if (tid < WAVE) {
            // Lane 0 takes the row above the range, lanes 1.. the range's keys in descending order, so a
            // prefix scan over the lanes counts the keys above each key.  The k-th largest key is the one
            // with  #above < k <= #above + #equal;  it is in the range iff that holds for a lane >= 1.
            const int rr = static_cast<int>(nf) - lane;
            const uint32_t full = rr >= 0 ? lh[rr] : 0u, part = rr >= 0 ? lp[rr] : 0u;
            const uint32_t incl = wave_inclusive_scan(full), incl_p = wave_inclusive_scan(part);
            const bool here = lane >= 1 && rr >= 0 && incl - full < k && k <= incl;
            const unsigned long long hit = __ballot(here);
            if (lane == 0) verdict = hit ? 1u : 0u;
            if (here) {
                bcast[0] = key_lo + static_cast<uint32_t>(rr);   // t
                bcast[1] = k - (incl - full);                     // m: how many keys equal to t are kept
                offs[0] = incl_p - part;                          // #{key > t} in the chunks before this one
                offs[1] = part;                                   // #{key == t} there
            }
        }
        __syncthreads();
        if (verdict) break;
        if (!predicted) return SEL_GAVE_UP;     // cannot happen with exact digits; the serial path would still answer
        predicted = false;                       // the sample misled: once more with the exact histogram
        missed = true;
        use_staged = false;
        __syncthreads();                         // everybody has read the verdict before it is written again
    }
    t = bcast[0];
    m = bcast[1];
    if (blockIdx.x == 0 && tid == 0) dev_store(&st->path, missed ? 2u : predicted ? 1u : 0u);
    uint32_t run_gt = offs[0], run_eq = offs[1];   // #{key > t}, #{key == t} before this chunk
    STAMP(6);

    // ---- ordered compaction -------------------------------------------------------
    // The kept elements of a tile occupy consecutive output slots; they are gathered in
    // LDS first so that the global stores are contiguous.
    auto keep = [&](uint32_t pos, uint32_t raw, int64_t i) {
        if (pos < k) {                     // always true for consistent counts
            vals[pos] = static_cast<RAW>(raw);
            idx[pos] = static_cast<int32_t>(i);
        }
    };
    auto emit_tile = [&](const u32x4 &q, int64_t v, bool live) {
        // bit e of gtm / eqm: element e of this thread's vector has key > t / key == t
        uint32_t gtm = 0, eqm = 0;
        for_each_raw(RAW(0), q, [&](uint32_t raw, int e) {
            const uint32_t key = raw & MASK;
            gtm |= (key > t ? 1u : 0u) << e;
            eqm |= (key == t ? 1u : 0u) << e;
        });
        if (!live) gtm = eqm = 0;
        const uint32_t cnt = __builtin_popcount(gtm) | (__builtin_popcount(eqm) << 16);
        uint32_t total;
        const uint32_t excl = block_exclusive_scan<SEL_THREADS>(cnt, wave_tot, total);
        const uint32_t tile_first = run_gt + min(run_eq, m);           // output slot of the tile's first kept element
        uint32_t my_gt = run_gt + (excl & 0xFFFFu);
        uint32_t my_eq = run_eq + (excl >> 16);
        const int64_t base = v * VEC;
        // A kept element (key > t, or one of the first m keys == t) goes to output slot
        // #gt-before + min(#eq-before, m): one formula for both cases.  Only the candidate
        // elements are visited (a tenth of them at gamma = 0.9): every LDS store a wavefront
        // issues costs its slot on the LDS pipe however few lanes take part.
        uint32_t todo = gtm | eqm;
        while (todo) {
            const int e = __builtin_ctz(todo);
            todo &= todo - 1;
            const bool gt = (gtm >> e) & 1u;
            if (gt || my_eq < m) {
                const uint32_t slot = my_gt + min(my_eq, m) - tile_first;
                uint32_t raw;
                if constexpr (F32) raw = q[e];
                else raw = (q[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
                stage_val[slot] = static_cast<RAW>(raw);
                stage_idx[slot] = static_cast<int32_t>(base + e);
            }
            my_gt += gt ? 1u : 0u;
            my_eq += gt ? 0u : 1u;
        }
        run_gt += total & 0xFFFFu;
        run_eq += total >> 16;
        const uint32_t tile_kept = run_gt + min(run_eq, m) - tile_first;
        __syncthreads();
        for (uint32_t s = tid; s < tile_kept; s += SEL_THREADS)
            if (tile_first + s < k) {      // always true for consistent counts
                vals[tile_first + s] = stage_val[s];
                idx[tile_first + s] = stage_idx[s];
            }
        // the next tile's scan starts with a barrier, which also protects the staging buffers
    };
    bool compacted = false;
    if constexpr (!F32) {
        if (use_staged) {
            // ---- compaction from the staged candidates: x is not read again ----
            const uint32_t n_w = wcount[wave];
            // #{key > t}, #{key == t} in the wavefronts' ranges, from their histograms: lane l adds up wavefront l's
            const uint32_t trel = t - key_lo;
            uint32_t g = 0, e = 0;
            if (lane < NW) {
                g = whist[lane][nf];
                for (uint32_t r = trel + 1; r < nf; ++r) g += whist[lane][r];
                e = whist[lane][trel];
            }
            const uint32_t gi = wave_inclusive_scan(g), ei = wave_inclusive_scan(e);
            uint32_t my_gt = run_gt + uint32_t(__builtin_amdgcn_readlane(int(gi - g), wave));
            uint32_t my_eq = run_eq + uint32_t(__builtin_amdgcn_readlane(int(ei - e), wave));
            run_gt += uint32_t(__builtin_amdgcn_readlane(int(gi), NW - 1));
            run_eq += uint32_t(__builtin_amdgcn_readlane(int(ei), NW - 1));
            const uint32_t flat0 = static_cast<uint32_t>(wv0 * VEC);
            for (uint32_t q0 = 0; q0 < n_w; q0 += 4 * WAVE) {
                const uint32_t q = q0 + lane * 4;
                u32x4 w4 = {0u, 0u, 0u, 0u};
                if (q < n_w) w4 = *reinterpret_cast<const u32x4 *>(seg + q);
                uint32_t gtm = 0, eqm = 0;                 // bit j: word j of this lane has key > t / key == t
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t key = (w4[j] >> 16) & MASK;
                    const bool there = q + j < n_w;
                    gtm |= (there && key > t) ? (1u << j) : 0u;
                    eqm |= (there && key == t) ? (1u << j) : 0u;
                }
                const uint32_t both = __builtin_popcount(gtm) | (__builtin_popcount(eqm) << 16);
                const uint32_t incl = wave_inclusive_scan(both);
                const uint32_t tot = uint32_t(__builtin_amdgcn_readlane(int(incl), WAVE - 1));
                uint32_t gb = my_gt + ((incl - both) & 0xFFFFu), eb = my_eq + ((incl - both) >> 16);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool gt = (gtm >> j) & 1u, eq = (eqm >> j) & 1u;
                    if (gt || (eq && eb < m)) keep(gb + min(eb, m), w4[j] >> 16, int64_t(flat0) + (w4[j] & 0xFFFFu));
                    gb += gt ? 1u : 0u;
                    eb += eq ? 1u : 0u;
                }
                my_gt += tot & 0xFFFFu;
                my_eq += tot >> 16;
            }
            if (tid == 0) __hip_atomic_fetch_add(&st->staged, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            compacted = true;
        }
    }
    if (!compacted) {
        __syncthreads();                       // histogram storage becomes staging storage
        // The chunk is compacted in super-tiles of FUSED_RES x 1024 vectors that sit in the parking
        // area: the first one is the parked head itself, the following ones are fetched (coalesced,
        // one super-tile ahead, through registers) into the same area.  Inside a super-tile each thread
        // takes `rows` CONSECUTIVE vectors (the other phases take every 1024th), so flat-index order is
        // thread order and one block scan serves the whole super-tile: two barriers + a gather + a
        // write-out per 49152 elements.  Bit (i * VEC + e) of the masks stands for element e of the
        // thread's i-th vector.  A super-tile that keeps more than the staging buffers hold (only when
        // most of the tensor is kept) falls back to one scan per 1024-vector row.
        constexpr int64_t SUPER = int64_t(FUSED_RES) * SEL_THREADS;
        auto fetch = [&](u32x4 (&pre)[FUSED_RES], int64_t sb) {       // vectors [sb, sb + SUPER) n [.., v1), clamped loads
    #pragma unroll
            for (int i = 0; i < FUSED_RES; ++i)
                pre[i] = (sb < v1) ? xv[min(sb + int64_t(i) * SEL_THREADS + tid, v1 - 1)] : u32x4{0, 0, 0, 0};
        };
        u32x4 pre[FUSED_RES];
        if (nres == 0 && v0 < v1) {            // nothing was parked (the staged form was abandoned): fetch the first super-tile now
            fetch(pre, v0);
    #pragma unroll
            for (int i = 0; i < FUSED_RES; ++i) res[i * SEL_THREADS + tid] = pre[i];
            __syncthreads();
        }
        for (int64_t sb = v0; sb < v1; sb += SUPER) {
            const int64_t count = min<int64_t>(v1 - sb, SUPER);          // vectors of this super-tile, all in `res`
            const int rows = static_cast<int>((count + SEL_THREADS - 1) / SEL_THREADS);
            const bool more = sb + SUPER < v1;
            if (more) fetch(pre, sb + SUPER);
            const int64_t mine0 = int64_t(tid) * rows;                    // first vector of this thread
            unsigned long long gtm = 0, eqm = 0;
    #pragma nounroll
            for (int i = 0; i < rows; ++i) {
                if (mine0 + i < count) {
                    uint32_t g = 0, q = 0;
                    for_each_raw(RAW(0), res[mine0 + i], [&](uint32_t raw, int e) {
                        const uint32_t key = raw & MASK;
                        g |= (key > t ? 1u : 0u) << e;
                        q |= (key == t ? 1u : 0u) << e;
                    });
                    gtm |= static_cast<unsigned long long>(g) << (i * VEC);
                    eqm |= static_cast<unsigned long long>(q) << (i * VEC);
                }
            }
            uint32_t ex_gt, ex_eq, tot_gt, tot_eq;
            block_exclusive_scan2<SEL_THREADS>(__builtin_popcountll(gtm), __builtin_popcountll(eqm), wave_tot2, ex_gt, ex_eq,
                                               tot_gt, tot_eq);
            const uint32_t part_first = run_gt + min(run_eq, m);
            const uint32_t part_kept = (run_gt + tot_gt) + min(run_eq + tot_eq, m) - part_first;
            // 16-bit elements are staged as ONE word each, value << 16 | position within the super-tile,
            // so the staging area holds half as many again (a super-tile that keeps a fifth of its
            // elements still fits) and the scatter issues one LDS store per kept element.
            constexpr bool PACKED = !F32;
            static_assert(F32 || SUPER * VEC <= 65536, "a position within a super-tile fits 16 bits");
            constexpr uint32_t STAGE_CAP = PACKED ? uint32_t(TILE + TILE / 2) : uint32_t(TILE);
            if (part_kept <= STAGE_CAP) {                                  // uniform over the workgroup
                uint32_t my_gt = run_gt + ex_gt, my_eq = run_eq + ex_eq;
                const RAW *res_raw = reinterpret_cast<const RAW *>(res);
                uint32_t *stage_pk = smem;
                unsigned long long todo = gtm | eqm;
                while (todo) {
                    const int b = __builtin_ctzll(todo);
                    todo &= todo - 1;
                    const bool gt = (gtm >> b) & 1ull;
                    if (gt || my_eq < m) {
                        const uint32_t slot = my_gt + min(my_eq, m) - part_first;
                        const uint32_t off = static_cast<uint32_t>(mine0) * VEC + b;
                        if constexpr (PACKED) {
                            stage_pk[slot] = (static_cast<uint32_t>(res_raw[off]) << 16) | off;
                        } else {
                            stage_val[slot] = res_raw[off];
                            stage_idx[slot] = static_cast<int32_t>(sb * VEC + off);
                        }
                    }
                    my_gt += gt ? 1u : 0u;
                    my_eq += gt ? 0u : 1u;
                }
                run_gt += tot_gt;
                run_eq += tot_eq;
                __syncthreads();
                for (uint32_t q = tid; q < part_kept; q += SEL_THREADS)
                    if (part_first + q < k) {          // always true for consistent counts
                        if constexpr (PACKED) {
                            const uint32_t w = stage_pk[q];
                            vals[part_first + q] = static_cast<RAW>(w >> 16);
                            idx[part_first + q] = static_cast<int32_t>(sb * VEC + (w & 0xFFFFu));
                        } else {
                            vals[part_first + q] = stage_val[q];
                            idx[part_first + q] = stage_idx[q];
                        }
                    }
            } else {
                for (int i = 0; i < rows; ++i) {       // row by row; a row's scan starts with a barrier, which frees the staging buffers
                    const int64_t v = sb + int64_t(i) * SEL_THREADS + tid;
                    emit_tile(res[i * SEL_THREADS + tid], v, v < v1);
                }
            }
            if (more) {
                __syncthreads();                       // everybody is done with this super-tile's vectors and staging
    #pragma unroll
                for (int i = 0; i < FUSED_RES; ++i) res[i * SEL_THREADS + tid] = pre[i];
                __syncthreads();
            }
        }
    }
    STAMP(7);
    if (last_chunk && tid == 0) {
        for (int64_t i = nvf * VEC; i < numel; ++i) {
            const RAW raw = x[i];
            const uint32_t key = raw & MASK;
            if (key > t) {
                keep(run_gt + min(run_eq, m), raw, i);
                ++run_gt;
            } else if (key == t) {
                if (run_eq < m) keep(run_gt + run_eq, raw, i);
                ++run_eq;
            }
        }
    }
#undef STAMP
    return SEL_DONE;
}

// The whole selection by ONE workgroup, phase after phase over the whole tensor: same digits,
// same slot formula, histograms in LDS, nothing read from the workspace.  Only ever runs after
// the parallel path gave up.  `lh` is LDS scratch of (1 << 13) + 2 * WAVE words.
template <typename RAW>
__device__ inline void select_serial(const RAW *__restrict__ x, int64_t numel, int64_t nvf, uint32_t k,
                                     RAW *__restrict__ vals, int32_t *__restrict__ idx, uint32_t *lh,
                                     uint32_t *wave_tot, uint32_t *bcast)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    constexpr uint32_t MASK = KeyTraits<RAW>::MASK;
    constexpr bool F32 = sizeof(RAW) == 4;
    constexpr int LAST_BITS = F32 ? 5 : 4;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const u32x4 *xv = reinterpret_cast<const u32x4 *>(x);
    auto for_all = [&](auto f) {
        for (int64_t v = tid; v < nvf; v += SEL_THREADS)
            for_each_raw(RAW(0), xv[v], [&](uint32_t raw, int) { f(raw); });
        if (tid == 0)
            for (int64_t i = nvf * VEC; i < numel; ++i) f(x[i]);
    };
    uint32_t prefix = 0, k_rem = k;
    auto pass = [&](auto shift_c, auto bits_c, auto first_c) {
        constexpr int SHIFT = decltype(shift_c)::value, BITS = decltype(bits_c)::value;
        constexpr bool FIRST = decltype(first_c)::value;
        constexpr int NB = 1 << BITS;
        __syncthreads();
        for (int i = tid; i < NB + 2 * WAVE; i += SEL_THREADS) lh[i] = 0;
        __syncthreads();
        const uint32_t zslot = NB + lane, dslot = NB + WAVE + lane;
        for_all([&](uint32_t raw) {
            const uint32_t key = raw & MASK;
            const uint32_t d = (key >> SHIFT) & (NB - 1);
            uint32_t a = d ? d : zslot;
            if (!FIRST) a = ((key >> (SHIFT + BITS)) == prefix) ? a : dslot;
            atomicAdd(&lh[a], 1u);
        });
        __syncthreads();
        if (tid < WAVE) {
            const uint32_t z = wave_sum(lh[NB + tid]);
            if (tid == 0) lh[0] += z;
        }
        __syncthreads();
        resolve_digit_local<NB, BITS>(lh, prefix, k_rem, wave_tot, bcast);
    };
    if constexpr (F32) {
        pass(std::integral_constant<int, 18>{}, std::integral_constant<int, 13>{}, std::true_type{});
        pass(std::integral_constant<int, 5>{}, std::integral_constant<int, 13>{}, std::false_type{});
    } else {
        pass(std::integral_constant<int, 4>{}, std::integral_constant<int, 11>{}, std::true_type{});
    }
    pass(std::integral_constant<int, 0>{}, std::integral_constant<int, LAST_BITS>{}, std::false_type{});
    const uint32_t t = prefix, m = k_rem;   // all digits resolved: the threshold key and its tie budget

    uint32_t run_gt = 0, run_eq = 0;
    auto keep = [&](uint32_t pos, uint32_t raw, int64_t i) {
        if (pos < k) {
            vals[pos] = static_cast<RAW>(raw);
            idx[pos] = static_cast<int32_t>(i);
        }
    };
    for (int64_t vb = 0; vb < nvf; vb += SEL_THREADS) {
        const int64_t v = vb + tid;
        const bool live = v < nvf;
        u32x4 q = u32x4{0, 0, 0, 0};
        if (live) q = xv[v];
        uint32_t cnt = 0;                  // low 16 bits: #gt, high 16 bits: #eq (tile <= 8192 elements)
        for_each_raw(RAW(0), q, [&](uint32_t raw, int) {
            const uint32_t key = raw & MASK;
            cnt += (key > t ? 1u : 0u) + (key == t ? 0x10000u : 0u);
        });
        if (!live) cnt = 0;
        uint32_t total;
        const uint32_t excl = block_exclusive_scan<SEL_THREADS>(cnt, wave_tot, total);
        uint32_t my_gt = run_gt + (excl & 0xFFFFu);
        uint32_t my_eq = run_eq + (excl >> 16);
        if (cnt) {
            for_each_raw(RAW(0), q, [&](uint32_t raw, int e) {
                const uint32_t key = raw & MASK;
                const bool gt = key > t, eq = key == t;
                if (gt || (eq && my_eq < m)) keep(my_gt + min(my_eq, m), raw, v * VEC + e);
                my_gt += gt ? 1u : 0u;
                my_eq += eq ? 1u : 0u;
            });
        }
        run_gt += total & 0xFFFFu;
        run_eq += total >> 16;
    }
    if (tid == 0) {
        for (int64_t i = nvf * VEC; i < numel; ++i) {
            const RAW raw = x[i];
            const uint32_t key = raw & MASK;
            const bool gt = key > t, eq = key == t;
            if (gt || (eq && run_eq < m)) keep(run_gt + min(run_eq, m), raw, i);
            run_gt += gt ? 1u : 0u;
            run_eq += eq ? 1u : 0u;
        }
    }
}

// ---- small tensors: one workgroup, everything in registers ------------------------------------------
// Up to SMALL_VECTORS 16-byte vectors per thread (64 K fp32 or 128 K 16-bit elements): the tensor is read
// once into registers and the whole selection -- the same digits, tie rule and slot formula as above --
// runs in ONE workgroup with workgroup barriers only.  No workspace, no grid barrier, no residency
// question; at this size the 256-workgroup form spends its time on its own machinery (a 64 KB tensor took
// 22 us there).  Thread t holds vectors t, t + 1024, ...; the compaction goes row by row (1024 vectors).
constexpr int SMALL_VECTORS = 8;

template <typename RAW>
__global__ void __launch_bounds__(SEL_THREADS)
select_small_kernel(const RAW *__restrict__ x, int64_t numel, int nvf, uint32_t k, RAW *__restrict__ vals,
                    int32_t *__restrict__ idx)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    constexpr uint32_t MASK = KeyTraits<RAW>::MASK;
    constexpr bool F32 = sizeof(RAW) == 4;
    constexpr int LAST_BITS = F32 ? 5 : 4;
    __shared__ uint32_t lh[(1 << MAX_HIST_BITS) + 2 * WAVE];
    __shared__ uint32_t wave_tot[SEL_THREADS / WAVE];
    __shared__ uint32_t bcast[2];
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    const u32x4 *xv = reinterpret_cast<const u32x4 *>(x);
    const int rows = (nvf + SEL_THREADS - 1) / SEL_THREADS;          // <= SMALL_VECTORS (checked by the host)
    u32x4 q[SMALL_VECTORS];
#pragma unroll
    for (int i = 0; i < SMALL_VECTORS; ++i) {
        const int v = tid + i * SEL_THREADS;
        q[i] = v < nvf ? xv[v] : u32x4{0u, 0u, 0u, 0u};
    }
    auto for_all = [&](auto f) {
#pragma unroll
        for (int i = 0; i < SMALL_VECTORS; ++i)
            if (tid + i * SEL_THREADS < nvf) for_each_raw(RAW(0), q[i], [&](uint32_t raw, int) { f(raw); });
        if (tid == 0)
            for (int64_t i = int64_t(nvf) * VEC; i < numel; ++i) f(x[i]);
    };
    uint32_t prefix = 0, k_rem = k;
    auto pass = [&](auto shift_c, auto bits_c, auto first_c) {
        constexpr int SHIFT = decltype(shift_c)::value, BITS = decltype(bits_c)::value;
        constexpr bool FIRST = decltype(first_c)::value;
        constexpr int NB = 1 << BITS;
        __syncthreads();
        for (int i = tid; i < NB + 2 * WAVE; i += SEL_THREADS) lh[i] = 0;
        __syncthreads();
        const uint32_t zslot = NB + lane, dslot = NB + WAVE + lane;
        for_all([&](uint32_t raw) {
            const uint32_t key = raw & MASK;
            const uint32_t d = (key >> SHIFT) & (NB - 1);
            uint32_t a = d ? d : zslot;
            if (!FIRST) a = ((key >> (SHIFT + BITS)) == prefix) ? a : dslot;
            atomicAdd(&lh[a], 1u);
        });
        __syncthreads();
        if (tid < WAVE) {
            const uint32_t z = wave_sum(lh[NB + tid]);
            if (tid == 0) lh[0] += z;
        }
        __syncthreads();
        resolve_digit_local<NB, BITS>(lh, prefix, k_rem, wave_tot, bcast);
    };
    if constexpr (F32) {
        pass(std::integral_constant<int, 18>{}, std::integral_constant<int, 13>{}, std::true_type{});
        pass(std::integral_constant<int, 5>{}, std::integral_constant<int, 13>{}, std::false_type{});
    } else {
        pass(std::integral_constant<int, 4>{}, std::integral_constant<int, 11>{}, std::true_type{});
    }
    pass(std::integral_constant<int, 0>{}, std::integral_constant<int, LAST_BITS>{}, std::false_type{});
    const uint32_t t = prefix, m = k_rem;   // all digits resolved: the threshold key and its tie budget

    uint32_t run_gt = 0, run_eq = 0;
    auto keep = [&](uint32_t pos, uint32_t raw, int64_t i) {
        if (pos < k) {
            vals[pos] = static_cast<RAW>(raw);
            idx[pos] = static_cast<int32_t>(i);
        }
    };
#pragma unroll
    for (int i = 0; i < SMALL_VECTORS; ++i) {
        if (i < rows) {                        // uniform over the workgroup
            const int v = tid + i * SEL_THREADS;
            uint32_t cnt = 0;                  // low 16 bits: #gt, high 16 bits: #eq (a row is <= 8192 elements)
            if (v < nvf)
                for_each_raw(RAW(0), q[i], [&](uint32_t raw, int) {
                    const uint32_t key = raw & MASK;
                    cnt += (key > t ? 1u : 0u) + (key == t ? 0x10000u : 0u);
                });
            uint32_t total;
            const uint32_t excl = block_exclusive_scan<SEL_THREADS>(cnt, wave_tot, total);
            uint32_t my_gt = run_gt + (excl & 0xFFFFu);
            uint32_t my_eq = run_eq + (excl >> 16);
            if (cnt) {
                for_each_raw(RAW(0), q[i], [&](uint32_t raw, int e) {
                    const uint32_t key = raw & MASK;
                    const bool gt = key > t, eq = key == t;
                    if (gt || (eq && my_eq < m)) keep(my_gt + min(my_eq, m), raw, int64_t(v) * VEC + e);
                    my_gt += gt ? 1u : 0u;
                    my_eq += eq ? 1u : 0u;
                });
            }
            run_gt += total & 0xFFFFu;
            run_eq += total >> 16;
        }
    }
    if (tid == 0) {
        for (int64_t i = int64_t(nvf) * VEC; i < numel; ++i) {
            const RAW raw = x[i];
            const uint32_t key = raw & MASK;
            const bool gt = key > t, eq = key == t;
            if (gt || (eq && run_eq < m)) keep(run_gt + min(run_eq, m), raw, i);
            run_gt += gt ? 1u : 0u;
            run_eq += eq ? 1u : 0u;
        }
    }
}

template <typename RAW>
__global__ void __launch_bounds__(SEL_THREADS)
select_fused_kernel(const RAW *__restrict__ x, int64_t numel, int64_t nvf, int64_t vpc, uint32_t k, SelState *st,
                    uint32_t *hist0, uint32_t *hist1, uint32_t *table, RAW *__restrict__ vals,
                    int32_t *__restrict__ idx, uint32_t spin_limit, unsigned long long gen)
{
    const SelOutcome outcome =
        select_fused_body<RAW>(x, numel, nvf, vpc, k, st, hist0, hist1, table, vals, idx, spin_limit, gen);
    // Exit protocol: one atomic per workgroup counts the leavers and, in the high half, those that
    // gave up at a barrier.  The last to leave sees whether anybody did.  Everything the others stored
    // to the outputs before leaving is either final or missing, never wrong, and the serial pass below
    // uses no workspace, so it needs no ordering against their remaining traffic.
    // A workgroup that never saw the exchange area published (workgroup 0, although dispatched first,
    // did not get through its first few microseconds within the waiting time: not expected to happen)
    // cannot rely on the counter either and simply redoes the selection itself; several doing so
    // write identical bytes.
    extern __shared__ __attribute__((aligned(16))) u32x4 dyn_smem[];
    __shared__ uint32_t s_redo;
    __shared__ uint32_t s_wave_tot[SEL_THREADS / WAVE];
    __shared__ uint32_t s_bcast[2];
    __syncthreads();
    if (threadIdx.x == 0) {
        s_redo = 1u;
        if (outcome != SEL_NEVER_READY) {
            const uint32_t mine = outcome == SEL_DONE ? 1u : 0x10001u;
            const uint32_t seen = __hip_atomic_fetch_add(&st->exited, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + mine;
            const bool last = (seen & 0xFFFFu) == gridDim.x;
            s_redo = (last && (seen >> 16) != 0) ? 1u : 0u;
            if (last) {
                // Nobody looks at the exchange area any more: un-publish it, so that the next launch that carries the
                // same generation number (a replay of a captured graph) cannot take this call's leftovers for its own.
                dev_store64(&st->ready, 0ull);
                if (s_redo) dev_store(&st->redo, 1u);
            }
        }
    }
    __syncthreads();
    if (s_redo)
        select_serial<RAW>(x, numel, nvf, k, vals, idx, reinterpret_cast<uint32_t *>(dyn_smem), s_wave_tot, s_bcast);
}

// ---- random dropping (Sec. 3.3, Random Elements) ------------------------------------------------
// Philox4x32 with 10 rounds (Salmon et al., SC'11): per round, counter words 0 and 2 are multiplied by two
// odd constants and the halves of the products are crossed with the other two words and the key; the key
// advances by two Weyl constants between rounds.
__device__ inline void philox_round(uint32_t (&c)[4], uint32_t k0, uint32_t k1)
{
    const uint32_t hi0 = __umulhi(0xD2511F53u, c[0]), lo0 = 0xD2511F53u * c[0];
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c[2]), lo1 = 0xCD9E8D57u * c[2];
    c[0] = hi1 ^ c[1] ^ k0;
    c[1] = lo1;
    c[2] = hi0 ^ c[3] ^ k1;
    c[3] = lo0;
}

// keys[4b .. 4b+3] = the four words of block b, each shifted right by one (31-bit keys, so that the
// select's sign-cleared order of fp32 bit patterns is their integer order).  `blocks` 16-byte stores.
__global__ void __launch_bounds__(256) random_keys_kernel(uint4 *keys, int64_t blocks, uint32_t seed_lo,
                                                          uint32_t seed_hi)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t b = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; b < blocks; b += stride) {
        uint32_t c[4] = {static_cast<uint32_t>(b), 0u, 0u, 0u};
        uint32_t k0 = seed_lo, k1 = seed_hi;
#pragma unroll
        for (int round = 0; round < 10; ++round) {
            if (round > 0) {
                k0 += 0x9E3779B9u;
                k1 += 0xBB67AE85u;
            }
            philox_round(c, k0, k1);
        }
        keys[b] = make_uint4(c[0] >> 1, c[1] >> 1, c[2] >> 1, c[3] >> 1);
    }
}

template <typename RAW>
__global__ void __launch_bounds__(256) gather_kernel(const RAW *__restrict__ x, const int32_t *__restrict__ idx,
                                                     int64_t k, RAW *__restrict__ vals)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t j = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; j < k; j += stride)
        vals[j] = x[idx[j]];
}

inline size_t round_up_256(size_t v) { return (v + 255) / 256 * 256; }

// Workspace of the random strategy: the select's own area, one key per element (padded to whole Philox
// blocks), and the keys the select writes out beside the indices (unused afterwards).
struct RandomWorkspace {
    size_t keys_off, keyvals_off, bytes;
    explicit RandomWorkspace(int64_t numel)
    {
        const size_t key_bytes = round_up_256((static_cast<size_t>(numel) + 3) / 4 * 16);
        keys_off = round_up_256(SelWorkspace::bytes);
        keyvals_off = keys_off + key_bytes;
        bytes = keyvals_off + key_bytes;
    }
};

struct Geometry {
    int64_t nvf, vpc;      // full 16-byte vectors, vectors per chunk
    int chunks;
};

template <typename RAW>
Geometry geometry(int64_t numel)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    Geometry g;
    g.nvf = numel / VEC;
    int64_t chunks = (g.nvf + SEL_THREADS - 1) / SEL_THREADS;
    if (chunks > SEL_MAX_CHUNKS) chunks = SEL_MAX_CHUNKS;
    if (chunks < 1) chunks = 1;
    g.vpc = (g.nvf + chunks - 1) / chunks;
    g.vpc = (g.vpc + 7) / 8 * 8;           // chunk starts on 128-byte lines
    if (g.vpc < 8) g.vpc = 8;
    g.chunks = static_cast<int>((g.nvf + g.vpc - 1) / g.vpc);
    if (g.chunks < 1) g.chunks = 1;        // a tensor shorter than one vector still needs a workgroup
    return g;
}

// A number no earlier call of this process has used (a random start, then a count), never 0.
unsigned long long next_generation()
{
    static std::atomic<unsigned long long> counter{[] {
        std::random_device rd;
        return (static_cast<unsigned long long>(rd()) << 32) ^ rd();
    }()};
    unsigned long long g = counter.fetch_add(1) + 1;
    return g ? g : counter.fetch_add(1) + 1;
}

template <typename RAW>
dropit_status run_compress(const void *x, int64_t numel, int64_t k, void *vals, int32_t *idx,
                           char *ws, hipStream_t stream)
{
    const Geometry g = geometry<RAW>(numel);
    SelState *st = reinterpret_cast<SelState *>(ws + SelWorkspace::state_off);
    uint32_t *hist0 = reinterpret_cast<uint32_t *>(ws + SelWorkspace::hist0_off);
    uint32_t *hist1 = reinterpret_cast<uint32_t *>(ws + SelWorkspace::hist1_off);
    uint32_t *table = reinterpret_cast<uint32_t *>(ws + SelWorkspace::table_off);
    uint32_t *off_gt = reinterpret_cast<uint32_t *>(ws + SelWorkspace::offgt_off);
    uint32_t *off_eq = reinterpret_cast<uint32_t *>(ws + SelWorkspace::offeq_off);
    const RAW *xr = static_cast<const RAW *>(x);

    auto clear_state = [&]() {                 // the separate kernels' clearing pass
        trace_mark(stream);
        init_kernel<<<32, 256, 0, stream>>>(reinterpret_cast<uint32_t *>(ws),
                                            static_cast<uint32_t>(SelWorkspace::zero_bytes / 4),
                                            static_cast<uint32_t>(k));
    };
    const int mode = select_mode();
    // Small tensors (default mode only: the other modes are there to exercise the other forms): one workgroup.
    if (mode == 0 && numel / KeyTraits<RAW>::VEC <= int64_t(SMALL_VECTORS) * SEL_THREADS) {
        trace_mark(stream);
        select_small_kernel<RAW><<<1, SEL_THREADS, 0, stream>>>(xr, numel, int(numel / KeyTraits<RAW>::VEC),
                                                                static_cast<uint32_t>(k), static_cast<RAW *>(vals), idx);
        trace_mark(stream);
        return launch_status();
    }
    // Preferred: one persistent kernel, one workgroup per compute unit.
    if (mode != 1) {
        constexpr int VEC = KeyTraits<RAW>::VEC;
        constexpr int TILE_WORDS = SEL_THREADS * VEC + SEL_THREADS * VEC * int(sizeof(RAW)) / 4;
        constexpr int HIST_WORDS = (sizeof(RAW) == 4 ? (1 << 13) : (1 << 11)) + 2 * WAVE;
        constexpr size_t parked_bytes = size_t(FUSED_RES) * SEL_THREADS * 16 +
                                        4 * size_t(TILE_WORDS > HIST_WORDS ? TILE_WORDS : HIST_WORDS);
        static_assert(parked_bytes <= FUSED_SMEM_BYTES, "both LDS layouts fit");
        // 16-bit types: everything the compute unit has, the staged form's segments take what the layouts leave
        constexpr size_t smem_bytes = sizeof(RAW) == 2 ? FUSED_SMEM_BYTES : parked_bytes;
        static_assert(size_t(FUSED_RES) * SEL_THREADS * 16 >= 4 * ((size_t(1) << 13) + 2 * WAVE),
                      "the serial fallback keeps its histogram where the chunk head was parked");
        // how many workgroups of this kernel each device holds at once (asked once per element type and device)
        static std::atomic<uint64_t> asked{0};
        static int capacity_of[64] = {};
        int dev = 0;
        (void)hipGetDevice(&dev);
        int fresh = -1;
        const bool ok = once_per_device(asked, [&] {
            hipDeviceProp_t prop;
            int per_cu = 0;
            if (hipGetDeviceProperties(&prop, dev) == hipSuccess &&
                hipFuncSetAttribute(reinterpret_cast<const void *>(select_fused_kernel<RAW>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    static_cast<int>(smem_bytes)) == hipSuccess &&
                hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, select_fused_kernel<RAW>, SEL_THREADS,
                                                             smem_bytes) == hipSuccess &&
                per_cu > 0 && prop.multiProcessorCount > 0)
                fresh = std::min(per_cu * prop.multiProcessorCount, SEL_MAX_CHUNKS);
            (void)hipGetLastError();
            if (dev >= 0 && dev < 64) capacity_of[dev] = fresh;
            return true;                       // a device that cannot hold the kernel is an answer too (-1)
        });
        const int capacity = !ok ? -1 : (dev >= 0 && dev < 64) ? capacity_of[dev] : fresh;
        if (capacity > 0) {
            // chunk geometry: at most one workgroup per resident slot, chunks start on 128-byte lines
            int64_t nvf = numel / VEC;
            int64_t chunks = std::min<int64_t>(std::max<int64_t>((nvf + SEL_THREADS - 1) / SEL_THREADS, 1), capacity);
            int64_t vpc = std::max<int64_t>(((nvf + chunks - 1) / chunks + 7) / 8 * 8, 8);
            chunks = std::max<int64_t>((nvf + vpc - 1) / vpc, 1);
            uint32_t k32 = static_cast<uint32_t>(k);
            uint32_t spin_limit = mode == 3 ? 0u : SPIN_LIMIT;
            RAW *vals_t = static_cast<RAW *>(vals);
            unsigned long long gen = next_generation();
            trace_mark(stream);
            if (mode == 2) {               // the runtime guarantees co-residency, at the price of slow queue switches
                void *args[] = {(void *)&xr, (void *)&numel, (void *)&nvf, (void *)&vpc, (void *)&k32, (void *)&st,
                                (void *)&hist0, (void *)&hist1, (void *)&table, (void *)&vals_t, (void *)&idx,
                                (void *)&spin_limit, (void *)&gen};
                if (hipLaunchCooperativeKernel(reinterpret_cast<const void *>(select_fused_kernel<RAW>),
                                               dim3(static_cast<unsigned>(chunks)), dim3(SEL_THREADS), args,
                                               smem_bytes, stream) == hipSuccess) {
                    trace_mark(stream);
                    return launch_status();
                }
                (void)hipGetLastError();   // cooperative launch unavailable (e.g. stream capture): ordinary launch
            }
            select_fused_kernel<RAW><<<dim3(static_cast<unsigned>(chunks)), dim3(SEL_THREADS), smem_bytes, stream>>>(
                xr, numel, nvf, vpc, k32, st, hist0, hist1, table, vals_t, idx, spin_limit, gen);
            trace_mark(stream);
            return launch_status();
        }
    }
    clear_state();
    const dim3 grid(g.chunks), block(SEL_THREADS);
    trace_mark(stream);
    if constexpr (sizeof(RAW) == 2) {
        hist_kernel<RAW, 4, 11, true><<<grid, block, 0, stream>>>(xr, numel, g.nvf, g.vpc, st, hist0, 0);
        trace_mark(stream);
        count_kernel<RAW, 4><<<grid, block, 0, stream>>>(xr, numel, g.nvf, g.vpc, st, table, off_gt, off_eq, 1);
    } else {
        hist_kernel<RAW, 18, 13, true><<<grid, block, 0, stream>>>(xr, numel, g.nvf, g.vpc, st, hist0, 0);
        trace_mark(stream);
        hist_kernel<RAW, 5, 13, false><<<grid, block, 0, stream>>>(xr, numel, g.nvf, g.vpc, st, hist1, 1);
        trace_mark(stream);
        count_kernel<RAW, 5><<<grid, block, 0, stream>>>(xr, numel, g.nvf, g.vpc, st, table, off_gt, off_eq, 2);
    }
    trace_mark(stream);
    compact_kernel<RAW><<<grid, block, 0, stream>>>(xr, numel, g.nvf, g.vpc, st, off_gt, off_eq,
                                                    static_cast<RAW *>(vals), idx);
    trace_mark(stream);
    return launch_status();
}

}  // namespace
}  // namespace dropit

dropit::TraceState &dropit::trace_state()
{
    static thread_local TraceState t = {nullptr, 0, 0};
    return t;
}

int &dropit::select_mode()
{
    static thread_local int mode = 0;
    return mode;
}

using namespace dropit;

extern "C" dropit_status dropit_set_select_mode(int mode)
{
    if (mode < 0 || mode > 3) return DROPIT_EINVAL;
    select_mode() = mode;
    return DROPIT_OK;
}

extern "C" void dropit_trace_events(void **events, int count)
{
    TraceState &t = trace_state();
    t.events = reinterpret_cast<hipEvent_t *>(events);
    t.count = (events != nullptr && count > 0) ? count : 0;
    t.next = 0;
}

extern "C" const char *dropit_status_string(dropit_status s)
{
    switch (s) {
    case DROPIT_OK: return "DROPIT_OK";
    case DROPIT_EINVAL: return "DROPIT_EINVAL: invalid argument";
    case DROPIT_EWORKSPACE: return "DROPIT_EWORKSPACE: workspace too small";
    case DROPIT_EUNSUPPORTED: return "DROPIT_EUNSUPPORTED: geometry not implemented";
    case DROPIT_EHIP: return "DROPIT_EHIP: HIP launch failed";
    }
    return "DROPIT: unknown status";
}

extern "C" int64_t dropit_keep_count(int64_t numel, double gamma)
{
    if (numel < 0 || numel > INT32_MAX) return -1;
    if (!(gamma >= 0.0 && gamma <= 1.0)) return -1;   // also rejects NaN
    // floor((1-gamma)*numel) == numel - ceil(gamma*numel); gamma*numel < 2^31 is exact enough in double
    const double dropped = __builtin_ceil(gamma * static_cast<double>(numel));
    int64_t k = numel - static_cast<int64_t>(dropped);
    if (k < 0) k = 0;
    return k;
}

extern "C" size_t dropit_compress_workspace_bytes(int64_t numel, dropit_dtype dt)
{
    if (numel < 1 || numel > INT32_MAX) return 0;
    if (dt != DROPIT_F32 && dt != DROPIT_BF16) return 0;
    return SelWorkspace::bytes;
}

extern "C" dropit_status dropit_compress(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                                         double gamma, void *vals, int32_t *idx, void *workspace,
                                         size_t workspace_bytes, void *hip_stream)
{
    if (dt != DROPIT_F32 && dt != DROPIT_BF16) return DROPIT_EINVAL;
    const int64_t numel = checked_numel(shape, ndim);
    if (numel < 1) return DROPIT_EINVAL;
    const int64_t k = dropit_keep_count(numel, gamma);
    if (k < 0) return DROPIT_EINVAL;
    if (x == nullptr || !aligned(x, 16)) return DROPIT_EINVAL;
    if (k == 0) return DROPIT_OK;
    if (vals == nullptr || idx == nullptr) return DROPIT_EINVAL;
    if (!aligned(vals, dt == DROPIT_F32 ? 4 : 2) || !aligned(idx, 4)) return DROPIT_EINVAL;
    if (workspace == nullptr || !aligned(workspace, 256)) return DROPIT_EINVAL;
    if (workspace_bytes < SelWorkspace::bytes) return DROPIT_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    if (dt == DROPIT_BF16) return run_compress<uint16_t>(x, numel, k, vals, idx, ws, stream);
    return run_compress<uint32_t>(x, numel, k, vals, idx, ws, stream);
}

// ---- dropit_compress for callers that cannot allocate ----------------------------------------------
// The select's exchange area (state, histograms, per-chunk table: SelWorkspace::bytes, about 170 KB, the
// same for every tensor size) as a device array of this library instead of a caller's workspace.  In
// host code `scratch` is only a handle for the runtime: the array's device address is asked for once
// per device (each device holds its own copy) and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[SelWorkspace::bytes];

namespace {
// Device address of `scratch` on the current device, nullptr if the runtime will not tell.
char *static_scratch()
{
    static std::atomic<uint64_t> known{0};
    static void *address_on[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    void *fresh = nullptr;
    const bool ok = once_per_device(known, [&] {
        if (hipGetSymbolAddress(&fresh, HIP_SYMBOL(scratch)) != hipSuccess || fresh == nullptr) {
            (void)hipGetLastError();
            return false;
        }
        if (dev >= 0 && dev < 64) address_on[dev] = fresh;
        return true;
    });
    if (!ok) return nullptr;
    return static_cast<char *>((dev >= 0 && dev < 64) ? address_on[dev] : fresh);
}
}  // namespace

extern "C" dropit_status dropit_compress_static(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                                                double gamma, void *vals, int32_t *idx, void *hip_stream)
{
    if (dt != DROPIT_F32 && dt != DROPIT_BF16) return DROPIT_EINVAL;
    const int64_t numel = checked_numel(shape, ndim);       // -1 beyond DROPIT_STATIC_MAX_NUMEL
    if (numel < 1) return DROPIT_EINVAL;
    const int64_t k = dropit_keep_count(numel, gamma);
    if (k < 0) return DROPIT_EINVAL;
    if (x == nullptr || !aligned(x, 16)) return DROPIT_EINVAL;
    if (k == 0) return DROPIT_OK;
    if (vals == nullptr || idx == nullptr) return DROPIT_EINVAL;
    if (!aligned(vals, dt == DROPIT_F32 ? 4 : 2) || !aligned(idx, 4)) return DROPIT_EINVAL;
    char *ws = static_scratch();
    if (ws == nullptr) return DROPIT_EHIP;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (dt == DROPIT_BF16) return run_compress<uint16_t>(x, numel, k, vals, idx, ws, stream);
    return run_compress<uint32_t>(x, numel, k, vals, idx, ws, stream);
}

extern "C" size_t dropit_compress_random_workspace_bytes(int64_t numel, dropit_dtype dt)
{
    if (numel < 1 || numel > INT32_MAX) return 0;
    if (dt != DROPIT_F32 && dt != DROPIT_BF16) return 0;
    return RandomWorkspace(numel).bytes;
}

extern "C" dropit_status dropit_compress_random(const void *x, const int64_t *shape, int ndim, dropit_dtype dt,
                                                double gamma, uint64_t seed, void *vals, int32_t *idx,
                                                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (dt != DROPIT_F32 && dt != DROPIT_BF16) return DROPIT_EINVAL;
    const int64_t numel = checked_numel(shape, ndim);
    if (numel < 1) return DROPIT_EINVAL;
    const int64_t k = dropit_keep_count(numel, gamma);
    if (k < 0) return DROPIT_EINVAL;
    if (x == nullptr || !aligned(x, 16)) return DROPIT_EINVAL;
    if (k == 0) return DROPIT_OK;
    if (vals == nullptr || idx == nullptr) return DROPIT_EINVAL;
    if (!aligned(vals, dt == DROPIT_F32 ? 4 : 2) || !aligned(idx, 4)) return DROPIT_EINVAL;
    if (workspace == nullptr || !aligned(workspace, 256)) return DROPIT_EINVAL;
    const RandomWorkspace rw(numel);
    if (workspace_bytes < rw.bytes) return DROPIT_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    uint4 *keys = reinterpret_cast<uint4 *>(ws + rw.keys_off);
    const int64_t blocks = (numel + 3) / 4;
    const unsigned grid = static_cast<unsigned>(std::min<int64_t>((blocks + 255) / 256, 256 * 16));
    trace_mark(stream);
    random_keys_kernel<<<grid, 256, 0, stream>>>(keys, blocks, static_cast<uint32_t>(seed & 0xFFFFFFFFu),
                                                 static_cast<uint32_t>(seed >> 32));
    // the drawn keys are 31-bit patterns: the fp32 select ranks them as integers
    dropit_status st = run_compress<uint32_t>(keys, numel, k, ws + rw.keyvals_off, idx, ws, stream);
    if (st != DROPIT_OK) return st;
    const unsigned ggrid = static_cast<unsigned>(std::min<int64_t>((k + 255) / 256, 256 * 16));
    if (dt == DROPIT_BF16)
        gather_kernel<uint16_t><<<ggrid, 256, 0, stream>>>(static_cast<const uint16_t *>(x), idx, k,
                                                           static_cast<uint16_t *>(vals));
    else
        gather_kernel<uint32_t><<<ggrid, 256, 0, stream>>>(static_cast<const uint32_t *>(x), idx, k,
                                                           static_cast<uint32_t *>(vals));
    trace_mark(stream);
    return launch_status();
}
