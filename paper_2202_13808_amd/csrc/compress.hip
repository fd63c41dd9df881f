// Min-k dropping D(a) = {a_Xr, Xr} (Sec. 3.2, Sec. 3.3 "Min-K Elements", Sec. 4.1)
// as a bandwidth-bound radix select + ordered stream compaction for gfx950.
//
// The magnitude key of an element is its bit pattern with the sign cleared
// (15 bits for bf16, 31 for fp32); unsigned key order == |x| order.
//
//   init      : clear histograms / tickets, seed the select state with k
//   hist pass : MSB-first digit histogram of the keys that match the digits
//               resolved so far (LDS histogram per workgroup, merged with
//               global atomics; the last workgroup to arrive resolves the digit)
//   count pass: resolves the last (4/5-bit) digit; every workgroup owns one
//               contiguous chunk of x and records, per chunk, how many keys
//               are above the resolved prefix and a small histogram of the
//               matching ones.  The last workgroup derives the threshold key
//               t, the tie budget m = k - #{key > t}, and the exclusive
//               per-chunk offsets of {key > t} and {key == t}.
//   compact   : each workgroup re-reads its chunk and writes (value, index)
//               pairs in ascending index order; of the keys equal to t only
//               the first m by flat index are kept.
//
// bf16: 11 + 4 bits (one hist pass); fp32: 13 + 13 + 5 bits (two hist passes).
// Nothing here synchronises with the host; counts are integer, so the result
// does not depend on the order in which workgroups run.
#include "common.hpp"

namespace dropit {
namespace {

constexpr int SEL_THREADS = 512;
constexpr int SEL_MAX_CHUNKS = 1024;
constexpr int SEL_UNROLL = 4;
constexpr int MAX_HIST_BITS = 13;
constexpr int MAX_LAST_BINS = 32;

struct SelState {
    uint32_t prefix;     // key digits resolved so far (key >> remaining bits)
    uint32_t k_rem;      // elements still to take among the keys matching prefix
    uint32_t t;          // threshold key (valid after the count pass)
    uint32_t m;          // how many keys equal to t are kept (lowest flat index first)
    uint32_t ticket[4];  // arrival counters, one per pass
    uint32_t pad[56];
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
    static constexpr size_t bytes = offeq_off + sizeof(uint32_t) * SEL_MAX_CHUNKS;
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

__device__ inline void unpack(const uint4 &q, uint16_t (&r)[8])
{
    r[0] = q.x & 0xFFFF; r[1] = q.x >> 16; r[2] = q.y & 0xFFFF; r[3] = q.y >> 16;
    r[4] = q.z & 0xFFFF; r[5] = q.z >> 16; r[6] = q.w & 0xFFFF; r[7] = q.w >> 16;
}
__device__ inline void unpack(const uint4 &q, uint32_t (&r)[4])
{
    r[0] = q.x; r[1] = q.y; r[2] = q.z; r[3] = q.w;
}

// Loads vector v (VEC consecutive elements, 16 bytes) of x; returns the number
// of valid elements (VEC except in the ragged last vector, 0 if v >= nvec).
template <typename RAW>
__device__ inline int load_vec(const RAW *__restrict__ x, int64_t v, int64_t nvec, int64_t numel,
                               RAW (&r)[KeyTraits<RAW>::VEC])
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    if (v >= nvec) return 0;
    const int64_t base = v * VEC;
    if (base + VEC <= numel) {
        const uint4 q = reinterpret_cast<const uint4 *>(x)[v];
        unpack(q, r);
        return VEC;
    }
    const int nv = static_cast<int>(numel - base);
#pragma unroll
    for (int e = 0; e < VEC; ++e) r[e] = (e < nv) ? x[base + e] : RAW(0);
    return nv;
}

__global__ void __launch_bounds__(256) init_kernel(uint32_t *ws, uint32_t nwords, uint32_t k)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < nwords; i += gridDim.x * blockDim.x)
        ws[i] = (i == offsetof(SelState, k_rem) / 4) ? k : 0u;
}

// Ticket: true in every thread of exactly one workgroup, the last to arrive.
__device__ inline bool last_block_to_arrive(uint32_t *ticket)
{
    __shared__ uint32_t s_last;
    __threadfence();                       // publish this workgroup's global writes
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t t = atomicAdd(ticket, 1u);
        s_last = (t == gridDim.x - 1) ? 1u : 0u;
    }
    __syncthreads();
    const bool last = s_last != 0;
    if (last) __threadfence();             // see every other workgroup's writes
    return last;
}

__device__ inline uint32_t coherent_load(const uint32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
        c[i] = (lo + i < NB) ? coherent_load(hist + lo + i) : 0u;
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

template <typename RAW, int BITS>
__global__ void __launch_bounds__(SEL_THREADS)
hist_kernel(const RAW *__restrict__ x, int64_t numel, int64_t nvec, int64_t vpc, SelState *st,
            uint32_t *ghist, int shift, int pass)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    constexpr int NB = 1 << BITS;
    __shared__ uint32_t lh[NB];
    __shared__ uint32_t scan[SEL_THREADS];
    const int tid = threadIdx.x;
    for (int i = tid; i < NB; i += SEL_THREADS) lh[i] = 0;
    const uint32_t prefix = st->prefix;
    __syncthreads();

    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * vpc;
    const int64_t v1 = min(v0 + vpc, nvec);
    uint32_t zero_digit = 0;               // digit 0 is counted in registers (exact zeros are common)
    for (int64_t vb = v0; vb < v1; vb += SEL_THREADS * SEL_UNROLL) {
        RAW r[SEL_UNROLL][VEC];
        int nv[SEL_UNROLL];
#pragma unroll
        for (int u = 0; u < SEL_UNROLL; ++u) {
            const int64_t v = vb + u * SEL_THREADS + tid;
            nv[u] = load_vec<RAW>(x, v < v1 ? v : nvec, nvec, numel, r[u]);
        }
#pragma unroll
        for (int u = 0; u < SEL_UNROLL; ++u) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const uint32_t key = r[u][e] & KeyTraits<RAW>::MASK;
                if (e < nv[u] && (key >> (shift + BITS)) == prefix) {
                    const uint32_t d = (key >> shift) & (NB - 1);
                    if (d == 0) ++zero_digit;
                    else atomicAdd(&lh[d], 1u);
                }
            }
        }
    }
    zero_digit = wave_sum(zero_digit);
    if ((tid & (WAVE - 1)) == 0 && zero_digit) atomicAdd(&lh[0], zero_digit);
    __syncthreads();
    for (int i = tid; i < NB; i += SEL_THREADS) {
        const uint32_t c = lh[i];
        if (c) atomicAdd(&ghist[i], c);
    }
    if (!last_block_to_arrive(&st->ticket[pass])) return;
    resolve_digit<NB, BITS>(ghist, st, scan);
}

template <typename RAW, int LAST_BITS>
__global__ void __launch_bounds__(SEL_THREADS)
count_kernel(const RAW *__restrict__ x, int64_t numel, int64_t nvec, int64_t vpc, SelState *st,
             uint32_t *table /*[LB+1][G]*/, uint32_t *off_gt, uint32_t *off_eq, int pass)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    constexpr int LB = 1 << LAST_BITS;
    __shared__ uint32_t lh[LB + 1];
    __shared__ uint32_t s_digit;
    __shared__ unsigned long long wave_tot[SEL_THREADS / WAVE];
    const int tid = threadIdx.x;
    const int G = gridDim.x;
    if (tid <= LB) lh[tid] = 0;
    const uint32_t prefix = st->prefix;    // == key >> LAST_BITS of the threshold
    __syncthreads();

    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * vpc;
    const int64_t v1 = min(v0 + vpc, nvec);
    uint32_t above = 0;
    for (int64_t vb = v0; vb < v1; vb += SEL_THREADS * SEL_UNROLL) {
        RAW r[SEL_UNROLL][VEC];
        int nv[SEL_UNROLL];
#pragma unroll
        for (int u = 0; u < SEL_UNROLL; ++u) {
            const int64_t v = vb + u * SEL_THREADS + tid;
            nv[u] = load_vec<RAW>(x, v < v1 ? v : nvec, nvec, numel, r[u]);
        }
#pragma unroll
        for (int u = 0; u < SEL_UNROLL; ++u) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const uint32_t key = r[u][e] & KeyTraits<RAW>::MASK;
                const uint32_t hi = key >> LAST_BITS;
                if (e < nv[u]) {
                    if (hi > prefix) ++above;
                    else if (hi == prefix) atomicAdd(&lh[key & (LB - 1)], 1u);
                }
            }
        }
    }
    above = wave_sum(above);
    if ((tid & (WAVE - 1)) == 0 && above) atomicAdd(&lh[LB], above);
    __syncthreads();
    if (tid <= LB) table[tid * G + blockIdx.x] = lh[tid];
    if (!last_block_to_arrive(&st->ticket[pass])) return;

    // ---- last workgroup: resolve the final digit, then per-chunk offsets ----
    if (tid <= LB) lh[tid] = 0;
    __syncthreads();
    for (int c = tid; c < G; c += SEL_THREADS) {
#pragma unroll
        for (int b = 0; b < LB; ++b) {
            const uint32_t n = coherent_load(table + b * G + c);
            if (n) atomicAdd(&lh[b], n);
        }
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
    // exclusive scan over chunks of (#{key > t}, #{key == t}); two chunks per thread
    constexpr int CPT = SEL_MAX_CHUNKS / SEL_THREADS;
    uint32_t gt[CPT], eq[CPT];
    unsigned long long mine = 0;
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = tid * CPT + i;
        gt[i] = eq[i] = 0;
        if (c < G) {
            uint32_t g = coherent_load(table + LB * G + c);
            for (int b = d + 1; b < LB; ++b) g += coherent_load(table + b * G + c);
            gt[i] = g;
            eq[i] = coherent_load(table + d * G + c);
        }
        mine += (static_cast<unsigned long long>(eq[i]) << 32) | gt[i];
    }
    unsigned long long total;
    unsigned long long run = block_exclusive_scan<SEL_THREADS>(mine, wave_tot, total);
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int c = tid * CPT + i;
        if (c < G) {
            off_gt[c] = static_cast<uint32_t>(run & 0xFFFFFFFFull);
            off_eq[c] = static_cast<uint32_t>(run >> 32);
        }
        run += (static_cast<unsigned long long>(eq[i]) << 32) | gt[i];
    }
}

template <typename RAW>
__global__ void __launch_bounds__(SEL_THREADS)
compact_kernel(const RAW *__restrict__ x, int64_t numel, int64_t nvec, int64_t vpc,
               const SelState *__restrict__ st, const uint32_t *__restrict__ off_gt,
               const uint32_t *__restrict__ off_eq, RAW *__restrict__ vals, int32_t *__restrict__ idx)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    __shared__ uint32_t wave_tot[SEL_THREADS / WAVE];
    const int tid = threadIdx.x;
    const uint32_t t = st->t;
    const uint32_t m = st->m;
    uint32_t run_gt = off_gt[blockIdx.x];  // #{key > t} before this tile
    uint32_t run_eq = off_eq[blockIdx.x];  // #{key == t} before this tile
    const int64_t v0 = static_cast<int64_t>(blockIdx.x) * vpc;
    const int64_t v1 = min(v0 + vpc, nvec);
    for (int64_t vb = v0; vb < v1; vb += SEL_THREADS) {
        const int64_t v = vb + tid;
        RAW r[VEC];
        const int nv = load_vec<RAW>(x, v < v1 ? v : nvec, nvec, numel, r);
        uint32_t cnt = 0;                  // low 16 bits: #gt, high 16 bits: #eq (tile <= 4096 elements)
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const uint32_t key = r[e] & KeyTraits<RAW>::MASK;
            if (e < nv) cnt += (key > t ? 1u : 0u) + (key == t ? 0x10000u : 0u);
        }
        uint32_t total;
        const uint32_t excl = block_exclusive_scan<SEL_THREADS>(cnt, wave_tot, total);
        uint32_t my_gt = run_gt + (excl & 0xFFFFu);
        uint32_t my_eq = run_eq + (excl >> 16);
        const int64_t base = v * VEC;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if (e < nv) {
                const uint32_t key = r[e] & KeyTraits<RAW>::MASK;
                if (key > t) {
                    const uint32_t pos = my_gt + min(my_eq, m);
                    vals[pos] = r[e];
                    idx[pos] = static_cast<int32_t>(base + e);
                    ++my_gt;
                } else if (key == t) {
                    if (my_eq < m) {
                        const uint32_t pos = my_gt + my_eq;
                        vals[pos] = r[e];
                        idx[pos] = static_cast<int32_t>(base + e);
                    }
                    ++my_eq;
                }
            }
        }
        run_gt += total & 0xFFFFu;
        run_eq += total >> 16;
    }
}

struct Geometry {
    int64_t nvec, vpc;
    int chunks;
};

template <typename RAW>
Geometry geometry(int64_t numel)
{
    constexpr int VEC = KeyTraits<RAW>::VEC;
    Geometry g;
    g.nvec = (numel + VEC - 1) / VEC;
    int64_t chunks = (g.nvec + SEL_THREADS - 1) / SEL_THREADS;
    if (chunks > SEL_MAX_CHUNKS) chunks = SEL_MAX_CHUNKS;
    if (chunks < 1) chunks = 1;
    g.vpc = (g.nvec + chunks - 1) / chunks;
    g.vpc = (g.vpc + 7) / 8 * 8;           // chunk starts on 128-byte lines
    g.chunks = static_cast<int>((g.nvec + g.vpc - 1) / g.vpc);
    return g;
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

    trace_mark(stream);
    init_kernel<<<32, 256, 0, stream>>>(reinterpret_cast<uint32_t *>(ws),
                                        static_cast<uint32_t>(SelWorkspace::zero_bytes / 4),
                                        static_cast<uint32_t>(k));
    const dim3 grid(g.chunks), block(SEL_THREADS);
    trace_mark(stream);
    if constexpr (sizeof(RAW) == 2) {
        hist_kernel<RAW, 11><<<grid, block, 0, stream>>>(xr, numel, g.nvec, g.vpc, st, hist0, 4, 0);
        trace_mark(stream);
        count_kernel<RAW, 4><<<grid, block, 0, stream>>>(xr, numel, g.nvec, g.vpc, st, table, off_gt, off_eq, 1);
    } else {
        hist_kernel<RAW, 13><<<grid, block, 0, stream>>>(xr, numel, g.nvec, g.vpc, st, hist0, 18, 0);
        hist_kernel<RAW, 13><<<grid, block, 0, stream>>>(xr, numel, g.nvec, g.vpc, st, hist1, 5, 1);
        trace_mark(stream);
        count_kernel<RAW, 5><<<grid, block, 0, stream>>>(xr, numel, g.nvec, g.vpc, st, table, off_gt, off_eq, 2);
    }
    trace_mark(stream);
    compact_kernel<RAW><<<grid, block, 0, stream>>>(xr, numel, g.nvec, g.vpc, st, off_gt, off_eq,
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

using namespace dropit;

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
