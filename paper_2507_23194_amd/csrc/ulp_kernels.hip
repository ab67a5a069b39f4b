// HIP kernels of the ulp-distance histogram for gfx950 (wave64): per (segment, candidate), how many
// elements lie how many steps of the tensor's own storage format away from the reference (the
// second half of the numeric error trace that the evaluator hands to the Reflector, GEAK sections
// 4.1 / 4.2; the paper does not define it).
//
//   distance  floating dtypes: steps on the ladder of the format's values ordered by value, -0 and
//             +0 one rung, +-Inf the rung after the largest finite value; with ord(x) = the
//             magnitude's bit pattern, negated for negative x, it is |ord(a) - ord(b)|.
//             integer dtypes: |a - b|.  Both exact in the unsigned type of the element's width.
//   bins      0: distance 0; j = 1..64: 2^(j-1) <= distance < 2^j; 65: a or b is NaN.
//
// histogram kernel -- the plan's work items and per-wave item lists are reused.  A wave keeps the
// ord values of its reference slice in registers and streams the candidates of the pass past them,
// one candidate's loads ahead of the compute.  Per element four cumulative classes (distance < 1,
// < 2, < 4, < 8) are counted with lane masks in scalar registers; only lanes beyond them (or NaN)
// touch the wave's histogram in LDS, one atomic add per lane.  Per (wave, segment run, candidate)
// the LDS rows are written, without atomics, to a partial table; the reduce kernel sums the
// partial rows of a segment.  A pass covers as many candidates as fit the wave's LDS rows.
#include <hip/hip_runtime.h>
#include "geak_internal.hpp"
#include "device_common.hpp"

namespace geak {
namespace {

// ---- per-dtype ord value of element e of a 16-byte vector -------------------------------------------
template <int DT> struct UlpTraits {
    typedef int Ord;                        // signed, as wide as the element (32 bits for the narrower ones)
    typedef uint32_t Dist;
};
template <> struct UlpTraits<GEAK_F64> { typedef long long Ord; typedef u64 Dist; };
template <> struct UlpTraits<GEAK_I64> { typedef long long Ord; typedef u64 Dist; };

template <int DT> constexpr bool kUlpFloating = (DT == GEAK_F32 || DT == GEAK_F16 || DT == GEAK_BF16 || DT == GEAK_F64);

// the magnitude pattern of +Inf, in the ord type
template <int DT> __device__ __forceinline__ typename UlpTraits<DT>::Ord ulp_inf()
{
    if constexpr (DT == GEAK_F32) return 0x7F800000;
    else if constexpr (DT == GEAK_F16) return 0x7C00;
    else if constexpr (DT == GEAK_BF16) return 0x7F80;
    else return 0x7FF0000000000000ll;
}

template <int DT>
__device__ __forceinline__ typename UlpTraits<DT>::Ord ulp_ord(const u32x4 &q, int e)
{
    if constexpr (DT == GEAK_F32) {
        const uint32_t bits = q[e];
        const int mag = (int)(bits & 0x7FFFFFFFu);
        return ((int)bits < 0) ? -mag : mag;
    } else if constexpr (DT == GEAK_F16 || DT == GEAK_BF16) {
        const uint32_t word = q[e >> 1];
        const uint32_t h = (e & 1) ? (word >> 16) : (word & 0xFFFFu);
        const int mag = (int)(h & 0x7FFFu);
        return (h & 0x8000u) ? -mag : mag;
    } else if constexpr (DT == GEAK_F64) {
        const u64 bits = (u64)q[2 * e] | ((u64)q[2 * e + 1] << 32);
        const long long mag = (long long)(bits & 0x7FFFFFFFFFFFFFFFull);
        return ((long long)bits < 0) ? -mag : mag;
    } else if constexpr (DT == GEAK_I32) {
        return (int)q[e];
    } else if constexpr (DT == GEAK_I64) {
        return (long long)((u64)q[2 * e] | ((u64)q[2 * e + 1] << 32));
    } else {
        const uint32_t v = (q[e >> 2] >> (8 * (e & 3))) & 0xFFu;
        return (DT == GEAK_I8) ? (int)(signed char)v : (int)v;
    }
}

template <int DT>
__device__ __forceinline__ bool ulp_is_nan(typename UlpTraits<DT>::Ord o)
{
    if constexpr (kUlpFloating<DT>) return (o < 0 ? -o : o) > ulp_inf<DT>();
    else return false;
}

template <int DT>
__device__ __forceinline__ typename UlpTraits<DT>::Dist ulp_dist(typename UlpTraits<DT>::Ord a, typename UlpTraits<DT>::Ord b)
{
    typedef typename UlpTraits<DT>::Dist D;
    return (a > b) ? (D)a - (D)b : (D)b - (D)a;          // exact: the true difference is below 2^width
}

__device__ __forceinline__ uint32_t bit_length(uint32_t d) { return 32u - (uint32_t)__builtin_clz(d | 1u) - (d == 0u); }
__device__ __forceinline__ uint32_t bit_length(u64 d) { return 64u - (uint32_t)__builtin_clzll(d | 1ull) - (d == 0ull); }

// ---- the wave's histogram rows in LDS: [candidate of the pass][slot], 32-bit counts ------------------
// slot j < nslots - 1 is bin j; the last slot is the NaN bin.
struct UlpState {
    uint32_t rows_off;       // LDS byte offset of the wave's rows
    uint32_t nslots;
};
__device__ __forceinline__ GEAK_AS_LDS uint32_t *ulp_row(const UlpState &st, uint32_t kk)
{
    return (GEAK_AS_LDS uint32_t *)(st.rows_off + kk * st.nslots * 4u);
}

// Counters of one (item, candidate): cumulative classes in scalar registers.
struct UlpCounts {
    uint32_t lt1, lt2, lt4, lt8, nan;
};

// One element position of all 64 lanes.
template <int DT>
__device__ __forceinline__ void ulp_element(typename UlpTraits<DT>::Ord oa, typename UlpTraits<DT>::Ord ob, bool ref_may_be_nan,
                                            UlpCounts &c, GEAK_AS_LDS uint32_t *row, int lane)
{
    typedef typename UlpTraits<DT>::Dist D;
    const D d = ulp_dist<DT>(oa, ob);
    u64 m1 = __builtin_amdgcn_ballot_w64(d < (D)1), m2 = __builtin_amdgcn_ballot_w64(d < (D)2);
    u64 m4 = __builtin_amdgcn_ballot_w64(d < (D)4), m8 = __builtin_amdgcn_ballot_w64(d < (D)8);
    u64 mn = 0;
    if constexpr (kUlpFloating<DT>) {
        mn = __builtin_amdgcn_ballot_w64(ulp_is_nan<DT>(oa));
        if (ref_may_be_nan) mn |= __builtin_amdgcn_ballot_w64(ulp_is_nan<DT>(ob));
        if (mn) {
            m1 &= ~mn; m2 &= ~mn; m4 &= ~mn; m8 &= ~mn;
            c.nan += (uint32_t)__builtin_popcountll(mn);
        }
    }
    c.lt1 += (uint32_t)__builtin_popcountll(m1);
    c.lt2 += (uint32_t)__builtin_popcountll(m2);
    c.lt4 += (uint32_t)__builtin_popcountll(m4);
    c.lt8 += (uint32_t)__builtin_popcountll(m8);
    const u64 rest = ~(m8 | mn);
    if (rest) {                                             // distance >= 8: straight into the LDS row
        if ((rest >> lane) & 1ull)
            (void)__hip_atomic_fetch_add(row + bit_length(d), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

// the scalar counters of one (item, candidate) go into the row; `pad` absent elements of a tail
// were read as 0 on both sides and counted as distance 0
__device__ __forceinline__ void ulp_commit(const UlpCounts &c, uint32_t pad, GEAK_AS_LDS uint32_t *row, uint32_t nslots, int lane)
{
    if (lane == 0) {
        const uint32_t b0 = c.lt1 - pad, b1 = c.lt2 - c.lt1, b2 = c.lt4 - c.lt2, b3 = c.lt8 - c.lt4;
        if (b0) (void)__hip_atomic_fetch_add(row + 0, b0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (b1) (void)__hip_atomic_fetch_add(row + 1, b1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (b2) (void)__hip_atomic_fetch_add(row + 2, b2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (b3) (void)__hip_atomic_fetch_add(row + 3, b3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (c.nan) (void)__hip_atomic_fetch_add(row + (nslots - 1), c.nan, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

// A (wave, segment) run ends: its rows go to the run's slot of the partial table and are cleared.
__device__ __forceinline__ void ulp_end_run(const UlpState &st, uint32_t *partials, uint32_t slot, uint32_t K, uint32_t k_begin,
                                            uint32_t k_count, int lane)
{
    GEAK_AS_LDS uint32_t *rows = (GEAK_AS_LDS uint32_t *)st.rows_off;
    GEAK_AS_GLOBAL uint32_t *out = (GEAK_AS_GLOBAL uint32_t *)partials + ((u64)slot * K + k_begin) * st.nslots;
    const uint32_t n = k_count * st.nslots;                 // rows of consecutive candidates are contiguous on both sides
    for (uint32_t i = lane; i < n; i += kWaveSize) {
        out[i] = rows[i];
        rows[i] = 0;
    }
}

struct UlpRunArgs {
    const geak_item *items;
    const unsigned char *ref;
    const unsigned char *const *cand;
    uint32_t *partials;
    uint32_t first_item;
    uint32_t num_items;
    uint32_t K, k_begin, k_count;
};

__device__ __forceinline__ uint32_t uniform32(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
template <typename T>
__device__ __forceinline__ T *uniform_ptr(T *p)
{
    const u64 v = reinterpret_cast<u64>(p);
    const u64 lo = uniform32((uint32_t)v), hi = uniform32((uint32_t)(v >> 32));
    return reinterpret_cast<T *>(lo | (hi << 32));
}

// A run of consecutive vector-loadable items of one dtype in the wave's list (FULL items: the whole
// run; a tail: that one item).  Returns the index of the wave's first item it did not process.
template <int DT>
__device__ __noinline__ uint32_t ulp_run(const UlpRunArgs in, const UlpState st_in)
{
    typedef typename UlpTraits<DT>::Ord Ord;
    constexpr int E = Traits<DT>::E;
    constexpr int N = kVecPerLane * E;
    constexpr bool kStageOrd = (N <= 32);                    // byte dtypes decode the reference again per candidate
    UlpState st;
    st.rows_off = uniform32(st_in.rows_off);
    st.nslots = uniform32(st_in.nslots);
    const geak_item *items = uniform_ptr(in.items);
    const unsigned char *ref_base = uniform_ptr(in.ref);
    const unsigned char *const *cand = uniform_ptr(in.cand);
    uint32_t *partials = uniform_ptr(in.partials);
    const uint32_t num_items = uniform32(in.num_items), K = uniform32(in.K);
    const uint32_t k_begin = uniform32(in.k_begin), k_count = uniform32(in.k_count);
    const int lane = threadIdx.x & (kWaveSize - 1);

    uint32_t j = uniform32(in.first_item);
    geak_item it = load_work_item(items, j);
    u32x4 cur[kVecPerLane];
    {
        const bool full = (it.flags & GEAK_ITEM_FULL) != 0;
#pragma unroll
        for (int v = 0; v < kVecPerLane; ++v) cur[v] = load_vec<DT>(ref_base + it.byte_offset, lane, v, it.numel, full);
    }
    for (;;) {
        const bool full = (it.flags & GEAK_ITEM_FULL) != 0;
        const uint32_t pad = (uint32_t)(kWaveSize * N) - it.numel;
        // does the wave's next item continue the run?  (only FULL items do: a tail ends it)
        const uint32_t jn = it.next;
        bool more = full && jn < num_items;
        geak_item nx = it;
        if (more) {
            nx = load_work_item(items, jn);
            more = nx.dtype == DT && (nx.flags & GEAK_ITEM_ALIGNED);
        }
        // stage the reference slice; its registers are refilled with the pass's first candidate
        Ord ob[kStageOrd ? N : 1];
        u32x4 raw[kStageOrd ? 1 : kVecPerLane];
        u64 ref_nan = 0;                                     // bit i: some lane's reference element i is NaN
        {
            const unsigned char *first = table_entry(cand, k_begin) + it.byte_offset;
#pragma unroll
            for (int v = 0; v < kVecPerLane; ++v) {
                if constexpr (kStageOrd) {
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        const Ord o = ulp_ord<DT>(cur[v], e);
                        ob[v * E + e] = o;
                        if constexpr (kUlpFloating<DT>)
                            if (__builtin_amdgcn_ballot_w64(ulp_is_nan<DT>(o))) ref_nan |= 1ull << (v * E + e);
                    }
                } else {
                    raw[v] = cur[v];
                }
                cur[v] = load_vec<DT>(first, lane, v, it.numel, full);
            }
        }
        for (uint32_t kk = 0; kk < k_count; ++kk) {
            const bool last = kk + 1 == k_count;
            const bool has_next = !last || more;
            const unsigned char *next = last ? ref_base + nx.byte_offset : table_entry(cand, k_begin + kk + 1) + it.byte_offset;
            const uint32_t next_n = last ? nx.numel : it.numel;
            const bool next_full = last ? (nx.flags & GEAK_ITEM_FULL) != 0 : full;
            GEAK_AS_LDS uint32_t *row = ulp_row(st, kk);
            UlpCounts c = {0u, 0u, 0u, 0u, 0u};
#pragma unroll
            for (int v = 0; v < kVecPerLane; ++v) {
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const Ord oa = ulp_ord<DT>(cur[v], e);
                    if constexpr (kStageOrd) ulp_element<DT>(oa, ob[v * E + e], (ref_nan >> (v * E + e)) & 1ull, c, row, lane);
                    else ulp_element<DT>(oa, ulp_ord<DT>(raw[v], e), false, c, row, lane);
                }
                if (has_next) cur[v] = load_vec<DT>(next, lane, v, next_n, next_full);
            }
            ulp_commit(c, pad, row, st.nslots, lane);
        }
        if (it.flags & GEAK_ITEM_LAST) ulp_end_run(st, partials, it.slot, K, k_begin, k_count, lane);
        if (!more) break;
        it = nx;
        j = jn;
    }
    return it.next;
}

// the few elements before a segment's first 16-byte boundary: element by element, every lane adding
// into the row itself
__device__ __forceinline__ void ulp_head(const geak_item &it, const unsigned char *ref, const unsigned char *const *cand,
                                         const UlpState &st, uint32_t k_begin, uint32_t k_count, int lane)
{
    for (uint32_t kk = 0; kk < k_count; ++kk) {
        const unsigned char *rb = ref + it.byte_offset, *cb = table_entry(cand, k_begin + kk) + it.byte_offset;
        GEAK_AS_LDS uint32_t *row = ulp_row(st, kk);
        for (uint32_t i = lane; i < it.numel; i += kWaveSize) {
            uint32_t slot;
            switch (it.dtype) {
            case GEAK_F32: case GEAK_F16: case GEAK_BF16: {
                const uint32_t width = it.dtype == GEAK_F32 ? 4u : 2u;
                const uint32_t pa = width == 4 ? reinterpret_cast<const uint32_t *>(cb)[i] : reinterpret_cast<const uint16_t *>(cb)[i];
                const uint32_t pb = width == 4 ? reinterpret_cast<const uint32_t *>(rb)[i] : reinterpret_cast<const uint16_t *>(rb)[i];
                const uint32_t sign = width == 4 ? 0x80000000u : 0x8000u;
                const uint32_t inf = it.dtype == GEAK_F32 ? 0x7F800000u : (it.dtype == GEAK_F16 ? 0x7C00u : 0x7F80u);
                const int ma = (int)(pa & (sign - 1u)), mb = (int)(pb & (sign - 1u));
                const int oa = (pa & sign) ? -ma : ma, ob = (pb & sign) ? -mb : mb;
                const uint32_t d = (oa > ob) ? (uint32_t)oa - (uint32_t)ob : (uint32_t)ob - (uint32_t)oa;
                slot = ((uint32_t)ma > inf || (uint32_t)mb > inf) ? st.nslots - 1 : bit_length(d);
                break;
            }
            case GEAK_F64: {
                const u64 pa = reinterpret_cast<const u64 *>(cb)[i], pb = reinterpret_cast<const u64 *>(rb)[i];
                const long long ma = (long long)(pa & 0x7FFFFFFFFFFFFFFFull), mb = (long long)(pb & 0x7FFFFFFFFFFFFFFFull);
                const long long oa = ((long long)pa < 0) ? -ma : ma, ob = ((long long)pb < 0) ? -mb : mb;
                const u64 d = (oa > ob) ? (u64)oa - (u64)ob : (u64)ob - (u64)oa;
                slot = (ma > 0x7FF0000000000000ll || mb > 0x7FF0000000000000ll) ? st.nslots - 1 : bit_length(d);
                break;
            }
            default: {
                const long long a = load_elem_int(cb, i, it.dtype), b = load_elem_int(rb, i, it.dtype);
                const u64 d = (a > b) ? (u64)a - (u64)b : (u64)b - (u64)a;
                slot = bit_length(d);
                break;
            }
            }
            (void)__hip_atomic_fetch_add(row + slot, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
}

__global__ __launch_bounds__(kBlockThreads, 4) void ulp_histogram_kernel(const UlpArgs p)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & (kWaveSize - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    UlpState st;
    st.nslots = p.nslots;
    st.rows_off = (uint32_t)(uintptr_t)(GEAK_AS_LDS unsigned char *)lds + wave * p.k_count * p.nslots * 4u;
    {
        GEAK_AS_LDS uint32_t *rows = (GEAK_AS_LDS uint32_t *)st.rows_off;
        for (uint32_t i = lane; i < p.k_count * p.nslots; i += kWaveSize) rows[i] = 0;
    }
    UlpRunArgs r;
    r.items = p.items;
    r.ref = p.ref;
    r.cand = p.cand_table;
    r.partials = p.partials;
    r.num_items = p.num_items;
    r.K = p.num_candidates;
    r.k_begin = p.k_begin;
    r.k_count = p.k_count;

    const GEAK_AS_CONSTANT uint32_t *wave_first = (const GEAK_AS_CONSTANT uint32_t *)p.wave_first;
    uint32_t j = wave_first[blockIdx.x * kWavesPerBlock + wave];
    while (j < p.num_items) {                                   // kNoItem ends the list
        const geak_item it = load_work_item(p.items, j);
        if (it.flags & GEAK_ITEM_ALIGNED) {
            r.first_item = j;
            uint32_t next_j;
            switch (it.dtype) {
            case GEAK_F32:  next_j = ulp_run<GEAK_F32>(r, st); break;
            case GEAK_F16:  next_j = ulp_run<GEAK_F16>(r, st); break;
            case GEAK_BF16: next_j = ulp_run<GEAK_BF16>(r, st); break;
            case GEAK_I32:  next_j = ulp_run<GEAK_I32>(r, st); break;
            case GEAK_I64:  next_j = ulp_run<GEAK_I64>(r, st); break;
            case GEAK_U8:   next_j = ulp_run<GEAK_U8>(r, st); break;
            case GEAK_F64:  next_j = ulp_run<GEAK_F64>(r, st); break;
            default:        next_j = ulp_run<GEAK_I8>(r, st); break;
            }
            j = __builtin_amdgcn_readfirstlane(next_j);
            continue;
        }
        ulp_head(it, p.ref, p.cand_table, st, p.k_begin, p.k_count, lane);
        if (it.flags & GEAK_ITEM_LAST) ulp_end_run(st, p.partials, it.slot, p.num_candidates, p.k_begin, p.k_count, lane);
        j = it.next;
    }
}

// ---- reduce: one block per (segment, candidate); thread t sums bin t over the segment's slots -----------
constexpr int kUlpReduceThreads = 128;
__global__ __launch_bounds__(kUlpReduceThreads) void ulp_reduce_kernel(const UlpReduceArgs p)
{
    const uint32_t K = p.num_candidates;
    const uint32_t seg = blockIdx.x / K, k = blockIdx.x % K;
    const uint32_t bin = threadIdx.x;
    if (bin >= GEAK_ULP_BINS) return;
    // bin -> slot of the partial rows: the NaN bin is the last slot; bins the plan's dtypes cannot reach hold nothing
    const bool reachable = (bin == GEAK_ULP_BINS - 1) || (bin < p.nslots - 1);
    const uint32_t slot_in_row = (bin == GEAK_ULP_BINS - 1) ? p.nslots - 1 : bin;
    u64 sum = 0;
    if (reachable) {
        const uint32_t s0 = p.slot_begin[seg], s1 = p.slot_begin[seg + 1];
        for (uint32_t s = s0; s < s1; ++s) sum += p.partials[((u64)s * K + k) * p.nslots + slot_in_row];
    }
    p.hist[(u64)blockIdx.x * GEAK_ULP_BINS + bin] = sum;
}

}  // namespace

int launch_ulp_histogram(const UlpArgs &args, uint32_t grid_blocks, uint32_t lds_bytes, void *stream)
{
    if (!args.num_items || !args.k_count) return (int)hipSuccess;
    hipLaunchKernelGGL(ulp_histogram_kernel, dim3(grid_blocks), dim3(kBlockThreads), lds_bytes, (hipStream_t)stream, args);
    return (int)hipGetLastError();
}

int launch_ulp_reduce(const UlpReduceArgs &args, void *stream)
{
    const uint64_t pairs = (uint64_t)args.num_segments * args.num_candidates;
    if (!pairs) return (int)hipSuccess;
    hipLaunchKernelGGL(ulp_reduce_kernel, dim3((uint32_t)pairs), dim3(kUlpReduceThreads), 0, (hipStream_t)stream, args);
    return (int)hipGetLastError();
}

}  // namespace geak
