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
// four 16-byte loads per lane in flight.  The low bins are counted without touching memory: for the
// 32- and 64-bit dtypes four cumulative classes (distance < 1, < 2, < 4, < 8) with lane masks in
// scalar registers; for the 16-bit dtypes, whose budget of instructions per byte is half as large,
// both halves of a word at once with packed arithmetic and two byte-permute tables that turn
// min(d, 8) into increments of per-lane counters.  Only lanes 8 or more steps away (or NaN) touch
// the wave's histogram rows in LDS, one atomic add per lane.  Per (wave, segment run, candidate) the
// rows are written, without atomics, to a partial table; the reduce kernel sums the partial rows of
// a segment.  A pass covers as many candidates as fit the wave's LDS rows.
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

template <int DT> constexpr bool kUlpFloating = (DT == GEAK_F32 || DT == GEAK_F16 || DT == GEAK_BF16 || DT == GEAK_F64 ||
                                                DT == GEAK_F8E4M3 || DT == GEAK_F8E5M2);

// the magnitude pattern of +Inf, in the ord type
template <int DT> __device__ __forceinline__ typename UlpTraits<DT>::Ord ulp_inf()
{
    if constexpr (DT == GEAK_F32) return 0x7F800000;
    else if constexpr (DT == GEAK_F16) return 0x7C00;
    else if constexpr (DT == GEAK_BF16) return 0x7F80;
    else if constexpr (DT == GEAK_F8E5M2) return 0x7C;
    else if constexpr (DT == GEAK_F8E4M3) return 0x7E;      // no infinities: the ladder ends at the largest finite value, the pattern above it is NaN
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
    } else if constexpr (DT == GEAK_F8E4M3 || DT == GEAK_F8E5M2) {
        const uint32_t v = (q[e >> 2] >> (8 * (e & 3))) & 0xFFu;
        const int mag = (int)(v & 0x7Fu);
        return (v & 0x80u) ? -mag : mag;
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

// Counters of one (item, candidate): cumulative classes (distance < 1, < 2, < 4, < 8) in scalar registers.
struct UlpCounts {
    uint32_t lt1, lt2, lt4, lt8;
};

// Floating elements where a or b is NaN carry the distance "all ones", a value no pair of numbers
// reaches (the largest distance, -Inf to +Inf, is twice the pattern of Inf).  Such lanes fall
// through the four classes like any far lane and are sorted out where the LDS row is addressed.
template <typename D, bool FLOATING>
__device__ __forceinline__ uint32_t ulp_slot(D d, uint32_t nslots)
{
    if (FLOATING && d == (D)~(D)0) return nslots - 1;
    // only lanes 8 or more steps away come here: d is not 0
    if constexpr (sizeof(D) == 8) return 64u - (uint32_t)__builtin_clzll((u64)d);
    else return 32u - (uint32_t)__builtin_clz((uint32_t)d);
}

// One element position of all 64 lanes: the four classes by lane mask, lanes beyond them straight
// into the LDS row (one atomic add per lane; equal addresses are serialised by the LDS).
template <typename D, bool FLOATING>
__device__ __forceinline__ void ulp_classify(D d, UlpCounts &c, GEAK_AS_LDS uint32_t *row, uint32_t nslots)
{
    const bool near = d < (D)8;
    const u64 m8 = __builtin_amdgcn_ballot_w64(near);
    c.lt1 += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(d < (D)1));
    c.lt2 += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(d < (D)2));
    c.lt4 += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(d < (D)4));
    c.lt8 += (uint32_t)__builtin_popcountll(m8);
    if (~m8) {
        if (__builtin_amdgcn_inverse_ballot_w64(~m8)) (void)__hip_atomic_fetch_add(row + ulp_slot<D, FLOATING>(d, nslots), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    // one element's lane masks at a time: the counters are a running chain in four scalar registers
    asm volatile("" : "+s"(c.lt1), "+s"(c.lt2), "+s"(c.lt4), "+s"(c.lt8));
}

// ---- the other dtypes: element by element ------------------------------------------------------------
// all ones if the ord value is that of a NaN
template <int DT>
__device__ __forceinline__ typename UlpTraits<DT>::Dist ulp_nan_mark(typename UlpTraits<DT>::Ord o)
{
    typedef typename UlpTraits<DT>::Ord Ord;
    typedef typename UlpTraits<DT>::Dist D;
    const Ord mag = o < 0 ? -o : o;
    // magnitudes above the pattern of Inf reach the sign bit when lifted by (largest magnitude - Inf)
    const D lifted = (D)mag + ((D)(~(D)0 >> 1) - (D)ulp_inf<DT>());
    return (D)((Ord)lifted >> (sizeof(Ord) * 8 - 1));
}

// the scalar counters of one (item, candidate) go into the row; `pad` absent elements of a tail
// were read as 0 on both sides and counted as distance 0
__device__ __forceinline__ void ulp_commit(const UlpCounts &c, uint32_t pad, GEAK_AS_LDS uint32_t *row, int lane)
{
    if (lane == 0) {
        const uint32_t b0 = c.lt1 - pad, b1 = c.lt2 - c.lt1, b2 = c.lt4 - c.lt2, b3 = c.lt8 - c.lt4;
        if (b0) (void)__hip_atomic_fetch_add(row + 0, b0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (b1) (void)__hip_atomic_fetch_add(row + 1, b1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (b2) (void)__hip_atomic_fetch_add(row + 2, b2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (b3) (void)__hip_atomic_fetch_add(row + 3, b3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
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
    const SegDesc *segments;
    const uint64_t *ref_item_offset;     // per item, for references with a layout of their own (null when the plan has none)
};

__device__ __forceinline__ uint32_t uniform32(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
template <typename T>
__device__ __forceinline__ T *uniform_ptr(T *p)
{
    const u64 v = reinterpret_cast<u64>(p);
    const u64 lo = uniform32((uint32_t)v), hi = uniform32((uint32_t)(v >> 32));
    return reinterpret_cast<T *>(lo | (hi << 32));
}

// The staged reference slice of one item and the comparison of one candidate vector against it.
template <int DT> struct UlpRef {
    typedef typename UlpTraits<DT>::Ord Ord;
    typedef typename UlpTraits<DT>::Dist D;
    static constexpr int E = Traits<DT>::E;
    typedef UlpCounts Counts;
    Ord ob[kVecPerLane * E];
    uint32_t nan_vectors;                                    // bit v: some lane's reference vector v holds a NaN
    static __device__ __forceinline__ Counts zero() { return Counts{0u, 0u, 0u, 0u}; }
    static __device__ __forceinline__ void commit(const Counts &c, uint32_t elements, GEAK_AS_LDS uint32_t *row, int lane)
    {
        ulp_commit(c, (uint32_t)(kWaveSize * kVecPerLane * E) - elements, row, lane);
    }

    template <int V> __device__ __forceinline__ void stage(const u32x4 &q)
    {
        if constexpr (V == 0) nan_vectors = 0;
        bool any_nan = false;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const Ord o = ulp_ord<DT>(q, e);
            ob[V * E + e] = o;
            if constexpr (kUlpFloating<DT>) any_nan |= ulp_is_nan<DT>(o);
        }
        if constexpr (kUlpFloating<DT>)
            if (__builtin_amdgcn_ballot_w64(any_nan)) nan_vectors |= 1u << V;
    }
    template <int V> __device__ __forceinline__ void compare(const u32x4 &q, UlpCounts &c, GEAK_AS_LDS uint32_t *row, uint32_t nslots) const
    {
        const bool ref_nan = kUlpFloating<DT> && ((nan_vectors >> V) & 1u);
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const Ord oa = ulp_ord<DT>(q, e);
            D d = ulp_dist<DT>(oa, ob[V * E + e]);
            if constexpr (kUlpFloating<DT>) {
                d |= ulp_nan_mark<DT>(oa);
                if (ref_nan) d |= ulp_nan_mark<DT>(ob[V * E + e]);
            }
            ulp_classify<D, kUlpFloating<DT>>(d, c, row, nslots);
        }
    }
};

// 16-bit floating dtypes: both halves of a word at once, with packed 16-bit integer arithmetic.
//   ord      magnitude, negated (two's complement, 16 bits) in a negative half
//   distance max - min of the two ord values; it is below 2^16, so the wrapping subtraction is exact
//   classes  t = min(d, 8) per half selects, as a byte selector of v_perm_b32, an entry of an 8-byte
//            table: 1 for d = 1 and 64 for d = 2, 3 in the first table, 1 for d = 4 .. 7 in the second;
//            d = 0 selects 0 and so does t = 8 (selector 8 yields the sign of table byte 1).  The upper
//            byte of each half of t is 0 and selects entry 0 as well.  Adding the results to two
//            per-lane accumulators counts the three classes in 6-bit fields of each half (a lane
//            sees 16 words per slice); they are summed over the wave once per candidate slice.
//   NaN      a NaN in the candidate needs no test while the reference vector holds nothing within 8
//            steps of Inf or beyond: its distance is then at least 8, and the far path, which looks
//            at the pattern again, sorts it out.  Reference vectors that do hold such a value take
//            the plain path, element by element.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u16x2 as_u16x2(uint32_t w) { return __builtin_bit_cast(u16x2, w); }
__device__ __forceinline__ s16x2 as_s16x2(uint32_t w) { return __builtin_bit_cast(s16x2, w); }
__device__ __forceinline__ uint32_t as_word(u16x2 v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ uint32_t as_word(s16x2 v) { return __builtin_bit_cast(uint32_t, v); }

__device__ __forceinline__ uint32_t ulp_dist_pair(uint32_t oa2, uint32_t ob2)
{
    const s16x2 a = as_s16x2(oa2), b = as_s16x2(ob2);
    const s16x2 hi = __builtin_elementwise_max(a, b), lo = __builtin_elementwise_min(a, b);
    return as_word(as_u16x2(as_word(hi)) - as_u16x2(as_word(lo)));
}
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b)
{
    uint32_t r;                       // as the instruction itself: from min() the compiler derives a compare and select per half
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
// Sum over the wave, wave-uniform result: four data-parallel-primitive steps inside each row of 16
// lanes (neighbour, other pair, other quad mirrored, other half mirrored), then one lane of each row.
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x)
{
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, false);     // quad_perm [1,0,3,2]
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, false);     // quad_perm [2,3,0,1]
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, false);    // row_half_mirror
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xF, 0xF, false);    // row_mirror
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 0) + (uint32_t)__builtin_amdgcn_readlane((int)x, 16) +
           (uint32_t)__builtin_amdgcn_readlane((int)x, 32) + (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
}

struct UlpCounts16 {
    uint32_t near12;          // per half, 6-bit fields: elements of this lane with d = 1 (bits 0-5) and d = 2, 3 (bits 6-11)
    uint32_t near4;           // per half: d = 4 .. 7 (bits 0-5)
    UlpCounts plain;          // what the plain path (reference vectors near Inf) counted, cumulative classes
    uint32_t far_lane;        // elements of this lane sent down the far path
};

// The same machinery serves the 8-bit floating formats: two bytes at a time are spread into the
// halves of a word (one byte permute), after which only the position of the sign bit differs.
template <int DT> struct UlpRefPacked {
    typedef UlpCounts16 Counts;
    static constexpr bool kBytes = (DT == GEAK_F8E4M3 || DT == GEAK_F8E5M2);
    static constexpr int E = Traits<DT>::E;
    static constexpr int kPairs = E / 2;                       // pair words per vector
    static constexpr uint32_t kMag = kBytes ? 0x7Fu : 0x7FFFu;
    static constexpr uint32_t kInf = (DT == GEAK_F16) ? 0x7C00u : (DT == GEAK_BF16) ? 0x7F80u : (DT == GEAK_F8E5M2) ? 0x7Cu : 0x7Eu;
    uint32_t ob2[kVecPerLane * kPairs];
    uint32_t edge_vectors;                                     // bit v: some lane's reference vector v holds a magnitude >= Inf - 8

    static __device__ __forceinline__ Counts zero() { return Counts{0u, 0u, UlpCounts{0u, 0u, 0u, 0u}, 0u}; }

    // elements 2j and 2j + 1 of a vector, one per half of a word
    template <int j> static __device__ __forceinline__ uint32_t pair_word(const u32x4 &q)
    {
        if constexpr (!kBytes) return q[j];
        else return __builtin_amdgcn_perm(0u, q[j >> 1], (j & 1) ? 0x0C030C02u : 0x0C010C00u);     // selector 0x0C yields 0
    }
    static __device__ __forceinline__ uint32_t ord_pair(uint32_t pw)
    {
        const uint32_t mag = pw & (kMag * 0x00010001u);
        const uint32_t up = kBytes ? as_word(as_u16x2(pw) << (unsigned short)8) : pw;     // sign bit to bit 15 of its half
        const uint32_t sign = as_word(as_s16x2(up) >> (short)15);                            // all ones in a negative half
        return as_word(as_u16x2(mag ^ sign) - as_u16x2(sign));                               // negated there
    }

    template <int V> __device__ __forceinline__ void stage(const u32x4 &q)
    {
        if constexpr (V == 0) edge_vectors = 0;
        bool edge = false;
        static_for<kPairs>([&](auto idx) {
            constexpr int j = decltype(idx)::value;
            const uint32_t pw = pair_word<j>(q);
            ob2[V * kPairs + j] = ord_pair(pw);
            edge |= (pw & kMag) >= kInf - 8u || ((pw >> 16) & kMag) >= kInf - 8u;
        });
        if (__builtin_amdgcn_ballot_w64(edge)) edge_vectors |= 1u << V;
    }

    // far path of one half: the lanes 8 or more steps away.  The slot is the distance's bit length,
    // addressed as (row + 32 slots) - 4 * leading zeros; a NaN among these lanes is the exception.
    static __device__ __forceinline__ void far(uint32_t pattern, uint32_t d, GEAK_AS_LDS uint32_t *row, uint32_t nslots)
    {
        const uint32_t row_bytes = (uint32_t)(uintptr_t)row;
        const uint32_t by_length = row_bytes + 128u - 4u * (uint32_t)__builtin_clz(d);
        const bool is_nan = (pattern & kMag) > kInf;
        if (__builtin_amdgcn_ballot_w64(is_nan) == 0) {
            (void)__hip_atomic_fetch_add((GEAK_AS_LDS uint32_t *)by_length, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        } else {
            uint32_t addr = is_nan ? row_bytes + 4u * (nslots - 1) : by_length;
            asm volatile("" : "+v"(addr));          // keeps the two cases apart: merged, both would pay for the selection
            (void)__hip_atomic_fetch_add((GEAK_AS_LDS uint32_t *)addr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }

    template <int V> __device__ __forceinline__ void compare(const u32x4 &q, Counts &c, GEAK_AS_LDS uint32_t *row, uint32_t nslots) const
    {
        if ((edge_vectors >> V) & 1u) {                      // rare: element by element, NaN tested on both sides
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const int oa = ulp_ord<DT>(q, e);
                const uint32_t pair = ob2[V * kPairs + (e >> 1)];
                const int ob = (e & 1) ? ((int)pair >> 16) : (int)(short)(pair & 0xFFFFu);
                const uint32_t d = ulp_dist<DT>(oa, ob) | ulp_nan_mark<DT>(oa) | ulp_nan_mark<DT>(ob);
                ulp_classify<uint32_t, true>(d, c.plain, row, nslots);
            }
            return;
        }
        uint32_t pw[kPairs], d2[kPairs], t2[kPairs], any = 0;
        static_for<kPairs>([&](auto idx) {
            constexpr int j = decltype(idx)::value;
            pw[j] = pair_word<j>(q);
            d2[j] = ulp_dist_pair(ord_pair(pw[j]), ob2[V * kPairs + j]);
            t2[j] = pk_min_u16(d2[j], 0x00080008u);
            c.near12 += __builtin_amdgcn_perm(0u, 0x40400100u, t2[j]);       // table bytes 0 .. 7: 0, 1, 64, 64, 0, 0, 0, 0
            c.near4 += __builtin_amdgcn_perm(0x01010101u, 0u, t2[j]);        //                     0, 0, 0, 0, 1, 1, 1, 1
            any |= t2[j];
        });
        if (__builtin_amdgcn_ballot_w64((any & 0x00080008u) != 0)) {
            // Some lane has elements 8 or more steps away.  Every lane walks through its own (bit i of
            // `todo`: half i of the vector), so the wave issues as many rounds of LDS atomics as the
            // worst lane has such elements, not one round per element position.
            uint32_t todo = 0;
#pragma unroll
            for (int j = 0; j < kPairs; ++j) todo |= (((t2[j] >> 3) & 1u) | ((t2[j] >> 18) & 2u)) << (2 * j);
            c.far_lane += (uint32_t)__builtin_popcount(todo);
            while (__builtin_amdgcn_ballot_w64(todo != 0)) {
                if (todo != 0) {
                    const uint32_t i = (uint32_t)__builtin_ctz(todo);
                    todo &= todo - 1u;
                    const uint32_t word = i >> 1, shift = (i & 1u) * 16u;
                    uint32_t dd = d2[0], qq = pw[0];
#pragma unroll
                    for (int j = 1; j < kPairs; ++j) {
                        dd = word == (uint32_t)j ? d2[j] : dd;
                        qq = word == (uint32_t)j ? pw[j] : qq;
                    }
                    far(qq >> shift, (dd >> shift) & 0xFFFFu, row, nslots);
                }
            }
        }
    }

    // `elements` of the slice (absent ones of a tail not counted) were compared.  Elements at distance 0
    // were counted nowhere on the packed path: they are what is left.  Of a plain-path vector's
    // positions (absent ones included, at distance 0) those outside its four classes went to the row there.
    __device__ __forceinline__ void commit(const Counts &c, uint32_t elements, GEAK_AS_LDS uint32_t *row, int lane) const
    {
        const uint32_t n1 = (c.near12 & 0x3Fu) + ((c.near12 >> 16) & 0x3Fu);
        const uint32_t n2 = ((c.near12 >> 6) & 0x3Fu) + ((c.near12 >> 22) & 0x3Fu);
        const uint32_t n4 = (c.near4 & 0x3Fu) + ((c.near4 >> 16) & 0x3Fu);
        // at most 64 per lane and class: two counts share a register through the wave sum (below 2^16 each)
        const uint32_t s12 = wave_sum_u32(n1 | (n2 << 16)), s4f = wave_sum_u32(n4 | (c.far_lane << 16));
        const uint32_t s4 = s4f & 0xFFFFu, far_total = s4f >> 16;
        if (lane == 0) {
            const uint32_t b1 = (s12 & 0xFFFFu) + (c.plain.lt2 - c.plain.lt1), b2 = (s12 >> 16) + (c.plain.lt4 - c.plain.lt2);
            const uint32_t b3 = s4 + (c.plain.lt8 - c.plain.lt4);
            const uint32_t plain_far = (uint32_t)__builtin_popcount(edge_vectors) * (uint32_t)(kWaveSize * E) - c.plain.lt8;
            const uint32_t b0 = elements - b1 - b2 - b3 - far_total - plain_far;
            if (b0) (void)__hip_atomic_fetch_add(row + 0, b0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (b1) (void)__hip_atomic_fetch_add(row + 1, b1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (b2) (void)__hip_atomic_fetch_add(row + 2, b2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (b3) (void)__hip_atomic_fetch_add(row + 3, b3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
};

// bytes (integers and the 8-bit floating formats): nothing staged but the vector itself; words that
// are equal in every lane are counted at once -- unless the reference vector holds a NaN, whose
// equal copy in a candidate is not at distance 0 but in the NaN bin.
template <int DT> struct UlpRefBytes {
    typedef UlpCounts Counts;
    u32x4 raw[kVecPerLane];
    uint32_t nan_vectors;
    static __device__ __forceinline__ Counts zero() { return Counts{0u, 0u, 0u, 0u}; }
    static __device__ __forceinline__ void commit(const Counts &c, uint32_t elements, GEAK_AS_LDS uint32_t *row, int lane)
    {
        ulp_commit(c, (uint32_t)(kWaveSize * kVecPerLane * 16) - elements, row, lane);
    }
    template <int V> __device__ __forceinline__ void stage(const u32x4 &q)
    {
        raw[V] = q;
        if constexpr (V == 0) nan_vectors = 0;
        if constexpr (kUlpFloating<DT>) {
            bool any_nan = false;
#pragma unroll
            for (int e = 0; e < 16; ++e) any_nan |= ulp_is_nan<DT>(ulp_ord<DT>(q, e));
            if (__builtin_amdgcn_ballot_w64(any_nan)) nan_vectors |= 1u << V;
        }
    }
    template <int V> __device__ __forceinline__ void compare(const u32x4 &q, Counts &c, GEAK_AS_LDS uint32_t *row, uint32_t nslots) const
    {
        const bool ref_nan = kUlpFloating<DT> && ((nan_vectors >> V) & 1u);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (!ref_nan && __builtin_amdgcn_ballot_w64(q[w] != raw[V][w]) == 0) {
                c.lt1 += 4 * kWaveSize; c.lt2 += 4 * kWaveSize; c.lt4 += 4 * kWaveSize; c.lt8 += 4 * kWaveSize;
                continue;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int a = ulp_ord<DT>(q, 4 * w + e), b = ulp_ord<DT>(raw[V], 4 * w + e);
                uint32_t d = ulp_dist<DT>(a, b);
                if constexpr (kUlpFloating<DT>) d |= ulp_nan_mark<DT>(a) | ulp_nan_mark<DT>(b);
                ulp_classify<uint32_t, kUlpFloating<DT>>(d, c, row, nslots);
            }
        }
    }
};

template <int DT> struct UlpRefOf { typedef UlpRef<DT> type; };
template <> struct UlpRefOf<GEAK_F16> { typedef UlpRefPacked<GEAK_F16> type; };
template <> struct UlpRefOf<GEAK_BF16> { typedef UlpRefPacked<GEAK_BF16> type; };
template <> struct UlpRefOf<GEAK_U8> { typedef UlpRefBytes<GEAK_U8> type; };
template <> struct UlpRefOf<GEAK_I8> { typedef UlpRefBytes<GEAK_I8> type; };
template <> struct UlpRefOf<GEAK_F8E4M3> { typedef UlpRefPacked<GEAK_F8E4M3> type; };
template <> struct UlpRefOf<GEAK_F8E5M2> { typedef UlpRefPacked<GEAK_F8E5M2> type; };

// TAIL = false: a run of consecutive FULL items of one dtype in the wave's list, every load an
// unguarded 16-byte load, the next item's reference slice fetched behind the last candidate.
// TAIL = true: one aligned item that is not a full one (a segment's tail, or a group of short rows of a
// pitched segment), guarded loads.
// Returns the index of the wave's first item it did not process.
template <int DT, bool TAIL, int KIND = kTailPlain>
__device__ __noinline__ uint32_t ulp_run(const UlpRunArgs in, const UlpState st_in)
{
    constexpr bool full = !TAIL;
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
    const ItemShape shape = item_shape<DT, KIND>(it, uniform_ptr(in.segments));
    const u64 shift_bytes = (u64)shape.skip * Traits<DT>::W;       // a shifted item is read from the boundary before it
    // vector v of this lane: unguarded inside a run of full items, by the item's shape (tail or row group) otherwise
    const auto fetch = [&](const unsigned char *base, int v, uint32_t n) {
        if constexpr (TAIL) return load_shaped<DT, KIND>(base - shift_bytes, lane, v, n, shape);
        else return load_vec<DT>(base, lane, v, n, full);
    };
    u32x4 cur[kVecPerLane];
    // a reference with a layout of its own: a full item's slice lies at the offset the plan's table gives (whole
    // vectors at any alignment); the other shapes go through the guarded loads of the mapped reference
    const GEAK_AS_CONSTANT unsigned long long *ref_table = (const GEAK_AS_CONSTANT unsigned long long *)uniform_ptr(in.ref_item_offset);
    const auto ref_offset_of = [&](const geak_item &item, uint32_t index) -> u64 {
        return (item.flags & GEAK_ITEM_REFMAP) ? ref_table[index] : item.byte_offset;
    };
    bool mapped = false;
    if constexpr (TAIL) mapped = (it.flags & GEAK_ITEM_REFMAP) != 0;          // uniform
    if (mapped) {
        const RefPlace place = ref_place<DT>(it, j, uniform_ptr(in.segments), uniform_ptr(in.ref_item_offset));
        uint32_t first;
#pragma unroll
        for (int v = 0; v < kVecPerLane; ++v)
            cur[v] = load_ref_slot<DT, KIND>(ref_base, place, (uint32_t)(v * kWaveSize + lane), it.numel, shape, first);
    } else {
#pragma unroll
        for (int v = 0; v < kVecPerLane; ++v) cur[v] = fetch(ref_base + ref_offset_of(it, j), v, it.numel);
    }
    typedef typename UlpRefOf<DT>::type Ref;
    Ref ref;
    for (;;) {
        const uint32_t jn = it.next;
        bool more = !TAIL && jn < num_items;
        geak_item nx = it;
        if (more) {
            nx = load_work_item(items, jn);
            more = nx.dtype == DT && (nx.flags & GEAK_ITEM_FULL);
        }
        // stage the reference slice; its registers are refilled with the pass's first candidate
        {
            const unsigned char *first = table_entry(cand, k_begin) + it.byte_offset;
            ref.template stage<0>(cur[0]); cur[0] = fetch(first, 0, it.numel);
            ref.template stage<1>(cur[1]); cur[1] = fetch(first, 1, it.numel);
            ref.template stage<2>(cur[2]); cur[2] = fetch(first, 2, it.numel);
            ref.template stage<3>(cur[3]); cur[3] = fetch(first, 3, it.numel);
        }
        for (uint32_t kk = 0; kk < k_count; ++kk) {
            const bool last = kk + 1 == k_count;
            // Every step refills its registers, so that the number of loads in flight is known at each wait:
            // behind the run's very last slice the same slice is simply read again (from the cache).
            const unsigned char *next = !last ? table_entry(cand, k_begin + kk + 1) + it.byte_offset
                                      : more ? ref_base + ref_offset_of(nx, jn)
                                             : table_entry(cand, k_begin + kk) + it.byte_offset;
            GEAK_AS_LDS uint32_t *row = ulp_row(st, kk);
            typename Ref::Counts c = Ref::zero();
            ref.template compare<0>(cur[0], c, row, st.nslots); cur[0] = fetch(next, 0, it.numel);
            ref.template compare<1>(cur[1], c, row, st.nslots); cur[1] = fetch(next, 1, it.numel);
            ref.template compare<2>(cur[2], c, row, st.nslots); cur[2] = fetch(next, 2, it.numel);
            ref.template compare<3>(cur[3], c, row, st.nslots); cur[3] = fetch(next, 3, it.numel);
            ref.commit(c, it.numel, row, lane);
        }
        if (it.flags & GEAK_ITEM_LAST) ulp_end_run(st, partials, it.slot, K, k_begin, k_count, lane);
        if (!more) break;
        it = nx;
        j = jn;
    }
    return it.next;
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
    r.segments = p.segments;
    r.ref_item_offset = p.ref_item_offset;

    const GEAK_AS_CONSTANT uint32_t *wave_first = (const GEAK_AS_CONSTANT uint32_t *)p.wave_first;
    uint32_t j = wave_first[table_range_of_block(blockIdx.x, gridDim.x, p.unit_groups, p.block_map) * kWavesPerBlock + wave];
    while (j < p.num_items) {                                   // kNoItem ends the list
        const geak_item it = load_work_item(p.items, j);
        r.first_item = j;
        uint32_t next_j = it.next;
        if (it.flags & GEAK_ITEM_FULL) {
            for_dtype(it.dtype, [&](auto dt) { next_j = ulp_run<decltype(dt)::value, false>(r, st); });
        } else if (it.flags & GEAK_ITEM_ROWS) {
            for_dtype(it.dtype, [&](auto dt) { next_j = ulp_run<decltype(dt)::value, true, kTailRows>(r, st); });
        } else if (it.flags & GEAK_ITEM_ALIGNED) {
            for_dtype(it.dtype, [&](auto dt) { next_j = ulp_run<decltype(dt)::value, true, kTailPlain>(r, st); });
        } else {
            for_dtype(it.dtype, [&](auto dt) { next_j = ulp_run<decltype(dt)::value, true, kTailShifted>(r, st); });
        }
        j = __builtin_amdgcn_readfirstlane(next_j);
    }
}

// ---- reduce: one block per (segment, candidate) ----------------------------------------------------
// The pair's partial rows (one per slot of the segment) are summed by 16 waves: a wave takes every
// 16th row, its lanes the row's slots (a row is contiguous), eight rows in flight at a time; the
// waves' sums meet in LDS.
constexpr int kUlpReduceThreads = 1024;
constexpr int kUlpReduceWaves = kUlpReduceThreads / kWaveSize;
__global__ __launch_bounds__(kUlpReduceThreads) void ulp_reduce_kernel(const UlpReduceArgs p)
{
    __shared__ u64 sums[kUlpReduceWaves][2 * kWaveSize];
    const uint32_t K = p.num_candidates, nslots = p.nslots;
    const uint32_t seg = blockIdx.x / K, k = blockIdx.x % K;
    const uint32_t lane = threadIdx.x & (kWaveSize - 1), wave = threadIdx.x / kWaveSize;
    const uint32_t s0 = p.slot_begin[seg], s1 = p.slot_begin[seg + 1];
    const bool has0 = lane < nslots, has1 = lane + kWaveSize < nslots;          // nslots <= 66: two slots per lane at most
    u64 acc0 = 0, acc1 = 0;
    constexpr uint32_t kAhead = 8;
    for (uint32_t s = s0 + wave; s < s1; s += kUlpReduceWaves * kAhead) {
        uint32_t v0[kAhead], v1[kAhead];
#pragma unroll
        for (uint32_t u = 0; u < kAhead; ++u) {
            const uint32_t row = s + u * kUlpReduceWaves;
            const uint32_t *r = p.partials + ((u64)row * K + k) * nslots;
            v0[u] = (row < s1 && has0) ? r[lane] : 0u;
            v1[u] = (row < s1 && has1) ? r[lane + kWaveSize] : 0u;
        }
#pragma unroll
        for (uint32_t u = 0; u < kAhead; ++u) { acc0 += v0[u]; acc1 += v1[u]; }
    }
    sums[wave][lane] = acc0;
    sums[wave][lane + kWaveSize] = acc1;
    __syncthreads();
    const uint32_t bin = threadIdx.x;
    if (bin < GEAK_ULP_BINS) {
        // bin -> slot of the partial rows: the NaN bin is the last slot; bins the plan's dtypes cannot reach hold nothing
        const bool reachable = (bin == GEAK_ULP_BINS - 1) || (bin < nslots - 1);
        const uint32_t slot_in_row = (bin == GEAK_ULP_BINS - 1) ? nslots - 1 : bin;
        u64 sum = 0;
        if (reachable)
            for (int w = 0; w < kUlpReduceWaves; ++w) sum += sums[w][slot_in_row];
        p.hist[(u64)blockIdx.x * GEAK_ULP_BINS + bin] = sum;
    }
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
