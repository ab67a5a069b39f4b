// HIP kernels of the output-equivalence check for gfx950 (wave64).
//
// The rule (GEAK section 3.1, tolerance-based comparison of output tensors against reference
// outputs; the reference is ground truth, section 3.3):
//     d = |a - b|, tol = atol + rtol*|b| (binary32, one rounding per step), close <=> d <= tol,
//     NaN: close only if equal_nan and both NaN; +-Inf: close only if a == b; integers: a == b.
//     fp16, bf16 and the 8-bit formats are widened exactly to binary32 first; binary64 runs the same
//     rule in binary64 arithmetic.
//
// compare kernel -- one wavefront per work item (4 KiB of every tensor).
//   * The wave loads its slice of the reference once, decodes it to binary32 and keeps b and tol
//     in registers (lane L holds the same element positions for the reference and every
//     candidate, so nothing has to be exchanged between lanes); the slice of each of the K
//     candidates is then streamed past it with 16-byte loads, one candidate ahead of the compute.
//     HBM traffic is K + 1 tensors.
//   * Reference elements for which the bare inequality is not the rule (b NaN or +-Inf, or tol
//     overflowed to +Inf) get tol = -1 ("poisoned"): the inequality then always reports a
//     suspect, and a per-candidate fix-up applies the NaN / Inf rule to exactly those slots.
//   * mismatch count: v_cmp -> 64-bit lane mask -> s_bcnt1, accumulated in LDS per (wave, k).
//   * max_abs_err / max_rel_err: the current maxima are read from a board of running maxima in the
//     workspace and used as wave-uniform thresholds.  The board holds R replicas per (segment,
//     candidate) -- a block reads and raises replica (block mod R), the reduce kernel takes the
//     maximum over them -- because many waves raising one address serialise at tens of
//     microseconds per atomic.  Per element only `d > max_abs` and the sign of
//     fma(max_rel, |b|, -d) matter (both folded over a lane's vector with three-operand max / min
//     and tested once): the fused result is the correctly rounded value of
//     max_rel*|b| - d and rounding keeps the sign of the exact value, so "negative" is exactly
//     "d/|b| would exceed max_rel", with no division.  When any lane trips, that vector is
//     evaluated exactly in registers (true binary32 division for the lanes that exceed what they
//     have seen) and the maxima are raised with a 64-bit atomic max on the bit patterns of the
//     non-negative doubles.  Rounding is monotone, so the maximum of the rounded quotients is the
//     rounded quotient of a tripping element.
//   * An item that is not a full one -- a segment's tail, a group of short rows of a pitched
//     segment, or the first item of a segment that starts off the 16-byte grid (read from the
//     boundary before it) -- is compared in batches of several candidates per round of loads, with
//     guarded loads that read everything outside the item as 0.
//   * first_mismatch: the wave only remembers the first of its items that holds a mismatch; the
//     reduce kernel re-reads that one item and finds the exact index.
// reduce kernel -- one block per (segment, candidate), or one wave when there are many pairs: sums
//   counts over the segment's slots, takes the least item index, rescans that item with the full
//   rule, folds the replicas of the maxima, writes the record.
//
// Blocks of the compare kernel start at different candidates so that the first, expensive, visit
// of a (segment, candidate) pair is spread out and later visitors find the maxima already raised:
// the blocks that share replica r of the board are r, r + R, r + 2R, ... and start at candidates
// 0, 1, 2, ... (k0 = (block / R) mod K).
#include <hip/hip_runtime.h>
#include <math.h>
#include "geak_internal.hpp"
#include "device_common.hpp"

namespace geak {
namespace {


// A value every lane holds alike (it came from a load all lanes made at one address), moved to scalar
// registers: what depends on it -- the threshold tests of every vector -- then runs on the scalar unit
// and as uniform branches instead of per-lane masks.
__device__ __forceinline__ u64 uniform64(u64 v)
{
    const u64 lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)v), hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return lo | (hi << 32);
}
__device__ __forceinline__ float uniform_f(float x)
{
    return __builtin_bit_cast(float, (uint32_t)__builtin_amdgcn_readfirstlane(__builtin_bit_cast(uint32_t, x)));
}
__device__ __forceinline__ double uniform_d(double x) { return __builtin_bit_cast(double, uniform64(__builtin_bit_cast(u64, x))); }
__device__ __forceinline__ float uniform_of(float x) { return uniform_f(x); }
__device__ __forceinline__ double uniform_of(double x) { return uniform_d(x); }

// ---- wave reductions (rare paths only) ---------------------------------------------------------
// Maximum over the wave, returned in every lane.  Data-parallel-primitive row shifts and the two
// row broadcasts of wave64 leave the maximum in lane 63 without going through LDS (a shuffle is an
// LDS-path instruction with a wait behind it: six of those per value made a trip of the maxima
// filters cost most of a microsecond).  Lanes that a shift gives no source keep their own value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float max_with_dpp(float x)
{
    const int self = __builtin_bit_cast(int, x);
    const float y = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(self, self, CTRL, ROW_MASK, 0xF, false));
    return (y > x) ? y : x;
}
__device__ __forceinline__ float wave_max_f(float x)
{
    x = max_with_dpp<0x111, 0xF>(x);          // row_shr:1
    x = max_with_dpp<0x112, 0xF>(x);          // row_shr:2
    x = max_with_dpp<0x114, 0xF>(x);          // row_shr:4
    x = max_with_dpp<0x118, 0xF>(x);          // row_shr:8: lane 15 of each row holds the row's maximum
    x = max_with_dpp<0x142, 0xA>(x);          // row_bcast:15 into rows 1 and 3
    x = max_with_dpp<0x143, 0xC>(x);          // row_bcast:31 into rows 2 and 3: lane 63 holds the wave's maximum
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}
__device__ __forceinline__ double wave_max_d(double x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double y = __shfl_xor(x, o, kWaveSize);
        x = (y > x) ? y : x;
    }
    return x;
}
__device__ __forceinline__ uint32_t wave_min_u(uint32_t x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t y = (uint32_t)__shfl_xor((int)x, o, kWaveSize);
        x = (y < x) ? y : x;
    }
    return x;
}

// Non-negative doubles order like their bit patterns, so the running maxima on the board are
// raised with an unsigned 64-bit atomic max.
__device__ __forceinline__ u64 load_bits(const double *p)
{
    // through the global address space: a flat load would also count against the LDS / scalar-load
    // counter, and the next wait for a scalar load would then wait for this one as well
    return __hip_atomic_load((const GEAK_AS_GLOBAL u64 *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_max(double *p, double v)
{
    (void)__hip_atomic_fetch_max((GEAK_AS_GLOBAL u64 *)p, __builtin_bit_cast(u64, v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The full rule for one floating element.
__device__ __forceinline__ bool close_exact(float a, float b, float atol_f, float rtol_f, int equal_nan)
{
    const bool a_nan = a != a, b_nan = b != b;
    if (a_nan || b_nan) return equal_nan && a_nan && b_nan;
    if (__builtin_fabsf(a) == kInfF || __builtin_fabsf(b) == kInfF) return a == b;
    const float d = __builtin_fabsf(a - b);
    const float prod = rtol_f * __builtin_fabsf(b);
    const float tol = atol_f + prod;
    return d <= tol;
}

__device__ __forceinline__ bool close_exact_d(double a, double b, double atol, double rtol, int equal_nan)
{
    const bool a_nan = a != a, b_nan = b != b;
    if (a_nan || b_nan) return equal_nan && a_nan && b_nan;
    if (__builtin_fabs(a) == kInfD || __builtin_fabs(b) == kInfD) return a == b;
    const double d = __builtin_fabs(a - b);
    const double prod = rtol * __builtin_fabs(b);
    const double tol = atol + prod;
    return d <= tol;
}

// max_rel filter.  An element can raise the running maximum r only if d/|b| > r, i.e. d > r*|b| in
// exact arithmetic.  e = fma(r, |b|, -d) is the correctly rounded value of r*|b| - d, and rounding
// keeps the sign of the exact value (a tiny negative value becomes -0, an exact tie becomes +0), so
// "e is negative, -0 included, and not NaN" is exactly the condition, at every magnitude, with no
// division and without flagging ties.  One v_fma_f32 and one v_cmp_class_f32.
//   NaN results (d NaN; Inf - Inf; 0 * Inf) mean "cannot raise" and are not flagged.
//   r = +Inf is handled by the caller (nothing exceeds it); b = 0 gives e = -d: flagged iff d > 0.
constexpr int kClassNegative = (1 << 2) | (1 << 3) | (1 << 4) | (1 << 5);   // -Inf, -normal, -subnormal, -0
__device__ __forceinline__ bool may_raise_rel(float r, float babs, float d)
{
    return __builtin_amdgcn_classf(__builtin_fmaf(r, babs, -d), kClassNegative);
}
// the same test in binary64 (v_fma_f64, v_cmp_class_f64)
__device__ __forceinline__ bool may_raise_rel_d(double r, double babs, double d)
{
    return __builtin_amdgcn_class(__builtin_fma(r, babs, -d), kClassNegative);
}

// int64 elements: |a - b| exact as an unsigned 64-bit integer and |b| (at most 2^63), each converted to
// binary64 with one rounding where a double is needed.
__device__ __forceinline__ double i64_abs_diff(long long a, long long x)
{
    const u64 d = (a >= x) ? ((u64)a - (u64)x) : ((u64)x - (u64)a);
    return (double)d;
}
__device__ __forceinline__ double i64_abs(long long x)
{
    const u64 m = (x < 0) ? (0ull - (u64)x) : (u64)x;
    return (double)m;
}

// ---- per-(wave, candidate) running state in LDS ----------------------------------------------
struct WaveState {
    uint32_t count_off;  // LDS byte offset of u64[K]: mismatching elements of the current (worker, segment) run
    uint32_t first_off;  // LDS byte offset of u32[K]: least item index of the run that holds a mismatch
    uint32_t tol_off;    // LDS byte offset of the wave's kTolBytesPerWave region for staged tolerances
};
// The state is addressed through the LDS address space (DS instructions), never through flat ones.
__device__ __forceinline__ GEAK_AS_LDS u64 *state_count(const WaveState &st) { return (GEAK_AS_LDS u64 *)st.count_off; }
__device__ __forceinline__ GEAK_AS_LDS uint32_t *state_first(const WaveState &st) { return (GEAK_AS_LDS uint32_t *)st.first_off; }

__device__ __forceinline__ void note_mismatches(const WaveState &st, uint32_t k, uint32_t n, uint32_t item, int lane)
{
    if (n && lane == 0) {
        (void)__hip_atomic_fetch_add(state_count(st) + k, (u64)n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        (void)__hip_atomic_fetch_min(state_first(st) + k, item, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
}

// A (worker, segment) run begins: clear the wave's running state.  It ends: write it to the run's slot.
__device__ __forceinline__ void begin_run(const WaveState &st, uint32_t K, int lane)
{
    for (uint32_t k = lane; k < K; k += kWaveSize) { state_count(st)[k] = 0; state_first(st)[k] = kNoItem; }
}
__device__ __forceinline__ void end_run(const WaveState &st, Partial *partials, uint32_t slot, uint32_t K, int lane)
{
    // one 16-byte record per candidate, written as a vector through the global address space
    static_assert(sizeof(Partial) == 16, "Partial is one 16-byte vector");
    GEAK_AS_GLOBAL u32x4 *out = (GEAK_AS_GLOBAL u32x4 *)partials + (u64)slot * K;
    for (uint32_t k = lane; k < K; k += kWaveSize) {
        const u64 count = state_count(st)[k];
        u32x4 r;
        r[0] = (uint32_t)count;
        r[1] = (uint32_t)(count >> 32);
        r[2] = state_first(st)[k];
        r[3] = 0;
        out[k] = r;
    }
}

// ---- full items, floating dtypes: reference slice staged in registers ---------------------------
// Lane mask of "x is negative (-0 included) and not NaN".  Written as the instruction itself: a
// ballot of the class builtin is materialised through a vector register and compared again.
__device__ __forceinline__ u64 negative_mask(float x)
{
    u64 m;
    asm("v_cmp_class_f32_e64 %0, %1, 60" : "=s"(m) : "v"(x));      // 60 = kClassNegative
    return m;
}

// binary16 operands are consumed straight from the packed registers by the mixed-precision FMA
// (f16 sources, f32 arithmetic, one rounding): a*1 - b is RN(a - b), the same value as converting
// both and subtracting, in one instruction instead of three.
template <bool HI>
__device__ __forceinline__ float f16_diff(uint32_t a2, uint32_t b2)
{
    float d;
    if constexpr (HI) asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,1] op_sel_hi:[1,0,1]" : "=v"(d) : "v"(a2), "v"(b2));
    else              asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,0] op_sel_hi:[1,0,1]" : "=v"(d) : "v"(a2), "v"(b2));
    return d;
}
// r*|b| - |d| with b a binary16 half of b2
template <bool HI>
__device__ __forceinline__ float f16_rel_margin(float r, uint32_t b2, float d)
{
    float e;
    if constexpr (HI) asm("v_fma_mix_f32 %0, %1, |%2|, -|%3| op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "=v"(e) : "v"(r), "v"(b2), "v"(d));
    else              asm("v_fma_mix_f32 %0, %1, |%2|, -|%3| op_sel:[0,0,0] op_sel_hi:[0,1,0]" : "=v"(e) : "v"(r), "v"(b2), "v"(d));
    return e;
}

// RN(r * |b|) with b a binary16 half of b2 (the added +0 changes nothing: the product is never -0)
template <bool HI>
__device__ __forceinline__ float f16_abs_scaled(float r, uint32_t b2)
{
    float e;
    if constexpr (HI) asm("v_fma_mix_f32 %0, %1, |%2|, 0 op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "=v"(e) : "v"(r), "v"(b2));
    else              asm("v_fma_mix_f32 %0, %1, |%2|, 0 op_sel:[0,0,0] op_sel_hi:[0,1,0]" : "=v"(e) : "v"(r), "v"(b2));
    return e;
}


// Arguments of a device function arrive in vector registers; everything here is the same for all
// lanes, so it is moved back to scalar registers once.
__device__ __forceinline__ uint32_t uniform32(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
template <typename T>
__device__ __forceinline__ T *uniform_ptr(T *p)
{
    const u64 v = reinterpret_cast<u64>(p);
    const u64 lo = uniform32((uint32_t)v), hi = uniform32((uint32_t)(v >> 32));
    return reinterpret_cast<T *>(lo | (hi << 32));
}
// One vector's worth of reference values / tolerances, decoded, as passed to the out-of-line
// versions of the rare paths (used where code size matters more than the call).
template <int DT> struct RefVec { float b[Traits<DT>::E]; };
template <int DT> struct TolVec { float t[Traits<DT>::E]; };
struct FloatPair { float abs, rel; };
struct DoublePair { double abs, rel; };
template <int DT>
__device__ uint32_t false_suspects_vector(const u32x4 q, const RefVec<DT> ref, const TolVec<DT> tol, const uint32_t slot_mask_in,
                                          const int equal_nan_in);
template <int DT>
__device__ FloatPair raise_vector(const u32x4 q, const RefVec<DT> ref, const float max_abs, const float max_rel, MaxPair *rec_in);
template <int DT>
__device__ __noinline__ DoublePair raise_vector_integer(const u32x4 q, const u32x4 b, const double max_abs, const double max_rel, MaxPair *rec_in);
template <typename T, typename Pair>
__device__ __forceinline__ Pair close_raise(T dm, T rm, const T max_abs, const T max_rel, MaxPair *rec);

// Tolerances of the staged reference slice, one per element the lane holds.  The 32-bit dtypes
// keep them in registers.  The 16-bit dtypes hold twice the elements per slice; their 32
// tolerances per lane live in the wave's own LDS region instead (the registers go to the loads in
// flight), laid out in chunks of four so that chunk c of lane L sits at c * 1024 + L * 16: every
// 16-byte access of the wave covers one contiguous KiB, free of bank conflicts.  A wave only ever
// reads what it wrote itself, and its DS operations execute in order, so no barrier is involved.
template <int E, bool IN_LDS> struct TolStore;
template <int E> struct TolStore<E, false> {
    float t[kVecPerLane * E];
    __device__ __forceinline__ void attach(uint32_t, int) {}
    template <int V> __device__ __forceinline__ void put(const float (&v)[E])
    {
#pragma unroll
        for (int e = 0; e < E; ++e) t[V * E + e] = v[e];
    }
    template <int V> __device__ __forceinline__ void get(float (&v)[E]) const
    {
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = t[V * E + e];
    }
    template <int I> __device__ __forceinline__ float one() const { return t[I]; }
};
template <int E> struct TolStore<E, true> {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    uint32_t base;                   // LDS byte offset of the lane's chunk 0
    __device__ __forceinline__ void attach(uint32_t region, int lane) { base = region + (uint32_t)lane * 16u; }
    template <int V> __device__ __forceinline__ void put(const float (&v)[E])
    {
#pragma unroll
        for (int c = 0; c < E / 4; ++c) {
            f32x4 x = {v[4 * c], v[4 * c + 1], v[4 * c + 2], v[4 * c + 3]};
            *(GEAK_AS_LDS f32x4 *)(base + (uint32_t)(V * (E / 4) + c) * 1024u) = x;
        }
    }
    template <int V> __device__ __forceinline__ void get(float (&v)[E]) const
    {
#pragma unroll
        for (int c = 0; c < E / 4; ++c) {
            const f32x4 x = *(const GEAK_AS_LDS f32x4 *)(base + (uint32_t)(V * (E / 4) + c) * 1024u);
            v[4 * c] = x[0]; v[4 * c + 1] = x[1]; v[4 * c + 2] = x[2]; v[4 * c + 3] = x[3];
        }
    }
    template <int I> __device__ __forceinline__ float one() const
    {
        return *(const GEAK_AS_LDS float *)(base + (uint32_t)(I / 4) * 1024u + (uint32_t)(I % 4) * 4u);
    }
};

template <int DT>
struct FloatItem {
    typedef float Hint;                 // the running maxima of floating segments are binary32 values
    static __device__ __forceinline__ float hint_from_bits(u64 bits) { return uniform_f((float)__builtin_bit_cast(double, bits)); }
    static constexpr int E = Traits<DT>::E;
    static constexpr int N = kVecPerLane * E;
    // Reference storage: binary32 and binary16 keep the vectors as loaded (binary32 needs no decode,
    // binary16 is read in place by the mixed-precision FMA); bfloat16 is unpacked once, because
    // unpacking it again for every candidate would cost an instruction per element.
    static constexpr int kRefRegs = (DT == GEAK_BF16) ? N : kVecPerLane * 4;
    uint32_t bref[kRefRegs];
    static constexpr bool kTolInLds = (E == 8);
    static constexpr bool kRaiseOutOfLine = false;
    TolStore<E, kTolInLds> tol;
    float tol_ahead[kTolInLds ? E : 1];     // the next vector's tolerances, on their way from LDS
    uint32_t poisoned_slots;        // wave-uniform: bit i set if any lane's element i is poisoned

    __device__ __forceinline__ void attach_lds(uint32_t region, int lane) { tol.attach(region, lane); }

    // Stage vector V of the reference slice: keep it (packed or unpacked, see above), compute the
    // tolerance of each of its elements once, and poison the elements the bare inequality cannot judge.
    template <int V>
    __device__ __forceinline__ void stage_vec(const u32x4 &q, const SegTol &tolerance)
    {
        const float atol_f = tolerance.atol_f, rtol_f = tolerance.rtol_f;
        if constexpr (V == 0) poisoned_slots = 0;
        if constexpr (DT != GEAK_BF16) {
#pragma unroll
            for (int w = 0; w < 4; ++w) bref[V * 4 + w] = q[w];
        }
        float tv[E];
        static_for<E>([&](auto idx) {
            constexpr int e = decltype(idx)::value;
            constexpr int i = V * E + e;
            float prod;
            if constexpr (DT == GEAK_F16) {
                prod = f16_abs_scaled<(e & 1) != 0>(rtol_f, q[e >> 1]);
            } else {
                const float x = decode<DT>(q, e);
                if constexpr (DT == GEAK_BF16) bref[i] = f_bits(x);
                prod = rtol_f * __builtin_fabsf(x);
            }
            const float t = atol_f + prod;
            tv[e] = t;
            // b NaN, b +-Inf, or the tolerance overflowed: rare, so the poison value is only worked
            // out under a wave-uniform branch.  It also records why: -1 b is NaN, -2 b is +-Inf,
            // -3 finite b with an infinite tolerance.
            const bool bad = !(t < kInfF);
            if (__builtin_amdgcn_ballot_w64(bad)) {
                const float x = decode<DT>(q, e);
                const float why = (x != x) ? -1.0f : (__builtin_fabsf(x) == kInfF ? -2.0f : -3.0f);
                tv[e] = bad ? why : t;
                poisoned_slots |= (1u << i);
            }
        });
        tol.template put<V>(tv);
        if constexpr (kTolInLds && V == kVecPerLane - 1) tol.template get<0>(tol_ahead);    // for the first candidate's vector 0
    }

    // reference element i = V*E + e as binary32 (rare paths)
    template <int V, int e>
    __device__ __forceinline__ float ref_value() const
    {
        if constexpr (DT == GEAK_F32) return bits_f(bref[V * 4 + e]);
        else if constexpr (DT == GEAK_BF16) return bits_f(bref[V * E + e]);
        else {
            const uint32_t word = bref[V * 4 + (e >> 1)];
            const uint16_t h = (e & 1) ? (uint16_t)(word >> 16) : (uint16_t)(word & 0xFFFFu);
            return (float)__builtin_bit_cast(_Float16, h);
        }
    }

    // a - b for element e of vector V, and r*|b| - |a - b|
    template <int V, int e>
    __device__ __forceinline__ float diff(const u32x4 &q) const
    {
        if constexpr (DT == GEAK_F16) return f16_diff<(e & 1) != 0>(q[e >> 1], bref[V * 4 + (e >> 1)]);
        else return decode<DT>(q, e) - ref_value<V, e>();
    }
    template <int V, int e>
    __device__ __forceinline__ float rel_margin(float r, float d) const
    {
        if constexpr (DT == GEAK_F16) return f16_rel_margin<(e & 1) != 0>(r, bref[V * 4 + (e >> 1)], d);
        else return __builtin_fmaf(r, __builtin_fabsf(ref_value<V, e>()), -__builtin_fabsf(d));
    }

    // Hot loop body for one 16-byte vector of one candidate.  Adds the suspects (elements with
    // !(d <= tol)) to `suspects` and ORs into `trip_abs` / `trip_rel` the lanes that may raise
    // max_abs_err / max_rel_err.  Four vector instructions per element (five for bfloat16).
    template <int V, bool AHEAD = true>
    __device__ __forceinline__ void compare_vec(const u32x4 &q, float max_abs, float max_rel, uint32_t &suspects,
                                                u64 &trip_abs, u64 &trip_rel, int equal_nan)
    {
        // tolerances of this vector; in the streaming routine (AHEAD: vectors 0, 1, 2, 3, 0, ... in
        // turn) those kept in LDS were fetched one vector ahead, and the next vector's are fetched
        // now, behind this vector's arithmetic
        float tv[E];
        if constexpr (kTolInLds && AHEAD) {
#pragma unroll
            for (int e = 0; e < E; ++e) tv[e] = tol_ahead[e];
            tol.template get<(V + 1) % kVecPerLane>(tol_ahead);
        } else {
            tol.template get<V>(tv);
        }
        // The two "may raise a maximum" tests are folded over the vector: a running greatest |d| and a
        // running least margin r|b| - |d| (three-operand max / min, which skip NaN as the comparisons
        // they stand for do), each tested once.
        float d_most = 0.0f, margin_least = kInfF;
        static_for<E / 2>([&](auto idx) {
            constexpr int e = 2 * decltype(idx)::value;
            const float d0 = diff<V, e>(q), d1 = diff<V, e + 1>(q);
            suspects += __builtin_popcountll(__builtin_amdgcn_ballot_w64(!(__builtin_fabsf(d0) <= tv[e])));
            suspects += __builtin_popcountll(__builtin_amdgcn_ballot_w64(!(__builtin_fabsf(d1) <= tv[e + 1])));
            d_most = __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(d0), __builtin_fabsf(d1)), d_most);
            margin_least = __builtin_fminf(__builtin_fminf(rel_margin<V, e>(max_rel, d0), rel_margin<V, e + 1>(max_rel, d1)), margin_least);
        });
        trip_abs |= __builtin_amdgcn_ballot_w64(d_most > max_abs);
        trip_rel |= negative_mask(margin_least);
        // Poisoned elements were all reported as suspects; take off those that the NaN / Inf rule
        // accepts.  In the streaming routine this happens here, while the vector's tolerances (which
        // say why an element is poisoned) are at hand.
        if constexpr (AHEAD) {
            constexpr uint32_t kVecMask = ((E == 8) ? 0xFFu : 0xFu) << (V * E);
            if (poisoned_slots & kVecMask) suspects -= false_suspects_vec<V>(q, tv, equal_nan);
        }
    }

    // Number of poisoned elements of vector V that the NaN / Inf rule accepts; tv: the vector's tolerances.
    template <int V>
    __device__ __forceinline__ uint32_t false_suspects_vec(const u32x4 &q, const float (&tv)[E], int equal_nan) const
    {
        uint32_t n = 0;
        static_for<E>([&](auto idx) {
            constexpr int e = decltype(idx)::value;
            constexpr int i = V * E + e;
            if (poisoned_slots & (1u << i)) {
                const float a = decode<DT>(q, e);
                const float x = ref_value<V, e>();
                float why = tv[e];
                asm volatile("" : "+v"(why));   // evaluate here, per candidate: hoisted lane masks would not fit the scalar file
                const bool ok = (why == -1.0f) ? (equal_nan && (a != a))
                              : (why == -2.0f) ? (a == x)
                              : (why == -3.0f) ? (__builtin_fabsf(a) < kInfF)   // any finite a is within an infinite tolerance
                              : false;
                n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(ok));
            }
        });
        return n;
    }

    // A lane of vector V may raise one of the maxima: evaluate the vector exactly, in registers, and
    // publish at once, so that the other waves (and this wave's next vectors) see the new thresholds.
    // Per lane the running maxima start from the wave-uniform ones, so the true division only runs
    // for elements that really exceed what the lane has seen.
    template <int V>
    __device__ __forceinline__ void raise_vec(const u32x4 &q, float &max_abs, float &max_rel, MaxPair *rec, int lane) const
    {
        float dm = max_abs, rm = max_rel;
        static_for<E>([&](auto idx) {
            constexpr int e = decltype(idx)::value;
            const float x = ref_value<V, e>();
            const float d = __builtin_fabsf(decode<DT>(q, e) - x);
            const float babs = __builtin_fabsf(x);
            dm = (d > dm) ? d : dm;                                          // false for NaN: skipped
            const bool hit = (rm < kInfF) && may_raise_rel(rm, babs, d);     // implies d > 0
            if (__builtin_amdgcn_ballot_w64(hit)) {
                const float r = d / babs;                                    // correctly rounded; d/0 = +Inf
                rm = (hit && r > rm) ? r : rm;
            }
        });
        dm = wave_max_f(dm);
        rm = wave_max_f(rm);
        if (lane == 0) {
            if (dm > max_abs) publish_max(&rec->abs, (double)dm);
            if (rm > max_rel) publish_max(&rec->rel, (double)rm);
        }
        max_abs = uniform_of(dm);           // all lanes hold the wave's maximum: back to scalar registers
        max_rel = uniform_of(rm);
    }

    // the same two rare paths through real functions (by-value arguments)
    template <int V>
    __device__ __forceinline__ uint32_t false_suspects_call(const u32x4 &q, int equal_nan) const
    {
        RefVec<DT> r;
        TolVec<DT> t;
        static_for<E>([&](auto idx) { constexpr int e = decltype(idx)::value; r.b[e] = ref_value<V, e>(); t.t[e] = tol.template one<V * E + e>(); });
        return false_suspects_vector<DT>(q, r, t, (poisoned_slots >> (V * E)) & ((1u << E) - 1u), equal_nan);
    }
    template <int V>
    __device__ __forceinline__ void raise_call(const u32x4 &q, float &max_abs, float &max_rel, MaxPair *rec) const
    {
        RefVec<DT> r;
        static_for<E>([&](auto idx) { constexpr int e = decltype(idx)::value; r.b[e] = ref_value<V, e>(); });
        const FloatPair out = raise_vector<DT>(q, r, max_abs, max_rel, rec);
        max_abs = uniform_of(out.abs);      // the callee returns the wave's maxima in every lane
        max_rel = uniform_of(out.rel);
    }
};

template <int DT>
__device__ __noinline__ uint32_t false_suspects_vector(const u32x4 q, const RefVec<DT> ref, const TolVec<DT> tol,
                                                       const uint32_t slot_mask_in, const int equal_nan_in)
{
    constexpr int E = Traits<DT>::E;
    const uint32_t slot_mask = uniform32(slot_mask_in);
    const int equal_nan = (int)uniform32((uint32_t)equal_nan_in);
    uint32_t n = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        if (slot_mask & (1u << e)) {
            const float a = decode<DT>(q, e);
            const float x = ref.b[e];
            const float why = tol.t[e];     // -1 b is NaN, -2 b is +-Inf, -3 finite b with tolerance +Inf, else not poisoned
            const bool ok = (why == -1.0f) ? (equal_nan && (a != a))
                          : (why == -2.0f) ? (a == x)
                          : (why == -3.0f) ? (__builtin_fabsf(a) < kInfF)
                          : false;
            n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(ok));
        }
    }
    return n;
}

template <int DT>
__device__ __noinline__ FloatPair raise_vector(const u32x4 q, const RefVec<DT> ref, const float max_abs, const float max_rel,
                                               MaxPair *rec_in)
{
    constexpr int E = Traits<DT>::E;
    MaxPair *rec = uniform_ptr(rec_in);
    float dm = max_abs, rm = max_rel;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const float x = ref.b[e];
        const float d = __builtin_fabsf(decode<DT>(q, e) - x);
        const float babs = __builtin_fabsf(x);
        dm = (d > dm) ? d : dm;                                          // false for NaN: skipped
        const bool hit = (rm < kInfF) && may_raise_rel(rm, babs, d);     // implies d > 0
        if (__builtin_amdgcn_ballot_w64(hit)) {
            const float r = d / babs;                                    // correctly rounded; d/0 = +Inf
            rm = (hit && r > rm) ? r : rm;
        }
    }
    return close_raise<float, FloatPair>(dm, rm, max_abs, max_rel, rec);
}

// ---- int32: same interface, exact equality ---------------------------------------------------------
struct IntItem {
    typedef double Hint;                // |a - b| reaches 2^32 - 1 and the quotient is binary64
    static __device__ __forceinline__ double hint_from_bits(u64 bits) { return __builtin_bit_cast(double, uniform64(bits)); }
    static constexpr int E = 4;
    // the exact evaluation is binary64 arithmetic with a division: inlined into the stream it costs
    // the loop its registers, so it is always called
    static constexpr bool kRaiseOutOfLine = true;
    uint32_t bref[kVecPerLane * 4];
    __device__ __forceinline__ void attach_lds(uint32_t, int) {}
    [[maybe_unused]] static constexpr uint32_t poisoned_slots = 0;

    template <int V>
    __device__ __forceinline__ void stage_vec(const u32x4 &q, const SegTol &)
    {
#pragma unroll
        for (int w = 0; w < 4; ++w) bref[V * 4 + w] = q[w];
    }
    // Any unequal element is a mismatch and the only kind of element that can raise a maximum.
    template <int V, bool AHEAD = true>
    __device__ __forceinline__ void compare_vec(const u32x4 &q, double, double, uint32_t &suspects, u64 &trip_abs, u64 &, int) const
    {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const u64 m = __builtin_amdgcn_ballot_w64(q[e] != bref[V * 4 + e]);
            suspects += __builtin_popcountll(m);
            trip_abs |= m;
        }
    }
    template <int V>
    __device__ __forceinline__ uint32_t false_suspects_call(const u32x4 &, int) const { return 0; }
    template <int V>
    __device__ __forceinline__ void raise_call(const u32x4 &q, double &max_abs, double &max_rel, MaxPair *rec) const
    {
        u32x4 b;
#pragma unroll
        for (int w = 0; w < 4; ++w) b[w] = bref[V * 4 + w];
        const DoublePair out = raise_vector_integer<GEAK_I32>(q, b, max_abs, max_rel, rec);
        max_abs = uniform_of(out.abs);      // the callee returns the wave's maxima in every lane
        max_rel = uniform_of(out.rel);
    }

    template <int V>
    __device__ __forceinline__ void raise_vec(const u32x4 &q, double &max_abs, double &max_rel, MaxPair *rec, int lane) const
    {
        double dm = max_abs, rm = max_rel;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const long long a = (int)q[e], x = (int)bref[V * 4 + e];
            const long long diff = a - x;
            const double d = (double)(diff < 0 ? -diff : diff);          // exact
            const double babs = (double)(x < 0 ? -x : x);
            dm = (d > dm) ? d : dm;
            // d/|b| > rm implies d > rm*|b|*(1 - 2^-30); the margin covers the product's rounding
            if (d > 0.0 && (rm < (double)kInfF) && d > rm * (1.0 - 0x1p-30) * babs) {
                const double r = d / babs;                               // binary64, correctly rounded; d/0 = +Inf
                rm = (r > rm) ? r : rm;
            }
        }
        dm = wave_max_d(dm);
        rm = wave_max_d(rm);
        if (lane == 0) {
            if (dm > max_abs) publish_max(&rec->abs, dm);
            if (rm > max_rel) publish_max(&rec->rel, rm);
        }
        max_abs = uniform_of(dm);           // all lanes hold the wave's maximum: back to scalar registers
        max_rel = uniform_of(rm);
    }
};

// Element e of a 16-byte vector of an integer dtype, widened exactly.
template <int DT>
__device__ __forceinline__ long long integer_element(const u32x4 &v, int e)
{
    if constexpr (DT == GEAK_I32) return (int)v[e];
    else if constexpr (DT == GEAK_I64) return (long long)((u64)v[2 * e] | ((u64)v[2 * e + 1] << 32));
    else {
        const uint32_t byte = (v[e >> 2] >> (8 * (e & 3))) & 0xFFu;
        return DT == GEAK_I8 ? (long long)(signed char)byte : (long long)byte;
    }
}
// What closes every raise routine: the wave's maxima, published by one lane where they grew, returned in every lane.
template <typename T, typename Pair>
__device__ __forceinline__ Pair close_raise(T dm, T rm, const T max_abs, const T max_rel, MaxPair *rec)
{
    if constexpr (sizeof(T) == 8) { dm = wave_max_d(dm); rm = wave_max_d(rm); }
    else { dm = wave_max_f(dm); rm = wave_max_f(rm); }
    if ((threadIdx.x & (kWaveSize - 1)) == 0) {
        if (dm > max_abs) publish_max(&rec->abs, (double)dm);
        if (rm > max_rel) publish_max(&rec->rel, (double)rm);
    }
    Pair out;
    out.abs = dm;
    out.rel = rm;
    return out;
}
// The rare path of the integer dtypes (int32, int64, uint8, int8), one routine: the exact |a - b| and
// |a - b| / |b| of a vector in which some lane saw a difference, folded into the running maxima.
template <int DT>
__device__ __noinline__ DoublePair raise_vector_integer(const u32x4 q, const u32x4 b, const double max_abs, const double max_rel,
                                                        MaxPair *rec_in)
{
    MaxPair *rec = uniform_ptr(rec_in);
    double dm = max_abs, rm = max_rel;
    constexpr int E = Traits<DT>::E, kPerWord = E / 4 > 0 ? E / 4 : 1;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        if constexpr (kPerWord > 1) {
            if (q[e / kPerWord] == b[e / kPerWord]) continue;            // bytes: most words of a tripping lane are equal
        }
        const long long a = integer_element<DT>(q, e), x = integer_element<DT>(b, e);
        double d, babs;
        if constexpr (DT == GEAK_I64) {
            d = i64_abs_diff(a, x);                                      // the difference may leave 64 bits: one rounding
            babs = i64_abs(x);
        } else {
            const long long diff = a - x;                                // narrower elements: exact in 64 bits
            d = (double)(diff < 0 ? -diff : diff);
            babs = (double)(x < 0 ? -x : x);
        }
        dm = (d > dm) ? d : dm;
        // d/|b| > rm implies d > rm*|b|*(1 - 2^-30); the margin covers the product's rounding
        if (d > 0.0 && (rm < (double)kInfF) && d > rm * (1.0 - 0x1p-30) * babs) {
            const double r = d / babs;                                   // binary64, correctly rounded; d/0 = +Inf
            rm = (r > rm) ? r : rm;
        }
    }
    return close_raise<double, DoublePair>(dm, rm, max_abs, max_rel, rec);
}

// ---- int64: two elements per 16-byte vector, exact equality ------------------------------------------
struct Int64Item {
    typedef double Hint;
    static __device__ __forceinline__ double hint_from_bits(u64 bits) { return __builtin_bit_cast(double, uniform64(bits)); }
    static constexpr int E = 2;
    static constexpr bool kRaiseOutOfLine = true;
    uint32_t bref[kVecPerLane * 4];
    __device__ __forceinline__ void attach_lds(uint32_t, int) {}
    [[maybe_unused]] static constexpr uint32_t poisoned_slots = 0;

    template <int V>
    __device__ __forceinline__ void stage_vec(const u32x4 &q, const SegTol &)
    {
#pragma unroll
        for (int w = 0; w < 4; ++w) bref[V * 4 + w] = q[w];
    }
    // Any unequal element is a mismatch and the only kind of element that can raise a maximum.
    template <int V, bool AHEAD = true>
    __device__ __forceinline__ void compare_vec(const u32x4 &q, double, double, uint32_t &suspects, u64 &trip_abs, u64 &, int) const
    {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const uint32_t differ = (q[2 * e] ^ bref[V * 4 + 2 * e]) | (q[2 * e + 1] ^ bref[V * 4 + 2 * e + 1]);
            const u64 m = __builtin_amdgcn_ballot_w64(differ != 0);
            suspects += __builtin_popcountll(m);
            trip_abs |= m;
        }
    }
    template <int V>
    __device__ __forceinline__ uint32_t false_suspects_call(const u32x4 &, int) const { return 0; }
    template <int V>
    __device__ __forceinline__ void raise_call(const u32x4 &q, double &max_abs, double &max_rel, MaxPair *rec) const
    {
        u32x4 b;
#pragma unroll
        for (int w = 0; w < 4; ++w) b[w] = bref[V * 4 + w];
        const DoublePair out = raise_vector_integer<GEAK_I64>(q, b, max_abs, max_rel, rec);
        max_abs = uniform_of(out.abs);      // the callee returns the wave's maxima in every lane
        max_rel = uniform_of(out.rel);
    }
    template <int V>
    __device__ __forceinline__ void raise_vec(const u32x4 &q, double &max_abs, double &max_rel, MaxPair *rec, int) const
    {
        raise_call<V>(q, max_abs, max_rel, rec);
    }
};

// ---- binary64: two elements per 16-byte vector, the floating rule in binary64 arithmetic -----------
// Lane mask of "x is negative (-0 included) and not NaN", binary64.
__device__ __forceinline__ u64 negative_mask_d(double x)
{
    u64 m;
    asm("v_cmp_class_f64_e64 %0, %1, 60" : "=s"(m) : "v"(x));      // 60 = kClassNegative
    return m;
}

__device__ __noinline__ DoublePair raise_vector_f64(const u32x4 q, const u32x4 b, const double max_abs, const double max_rel,
                                                    MaxPair *rec_in)
{
    MaxPair *rec = uniform_ptr(rec_in);
    double dm = max_abs, rm = max_rel;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const double x = bits_d(b[2 * e], b[2 * e + 1]);
        const double d = __builtin_fabs(bits_d(q[2 * e], q[2 * e + 1]) - x);
        const double babs = __builtin_fabs(x);
        dm = (d > dm) ? d : dm;                                          // false for NaN: skipped
        const bool hit = (rm < kInfD) && may_raise_rel_d(rm, babs, d);   // implies d > 0
        if (__builtin_amdgcn_ballot_w64(hit)) {
            const double r = d / babs;                                   // correctly rounded; d/0 = +Inf
            rm = (hit && r > rm) ? r : rm;
        }
    }
    return close_raise<double, DoublePair>(dm, rm, max_abs, max_rel, rec);
}

struct DoubleItem {
    typedef double Hint;
    static __device__ __forceinline__ double hint_from_bits(u64 bits) { return __builtin_bit_cast(double, uniform64(bits)); }
    static constexpr int E = 2;
    static constexpr bool kRaiseOutOfLine = true;    // binary64 division: kept out of the stream, like the integer items'
    uint32_t bref[kVecPerLane * 4];
    double tol[kVecPerLane * E];
    uint32_t poisoned_slots;        // wave-uniform: bit i set if any lane's element i is poisoned
    __device__ __forceinline__ void attach_lds(uint32_t, int) {}

    template <int V, int e>
    __device__ __forceinline__ double ref_value() const { return bits_d(bref[V * 4 + 2 * e], bref[V * 4 + 2 * e + 1]); }

    // Stage vector V of the reference slice: the tolerance of each element, computed once with two
    // roundings, or a poison value where the bare inequality cannot judge (-1 b is NaN, -2 b is
    // +-Inf, -3 finite b with an infinite tolerance).
    template <int V>
    __device__ __forceinline__ void stage_vec(const u32x4 &q, const SegTol &tolerance)
    {
        if constexpr (V == 0) poisoned_slots = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) bref[V * 4 + w] = q[w];
        static_for<E>([&](auto idx) {
            constexpr int e = decltype(idx)::value;
            constexpr int i = V * E + e;
            const double x = bits_d(q[2 * e], q[2 * e + 1]);
            const double prod = tolerance.rtol * __builtin_fabs(x);
            const double t = tolerance.atol + prod;
            tol[i] = t;
            const bool bad = !(t < kInfD);
            if (__builtin_amdgcn_ballot_w64(bad)) {
                const double why = (x != x) ? -1.0 : (__builtin_fabs(x) == kInfD ? -2.0 : -3.0);
                tol[i] = bad ? why : t;
                poisoned_slots |= (1u << i);
            }
        });
    }

    // Hot loop body for one 16-byte vector of one candidate: suspects (elements with !(d <= tol)) and
    // the lanes that may raise one of the maxima.  Five binary64 instructions per element.
    template <int V, bool AHEAD = true>
    __device__ __forceinline__ void compare_vec(const u32x4 &q, double max_abs, double max_rel, uint32_t &suspects,
                                                u64 &trip_abs, u64 &trip_rel, int equal_nan) const
    {
        static_for<E>([&](auto idx) {
            constexpr int e = decltype(idx)::value;
            const double x = ref_value<V, e>();
            const double d = bits_d(q[2 * e], q[2 * e + 1]) - x;
            suspects += __builtin_popcountll(__builtin_amdgcn_ballot_w64(!(__builtin_fabs(d) <= tol[V * E + e])));
            trip_abs |= __builtin_amdgcn_ballot_w64(__builtin_fabs(d) > max_abs);
            trip_rel |= negative_mask_d(__builtin_fma(max_rel, __builtin_fabs(x), -__builtin_fabs(d)));
        });
        // poisoned elements were all reported as suspects; take off those that the NaN / Inf rule accepts
        if constexpr (AHEAD) {
            constexpr uint32_t kVecMask = ((1u << E) - 1u) << (V * E);
            if (poisoned_slots & kVecMask) suspects -= false_suspects_call<V>(q, equal_nan);
        }
    }

    // Number of poisoned elements of vector V that the NaN / Inf rule accepts.
    template <int V>
    __device__ __forceinline__ uint32_t false_suspects_call(const u32x4 &q, int equal_nan) const
    {
        uint32_t n = 0;
        static_for<E>([&](auto idx) {
            constexpr int e = decltype(idx)::value;
            constexpr int i = V * E + e;
            if (poisoned_slots & (1u << i)) {
                const double a = bits_d(q[2 * e], q[2 * e + 1]);
                const double x = ref_value<V, e>();
                const double why = tol[i];
                const bool ok = (why == -1.0) ? (equal_nan && (a != a))
                              : (why == -2.0) ? (a == x)
                              : (why == -3.0) ? (__builtin_fabs(a) < kInfD)   // any finite a is within an infinite tolerance
                              : false;
                n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(ok));
            }
        });
        return n;
    }

    template <int V>
    __device__ __forceinline__ void raise_call(const u32x4 &q, double &max_abs, double &max_rel, MaxPair *rec) const
    {
        u32x4 b;
#pragma unroll
        for (int w = 0; w < 4; ++w) b[w] = bref[V * 4 + w];
        const DoublePair out = raise_vector_f64(q, b, max_abs, max_rel, rec);
        max_abs = uniform_of(out.abs);      // the callee returns the wave's maxima in every lane
        max_rel = uniform_of(out.rel);
    }
    template <int V>
    __device__ __forceinline__ void raise_vec(const u32x4 &q, double &max_abs, double &max_rel, MaxPair *rec, int) const
    {
        raise_call<V>(q, max_abs, max_rel, rec);
    }
};

// ---- 8-bit floating formats: sixteen elements per 16-byte vector, the binary32 rule ----------------------
// A lane holds 64 elements of the slice: the decoded reference does not fit the registers, and of its
// tolerances only half fit the wave's LDS region (four blocks per compute unit share the LDS).  The
// reference stays packed and is widened again for every candidate (one conversion per two
// elements); the tolerances of vectors 0 and 1 are staged in LDS, those of vectors 2 and 3 computed
// again (one multiplication, one addition): five and seven vector instructions per element,
// against four for the wider dtypes, and a budget of 4.9 per byte at the memory's speed -- this
// path is bound by arithmetic.  Elements the bare inequality cannot judge (b NaN, b +-Inf, tolerance
// overflowed) are only marked when the slice is staged; vectors that hold one are counted again
// with the full rule.
// The block-scaled element formats (payload byte plus the scale of the vector's block) take the same path:
// wherever an element is widened it is multiplied by its vector's scale, `sa` for the candidate's and `sb` for
// the reference's vector (both 1 and not applied for the plain 8-bit formats).
template <int DT>
__device__ FloatPair raise_vector_f8(const u32x4 q, const u32x4 b, const float max_abs, const float max_rel, MaxPair *rec_in,
                                     const float sa, const float sb);
template <int DT>
__device__ int recount_vector_f8(const u32x4 q, const u32x4 b, const uint32_t marked_in, const float atol_in, const float rtol_in,
                                 const int equal_nan_in, const float sa, const float sb);
template <int DT, int BYTE>
__device__ __forceinline__ float f8_value(uint32_t word, [[maybe_unused]] float scale)
{
    if constexpr (kScaled<DT>) return f8_to_f32<DT, BYTE>(word) * scale;
    else return f8_to_f32<DT, BYTE>(word);
}

template <int DT>
struct Fp8Item {
    typedef float Hint;
    static __device__ __forceinline__ float hint_from_bits(u64 bits) { return uniform_f((float)__builtin_bit_cast(double, bits)); }
    static constexpr int E = 16;
    static constexpr bool kRaiseOutOfLine = true;
    uint32_t bref[kVecPerLane * 4];
    float atol_f, rtol_f;           // wave-uniform
    u64 poisoned_slots;             // wave-uniform: bit i set if any lane's element i is poisoned
    // block-scaled formats only: the scales of the reference's four vectors, and of the candidate's vector that is
    // compared next (set by the caller before each vector)
    float sb[kVecPerLane];
    float sa;
    template <int V> __device__ __forceinline__ void stage_scale(uint32_t byte) { sb[V] = scale_of_byte<DT>(byte); }
    __device__ __forceinline__ void candidate_scale(uint32_t byte) { sa = scale_of_byte<DT>(byte); }
    template <int V> __device__ __forceinline__ float ref_scale() const
    {
        if constexpr (kScaled<DT>) return sb[V];
        else return 1.0f;
    }
    __device__ __forceinline__ float cand_scale() const
    {
        if constexpr (kScaled<DT>) return sa;
        else return 1.0f;
    }
    // The wave's LDS region holds the tolerances of half the slice (vectors 0 and 1: 32 per lane);
    // those of the other half are computed again for every candidate.
    static constexpr int kStoredVectors = 2;
    TolStore<E, true> tol;
    __device__ __forceinline__ void attach_lds(uint32_t region, int lane) { tol.attach(region, lane); }


    template <int V>
    __device__ __forceinline__ void stage_vec(const u32x4 &q, const SegTol &tolerance)
    {
        if constexpr (V == 0) { poisoned_slots = 0; atol_f = tolerance.atol_f; rtol_f = tolerance.rtol_f; }
#pragma unroll
        for (int w = 0; w < 4; ++w) bref[V * 4 + w] = q[w];
        float tv[E];
        static_for<E>([&](auto idx) {
            constexpr int e = decltype(idx)::value;
            const float x = f8_value<DT, e & 3>(q[e >> 2], ref_scale<V>());
            const float prod = rtol_f * __builtin_fabsf(x);
            const float t = atol_f + prod;
            tv[e] = t;
            if (__builtin_amdgcn_ballot_w64(!(t < kInfF))) poisoned_slots |= 1ull << (V * E + e);
        });
        if constexpr (V < kStoredVectors) tol.template put<V>(tv);
    }

    template <int V, bool AHEAD = true>
    __device__ __forceinline__ void compare_vec(const u32x4 &q, float max_abs, float max_rel, uint32_t &suspects,
                                                u64 &trip_abs, u64 &trip_rel, int equal_nan) const
    {
        // The packed reference words are made opaque for each candidate: otherwise the 64 widened values
        // and their 64 tolerances are computed once per item and kept -- in scratch memory.
        uint32_t words[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            words[w] = bref[V * 4 + w];
            asm volatile("" : "+v"(words[w]));
        }
        // Two elements per step: one conversion widens both, and the two "may raise a maximum" tests
        // are folded into a running greatest |d| and a running least margin r|b| - |d| (three-operand
        // max / min, which skip NaN as the comparisons they replace did), tested once per vector.
        float d_most = 0.0f, margin_least = kInfF;
        [[maybe_unused]] float tv[E];
        if constexpr (V < kStoredVectors) tol.template get<V>(tv);
        static_for<E / 2>([&](auto idx) {
            constexpr int p = decltype(idx)::value;
            F32Pair x = f8_pair_to_f32<DT, (p & 1) != 0>(words[p >> 1]);
            F32Pair a = f8_pair_to_f32<DT, (p & 1) != 0>(q[p >> 1]);
            if constexpr (kScaled<DT>) {
                x.lo *= sb[V]; x.hi *= sb[V];
                a.lo *= sa; a.hi *= sa;
            }
            const float d0 = a.lo - x.lo, d1 = a.hi - x.hi;
            float t0, t1;
            if constexpr (V < kStoredVectors) {
                t0 = tv[2 * p];
                t1 = tv[2 * p + 1];
            } else {
                const float prod0 = rtol_f * __builtin_fabsf(x.lo), prod1 = rtol_f * __builtin_fabsf(x.hi);
                t0 = atol_f + prod0;
                t1 = atol_f + prod1;
            }
            suspects += __builtin_popcountll(__builtin_amdgcn_ballot_w64(!(__builtin_fabsf(d0) <= t0)));
            suspects += __builtin_popcountll(__builtin_amdgcn_ballot_w64(!(__builtin_fabsf(d1) <= t1)));
            d_most = __builtin_fmaxf(__builtin_fmaxf(__builtin_fabsf(d0), __builtin_fabsf(d1)), d_most);
            const float m0 = __builtin_fmaf(max_rel, __builtin_fabsf(x.lo), -__builtin_fabsf(d0));
            const float m1 = __builtin_fmaf(max_rel, __builtin_fabsf(x.hi), -__builtin_fabsf(d1));
            margin_least = __builtin_fminf(__builtin_fminf(m0, m1), margin_least);
        });
        trip_abs |= __builtin_amdgcn_ballot_w64(d_most > max_abs);
        trip_rel |= negative_mask(margin_least);
        if constexpr (AHEAD) {
            if ((poisoned_slots >> (V * E)) & 0xFFFFull) suspects += (uint32_t)recount<V>(q, equal_nan);
        }
    }

    // For the marked element positions of vector V: what the full rule counts minus what the bare
    // inequality counted above.  A real function: inlined, its sixteen rarely taken branches cost the
    // stream its registers.
    template <int V>
    __device__ __forceinline__ int recount(const u32x4 &q, int equal_nan) const
    {
        u32x4 b;
#pragma unroll
        for (int w = 0; w < 4; ++w) b[w] = bref[V * 4 + w];
        return recount_vector_f8<DT>(q, b, (uint32_t)(poisoned_slots >> (V * E)) & 0xFFFFu, atol_f, rtol_f, equal_nan, cand_scale(), ref_scale<V>());
    }
    template <int V>
    __device__ __forceinline__ uint32_t false_suspects_call(const u32x4 &q, int equal_nan) const
    {
        return (uint32_t)(-recount<V>(q, equal_nan));        // the caller subtracts
    }

    template <int V>
    __device__ __forceinline__ void raise_call(const u32x4 &q, float &max_abs, float &max_rel, MaxPair *rec) const
    {
        u32x4 b;
#pragma unroll
        for (int w = 0; w < 4; ++w) b[w] = bref[V * 4 + w];
        const FloatPair out = raise_vector_f8<DT>(q, b, max_abs, max_rel, rec, cand_scale(), ref_scale<V>());
        max_abs = uniform_of(out.abs);      // the callee returns the wave's maxima in every lane
        max_rel = uniform_of(out.rel);
    }
    template <int V>
    __device__ __forceinline__ void raise_vec(const u32x4 &q, float &max_abs, float &max_rel, MaxPair *rec, int) const
    {
        raise_call<V>(q, max_abs, max_rel, rec);
    }
};

template <int DT>
__device__ __noinline__ int recount_vector_f8(const u32x4 q, const u32x4 b, const uint32_t marked_in, const float atol_in,
                                              const float rtol_in, const int equal_nan_in, const float sa, const float sb)
{
    const uint32_t marked = uniform32(marked_in);
    const float atol_f = bits_f(uniform32(f_bits(atol_in))), rtol_f = bits_f(uniform32(f_bits(rtol_in)));
    const int equal_nan = (int)uniform32((uint32_t)equal_nan_in);
    int delta = 0;
    static_for<16>([&](auto idx) {
        constexpr int e = decltype(idx)::value;
        if (marked & (1u << e)) {
            const float x = f8_value<DT, e & 3>(b[e >> 2], sb), a = f8_value<DT, e & 3>(q[e >> 2], sa);
            const float prod = rtol_f * __builtin_fabsf(x);
            const float t = atol_f + prod;
            const float d = __builtin_fabsf(a - x);
            delta += __builtin_popcountll(__builtin_amdgcn_ballot_w64(!close_exact(a, x, atol_f, rtol_f, equal_nan)));
            delta -= __builtin_popcountll(__builtin_amdgcn_ballot_w64(!(d <= t)));
        }
    });
    return delta;
}

template <int DT>
__device__ __noinline__ FloatPair raise_vector_f8(const u32x4 q, const u32x4 b, const float max_abs, const float max_rel,
                                                  MaxPair *rec_in, const float sa, const float sb)
{
    MaxPair *rec = uniform_ptr(rec_in);
    float dm = max_abs, rm = max_rel;
    static_for<16>([&](auto idx) {
        constexpr int e = decltype(idx)::value;
        const float x = f8_value<DT, e & 3>(b[e >> 2], sb);
        const float d = __builtin_fabsf(f8_value<DT, e & 3>(q[e >> 2], sa) - x);
        const float babs = __builtin_fabsf(x);
        dm = (d > dm) ? d : dm;                                          // false for NaN: skipped
        const bool hit = (rm < kInfF) && may_raise_rel(rm, babs, d);     // implies d > 0
        if (__builtin_amdgcn_ballot_w64(hit)) {
            const float r = d / babs;                                    // correctly rounded; d/0 = +Inf
            rm = (hit && r > rm) ? r : rm;
        }
    });
    return close_raise<float, FloatPair>(dm, rm, max_abs, max_rel, rec);
}

// ---- uint8 / int8: sixteen elements per 16-byte vector, exact equality ---------------------------
__device__ __forceinline__ uint32_t wave_sum_u(uint32_t x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += (uint32_t)__shfl_xor((int)x, o, kWaveSize);
    return x;
}
// number of bytes of x that are not zero
__device__ __forceinline__ uint32_t nonzero_bytes(uint32_t x)
{
    const uint32_t t = (((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x) & 0x80808080u;
    return (uint32_t)__builtin_popcount(t);
}
template <bool SIGNED>
struct ByteItem {
    typedef double Hint;
    static __device__ __forceinline__ double hint_from_bits(u64 bits) { return __builtin_bit_cast(double, uniform64(bits)); }
    static constexpr int E = 16;
    static constexpr bool kRaiseOutOfLine = true;
    uint32_t bref[kVecPerLane * 4];
    __device__ __forceinline__ void attach_lds(uint32_t, int) {}
    [[maybe_unused]] static constexpr uint32_t poisoned_slots = 0;

    template <int V>
    __device__ __forceinline__ void stage_vec(const u32x4 &q, const SegTol &)
    {
#pragma unroll
        for (int w = 0; w < 4; ++w) bref[V * 4 + w] = q[w];
    }
    // A vector whose sixteen bytes all equal the reference's costs four XORs, two ORs and one compare;
    // only a wave that sees a difference counts the differing bytes (per lane, then summed).
    template <int V, bool AHEAD = true>
    __device__ __forceinline__ void compare_vec(const u32x4 &q, double, double, uint32_t &suspects, u64 &trip_abs, u64 &, int) const
    {
        const uint32_t x0 = q[0] ^ bref[V * 4 + 0], x1 = q[1] ^ bref[V * 4 + 1];
        const uint32_t x2 = q[2] ^ bref[V * 4 + 2], x3 = q[3] ^ bref[V * 4 + 3];
        const u64 m = __builtin_amdgcn_ballot_w64((x0 | x1 | x2 | x3) != 0);
        if (m) {
            suspects += wave_sum_u(nonzero_bytes(x0) + nonzero_bytes(x1) + nonzero_bytes(x2) + nonzero_bytes(x3));
            trip_abs |= m;
        }
    }
    template <int V>
    __device__ __forceinline__ uint32_t false_suspects_call(const u32x4 &, int) const { return 0; }
    template <int V>
    __device__ __forceinline__ void raise_call(const u32x4 &q, double &max_abs, double &max_rel, MaxPair *rec) const
    {
        u32x4 b;
#pragma unroll
        for (int w = 0; w < 4; ++w) b[w] = bref[V * 4 + w];
        const DoublePair out = raise_vector_integer<SIGNED ? GEAK_I8 : GEAK_U8>(q, b, max_abs, max_rel, rec);
        max_abs = uniform_of(out.abs);      // the callee returns the wave's maxima in every lane
        max_rel = uniform_of(out.rel);
    }
    template <int V>
    __device__ __forceinline__ void raise_vec(const u32x4 &q, double &max_abs, double &max_rel, MaxPair *rec, int) const
    {
        raise_call<V>(q, max_abs, max_rel, rec);
    }
};

template <int DT> struct ItemOf { typedef FloatItem<DT> type; };
template <> struct ItemOf<GEAK_U8> { typedef ByteItem<false> type; };
template <> struct ItemOf<GEAK_I8> { typedef ByteItem<true> type; };
template <> struct ItemOf<GEAK_I32> { typedef IntItem type; };
template <> struct ItemOf<GEAK_I64> { typedef Int64Item type; };
template <> struct ItemOf<GEAK_F64> { typedef DoubleItem type; };
template <> struct ItemOf<GEAK_F8E4M3> { typedef Fp8Item<GEAK_F8E4M3> type; };
template <> struct ItemOf<GEAK_F8E5M2> { typedef Fp8Item<GEAK_F8E5M2> type; };
template <> struct ItemOf<GEAK_MXFP8_E4M3> { typedef Fp8Item<GEAK_MXFP8_E4M3> type; };
template <> struct ItemOf<GEAK_MXFP8_E5M2> { typedef Fp8Item<GEAK_MXFP8_E5M2> type; };
template <> struct ItemOf<GEAK_MXINT8> { typedef Fp8Item<GEAK_MXINT8> type; };
template <> struct ItemOf<GEAK_MXFP4_E2M1> { typedef Fp8Item<GEAK_MXFP4_E2M1> type; };
template <> struct ItemOf<GEAK_MXFP6_E2M3> { typedef Fp8Item<GEAK_MXFP6_E2M3> type; };
template <> struct ItemOf<GEAK_MXFP6_E3M2> { typedef Fp8Item<GEAK_MXFP6_E3M2> type; };

__device__ __forceinline__ WaveState uniform_state(const WaveState &in)
{
    WaveState st;
    st.count_off = uniform32(in.count_off);
    st.first_off = uniform32(in.first_off);
    st.tol_off = uniform32(in.tol_off);
    return st;
}

// Instruction issue on a SIMD favours the oldest resident wave, and the four waves that share a
// SIMD come from four blocks dispatched one after another: with equal work the first-dispatched
// finishes 10 % ahead of the last, which then sets the kernel's end.  Each wave therefore walks
// through the four issue priorities, one per candidate slice, starting from a phase that differs
// between the waves of a SIMD, so that every wave spends the same share of its time at every
// priority.
__device__ __forceinline__ void set_issue_priority(uint32_t p)
{
    switch (p & 3u) {
    case 0: __builtin_amdgcn_s_setprio(0); break;
    case 1: __builtin_amdgcn_s_setprio(1); break;
    case 2: __builtin_amdgcn_s_setprio(2); break;
    default: __builtin_amdgcn_s_setprio(3); break;
    }
}

// Arguments of a run of vector-loadable items of one wave.
struct RunArgs {
    const geak_item *items;
    const unsigned char *ref;            // buffer base
    const unsigned char *const *cand;    // device table of K candidate bases
    MaxPair *board;                      // running maxima: [segment][candidate][replica]
    Partial *partials;
    uint32_t replicas;                   // power of two
    uint32_t replica;                    // the one this block reads and raises
    uint32_t first_item;                 // index of the run's first item; the wave follows the items' next links
    uint32_t num_items;                  // table length: no link is followed past it
    uint32_t K;
    uint32_t k0;
    uint32_t priority_phase;             // dispatch round of the block: (block * 4) / grid
    const SegTol *seg_tol;               // per-segment tolerances
    const SegDesc *segments;             // row geometry of row-group items, layout of mapped references
    const uint64_t *ref_item_offset;     // per item, for mapped references (null when the plan has none)
    int equal_nan;
};

// One vector step of the stream: compare vector V of the current candidate, then reuse its
// registers for the same vector of the next element of the wave's stream (the next candidate, or
// the reference slice of the wave's next item).  Four loads per lane stay in flight and each has a
// whole element's worth of compute to land.
template <int DT, int V, bool OUTLINE = false, bool ROWS = false, typename Item>
__device__ __forceinline__ void stream_step(Item &ref, u32x4 &slot, const unsigned char *next, bool has_next,
                                            uint32_t next_n, const bool next_full, typename Item::Hint &max_abs,
                                            typename Item::Hint &max_rel, int equal_nan, MaxPair *rec, int lane,
                                            uint32_t &bad, [[maybe_unused]] uint32_t *scale_byte = nullptr,
                                            [[maybe_unused]] const unsigned char *next_scales = nullptr,
                                            [[maybe_unused]] uint32_t next_off = 0, [[maybe_unused]] bool next_splat = false,
                                            [[maybe_unused]] bool next_active = true)
{
    u64 trip_abs = 0, trip_rel = 0;
    // block-scaled formats: the vector's scale byte travels beside it and is refilled with it
    if constexpr (kScaled<DT>) ref.candidate_scale(*scale_byte);
    ref.template compare_vec<V, !OUTLINE>(slot, max_abs, max_rel, bad, trip_abs, trip_rel, equal_nan);
    if constexpr (OUTLINE && (DT == GEAK_F32 || DT == GEAK_F16 || DT == GEAK_BF16 || DT == GEAK_F64 || DT == GEAK_F8E4M3 ||
                              DT == GEAK_F8E5M2 || kScaled<DT>)) {      // only floating items poison slots
        constexpr u64 kVecMask = ((Traits<DT>::E == 16) ? 0xFFFFull : ((1ull << Traits<DT>::E) - 1ull)) << (V * Traits<DT>::E);
        if (ref.poisoned_slots & kVecMask) bad -= ref.template false_suspects_call<V>(slot, equal_nan);
    }
    if (max_rel == (typename Item::Hint)kInfF) trip_rel = 0;       // nothing exceeds +Inf
    if (trip_abs | trip_rel) {
        if constexpr (OUTLINE || Item::kRaiseOutOfLine) ref.template raise_call<V>(slot, max_abs, max_rel, rec);
        else ref.template raise_vec<V>(slot, max_abs, max_rel, rec, lane);
    }
    if (has_next) {
        if constexpr (ROWS) {                              // a row group: this lane's vector of its row, or its row's one reference element;
            slot = u32x4{0u, 0u, 0u, 0u};                  // a slot behind the group's last row is not loaded and reads as 0 in every tensor
            if (next_active) {
                if (next_splat) slot = splat_element<DT>(next + next_off);
                else slot = __builtin_nontemporal_load((global_vec_ptr)(next + next_off));
            }
        }
        else slot = load_vec<DT>(next, lane, V, next_n, next_full);
        if constexpr (kScaled<DT>) *scale_byte = load_scale_byte(next_scales, (uint32_t)(V * kWaveSize + lane), next_n);
    }
}

// Each dtype's routine is a real function, so that its register allocation stands alone instead of
// being merged with the other dtypes' inside the kernel.  It processes a whole run of consecutive
// FULL items of the dtype: the wave's loads form one stream -- reference slice, K candidate slices,
// next reference slice, ... -- that never drains at an item boundary, and every load is an
// unguarded 16-byte vector load.  Returns the index of the wave's first item it did not process.
// ROWS: the same stream for row groups of one pitched segment whose rows are whole vectors (GEAK_ITEM_STREAM; slots
// behind the group's last row are not loaded and read as 0 on every side): a lane's vector v is vector `vec` of row `row` of the group, `row * pitch + 16 vec`
// bytes behind the item's start -- in the reference, when it has a layout of its own, with its own pitch.
template <int DT, bool ROWS = false>
__device__ __noinline__ uint32_t process_run(const RunArgs in, const WaveState st_in)
{
    typedef typename ItemOf<DT>::type Item;
    typedef typename Item::Hint Hint;
    const WaveState st = uniform_state(st_in);
    const geak_item *items = uniform_ptr(in.items);
    const unsigned char *ref_base = uniform_ptr(in.ref);
    const unsigned char *const *cand = uniform_ptr(in.cand);
    MaxPair *board = uniform_ptr(in.board);
    Partial *partials = uniform_ptr(in.partials);
    const uint32_t replicas = uniform32(in.replicas), replica = uniform32(in.replica);
    const uint32_t num_items = uniform32(in.num_items), K = uniform32(in.K), k0 = uniform32(in.k0);
    uint32_t priority = uniform32(in.priority_phase);
    const SegTol *seg_tol = uniform_ptr(in.seg_tol);
    const int equal_nan = (int)uniform32((uint32_t)in.equal_nan);
    const int lane = threadIdx.x & (kWaveSize - 1);

    uint32_t j = uniform32(in.first_item);
    geak_item it = load_work_item(items, j);
    SegTol tolerance = load_tol(seg_tol, it.segment);
    Item ref;
    ref.attach_lds(st.tol_off, lane);
    u32x4 cur[kVecPerLane];
    constexpr bool full = true;
    // Where an item's reference slice lies: at the item's own offset, or -- a segment whose reference has a layout
    // of its own, contiguous along the row -- at the offset the plan's table gives (any alignment: whole vectors).
    const GEAK_AS_CONSTANT unsigned long long *ref_table = (const GEAK_AS_CONSTANT unsigned long long *)uniform_ptr(in.ref_item_offset);
    const auto ref_offset_of = [&](const geak_item &item, uint32_t index) -> u64 {
        return (item.flags & GEAK_ITEM_REFMAP) ? ref_table[index] : item.byte_offset;
    };
    u64 next_ref_off = 0;
    [[maybe_unused]] uint32_t cand_off[kVecPerLane] = {0u, 0u, 0u, 0u}, ref_off[kVecPerLane] = {0u, 0u, 0u, 0u};
    [[maybe_unused]] bool ref_splat = false;
    if constexpr (ROWS) {
        const ItemShape sh = item_shape<DT, kTailRows>(it, uniform_ptr(in.segments));
        const GEAK_AS_CONSTANT unsigned long long *g = (const GEAK_AS_CONSTANT unsigned long long *)(uniform_ptr(in.segments) + it.segment);
        const uint32_t pitch = (uint32_t)sh.pitch, ref_pitch = (it.flags & GEAK_ITEM_REFMAP) ? (uint32_t)g[6] : pitch;     // the planner admits pitches whose group fits 32 bits
        ref_splat = (it.flags & GEAK_ITEM_REFMAP) && ((uint32_t)(g[4] >> 32) >> kRefStrideShift) == 0;                     // one reference element per row
#pragma unroll
        for (int v = 0; v < kVecPerLane; ++v) {
            const uint32_t slot = (uint32_t)(v * kWaveSize + lane), row = (slot * sh.inv) >> 16, vec = slot - row * sh.vpr;
            cand_off[v] = row * pitch + vec * 16u;
            ref_off[v] = row * ref_pitch + (ref_splat ? 0u : vec * 16u);
        }
    }
#pragma unroll
    for (int v = 0; v < kVecPerLane; ++v) {                // the only loads of the run that nothing hides
        if constexpr (ROWS) {
            // the group's rows are whole vectors: numel / E of the item's 256 slots hold them, the others read as 0
            const unsigned char *at = ref_base + ref_offset_of(it, j) + ref_off[v];
            cur[v] = u32x4{0u, 0u, 0u, 0u};
            if ((uint32_t)(v * kWaveSize + lane) < (uint32_t)it.numel / (uint32_t)Traits<DT>::E) {
                if (ref_splat) cur[v] = splat_element<DT>(at);
                else cur[v] = __builtin_nontemporal_load((global_vec_ptr)at);
            }
        } else {
            cur[v] = load_vec<DT>(ref_base + ref_offset_of(it, j), lane, v, it.numel, full);
        }
    }
    // block-scaled formats: the scale byte of each vector's block, loaded and refilled beside the vector
    [[maybe_unused]] uint32_t sc[kVecPerLane] = {0u, 0u, 0u, 0u};
    [[maybe_unused]] u64 scale_off = 0, next_scale_off = 0;
    if constexpr (kScaled<DT>) {
        scale_off = item_scale_offset(it, uniform_ptr(in.segments));
#pragma unroll
        for (int v = 0; v < kVecPerLane; ++v) sc[v] = load_scale_byte(ref_base + scale_off, (uint32_t)(v * kWaveSize + lane), it.numel);
    }

    for (;;) {
        // look ahead: does the wave's next item continue the run?
        const uint32_t jn = it.next;
        bool more = jn < num_items;                 // kNoItem ends the list
        geak_item nx = it;
        if (more) {
            nx = load_work_item(items, jn);
            if constexpr (ROWS) more = (nx.flags & GEAK_ITEM_STREAM) && nx.dtype == DT && nx.segment == it.segment;     // the same rows: the same offsets
            else more = (nx.flags & GEAK_ITEM_FULL) && nx.dtype == DT;
        }
        if (more) next_ref_off = ref_offset_of(nx, jn);
        const SegTol cur_tol = tolerance;
        if (more) tolerance = load_tol(seg_tol, nx.segment);          // the next item's, a whole item ahead of its use
        if constexpr (kScaled<DT>) {
            if (more) next_scale_off = item_scale_offset(nx, uniform_ptr(in.segments));
        }
        if (it.flags & GEAK_ITEM_FIRST) begin_run(st, K, lane);
        MaxPair *recs = board + (u64)it.segment * K * replicas + replica;     // candidate k: recs[k * replicas]

        // reference element: stage it, refilling each vector with the first candidate's
        uint32_t k = k0;
        {
            const unsigned char *first = table_entry(cand, k) + it.byte_offset;
            if constexpr (kScaled<DT>) {
                const unsigned char *first_scales = table_entry(cand, k) + scale_off;
                static_for<kVecPerLane>([&](auto idx) {
                    constexpr int v = decltype(idx)::value;
                    ref.template stage_scale<v>(sc[v]);
                    sc[v] = load_scale_byte(first_scales, (uint32_t)(v * kWaveSize + lane), it.numel);
                });
            }
            const auto first_vec = [&](auto idx) -> u32x4 {
                constexpr int v = decltype(idx)::value;
                if constexpr (ROWS) {
                    u32x4 q = {0u, 0u, 0u, 0u};
                    if ((uint32_t)(v * kWaveSize + lane) < (uint32_t)it.numel / (uint32_t)Traits<DT>::E) q = __builtin_nontemporal_load((global_vec_ptr)(first + cand_off[v]));
                    return q;
                } else {
                    return load_vec<DT>(first, lane, v, it.numel, full);
                }
            };
            ref.template stage_vec<0>(cur[0], cur_tol); cur[0] = first_vec(Index<0>{});
            ref.template stage_vec<1>(cur[1], cur_tol); cur[1] = first_vec(Index<1>{});
            ref.template stage_vec<2>(cur[2], cur_tol); cur[2] = first_vec(Index<2>{});
            ref.template stage_vec<3>(cur[3], cur_tol); cur[3] = first_vec(Index<3>{});
        }
        u64 abs_bits = load_bits(&recs[k * replicas].abs), rel_bits = load_bits(&recs[k * replicas].rel);

        for (uint32_t step = 0; step < K; ++step) {
            set_issue_priority(priority++);
            const uint32_t kn = (k + 1 == K) ? 0 : k + 1;
            const bool last = step + 1 == K;
            const bool has_next = !last || more;
            const unsigned char *next = last ? ref_base + next_ref_off : table_entry(cand, kn) + it.byte_offset;
            const uint32_t next_n = last ? nx.numel : it.numel;
            [[maybe_unused]] const unsigned char *next_scales = nullptr;
            if constexpr (kScaled<DT>) next_scales = last ? ref_base + next_scale_off : table_entry(cand, kn) + scale_off;

            Hint max_abs = Item::hint_from_bits(abs_bits);      // exact: floating maxima are published from binary32
            Hint max_rel = Item::hint_from_bits(rel_bits);
            if (!last) {
                abs_bits = load_bits(&recs[kn * replicas].abs);
                rel_bits = load_bits(&recs[kn * replicas].rel);
            }
            uint32_t bad = 0;
            stream_step<DT, 0, false, ROWS>(ref, cur[0], next, has_next, next_n, full, max_abs, max_rel, equal_nan, &recs[k * replicas], lane, bad, &sc[0], next_scales, last ? ref_off[0] : cand_off[0], last && ref_splat,
                                            (uint32_t)(0 * kWaveSize + lane) < (uint32_t)(last ? nx.numel : it.numel) / (uint32_t)Traits<DT>::E);
            stream_step<DT, 1, false, ROWS>(ref, cur[1], next, has_next, next_n, full, max_abs, max_rel, equal_nan, &recs[k * replicas], lane, bad, &sc[1], next_scales, last ? ref_off[1] : cand_off[1], last && ref_splat,
                                            (uint32_t)(1 * kWaveSize + lane) < (uint32_t)(last ? nx.numel : it.numel) / (uint32_t)Traits<DT>::E);
            stream_step<DT, 2, false, ROWS>(ref, cur[2], next, has_next, next_n, full, max_abs, max_rel, equal_nan, &recs[k * replicas], lane, bad, &sc[2], next_scales, last ? ref_off[2] : cand_off[2], last && ref_splat,
                                            (uint32_t)(2 * kWaveSize + lane) < (uint32_t)(last ? nx.numel : it.numel) / (uint32_t)Traits<DT>::E);
            stream_step<DT, 3, false, ROWS>(ref, cur[3], next, has_next, next_n, full, max_abs, max_rel, equal_nan, &recs[k * replicas], lane, bad, &sc[3], next_scales, last ? ref_off[3] : cand_off[3], last && ref_splat,
                                            (uint32_t)(3 * kWaveSize + lane) < (uint32_t)(last ? nx.numel : it.numel) / (uint32_t)Traits<DT>::E);
            note_mismatches(st, k, bad, j, lane);
            k = kn;
        }
        if (it.flags & GEAK_ITEM_LAST) end_run(st, partials, it.slot, K, lane);
        if (!more) break;
        it = nx;
        j = jn;
        scale_off = next_scale_off;
    }
    return it.next;
}

// ---- a segment's tail: one item that starts aligned but is shorter than a full item -----------------
// A wave is latency-bound per load round trip whatever the slice length, so a short tail is not
// streamed candidate by candidate: the four vector registers per lane are packed with as many
// candidates as fit (four when the tail needs one vector per lane, two when it needs two), the
// loads of a batch -- and, for the first batch, of the reference -- are issued together, and the
// whole batch is compared after a single wait.  Absent elements read as 0 on both sides.  A row
// group (short rows of a pitched segment, a pitch apart) goes the same way: only the address and the
// number of valid elements of a lane's vector differ.  So does an item that starts off the 16-byte
// grid (a segment's or a row's first item): it is read from the boundary before it.
// MAPPED: the segment's reference has a layout of its own; only where the reference's vectors are loaded
// from differs.
template <int DT, int KIND, bool MAPPED>
__device__ __noinline__ void process_tail(const RunArgs in, const WaveState st_in)
{
    typedef typename ItemOf<DT>::type Item;
    typedef typename Item::Hint Hint;
    const WaveState st = uniform_state(st_in);
    const geak_item *items = uniform_ptr(in.items);
    const unsigned char *ref_base = uniform_ptr(in.ref);
    const unsigned char *const *cand = uniform_ptr(in.cand);
    MaxPair *board = uniform_ptr(in.board);
    Partial *partials = uniform_ptr(in.partials);
    const uint32_t replicas = uniform32(in.replicas), replica = uniform32(in.replica);
    const uint32_t K = uniform32(in.K);
    const SegTol *seg_tol = uniform_ptr(in.seg_tol);
    const int equal_nan = (int)uniform32((uint32_t)in.equal_nan);
    const int lane = threadIdx.x & (kWaveSize - 1);
    const uint32_t j = uniform32(in.first_item);
    const geak_item it = load_work_item(items, j);
    const SegTol tolerance = load_tol(seg_tol, it.segment);
    const ItemShape shape = item_shape<DT, KIND>(it, uniform_ptr(in.segments));
    const uint32_t n = it.numel;
    const u64 offset = it.byte_offset - (u64)shape.skip * Traits<DT>::W;                    // of vector slot 0
    const uint32_t vectors = shape_vectors<DT>(shape, n);                                   // 1..4 per lane
    const uint32_t per_batch = vectors == 1 ? 4 : (vectors == 2 ? 2 : 1);                       // candidates per batch
    MaxPair *recs = board + (u64)it.segment * K * replicas + replica;         // candidate k: recs[k * replicas]

    // loads of one batch: candidate kb + c occupies registers [c * (4 / per_batch), ...); for the block-scaled
    // formats the scale byte of each register's vector is loaded beside it (such items are plain tails)
    u32x4 cur[kVecPerLane];
    [[maybe_unused]] uint32_t cs[kVecPerLane] = {127u, 127u, 127u, 127u};
    [[maybe_unused]] u64 scale_off = 0;
    if constexpr (kScaled<DT>) scale_off = item_scale_offset(it, uniform_ptr(in.segments));
    const auto load_register = [&](int reg, uint32_t k, int v) {
        cur[reg] = load_shaped<DT, KIND>(table_entry(cand, k) + offset, lane, v, n, shape);
        if constexpr (kScaled<DT>) cs[reg] = load_scale_byte(table_entry(cand, k) + scale_off, (uint32_t)(v * kWaveSize + lane), n);
    };
    const auto load_batch = [&](uint32_t kb) {
        if (per_batch == 4) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (kb + c < K) load_register(c, kb + c, 0);
        } else if (per_batch == 2) {
#pragma unroll
            for (int c = 0; c < 2; ++c)
                if (kb + c < K) {
                    load_register(2 * c + 0, kb + c, 0);
                    load_register(2 * c + 1, kb + c, 1);
                }
        } else {
#pragma unroll
            for (int v = 0; v < kVecPerLane; ++v) load_register(v, kb, v);
        }
    };

    Item ref;
    ref.attach_lds(st.tol_off, lane);
    {
        u32x4 r[kVecPerLane];
        if constexpr (MAPPED) {
            const RefPlace place = ref_place<DT>(it, j, uniform_ptr(in.segments), uniform_ptr(in.ref_item_offset));
            uint32_t first;
#pragma unroll
            for (int v = 0; v < kVecPerLane; ++v)
                r[v] = load_ref_slot<DT, KIND>(ref_base, place, (uint32_t)(v * kWaveSize + lane), n, shape, first);
        } else {
#pragma unroll
            for (int v = 0; v < kVecPerLane; ++v) r[v] = load_shaped<DT, KIND>(ref_base + offset, lane, v, n, shape);
        }
        [[maybe_unused]] uint32_t rs[kVecPerLane];
        if constexpr (kScaled<DT>) {
#pragma unroll
            for (int v = 0; v < kVecPerLane; ++v) rs[v] = load_scale_byte(ref_base + scale_off, (uint32_t)(v * kWaveSize + lane), n);
        }
        load_batch(0);                                     // in flight together with the reference
        if constexpr (kScaled<DT>) {
            static_for<kVecPerLane>([&](auto idx) { ref.template stage_scale<decltype(idx)::value>(rs[decltype(idx)::value]); });
        }
        ref.template stage_vec<0>(r[0], tolerance);
        ref.template stage_vec<1>(r[1], tolerance);
        ref.template stage_vec<2>(r[2], tolerance);
        ref.template stage_vec<3>(r[3], tolerance);
    }
    if (it.flags & GEAK_ITEM_FIRST) begin_run(st, K, lane);

    // compare register vector `q` as vector V of candidate k, accumulating into bad
    const auto one = [&](auto vtag, int reg, uint32_t k, Hint &max_abs, Hint &max_rel, uint32_t &bad) {
        constexpr int V = decltype(vtag)::value;
        u32x4 slot = cur[reg];
        stream_step<DT, V, true>(ref, slot, nullptr, false, 0, false, max_abs, max_rel, equal_nan, &recs[k * replicas], lane, bad, &cs[reg]);
    };
    const auto hints = [&](uint32_t k, Hint &max_abs, Hint &max_rel) {
        max_abs = Item::hint_from_bits(load_bits(&recs[k * replicas].abs));
        max_rel = Item::hint_from_bits(load_bits(&recs[k * replicas].rel));
    };

    for (uint32_t kb = 0; kb < K; kb += per_batch) {
        if (kb) load_batch(kb);
        if (per_batch == 4) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (kb + c < K) {
                    Hint ma, mr;
                    hints(kb + c, ma, mr);
                    uint32_t bad = 0;
                    one(Index<0>{}, c, kb + c, ma, mr, bad);
                    note_mismatches(st, kb + c, bad, j, lane);
                }
        } else if (per_batch == 2) {
#pragma unroll
            for (int c = 0; c < 2; ++c)
                if (kb + c < K) {
                    Hint ma, mr;
                    hints(kb + c, ma, mr);
                    uint32_t bad = 0;
                    one(Index<0>{}, 2 * c + 0, kb + c, ma, mr, bad);
                    one(Index<1>{}, 2 * c + 1, kb + c, ma, mr, bad);
                    note_mismatches(st, kb + c, bad, j, lane);
                }
        } else {
            Hint ma, mr;
            hints(kb, ma, mr);
            uint32_t bad = 0;
            one(Index<0>{}, 0, kb, ma, mr, bad);
            one(Index<1>{}, 1, kb, ma, mr, bad);
            one(Index<2>{}, 2, kb, ma, mr, bad);
            one(Index<3>{}, 3, kb, ma, mr, bad);
            note_mismatches(st, kb, bad, j, lane);
        }
    }
    if (it.flags & GEAK_ITEM_LAST) end_run(st, partials, it.slot, K, lane);
}

__global__ __launch_bounds__(kBlockThreads, 4) void compare_kernel(const CompareArgs p)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t K = p.num_candidates;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t range = table_range_of_block(blockIdx.x, gridDim.x, p.unit_groups, p.block_map);
    WaveState st;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(GEAK_AS_LDS unsigned char *)lds;
    st.count_off = lds_base + (uint32_t)sizeof(u64) * wave * K;
    st.first_off = lds_base + (uint32_t)sizeof(u64) * kWavesPerBlock * K + (uint32_t)sizeof(uint32_t) * wave * K;
    st.tol_off = lds_base + lds_state_bytes((int)K) + kTolBytesPerWave * wave;

    RunArgs r;
    r.items = p.items;
    r.ref = p.ref;
    r.cand = p.cand_table;
    r.board = p.board;
    r.replicas = p.replicas;
    r.replica = range & (p.replicas - 1);
    r.partials = p.partials;
    r.num_items = p.num_items;
    r.K = K;
    r.k0 = (range / p.replicas) % K;
    r.priority_phase = (blockIdx.x * 4u) / gridDim.x;
    r.seg_tol = p.seg_tol;
    r.segments = p.segments;
    r.ref_item_offset = p.ref_item_offset;
    r.equal_nan = p.equal_nan;

    // the wave's list of items: its first one from the wave table, then along the next links
    const GEAK_AS_CONSTANT uint32_t *wave_first = (const GEAK_AS_CONSTANT uint32_t *)p.wave_first;
    uint32_t j = wave_first[range * kWavesPerBlock + wave];
    while (j < p.num_items) {                                   // kNoItem ends the list; nothing past the table is read
        const geak_item it = load_work_item(p.items, j);
        // a run of full items, or one item of another shape: handled, state bookkeeping included, by the dtype's routine
        r.first_item = j;
        uint32_t next_j = it.next;
        if (it.dtype >= GEAK_MXFP8_E4M3) {                  // block-scaled: contiguous, on the grid, so full items and plain tails only
            if (it.flags & GEAK_ITEM_FULL) for_scaled_dtype(it.dtype, [&](auto dt) { next_j = process_run<decltype(dt)::value>(r, st); });
            else for_scaled_dtype(it.dtype, [&](auto dt) { process_tail<decltype(dt)::value, kTailPlain, false>(r, st); });
        } else if (it.flags & GEAK_ITEM_FULL) {
            for_dtype(it.dtype, [&](auto dt) { next_j = process_run<decltype(dt)::value>(r, st); });
        } else if (it.flags & GEAK_ITEM_STREAM) {            // whole row groups: streamed like full items
            for_dtype(it.dtype, [&](auto dt) { next_j = process_run<decltype(dt)::value, true>(r, st); });
        } else if (it.flags & GEAK_ITEM_REFMAP) {
            if (it.flags & GEAK_ITEM_ROWS) for_dtype(it.dtype, [&](auto dt) { process_tail<decltype(dt)::value, kTailRows, true>(r, st); });
            else if (it.flags & GEAK_ITEM_ALIGNED) for_dtype(it.dtype, [&](auto dt) { process_tail<decltype(dt)::value, kTailPlain, true>(r, st); });
            else for_dtype(it.dtype, [&](auto dt) { process_tail<decltype(dt)::value, kTailShifted, true>(r, st); });
        } else if (it.flags & GEAK_ITEM_ROWS) {
            for_dtype(it.dtype, [&](auto dt) { process_tail<decltype(dt)::value, kTailRows, false>(r, st); });
        } else if (it.flags & GEAK_ITEM_ALIGNED) {
            for_dtype(it.dtype, [&](auto dt) { process_tail<decltype(dt)::value, kTailPlain, false>(r, st); });
        } else {
            for_dtype(it.dtype, [&](auto dt) { process_tail<decltype(dt)::value, kTailShifted, false>(r, st); });
        }
        j = __builtin_amdgcn_readfirstlane(next_j);
    }
}

// ---- init: neutral records (also final for empty segments) and the candidate pointer table --------
__global__ void init_kernel(const InitArgs p)
{
    const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < p.num_results) {
        geak_result r;
        r.pass = 1;
        r.reserved = 0;
        r.mismatch_count = 0;
        r.first_mismatch = -1;
        r.max_abs_err = 0.0;
        r.max_rel_err = 0.0;
        p.results[i] = r;
    }
    if (p.cand_table && i < p.num_candidates) p.cand_table[i] = p.cand[i];
    for (u64 e = i; e < p.num_board; e += (u64)gridDim.x * blockDim.x) {      // running maxima start at +0
        p.board[e].abs = 0.0;
        p.board[e].rel = 0.0;
    }
}

// ---- reduce: one block per (segment, candidate) ----------------------------------------------
constexpr int kReduceThreads = 256;
constexpr uint64_t kReduceWavePairs = 1024;        // from this many (segment, candidate) pairs on, one wave per pair

// Least element of one 16-byte vector pair that is not close, or kNoItem: the rescan of an item's
// first mismatch, one vector per thread.  `valid` elements of the vector lie inside the item.
template <int DT>
__device__ __forceinline__ uint32_t first_bad_in_vector(const u32x4 &qa, const u32x4 &qb, uint32_t valid, const SegTol &tolerance,
                                                        int equal_nan, [[maybe_unused]] float sa = 1.0f, [[maybe_unused]] float sb = 1.0f)
{
    constexpr int E = Traits<DT>::E;
    uint32_t best = kNoItem;
    static_for<E>([&](auto idx) {
        constexpr int e = E - 1 - decltype(idx)::value;                 // downwards, so that the least index is kept
        bool close;
        if constexpr (DT == GEAK_I32) close = qa[e] == qb[e];
        else if constexpr (DT == GEAK_I64) close = qa[2 * e] == qb[2 * e] && qa[2 * e + 1] == qb[2 * e + 1];
        else if constexpr (DT == GEAK_U8 || DT == GEAK_I8) close = ((qa[e >> 2] ^ qb[e >> 2]) >> (8 * (e & 3)) & 0xFFu) == 0;
        else if constexpr (DT == GEAK_F64)
            close = close_exact_d(bits_d(qa[2 * e], qa[2 * e + 1]), bits_d(qb[2 * e], qb[2 * e + 1]), tolerance.atol, tolerance.rtol, equal_nan);
        else if constexpr (DT == GEAK_F8E4M3 || DT == GEAK_F8E5M2 || kScaled<DT>)
            close = close_exact(f8_value<DT, e & 3>(qa[e >> 2], sa), f8_value<DT, e & 3>(qb[e >> 2], sb), tolerance.atol_f, tolerance.rtol_f, equal_nan);
        else close = close_exact(decode<DT>(qa, e), decode<DT>(qb, e), tolerance.atol_f, tolerance.rtol_f, equal_nan);
        if ((uint32_t)e < valid && !close) best = (uint32_t)e;
    });
    return best;
}
template <int DT, int KIND>
__device__ __forceinline__ uint32_t first_bad_of_slot(const unsigned char *ref, const unsigned char *cand, uint32_t slot, const geak_item &it,
                                                      uint32_t item_index, const SegDesc *segments, const uint64_t *ref_item_offset,
                                                      const SegTol &tolerance, int equal_nan)
{
    const ItemShape shape = item_shape<DT, KIND>(it, segments);
    const u64 offset = it.byte_offset - (u64)shape.skip * Traits<DT>::W;         // of vector slot 0
    uint32_t first;
    u32x4 qb;
    if (it.flags & GEAK_ITEM_REFMAP) qb = load_ref_slot<DT, KIND>(ref, ref_place<DT>(it, item_index, segments, ref_item_offset), slot, it.numel, shape, first);
    else qb = load_slot<DT, KIND>(ref + offset, slot, it.numel, shape, first);
    const u32x4 qa = load_slot<DT, KIND>(cand + offset, slot, it.numel, shape, first);
    // positions outside the item read as 0 on both sides and are close under every rule
    uint32_t e;
    if constexpr (kScaled<DT>) {
        const u64 scale_off = item_scale_offset(it, segments);
        e = first_bad_in_vector<DT>(qa, qb, (uint32_t)Traits<DT>::E, tolerance, equal_nan,
                                    scale_of_byte<DT>(load_scale_byte(cand + scale_off, slot, it.numel)),
                                    scale_of_byte<DT>(load_scale_byte(ref + scale_off, slot, it.numel)));
    } else {
        e = first_bad_in_vector<DT>(qa, qb, (uint32_t)Traits<DT>::E, tolerance, equal_nan);
    }
    return e == kNoItem ? kNoItem : first + e;
}
template <int DT>
__device__ __forceinline__ uint32_t first_bad_of_thread(const unsigned char *ref, const unsigned char *cand, int tid, const geak_item &it,
                                                        uint32_t item_index, const SegDesc *segments, const uint64_t *ref_item_offset,
                                                        const SegTol &tolerance, int equal_nan)
{
    // the three branches are uniform
    if (it.flags & GEAK_ITEM_ROWS)
        return first_bad_of_slot<DT, kTailRows>(ref, cand, (uint32_t)tid, it, item_index, segments, ref_item_offset, tolerance, equal_nan);
    if (it.flags & GEAK_ITEM_ALIGNED)
        return first_bad_of_slot<DT, kTailPlain>(ref, cand, (uint32_t)tid, it, item_index, segments, ref_item_offset, tolerance, equal_nan);
    return first_bad_of_slot<DT, kTailShifted>(ref, cand, (uint32_t)tid, it, item_index, segments, ref_item_offset, tolerance, equal_nan);
}

__global__ __launch_bounds__(kReduceThreads) void reduce_kernel(const ReduceArgs p)
{
    __shared__ u64 s_count[kReduceThreads / kWaveSize];
    __shared__ uint32_t s_first[kReduceThreads / kWaveSize];
    __shared__ uint32_t s_best[kReduceThreads / kWaveSize];
    const uint32_t K = p.num_candidates;
    const uint32_t seg = blockIdx.x / K, k = blockIdx.x % K;
    const int tid = threadIdx.x, lane = tid & (kWaveSize - 1), wave = tid / kWaveSize;
    const uint32_t sb = p.slot_begin[seg], se = p.slot_begin[seg + 1];
    if (sb == se) return;                       // empty segment: the neutral record stands (uniform exit)

    // sum of the counts and least first-item index over the segment's slots; eight independent loads
    // per thread are in flight at a time
    u64 count = 0;
    uint32_t first_item = kNoItem;
    for (uint32_t s0 = sb + tid; s0 < se; s0 += 8 * kReduceThreads) {
        Partial r[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t s = s0 + u * kReduceThreads;
            r[u].count = 0;
            r[u].first_item = kNoItem;
            if (s < se) r[u] = p.partials[(u64)s * K + k];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            count += r[u].count;
            first_item = r[u].first_item < first_item ? r[u].first_item : first_item;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) count += (u64)__shfl_xor((long long)count, o, kWaveSize);
    first_item = wave_min_u(first_item);
    if (lane == 0) { s_count[wave] = count; s_first[wave] = first_item; }
    __syncthreads();
    count = 0;
    first_item = kNoItem;
#pragma unroll
    for (int w = 0; w < kReduceThreads / kWaveSize; ++w) {
        count += s_count[w];
        first_item = s_first[w] < first_item ? s_first[w] : first_item;
    }

    // exact first index: re-read the first item that holds a mismatch, every thread one 16-byte vector of
    // the reference and of the candidate (256 threads x 16 bytes: the whole item; whatever the item's shape,
    // its vector slots ascend with the element index)
    long long first = -1;
    if (first_item != kNoItem) {                // uniform: every thread holds the same first_item
        const geak_item it = p.items[first_item];
        const SegTol tolerance = p.seg_tol[seg];
        uint32_t best = kNoItem;
        const auto rescan = [&](auto dt) {
            best = first_bad_of_thread<decltype(dt)::value>(p.ref, p.cand_table[k], tid, it, first_item, p.segments, p.ref_item_offset, tolerance, p.equal_nan);
        };
        if (it.dtype >= GEAK_MXFP8_E4M3) for_scaled_dtype(it.dtype, rescan);
        else for_dtype(it.dtype, rescan);
        best = wave_min_u(best);
        if (lane == 0) s_best[wave] = best;
        __syncthreads();
        best = kNoItem;
#pragma unroll
        for (int w = 0; w < kReduceThreads / kWaveSize; ++w) best = s_best[w] < best ? s_best[w] : best;
        first = (long long)it.elem_start + (long long)best;
    }
    if (wave == 0) {
        // the two maxima: largest bit pattern over the replicas (non-negative doubles order like their bits)
        const MaxPair *mp = p.board + ((u64)seg * K + k) * p.replicas;
        u64 a = 0, r = 0;
        for (uint32_t i = lane; i < p.replicas; i += kWaveSize) {
            const u64 ai = __builtin_bit_cast(u64, mp[i].abs), ri = __builtin_bit_cast(u64, mp[i].rel);
            a = ai > a ? ai : a;
            r = ri > r ? ri : r;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const u64 ao = (u64)__shfl_xor((long long)a, o, kWaveSize), ro = (u64)__shfl_xor((long long)r, o, kWaveSize);
            a = ao > a ? ao : a;
            r = ro > r ? ro : r;
        }
        if (lane == 0) {
            geak_result *rec = p.results + (u64)seg * K + k;
            rec->pass = (count == 0);
            rec->mismatch_count = count;
            rec->first_mismatch = first;
            rec->max_abs_err = __builtin_bit_cast(double, a);
            rec->max_rel_err = __builtin_bit_cast(double, r);
        }
    }
}

// The same reduction with one wave per (segment, candidate) and no barrier: for plans with many pairs
// (ragged batches), where a whole block per pair leaves most of its threads without a slot to read
// and the number of blocks, not the work, sets the time.  A lane takes four vector slots of the
// item that is scanned again.
template <int DT>
__device__ __forceinline__ uint32_t first_bad_of_lane(const unsigned char *ref, const unsigned char *cand, int lane, const geak_item &it,
                                                      uint32_t item_index, const SegDesc *segments, const uint64_t *ref_item_offset,
                                                      const SegTol &tolerance, int equal_nan)
{
    uint32_t best = kNoItem;
#pragma unroll
    for (int v = kVecPerLane - 1; v >= 0; --v) {            // downwards, so that the least index is kept
        const uint32_t b = first_bad_of_thread<DT>(ref, cand, v * kWaveSize + lane, it, item_index, segments, ref_item_offset, tolerance, equal_nan);
        best = b < best ? b : best;
    }
    return best;
}

__global__ __launch_bounds__(kReduceThreads) void reduce_wave_kernel(const ReduceArgs p)
{
    const uint32_t K = p.num_candidates;
    const int tid = threadIdx.x, lane = tid & (kWaveSize - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane((uint32_t)tid / kWaveSize);
    const u64 pair = (u64)blockIdx.x * (kReduceThreads / kWaveSize) + wave;
    if (pair >= (u64)p.num_segments * K) return;
    const uint32_t seg = (uint32_t)(pair / K), k = (uint32_t)(pair % K);
    const uint32_t sb = p.slot_begin[seg], se = p.slot_begin[seg + 1];
    if (sb == se) return;                       // empty segment: the neutral record stands

    // the two maxima: asked for first, used last
    const MaxPair *mp = p.board + ((u64)seg * K + k) * p.replicas;
    u64 a = 0, r = 0;
    for (uint32_t i = lane; i < p.replicas; i += kWaveSize) {
        const u64 ai = __builtin_bit_cast(u64, mp[i].abs), ri = __builtin_bit_cast(u64, mp[i].rel);
        a = ai > a ? ai : a;
        r = ri > r ? ri : r;
    }

    u64 count = 0;
    uint32_t first_item = kNoItem;
    for (uint32_t s0 = sb + lane; s0 < se; s0 += 8 * kWaveSize) {
        Partial q[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t s = s0 + u * kWaveSize;
            q[u].count = 0;
            q[u].first_item = kNoItem;
            if (s < se) q[u] = p.partials[(u64)s * K + k];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            count += q[u].count;
            first_item = q[u].first_item < first_item ? q[u].first_item : first_item;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) count += (u64)__shfl_xor((long long)count, o, kWaveSize);
    first_item = wave_min_u(first_item);

    long long first = -1;
    if (first_item != kNoItem) {                // uniform over the wave
        const geak_item it = p.items[first_item];
        const SegTol tolerance = p.seg_tol[seg];
        uint32_t best = kNoItem;
        const auto rescan = [&](auto dt) {
            best = first_bad_of_lane<decltype(dt)::value>(p.ref, p.cand_table[k], lane, it, first_item, p.segments, p.ref_item_offset, tolerance, p.equal_nan);
        };
        if (it.dtype >= GEAK_MXFP8_E4M3) for_scaled_dtype(it.dtype, rescan);
        else for_dtype(it.dtype, rescan);
        best = wave_min_u(best);
        first = (long long)it.elem_start + (long long)best;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const u64 ao = (u64)__shfl_xor((long long)a, o, kWaveSize), ro = (u64)__shfl_xor((long long)r, o, kWaveSize);
        a = ao > a ? ao : a;
        r = ro > r ? ro : r;
    }
    if (lane == 0) {
        geak_result *rec = p.results + pair;
        rec->pass = (count == 0);
        rec->mismatch_count = count;
        rec->first_mismatch = first;
        rec->max_abs_err = __builtin_bit_cast(double, a);
        rec->max_rel_err = __builtin_bit_cast(double, r);
    }
}

// ---- mismatch report: the first elements of each pair that are not close ----------------------------
// One block per (segment, candidate).  The pair's record says where its first mismatch is and how
// many there are; the block walks the segment from there in tiles of 4096 elements (thread t looks
// at elements t, t + 256, ... of the tile, all of its loads in flight together), ranks the
// mismatches of a tile in index order with lane masks and one LDS table, writes those that still fit
// and stops when it has min(max_records, mismatch_count) of them.
constexpr int kReportThreads = 256;
constexpr int kReportPerThread = 16;

// one element straight from memory, by compile-time dtype (all of a thread's loads can then be issued together)
template <int DT>
__device__ __forceinline__ float elem_f(const unsigned char *base, u64 idx)
{
    if constexpr (DT == GEAK_F32) return reinterpret_cast<const float *>(base)[idx];
    else if constexpr (DT == GEAK_MXFP4_E2M1) {             // element idx is a nibble of byte idx / 2; its E4M3 code from the same table as the loads'
        const uint32_t nib = ((uint32_t)base[idx >> 1] >> (4 * (uint32_t)(idx & 1))) & 0xFu;
        const uint32_t code = (uint32_t)((0x4C4844403C383000ull >> (8 * (nib & 7u))) & 0xFFu) | ((nib & 8u) << 4);
        return f8_to_f32<DT, 0>(code);
    }
    else if constexpr (kFp6<DT>) {                           // element idx is the six bits from bit 6 idx on; its E4M3 code as the loads form it
        const u64 bit = 6 * idx;
        const uint32_t lo = base[bit >> 3], hi = (bit & 7) > 2 ? (uint32_t)base[(bit >> 3) + 1] : 0u;       // the code may straddle two bytes
        return f8_to_f32<DT, 0>(fp6_four<DT>(((lo | (hi << 8)) >> (bit & 7)) & 0x3Fu));
    }
    else if constexpr (DT == GEAK_F8E4M3 || DT == GEAK_F8E5M2 || kScaled<DT>) return f8_to_f32<DT, 0>(base[idx]);     // block-scaled: the bare code's value
    else if constexpr (DT == GEAK_F16) return (float)__builtin_bit_cast(_Float16, reinterpret_cast<const uint16_t *>(base)[idx]);
    else return bits_f((uint32_t)reinterpret_cast<const uint16_t *>(base)[idx] << 16);
}

template <int DT> constexpr bool kIntegerDtype = (DT == GEAK_I32 || DT == GEAK_I64 || DT == GEAK_U8 || DT == GEAK_I8);

template <int DT>
__device__ __forceinline__ void report_pair(const ReportArgs &p, const SegTol tolerance, const SegDesc &sg, const geak_result &rec, u64 want,
                                            const unsigned char *rb, const unsigned char *cb, geak_mismatch *out,
                                            uint32_t (&s_cnt)[kReportPerThread][kReportThreads / kWaveSize])
{
    const int tid = threadIdx.x, lane = tid & (kWaveSize - 1), wave = tid / kWaveSize;
    // a pitched segment: flat index i sits in row i / row_elems; in units of elements the rows are pitch_elems apart
    const bool pitched = sg.row_elems != sg.numel;
    const u64 pitch_elems = sg.pitch_bytes / (u64)Traits<DT>::W;
    // a reference with a layout of its own: its rows are ref_pitch_elems apart and hold the row's elements or one for all
    const bool mapped = seg_ref_mapped(sg);
    const u64 ref_stride = seg_ref_stride(sg);          // elements between neighbours of a reference row
    const u64 ref_pitch_elems = sg.ref_pitch_bytes / (u64)Traits<DT>::W;
    // a block-scaled segment: its scale bytes, one per 32 elements, in the same buffers
    [[maybe_unused]] const unsigned char *rscales = p.ref + sg.ref_byte_offset, *cscales = p.cand_table[blockIdx.x % p.num_candidates] + sg.ref_byte_offset;
    // an N-d segment: the rows above are those of one 2-D block; block (o0, o1) lies at its own offsets in both tensors
    const bool is_nd = seg_is_nd(sg) && p.nd != nullptr;
    SegNd outer{1, {1, 1}, {0, 0}, {0, 0}};
    if (is_nd) outer = p.nd[blockIdx.x / p.num_candidates];
    const u64 block_elems = outer.inner_rows * sg.row_elems;
    const u64 outer_elems[2] = {outer.outer_stride[0] / (u64)Traits<DT>::W, outer.outer_stride[1] / (u64)Traits<DT>::W};
    const u64 outer_ref_elems[2] = {outer.outer_ref_stride[0] / (u64)Traits<DT>::W, outer.outer_ref_stride[1] / (u64)Traits<DT>::W};
    u64 found = 0;
    for (u64 base = (u64)rec.first_mismatch; base < sg.numel && found < want; base += kReportThreads * kReportPerThread) {
        // all loads of the tile first, then the rule
        float av[kReportPerThread], bv[kReportPerThread];
        long long ai[kReportPerThread], bi[kReportPerThread];
#pragma unroll
        for (int u = 0; u < kReportPerThread; ++u) {
            const u64 i = base + (u64)u * kReportThreads + tid;
            const bool in = i < sg.numel;
            u64 j = (pitched && in) ? (i / sg.row_elems) * pitch_elems + i % sg.row_elems : i;     // where element i is stored
            u64 jr = (mapped && in) ? (i / sg.row_elems) * ref_pitch_elems + (i % sg.row_elems) * ref_stride : j;   // and what it is compared with
            if (is_nd && in) {
                const u64 block = i / block_elems, within = i % block_elems;             // row-major over (o0, o1, row, column)
                const u64 o0 = block / outer.outer_shape[1], o1 = block % outer.outer_shape[1];
                const u64 row = within / sg.row_elems, col = within % sg.row_elems;
                j = o0 * outer_elems[0] + o1 * outer_elems[1] + row * pitch_elems + col;
                jr = o0 * outer_ref_elems[0] + o1 * outer_ref_elems[1] + row * ref_pitch_elems + col * ref_stride;
            }
            if constexpr (DT == GEAK_I32) {
                ai[u] = in ? reinterpret_cast<const int *>(cb)[j] : 0;
                bi[u] = in ? reinterpret_cast<const int *>(rb)[jr] : 0;
            } else if constexpr (DT == GEAK_I64 || DT == GEAK_F64) {     // binary64 travels as its bit pattern
                ai[u] = in ? reinterpret_cast<const long long *>(cb)[j] : 0;
                bi[u] = in ? reinterpret_cast<const long long *>(rb)[jr] : 0;
            } else if constexpr (DT == GEAK_U8 || DT == GEAK_I8) {
                ai[u] = in ? load_elem_int(cb, j, DT) : 0;
                bi[u] = in ? load_elem_int(rb, jr, DT) : 0;
            } else if constexpr (kScaled<DT>) {             // the value: the code's times the scale of its block
                av[u] = in ? elem_f<DT>(cb, j) * scale_of_byte<DT>(cscales[j >> 5]) : 0.0f;
                bv[u] = in ? elem_f<DT>(rb, j) * scale_of_byte<DT>(rscales[j >> 5]) : 0.0f;
            } else {
                av[u] = in ? elem_f<DT>(cb, j) : 0.0f;
                bv[u] = in ? elem_f<DT>(rb, jr) : 0.0f;
            }
        }
        bool bad[kReportPerThread];
        int any = 0;
        uint32_t before[kReportPerThread];               // mismatches of lower lanes of this wave in row u
#pragma unroll
        for (int u = 0; u < kReportPerThread; ++u) {
            const u64 i = base + (u64)u * kReportThreads + tid;
            if constexpr (kIntegerDtype<DT>) bad[u] = (i < sg.numel) && ai[u] != bi[u];
            else if constexpr (DT == GEAK_F64)
                bad[u] = (i < sg.numel) && !close_exact_d(__builtin_bit_cast(double, ai[u]), __builtin_bit_cast(double, bi[u]),
                                                          tolerance.atol, tolerance.rtol, p.equal_nan);
            else bad[u] = (i < sg.numel) && !close_exact(av[u], bv[u], tolerance.atol_f, tolerance.rtol_f, p.equal_nan);
            const u64 mask = __builtin_amdgcn_ballot_w64(bad[u]);
            before[u] = (uint32_t)__builtin_popcountll(mask & ((1ull << lane) - 1ull));
            if (lane == 0) s_cnt[u][wave] = (uint32_t)__builtin_popcountll(mask);
            any |= bad[u];
        }
        if (!__syncthreads_or(any)) continue;                // a clean tile (the common case when mismatches are sparse)
        u64 rank = found;                                    // mismatches before row u
        u64 tile_total = 0;
#pragma unroll
        for (int u = 0; u < kReportPerThread; ++u) {
            uint32_t row_before = 0, row_total = 0;
#pragma unroll
            for (int w = 0; w < kReportThreads / kWaveSize; ++w) {
                const uint32_t c = s_cnt[u][w];
                row_before += (w < wave) ? c : 0u;
                row_total += c;
            }
            const u64 pos = rank + row_before + before[u];
            if (bad[u] && pos < want) {
                geak_mismatch m;
                m.index = (long long)(base + (u64)u * kReportThreads + tid);
                if constexpr (kIntegerDtype<DT>) {
                    m.a = (double)ai[u];                     // int64: one rounding each
                    m.b = (double)bi[u];
                    m.d = i64_abs_diff(ai[u], bi[u]);
                    m.tol = 0.0;
                } else if constexpr (DT == GEAK_F64) {
                    const double a = __builtin_bit_cast(double, ai[u]), b = __builtin_bit_cast(double, bi[u]);
                    const double prod = tolerance.rtol * __builtin_fabs(b);
                    m.a = a;
                    m.b = b;
                    m.d = __builtin_fabs(a - b);
                    m.tol = tolerance.atol + prod;
                } else {
                    const float prod = tolerance.rtol_f * __builtin_fabsf(bv[u]);
                    m.a = (double)av[u];
                    m.b = (double)bv[u];
                    m.d = (double)__builtin_fabsf(av[u] - bv[u]);
                    m.tol = (double)(tolerance.atol_f + prod);
                }
                out[pos] = m;
            }
            rank += row_total;
            tile_total += row_total;
        }
        found += tile_total;
        __syncthreads();                                     // the table is rewritten by the next tile
    }
}

__global__ __launch_bounds__(kReportThreads) void report_kernel(const ReportArgs p)
{
    __shared__ uint32_t s_cnt[kReportPerThread][kReportThreads / kWaveSize];
    const uint32_t K = p.num_candidates;
    const uint32_t seg = blockIdx.x / K, k = blockIdx.x % K;
    const geak_result rec = p.results[blockIdx.x];
    const u64 want = rec.mismatch_count < p.max_records ? rec.mismatch_count : (u64)p.max_records;
    if (threadIdx.x == 0) p.counts[blockIdx.x] = (uint32_t)want;
    if (want == 0) return;                                   // uniform
    const SegDesc sg = p.segments[seg];
    const SegTol tolerance = p.seg_tol[seg];
    const unsigned char *rb = p.ref + (seg_ref_mapped(sg) ? sg.ref_byte_offset : sg.byte_offset), *cb = p.cand_table[k] + sg.byte_offset;
    geak_mismatch *out = p.records + (u64)blockIdx.x * p.max_records;
    const auto report = [&](auto dt) { report_pair<decltype(dt)::value>(p, tolerance, sg, rec, want, rb, cb, out, s_cnt); };
    if (sg.dtype >= GEAK_MXFP8_E4M3) for_scaled_dtype(sg.dtype, report);          // uniform
    else for_dtype(sg.dtype, report);
}

// ---- read probe: what a kernel that only reads the same bytes achieves ---------------------------
// Every lane keeps eight 16-byte non-temporal loads in flight over a grid-stride walk of each buffer
// and folds what it reads into one word, which is stored only if it has a value it cannot have.
__global__ __launch_bounds__(256) void read_probe_kernel(const ProbeArgs p)
{
    const u64 vectors = p.bytes_each / 16;
    const u64 stride = (u64)gridDim.x * blockDim.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (uint32_t t = 0; t < p.num_buffers; ++t) {
        global_vec_ptr base = (global_vec_ptr)table_entry(p.buffers, t);
        u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
        for (; i + 7 * stride < vectors; i += 8 * stride) {
            u32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(base + i + u * stride);
#pragma unroll
            for (int u = 0; u < 8; ++u) acc ^= v[u];
        }
        for (; i < vectors; i += stride) acc ^= __builtin_nontemporal_load(base + i);
    }
    const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (x == 0x9E3779B9u && p.sink) p.sink[0] = x;       // keeps the loads alive; practically never taken
}

}  // namespace

int launch_report(const ReportArgs &args, void *stream)
{
    const uint64_t pairs = (uint64_t)args.num_segments * args.num_candidates;
    if (!pairs) return (int)hipSuccess;
    hipLaunchKernelGGL(report_kernel, dim3((uint32_t)pairs), dim3(kReportThreads), 0, (hipStream_t)stream, args);
    return (int)hipGetLastError();
}

int launch_read_probe(const ProbeArgs &args, uint32_t grid_blocks, void *stream)
{
    if (!args.num_buffers || args.bytes_each < 16) return (int)hipSuccess;
    hipLaunchKernelGGL(read_probe_kernel, dim3(grid_blocks), dim3(256), 0, (hipStream_t)stream, args);
    return (int)hipGetLastError();
}

int launch_init(const InitArgs &args, void *stream)
{
    uint64_t n = args.num_results > args.num_candidates ? args.num_results : args.num_candidates;
    if (args.num_board > n) n = args.num_board;
    if (!n) return (int)hipSuccess;
    const uint32_t threads = 256;
    uint64_t blocks = (n + threads - 1) / threads;
    const uint64_t need = ((args.num_results > args.num_candidates ? args.num_results : args.num_candidates) + threads - 1) / threads;
    if (blocks > 4096) blocks = 4096 > need ? 4096 : need;     // the board is zeroed with a grid-stride loop
    hipLaunchKernelGGL(init_kernel, dim3((uint32_t)blocks), dim3(threads), 0, (hipStream_t)stream, args);
    return (int)hipGetLastError();
}

int launch_compare(const CompareArgs &args, uint32_t grid_blocks, uint32_t lds_bytes, void *stream)
{
    if (!args.num_items) return (int)hipSuccess;
    hipLaunchKernelGGL(compare_kernel, dim3(grid_blocks), dim3(kBlockThreads), lds_bytes, (hipStream_t)stream, args);
    return (int)hipGetLastError();
}

int launch_reduce(const ReduceArgs &args, void *stream)
{
    const uint64_t pairs = (uint64_t)args.num_segments * args.num_candidates;
    if (!pairs) return (int)hipSuccess;
    // Few pairs: a block each, so that a pair's many slots are read by many threads.  Many pairs: a wave each.
    if (pairs < kReduceWavePairs) {
        hipLaunchKernelGGL(reduce_kernel, dim3((uint32_t)pairs), dim3(kReduceThreads), 0, (hipStream_t)stream, args);
    } else {
        const uint64_t per_block = kReduceThreads / kWaveSize;
        hipLaunchKernelGGL(reduce_wave_kernel, dim3((uint32_t)((pairs + per_block - 1) / per_block)), dim3(kReduceThreads), 0,
                           (hipStream_t)stream, args);
    }
    return (int)hipGetLastError();
}

int compare_blocks_per_cu(uint32_t lds_bytes)
{
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, compare_kernel, kBlockThreads, lds_bytes) != hipSuccess) return -1;
    return n;
}

}  // namespace geak
