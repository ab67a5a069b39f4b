// Device-side helpers shared by the kernel files: vector and address-space types, scalar reads of
// the plan's tables, per-dtype vector geometry, and the guarded 16-byte loads.
#pragma once
#include <hip/hip_runtime.h>
#include "geak_internal.hpp"

namespace geak {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;

constexpr float kInfF = __builtin_huge_valf();
constexpr double kInfD = __builtin_huge_val();

// Explicit address spaces.  Tables that are written before the kernel starts and never during it
// (work items, candidate base pointers) are read through the constant address space, so that a
// wave-uniform index turns into a scalar load instead of a vector load the wave has to wait for;
// tensor data is read through the global address space (no flat instructions).
#define GEAK_AS_GLOBAL   __attribute__((address_space(1)))
#define GEAK_AS_CONSTANT __attribute__((address_space(4)))
#define GEAK_AS_LDS      __attribute__((address_space(3)))
typedef const GEAK_AS_GLOBAL u32x4 *global_vec_ptr;

// A work item read with scalar loads (four 64-bit words; layout of geak_item).
__device__ __forceinline__ geak_item load_work_item(const geak_item *items, uint32_t j)
{
    static_assert(sizeof(geak_item) == 32, "geak_item is four 64-bit words");
    const GEAK_AS_CONSTANT unsigned long long *w = (const GEAK_AS_CONSTANT unsigned long long *)(items + j);
    const unsigned long long w2 = w[2], w3 = w[3];
    geak_item it;
    it.byte_offset = w[0];
    it.elem_start = w[1];
    it.segment = (uint32_t)w2;
    it.slot = (uint32_t)(w2 >> 32);
    it.numel = (uint16_t)w3;
    it.dtype = (uint8_t)(w3 >> 16);
    it.flags = (uint8_t)(w3 >> 24);
    it.next = (uint32_t)(w3 >> 32);
    return it;
}

__device__ __forceinline__ const unsigned char *table_entry(const unsigned char *const *table, uint32_t k)
{
    const GEAK_AS_CONSTANT unsigned long long *t = (const GEAK_AS_CONSTANT unsigned long long *)table;
    return reinterpret_cast<const unsigned char *>(t[k]);
}

// The range of the plan's block table that block `block` of a grid of `grid` blocks runs.  A grid that fills the
// chip is dispatched round by round: block b goes to XCD b mod 8 and there to compute unit u = b mod units, in
// round q = b / units (measured; the same in every run).
//   GEAK_MAP_PLAIN    range b.
//   GEAK_MAP_ROTATED  range q * units + g: the plain table, but within every stripe of eight ranges the XCDs take
//                     turns (g = u with its three low bits rotated by the three bits above them).  With range b
//                     every eighth range goes to the same XCD, whose addresses then differ from the other XCDs' in a
//                     few fixed bits; a bfloat16 tensor of 2^28 elements ran 2.5 % slower that way.
//   GEAK_MAP_BY_UNIT  range g * (grid / units) + q: the planner laid the ranges of the blocks that share a compute
//                     unit side by side (group g of the table belongs to one unit), the XCDs rotated as above --
//                     unrotated, dense tensors ran 5 - 15 % slower in this layout.
__device__ __forceinline__ uint32_t table_range_of_block(uint32_t block, uint32_t grid, uint32_t units, uint32_t block_map)
{
    if (block_map == GEAK_MAP_PLAIN || units <= 1) return block;
    const uint32_t unit = block % units, round = block / units;
    const uint32_t group = unit ^ ((unit >> 3) & 7u);
    return block_map == GEAK_MAP_BY_UNIT ? group * (grid / units) + round : round * units + group;
}

// A segment's tolerances, read with scalar loads when the segment index is wave-uniform.
__device__ __forceinline__ SegTol load_tol(const SegTol *table, uint32_t segment)
{
    const GEAK_AS_CONSTANT unsigned long long *t = (const GEAK_AS_CONSTANT unsigned long long *)(table + segment);
    const unsigned long long w = t[0];
    SegTol out;
    out.atol_f = __builtin_bit_cast(float, (uint32_t)w);
    out.rtol_f = __builtin_bit_cast(float, (uint32_t)(w >> 32));
    out.atol = __builtin_bit_cast(double, t[1]);
    out.rtol = __builtin_bit_cast(double, t[2]);
    return out;
}

template <int DT> struct Traits;
template <> struct Traits<GEAK_F32>  { static constexpr int E = 4, W = 4; };
template <> struct Traits<GEAK_F16>  { static constexpr int E = 8, W = 2; };
template <> struct Traits<GEAK_BF16> { static constexpr int E = 8, W = 2; };
template <> struct Traits<GEAK_I32>  { static constexpr int E = 4, W = 4; };
template <> struct Traits<GEAK_I64>  { static constexpr int E = 2, W = 8; };
template <> struct Traits<GEAK_U8>   { static constexpr int E = 16, W = 1; };
template <> struct Traits<GEAK_I8>   { static constexpr int E = 16, W = 1; };
template <> struct Traits<GEAK_F64>  { static constexpr int E = 2, W = 8; };
template <> struct Traits<GEAK_F8E4M3> { static constexpr int E = 16, W = 1; };
template <> struct Traits<GEAK_F8E5M2> { static constexpr int E = 16, W = 1; };
template <> struct Traits<GEAK_MXFP8_E4M3> { static constexpr int E = 16, W = 1; };
template <> struct Traits<GEAK_MXFP8_E5M2> { static constexpr int E = 16, W = 1; };
template <> struct Traits<GEAK_MXINT8>     { static constexpr int E = 16, W = 1; };
// The four-bit format never reaches the arithmetic as such: the loads rewrite sixteen E2M1 codes (8 bytes) as the
// sixteen E4M3 byte codes of the same values, so a lane's "vector" is sixteen elements here too.
template <> struct Traits<GEAK_MXFP4_E2M1> { static constexpr int E = 16, W = 1; };
// The same for the six-bit formats: sixteen codes (12 bytes) become sixteen E4M3 byte codes (every E2M3 and E3M2
// value is an E4M3 value).
template <> struct Traits<GEAK_MXFP6_E2M3> { static constexpr int E = 16, W = 1; };
template <> struct Traits<GEAK_MXFP6_E3M2> { static constexpr int E = 16, W = 1; };
// Block-scaled element formats: a 16-byte vector holds half a block of 32 elements, so one scale byte
// belongs to every vector.
template <int DT> constexpr bool kScaled = (DT == GEAK_MXFP8_E4M3 || DT == GEAK_MXFP8_E5M2 || DT == GEAK_MXINT8 || DT == GEAK_MXFP4_E2M1 ||
                                           DT == GEAK_MXFP6_E2M3 || DT == GEAK_MXFP6_E3M2);
// formats whose loads rewrite sub-byte codes as E4M3 byte codes
template <int DT> constexpr bool kFp6 = (DT == GEAK_MXFP6_E2M3 || DT == GEAK_MXFP6_E3M2);
template <int DT> constexpr bool kSubByte = (DT == GEAK_MXFP4_E2M1 || kFp6<DT>);

__device__ __forceinline__ float bits_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ double bits_d(uint32_t lo, uint32_t hi) { return __builtin_bit_cast(double, (u64)lo | ((u64)hi << 32)); }
__device__ __forceinline__ uint32_t f_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// Element e (0 .. E-1) of a 16-byte vector, decoded exactly to binary32.
template <int DT>
__device__ __forceinline__ float decode(const u32x4 &q, int e)
{
    if constexpr (DT == GEAK_F32) {
        return bits_f(q[e]);
    } else if constexpr (DT == GEAK_F16) {
        const uint32_t word = q[e >> 1];
        const uint16_t h = (e & 1) ? (uint16_t)(word >> 16) : (uint16_t)(word & 0xFFFFu);
        return (float)__builtin_bit_cast(_Float16, h);
    } else {  // bf16: upper half of a binary32
        const uint32_t word = q[e >> 1];
        return bits_f((e & 1) ? (word & 0xFFFF0000u) : (word << 16));
    }
}

// ---- loads -------------------------------------------------------------------------------------
// Elements [lo, valid) of the 16-byte vector at p, the rest 0.  With p on a 16-byte boundary (the
// tensor's base pointer is 16-byte aligned) a vector that holds any element of the item is loaded
// whole and the bytes of the other elements are cleared: the vector is one aligned 16-byte granule
// of the buffer, so it lies in the same page as the item's own bytes in it and the load touches
// nothing the item's bytes do not already map.  With p off the grid (a base pointer that is only
// element-aligned, such as a slice of a larger tensor) a vector that lies wholly inside the item is
// still one 16-byte load -- the hardware takes global loads at any address -- and a vector that holds
// only part of the item is read byte by byte.  A vector without any element of the item is not loaded
// at all.
// Bytes [first_byte, end_byte) of the vector kept, the others cleared.
__device__ __forceinline__ u32x4 cut_vector_inline(u32x4 q, const int first_byte, const int end_byte)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int keep_from = first_byte - 4 * j, keep_to = end_byte - 4 * j;          // relative to word j
        const uint32_t below_to = keep_to <= 0 ? 0u : (keep_to >= 4 ? 0xFFFFFFFFu : (1u << (8 * keep_to)) - 1u);
        const uint32_t below_from = keep_from <= 0 ? 0u : (keep_from >= 4 ? 0xFFFFFFFFu : (1u << (8 * keep_from)) - 1u);
        q[j] &= below_to & ~below_from;
    }
    return q;
}
__device__ __noinline__ u32x4 cut_vector_call(const u32x4 q, const int first_byte, const int end_byte)
{
    return cut_vector_inline(q, first_byte, end_byte);
}

// Bytes [first_byte, end_byte) of the 16 bytes at p, read one by one, the others 0: for a vector that holds
// only part of an item in a tensor whose base pointer is not 16-byte aligned.  There the vector is no
// aligned granule, may straddle a page, and nothing outside the item's own bytes may be touched.  Rare
// (the first and last vector of an item that is not a full one, in such a tensor only): a real function.
__device__ __noinline__ u32x4 load_bytes_call(const GEAK_AS_GLOBAL unsigned char *p, const int first_byte, const int end_byte)
{
    u32x4 q = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int b = 0; b < 16; ++b)
        if (b >= first_byte && b < end_byte) q[b >> 2] |= (uint32_t)p[b] << (8 * (b & 3));
    return q;
}

template <int DT>
__device__ __forceinline__ u32x4 load_partial_from(global_vec_ptr p, uint32_t lo, uint32_t valid)
{
    constexpr uint32_t E = Traits<DT>::E, W = Traits<DT>::W;
    u32x4 q = {0u, 0u, 0u, 0u};
    const bool partial = valid > lo && (lo != 0 || valid < E);
    const bool off_grid = ((uint32_t)reinterpret_cast<u64>(p) & 15u) != 0;       // a property of the tensor's base (and, for a mapped reference, of its rows' pitch)
    if (valid > lo && !(partial && off_grid)) q = __builtin_nontemporal_load(p);
    if (__builtin_amdgcn_ballot_w64(partial && off_grid)) {
        if (partial && off_grid)
            q = load_bytes_call((const GEAK_AS_GLOBAL unsigned char *)p, (int)(lo * W), (int)((valid < E ? valid : E) * W));
    }
    // The wave branches around the cut as a whole (in a tail only one lane of the last vector needs
    // it); inside, a lane whose vector is whole keeps all of it.  The routines of the 16-bit dtypes
    // have no registers to spare, so there the cut is a call.
    if (__builtin_amdgcn_ballot_w64(valid > lo && (lo != 0 || valid < E))) {
        const int first_byte = (int)(lo * W), end_byte = (int)((valid < E ? valid : E) * W);
        if constexpr (E == 8) q = cut_vector_call(q, first_byte, end_byte);
        else q = cut_vector_inline(q, first_byte, end_byte);
    }
    return q;
}
template <int DT>
__device__ __forceinline__ u32x4 load_partial(global_vec_ptr p, uint32_t valid)
{
    return load_partial_from<DT>(p, 0u, valid);
}

// Vector V of lane L of an item that starts 16-byte aligned but may be shorter than a full item
// (a segment's tail): whole vectors inside the item are loaded as such, the one vector that
// straddles the end is loaded and cut, vectors past the end are not loaded, and everything past the
// end reads as 0 -- in the reference and in every candidate alike, so that those positions compare
// as close and add nothing to either maximum.
// Sixteen E2M1 codes -- two per byte, the even element in the low nibble: the 64 bits {lo, hi} -- rewritten as
// the sixteen E4M3 byte codes of the same values (0, 0.5, 1, 1.5, 2, 3, 4, 6 are 0x00, 0x30, 0x38, 0x3C, 0x40, 0x44,
// 0x48, 0x4C; bit 3 of a nibble is the sign): the nibbles of 16 bits are spread into four bytes, and one byte permute
// looks all four magnitudes up.
__device__ __forceinline__ uint32_t e2m1_four(uint32_t h16)
{
    const uint32_t t = (h16 | (h16 << 8)) & 0x00FF00FFu;
    const uint32_t u = (t | (t << 4)) & 0x0F0F0F0Fu;
    const uint32_t code = __builtin_amdgcn_perm(0x4C484440u, 0x3C383000u, u & 0x07070707u);     // selector i: byte i of the table
    return code | ((u & 0x08080808u) << 4);
}
__device__ __forceinline__ u32x4 expand_e2m1(uint32_t lo, uint32_t hi)
{
    u32x4 q;
    q[0] = e2m1_four(lo & 0xFFFFu); q[1] = e2m1_four(lo >> 16);
    q[2] = e2m1_four(hi & 0xFFFFu); q[3] = e2m1_four(hi >> 16);
    return q;
}
// Slot `slot` of an item of the four-bit format: 8 bytes of payload, as sixteen byte codes.
__device__ __forceinline__ u32x4 load_e2m1_slot(const unsigned char *base, uint32_t slot)
{
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 w = __builtin_nontemporal_load((const GEAK_AS_GLOBAL u32x2 *)base + slot);
    return expand_e2m1(w[0], w[1]);
}

// Four six-bit codes, one in the low bits of each byte of u (bit 5 the sign), as the E4M3 byte codes of the same values.
//   E2M3 (bias 1): magnitude code c = e e m m m.  c >= 8: 2^(e-1) * (1 + m/8), E4M3 exponent field e + 6, the same
//                  mantissa: code c + 0x30.  c < 8: the subnormal c / 8 = 0, 2^-3, 2^-2, 1.5 * 2^-2, 2^-1, 1.25 * 2^-1,
//                  1.5 * 2^-1, 1.75 * 2^-1: codes 0x00, 0x20, 0x28, 0x2C, 0x30, 0x32, 0x34, 0x36 (a byte-permute table).
//   E3M2 (bias 3): c = e e e m m.  c >= 4: 2^(e-3) * (1 + m/4), exponent field e + 4, mantissa m0: code 2 c + 0x20.
//                  c < 4: c / 16 = 0, 2^-4, 2^-3, 1.5 * 2^-3: codes 0x00, 0x18, 0x20, 0x24.
template <int DT>
__device__ __forceinline__ uint32_t fp6_four(uint32_t u)
{
    constexpr uint32_t kLeastNormal = DT == GEAK_MXFP6_E2M3 ? 8u : 4u;
    const uint32_t mag = u & 0x1F1F1F1Fu;
    const uint32_t top = (mag + (0x80u - kLeastNormal) * 0x01010101u) & 0x80808080u;      // bit 7 of a byte: its code is a normal number's
    const uint32_t normal_bytes = (top - (top >> 7)) | top;                              // 0xFF in those bytes
    uint32_t normal, subnormal;
    if constexpr (DT == GEAK_MXFP6_E2M3) {
        normal = mag + 0x30303030u;
        subnormal = __builtin_amdgcn_perm(0x36343230u, 0x2C282000u, mag & 0x07070707u);     // selector i: byte i of the table
    } else {
        normal = (mag << 1) + 0x20202020u;                                                  // mag <= 31: no bit leaves its byte
        subnormal = __builtin_amdgcn_perm(0u, 0x24201800u, mag & 0x03030303u);
    }
    const uint32_t code = (normal & normal_bytes) | (subnormal & ~normal_bytes);
    return code | ((u & 0x20202020u) << 2);
}
// Sixteen six-bit codes -- element i in bits 6 i .. 6 i + 5 of the 96 bits {w0, w1, w2} -- as sixteen E4M3 byte codes.
template <int DT>
__device__ __forceinline__ u32x4 expand_fp6(uint32_t w0, uint32_t w1, uint32_t w2)
{
    // elements 4 j .. 4 j + 3 are the 24 bits from bit 24 j on
    const uint32_t x[4] = {w0, __builtin_amdgcn_alignbit(w1, w0, 24), __builtin_amdgcn_alignbit(w2, w1, 16), w2 >> 8};
    u32x4 q;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t spread = (x[j] & 0x3Fu) | ((x[j] << 2) & 0x3F00u) | ((x[j] << 4) & 0x3F0000u) | ((x[j] << 6) & 0x3F000000u);
        q[j] = fp6_four<DT>(spread);
    }
    return q;
}
// Slot `slot` of an item of a six-bit format: 12 bytes of payload (on a 4-byte boundary), as sixteen byte codes.
template <int DT>
__device__ __forceinline__ u32x4 load_fp6_slot(const unsigned char *base, uint32_t slot)
{
    const GEAK_AS_GLOBAL uint32_t *w = (const GEAK_AS_GLOBAL uint32_t *)(base + (u64)slot * 12u);
    const uint32_t w0 = __builtin_nontemporal_load(w), w1 = __builtin_nontemporal_load(w + 1), w2 = __builtin_nontemporal_load(w + 2);
    return expand_fp6<DT>(w0, w1, w2);
}
// A slot of a format narrower than a byte.
template <int DT>
__device__ __forceinline__ u32x4 load_sub_byte_slot(const unsigned char *base, uint32_t slot)
{
    if constexpr (kFp6<DT>) return load_fp6_slot<DT>(base, slot);
    else return load_e2m1_slot(base, slot);
}

template <int DT>
__device__ __forceinline__ u32x4 load_vec(const unsigned char *base, int lane, int v, uint32_t n, bool full)
{
    constexpr uint32_t E = Traits<DT>::E;
    if constexpr (kSubByte<DT>) {                       // whole blocks only: a slot is inside the item or behind it
        const uint32_t slot = (uint32_t)(v * kWaveSize + lane);
        if (full || slot * E < n) return load_sub_byte_slot<DT>(base, slot);
        return u32x4{0u, 0u, 0u, 0u};
    }
    global_vec_ptr p = (global_vec_ptr)base + (v * kWaveSize + lane);
    if (full) return __builtin_nontemporal_load(p);
    const uint32_t first = (uint32_t)(v * kWaveSize + lane) * E;
    return load_partial<DT>(p, first < n ? n - first : 0u);
}

// Where the vectors of an item that is not a full one lie; three kinds.
//   plain    a tail: starts on a 16-byte boundary, contiguous, vector slot i at byte 16 i.
//   rows     a row group (GEAK_ITEM_ROWS: several short rows of a pitched segment, each starting on a
//            16-byte boundary): every row takes `vpr` slots, the last of them partial when the row's bytes
//            are no multiple of 16, and row r lies at byte r * pitch; slot i is vector i % vpr of row i / vpr.
//   shifted  an item that starts off the 16-byte grid (GEAK_ITEM_ALIGNED not set): read from the
//            boundary before it, so that slot 0 holds `skip` foreign elements in front, which read as 0
//            like everything behind the item's end.
// In all three the slots ascend with the element index.  All fields wave-uniform.
enum TailKind { kTailPlain = 0, kTailRows = 1, kTailShifted = 2 };
struct ItemShape {
    uint32_t rows;          // rows: their number
    uint32_t vpr;           // rows: vectors per row
    uint32_t inv;           // rows: ceil(2^16 / vpr): (i * inv) >> 16 == i / vpr for i < 256
    uint32_t row_elems;     // rows
    u64 pitch;              // rows: bytes from one row to the next
    uint32_t skip;          // shifted: elements between the 16-byte boundary and the item's first
};

template <int DT, int KIND>
__device__ __forceinline__ ItemShape item_shape(const geak_item &it, const SegDesc *segments)
{
    ItemShape sh{0u, 1u, 0u, 0u, 0ull, 0u};
    if constexpr (KIND == kTailRows) {
        const GEAK_AS_CONSTANT unsigned long long *g = (const GEAK_AS_CONSTANT unsigned long long *)(segments + it.segment);
        sh.row_elems = (uint32_t)g[2];                    // SegDesc: byte_offset, numel, row_elems, pitch_bytes, ...
        sh.pitch = g[3];
        sh.vpr = (sh.row_elems + Traits<DT>::E - 1) / Traits<DT>::E;
        sh.inv = (65536u + sh.vpr - 1u) / sh.vpr;
        sh.rows = (uint32_t)it.numel / sh.row_elems;
    } else if constexpr (KIND == kTailShifted) {
        sh.skip = ((uint32_t)it.byte_offset & 15u) / (uint32_t)Traits<DT>::W;
    }
    return sh;
}

// Number of vector slots per lane (1 .. 4) that an item of this shape with n elements occupies.
template <int DT>
__device__ __forceinline__ uint32_t shape_vectors(const ItemShape &sh, uint32_t n)
{
    const uint32_t slots = sh.rows ? sh.rows * sh.vpr : (sh.skip + n + Traits<DT>::E - 1) / Traits<DT>::E;
    return (slots + kWaveSize - 1) / kWaveSize;
}

// Vector slot `slot` (= v * 64 + lane) of an item of n elements whose first slot lies at `base` (for
// a shifted item: the boundary before its first element).  `first`: index within the item of the
// slot's element 0 (meaningless when nothing is valid; for slot 0 of a shifted item it wraps below
// zero, and first + e is right again for every valid e).
struct SlotPlace {
    uint32_t row, vec;       // the slot is vector `vec` of row `row` (one row unless the item is a row group)
    uint32_t lo, valid;      // elements [lo, valid) of the vector belong to the item (valid may exceed the vector)
    uint32_t first;          // see above
};
template <int DT, int KIND>
__device__ __forceinline__ SlotPlace slot_place(uint32_t slot, uint32_t n, const ItemShape &sh)
{
    constexpr uint32_t E = Traits<DT>::E;
    if constexpr (KIND == kTailRows) {
        const uint32_t row = (slot * sh.inv) >> 16, vec = slot - row * sh.vpr, col = vec * E;
        return SlotPlace{row, vec, 0u, row < sh.rows ? sh.row_elems - col : 0u, row * sh.row_elems + col};   // col < row_elems by construction of vpr
    } else if constexpr (KIND == kTailShifted) {
        const uint32_t end = sh.skip + n;                                  // in slot positions
        return SlotPlace{0u, slot, slot == 0 ? sh.skip : 0u, slot * E < end ? end - slot * E : 0u, slot * E - sh.skip};
    } else {
        return SlotPlace{0u, slot, 0u, slot * E < n ? n - slot * E : 0u, slot * E};
    }
}
template <int DT, int KIND>
__device__ __forceinline__ u32x4 load_slot(const unsigned char *base, uint32_t slot, uint32_t n, const ItemShape &sh, uint32_t &first)
{
    const SlotPlace sp = slot_place<DT, KIND>(slot, n, sh);
    first = sp.first;
    if constexpr (kSubByte<DT>) {                       // plain tails of whole blocks only
        if (sp.valid > 0) return load_sub_byte_slot<DT>(base, sp.vec);
        return u32x4{0u, 0u, 0u, 0u};
    }
    if constexpr (KIND == kTailRows) return load_partial_from<DT>((global_vec_ptr)(base + (u64)sp.row * sh.pitch) + sp.vec, sp.lo, sp.valid);
    else return load_partial_from<DT>((global_vec_ptr)base + sp.vec, sp.lo, sp.valid);
}

// Where the reference's elements of an item lie when the segment's reference has a layout of its own
// (GEAK_ITEM_REFMAP): the candidates' slots keep their shape, the reference's rows have their own pitch
// -- possibly 0: one row for all -- and either lie as the candidates' rows do or hold one element that
// every element of the row is compared with.  All fields wave-uniform.
struct RefPlace {
    u64 offset;              // byte offset in the reference buffer of what the item's first element is compared with
    u64 pitch;               // bytes between the reference's rows
    uint32_t stride;         // elements between neighbours of a reference row: 1 contiguous, 0 one element per row
};
template <int DT>
__device__ __forceinline__ RefPlace ref_place(const geak_item &it, uint32_t item_index, const SegDesc *segments, const uint64_t *ref_item_offset)
{
    const GEAK_AS_CONSTANT unsigned long long *g = (const GEAK_AS_CONSTANT unsigned long long *)(segments + it.segment);
    const GEAK_AS_CONSTANT unsigned long long *t = (const GEAK_AS_CONSTANT unsigned long long *)ref_item_offset;
    // SegDesc: byte_offset, numel, row_elems, pitch_bytes, {dtype, layout}, ref_byte_offset, ref_pitch_bytes
    return RefPlace{t[item_index], g[6], (uint32_t)(g[4] >> 32) >> kRefStrideShift};
}
// Elements [lo, hi) of a 16-byte vector gathered one by one: element e from `first` + e * stride_bytes, the others 0.
// The reference of a segment whose reference row is strided (a transposed reference, a column of a wider
// matrix); rare and slow by nature: a real function.
template <int DT>
__device__ __noinline__ u32x4 gather_elements_call(const unsigned char *first, const u64 stride_bytes, const uint32_t lo, const uint32_t hi)
{
    constexpr int E = Traits<DT>::E, W = Traits<DT>::W;
    u32x4 q = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < E; ++e) {
        if ((uint32_t)e < lo || (uint32_t)e >= hi) continue;
        const GEAK_AS_GLOBAL unsigned char *p = (const GEAK_AS_GLOBAL unsigned char *)(first + (u64)e * stride_bytes);
        if constexpr (W == 1) q[e >> 2] |= (uint32_t)p[0] << (8 * (e & 3));
        else if constexpr (W == 2) q[e >> 1] |= (uint32_t)*(const GEAK_AS_GLOBAL uint16_t *)p << (16 * (e & 1));
        else if constexpr (W == 4) q[e] = *(const GEAK_AS_GLOBAL uint32_t *)p;
        else { q[2 * e] = ((const GEAK_AS_GLOBAL uint32_t *)p)[0]; q[2 * e + 1] = ((const GEAK_AS_GLOBAL uint32_t *)p)[1]; }
    }
    return q;
}
// A 16-byte vector filled with the one element at `at`.
template <int DT>
__device__ __forceinline__ u32x4 splat_element(const unsigned char *at)
{
    constexpr uint32_t W = Traits<DT>::W;
    const GEAK_AS_GLOBAL unsigned char *one = (const GEAK_AS_GLOBAL unsigned char *)at;
    uint32_t w0, w1 = 0u;
    if constexpr (W == 1) { w0 = *one; w0 |= w0 << 8; w0 |= w0 << 16; w1 = w0; }
    else if constexpr (W == 2) { w0 = *(const GEAK_AS_GLOBAL uint16_t *)one; w0 |= w0 << 16; w1 = w0; }
    else if constexpr (W == 4) { w0 = *(const GEAK_AS_GLOBAL uint32_t *)one; w1 = w0; }
    else { w0 = ((const GEAK_AS_GLOBAL uint32_t *)one)[0]; w1 = ((const GEAK_AS_GLOBAL uint32_t *)one)[1]; }
    return u32x4{w0, w1, w0, w1};
}
// Vector slot `slot` of the reference side of such an item: the elements that the same slot of a
// candidate is compared with, zero where the candidate's slot reads as zero.
template <int DT, int KIND>
__device__ __forceinline__ u32x4 load_ref_slot(const unsigned char *ref_base, const RefPlace &rp, uint32_t slot, uint32_t n, const ItemShape &sh,
                                               uint32_t &first)
{
    constexpr uint32_t E = Traits<DT>::E, W = Traits<DT>::W;
    const SlotPlace sp = slot_place<DT, KIND>(slot, n, sh);
    first = sp.first;
    const unsigned char *row = ref_base + rp.offset + (u64)sp.row * rp.pitch;
    if (rp.stride == 1) {
        // a shifted item's slot 0 starts `skip` elements before the item: so does the reference's (those are not read
        // unless they share an aligned 16-byte granule with the item's own)
        if constexpr (KIND == kTailShifted) row -= (u64)sh.skip * W;
        return load_partial_from<DT>((global_vec_ptr)row + sp.vec, sp.lo, sp.valid);
    }
    u32x4 q = {0u, 0u, 0u, 0u};
    if (rp.stride != 0) {
        // column of the slot's element 0 within its row (for slot 0 of a shifted item it lies before the item's first
        // element: only elements from `lo` on are touched)
        long long col = (long long)sp.vec * E;
        if constexpr (KIND == kTailShifted) col -= sh.skip;
        if (__builtin_amdgcn_ballot_w64(sp.valid > sp.lo)) {
            if (sp.valid > sp.lo)
                q = gather_elements_call<DT>(row + col * (long long)((u64)rp.stride * W), (u64)rp.stride * W, sp.lo, sp.valid < E ? sp.valid : E);
        }
        return q;
    }
    if (sp.valid > sp.lo) {
        q = splat_element<DT>(row);                                                                 // the row's one element
        if (sp.lo != 0 || sp.valid < E) q = cut_vector_call(q, (int)(sp.lo * W), (int)((sp.valid < E ? sp.valid : E) * W));
    }
    return q;
}
// Vector v of this lane.
template <int DT, int KIND>
__device__ __forceinline__ u32x4 load_shaped(const unsigned char *base, int lane, int v, uint32_t n, const ItemShape &sh)
{
    uint32_t first;
    return load_slot<DT, KIND>(base, (uint32_t)(v * kWaveSize + lane), n, sh, first);
}

// The 8-bit floating formats are widened by the conversion instructions (v_cvt_f32_fp8 for E4M3,
// v_cvt_f32_bf8 for E5M2), which on gfx950 implement the OCP formats: NaN and, for E5M2, the
// infinities arrive as such.  BYTE selects the byte of the word.
template <int DT, int BYTE>
__device__ __forceinline__ float f8_to_f32(uint32_t word)
{
    if constexpr (DT == GEAK_F8E4M3 || DT == GEAK_MXFP8_E4M3 || kSubByte<DT>) return __builtin_amdgcn_cvt_f32_fp8((int)word, BYTE);
    else if constexpr (DT == GEAK_MXINT8) return (float)((int)(word << (24 - 8 * BYTE)) >> 24);     // the code as an integer; the scale carries the 1/64
    else return __builtin_amdgcn_cvt_f32_bf8((int)word, BYTE);
}

// Two neighbouring bytes of the word (the low pair, or with HI the high pair) widened by one instruction.
struct F32Pair { float lo, hi; };
template <int DT, bool HI>
__device__ __forceinline__ F32Pair f8_pair_to_f32(uint32_t word)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    if constexpr (DT == GEAK_MXINT8) {
        return F32Pair{f8_to_f32<DT, HI ? 2 : 0>(word), f8_to_f32<DT, HI ? 3 : 1>(word)};
    } else {
        f32x2 v;
        if constexpr (DT == GEAK_F8E4M3 || DT == GEAK_MXFP8_E4M3 || kSubByte<DT>) v = __builtin_amdgcn_cvt_pk_f32_fp8((int)word, HI);
        else v = __builtin_amdgcn_cvt_pk_f32_bf8((int)word, HI);
        return F32Pair{v[0], v[1]};
    }
}

// The factor a scale byte X stands for, as binary32: 2^(X - 127), NaN for X = 0xFF.  2^-127 is a binary32
// subnormal.  For the integer element format the element's own 2^-6 is folded in (2^(X - 133), subnormal for
// X <= 6); multiplying the code's integer value by it is exact.
template <int DT>
__device__ __forceinline__ float scale_of_byte(uint32_t x)
{
    constexpr int kFold = DT == GEAK_MXINT8 ? 6 : 0;
    const int e = (int)x - 127 - kFold;                                       // -133 .. 127
    const uint32_t bits = e >= -126 ? (uint32_t)(e + 127) << 23 : 1u << (e + 149);
    return bits_f(x == 0xFFu ? 0x7FC00000u : bits);
}
// The scale byte of vector slot `slot` (= v * 64 + lane) of an item of n elements whose first block's scale
// lies at `scales`: sixteen elements per vector, two vectors per block.  A slot behind the item's end has no
// elements (they read as 0 in every tensor) and gets the byte of 2^0.
__device__ __forceinline__ uint32_t load_scale_byte(const unsigned char *scales, uint32_t slot, uint32_t n)
{
    return slot * 16u < n ? (uint32_t)((const GEAK_AS_GLOBAL unsigned char *)scales)[slot >> 1] : 127u;
}
// Byte offset in every packed buffer of the scale of an item's first block: the segment's scales begin at the
// record's sixth word, one byte per block of 32 elements (items of such segments start on block boundaries).
__device__ __forceinline__ u64 item_scale_offset(const geak_item &it, const SegDesc *segments)
{
    const GEAK_AS_CONSTANT unsigned long long *g = (const GEAK_AS_CONSTANT unsigned long long *)(segments + it.segment);
    return g[5] + (it.elem_start >> 5);
}

// One integer element straight from memory, widened exactly to 64 bits.
__device__ __forceinline__ long long load_elem_int(const unsigned char *base, u64 idx, int dtype)
{
    if (dtype == GEAK_I32) return reinterpret_cast<const int *>(base)[idx];
    if (dtype == GEAK_I64) return reinterpret_cast<const long long *>(base)[idx];
    if (dtype == GEAK_U8) return base[idx];
    return reinterpret_cast<const signed char *>(base)[idx];
}

// Compile-time loop: f is called with Index<0>, Index<1>, ... so that the index can select a register
// or an instruction's byte selector.
template <int I> struct Index { static constexpr int value = I; };
template <int N, typename F, int I = 0>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(Index<I>{});
        static_for<N, F, I + 1>(static_cast<F &&>(f));
    }
}

// Calls f(Index<DT>{}) for the dtype code `dtype` (validated when the plan is built): the one place
// where a run-time dtype selects a routine's instantiation.
template <typename F>
__device__ __forceinline__ void for_dtype(int dtype, F &&f)
{
    switch (dtype) {
    case GEAK_F32:    f(Index<GEAK_F32>{}); break;
    case GEAK_F16:    f(Index<GEAK_F16>{}); break;
    case GEAK_BF16:   f(Index<GEAK_BF16>{}); break;
    case GEAK_I32:    f(Index<GEAK_I32>{}); break;
    case GEAK_I64:    f(Index<GEAK_I64>{}); break;
    case GEAK_U8:     f(Index<GEAK_U8>{}); break;
    case GEAK_I8:     f(Index<GEAK_I8>{}); break;
    case GEAK_F64:    f(Index<GEAK_F64>{}); break;
    case GEAK_F8E4M3: f(Index<GEAK_F8E4M3>{}); break;
    default:          f(Index<GEAK_F8E5M2>{}); break;
    }
}

// The same for the element formats of block-scaled segments.
template <typename F>
__device__ __forceinline__ void for_scaled_dtype(int dtype, F &&f)
{
    switch (dtype) {
    case GEAK_MXFP8_E4M3: f(Index<GEAK_MXFP8_E4M3>{}); break;
    case GEAK_MXFP8_E5M2: f(Index<GEAK_MXFP8_E5M2>{}); break;
    case GEAK_MXFP4_E2M1: f(Index<GEAK_MXFP4_E2M1>{}); break;
    case GEAK_MXFP6_E2M3: f(Index<GEAK_MXFP6_E2M3>{}); break;
    case GEAK_MXFP6_E3M2: f(Index<GEAK_MXFP6_E3M2>{}); break;
    default:              f(Index<GEAK_MXINT8>{}); break;
    }
}

}  // namespace
}  // namespace geak
