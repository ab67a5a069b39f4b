// Internal definitions shared by the host planner, the API layer and the kernels.
#pragma once
#include <cstdint>
#include <vector>
#include "geak_check.h"

namespace geak {

constexpr int kWaveSize = 64;
constexpr int kVecPerLane = 4;                                   // 16-byte vectors per lane, per tensor, per item
constexpr int kItemBytes = kVecPerLane * kWaveSize * 16;         // 4096 bytes of each tensor per work item
constexpr int kWavesPerBlock = 4;
constexpr int kBlockThreads = kWavesPerBlock * kWaveSize;
constexpr int kDefaultComputeUnits = 256;                        // host-only plans
constexpr int kDefaultBlocksPerCU = 4;
constexpr uint32_t kNoItem = 0xFFFFFFFFu;

inline int elem_size(int dtype)
{
    switch (dtype) {
    case GEAK_F16: case GEAK_BF16: return 2;
    case GEAK_I64: case GEAK_F64: return 8;
    case GEAK_U8: case GEAK_I8: case GEAK_F8E4M3: case GEAK_F8E5M2: return 1;
    case GEAK_MXFP8_E4M3: case GEAK_MXFP8_E5M2: case GEAK_MXINT8: return 1;       // the payload's elements
    case GEAK_MXFP4_E2M1: case GEAK_MXFP6_E2M3: case GEAK_MXFP6_E3M2: return 1;   // nominal: narrower than a byte (payload_bytes)
    default: return 4;
    }
}

// Bytes that n elements of a dtype occupy (n a multiple of 2 for the four-bit format, of 4 for the six-bit ones),
// and elements of one full work item.
inline bool is_fp6_dtype(int dtype) { return dtype == GEAK_MXFP6_E2M3 || dtype == GEAK_MXFP6_E3M2; }
inline uint64_t payload_bytes(int dtype, uint64_t n)
{
    return dtype == GEAK_MXFP4_E2M1 ? n / 2 : is_fp6_dtype(dtype) ? n / 4 * 3 : n * (uint64_t)elem_size(dtype);
}
inline uint64_t elems_per_item(int dtype)
{
    // the four- and six-bit codes are rewritten as byte codes when they are loaded: an item is 4096 of them, 2 KiB
    // and 3 KiB of payload
    return (dtype == GEAK_MXFP4_E2M1 || is_fp6_dtype(dtype)) ? (uint64_t)kItemBytes : (uint64_t)kItemBytes / (uint64_t)elem_size(dtype);
}

// Partial result of one (worker, segment) run for one candidate; 16 bytes.
struct Partial {
    unsigned long long count;   // mismatching elements seen by the run
    uint32_t first_item;        // least item index of the run that holds a mismatch, kNoItem if none
    uint32_t reserved;
};

// LDS of one block: per wave and candidate a 64-bit count and a 32-bit first-item index (rounded
// up to 16 bytes in total), then per wave a region for the staged tolerances of a 16-bit slice
// (2048 elements x 4 bytes).
constexpr uint32_t kTolBytesPerWave = kItemBytes / 2 * 4;
constexpr uint32_t lds_state_bytes(int num_candidates) {
    return ((uint32_t)(kWavesPerBlock * num_candidates * (sizeof(unsigned long long) + sizeof(uint32_t))) + 15u) & ~15u;
}
inline uint32_t lds_bytes_for(int num_candidates) {
    return lds_state_bytes(num_candidates) + kWavesPerBlock * kTolBytesPerWave;
}

// Tolerances of one segment: converted once to binary32 for the dtypes whose rule runs in binary32,
// and as given for binary64 segments.  Three 64-bit words.
struct SegTol {
    float atol_f;
    float rtol_f;
    double atol;
    double rtol;
};
static_assert(sizeof(SegTol) == 24, "SegTol is read as three 64-bit words");

// A segment as the planner and the kernels see it: `numel` elements in rows of `row_elems`, row r starting
// pitch_bytes * r behind byte_offset.  A contiguous segment is one row.  `layout` says where the reference's
// elements lie: 0 at the candidates' own offsets; kRefMapped (bit 0) with the reference's element stride in the
// bits from kRefStrideShift up: element (r, c) at ref_byte_offset + r * ref_pitch_bytes + c * stride * element size
// (stride 0: one element per row; stride 1: the row is contiguous; more: its elements are gathered one by one).
// kMxScaled: a block-scaled segment (dtype one of the GEAK_MX* codes, contiguous, whole blocks of kMxBlock
// elements); ref_byte_offset then holds the offset of its scale bytes, one per block, in every packed buffer.
// kSegNd (bit 1, with kRefMapped): the rows x row_elems of the record are one 2-D block of an N-d segment; the
// segment's SegNd entry says how many rows a block has and where the blocks lie.
// Seven 64-bit words: device code reads the record word by word.
constexpr int32_t kRefMapped = 1, kSegNd = 2, kMxScaled = 4;
constexpr int kRefStrideShift = 8;
constexpr uint64_t kMaxRefStride = (1ull << 22) - 1;
constexpr uint64_t kMxBlock = 32;
inline bool is_mx_dtype(int dtype) { return dtype >= GEAK_MXFP8_E4M3 && dtype <= GEAK_MXFP6_E3M2; }
struct SegDesc {
    uint64_t byte_offset;
    uint64_t numel;
    uint64_t row_elems;                  // >= 1
    uint64_t pitch_bytes;
    int32_t dtype;
    int32_t layout;
    uint64_t ref_byte_offset;
    uint64_t ref_pitch_bytes;
};
static_assert(sizeof(SegDesc) == 56, "SegDesc is read as seven 64-bit words");
// The dimensions of an N-d segment above its 2-D blocks (up to two; extent 1 and stride 0 where unused): block
// (o0, o1) starts outer_stride[0] * o0 + outer_stride[1] * o1 bytes behind the segment's byte_offset in the
// candidates, and outer_ref_stride likewise behind ref_byte_offset in the reference (0: broadcast); element
// indices are row-major over (outer_shape[0], outer_shape[1], inner_rows, row_elems).  Seven 64-bit words.
struct SegNd {
    uint64_t inner_rows;
    uint64_t outer_shape[2];
    uint64_t outer_stride[2];
    uint64_t outer_ref_stride[2];
};
static_assert(sizeof(SegNd) == 56, "SegNd is seven 64-bit words");
constexpr bool seg_is_nd(const SegDesc &g) { return g.layout != kMxScaled && (g.layout & kSegNd) != 0; }
inline uint64_t seg_rows(const SegDesc &g) { return g.numel / g.row_elems; }
constexpr bool seg_ref_mapped(const SegDesc &g) { return g.layout != kMxScaled && (g.layout & kRefMapped) != 0; }
constexpr uint64_t seg_ref_stride(const SegDesc &g) { return (uint32_t)g.layout >> kRefStrideShift; }       // of a mapped segment
// bytes from the segment's first to behind its last element
inline uint64_t seg_span(const SegDesc &g)
{
    return g.numel ? (seg_rows(g) - 1) * g.pitch_bytes + payload_bytes(g.dtype, g.row_elems) : 0;
}
// bytes of one row of a mapped segment's reference, first to behind last element (the planner refuses what would overflow)
inline uint64_t seg_ref_row_span(const SegDesc &g)
{
    return ((g.row_elems - 1) * seg_ref_stride(g) + 1) * (uint64_t)elem_size(g.dtype);
}
// the same for all rows
inline uint64_t seg_ref_span(const SegDesc &g)
{
    return g.numel ? (seg_rows(g) - 1) * g.ref_pitch_bytes + seg_ref_row_span(g) : 0;
}

// Host side of a plan: everything that can be decided without a device.
struct HostPlan {
    std::vector<SegDesc> segments;
    std::vector<SegNd> nd;                 // per segment, only when a segment is N-d (else empty)
    std::vector<geak_item> items;
    std::vector<uint64_t> ref_item_offset; // per item, only when a segment is mapped: byte offset of the reference element
                                           // that the item's first element is compared with
    std::vector<uint32_t> slot_begin;      // per segment, size nsegs + 1; slots of a segment are contiguous
    uint64_t algorithmic_bytes = 0;
    int num_candidates = 0;
    std::vector<SegTol> seg_tol;          // per segment
    int equal_nan = 0;
    uint32_t grid_blocks = 1;
    uint32_t replicas = 1;                 // replicas of the running maxima per (segment, candidate)
    std::vector<uint32_t> block_first;     // size grid_blocks + 1: block b owns items [block_first[b], block_first[b + 1])
    std::vector<uint32_t> wave_first;      // size grid_blocks * kWavesPerBlock: first item of each wave's list (kNoItem: none)
    uint32_t max_blocks = 1;               // compute units x resident blocks per unit
    uint32_t unit_groups = 1;              // compute units, when a full grid's blocks take the table's ranges by GEAK_MAP_ROTATED or _BY_UNIT
    uint32_t block_map = GEAK_MAP_PLAIN;   // which block runs which range: table_range_of_block() in device_common.hpp
};

// Validates and builds the work table for a persistent grid of at most `max_blocks` blocks.
// `nd`: one entry per segment when any segment carries kSegNd (entries of the other segments are ignored), else null.
geak_status build_host_plan(HostPlan &hp, const SegDesc *segs, const geak_tolerance *tols, uint64_t nsegs,
                            int32_t num_candidates, int32_t equal_nan, uint32_t max_blocks, uint32_t compute_units,
                            const SegNd *nd = nullptr);

// Running maxima of one (segment, candidate, replica): non-negative doubles, raised by atomic max on
// their bit patterns.
struct MaxPair {
    double abs;
    double rel;
};

// Workspace layout: [candidate pointer table, kCandTableBytes][board: segments x K x replicas MaxPair]
// [partials: num_slots x K].
constexpr uint64_t kCandTableBytes = GEAK_MAX_CANDIDATES * sizeof(void *);
constexpr uint32_t kMaxReplicas = 64;
constexpr uint32_t kMinReplicas = 4;
constexpr uint64_t kBoardBudgetBytes = 16ull << 20;      // replicas are halved until the board fits

// Init kernel: neutral result records, and the candidate base pointers copied from the kernel
// argument block into the workspace so that the other kernels index them from memory.
struct InitArgs {
    geak_result *results;
    const unsigned char **cand_table;
    MaxPair *board;
    uint64_t num_board;                  // segments x K x replicas
    uint64_t num_results;
    uint32_t num_candidates;
    uint32_t reserved;
    const unsigned char *cand[GEAK_MAX_CANDIDATES];
};

struct CompareArgs {
    const geak_item *items;
    const unsigned char *ref;
    const unsigned char *const *cand_table;
    Partial *partials;
    MaxPair *board;
    uint32_t replicas;                   // power of two
    uint32_t unit_groups;                // HostPlan::unit_groups and, below, block_map: which range of the wave table a block runs
    uint32_t num_items;
    uint32_t num_candidates;
    const SegTol *seg_tol;               // device table, one entry per segment
    int equal_nan;
    uint32_t block_map;
    const uint32_t *wave_first;          // grid_blocks * kWavesPerBlock entries
    const SegDesc *segments;             // device table: the row geometry of row-group items, the reference's layout
    const uint64_t *ref_item_offset;     // device table, per item; null when no segment's reference is mapped
};

struct ReduceArgs {
    const geak_item *items;
    const uint32_t *slot_begin;
    const Partial *partials;
    const MaxPair *board;
    geak_result *results;
    const unsigned char *ref;
    const unsigned char *const *cand_table;
    uint32_t num_segments;
    uint32_t num_candidates;
    const SegTol *seg_tol;               // device table, one entry per segment
    int equal_nan;
    uint32_t replicas;
    const SegDesc *segments;             // device table: the row geometry of row-group items, the reference's layout
    const uint64_t *ref_item_offset;     // device table, per item; null when no segment's reference is mapped
};

// Read probe: num_buffers device buffers (pointer table in the workspace), bytes_each bytes of each.
struct ProbeArgs {
    const unsigned char *const *buffers;
    uint32_t *sink;
    uint64_t bytes_each;
    uint32_t num_buffers;
    uint32_t reserved;
};

struct ReportArgs {
    const SegDesc *segments;             // device copy of the segment table
    const geak_result *results;
    const unsigned char *ref;
    const unsigned char *const *cand_table;
    geak_mismatch *records;
    uint32_t *counts;
    uint32_t num_segments;
    uint32_t num_candidates;
    uint32_t max_records;
    const SegTol *seg_tol;               // device table, one entry per segment
    int equal_nan;
    int reserved;
    const SegNd *nd;                     // device table, per segment; null when no segment is N-d
};

// ---- ulp-distance histogram ------------------------------------------------------------------------
// Slots of a histogram row for one dtype: the bins its distances can reach (0 .. bit length of the
// largest distance) plus one for NaN.  A plan uses the largest over its segments.
inline uint32_t ulp_slots_of(int dtype)
{
    switch (dtype) {
    case GEAK_F16: case GEAK_BF16: return 18;            // distances below 2^16
    case GEAK_U8: case GEAK_I8: case GEAK_F8E4M3: case GEAK_F8E5M2: return 10;     // at most 255
    case GEAK_F64: case GEAK_I64: return 66;             // below 2^64
    default: return 34;                                  // binary32, int32: below 2^32
    }
}
constexpr uint32_t kUlpLdsBudgetPerWave = 10u << 10;     // rows of one pass: candidates x slots x 4 bytes

// Workspace of the histogram: [candidate pointer table, kCandTableBytes][partial rows: slots x K x nslots, 32-bit].
struct UlpArgs {
    const geak_item *items;
    const unsigned char *ref;
    const unsigned char *const *cand_table;
    uint32_t *partials;
    const uint32_t *wave_first;
    uint32_t num_items;
    uint32_t num_candidates;
    uint32_t k_begin;                    // candidates [k_begin, k_begin + k_count) are counted by this pass
    uint32_t k_count;
    uint32_t nslots;
    uint32_t unit_groups;                // as in CompareArgs
    uint32_t block_map;
    uint32_t reserved;
    const SegDesc *segments;             // device table: the row geometry of row-group items, the reference's layout
    const uint64_t *ref_item_offset;     // device table, per item; null when no segment's reference is mapped
};

struct UlpReduceArgs {
    const uint32_t *slot_begin;
    const uint32_t *partials;
    unsigned long long *hist;            // [segment][candidate][GEAK_ULP_BINS]
    uint32_t num_segments;
    uint32_t num_candidates;
    uint32_t nslots;
    uint32_t reserved;
};

int launch_ulp_histogram(const UlpArgs &args, uint32_t grid_blocks, uint32_t lds_bytes, void *stream);   // ulp_kernels.hip
int launch_ulp_reduce(const UlpReduceArgs &args, void *stream);

// Per-candidate verdict over all segments (verdict_kernel.hip).
struct VerdictArgs {
    const geak_result *results;          // [segment][candidate]
    int32_t *verdicts;                   // [candidate]: 1 iff every segment passes
    uint32_t *failed_tests;              // [candidate]: segments that fail; may be null
    uint32_t num_segments;
    uint32_t num_candidates;
};
int launch_verdicts(const VerdictArgs &args, void *stream);

// Kernel launchers (kernels.hip).  Return the hipError_t of the launch as int.
int launch_init(const InitArgs &args, void *stream);
int launch_compare(const CompareArgs &args, uint32_t grid_blocks, uint32_t lds_bytes, void *stream);
int launch_reduce(const ReduceArgs &args, void *stream);
int launch_report(const ReportArgs &args, void *stream);
int launch_read_probe(const ProbeArgs &args, uint32_t grid_blocks, void *stream);
int compare_blocks_per_cu(uint32_t lds_bytes);   // occupancy query on the current device; <= 0 on failure
// Address of `device`'s copy of the library's static scratch array (static_scratch.hip); hipError_t as int.
int static_scratch_address(int device, void **out);

}  // namespace geak
