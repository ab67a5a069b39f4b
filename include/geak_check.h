/*
 * geak_check -- output-equivalence check of K candidate tensors against one reference tensor,
 * on one MI355X (gfx950).  C ABI; plain pointers and sizes only.
 *
 * What it computes.  The evaluator of the GEAK kernel-generation agent (arXiv 2507.23194) judges
 * a candidate kernel by comparing the tensors its unit tests produce with reference outputs,
 * element by element and within a tolerance (section 3.1, second enhancement bullet); a kernel is
 * correct only if it satisfies all unit tests and the reference kernels are the ground truth
 * (section 3.3); the check runs once per candidate x unit test x refinement iteration x parallel
 * run (sections 4.1, 4.2, 5.2).  The paper gives no formula, so this library fixes one:
 *
 *   fp32, fp16, bf16 and the 8-bit formats E4M3 (no infinities, one NaN pattern per sign, largest value
 *   448) and E5M2 (an IEEE-like format), each widened exactly to binary32: a = candidate element,
 *   b = reference element, all steps in IEEE binary32,
 *   round-to-nearest-even, one rounding per step, no fused multiply-add, subnormals honoured:
 *       d = |a - b|,  tol = atol_f + (rtol_f * |b|),  close <=> d <= tol
 *       a or b NaN   : close <=> equal_nan and both NaN
 *       a or b +-Inf : close <=> a == b
 *   fp64: the same rule with every step in IEEE binary64 and atol, rtol as given (not narrowed)
 *   int32, int64, uint8, int8:
 *                      close <=> a == b   (atol, rtol, equal_nan ignored; d = |a - b| exact; for int64
 *                      d (up to 2^64 - 1) and |b| are each rounded once to binary64 where a double is
 *                      needed: max_abs_err, max_rel_err, the mismatch report)
 *
 *   and reduces, for every (segment, candidate) pair, the record `geak_result`:
 *       mismatch_count  number of elements that are not close
 *       first_mismatch  least flat 0-based index (within the segment) that is not close, else -1
 *       pass            1 iff mismatch_count == 0 (an empty segment passes)
 *       max_abs_err     max of d over ALL elements, NaN d skipped, +Inf kept, starting at +0
 *       max_rel_err     max over all elements of (d == 0 ? 0 : d / |b|) (binary32 division for
 *                       fp32 / fp16 / bf16 / E4M3 / E5M2, binary64 for fp64 and the integer dtypes;
 *                       x/0 = +Inf; NaN skipped), from +0
 *   Every field is an order-independent reduction, so results are bit-reproducible.
 *
 * Memory model.  The caller owns every device buffer (reference, candidates, workspace, results)
 * and the HIP stream.  The library owns only the opaque plan: a host structure plus a small device
 * work table allocated in geak_check_plan and freed in geak_check_destroy.  geak_check_run is
 * asynchronous on the given stream, never synchronises and never allocates.
 */
#ifndef GEAK_CHECK_H
#define GEAK_CHECK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GEAK_OK = 0,
    GEAK_EINVAL = 1,     /* null pointer, nsegs == 0, K out of range, bad atol/rtol/equal_nan, host-only plan run */
    GEAK_EDTYPE = 2,     /* unknown dtype code */
    GEAK_EALIGN = 3,     /* byte_offset or a tensor's base pointer not a multiple of the element size; workspace or results misaligned */
    GEAK_EBOUNDS = 4,    /* byte_offset + numel * size overflows, segments overlap, or too many elements */
    GEAK_ENOMEM = 5,     /* host or device allocation failed while planning */
    GEAK_EWORKSPACE = 6, /* workspace pointer missing although geak_check_workspace_bytes() > 0 */
    GEAK_EHIP = 7        /* a HIP runtime call failed (no device, launch error) */
} geak_status;

typedef enum { GEAK_F32 = 0, GEAK_F16 = 1, GEAK_BF16 = 2, GEAK_I32 = 3, GEAK_I64 = 4,
               GEAK_U8 = 5 /* also boolean masks stored as bytes */, GEAK_I8 = 6, GEAK_F64 = 7,
               GEAK_F8E4M3 = 8, GEAK_F8E5M2 = 9, /* the 8-bit formats of the OCP 8-bit floating point specification */
               /* element formats of block-scaled segments (geak_segment_mx only) */
               GEAK_MXFP8_E4M3 = 10, GEAK_MXFP8_E5M2 = 11, GEAK_MXINT8 = 12, GEAK_MXFP4_E2M1 = 13,
               GEAK_MXFP6_E2M3 = 14, GEAK_MXFP6_E3M2 = 15 } geak_dtype;

#define GEAK_MAX_CANDIDATES 256
#define GEAK_MAX_SEGMENT_NUMEL (1ull << 40)

/* One tensor of a packed (ragged) batch.  Every buffer -- the reference and each candidate -- is
 * packed with the same table.  byte_offset must be a multiple of the element size; a start off the
 * 16-byte grid costs the segment one shorter first work item, read from the boundary before it.
 * numel == 0 is legal.  Segments must not overlap.  In a tensor whose base pointer is 16-byte aligned the
 * kernels load whole 16-byte aligned vectors: the up to 15 bytes between such a boundary and a segment's first
 * byte, and between its last byte and the next boundary, may be read (never compared, never written); they lie
 * in pages the segment occupies.  In a tensor whose base pointer is only element-aligned nothing outside the
 * segments is read. */
typedef struct {
    uint64_t byte_offset;
    uint64_t numel;
    int32_t  dtype;      /* geak_dtype */
    int32_t  reserved;   /* must be 0 */
} geak_segment;

/* One record per (segment, candidate); see the file comment for field meaning.  40 bytes. */
typedef struct {
    int32_t  pass;
    int32_t  reserved;
    uint64_t mismatch_count;
    int64_t  first_mismatch;
    double   max_abs_err;
    double   max_rel_err;
} geak_result;

typedef struct geak_plan geak_plan; /* opaque */

/*
 * Plan a check of `num_candidates` packed candidate buffers against one packed reference buffer
 * (section 3.3: a kernel has many unit-test outputs and must satisfy all of them -- one segment per
 * output).  Validates the arguments, cuts the segments into fixed-size work items, assigns them to
 * the persistent grid and sizes the workspace.
 *   out            receives the plan; untouched on failure
 *   segs, nsegs    host array, copied; nsegs >= 1
 *   num_candidates 1 .. GEAK_MAX_CANDIDATES
 *   atol, rtol     finite, >= 0; converted once to binary32 (fp64 segments use them as given)
 *   equal_nan      0 or 1
 *   device         HIP device ordinal that geak_check_run will use; -1 builds a host-only plan
 *                  (for inspection; geak_check_run then returns GEAK_EINVAL) laid out for 256 compute units
 * Returns GEAK_OK or an error code; never throws, aborts or prints.
 */
geak_status geak_check_plan(geak_plan **out, const geak_segment *segs, uint64_t nsegs,
                            int32_t num_candidates, double atol, double rtol, int32_t equal_nan,
                            int32_t device);

/* One tolerance pair per segment.  The unit tests of one kernel produce outputs of different
 * magnitude and precision (section 3.3: a kernel is checked on all of its unit tests), so each
 * packed output may be judged with its own atol / rtol; integer segments ignore theirs. */
typedef struct {
    double atol;
    double rtol;
} geak_tolerance;

/* Like geak_check_plan, with `tols[s]` applying to segment s (host array of nsegs entries, copied;
 * each value finite and >= 0, for every dtype but fp64 also after conversion to binary32). */
geak_status geak_check_plan_tolerances(geak_plan **out, const geak_segment *segs, const geak_tolerance *tols,
                                       uint64_t nsegs, int32_t num_candidates, int32_t equal_nan, int32_t device);

/* A segment stored as `rows` rows of `row_elems` elements, row r starting pitch_bytes * r behind byte_offset:
 * outputs that kernels write into padded buffers (section 3.3: every unit-test output is checked; repacking
 * them first would cost another pass over the data).  The reference and every candidate use the same layout.
 * Indices (first_mismatch, the report) are flat and row-major over the rows * row_elems elements, padding
 * not counted.  pitch_bytes must be a multiple of the element size and at least one row long; segments may not
 * interleave (their spans from first to last byte must not overlap).  Rows that start 16-byte aligned and are at
 * least 4 KiB long run at the speed of contiguous data; rows of at most 2 KiB that all start 16-byte aligned
 * (byte_offset and pitch_bytes multiples of 16) are grouped, several whole rows to a work item; other short rows
 * are handled one by one. */
typedef struct {
    uint64_t byte_offset;
    uint64_t rows;
    uint64_t row_elems;
    uint64_t pitch_bytes;
    int32_t  dtype;
    int32_t  reserved;   /* must be 0 */
} geak_segment2d;

/* Like geak_check_plan_tolerances for pitched segments; `tols` may be null, then atol / rtol apply to all. */
geak_status geak_check_plan_pitched(geak_plan **out, const geak_segment2d *segs, const geak_tolerance *tols,
                                    uint64_t nsegs, int32_t num_candidates, double atol, double rtol,
                                    int32_t equal_nan, int32_t device);

/* A segment whose reference has a layout of its own.  The candidates store it like a geak_segment2d (rows x
 * row_elems elements, rows pitch_bytes apart, the first at byte_offset of every candidate buffer); the reference
 * buffer holds the value that candidate element (r, c) is compared with at
 *     ref_byte_offset + r * ref_pitch_bytes + c * ref_elem_stride * element size.
 * The paper's benchmark kernels include reductions, normalisations and elementwise kernels (section 4.1, Table 1)
 * whose expected output is naturally one row, one column or one value for the whole output; the rule of section 3.1
 * is unchanged, only where b is read differs.
 *   ref_pitch_bytes   bytes between the reference's rows; any multiple of the element size, also one below a row's
 *                     length (overlapping rows) and 0: one reference row for all rows
 *   ref_elem_stride   elements between neighbours of a reference row.  1: the row is contiguous; 0: one reference
 *                     element for the whole row (with ref_pitch_bytes == 0: one element for the whole segment);
 *                     more (below 2^22): a strided row -- a reference stored transposed is ref_pitch_bytes = element
 *                     size, ref_elem_stride = rows of the reference's own storage
 * Reference regions of different segments may overlap each other; the candidates' spans may not, as for every
 * other plan.  Indices in the results are flat over the candidates' rows * row_elems elements.  A reference element
 * that several candidate elements share is read once per work item that needs it: the algorithmic bytes of such a
 * plan count the candidates' elements K times and the reference's distinct elements once.  With a contiguous
 * reference row (stride 1), rows that start 16-byte aligned and are at least 4 KiB long run as full work items;
 * with one element per row every item takes the guarded path of a segment's tail, and a strided row is gathered
 * element by element (correct, far from the memory's rate). */
typedef struct {
    uint64_t byte_offset;
    uint64_t rows;
    uint64_t row_elems;
    uint64_t pitch_bytes;
    uint64_t ref_byte_offset;
    uint64_t ref_pitch_bytes;
    int32_t  ref_elem_stride;    /* >= 0 */
    int32_t  dtype;
} geak_segment_mapped;

/* Like geak_check_plan_pitched for segments whose reference has its own layout; `tols` may be null, then
 * atol / rtol apply to all.  GEAK_EINVAL for a negative stride, GEAK_EALIGN for reference offsets or pitches that
 * are no multiple of the element size, GEAK_EBOUNDS for a stride of 2^22 or more or when the reference region
 * leaves the address space. */
geak_status geak_check_plan_mapped(geak_plan **out, const geak_segment_mapped *segs, const geak_tolerance *tols,
                                   uint64_t nsegs, int32_t num_candidates, double atol, double rtol,
                                   int32_t equal_nan, int32_t device);

/* A block-scaled segment (OCP Microscaling Formats (MX) specification v1.0): a payload of numel one-byte
 * elements and one shared scale byte (E8M0: 2^(X - 127), X = 0xFF is NaN) per block of 32 consecutive elements.
 * Quantising kernels -- the benchmark kernels of section 4.1, Table 1 include an MXFP matmul and fp8 kernels --
 * write such outputs; a candidate may choose other scales than the reference and still encode the same numbers,
 * so the rule of section 3.1 is applied to the VALUES: element i stands for scale(block of i) * value(payload
 * code), formed in binary32 -- exact, except that a product beyond binary32's range becomes an infinity of its
 * sign (the specification leaves that case open) -- and the binary32 rule of the other narrow floating dtypes
 * judges them.  A NaN scale makes its 32 elements NaN; the payload's own NaN and infinity codes stay what they
 * are under any scale.
 *   dtype               GEAK_MXFP8_E4M3, GEAK_MXFP8_E5M2 (payload codes as GEAK_F8E4M3 / GEAK_F8E5M2), GEAK_MXINT8
 *                       (two's complement, value code / 64), GEAK_MXFP4_E2M1 (two four-bit codes per byte, element
 *                       2j in the low nibble of byte j: sign, two exponent bits, one mantissa bit; magnitudes 0, 0.5,
 *                       1, 1.5, 2, 3, 4, 6), GEAK_MXFP6_E2M3 or GEAK_MXFP6_E3M2 (six-bit codes: sign, exponent,
 *                       mantissa, bias 1 and 3, no infinities and no NaN, largest values 7.5 and 28; the
 *                       specification leaves their place in memory open: here they are packed without gaps, element
 *                       i in bits 6 i .. 6 i + 5 of the payload read as one little-endian number, a block of 32
 *                       elements in 24 bytes)
 *   byte_offset         of the payload within every packed buffer; a multiple of 16
 *   numel               a multiple of 32 (whole blocks); the payload is numel bytes, numel / 2 for the four-bit
 *                       format, numel * 3 / 4 for the six-bit ones
 *   scale_byte_offset   of the numel / 32 scale bytes within the same buffer
 * Payloads and scale regions of a plan may not overlap each other.  The algorithmic bytes count payload and
 * scales of every tensor once.  A full work item of the four- and six-bit formats is 4096 elements, 2 KiB and
 * 3 KiB of payload.  The ulp histogram is not defined for such plans (GEAK_EDTYPE). */
typedef struct {
    uint64_t byte_offset;
    uint64_t numel;
    uint64_t scale_byte_offset;
    int32_t  dtype;
    int32_t  reserved;   /* must be 0 */
} geak_segment_mx;

/* Like geak_check_plan_tolerances for block-scaled segments; `tols` may be null, then atol / rtol apply to all.
 * GEAK_EDTYPE for another dtype, GEAK_EALIGN for a payload off the 16-byte grid, GEAK_EINVAL for a ragged last
 * block, GEAK_EBOUNDS for overlapping regions. */
geak_status geak_check_plan_mx(geak_plan **out, const geak_segment_mx *segs, const geak_tolerance *tols,
                               uint64_t nsegs, int32_t num_candidates, double atol, double rtol,
                               int32_t equal_nan, int32_t device);

/* N-d segments (section 3.1: the outputs that are compared are tensors, and what a reference implementation returns
 * need not be laid out like what a generated kernel writes): every tensor of the unit test is an N-d array of up
 * to GEAK_MAX_DIMS dimensions and the reference has strides of its own -- 0 along a dimension where it is broadcast
 * against the candidates, a permutation of the candidates' where it is a transposed view, anything else that
 * numpy-style strides express.  The rule is applied to element (i0, i1, ...) of the candidate against element
 * (i0, i1, ...) of the reference; flat indices (first_mismatch, the mismatch report) are row-major over `shape`.
 *   byte_offset        of the candidates' element (0, ..., 0) within every candidate buffer
 *   ref_byte_offset    of the reference's element (0, ..., 0) within the reference buffer
 *   shape              extents, outermost first; the first ndim entries are used (ndim 0: one element)
 *   stride_bytes       candidates: bytes from one index of a dimension to the next; multiples of the element size;
 *                      the innermost is the element size, and every other one at least the bytes that the dimensions
 *                      inside it span (no two elements share a byte: a slice of a larger array, a padded layout)
 *   ref_stride_bytes   reference: multiples of the element size, 0 where broadcast; the innermost at most
 *                      (2^22 - 1) elements; the reference's elements may overlap and coincide freely
 *   dtype              any but the block-scaled element formats
 * Neighbouring dimensions that both tensors step through in one stride are merged and extents of 1 dropped; what
 * is left as one or two dimensions is exactly a geak_segment_mapped, three or four are cut into 2-D blocks, one per
 * index of the outer dimensions.  GEAK_EINVAL: ndim outside 0 .. GEAK_MAX_DIMS, the candidates' innermost stride not
 * the element size; GEAK_EALIGN: a stride or offset off the element grid; GEAK_EBOUNDS: candidates' dimensions that
 * run into each other, more than GEAK_MAX_SEGMENT_NUMEL elements, offsets beyond the address space, a reference
 * stride too large.  The read probe is not defined for such plans (GEAK_EINVAL), as for geak_check_plan_mapped. */
#define GEAK_MAX_DIMS 4
typedef struct {
    uint64_t byte_offset;
    uint64_t ref_byte_offset;
    uint64_t shape[GEAK_MAX_DIMS];
    uint64_t stride_bytes[GEAK_MAX_DIMS];
    uint64_t ref_stride_bytes[GEAK_MAX_DIMS];
    int32_t  ndim;
    int32_t  dtype;
} geak_segment_nd;

/* `tols` may be null, then atol / rtol apply to all. */
geak_status geak_check_plan_nd(geak_plan **out, const geak_segment_nd *segs, const geak_tolerance *tols,
                               uint64_t nsegs, int32_t num_candidates, double atol, double rtol,
                               int32_t equal_nan, int32_t device);

/* One table for a batch whose unit-test outputs are of different kinds (section 3.3: a kernel is checked on all of
 * its unit tests, and those need not produce the same kind of output): every entry is a plain or padded segment, a
 * segment whose reference has a layout of its own, or a block-scaled segment, with the fields of geak_segment2d,
 * geak_segment_mapped or geak_segment_mx and the same rules.
 *   kind GEAK_KIND_PITCHED   byte_offset, rows, row_elems, pitch_bytes, dtype (a contiguous segment: rows = 1 and
 *                            pitch_bytes = its length in bytes); the other fields 0
 *   kind GEAK_KIND_MAPPED    all fields, as in geak_segment_mapped
 *   kind GEAK_KIND_MX        byte_offset, rows = 1, row_elems = the element count, aux_byte_offset = the scales' offset,
 *                            dtype one of the GEAK_MX* formats; pitch_bytes, aux_pitch_bytes and ref_elem_stride 0
 * One plan, one launch, one result table in the entries' order; the ulp histogram is refused when any entry is
 * block-scaled, the read probe when any entry's reference has its own layout. */
enum { GEAK_KIND_PITCHED = 0, GEAK_KIND_MAPPED = 1, GEAK_KIND_MX = 2 };
typedef struct {
    uint64_t byte_offset;
    uint64_t rows;
    uint64_t row_elems;
    uint64_t pitch_bytes;
    uint64_t aux_byte_offset;    /* MAPPED: the reference's byte offset; MX: the scales' */
    uint64_t aux_pitch_bytes;    /* MAPPED: bytes between the reference's rows */
    int32_t  ref_elem_stride;    /* MAPPED */
    int32_t  dtype;
    int32_t  kind;               /* GEAK_KIND_* */
    int32_t  reserved;           /* must be 0 */
} geak_segment_any;

/* `tols` may be null, then atol / rtol apply to all.  Errors as for the entry point of each kind; GEAK_EINVAL for an
 * unknown kind or a field that the kind asks to be 0 and is not. */
geak_status geak_check_plan_table(geak_plan **out, const geak_segment_any *segs, const geak_tolerance *tols,
                                  uint64_t nsegs, int32_t num_candidates, double atol, double rtol,
                                  int32_t equal_nan, int32_t device);

/* Dense convenience (section 3.1: one output tensor against its reference): a single segment at
 * offset 0 with prod(shape) elements; shape is a host array of ndim >= 0 non-negative extents
 * (ndim == 0 is a scalar).  Only the element count matters: indices are flat, row-major. */
geak_status geak_check_plan_dense(geak_plan **out, int32_t dtype, const int64_t *shape, int32_t ndim,
                                  int32_t num_candidates, double atol, double rtol, int32_t equal_nan,
                                  int32_t device);

/* Bytes of device workspace geak_check_run needs (may be 0); the buffer must be 16-byte aligned. */
uint64_t geak_check_workspace_bytes(const geak_plan *plan);

/* Number of result records = nsegs * num_candidates; record index = segment * num_candidates + candidate. */
uint64_t geak_check_result_count(const geak_plan *plan);

/*
 * Run the planned check (the comparison of section 3.1 for all candidates in one pass: the
 * reference is read once and every candidate once).
 *   ref_dev      device pointer, packed reference buffer, aligned to the largest element size among the
 *                plan's segments -- a slice of a larger tensor will do; 16-byte aligned bases are read a
 *                little faster (may be NULL, like the candidate pointers, when every segment is empty:
 *                nothing is read then)
 *   cand_dev     HOST array of num_candidates DEVICE pointers, each aligned and packed like ref_dev (the
 *                tensors need not share an alignment)
 *   workspace    device pointer to geak_check_workspace_bytes() bytes (ignored when that is 0)
 *   results_dev  device pointer to geak_check_result_count() records; fully overwritten
 *   hip_stream   hipStream_t (NULL = default stream); three kernels are enqueued on it
 * Results are valid once the caller has synchronised the stream.  Concurrent runs of one plan are
 * allowed when they use distinct workspace and results buffers.
 */
geak_status geak_check_run(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                           void *workspace_dev, geak_result *results_dev, void *hip_stream);

/*
 * geak_check_run for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The workspace is a static device array of
 * GEAK_STATIC_SCRATCH_BYTES that is part of the library (every GPU the library runs on holds its own copy
 * until the process ends); the call itself allocates nothing.  Arguments and results as for
 * geak_check_run, without the workspace.  GEAK_EWORKSPACE when geak_check_workspace_bytes(plan) exceeds
 * GEAK_STATIC_SCRATCH_BYTES (8 MiB hold the five benchmark workloads, up to 2^30 elements x 32 candidates).
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams or
 * threads) race; calls on one stream, one after the other, are fine -- nothing is carried over from
 * one call to the next, every byte a call reads from the array it has written before.  The array's
 * address is looked up when a plan is built for the device, so the run itself makes no such call.
 */
#define GEAK_STATIC_SCRATCH_BYTES (8u << 20)
geak_status geak_check_run_static(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                                  geak_result *results_dev, void *hip_stream);

void geak_check_destroy(geak_plan *plan);

const char *geak_status_string(geak_status status);

/* Digest (16 hex digits of a SHA-256) of the source files the loaded library was built from: the build script,
 * this header and every file of csrc/, concatenated in bytewise path order.  A harness compares it with the
 * digest of the sources it sits beside and refuses a library that was built from other sources. */
const char *geak_check_build_id(void);

/* ---- inspection (host only; used by tests and the benchmark's reporting) ---------------------- */

typedef struct {
    uint64_t num_segments;
    uint64_t num_items;          /* work items (one wavefront processes one item against all candidates) */
    uint64_t num_slots;          /* partial-result slots in the workspace */
    uint64_t algorithmic_bytes;  /* (K + 1) * sum(numel * element size): every element of every tensor once (a mapped
                                    segment's reference: its distinct elements once) */
    uint32_t num_candidates;
    uint32_t grid_blocks;        /* persistent grid of the compare kernel */
    uint32_t block_threads;
    uint32_t lds_bytes;          /* dynamic LDS per block */
    uint32_t item_bytes;         /* bytes of one full work item per tensor */
    int32_t  device;
    uint32_t unit_groups;        /* compute units of the device, when block_map is not GEAK_MAP_PLAIN; else 1 */
    uint32_t block_map;          /* GEAK_MAP_*: which block of the compare kernel runs which range of the block
                                    table (geak_check_plan_blocks) */
} geak_plan_info;

/* One work item, as the compare kernel sees it.  32 bytes. */
typedef struct {
    uint64_t byte_offset;  /* of the item's first element, within every packed buffer */
    uint64_t elem_start;   /* flat index of that element within its segment */
    uint32_t segment;
    uint32_t slot;         /* workspace slot its run accumulates into */
    uint16_t numel;        /* 1 .. item_bytes / element size (at most 4096) */
    uint8_t  dtype;
    uint8_t  flags;        /* GEAK_ITEM_* */
    uint32_t next;         /* index of the next item of the same wavefront, GEAK_NO_ITEM after its last */
} geak_item;

#define GEAK_NO_ITEM 0xFFFFFFFFu
#define GEAK_ITEM_FULL  1u /* 16-byte aligned start and exactly item_bytes long: unguarded vector loads */
#define GEAK_ITEM_FIRST 2u /* first item of its (wavefront, segment) run: running state is reset */
#define GEAK_ITEM_LAST  4u /* last item of its run: running state is written to the slot */
#define GEAK_ITEM_ALIGNED 8u /* 16-byte aligned start (FULL implies it): vector loads, guarded at the end.  Not set: the
                                first item of a segment or row that starts off the 16-byte grid; it ends where a full
                                item read from the boundary before it would end, or with the segment or row */
#define GEAK_ITEM_ROWS 16u /* several whole rows of a pitched segment whose rows are short and start on 16-byte
                              boundaries: numel / row_elems rows, pitch_bytes apart, the first at byte_offset;
                              elem_start is the flat index of the first row's first element (ALIGNED is set) */
#define GEAK_ITEM_STREAM 64u /* with ROWS: the rows are whole 16-byte vectors (and the reference's rows, if it has a layout of
                                its own, are contiguous or one element each): the compare kernel streams such groups like full items */
#define GEAK_ITEM_REFMAP 32u /* the segment's reference has a layout of its own (geak_segment_mapped): the item's
                                reference elements are found through the segment's mapping, not at byte_offset */

geak_status geak_check_plan_info(const geak_plan *plan, geak_plan_info *out);

/* values of geak_plan_info.block_map */
#define GEAK_MAP_PLAIN 0u
#define GEAK_MAP_ROTATED 1u
#define GEAK_MAP_BY_UNIT 2u

/* Copies up to `capacity` entries of the block table into `out` (host); returns its length,
 * grid_blocks + 1.  Range r of the table is the items [table[r], table[r + 1]); the ranges partition
 * the item table in order and none is empty.  Which block runs range r depends on block_map; a grid
 * that fills the chip is dispatched round by round, block b to XCD b mod 8 and to compute unit
 * u = b mod unit_groups in round q = b / unit_groups, and with g = u ^ ((u >> 3) & 7):
 *   GEAK_MAP_PLAIN    block b runs range b (grids that do not fill the chip).
 *   GEAK_MAP_ROTATED  block b runs range q * unit_groups + g: the same table, the XCDs taking turns
 *                     within every eight ranges instead of each keeping every eighth one.
 *   GEAK_MAP_BY_UNIT  block b runs range g * per_unit + q, per_unit = grid_blocks / unit_groups.  The
 *                     waves of a compute unit finish together; for a batch whose plain ranges would
 *                     load the units unequally the table is cut so that every unit streams the same
 *                     number of bytes, the ranges of the blocks that share a unit side by side. */
uint64_t geak_check_plan_blocks(const geak_plan *plan, uint32_t *out, uint64_t capacity);

/* Copies up to `capacity` entries of the wavefront table into `out` (host); returns its length,
 * grid_blocks * (block_threads / 64).  Entry r * (block_threads / 64) + w is the first item of
 * wavefront w of the block that runs range r (GEAK_NO_ITEM if it has none); the wavefront then
 * follows the items' `next` links, which stay inside the range and ascend. */
uint64_t geak_check_plan_waves(const geak_plan *plan, uint32_t *out, uint64_t capacity);

/* Copies up to `capacity` items into `out` (host); returns the total number of items. */
uint64_t geak_check_plan_items(const geak_plan *plan, geak_item *out, uint64_t capacity);

/* For a plan built by geak_check_plan_mapped: copies up to `capacity` entries of the per-item table of reference
 * offsets into `out` (host) and returns its length, the number of items; entry i is the byte offset in the
 * reference buffer of the element that item i's first element is compared with.  Returns 0 for every other plan. */
uint64_t geak_check_plan_ref_offsets(const geak_plan *plan, uint64_t *out, uint64_t capacity);

/* ---- optional device timing of the compare kernel (a measurement aid of this library, used by its
 * benchmark; not something the paper describes) -------------------------------------------------
 * After geak_check_profile_enable(plan, n) every geak_check_run records a HIP event pair around the
 * compare kernel on the run's stream, into a ring of n pairs (no synchronisation is added).
 * geak_check_profile_read must be called after the caller has synchronised the stream(s); it
 * returns the number of milliseconds values written (oldest first, at most capacity) and resets the
 * ring.  While profiling is enabled, runs of this plan must not overlap.  n == 0 disables it. */
geak_status geak_check_profile_enable(geak_plan *plan, uint32_t num_pairs);
uint64_t    geak_check_profile_read(geak_plan *plan, float *ms_out, uint64_t capacity);

/* ---- mismatch report -----------------------------------------------------------------------------
 * When the functionality test fails, the evaluator hands an error trace to the Reflector, which has
 * to work out what went wrong (sections 4.1 and 4.2, Reflexion).  The paper does not say what the
 * trace holds; this library reports, per (segment, candidate), the first elements that are not
 * close, in ascending index order, each with what the rule saw:
 *     index  flat 0-based index within the segment
 *     a, b   candidate and reference element, widened exactly to binary64
 *     d      |a - b| as the rule computed it (binary32 value widened, binary64 for fp64; exact for
 *            integers up to the one rounding of int64); NaN when a or b is NaN or both are the same
 *            infinity, +Inf when one of them is infinite
 *     tol    atol + rtol * |b| as the rule computed it (two roundings, in binary32 and widened, or in
 *            binary64 for fp64; NaN or +Inf when b is); 0 for integers
 * NaN payloads are not specified. */
typedef struct {
    int64_t index;
    double  a;
    double  b;
    double  d;
    double  tol;
} geak_mismatch; /* 40 bytes */

/*
 * Enqueue the report of a completed check.  Must follow, on the same stream, the geak_check_run that
 * produced `results_dev` from the same tensors (its records tell where each pair's mismatches start
 * and how many there are); the workspace is reused.
 *   max_records  how many mismatches to report per (segment, candidate) pair, >= 1
 *   records_dev  device array of geak_check_result_count() x max_records entries; pair p owns
 *                [p * max_records, (p + 1) * max_records); entries past its count are left untouched
 *   counts_dev   device array of geak_check_result_count() entries: min(max_records, mismatch_count)
 * One block per pair scans its segment from the pair's first mismatch and stops as soon as it has
 * what it needs, so the cost is that of reading the segment up to the last reported element (all
 * of it when the pair has fewer than max_records mismatches spread to its end).
 */
geak_status geak_check_report(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                              void *workspace_dev, const geak_result *results_dev, uint32_t max_records,
                              geak_mismatch *records_dev, uint32_t *counts_dev, void *hip_stream);

/* ---- ulp-distance histogram ------------------------------------------------------------------------
 * The other half of the numeric error trace for the Reflector (sections 4.1 and 4.2): whether a
 * failing candidate is off by rounding or by wrong values.  The paper does not define it; this
 * library counts, per (segment, candidate), ALL elements of the pair by their distance in units in
 * the last place of the tensor's own storage format:
 *     floating dtypes  distance = number of steps between a and b on the ladder of the format's
 *                      values ordered by value, -0 and +0 being one rung and +-Inf the rung after
 *                      the largest finite value
 *     integer dtypes   distance = |a - b|, exact
 *     bin 0            distance 0
 *     bin j, 1..64     2^(j-1) <= distance < 2^j
 *     bin 65           a or b is NaN (equal_nan plays no part)
 * The bins of a pair sum to the segment's numel.  A full pass over the reference and every
 * candidate; candidates are counted in passes of as many as fit the per-wave rows in LDS (the
 * reference is read once per pass). */
#define GEAK_ULP_BINS 66

/* Bytes of device scratch the histogram needs (its own, not the workspace of geak_check_run);
 * 0 for a null plan. */
uint64_t geak_check_ulp_workspace_bytes(const geak_plan *plan);

/*
 * Enqueue the histogram on `hip_stream`.  Independent of geak_check_run (no results are needed).
 *   ref_dev, cand_dev   as for geak_check_run
 *   ulp_workspace_dev   device scratch of geak_check_ulp_workspace_bytes() bytes, 16-byte aligned;
 *                       contents need not be preserved or cleared
 *   hist_dev            device array of geak_check_result_count() x GEAK_ULP_BINS 64-bit counts,
 *                       row-major [segment][candidate][bin], 8-byte aligned; every entry is written
 * Returns GEAK_OK or an error code; asynchronous, never allocates.
 */
geak_status geak_check_ulp_histogram(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                                     void *ulp_workspace_dev, uint64_t *hist_dev, void *hip_stream);

/* ---- verdicts and the evaluation metrics built on them --------------------------------------------
 * A kernel is correct only if it satisfies all of its unit tests (section 3.3); the metrics of the
 * paper's "Evaluation Metrics" section are computed from these verdicts. */

/* Enqueue, after the geak_check_run that produced `results_dev` and on the same stream:
 *   verdicts_dev[k]      1 iff every segment's record of candidate k passes (device, num_candidates int32)
 *   failed_tests_dev[k]  number of segments candidate k fails (device, num_candidates uint32); may be null */
geak_status geak_check_verdicts(const geak_plan *plan, const geak_result *results_dev, int32_t *verdicts_dev,
                                uint32_t *failed_tests_dev, void *hip_stream);

/* Host arithmetic, host pointers.
 * Call accuracy = kernels that compile and run / all kernels; execution accuracy = kernels that
 * satisfy all unit tests / kernels that compile (NaN when the denominator is 0).  compiled[i] and
 * correct[i] are flags of kernel i; `correct` only counts where `compiled` is set. */
geak_status geak_metrics_accuracy(const int32_t *compiled, const int32_t *correct, uint64_t n,
                                  double *call_accuracy, double *execution_accuracy);

/* Speedup of one correct kernel: the mean over its unit tests of (median reference latency of the
 * test / median generated latency of the test), accumulated in test order in binary64.  Latencies are
 * row-major [test][repetition]; the median of an even count is the mean of the two middle values.
 * NaN when there is no test or no repetition. */
geak_status geak_metrics_speedup(const double *ref_latencies, uint64_t ref_reps, const double *gen_latencies,
                                 uint64_t gen_reps, uint64_t num_tests, double *speedup);

/* ---- latencies for the speedup ---------------------------------------------------------------------
 * Code that passes the functionality test goes on to the performance test, which measures its latency
 * (section 4.1); the speedup compares the median latency of the reference kernel and of the generated
 * kernel on every unit test (section 3.3).  The paper does not say how a latency is taken.  Here every
 * repetition starts from cold caches and is bracketed by two events on the caller's stream. */

/* Enqueue, on `hip_stream`, a kernel that overwrites scratch_bytes (>= 16; a multiple of 16 is used) of
 * `scratch_dev` (device, 16-byte aligned, the caller's): with a buffer larger than the last-level cache
 * (512 MiB on this part: twice its 256 MB) whatever the next kernel reads comes from memory. */
geak_status geak_timing_flush(void *scratch_dev, uint64_t scratch_bytes, void *hip_stream);

/* The kernel under test, enqueued by the caller on the stream it is handed; returns 0 on success. */
typedef int (*geak_launch_fn)(void *user, void *hip_stream);

/* warmup + repetitions times: flush the caches (skipped when flush_scratch_dev is null: warm measurement),
 * record an event, call launch(user, hip_stream), record an event, wait for it.  The elapsed times of the
 * last `repetitions` rounds are written to latency_ms_out (host, `repetitions` doubles), in order: one
 * row of the [test][repetition] tables geak_metrics_speedup takes.  Synchronises the stream once per round;
 * creates and destroys two events.  GEAK_EINVAL for null launch / output, repetitions == 0, or a launch that fails. */
geak_status geak_timing_measure(geak_launch_fn launch, void *user, uint32_t warmup, uint32_t repetitions, void *flush_scratch_dev,
                                uint64_t flush_bytes, void *hip_stream, double *latency_ms_out);

/* pass@k (section 4.2: accuracy under parallel scaling is estimated with pass@k; the paper prints no
 * formula, this is the usual unbiased estimator): the probability 1 - C(n - c, k) / C(n, k) that a
 * k-subset of n samples, c of them correct, holds a correct one.  GEAK_EINVAL unless c <= n, 1 <= k <= n. */
geak_status geak_metrics_pass_at_k(uint64_t n, uint64_t c, uint64_t k, double *out);

/* ---- read probe (measurement aid, not part of the check) -------------------------------------
 * Enqueues a kernel that only reads, with 16-byte loads, the same bytes a run of this plan reads
 * (the span of the packed reference and of every candidate that the segments cover) and computes
 * nothing from them: the rate it reaches is what this machine's memory system delivers to any
 * kernel with this traffic, the yardstick beside the nominal HBM peak.  Arguments as for
 * geak_check_run (at most GEAK_MAX_CANDIDATES - 1 candidates); the workspace is used as scratch and
 * no results are produced.  The caller times it on its stream.  GEAK_EINVAL for a plan built by
 * geak_check_plan_mapped: its reference need not be as long as the candidates. */
geak_status geak_check_read_probe(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                                  void *workspace_dev, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GEAK_CHECK_H */
