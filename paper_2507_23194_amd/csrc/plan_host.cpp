// Host planner: argument validation and the work table of the compare kernel.  No HIP calls here,
// so all of it runs (and is tested) without a device.
//
// The evaluator hands over many test outputs per kernel (GEAK section 3.3: a kernel must satisfy
// all unit tests); they arrive packed in one buffer with a segment table.  Each segment is cut into
// work items of kItemBytes per tensor; one wavefront takes one item, keeps the reference slice in
// registers and streams the same slice of every candidate past it.
#include <algorithm>
#include <cmath>
#include <new>
#include "geak_internal.hpp"

namespace geak {

static bool mul_overflows(uint64_t a, uint64_t b) { return b != 0 && a > UINT64_MAX / b; }

// what a start and a tail cost a compute unit, in sixteenths of a slice (see the partition below)
constexpr uint64_t kUnitStart = 110, kUnitTailMul16 = 10, kUnitTailFix = 8;
// the one-step ranges are kept while the lightest unit's load is within this fraction of the heaviest's
constexpr uint64_t kUnitSpreadNum = 8, kUnitSpreadDen = 100;

geak_status build_host_plan(HostPlan &hp, const SegDesc *segs, const geak_tolerance *tols, uint64_t nsegs,
                            int32_t num_candidates, int32_t equal_nan, uint32_t max_blocks, uint32_t compute_units, const SegNd *nd)
{
    if (!segs || !tols || nsegs == 0 || nsegs > 0x7FFFFFFFull) return GEAK_EINVAL;
    if (num_candidates < 1 || num_candidates > GEAK_MAX_CANDIDATES) return GEAK_EINVAL;
    if (equal_nan != 0 && equal_nan != 1) return GEAK_EINVAL;
    if (max_blocks == 0 || compute_units == 0) return GEAK_EINVAL;
    for (uint64_t s = 0; s < nsegs; ++s) {
        const double atol = tols[s].atol, rtol = tols[s].rtol;
        if (!(atol >= 0.0) || !(rtol >= 0.0) || std::isinf(atol) || std::isinf(rtol)) return GEAK_EINVAL;
    }

    // per-segment checks
    uint64_t total_bytes = 0, total_ref_bytes = 0;       // the candidates' elements; the reference's distinct elements
    bool any_mapped = false, any_nd = false;
    std::vector<uint64_t> span_of;                        // bytes from a segment's first to behind its last element, candidates' side
    try {
        span_of.assign(nsegs, 0);
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    // rows of one 2-D block of a segment: all its rows, unless it is N-d
    const auto block_rows = [&](uint64_t s) { return seg_is_nd(segs[s]) ? nd[s].inner_rows : seg_rows(segs[s]); };
    for (uint64_t s = 0; s < nsegs; ++s) {
        const SegDesc &g = segs[s];
        if (g.dtype < GEAK_F32 || g.dtype > GEAK_MXFP6_E3M2) return GEAK_EDTYPE;
        if (is_mx_dtype(g.dtype) != (g.layout == kMxScaled)) return GEAK_EDTYPE;     // block-scaled element formats belong to block-scaled segments only
        if (g.layout != kMxScaled && g.layout != 0 && (!(g.layout & kRefMapped) || (g.layout & 0xFC) != 0 || g.layout < 0 ||
                                                       seg_ref_stride(g) > kMaxRefStride)) return GEAK_EINVAL;
        any_mapped |= seg_ref_mapped(g);
        if (seg_is_nd(g)) {
            if (!nd) return GEAK_EINVAL;
            any_nd = true;
        }
        if (g.layout == kMxScaled) {
            // payload on the 16-byte grid (a vector then lies inside one block), whole blocks, one contiguous row
            if (g.byte_offset % 16 != 0) return GEAK_EALIGN;
            if (g.numel % kMxBlock != 0 || (g.numel && g.row_elems != g.numel)) return GEAK_EINVAL;
            if (g.ref_byte_offset > UINT64_MAX - g.numel / kMxBlock) return GEAK_EBOUNDS;
        }
        if (g.row_elems == 0 || g.numel % g.row_elems != 0) return GEAK_EINVAL;
        if (seg_is_nd(g)) {                                  // numel = outer extents x rows of a block x row_elems (all <= 2^40: no overflow)
            const SegNd &o = nd[s];
            if (!o.inner_rows || !o.outer_shape[0] || !o.outer_shape[1]) return GEAK_EINVAL;
            if (o.inner_rows > GEAK_MAX_SEGMENT_NUMEL || o.outer_shape[0] > GEAK_MAX_SEGMENT_NUMEL || o.outer_shape[1] > GEAK_MAX_SEGMENT_NUMEL) return GEAK_EBOUNDS;
            if (g.numel) {
                const uint64_t rows = seg_rows(g);
                if (rows % o.inner_rows || (rows / o.inner_rows) % o.outer_shape[1] || rows / o.inner_rows / o.outer_shape[1] != o.outer_shape[0])
                    return GEAK_EINVAL;
            }
        }
        // the rule of every dtype but binary64 runs in binary32: its tolerances must be finite there too
        if (g.dtype != GEAK_F64 && (std::isinf((float)tols[s].atol) || std::isinf((float)tols[s].rtol))) return GEAK_EINVAL;
        const uint64_t w = (uint64_t)elem_size(g.dtype);
        if (g.byte_offset % w != 0 || g.pitch_bytes % w != 0) return GEAK_EALIGN;
        if (g.numel > GEAK_MAX_SEGMENT_NUMEL) return GEAK_EBOUNDS;
        if (mul_overflows(g.numel, w)) return GEAK_EBOUNDS;
        const uint64_t bytes = payload_bytes(g.dtype, g.numel);
        // rows must not run into each other, and the last one must end inside the address space
        if (g.numel) {
            const uint64_t row_bytes = payload_bytes(g.dtype, g.row_elems);     // <= bytes: no overflow
            const uint64_t rows = block_rows(s);
            if (g.pitch_bytes < row_bytes) return GEAK_EBOUNDS;
            if (mul_overflows(rows - 1, g.pitch_bytes)) return GEAK_EBOUNDS;
            if ((rows - 1) * g.pitch_bytes > UINT64_MAX - row_bytes) return GEAK_EBOUNDS;
            uint64_t span = (rows - 1) * g.pitch_bytes + row_bytes;
            if (seg_is_nd(g)) {
                // the blocks: element-aligned, nested from the inside out (a block ends before the next one begins)
                for (int d = 1; d >= 0; --d) {
                    const uint64_t extent = nd[s].outer_shape[d], stride = nd[s].outer_stride[d];
                    if (extent == 1) continue;
                    if (stride % w != 0) return GEAK_EALIGN;
                    if (stride < span) return GEAK_EBOUNDS;
                    if (mul_overflows(extent - 1, stride) || (extent - 1) * stride > UINT64_MAX - span) return GEAK_EBOUNDS;
                    span += (extent - 1) * stride;
                }
            }
            if (g.byte_offset > UINT64_MAX - span) return GEAK_EBOUNDS;
            span_of[s] = span;
        }
        // what one tensor holds of the segment: its elements, and for a block-scaled one its scale bytes (numel <= 2^40)
        const uint64_t tensor_bytes = bytes + (g.layout == kMxScaled ? g.numel / kMxBlock : 0);
        if (total_bytes > UINT64_MAX - tensor_bytes) return GEAK_EBOUNDS;
        total_bytes += tensor_bytes;
        // the reference's side of a mapped segment: element-aligned, inside the address space; its rows may
        // overlap or coincide, so its distinct bytes are at most its span
        uint64_t ref_bytes = tensor_bytes;
        if (seg_ref_mapped(g)) {
            if (g.ref_byte_offset % w != 0 || g.ref_pitch_bytes % w != 0) return GEAK_EALIGN;
            if (g.numel) {
                const uint64_t rows = block_rows(s);
                if (mul_overflows(rows - 1, g.ref_pitch_bytes)) return GEAK_EBOUNDS;
                if (seg_ref_stride(g) && g.row_elems - 1 > (UINT64_MAX / 16) / seg_ref_stride(g)) return GEAK_EBOUNDS;
                const uint64_t ref_row_span = seg_ref_row_span(g);                       // fits: checked in the line above
                if ((rows - 1) * g.ref_pitch_bytes > UINT64_MAX - ref_row_span) return GEAK_EBOUNDS;
                uint64_t ref_span = (rows - 1) * g.ref_pitch_bytes + ref_row_span;
                const uint64_t ref_rows = g.ref_pitch_bytes ? rows : 1;
                const uint64_t ref_row_bytes = (seg_ref_stride(g) ? g.row_elems : 1) * w;    // distinct elements of a row
                uint64_t distinct = mul_overflows(ref_rows, ref_row_bytes) ? UINT64_MAX : ref_rows * ref_row_bytes;
                if (seg_is_nd(g)) {
                    for (int d = 1; d >= 0; --d) {
                        const uint64_t extent = nd[s].outer_shape[d], stride = nd[s].outer_ref_stride[d];
                        if (extent == 1) continue;
                        if (stride % w != 0) return GEAK_EALIGN;
                        if (mul_overflows(extent - 1, stride) || (extent - 1) * stride > UINT64_MAX - ref_span) return GEAK_EBOUNDS;
                        ref_span += (extent - 1) * stride;
                        if (stride) distinct = mul_overflows(distinct, extent) ? UINT64_MAX : distinct * extent;
                    }
                }
                if (g.ref_byte_offset > UINT64_MAX - ref_span) return GEAK_EBOUNDS;
                ref_bytes = std::min(std::min(ref_span, distinct), tensor_bytes);           // overlapping reference blocks: never more than the candidates' bytes
            }
        }
        total_ref_bytes += ref_bytes;                        // <= total_bytes: no overflow
    }
    if (mul_overflows(total_bytes, (uint64_t)num_candidates + 1)) return GEAK_EBOUNDS;

    try {
        // overlap check on the non-empty segments, sorted by start
        std::vector<std::pair<uint64_t, uint64_t>> spans;
        spans.reserve(nsegs);
        for (uint64_t s = 0; s < nsegs; ++s)
            if (segs[s].numel) {
                spans.emplace_back(segs[s].byte_offset, segs[s].byte_offset + span_of[s]);   // pitched and N-d segments: first to last byte
                if (segs[s].layout == kMxScaled)                                                     // and a block-scaled segment's scales
                    spans.emplace_back(segs[s].ref_byte_offset, segs[s].ref_byte_offset + segs[s].numel / kMxBlock);
            }
        std::sort(spans.begin(), spans.end());
        for (size_t i = 1; i < spans.size(); ++i)
            if (spans[i].first < spans[i - 1].second) return GEAK_EBOUNDS;

        // Count items first, in closed form (a segment may have 2^40 one-element rows): a group of short rows
        // is one item; otherwise a row gives a shorter first item where it starts off the 16-byte grid, full
        // items and a tail, and the rows' starts repeat modulo 16 with a period of at most 16 rows.
        // items of one 2-D block of segment s whose first row starts at byte `base`
        const auto count_block = [&](uint64_t s, uint64_t base) -> uint64_t {
            const SegDesc &g = segs[s];
            const uint64_t w = elem_size(g.dtype), per = elems_per_item(g.dtype);
            const uint64_t rows = block_rows(s);
            const uint64_t row_vectors = (g.row_elems * w + 15) / 16;
            if (rows > 1 && base % 16 == 0 && g.pitch_bytes % 16 == 0 && row_vectors <= kItemBytes / 32) {
                const uint64_t group = (kItemBytes / 16) / row_vectors;
                return (rows + group - 1) / group;
            }
            uint64_t period = 1, total = 0;
            while ((g.pitch_bytes * period) % 16 != 0) period *= 2;        // 1, 2, 4, 8 or 16
            for (uint64_t r = 0; r < period && r < rows; ++r) {
                uint64_t n = g.row_elems, count = 0;
                const uint64_t skip = ((base + r * g.pitch_bytes) % 16) / w;
                if (skip) { ++count; n -= std::min<uint64_t>(n, per - skip); }
                count += n / per + (n % per ? 1 : 0);
                total += count * ((rows - r + period - 1) / period);     // rows r, r + period, r + 2 period, ...
            }
            return total;
        };
        uint64_t n_items = 0;
        for (uint64_t s = 0; s < nsegs; ++s) {
            const SegDesc &g = segs[s];
            if (!g.numel) continue;
            if (!seg_is_nd(g)) {
                n_items += count_block(s, g.byte_offset);
            } else {
                // block by block: every block holds at least one item, so more blocks than the table can hold items are
                // refused before they are walked, and the loop ends with the item limit
                if (nd[s].outer_shape[0] >= 0x7FFFFFFFull / nd[s].outer_shape[1]) return GEAK_EBOUNDS;
                for (uint64_t o0 = 0; o0 < nd[s].outer_shape[0] && n_items < 0x7FFFFFFFull; ++o0)
                    for (uint64_t o1 = 0; o1 < nd[s].outer_shape[1] && n_items < 0x7FFFFFFFull; ++o1)
                        n_items += count_block(s, g.byte_offset + o0 * nd[s].outer_stride[0] + o1 * nd[s].outer_stride[1]);
            }
            if (n_items >= 0x7FFFFFFFull) return GEAK_EBOUNDS;
        }
        if (n_items >= 0x7FFFFFFFull) return GEAK_EBOUNDS;

        hp.segments.assign(segs, segs + nsegs);
        hp.nd.clear();
        if (any_nd) hp.nd.assign(nd, nd + nsegs);
        hp.items.clear();
        hp.items.reserve(n_items);
        hp.ref_item_offset.clear();
        if (any_mapped) hp.ref_item_offset.reserve(n_items);
        hp.slot_begin.assign(nsegs + 1, 0);
        hp.num_candidates = num_candidates;
        hp.seg_tol.resize(nsegs);
        for (uint64_t s = 0; s < nsegs; ++s) hp.seg_tol[s] = SegTol{(float)tols[s].atol, (float)tols[s].rtol, tols[s].atol, tols[s].rtol};
        hp.equal_nan = equal_nan;
        hp.algorithmic_bytes = total_bytes * (uint64_t)num_candidates + total_ref_bytes;
        hp.max_blocks = max_blocks;
        // Replicas of the running maxima.  Many waves raising one address serialise, so few
        // candidates (few addresses per segment) want many replicas; but every replica has to learn
        // its maxima by itself, so many candidates want few.  About 512 addresses per segment, within
        // 4 .. 64 replicas, and fewer when so many (segment, candidate) pairs exist that the board
        // would outgrow its budget.
        hp.replicas = kMaxReplicas;
        while (hp.replicas > kMinReplicas && (uint64_t)hp.replicas * (uint64_t)num_candidates > 512) hp.replicas /= 2;
        while (hp.replicas > 1 && (uint64_t)nsegs * (uint64_t)num_candidates * hp.replicas * sizeof(MaxPair) > kBoardBudgetBytes)
            hp.replicas /= 2;

        // The items of one 2-D block of segment s: `rows` rows whose first starts at byte cand_base in the candidates and
        // is compared with what lies at ref_base in the reference; the block's first element has flat index elem_base.
        const auto emit_block = [&](uint64_t s, uint64_t cand_base, uint64_t ref_base, uint64_t elem_base, uint64_t rows) {
            const SegDesc &g = segs[s];
            const uint64_t w = elem_size(g.dtype), per = elems_per_item(g.dtype);
            const bool mapped = seg_ref_mapped(g);
            const uint64_t ref_stride = mapped ? seg_ref_stride(g) : 1;
            // Short rows of a pitched segment that all start on 16-byte boundaries: whole rows are
            // grouped into one item, as many as its 256 vector slots hold (a row takes
            // ceil(row bytes / 16) of them), instead of one mostly idle item per row.
            const uint64_t row_vectors = (g.row_elems * w + 15) / 16;
            if (rows > 1 && cand_base % 16 == 0 && g.pitch_bytes % 16 == 0 && row_vectors <= kItemBytes / 32) {
                const uint64_t group = (kItemBytes / 16) / row_vectors;             // >= 2 rows per item
                for (uint64_t r = 0; r < rows; r += group) {
                    const uint64_t rows_here = std::min<uint64_t>(group, rows - r);
                    geak_item it{};
                    it.byte_offset = cand_base + r * g.pitch_bytes;
                    it.elem_start = elem_base + r * g.row_elems;
                    it.segment = (uint32_t)s;
                    it.numel = (uint16_t)(rows_here * g.row_elems);                 // at most 4096 / w elements
                    it.next = kNoItem;
                    it.dtype = (uint8_t)g.dtype;
                    // rows of whole vectors, a group's offsets within 32 bits, the reference's rows (if they are its own)
                    // contiguous or one element each: streamed like a full item (slots that the group leaves idle read as 0)
                    constexpr uint64_t kOffsetLimit = (1ull << 32) - kItemBytes;      // a row's offset plus a vector's within the row: 32 bits
                    const bool stream = (g.row_elems * w) % 16 == 0 && (group - 1) * g.pitch_bytes < kOffsetLimit &&
                                        (!mapped || (ref_stride <= 1 && (group - 1) * g.ref_pitch_bytes < kOffsetLimit));
                    it.flags = (uint8_t)(GEAK_ITEM_ALIGNED | GEAK_ITEM_ROWS | (mapped ? GEAK_ITEM_REFMAP : 0) | (stream ? GEAK_ITEM_STREAM : 0));
                    hp.items.push_back(it);
                    if (any_mapped) hp.ref_item_offset.push_back(mapped ? ref_base + r * g.ref_pitch_bytes : it.byte_offset);
                }
                return;
            }
            // Row by row (a contiguous segment is one row): full items and a tail.  A row that starts off the
            // 16-byte grid begins with one item that ends where a full item read from the boundary before
            // it would end (the kernels read it from that boundary and ignore the foreign elements in
            // front), so that everything behind it is aligned again.
            for (uint64_t r = 0; r < rows; ++r) {
                const uint64_t row_start = cand_base + r * g.pitch_bytes;
                uint64_t done = 0;
                auto push = [&](uint64_t n, bool full) {
                    geak_item it{};
                    it.byte_offset = row_start + payload_bytes(g.dtype, done);     // done is a multiple of 4096 for the sub-byte formats
                    it.elem_start = elem_base + r * g.row_elems + done;
                    it.segment = (uint32_t)s;
                    it.numel = (uint16_t)n;
                    it.next = kNoItem;
                    it.dtype = (uint8_t)g.dtype;
                    // a full item needs a contiguous reference slice: with one reference element per row, or a strided
                    // reference row, the item takes the guarded path
                    it.flags = (uint8_t)((full && ref_stride == 1 ? GEAK_ITEM_FULL : 0) | (it.byte_offset % 16 == 0 ? GEAK_ITEM_ALIGNED : 0) |
                                         (mapped ? GEAK_ITEM_REFMAP : 0));
                    hp.items.push_back(it);
                    if (any_mapped)
                        hp.ref_item_offset.push_back(!mapped ? it.byte_offset
                                                     : ref_base + r * g.ref_pitch_bytes + done * ref_stride * w);
                    done += n;
                };
                const uint64_t skip = (row_start % 16) / w;
                if (skip) push(std::min<uint64_t>(g.row_elems, per - skip), false);
                while (g.row_elems - done >= per) push(per, true);
                if (g.row_elems - done) push(g.row_elems - done, false);
            }
        };
        for (uint64_t s = 0; s < nsegs; ++s) {
            const SegDesc &g = segs[s];
            if (!g.numel) continue;
            if (!seg_is_nd(g)) {
                emit_block(s, g.byte_offset, g.ref_byte_offset, 0, seg_rows(g));
                continue;
            }
            const SegNd &o = nd[s];                           // blocks in row-major order of the outer dimensions
            const uint64_t block_elems = o.inner_rows * g.row_elems;
            for (uint64_t o0 = 0; o0 < o.outer_shape[0]; ++o0)
                for (uint64_t o1 = 0; o1 < o.outer_shape[1]; ++o1)
                    emit_block(s, g.byte_offset + o0 * o.outer_stride[0] + o1 * o.outer_stride[1],
                               g.ref_byte_offset + o0 * o.outer_ref_stride[0] + o1 * o.outer_ref_stride[1],
                               (o0 * o.outer_shape[1] + o1) * block_elems, o.inner_rows);
        }

        if (hp.items.size() != n_items) return GEAK_EINVAL;     // the closed-form count and the table must agree

        // Partition of the table over the persistent grid.  Block b owns the contiguous item range
        // [block_first[b], block_first[b + 1]); its four waves interleave inside it (wave w takes every
        // fourth item starting at w).  A wave's consecutive items are then neighbours in memory and
        // mostly of one segment, so the running maxima it has just raised are the right thresholds
        // for its next item.  Ranges are cut at equal estimated cost, not equal item count.  A wave is
        // latency-bound per 4 KiB slice, so an item costs about one unit per slice it streams
        // (reference + K candidates); measured per wave on mixed batches, a binary16 slice (twice the
        // elements) takes about 1.3 times, a bfloat16 slice 1.2 times and an int32 slice 0.8 times as
        // long as a binary32 one.  Every fresh start of the stream (a new segment, a tail) is priced at
        // about six slice times whatever K is -- nothing hides its first loads, and waves with many
        // starts were the last to finish until they were priced this high -- and a tail at a full
        // item on top of that, whatever its length.  Units: sixteenths of a binary32 slice.  A regression of
        // per-wave durations on what each wave's list holds, over four seeds of the ragged batch at K = 4 and
        // batches at K = 8 and K = 16, gives 16 / 20 / 19 / 13 per binary32 / binary16 / bfloat16 / int32 slice,
        // about 50 for a start and 1.3 slices' worth plus 80 for a tail; planning with those instead moves the
        // kernel's duration by -1.8 % to +2.4 % depending on the seed, inside the run-to-run spread, so the
        // constants below stand.  What the model cannot see -- which compute unit a block lands on, how many of
        // a segment's elements trip the maxima filters -- leaves blocks of equal estimated cost 5 % apart.
        const uint64_t blocks_wanted = (n_items + kWavesPerBlock - 1) / kWavesPerBlock;
        const uint64_t target_blocks = std::max<uint64_t>(1, std::min<uint64_t>(max_blocks, blocks_wanted));
        const uint64_t slices = (uint64_t)num_candidates + 1;
        auto item_cost = [&](const geak_item &it, bool starts_run) -> uint64_t {
            const uint64_t per_slice = is_mx_dtype(it.dtype) ? 48 : (it.dtype == GEAK_F8E4M3 || it.dtype == GEAK_F8E5M2) ? 40 : (it.dtype == GEAK_F32 || it.dtype == GEAK_F64) ? 16 : it.dtype == GEAK_BF16 ? 19 : it.dtype == GEAK_F16 ? 21 : 13;   // integers: 13
            if (!(it.flags & (GEAK_ITEM_FULL | GEAK_ITEM_STREAM))) return per_slice * slices + 140;       // tails, ragged row groups, starts off the grid
            return per_slice * slices + (starts_run ? 100 : 0);
        };
        // What the blocks that share a compute unit cost it together.  The waves of a compute unit slow each other
        // down until they finish nearly together (measured on mixed batches: 4 us of spread between the blocks of a
        // unit, 11 us between units when only the blocks are balanced), and what their common duration follows is
        // the number of slices the unit streams, whatever their dtype: the heavier arithmetic of a 16-bit slice
        // delays its own wave inside the unit, not the unit.  A start costs the unit about seven slices, a tail
        // about two thirds of a full item.  (The 8-bit floating and block-scaled formats are bound by arithmetic
        // for the unit as a whole and keep their per-wave weight.)  Balancing the units this way takes the spread
        // of their mean durations from 11 to 7 us on the ragged benchmark batch and its kernel from 241 to 234 us;
        // what is left does not follow anything the planner can count.
        auto unit_cost = [&](const geak_item &it, bool starts_run) -> uint64_t {
            const uint64_t per_slice = is_mx_dtype(it.dtype) ? 48 : (it.dtype == GEAK_F8E4M3 || it.dtype == GEAK_F8E5M2) ? 40 : 16;
            if (!(it.flags & (GEAK_ITEM_FULL | GEAK_ITEM_STREAM))) return per_slice * slices * kUnitTailMul16 / 16 + kUnitTailFix;
            return per_slice * slices + (starts_run ? kUnitStart : 0);
        };
        const auto starts = [&](uint64_t j) { return j > 0 && hp.items[j - 1].segment != hp.items[j].segment; };
        // Cuts items [begin, end) into `parts` contiguous ranges of equal cost, none of them with fewer than `least`
        // items (end - begin >= parts * least); the boundaries after the first are appended to `out`.
        const auto cut = [&](uint64_t begin, uint64_t end, uint64_t parts, uint64_t least, auto &&cost, std::vector<uint32_t> &out) {
            uint64_t total = 0, acc = 0, opened = 1, last = begin;
            for (uint64_t j = begin; j < end; ++j) total += cost(hp.items[j], starts(j));
            for (uint64_t j = begin; j < end; ++j) {
                // close the current range before item j once its share of the total is reached, or when the ranges
                // still to open need every item that is left
                if (opened < parts && j - last >= least && (acc * parts >= total * opened || end - j <= (parts - opened) * least)) {
                    out.push_back((uint32_t)j);
                    last = j;
                    ++opened;
                }
                acc += cost(hp.items[j], starts(j));
            }
        };
        // One step: ranges of equal cost to a wave.
        hp.block_first.clear();
        hp.block_first.push_back(0);
        cut(0, hp.items.size(), target_blocks, 1, item_cost, hp.block_first);
        hp.unit_groups = 1;
        hp.block_map = GEAK_MAP_PLAIN;
        // A grid that fills the chip is dispatched round by round: block b lands on compute unit b mod (number of
        // units), so blocks b, b + units, b + 2 units, ... share one.  Where the one-step ranges would leave the units
        // with unequal loads (a batch of mixed dtypes and sizes; never a dense tensor), the table is cut in two steps
        // instead: into as many ranges as there are units, equal in what they cost a unit, and each of those into the
        // ranges of the unit's blocks, equal in what they cost a wave.  Which block runs which range of the table:
        // hp.block_map and table_range_of_block() (device_common.hpp).
        const uint64_t per_unit = target_blocks / compute_units;
        if (target_blocks == max_blocks && per_unit >= 2 && per_unit * compute_units == target_blocks && compute_units % 8 == 0 &&
            hp.items.size() >= target_blocks) {
            hp.unit_groups = compute_units;
            hp.block_map = GEAK_MAP_ROTATED;               // the plain table; only the XCDs take turns (device_common.hpp)
            std::vector<uint64_t> load(compute_units, 0);
            for (uint64_t r = 0; r < target_blocks; ++r) {
                const uint64_t end = r + 1 < target_blocks ? hp.block_first[r + 1] : hp.items.size();
                for (uint64_t j = hp.block_first[r]; j < end; ++j) load[r % compute_units] += unit_cost(hp.items[j], starts(j));
            }
            const uint64_t least = *std::min_element(load.begin(), load.end()), most = *std::max_element(load.begin(), load.end());
            if ((most - least) * kUnitSpreadDen > most * kUnitSpreadNum) {
                std::vector<uint32_t> unit_first, ranges;
                unit_first.push_back(0);
                cut(0, hp.items.size(), compute_units, per_unit, unit_cost, unit_first);
                unit_first.push_back((uint32_t)hp.items.size());
                ranges.push_back(0);
                for (uint64_t u = 0; u < compute_units; ++u) {
                    if (u) ranges.push_back(unit_first[u]);
                    cut(unit_first[u], unit_first[u + 1], per_unit, 1, item_cost, ranges);
                }
                if (ranges.size() == target_blocks) {       // always: every unit's range holds at least per_unit items
                    hp.block_first.swap(ranges);
                    hp.block_map = GEAK_MAP_BY_UNIT;
                }
            }
        }
        hp.block_first.push_back((uint32_t)hp.items.size());
        hp.grid_blocks = (uint32_t)(hp.block_first.size() - 1);    // >= 1; the last entry closes the last block
        if (hp.items.empty()) hp.grid_blocks = 1;

        // Inside a block every item goes to the wave that has the least estimated cost so far (in
        // table order, so a wave's list ascends and neighbouring items mostly go to neighbouring
        // waves): with equal items that is a plain interleave, and a tail, a start off the grid or a heavier dtype
        // no longer makes one wave of the block finish an item or two after the others.  Each wave
        // follows its list through the items' `next` links.
        //
        // Runs and slots.  Scanning the table in order, a wave opens a new run (and a new slot)
        // whenever the segment of its next item differs from the segment of its previous one.
        // Items of one segment are contiguous in the table, so the slots opened while scanning a
        // segment are contiguous too.
        const uint64_t workers = (uint64_t)hp.grid_blocks * kWavesPerBlock;
        hp.wave_first.assign(workers, kNoItem);
        std::vector<uint32_t> run_segment(workers, 0xFFFFFFFFu), run_slot(workers, 0), last_item(workers, kNoItem);
        std::vector<uint64_t> load(workers, 0);
        uint64_t slot_cursor = 0;
        uint64_t seg_cursor = 0;
        uint64_t block = 0;
        for (uint64_t j = 0; j < hp.items.size(); ++j) {
            geak_item &it = hp.items[j];
            while (seg_cursor <= it.segment) hp.slot_begin[seg_cursor++] = (uint32_t)slot_cursor;
            while (j >= hp.block_first[block + 1]) ++block;
            uint64_t worker = block * kWavesPerBlock;
            for (uint64_t w = worker + 1; w < (block + 1) * kWavesPerBlock; ++w)
                if (load[w] < load[worker]) worker = w;
            const bool new_run = run_segment[worker] != it.segment;
            load[worker] += item_cost(it, new_run);
            if (last_item[worker] == kNoItem) hp.wave_first[worker] = (uint32_t)j;
            else hp.items[last_item[worker]].next = (uint32_t)j;
            if (new_run) {
                if (last_item[worker] != kNoItem) hp.items[last_item[worker]].flags |= GEAK_ITEM_LAST;
                run_segment[worker] = it.segment;
                run_slot[worker] = (uint32_t)slot_cursor++;
                it.flags |= GEAK_ITEM_FIRST;
                if (slot_cursor >= 0x7FFFFFFFull) return GEAK_EBOUNDS;
            }
            it.slot = run_slot[worker];
            last_item[worker] = (uint32_t)j;
        }
        for (uint64_t wk = 0; wk < workers; ++wk)
            if (last_item[wk] != kNoItem) hp.items[last_item[wk]].flags |= GEAK_ITEM_LAST;
        while (seg_cursor <= nsegs) hp.slot_begin[seg_cursor++] = (uint32_t)slot_cursor;
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    return GEAK_OK;
}

}  // namespace geak
