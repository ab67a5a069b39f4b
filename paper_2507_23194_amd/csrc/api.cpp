// C-ABI entry points: plan lifetime, argument checks, kernel enqueue.  See include/geak_check.h.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cstring>
#include <new>
#include "geak_internal.hpp"

using namespace geak;

struct geak_plan {
    HostPlan host;
    int device = -1;
    uint32_t lds_bytes = 0;
    // device copies of the work table
    geak_item *items_dev = nullptr;
    uint32_t *slot_begin_dev = nullptr;
    uint32_t *wave_first_dev = nullptr;
    SegDesc *segments_dev = nullptr;
    SegTol *seg_tol_dev = nullptr;
    uint64_t *ref_item_offset_dev = nullptr;     // only when a segment's reference has a layout of its own
    SegNd *nd_dev = nullptr;                     // only when a segment is N-d
    // optional timing ring
    std::vector<hipEvent_t> ev_start, ev_stop;
    uint32_t ev_next = 0, ev_used = 0;
};

namespace {

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
    }
    ~DeviceGuard() {
        int cur = -1;
        if (ok && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

void free_device_side(geak_plan *p)
{
    if (p->device < 0) return;
    DeviceGuard g(p->device);
    if (p->items_dev) (void)hipFree(p->items_dev);
    if (p->slot_begin_dev) (void)hipFree(p->slot_begin_dev);
    if (p->wave_first_dev) (void)hipFree(p->wave_first_dev);
    if (p->segments_dev) (void)hipFree(p->segments_dev);
    if (p->seg_tol_dev) (void)hipFree(p->seg_tol_dev);
    if (p->ref_item_offset_dev) (void)hipFree(p->ref_item_offset_dev);
    if (p->nd_dev) (void)hipFree(p->nd_dev);
    for (auto e : p->ev_start) (void)hipEventDestroy(e);
    for (auto e : p->ev_stop) (void)hipEventDestroy(e);
    p->items_dev = nullptr;
    p->slot_begin_dev = nullptr;
    p->wave_first_dev = nullptr;
    p->segments_dev = nullptr;
    p->seg_tol_dev = nullptr;
    p->ref_item_offset_dev = nullptr;
    p->nd_dev = nullptr;
    p->ev_start.clear();
    p->ev_stop.clear();
}

}  // namespace

extern "C" {

geak_status geak_check_plan(geak_plan **out, const geak_segment *segs, uint64_t nsegs, int32_t num_candidates,
                            double atol, double rtol, int32_t equal_nan, int32_t device)
{
    if (!segs || nsegs == 0 || nsegs > 0x7FFFFFFFull) return GEAK_EINVAL;
    std::vector<geak_tolerance> tols;
    try {
        tols.assign(nsegs, geak_tolerance{atol, rtol});
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    return geak_check_plan_tolerances(out, segs, tols.data(), nsegs, num_candidates, equal_nan, device);
}

static geak_status plan_from_descs(geak_plan **out, const SegDesc *segs, const geak_tolerance *tols, uint64_t nsegs,
                                   int32_t num_candidates, int32_t equal_nan, int32_t device, const SegNd *nd = nullptr);

geak_status geak_check_plan_tolerances(geak_plan **out, const geak_segment *segs, const geak_tolerance *tols,
                                       uint64_t nsegs, int32_t num_candidates, int32_t equal_nan, int32_t device)
{
    if (!segs || nsegs == 0 || nsegs > 0x7FFFFFFFull) return GEAK_EINVAL;
    std::vector<SegDesc> descs;
    try {
        descs.resize(nsegs);
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    for (uint64_t s = 0; s < nsegs; ++s) {                 // a contiguous segment is one row
        const geak_segment &g = segs[s];
        const uint64_t w = (g.dtype >= GEAK_F32 && g.dtype <= GEAK_F8E5M2) ? (uint64_t)elem_size(g.dtype) : 1;
        descs[s] = SegDesc{g.byte_offset, g.numel, g.numel ? g.numel : 1, g.numel <= UINT64_MAX / w ? g.numel * w : 0, g.dtype, 0, 0, 0};
        if (g.reserved != 0) return GEAK_EINVAL;
    }
    return plan_from_descs(out, descs.data(), tols, nsegs, num_candidates, equal_nan, device);
}

geak_status geak_check_plan_pitched(geak_plan **out, const geak_segment2d *segs, const geak_tolerance *tols, uint64_t nsegs,
                                    int32_t num_candidates, double atol, double rtol, int32_t equal_nan, int32_t device)
{
    if (!segs || nsegs == 0 || nsegs > 0x7FFFFFFFull) return GEAK_EINVAL;
    std::vector<SegDesc> descs;
    std::vector<geak_tolerance> same;
    try {
        descs.resize(nsegs);
        if (!tols) same.assign(nsegs, geak_tolerance{atol, rtol});
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    for (uint64_t s = 0; s < nsegs; ++s) {
        const geak_segment2d &g = segs[s];
        if (g.rows && g.row_elems > GEAK_MAX_SEGMENT_NUMEL / g.rows) return GEAK_EBOUNDS;
        const uint64_t numel = g.rows * g.row_elems;
        const uint64_t w = (g.dtype >= GEAK_F32 && g.dtype <= GEAK_F8E5M2) ? (uint64_t)elem_size(g.dtype) : 1;
        if (g.reserved != 0) return GEAK_EINVAL;
        SegDesc d{g.byte_offset, numel, numel ? g.row_elems : 1, g.pitch_bytes, g.dtype, 0, 0, 0};
        if (numel && g.row_elems <= UINT64_MAX / w && g.pitch_bytes == g.row_elems * w) {    // rows back to back: one row
            d.row_elems = numel;
            d.pitch_bytes = numel * w;                  // numel <= 2^40
        }
        if (!numel) d.pitch_bytes = 0;
        descs[s] = d;
    }
    return plan_from_descs(out, descs.data(), tols ? tols : same.data(), nsegs, num_candidates, equal_nan, device);
}

geak_status geak_check_plan_mx(geak_plan **out, const geak_segment_mx *segs, const geak_tolerance *tols, uint64_t nsegs,
                               int32_t num_candidates, double atol, double rtol, int32_t equal_nan, int32_t device)
{
    if (!segs || nsegs == 0 || nsegs > 0x7FFFFFFFull) return GEAK_EINVAL;
    std::vector<SegDesc> descs;
    std::vector<geak_tolerance> same;
    try {
        descs.resize(nsegs);
        if (!tols) same.assign(nsegs, geak_tolerance{atol, rtol});
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    for (uint64_t s = 0; s < nsegs; ++s) {
        const geak_segment_mx &g = segs[s];
        if (g.reserved != 0) return GEAK_EINVAL;
        if (!is_mx_dtype(g.dtype)) return GEAK_EDTYPE;
        // one contiguous row of one-byte elements; the scales' offset travels in the record's reference field
        descs[s] = SegDesc{g.byte_offset, g.numel, g.numel ? g.numel : 1, payload_bytes(g.dtype, g.numel), g.dtype, kMxScaled, g.scale_byte_offset, 0};
    }
    return plan_from_descs(out, descs.data(), tols ? tols : same.data(), nsegs, num_candidates, equal_nan, device);
}

geak_status geak_check_plan_table(geak_plan **out, const geak_segment_any *segs, const geak_tolerance *tols, uint64_t nsegs,
                                  int32_t num_candidates, double atol, double rtol, int32_t equal_nan, int32_t device)
{
    if (!segs || nsegs == 0 || nsegs > 0x7FFFFFFFull) return GEAK_EINVAL;
    std::vector<SegDesc> descs;
    std::vector<geak_tolerance> same;
    try {
        descs.resize(nsegs);
        if (!tols) same.assign(nsegs, geak_tolerance{atol, rtol});
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    for (uint64_t s = 0; s < nsegs; ++s) {                 // each kind exactly as its own entry point builds it
        const geak_segment_any &g = segs[s];
        if (g.reserved != 0) return GEAK_EINVAL;
        if (g.rows && g.row_elems > GEAK_MAX_SEGMENT_NUMEL / g.rows) return GEAK_EBOUNDS;
        const uint64_t numel = g.rows * g.row_elems;
        if (g.kind == GEAK_KIND_PITCHED) {
            if (g.aux_byte_offset || g.aux_pitch_bytes || g.ref_elem_stride) return GEAK_EINVAL;
            if (is_mx_dtype(g.dtype)) return GEAK_EDTYPE;
            const uint64_t w = (g.dtype >= GEAK_F32 && g.dtype <= GEAK_F8E5M2) ? (uint64_t)elem_size(g.dtype) : 1;
            SegDesc d{g.byte_offset, numel, numel ? g.row_elems : 1, g.pitch_bytes, g.dtype, 0, 0, 0};
            if (numel && g.row_elems <= UINT64_MAX / w && g.pitch_bytes == g.row_elems * w) {    // rows back to back: one row
                d.row_elems = numel;
                d.pitch_bytes = numel * w;
            }
            if (!numel) d.pitch_bytes = 0;
            descs[s] = d;
        } else if (g.kind == GEAK_KIND_MAPPED) {
            if (g.ref_elem_stride < 0) return GEAK_EINVAL;
            if ((uint64_t)g.ref_elem_stride > kMaxRefStride) return GEAK_EBOUNDS;
            if (is_mx_dtype(g.dtype)) return GEAK_EDTYPE;
            descs[s] = SegDesc{g.byte_offset, numel, numel ? g.row_elems : 1, numel ? g.pitch_bytes : 0, g.dtype,
                               kRefMapped | (int32_t)((uint32_t)g.ref_elem_stride << kRefStrideShift), g.aux_byte_offset,
                               numel ? g.aux_pitch_bytes : 0};
        } else if (g.kind == GEAK_KIND_MX) {
            if (g.rows > 1 || g.pitch_bytes || g.aux_pitch_bytes || g.ref_elem_stride) return GEAK_EINVAL;
            if (!is_mx_dtype(g.dtype)) return GEAK_EDTYPE;
            descs[s] = SegDesc{g.byte_offset, numel, numel ? numel : 1, payload_bytes(g.dtype, numel), g.dtype, kMxScaled, g.aux_byte_offset, 0};
        } else {
            return GEAK_EINVAL;
        }
    }
    return plan_from_descs(out, descs.data(), tols ? tols : same.data(), nsegs, num_candidates, equal_nan, device);
}

geak_status geak_check_plan_mapped(geak_plan **out, const geak_segment_mapped *segs, const geak_tolerance *tols, uint64_t nsegs,
                                   int32_t num_candidates, double atol, double rtol, int32_t equal_nan, int32_t device)
{
    if (!segs || nsegs == 0 || nsegs > 0x7FFFFFFFull) return GEAK_EINVAL;
    std::vector<SegDesc> descs;
    std::vector<geak_tolerance> same;
    try {
        descs.resize(nsegs);
        if (!tols) same.assign(nsegs, geak_tolerance{atol, rtol});
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    for (uint64_t s = 0; s < nsegs; ++s) {
        const geak_segment_mapped &g = segs[s];
        if (g.ref_elem_stride < 0) return GEAK_EINVAL;
        if ((uint64_t)g.ref_elem_stride > kMaxRefStride) return GEAK_EBOUNDS;
        if (g.rows && g.row_elems > GEAK_MAX_SEGMENT_NUMEL / g.rows) return GEAK_EBOUNDS;
        const uint64_t numel = g.rows * g.row_elems;
        // the rows stay rows, also when the candidates store them back to back: the reference's row differs
        SegDesc d{g.byte_offset, numel, numel ? g.row_elems : 1, numel ? g.pitch_bytes : 0, g.dtype,
                  kRefMapped | (int32_t)((uint32_t)g.ref_elem_stride << kRefStrideShift), g.ref_byte_offset, numel ? g.ref_pitch_bytes : 0};
        descs[s] = d;
    }
    return plan_from_descs(out, descs.data(), tols ? tols : same.data(), nsegs, num_candidates, equal_nan, device);
}

geak_status geak_check_plan_nd(geak_plan **out, const geak_segment_nd *segs, const geak_tolerance *tols, uint64_t nsegs,
                               int32_t num_candidates, double atol, double rtol, int32_t equal_nan, int32_t device)
{
    if (!segs || nsegs == 0 || nsegs > 0x7FFFFFFFull) return GEAK_EINVAL;
    std::vector<SegDesc> descs;
    std::vector<SegNd> nds;
    std::vector<geak_tolerance> same;
    try {
        descs.resize(nsegs);
        nds.assign(nsegs, SegNd{1, {1, 1}, {0, 0}, {0, 0}});
        if (!tols) same.assign(nsegs, geak_tolerance{atol, rtol});
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    bool any_nd = false;
    for (uint64_t s = 0; s < nsegs; ++s) {
        const geak_segment_nd &g = segs[s];
        if (g.ndim < 0 || g.ndim > GEAK_MAX_DIMS) return GEAK_EINVAL;
        if (g.dtype < GEAK_F32 || g.dtype > GEAK_F8E5M2) return GEAK_EDTYPE;
        const uint64_t w = (uint64_t)elem_size(g.dtype);
        // the dimensions that matter, outermost first: extents of 1 dropped, neighbours that both tensors step through
        // in one stride merged (an empty tensor has no dimensions to look at)
        uint64_t shape[GEAK_MAX_DIMS], stride[GEAK_MAX_DIMS], ref_stride[GEAK_MAX_DIMS], numel = 1;
        int n = 0;
        bool empty = false;
        for (int d = 0; d < g.ndim; ++d) empty |= g.shape[d] == 0;
        for (int d = 0; d < g.ndim && !empty; ++d) {
            if (g.shape[d] > GEAK_MAX_SEGMENT_NUMEL || numel > GEAK_MAX_SEGMENT_NUMEL / g.shape[d]) return GEAK_EBOUNDS;
            numel *= g.shape[d];
            if (g.shape[d] == 1) continue;                      // its strides are never stepped
            if (g.stride_bytes[d] % w || g.ref_stride_bytes[d] % w) return GEAK_EALIGN;
            // dimension n - 1 steps over all of dimension d in both tensors: one dimension (products below 2^40 * 2^64 are
            // compared by division)
            if (n && g.stride_bytes[d] && stride[n - 1] / g.shape[d] == g.stride_bytes[d] && stride[n - 1] % g.shape[d] == 0 &&
                ((ref_stride[n - 1] == 0 && g.ref_stride_bytes[d] == 0) ||
                 (g.ref_stride_bytes[d] && ref_stride[n - 1] / g.shape[d] == g.ref_stride_bytes[d] && ref_stride[n - 1] % g.shape[d] == 0))) {
                shape[n - 1] *= g.shape[d];
                stride[n - 1] = g.stride_bytes[d];
                ref_stride[n - 1] = g.ref_stride_bytes[d];
            } else {
                shape[n] = g.shape[d];
                stride[n] = g.stride_bytes[d];
                ref_stride[n] = g.ref_stride_bytes[d];
                ++n;
            }
        }
        if (empty) numel = 0;
        if (numel == 0) {
            descs[s] = SegDesc{g.byte_offset, 0, 1, 0, g.dtype, kRefMapped | (1 << kRefStrideShift), g.ref_byte_offset, 0};
            continue;
        }
        if (n == 0) { shape[0] = 1; stride[0] = w; ref_stride[0] = w; n = 1; }          // one element
        if (stride[n - 1] != w) {
            // the candidates' innermost dimension must be contiguous -- unless its extent is 1 (a column of a wider array:
            // dropped above), then the rows are one element long
            if (g.shape[g.ndim - 1] != 1) return GEAK_EINVAL;
            shape[n] = 1; stride[n] = w; ref_stride[n] = w;    // n <= GEAK_MAX_DIMS - 1: the innermost dimension was dropped
            ++n;
        }
        if (ref_stride[n - 1] / w > kMaxRefStride) return GEAK_EBOUNDS;
        const uint64_t row_elems = shape[n - 1];
        const uint64_t rows = n >= 2 ? shape[n - 2] : 1;
        int32_t layout = kRefMapped | (int32_t)((uint32_t)(ref_stride[n - 1] / w) << kRefStrideShift);
        if (n > 2) {
            layout |= kSegNd;
            any_nd = true;
            SegNd &o = nds[s];
            o.inner_rows = rows;
            // dimensions n - 3 and, if there is one, n - 4: the inner of the two in slot 1
            o.outer_shape[1] = shape[n - 3];
            o.outer_stride[1] = stride[n - 3];
            o.outer_ref_stride[1] = ref_stride[n - 3];
            if (n == 4) {
                o.outer_shape[0] = shape[0];
                o.outer_stride[0] = stride[0];
                o.outer_ref_stride[0] = ref_stride[0];
            }
        }
        descs[s] = SegDesc{g.byte_offset, numel, row_elems, n >= 2 ? stride[n - 2] : row_elems * w, g.dtype, layout, g.ref_byte_offset,
                           n >= 2 ? ref_stride[n - 2] : 0};
    }
    return plan_from_descs(out, descs.data(), tols ? tols : same.data(), nsegs, num_candidates, equal_nan, device, any_nd ? nds.data() : nullptr);
}

static geak_status plan_from_descs(geak_plan **out, const SegDesc *segs, const geak_tolerance *tols, uint64_t nsegs,
                                   int32_t num_candidates, int32_t equal_nan, int32_t device, const SegNd *nd)
{
    if (!out) return GEAK_EINVAL;
    if (device < -1) return GEAK_EINVAL;
    if (num_candidates < 1 || num_candidates > GEAK_MAX_CANDIDATES) return GEAK_EINVAL;
    if (nsegs > 0x7FFFFFFFull / GEAK_MAX_CANDIDATES) return GEAK_EINVAL;   // one reduce block per record

    geak_plan *p = new (std::nothrow) geak_plan;
    if (!p) return GEAK_ENOMEM;
    p->device = device;
    p->lds_bytes = lds_bytes_for(num_candidates);

    uint32_t max_blocks = (uint32_t)(kDefaultComputeUnits * kDefaultBlocksPerCU), compute_units = (uint32_t)kDefaultComputeUnits;
    if (device >= 0) {
        int n_dev = 0;
        if (hipGetDeviceCount(&n_dev) != hipSuccess || device >= n_dev) { delete p; return GEAK_EHIP; }
        DeviceGuard g(device);
        hipDeviceProp_t prop;
        if (!g.ok || hipGetDeviceProperties(&prop, device) != hipSuccess) { delete p; return GEAK_EHIP; }
        const int per_cu = compare_blocks_per_cu(p->lds_bytes);
        if (per_cu <= 0 || prop.multiProcessorCount <= 0) { delete p; return GEAK_EHIP; }
        max_blocks = (uint32_t)prop.multiProcessorCount * (uint32_t)per_cu;
        compute_units = (uint32_t)prop.multiProcessorCount;
    }

    geak_status st = build_host_plan(p->host, segs, tols, nsegs, num_candidates, equal_nan, max_blocks, compute_units, nd);
    if (st != GEAK_OK) { delete p; return st; }

    if (device >= 0) {
        DeviceGuard g(device);
        const size_t item_bytes = p->host.items.size() * sizeof(geak_item);
        const size_t slot_bytes = p->host.slot_begin.size() * sizeof(uint32_t);
        bool ok = g.ok;
        if (ok && item_bytes) ok = hipMalloc((void **)&p->items_dev, item_bytes) == hipSuccess;
        const size_t wave_bytes = p->host.wave_first.size() * sizeof(uint32_t);
        if (ok) ok = hipMalloc((void **)&p->slot_begin_dev, slot_bytes) == hipSuccess;
        if (ok) ok = hipMalloc((void **)&p->wave_first_dev, wave_bytes) == hipSuccess;
        const size_t seg_bytes = p->host.segments.size() * sizeof(SegDesc);
        if (ok) ok = hipMalloc((void **)&p->segments_dev, seg_bytes) == hipSuccess;
        const size_t tol_bytes = p->host.seg_tol.size() * sizeof(SegTol);
        if (ok) ok = hipMalloc((void **)&p->seg_tol_dev, tol_bytes) == hipSuccess;
        const size_t ref_off_bytes = p->host.ref_item_offset.size() * sizeof(uint64_t);
        if (ok && ref_off_bytes) ok = hipMalloc((void **)&p->ref_item_offset_dev, ref_off_bytes) == hipSuccess;
        const size_t nd_bytes = p->host.nd.size() * sizeof(SegNd);
        if (ok && nd_bytes) ok = hipMalloc((void **)&p->nd_dev, nd_bytes) == hipSuccess;
        if (!ok) { free_device_side(p); delete p; return GEAK_ENOMEM; }
        if (item_bytes) ok = hipMemcpy(p->items_dev, p->host.items.data(), item_bytes, hipMemcpyHostToDevice) == hipSuccess;
        if (ok) ok = hipMemcpy(p->slot_begin_dev, p->host.slot_begin.data(), slot_bytes, hipMemcpyHostToDevice) == hipSuccess;
        if (ok) ok = hipMemcpy(p->wave_first_dev, p->host.wave_first.data(), wave_bytes, hipMemcpyHostToDevice) == hipSuccess;
        if (ok) ok = hipMemcpy(p->segments_dev, p->host.segments.data(), seg_bytes, hipMemcpyHostToDevice) == hipSuccess;
        if (ok) ok = hipMemcpy(p->seg_tol_dev, p->host.seg_tol.data(), tol_bytes, hipMemcpyHostToDevice) == hipSuccess;
        if (ok && ref_off_bytes)
            ok = hipMemcpy(p->ref_item_offset_dev, p->host.ref_item_offset.data(), ref_off_bytes, hipMemcpyHostToDevice) == hipSuccess;
        if (ok && nd_bytes) ok = hipMemcpy(p->nd_dev, p->host.nd.data(), nd_bytes, hipMemcpyHostToDevice) == hipSuccess;
        if (!ok) { free_device_side(p); delete p; return GEAK_EHIP; }
        // set-up is the place to look up the device's copy of the static scratch array: geak_check_run_static
        // then finds the address there (a failure here only surfaces if that entry point is used)
        (void)static_scratch_address(device, nullptr);
    }
    *out = p;
    return GEAK_OK;
}

geak_status geak_check_plan_dense(geak_plan **out, int32_t dtype, const int64_t *shape, int32_t ndim,
                                  int32_t num_candidates, double atol, double rtol, int32_t equal_nan, int32_t device)
{
    if (ndim < 0 || (ndim > 0 && !shape)) return GEAK_EINVAL;
    uint64_t numel = 1;
    for (int i = 0; i < ndim; ++i) {
        if (shape[i] < 0) return GEAK_EINVAL;
        const uint64_t e = (uint64_t)shape[i];
        if (e != 0 && numel > GEAK_MAX_SEGMENT_NUMEL / e) {
            // keep scanning: a later zero extent makes the tensor empty
            bool zero_later = false;
            for (int j = i + 1; j < ndim; ++j) zero_later |= (shape[j] == 0);
            if (!zero_later) return GEAK_EBOUNDS;
            numel = 0;
            break;
        }
        numel *= e;
    }
    geak_segment seg;
    seg.byte_offset = 0;
    seg.numel = numel;
    seg.dtype = dtype;
    seg.reserved = 0;
    return geak_check_plan(out, &seg, 1, num_candidates, atol, rtol, equal_nan, device);
}

uint64_t geak_check_workspace_bytes(const geak_plan *plan)
{
    if (!plan || plan->host.items.empty()) return 0;
    const HostPlan &hp = plan->host;
    const uint64_t board = (uint64_t)hp.segments.size() * (uint64_t)hp.num_candidates * hp.replicas * sizeof(MaxPair);
    return kCandTableBytes + board + (uint64_t)hp.slot_begin.back() * (uint64_t)hp.num_candidates * sizeof(Partial);
}

uint64_t geak_check_result_count(const geak_plan *plan)
{
    if (!plan) return 0;
    return (uint64_t)plan->host.segments.size() * (uint64_t)plan->host.num_candidates;
}

// The tensor arguments of a call: the reference and the K candidate base pointers must be there
// when the plan reads any data, and aligned to the largest element size among the plan's segments
// (every element then sits at a multiple of its size).  Nothing more: a base off the 16-byte grid --
// a slice of a larger tensor -- is read with vector loads at odd addresses.
static geak_status check_tensor_pointers(const HostPlan &hp, const void *ref_dev, const void *const *cand_dev)
{
    const bool reads_data = !hp.items.empty();          // a plan of empty segments touches no tensor
    uintptr_t mask = 0;
    for (const SegDesc &g : hp.segments) mask |= (uintptr_t)elem_size(g.dtype) - 1u;
    if (reads_data && !ref_dev) return GEAK_EINVAL;
    if ((uintptr_t)ref_dev & mask) return GEAK_EALIGN;
    for (int k = 0; k < hp.num_candidates; ++k) {
        if (reads_data && !cand_dev[k]) return GEAK_EINVAL;
        if ((uintptr_t)cand_dev[k] & mask) return GEAK_EALIGN;
    }
    return GEAK_OK;
}

geak_status geak_check_run(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                           void *workspace_dev, geak_result *results_dev, void *hip_stream)
{
    if (!plan || !cand_dev || !results_dev) return GEAK_EINVAL;
    if (plan->device < 0) return GEAK_EINVAL;
    const HostPlan &hp = plan->host;
    const int K = hp.num_candidates;
    if (const geak_status st = check_tensor_pointers(hp, ref_dev, cand_dev)) return st;
    if ((uintptr_t)results_dev & 7u) return GEAK_EALIGN;
    const uint64_t ws_bytes = geak_check_workspace_bytes(plan);
    if (ws_bytes && !workspace_dev) return GEAK_EWORKSPACE;
    if (ws_bytes && ((uintptr_t)workspace_dev & 15u)) return GEAK_EALIGN;

    DeviceGuard g(plan->device);
    if (!g.ok) return GEAK_EHIP;

    // workspace: [candidate pointer table][partials]
    const uint64_t num_board = hp.items.empty() ? 0 : (uint64_t)hp.segments.size() * (uint64_t)K * hp.replicas;
    const unsigned char **cand_table = hp.items.empty() ? nullptr : (const unsigned char **)workspace_dev;
    MaxPair *board = hp.items.empty() ? nullptr : (MaxPair *)((unsigned char *)workspace_dev + kCandTableBytes);
    Partial *partials = hp.items.empty() ? nullptr : (Partial *)((unsigned char *)board + num_board * sizeof(MaxPair));

    InitArgs ia;
    ia.results = results_dev;
    ia.cand_table = cand_table;
    ia.board = board;
    ia.num_board = num_board;
    ia.num_results = geak_check_result_count(plan);
    ia.num_candidates = (uint32_t)K;
    ia.reserved = 0;
    for (int k = 0; k < GEAK_MAX_CANDIDATES; ++k) ia.cand[k] = (k < K) ? (const unsigned char *)cand_dev[k] : nullptr;
    if (launch_init(ia, hip_stream) != (int)hipSuccess) return GEAK_EHIP;

    if (!hp.items.empty()) {
        CompareArgs ca;
        ca.items = plan->items_dev;
        ca.ref = (const unsigned char *)ref_dev;
        ca.cand_table = cand_table;
        ca.partials = partials;
        ca.board = board;
        ca.replicas = hp.replicas;
        ca.unit_groups = hp.unit_groups;
        ca.num_items = (uint32_t)hp.items.size();
        ca.num_candidates = (uint32_t)K;
        ca.seg_tol = plan->seg_tol_dev;
        ca.equal_nan = hp.equal_nan;
        ca.block_map = hp.block_map;
        ca.wave_first = plan->wave_first_dev;
        ca.segments = plan->segments_dev;
        ca.ref_item_offset = plan->ref_item_offset_dev;

        geak_plan *mp = const_cast<geak_plan *>(plan);      // timing ring only; documented as not re-entrant
        const bool timed = !mp->ev_start.empty();
        const uint32_t slot = mp->ev_next;
        if (timed && hipEventRecord(mp->ev_start[slot], (hipStream_t)hip_stream) != hipSuccess) return GEAK_EHIP;
        if (launch_compare(ca, hp.grid_blocks, plan->lds_bytes, hip_stream) != (int)hipSuccess) return GEAK_EHIP;
        if (timed) {
            if (hipEventRecord(mp->ev_stop[slot], (hipStream_t)hip_stream) != hipSuccess) return GEAK_EHIP;
            mp->ev_next = (slot + 1) % (uint32_t)mp->ev_start.size();
            if (mp->ev_used < mp->ev_start.size()) ++mp->ev_used;
        }

        ReduceArgs ra;
        ra.items = plan->items_dev;
        ra.slot_begin = plan->slot_begin_dev;
        ra.partials = partials;
        ra.board = board;
        ra.results = results_dev;
        ra.ref = (const unsigned char *)ref_dev;
        ra.cand_table = cand_table;
        ra.num_segments = (uint32_t)hp.segments.size();
        ra.num_candidates = (uint32_t)K;
        ra.seg_tol = plan->seg_tol_dev;
        ra.equal_nan = hp.equal_nan;
        ra.replicas = hp.replicas;
        ra.segments = plan->segments_dev;
        ra.ref_item_offset = plan->ref_item_offset_dev;
        if (launch_reduce(ra, hip_stream) != (int)hipSuccess) return GEAK_EHIP;
    }
    return GEAK_OK;
}

void geak_check_destroy(geak_plan *plan)
{
    if (!plan) return;
    free_device_side(plan);
    delete plan;
}

#ifndef GEAK_BUILD_ID
#define GEAK_BUILD_ID "unknown"
#endif
const char *geak_check_build_id(void) { return GEAK_BUILD_ID; }

const char *geak_status_string(geak_status status)
{
    switch (status) {
    case GEAK_OK: return "ok";
    case GEAK_EINVAL: return "invalid argument";
    case GEAK_EDTYPE: return "unknown dtype";
    case GEAK_EALIGN: return "misaligned offset or pointer";
    case GEAK_EBOUNDS: return "segment out of bounds, overlapping or too large";
    case GEAK_ENOMEM: return "out of memory";
    case GEAK_EWORKSPACE: return "workspace missing";
    case GEAK_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

geak_status geak_check_plan_info(const geak_plan *plan, geak_plan_info *out)
{
    if (!plan || !out) return GEAK_EINVAL;
    const HostPlan &hp = plan->host;
    out->num_segments = hp.segments.size();
    out->num_items = hp.items.size();
    out->num_slots = hp.slot_begin.back();
    out->algorithmic_bytes = hp.algorithmic_bytes;
    out->num_candidates = (uint32_t)hp.num_candidates;
    out->grid_blocks = hp.grid_blocks;
    out->block_threads = kBlockThreads;
    out->lds_bytes = plan->lds_bytes;
    out->item_bytes = kItemBytes;
    out->device = plan->device;
    out->unit_groups = hp.unit_groups;
    out->block_map = hp.block_map;
    return GEAK_OK;
}

uint64_t geak_check_plan_blocks(const geak_plan *plan, uint32_t *out, uint64_t capacity)
{
    if (!plan) return 0;
    const auto &bf = plan->host.block_first;
    if (out) {
        const uint64_t n = capacity < bf.size() ? capacity : bf.size();
        if (n) std::memcpy(out, bf.data(), n * sizeof(uint32_t));
    }
    return bf.size();
}

uint64_t geak_check_plan_waves(const geak_plan *plan, uint32_t *out, uint64_t capacity)
{
    if (!plan) return 0;
    const auto &wf = plan->host.wave_first;
    if (out) {
        const uint64_t n = capacity < wf.size() ? capacity : wf.size();
        if (n) std::memcpy(out, wf.data(), n * sizeof(uint32_t));
    }
    return wf.size();
}

uint64_t geak_check_plan_items(const geak_plan *plan, geak_item *out, uint64_t capacity)
{
    if (!plan) return 0;
    const auto &items = plan->host.items;
    if (out) {
        const uint64_t n = capacity < items.size() ? capacity : items.size();
        if (n) std::memcpy(out, items.data(), n * sizeof(geak_item));
    }
    return items.size();
}

uint64_t geak_check_plan_ref_offsets(const geak_plan *plan, uint64_t *out, uint64_t capacity)
{
    if (!plan) return 0;
    const auto &table = plan->host.ref_item_offset;
    if (out) {
        const uint64_t n = capacity < table.size() ? capacity : table.size();
        if (n) std::memcpy(out, table.data(), n * sizeof(uint64_t));
    }
    return table.size();
}

geak_status geak_check_report(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                              void *workspace_dev, const geak_result *results_dev, uint32_t max_records,
                              geak_mismatch *records_dev, uint32_t *counts_dev, void *hip_stream)
{
    if (!plan || !cand_dev || !results_dev || !records_dev || !counts_dev || max_records == 0) return GEAK_EINVAL;
    if (plan->device < 0) return GEAK_EINVAL;
    const HostPlan &hp = plan->host;
    const int K = hp.num_candidates;
    const bool reads_data = !hp.items.empty();
    if (const geak_status st = check_tensor_pointers(hp, ref_dev, cand_dev)) return st;
    if (((uintptr_t)results_dev & 7u) || ((uintptr_t)records_dev & 7u) || ((uintptr_t)counts_dev & 3u)) return GEAK_EALIGN;
    const uint64_t ws_bytes = geak_check_workspace_bytes(plan);
    if (ws_bytes && !workspace_dev) return GEAK_EWORKSPACE;
    if (ws_bytes && ((uintptr_t)workspace_dev & 15u)) return GEAK_EALIGN;
    DeviceGuard g(plan->device);
    if (!g.ok) return GEAK_EHIP;

    // the candidate pointer table is written again (the caller may have reused the workspace)
    const unsigned char **cand_table = reads_data ? (const unsigned char **)workspace_dev : nullptr;
    InitArgs ia;
    ia.results = nullptr;
    ia.cand_table = cand_table;
    ia.board = nullptr;
    ia.num_board = 0;
    ia.num_results = 0;
    ia.num_candidates = (uint32_t)K;
    ia.reserved = 0;
    for (int k = 0; k < GEAK_MAX_CANDIDATES; ++k) ia.cand[k] = (k < K) ? (const unsigned char *)cand_dev[k] : nullptr;
    if (reads_data && launch_init(ia, hip_stream) != (int)hipSuccess) return GEAK_EHIP;

    ReportArgs ra;
    ra.segments = plan->segments_dev;
    ra.results = results_dev;
    ra.ref = (const unsigned char *)ref_dev;
    ra.cand_table = cand_table;
    ra.records = records_dev;
    ra.counts = counts_dev;
    ra.num_segments = (uint32_t)hp.segments.size();
    ra.num_candidates = (uint32_t)K;
    ra.max_records = max_records;
    ra.seg_tol = plan->seg_tol_dev;
    ra.equal_nan = hp.equal_nan;
    ra.reserved = 0;
    ra.nd = plan->nd_dev;
    if (launch_report(ra, hip_stream) != (int)hipSuccess) return GEAK_EHIP;
    return GEAK_OK;
}

static uint32_t ulp_slots(const HostPlan &hp)
{
    uint32_t n = 0;
    for (const SegDesc &g : hp.segments) n = std::max(n, ulp_slots_of(g.dtype));
    return n;
}

uint64_t geak_check_ulp_workspace_bytes(const geak_plan *plan)
{
    if (!plan) return 0;
    const HostPlan &hp = plan->host;
    return kCandTableBytes + (uint64_t)hp.slot_begin.back() * (uint64_t)hp.num_candidates * ulp_slots(hp) * sizeof(uint32_t);
}

geak_status geak_check_ulp_histogram(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                                     void *ulp_workspace_dev, uint64_t *hist_dev, void *hip_stream)
{
    if (!plan || !cand_dev || !hist_dev || !ulp_workspace_dev) return GEAK_EINVAL;
    if (plan->device < 0) return GEAK_EINVAL;
    const HostPlan &hp = plan->host;
    for (const SegDesc &sg : hp.segments)
        if (sg.layout == kMxScaled) return GEAK_EDTYPE;          // a distance in code steps says nothing across different scales
    const int K = hp.num_candidates;
    const bool reads_data = !hp.items.empty();
    if (const geak_status st = check_tensor_pointers(hp, ref_dev, cand_dev)) return st;
    if (((uintptr_t)ulp_workspace_dev & 15u) || ((uintptr_t)hist_dev & 7u)) return GEAK_EALIGN;
    DeviceGuard g(plan->device);
    if (!g.ok) return GEAK_EHIP;

    const uint32_t nslots = ulp_slots(hp);
    const unsigned char **cand_table = (const unsigned char **)ulp_workspace_dev;
    uint32_t *partials = (uint32_t *)((unsigned char *)ulp_workspace_dev + kCandTableBytes);
    if (reads_data) {
        InitArgs ia;
        ia.results = nullptr;
        ia.cand_table = cand_table;
        ia.board = nullptr;
        ia.num_board = 0;
        ia.num_results = 0;
        ia.num_candidates = (uint32_t)K;
        ia.reserved = 0;
        for (int k = 0; k < GEAK_MAX_CANDIDATES; ++k) ia.cand[k] = (k < K) ? (const unsigned char *)cand_dev[k] : nullptr;
        if (launch_init(ia, hip_stream) != (int)hipSuccess) return GEAK_EHIP;

        // candidates per pass: what fits the per-wave rows
        const uint32_t per_pass = std::max<uint32_t>(1u, std::min<uint32_t>((uint32_t)K, kUlpLdsBudgetPerWave / (nslots * 4u)));
        for (uint32_t k0 = 0; k0 < (uint32_t)K; k0 += per_pass) {
            UlpArgs ua;
            ua.items = plan->items_dev;
            ua.ref = (const unsigned char *)ref_dev;
            ua.cand_table = cand_table;
            ua.partials = partials;
            ua.wave_first = plan->wave_first_dev;
            ua.num_items = (uint32_t)hp.items.size();
            ua.num_candidates = (uint32_t)K;
            ua.k_begin = k0;
            ua.k_count = std::min<uint32_t>(per_pass, (uint32_t)K - k0);
            ua.nslots = nslots;
            ua.unit_groups = hp.unit_groups;
            ua.block_map = hp.block_map;
            ua.reserved = 0;
            ua.segments = plan->segments_dev;
            ua.ref_item_offset = plan->ref_item_offset_dev;
            const uint32_t lds = kWavesPerBlock * ua.k_count * nslots * 4u;
            if (launch_ulp_histogram(ua, hp.grid_blocks, lds, hip_stream) != (int)hipSuccess) return GEAK_EHIP;
        }
    }
    UlpReduceArgs ra;
    ra.slot_begin = plan->slot_begin_dev;
    ra.partials = partials;
    ra.hist = (unsigned long long *)hist_dev;
    ra.num_segments = (uint32_t)hp.segments.size();
    ra.num_candidates = (uint32_t)K;
    ra.nslots = nslots;
    ra.reserved = 0;
    if (launch_ulp_reduce(ra, hip_stream) != (int)hipSuccess) return GEAK_EHIP;
    return GEAK_OK;
}

geak_status geak_check_verdicts(const geak_plan *plan, const geak_result *results_dev, int32_t *verdicts_dev,
                                uint32_t *failed_tests_dev, void *hip_stream)
{
    if (!plan || !results_dev || !verdicts_dev) return GEAK_EINVAL;
    if (plan->device < 0) return GEAK_EINVAL;
    if (((uintptr_t)results_dev & 7u) || ((uintptr_t)verdicts_dev & 3u) || ((uintptr_t)failed_tests_dev & 3u)) return GEAK_EALIGN;
    DeviceGuard g(plan->device);
    if (!g.ok) return GEAK_EHIP;
    VerdictArgs va;
    va.results = results_dev;
    va.verdicts = verdicts_dev;
    va.failed_tests = failed_tests_dev;
    va.num_segments = (uint32_t)plan->host.segments.size();
    va.num_candidates = (uint32_t)plan->host.num_candidates;
    if (launch_verdicts(va, hip_stream) != (int)hipSuccess) return GEAK_EHIP;
    return GEAK_OK;
}

geak_status geak_check_read_probe(const geak_plan *plan, const void *ref_dev, const void *const *cand_dev,
                                  void *workspace_dev, void *hip_stream)
{
    if (!plan || !cand_dev) return GEAK_EINVAL;
    if (plan->device < 0) return GEAK_EINVAL;
    const HostPlan &hp = plan->host;
    if (hp.items.empty()) return GEAK_OK;
    if (!workspace_dev) return GEAK_EINVAL;
    if (const geak_status st = check_tensor_pointers(hp, ref_dev, cand_dev)) return st;
    if ((uintptr_t)workspace_dev & 15u) return GEAK_EALIGN;
    // the probe reads the same span of every buffer: a reference with a layout of its own may be far shorter
    for (const SegDesc &sg : hp.segments)
        if (seg_ref_mapped(sg)) return GEAK_EINVAL;
    const int K = hp.num_candidates;
    // the span of the packed buffers that the plan's segments cover
    uint64_t end = 0;
    for (const SegDesc &g : hp.segments)
        if (g.numel) {
            end = std::max<uint64_t>(end, g.byte_offset + seg_span(g));
            if (g.layout == kMxScaled) end = std::max<uint64_t>(end, g.ref_byte_offset + g.numel / kMxBlock);     // its scale bytes
        }
    DeviceGuard g(plan->device);
    if (!g.ok) return GEAK_EHIP;
    // the candidate pointer table of a run is reused; the reference pointer goes behind it
    InitArgs ia;
    ia.results = nullptr;
    ia.cand_table = (const unsigned char **)workspace_dev;
    ia.board = nullptr;
    ia.num_board = 0;
    ia.num_results = 0;
    ia.num_candidates = (uint32_t)K + 1;
    ia.reserved = 0;
    if (K + 1 > GEAK_MAX_CANDIDATES) return GEAK_EINVAL;      // the table has room for 256 pointers
    for (int k = 0; k < GEAK_MAX_CANDIDATES; ++k)
        ia.cand[k] = (k < K) ? (const unsigned char *)cand_dev[k] : (k == K ? (const unsigned char *)ref_dev : nullptr);
    if (launch_init(ia, hip_stream) != (int)hipSuccess) return GEAK_EHIP;
    ProbeArgs pa;
    pa.buffers = (const unsigned char *const *)workspace_dev;
    pa.sink = (uint32_t *)((unsigned char *)workspace_dev + kCandTableBytes);      // the first queue/board word: scratch
    pa.bytes_each = end;
    pa.num_buffers = (uint32_t)K + 1;
    pa.reserved = 0;
    if (launch_read_probe(pa, hp.max_blocks * 2, hip_stream) != (int)hipSuccess) return GEAK_EHIP;
    return GEAK_OK;
}

geak_status geak_check_profile_enable(geak_plan *plan, uint32_t num_pairs)
{
    if (!plan || plan->device < 0) return GEAK_EINVAL;
    DeviceGuard g(plan->device);
    if (!g.ok) return GEAK_EHIP;
    for (auto e : plan->ev_start) (void)hipEventDestroy(e);
    for (auto e : plan->ev_stop) (void)hipEventDestroy(e);
    plan->ev_start.clear();
    plan->ev_stop.clear();
    plan->ev_next = plan->ev_used = 0;
    try {
        plan->ev_start.reserve(num_pairs);                  // so that the two rings cannot end up of different lengths
        plan->ev_stop.reserve(num_pairs);
        for (uint32_t i = 0; i < num_pairs; ++i) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess) return GEAK_EHIP;
            if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return GEAK_EHIP; }
            plan->ev_start.push_back(a);
            plan->ev_stop.push_back(b);
        }
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    return GEAK_OK;
}

uint64_t geak_check_profile_read(geak_plan *plan, float *ms_out, uint64_t capacity)
{
    if (!plan || !ms_out || plan->ev_start.empty()) return 0;
    const uint32_t ring = (uint32_t)plan->ev_start.size();
    const uint32_t used = plan->ev_used;
    const uint32_t oldest = (plan->ev_next + ring - used) % ring;
    uint64_t n = 0;
    for (uint32_t i = 0; i < used && n < capacity; ++i) {
        const uint32_t s = (oldest + i) % ring;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, plan->ev_start[s], plan->ev_stop[s]) == hipSuccess) ms_out[n++] = ms;
    }
    plan->ev_next = plan->ev_used = 0;
    return n;
}

}  // extern "C"
