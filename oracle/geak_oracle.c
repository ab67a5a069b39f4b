/*
 * CPU oracle for the evaluator's output-equivalence check.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, element-by-element
 * statement of what the check computes.  It is called by the tests, by the
 * smoke check and by the benchmark's CPU-baseline leg, never by the product
 * path, and it shares no code with the HIP implementation.
 *
 * What it follows: GEAK (arXiv 2507.23194) section 3.1, second enhancement
 * bullet -- candidate kernels are judged by a tolerance-based comparison of
 * the output tensors of their test functions against reference outputs -- and
 * section 3.3, where a kernel counts as correct only if it satisfies every
 * unit test and the reference kernels are the ground truth.  The paper prints
 * no formula, tolerance value or NaN policy; the rule below is the reading
 * this project fixes (every point is listed in the design notes):
 *
 *   floating dtypes (binary32, binary16, bfloat16, and the 8-bit formats E4M3 and E5M2 of the OCP
 *   specification, all widened exactly to binary32), a = candidate, b = reference,
 *   all arithmetic in IEEE binary32, round-to-nearest-even, one rounding per
 *   operation, no fused multiply-add, subnormals honoured:
 *     R1  d   = | a (-) b |
 *         tol = atol_f (+) ( rtol_f (x) |b| ),  atol_f = (float)atol, rtol_f = (float)rtol
 *         close <=> d <= tol            (inclusive; tolerance scales with the reference)
 *     R3  if a or b is NaN:   close <=> equal_nan and both are NaN
 *     R4  else if a or b is +-Inf: close <=> a == b
 *     R5  -0 vs +0 gives d = 0, hence close
 *   binary64 inputs:
 *     R2' the same rules R1, R3, R4, R5, R8, R9 with every operation in IEEE binary64 (one rounding per
 *         operation, no fused multiply-add) and atol, rtol used as given: converting the inputs to
 *         binary32 would throw away the precision such outputs are checked for
 *   int32:
 *     R6  close <=> a == b; d = |a - b| exactly (64-bit), tolerances ignored
 *   uint8 (also the storage of boolean masks) and int8:
 *     R6" close <=> a == b; d = |a - b| exactly (at most 255); R8 and R9 as for int32
 *   int64 (index outputs of sort / argmax-like kernels):
 *     R6' close <=> a == b; d = |a - b| exactly as an unsigned 64-bit integer (at most 2^64 - 1);
 *         where a binary64 value is needed (R8, R9, the report) d and |b| (at most 2^63) are each
 *         converted to binary64 with one rounding to nearest even
 *   reductions per (segment, candidate):
 *     R7  mismatch_count = #{i : not close_i}; first_mismatch = least such i, else -1;
 *         pass = (mismatch_count == 0); an empty segment passes
 *     R8  max_abs_err = maximum of d_i over ALL i, skipping NaN d_i, +Inf included,
 *         starting from +0
 *     R9  max_rel_err = maximum over all i of r_i, r_i = 0 when d_i == 0, else
 *         d_i (/) |b_i| (binary32 division; x/0 = +Inf; NaN skipped), starting from +0.
 *         int32: r_i = (double)d_i / (double)|b_i| in binary64, same conventions
 *     R10 indices are flat, 0-based, within the segment
 *
 *   mismatch report (oracle_report_segment, below): the first M elements that are not close,
 *         with index, a, b, d and tol as the rule computed them
 *   ulp histogram (oracle_ulp_histogram_segment, below): per pair, how many elements lie how many
 *         steps of the storage format apart (rules U1-U4 there)
 *
 * Pins (tests/test_oracle_pins.py, tests/golden/): hand-derived records for
 * boundary, NaN, Inf, signed-zero, subnormal and integer cases; an exact
 * rational-arithmetic model of the rounding steps; structural invariants;
 * agreement with numpy.isclose away from the boundary; generator-known
 * mismatch counts on the synthetic workloads.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC (see oracle.py).
 */
#include <stdint.h>
#include <string.h>
#include <math.h>

#if defined(__SSE2__)
#include <xmmintrin.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2, ORACLE_I32 = 3, ORACLE_I64 = 4, ORACLE_U8 = 5, ORACLE_I8 = 6, ORACLE_F64 = 7,
       ORACLE_F8E4M3 = 8, ORACLE_F8E5M2 = 9 };

typedef struct {
    int32_t  pass;
    int32_t  reserved;
    uint64_t mismatch_count;
    int64_t  first_mismatch;
    double   max_abs_err;
    double   max_rel_err;
} oracle_record;

static float bits_to_float(uint32_t u)
{
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* binary16 -> binary32, exact, by bit manipulation (R13: own decoder). */
static float decode_f16(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t exp  = (h >> 10) & 0x1Fu;
    uint32_t man  = h & 0x3FFu;
    if (exp == 0x1Fu)                         /* Inf / NaN: keep payload */
        return bits_to_float(sign | 0x7F800000u | (man << 13));
    if (exp == 0) {
        if (man == 0)
            return bits_to_float(sign);       /* signed zero */
        /* subnormal: value = man * 2^-24; normalise */
        int shift = 0;
        while ((man & 0x400u) == 0) { man <<= 1; ++shift; }
        man &= 0x3FFu;
        exp = (uint32_t)(127 - 15 + 1 - shift);
        return bits_to_float(sign | (exp << 23) | (man << 13));
    }
    return bits_to_float(sign | ((exp + (127 - 15)) << 23) | (man << 13));
}

/* bfloat16 is the upper half of a binary32. */
static float decode_bf16(uint16_t h)
{
    return bits_to_float((uint32_t)h << 16);
}

/* 8-bit floating formats of the OCP 8-bit floating point specification, decoded by their definition:
 * sign, biased exponent, mantissa; value = (-1)^s * 2^(e - bias) * (1 + m / 2^mbits), or
 * (-1)^s * 2^(1 - bias) * (m / 2^mbits) when e = 0.
 *   E4M3: 4 exponent bits (bias 7), 3 mantissa bits; no infinities; S.1111.111 is NaN; largest value 448
 *   E5M2: 5 exponent bits (bias 15), 2 mantissa bits; e = 31 is Inf (m = 0) or NaN, as in IEEE formats */
static float decode_f8e4m3(uint8_t x)
{
    int sign = x >> 7, e = (x >> 3) & 0xF, m = x & 0x7;
    float v;
    if (e == 0xF && m == 0x7)
        v = NAN;
    else if (e == 0)
        v = ldexpf((float)m, 1 - 7 - 3);
    else
        v = ldexpf((float)(8 + m), e - 7 - 3);
    return sign ? -v : v;
}
static float decode_f8e5m2(uint8_t x)
{
    int sign = x >> 7, e = (x >> 2) & 0x1F, m = x & 0x3;
    float v;
    if (e == 0x1F)
        v = m ? NAN : INFINITY;
    else if (e == 0)
        v = ldexpf((float)m, 1 - 15 - 2);
    else
        v = ldexpf((float)(4 + m), e - 15 - 2);
    return sign ? -v : v;
}

/* element i of a tensor of one of the dtypes whose rule runs in binary32, widened exactly */
static float load_as_f32(const void *p, uint64_t i, int dtype)
{
    switch (dtype) {
    case ORACLE_F32:    return ((const float *)p)[i];
    case ORACLE_F16:    return decode_f16(((const uint16_t *)p)[i]);
    case ORACLE_BF16:   return decode_bf16(((const uint16_t *)p)[i]);
    case ORACLE_F8E4M3: return decode_f8e4m3(((const uint8_t *)p)[i]);
    default:            return decode_f8e5m2(((const uint8_t *)p)[i]);
    }
}

static int is_nan_f(float x) { return x != x; }
static int is_inf_f(float x) { return x == INFINITY || x == -INFINITY; }

/*
 * One (segment, candidate) pair.  ref and cand point at the first element of
 * the segment; numel elements of the given dtype follow contiguously.
 * Returns 0, or -1 for an unknown dtype / null output.
 */
int oracle_check_segment(const void *ref, const void *cand, uint64_t numel, int dtype,
                         double atol, double rtol, int equal_nan, oracle_record *out)
{
    if (!out || dtype < 0 || dtype > 9)
        return -1;

#if defined(__SSE2__)
    /* Subnormals must be honoured: drop FTZ/DAZ if some library set them on this thread. */
    unsigned int csr_saved = _mm_getcsr();
    _mm_setcsr(csr_saved & ~0x8040u);
#endif

    uint64_t count = 0;
    int64_t  first = -1;
    double   max_abs = 0.0;
    double   max_rel = 0.0;

    if (dtype == ORACLE_F64) {
        const double *pb = (const double *)ref;
        const double *pa = (const double *)cand;
        for (uint64_t i = 0; i < numel; ++i) {
            double a = pa[i], b = pb[i];
            double diff = a - b;                             /* each operation rounded to binary64 on its own */
            double d = fabs(diff);                           /* R1 */
            double babs = fabs(b);
            int close;
            if (a != a || b != b) {                          /* R3 */
                close = equal_nan && (a != a) && (b != b);
            } else if (isinf(a) || isinf(b)) {               /* R4 */
                close = (a == b);
            } else {
                double prod = rtol * babs;                   /* rounded */
                double tol  = atol + prod;                   /* rounded again: no FMA */
                close = (d <= tol);
            }
            if (!close) {
                ++count;
                if (first < 0) first = (int64_t)i;
            }
            if (!(d != d) && d > max_abs)                    /* R8 */
                max_abs = d;
            double r;
            if (d == 0.0) {
                r = 0.0;                                     /* R9 */
            } else {
                r = d / babs;                                /* binary64 division */
            }
            if (!(r != r) && r > max_rel)
                max_rel = r;
        }
    } else if (dtype == ORACLE_I64) {
        const int64_t *pb = (const int64_t *)ref;
        const int64_t *pa = (const int64_t *)cand;
        for (uint64_t i = 0; i < numel; ++i) {
            int64_t a = pa[i], b = pb[i];
            /* |a - b| without overflow: subtract the smaller from the larger in unsigned arithmetic */
            uint64_t d = (a >= b) ? ((uint64_t)a - (uint64_t)b) : ((uint64_t)b - (uint64_t)a);
            if (a != b) {                                    /* R6' */
                ++count;
                if (first < 0) first = (int64_t)i;
            }
            double dd = (double)d;                           /* one rounding */
            if (dd > max_abs) max_abs = dd;                  /* R8 */
            double r;
            if (d == 0) {
                r = 0.0;
            } else {
                uint64_t babs_u = (b < 0) ? (0 - (uint64_t)b) : (uint64_t)b;     /* |INT64_MIN| = 2^63 fits */
                r = dd / (double)babs_u;                     /* R9, binary64; x/0 = +Inf */
            }
            if (r > max_rel) max_rel = r;
        }
    } else if (dtype == ORACLE_I32 || dtype == ORACLE_U8 || dtype == ORACLE_I8) {
        for (uint64_t i = 0; i < numel; ++i) {
            int64_t a, b;
            if (dtype == ORACLE_I32) {
                a = ((const int32_t *)cand)[i];
                b = ((const int32_t *)ref)[i];
            } else if (dtype == ORACLE_U8) {
                a = ((const uint8_t *)cand)[i];
                b = ((const uint8_t *)ref)[i];
            } else {
                a = ((const int8_t *)cand)[i];
                b = ((const int8_t *)ref)[i];
            }
            int64_t diff = a - b;
            uint64_t d = (uint64_t)(diff < 0 ? -diff : diff);
            if (a != b) {                                    /* R6 */
                ++count;
                if (first < 0) first = (int64_t)i;
            }
            double dd = (double)d;
            if (dd > max_abs) max_abs = dd;                  /* R8 */
            double r;
            if (d == 0) {
                r = 0.0;
            } else {
                double babs = (double)(b < 0 ? -b : b);
                r = dd / babs;                               /* R9, binary64 */
            }
            if (r > max_rel) max_rel = r;
        }
    } else {
        const float atol_f = (float)atol;
        const float rtol_f = (float)rtol;
        for (uint64_t i = 0; i < numel; ++i) {
            float a = load_as_f32(cand, i, dtype), b = load_as_f32(ref, i, dtype);

            /* each operation rounded to binary32 on its own */
            float diff = a - b;
            float d = fabsf(diff);                           /* R1 */
            float babs = fabsf(b);

            int close;
            if (is_nan_f(a) || is_nan_f(b)) {                /* R3 */
                close = equal_nan && is_nan_f(a) && is_nan_f(b);
            } else if (is_inf_f(a) || is_inf_f(b)) {         /* R4 */
                close = (a == b);
            } else {
                float prod = rtol_f * babs;             /* rounded */
                float tol  = atol_f + prod;             /* rounded again: no FMA */
                close = (d <= tol);                          /* R1 */
            }
            if (!close) {                                    /* R7 */
                ++count;
                if (first < 0) first = (int64_t)i;
            }

            if (!is_nan_f(d) && (double)d > max_abs)         /* R8 */
                max_abs = (double)d;

            float r;
            if (d == 0.0f) {
                r = 0.0f;                                    /* R9: covers 0/0 and +-0 */
            } else {
                r = d / babs;                               /* binary32 division */
            }
            if (!is_nan_f(r) && (double)r > max_rel)         /* NaN d gives NaN r: skipped */
                max_rel = (double)r;
        }
    }

    out->pass = (count == 0);
    out->reserved = 0;
    out->mismatch_count = count;
    out->first_mismatch = first;
    out->max_abs_err = max_abs;
    out->max_rel_err = max_rel;

#if defined(__SSE2__)
    _mm_setcsr(csr_saved);
#endif
    return 0;
}

/*
 * Mismatch report for one (segment, candidate) pair: the first max_records elements that are not
 * close, in ascending index order, each with what the rule saw.  GEAK section 4.1 feeds the error
 * trace of a failed functionality test to the Reflector, and section 4.2 (Reflexion) has the agent
 * analyse it; the paper does not say what the trace holds, so this is the reading: for every
 * reported element its flat index, a and b widened exactly to binary64, d = |a (-) b| and
 * tol = atol_f (+) (rtol_f (x) |b|) exactly as rules R1 / R6 compute them (binary32 values widened;
 * for int32 d is exact and tol is 0; for int64 a, b and d are each converted to binary64 with one
 * rounding).  d and tol may be NaN or infinite when a or b is.
 * Returns the number of records written (at most max_records), or -1 on a bad argument.
 */
typedef struct {
    int64_t index;
    double  a;
    double  b;
    double  d;
    double  tol;
} oracle_mismatch;

int64_t oracle_report_segment(const void *ref, const void *cand, uint64_t numel, int dtype,
                              double atol, double rtol, int equal_nan, uint64_t max_records,
                              oracle_mismatch *out)
{
    if ((!out && max_records) || dtype < 0 || dtype > 9)
        return -1;
#if defined(__SSE2__)
    unsigned int csr_saved = _mm_getcsr();
    _mm_setcsr(csr_saved & ~0x8040u);
#endif
    uint64_t written = 0;
    const float atol_f = (float)atol;
    const float rtol_f = (float)rtol;
    for (uint64_t i = 0; i < numel && written < max_records; ++i) {
        oracle_mismatch m;
        int close;
        if (dtype == ORACLE_F64) {
            double a = ((const double *)cand)[i], b = ((const double *)ref)[i];
            double diff = a - b;
            double d = fabs(diff);
            double prod = rtol * fabs(b);
            double tol = atol + prod;
            if (a != a || b != b)                                /* R3 */
                close = equal_nan && (a != a) && (b != b);
            else if (isinf(a) || isinf(b))                       /* R4 */
                close = (a == b);
            else
                close = (d <= tol);
            m.a = a;
            m.b = b;
            m.d = d;
            m.tol = tol;
        } else if (dtype == ORACLE_I64) {
            int64_t a = ((const int64_t *)cand)[i], b = ((const int64_t *)ref)[i];
            uint64_t d = (a >= b) ? ((uint64_t)a - (uint64_t)b) : ((uint64_t)b - (uint64_t)a);
            close = (a == b);                                    /* R6' */
            m.a = (double)a;                                     /* one rounding each */
            m.b = (double)b;
            m.d = (double)d;
            m.tol = 0.0;
        } else if (dtype == ORACLE_I32 || dtype == ORACLE_U8 || dtype == ORACLE_I8) {
            int64_t a, b;
            if (dtype == ORACLE_I32) {
                a = ((const int32_t *)cand)[i];
                b = ((const int32_t *)ref)[i];
            } else if (dtype == ORACLE_U8) {
                a = ((const uint8_t *)cand)[i];
                b = ((const uint8_t *)ref)[i];
            } else {
                a = ((const int8_t *)cand)[i];
                b = ((const int8_t *)ref)[i];
            }
            int64_t diff = a - b;
            close = (a == b);                                    /* R6 */
            m.a = (double)a;
            m.b = (double)b;
            m.d = (double)(diff < 0 ? -diff : diff);
            m.tol = 0.0;
        } else {
            float a = load_as_f32(cand, i, dtype), b = load_as_f32(ref, i, dtype);
            float diff = a - b;
            float d = fabsf(diff);                               /* R1 */
            float prod = rtol_f * fabsf(b);
            float tol = atol_f + prod;
            if (is_nan_f(a) || is_nan_f(b))                      /* R3 */
                close = equal_nan && is_nan_f(a) && is_nan_f(b);
            else if (is_inf_f(a) || is_inf_f(b))                 /* R4 */
                close = (a == b);
            else
                close = (d <= tol);
            m.a = (double)a;
            m.b = (double)b;
            m.d = (double)d;
            m.tol = (double)tol;
        }
        if (!close) {
            m.index = (int64_t)i;
            out[written++] = m;
        }
    }
#if defined(__SSE2__)
    _mm_setcsr(csr_saved);
#endif
    return (int64_t)written;
}

/*
 * Histogram of unit-in-the-last-place distances for one (segment, candidate) pair: the second half
 * of the numeric error trace (GEAK sections 4.1 / 4.2: the Reflector analyses why the functionality
 * test failed).  It separates rounding-level deviations (a few steps of the format) from structural
 * ones (wrong values).  The paper does not define it; the reading:
 *
 *   U1  floating dtypes: the distance of a and b is the number of steps between them on the ladder
 *       of the values of the tensor's OWN storage format (binary16, bfloat16, binary32, binary64),
 *       ordered by value, -0 and +0 being one rung, +-Inf the rung after the largest finite value.
 *       For values of one sign that is the difference of the magnitudes' bit patterns, for values of
 *       opposite sign their sum (both exact in 64 bits unsigned).
 *   U2  integer dtypes: the distance is |a - b|, exact (at most 2^64 - 1).
 *   U3  bins: 0 holds distance 0; bin j, 1 <= j <= 64, holds 2^(j-1) <= distance < 2^j;
 *       bin 65 holds every element where a or b is NaN (equal_nan plays no part).
 *   U4  out[66] counts all elements of the segment: the bins sum to numel.
 * Returns 0, or -1 on a bad argument.
 */
#define ORACLE_ULP_BINS 66

static int bit_length_u64(uint64_t x)
{
    int n = 0;
    while (x) { ++n; x >>= 1; }
    return n;
}

int oracle_ulp_histogram_segment(const void *ref, const void *cand, uint64_t numel, int dtype,
                                 uint64_t *out)
{
    if (!out || dtype < 0 || dtype > 9)
        return -1;
    for (int j = 0; j < ORACLE_ULP_BINS; ++j) out[j] = 0;
    for (uint64_t i = 0; i < numel; ++i) {
        uint64_t distance;
        if (dtype == ORACLE_I32 || dtype == ORACLE_U8 || dtype == ORACLE_I8 || dtype == ORACLE_I64) {
            int64_t a, b;                                        /* U2 */
            if (dtype == ORACLE_I32) {
                a = ((const int32_t *)cand)[i];  b = ((const int32_t *)ref)[i];
            } else if (dtype == ORACLE_U8) {
                a = ((const uint8_t *)cand)[i];  b = ((const uint8_t *)ref)[i];
            } else if (dtype == ORACLE_I8) {
                a = ((const int8_t *)cand)[i];   b = ((const int8_t *)ref)[i];
            } else {
                a = ((const int64_t *)cand)[i];  b = ((const int64_t *)ref)[i];
            }
            distance = (a >= b) ? ((uint64_t)a - (uint64_t)b) : ((uint64_t)b - (uint64_t)a);
        } else {
            /* sign, magnitude pattern and NaN test in the format's own fields (U1) */
            uint64_t pa, pb, sign_bit, inf_pattern;
            if (dtype == ORACLE_F64) {
                pa = ((const uint64_t *)cand)[i];  pb = ((const uint64_t *)ref)[i];
                sign_bit = 1ull << 63;  inf_pattern = 0x7FF0000000000000ull;
            } else if (dtype == ORACLE_F32) {
                pa = ((const uint32_t *)cand)[i];  pb = ((const uint32_t *)ref)[i];
                sign_bit = 1ull << 31;  inf_pattern = 0x7F800000ull;
            } else if (dtype == ORACLE_F16 || dtype == ORACLE_BF16) {
                pa = ((const uint16_t *)cand)[i];  pb = ((const uint16_t *)ref)[i];
                sign_bit = 1ull << 15;
                inf_pattern = (dtype == ORACLE_F16) ? 0x7C00ull : 0x7F80ull;
            } else {
                pa = ((const uint8_t *)cand)[i];  pb = ((const uint8_t *)ref)[i];
                sign_bit = 1ull << 7;
                /* E5M2 has Inf at 0x7C; E4M3 has none: its ladder ends at the largest finite value 0x7E and
                 * the one pattern above it is NaN, so that value stands in for Inf in the NaN test */
                inf_pattern = (dtype == ORACLE_F8E5M2) ? 0x7Cull : 0x7Eull;
            }
            uint64_t ma = pa & (sign_bit - 1), mb = pb & (sign_bit - 1);
            if (ma > inf_pattern || mb > inf_pattern) {          /* U3: NaN */
                out[65] += 1;
                continue;
            }
            int neg_a = (pa & sign_bit) != 0, neg_b = (pb & sign_bit) != 0;
            if (neg_a == neg_b)
                distance = (ma >= mb) ? (ma - mb) : (mb - ma);
            else
                distance = ma + mb;                              /* across zero; +-0 add nothing */
        }
        out[bit_length_u64(distance)] += 1;                      /* U3 */
    }
    return 0;
}

/* Decoders exported so the pins can check them on all 65536 bit patterns. */
float oracle_decode_f16(uint16_t h)  { return decode_f16(h); }
float oracle_decode_bf16(uint16_t h) { return decode_bf16(h); }
float oracle_decode_f8e4m3(uint8_t x) { return decode_f8e4m3(x); }
float oracle_decode_f8e5m2(uint8_t x) { return decode_f8e5m2(x); }
