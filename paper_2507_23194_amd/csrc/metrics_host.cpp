// Host-side evaluation metrics that consume the check's verdicts (GEAK section "Evaluation
// Metrics": call accuracy, execution accuracy, speedup; section 4.2: accuracy estimated with pass@k).
#include <algorithm>
#include <cmath>
#include <limits>
#include <new>
#include <vector>
#include "geak_check.h"

namespace {

// median of n values (n >= 1); the buffer is reordered
double median_of(double *v, uint64_t n)
{
    double *mid = v + n / 2;
    std::nth_element(v, mid, v + n);
    if (n % 2) return *mid;
    const double below = *std::max_element(v, mid);        // the largest of the lower half
    return 0.5 * (below + *mid);
}

}  // namespace

extern "C" {

geak_status geak_metrics_accuracy(const int32_t *compiled, const int32_t *correct, uint64_t n,
                                  double *call_accuracy, double *execution_accuracy)
{
    if ((n && (!compiled || !correct)) || !call_accuracy || !execution_accuracy) return GEAK_EINVAL;
    uint64_t n_compiled = 0, n_correct = 0;
    for (uint64_t i = 0; i < n; ++i) {
        n_compiled += compiled[i] != 0;
        n_correct += compiled[i] != 0 && correct[i] != 0;
    }
    const double nan = std::numeric_limits<double>::quiet_NaN();
    *call_accuracy = n ? (double)n_compiled / (double)n : nan;
    *execution_accuracy = n_compiled ? (double)n_correct / (double)n_compiled : nan;
    return GEAK_OK;
}

geak_status geak_metrics_speedup(const double *ref_latencies, uint64_t ref_reps, const double *gen_latencies,
                                 uint64_t gen_reps, uint64_t num_tests, double *speedup)
{
    if (!speedup) return GEAK_EINVAL;
    if (!num_tests || !ref_reps || !gen_reps) { *speedup = std::numeric_limits<double>::quiet_NaN(); return GEAK_OK; }
    if (!ref_latencies || !gen_latencies) return GEAK_EINVAL;
    try {
        std::vector<double> buf(std::max(ref_reps, gen_reps));
        double total = 0.0;
        for (uint64_t t = 0; t < num_tests; ++t) {
            std::copy(ref_latencies + t * ref_reps, ref_latencies + (t + 1) * ref_reps, buf.begin());
            const double ref_median = median_of(buf.data(), ref_reps);
            std::copy(gen_latencies + t * gen_reps, gen_latencies + (t + 1) * gen_reps, buf.begin());
            const double gen_median = median_of(buf.data(), gen_reps);
            total = total + ref_median / gen_median;                  // in test order
        }
        *speedup = total / (double)num_tests;
    } catch (const std::bad_alloc &) {
        return GEAK_ENOMEM;
    }
    return GEAK_OK;
}

geak_status geak_metrics_pass_at_k(uint64_t n, uint64_t c, uint64_t k, double *out)
{
    if (!out || c > n || k < 1 || k > n) return GEAK_EINVAL;
    if (n - c < k) { *out = 1.0; return GEAK_OK; }                   // every k-subset holds a correct sample
    // C(n - c, k) / C(n, k) = prod_{i = n - c + 1 .. n} (1 - k / i): c factors in (0, 1], no large binomials
    double miss = 1.0;
    for (uint64_t i = n - c + 1; i <= n; ++i) miss *= 1.0 - (double)k / (double)i;
    *out = 1.0 - miss;
    return GEAK_OK;
}

}  // extern "C"
