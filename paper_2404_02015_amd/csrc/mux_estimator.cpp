// Throughput estimator of MuxServe (Section 3.3, Eq. 3; Appendix A.2) and the batch-size search
// built on it.  Host arithmetic only.
#include <cmath>

#include "mux_internal.h"

extern "C" {

double mux_estimate_tpt(int32_t n_models, const double *batch, const double *t_prefill, const double *t_decode,
                        const double *gen_len, int32_t m, double rate_cap)
{
    const double bad = std::nan("");
    if (n_models <= 0 || !batch || !t_prefill || !t_decode || !gen_len || m < 0 || m >= n_models) return bad;
    double prefill_sum = 0.0;
    for (int32_t i = 0; i < n_models; ++i) {
        if (!(batch[i] >= 0.0) || !(t_prefill[i] >= 0.0) || !(t_decode[i] >= 0.0) || !(gen_len[i] >= 0.0)) return bad;
        if (batch[i] > 0.0) prefill_sum += t_prefill[i];   // a model without requests runs no prefill
    }
    if (!(rate_cap >= 0.0)) return bad;
    const double period = prefill_sum + t_decode[m] * gen_len[m];
    if (!(period > 0.0)) return batch[m] > 0.0 ? rate_cap : 0.0;
    return std::fmin(batch[m] / period, rate_cap);
}

int64_t mux_find_batch_size(double rate, int64_t max_batch, double p0, double p1, double d0, double d1, double gen_len,
                            double other_prefill)
{
    if (!(rate >= 0.0) || max_batch < 1 || !(p0 >= 0.0) || !(p1 >= 0.0) || !(d0 >= 0.0) || !(d1 >= 0.0) || !(gen_len >= 0.0) ||
        !(other_prefill >= 0.0))
        return MUX_ERR_INVALID;
    auto tpt = [&](int64_t b) {
        const double x = static_cast<double>(b);
        const double period = other_prefill + (p0 + p1 * x) + (d0 + d1 * x) * gen_len;   // in this order: the comparison below decides an integer
        return period > 0.0 ? x / period : INFINITY;
    };
    if (tpt(max_batch) < rate) return 0;   // even the largest batch cannot keep up
    int64_t lo = 1, hi = max_batch;        // tpt is non-decreasing in b: the first b with tpt(b) >= rate
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (tpt(mid) >= rate)
            hi = mid;
        else
            lo = mid + 1;
    }
    return lo;
}

}  // extern "C"
