// Host-side scheduling model that consumes the predicted lengths (Section 4.3 and the appendix on
// end-to-end system metrics): shortest-predicted-job-first order, consecutive batches, padding
// ratio / completion time / throughput.  Integer arithmetic throughout.
#include "../../include/egtp_sched.h"

#include <algorithm>
#include <cmath>
#include <new>
#include <numeric>
#include <vector>

extern "C" {

egtp_status egtp_sjf_order(const float *pred, int32_t n, int32_t *order_out)
{
    if (n < 0)
        return EGTP_ERR_SHAPE;
    if (n == 0)
        return EGTP_OK;
    if (!pred || !order_out)
        return EGTP_ERR_NULL;
    std::iota(order_out, order_out + n, 0);
    // NaN compares false both ways; send it behind every number explicitly so that the
    // comparison stays a strict weak order
    std::stable_sort(order_out, order_out + n, [pred](int32_t a, int32_t b) {
        const bool na = std::isnan(pred[a]), nb = std::isnan(pred[b]);
        if (na || nb)
            return !na && nb;
        return pred[a] < pred[b];
    });
    return EGTP_OK;
}

egtp_status egtp_simulate_batches(const int32_t *order, const int32_t *true_len, int32_t n, int32_t batch_size,
                                  egtp_sched_report *report, int64_t *completion_out, int32_t *batch_of_out)
{
    if (n < 0 || batch_size < 1)
        return EGTP_ERR_SHAPE;
    if (!report || (n > 0 && (!order || !true_len)))
        return EGTP_ERR_NULL;
    std::vector<char> seen;
    try {
        seen.assign((size_t)n, 0);
    } catch (const std::bad_alloc &) {
        return EGTP_ERR_HIP;
    }
    for (int32_t i = 0; i < n; ++i) {
        const int32_t j = order[i];
        if (j < 0 || j >= n || seen[j])
            return EGTP_ERR_OFFSETS;
        seen[j] = 1;
        if (true_len[j] < 0)
            return EGTP_ERR_SHAPE;
    }
    egtp_sched_report r = {};
    int64_t clock = 0;
    for (int32_t lo = 0; lo < n; lo += batch_size) {
        const int32_t hi = std::min<int64_t>((int64_t)lo + batch_size, n);
        int64_t longest = 0;
        for (int32_t i = lo; i < hi; ++i)
            longest = std::max<int64_t>(longest, true_len[order[i]]);
        for (int32_t i = lo; i < hi; ++i) {
            const int32_t j = order[i];
            const int64_t done = clock + true_len[j];
            r.actual_tokens += true_len[j];
            r.sum_jct_steps += done;
            if (completion_out)
                completion_out[j] = done;
            if (batch_of_out)
                batch_of_out[j] = r.n_batches;
        }
        r.allocated_tokens += (int64_t)(hi - lo) * longest;
        clock += longest;
        ++r.n_batches;
    }
    r.makespan_steps = clock;
    r.padding_ratio = r.actual_tokens > 0 ? (double)(r.allocated_tokens - r.actual_tokens) / (double)r.actual_tokens : 0.0;
    r.avg_jct_steps = n > 0 ? (double)r.sum_jct_steps / (double)n : 0.0;
    r.throughput = clock > 0 ? (double)n / (double)clock : 0.0;
    *report = r;
    return EGTP_OK;
}

}  // extern "C"
