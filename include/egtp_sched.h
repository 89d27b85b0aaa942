/*
 * egtp_sched.h -- host-side consumer of the length predictions: shortest-predicted-job-first
 * ordering, length-bucketed static batches and the end-to-end metrics of the paper's system
 * evaluation (Section 4.3; metric definitions in the appendix on end-to-end system metrics:
 * throughput, job completion time, padding ratio).
 *
 * The paper couples its predictor to an SJF scheduler inside a serving engine and reports the
 * three metrics; it does not describe the scheduler further.  What is modelled here is the
 * plainest system those metrics are defined on:
 *   - all n jobs are submitted at time 0; one engine runs one batch at a time;
 *   - jobs are taken in the given order and cut into batches of `batch_size` consecutive jobs
 *     (the last batch may be smaller) -- sorting by predicted length first makes these
 *     length buckets;
 *   - a batch decodes in lock step for as many steps as its longest member really needs
 *     (true lengths, in tokens); every member holds its slot until the batch ends, so the batch
 *     is allocated  |batch| * max length  token slots;
 *   - a job completes at the step its own last token is produced (batch start + its length).
 * Time is counted in decode steps (integers), so everything below is exact integer work except
 * the final ratios, which are one double division each.
 *
 * All pointers are HOST pointers, borrowed.  Nothing here touches the GPU.
 */
#ifndef EGTP_SCHED_H
#define EGTP_SCHED_H

#include <stdint.h>

#include "egtp.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Shortest-job-first order from predicted lengths: order_out[0..n) is the permutation of
 * 0..n-1 that sorts pred ascending; equal predictions keep their submission order; NaN
 * predictions go last (in submission order).  n == 0 is fine.
 * EGTP_ERR_NULL / EGTP_ERR_SHAPE (n < 0). */
egtp_status egtp_sjf_order(const float *pred, int32_t n, int32_t *order_out);

typedef struct {
    int32_t n_batches;
    int64_t actual_tokens;    /* R_actual    = sum of true lengths                              */
    int64_t allocated_tokens; /* R_allocated = sum over batches of |batch| * max true length    */
    int64_t makespan_steps;   /* decode steps until the last batch ends                         */
    int64_t sum_jct_steps;    /* sum over jobs of completion step (submission is step 0)        */
    double padding_ratio;     /* (R_allocated - R_actual) / R_actual; 0 when R_actual == 0      */
    double avg_jct_steps;     /* sum_jct_steps / n; 0 when n == 0                               */
    double throughput;        /* n / makespan_steps (jobs per decode step); 0 when makespan == 0 */
} egtp_sched_report;

/* Runs the model above on jobs taken in `order` (a permutation of 0..n-1, checked:
 * EGTP_ERR_OFFSETS if it is not one) with true lengths true_len[n] (>= 0, EGTP_ERR_SHAPE
 * otherwise; batch_size >= 1).  completion_out[n] (optional) receives each job's completion
 * step, batch_of_out[n] (optional) the batch each job ran in. */
egtp_status egtp_simulate_batches(const int32_t *order, const int32_t *true_len, int32_t n,
                                  int32_t batch_size, egtp_sched_report *report,
                                  int64_t *completion_out, int32_t *batch_of_out);

#ifdef __cplusplus
}
#endif
#endif /* EGTP_SCHED_H */
