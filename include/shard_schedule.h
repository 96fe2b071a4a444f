/*
 * Host-side model of EdgeShard's pipeline execution (Sec. 4.2 "Pipeline Execution
 * Optimization", Fig. 5): S pipeline stages (the devices of a throughput plan, in layer
 * order), MB micro-batches, each of which runs one prefill iteration and then n_decode
 * autoregressive iterations.  Iteration i+1 of a micro-batch cannot enter stage 0 before
 * its iteration i has left the last stage and the generated token is back at the source
 * (the autoregressive dependency that causes the bubbles).  Pure CPU code.
 *
 * Task (m, i, s) = micro-batch m, iteration i, stage s.  It may start when
 *   - s > 0: task (m, i, s-1) has finished and its activation has crossed link s-1 -> s;
 *   - s = 0, i > 0: task (m, i-1, S-1) has finished and the token has crossed the return
 *     link to stage 0;
 *   - the stage is free: a stage runs one task at a time, without preemption, and takes
 *     the waiting task that became ready first (ties: lower iteration, then lower m).
 * Two strategies (the paper defines them by the figure and its caption; this is the
 * reading taken):
 *   - Bubbles: iteration i+1 of ANY micro-batch enters stage 0 only after iteration i of
 *     ALL micro-batches has finished and returned (a barrier per iteration);
 *   - No-bubbles: only the per-micro-batch dependency above.
 */
#ifndef SHARD_SCHEDULE_H
#define SHARD_SCHEDULE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t n_stages;        /* S >= 1 */
    int32_t n_micro;         /* MB >= 1 */
    int32_t n_decode;        /* autoregressive iterations after the prefill, >= 0 */
    const double *t_prefill; /* [S] seconds of one micro-batch's prefill on stage s, host pointer */
    const double *t_decode;  /* [S] seconds of one decode iteration on stage s */
    const double *c_prefill; /* [S-1] transfer of a prefill activation, stage s -> s+1 (NULL if S == 1) */
    const double *c_decode;  /* [S-1] the same for one decode iteration */
    double c_return;         /* transfer of a generated token from the last stage to stage 0 */
} shard_pipeline_problem;

/* Simulate the schedule.  no_bubbles: 0 = Bubbles, otherwise No-bubbles.
 * makespan_s (out): time at which the last token is back at the source.
 * busy_s (out, host array [S], may be NULL): seconds each stage spent computing.
 * Tokens produced: MB * (1 + n_decode) per sequence of a micro-batch; throughput is that
 * count times the micro-batch size divided by the makespan.
 * Returns 0, -1 on bad arguments (NULL, sizes out of range, negative or non-finite times), or
 * -3 when a host allocation failed. */
int shard_simulate_pipeline(const shard_pipeline_problem *p, int32_t no_bubbles,
                            double *makespan_s, double *busy_s);

#ifdef __cplusplus
}
#endif
#endif /* SHARD_SCHEDULE_H */
