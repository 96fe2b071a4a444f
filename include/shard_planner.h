/*
 * Host-side planner: EdgeShard's joint device selection and layer partition (Sec. 4),
 * fed by the per-layer profiles shard_profile() measures.  Pure CPU code; it is not part
 * of the GPU hot path.
 *
 * Model (Sec. 4 "System Model"): N layers, M devices; t_comp[i][j] = time of layer i on
 * device j; act_bytes[i] = O_i, the size of layer i's output activation; req_bytes[i] =
 * Req_i; mem_bytes[j] = Mem_j; bandwidth[k][j] = B_{k,j} in bytes per second.  Sending
 * layer i's activation from k to j costs O_i / B_{k,j}, and nothing when k == j (Eq. 1).
 * Layer 0 is pinned to device 0, the source node (Eq. 4).
 */
#ifndef SHARD_PLANNER_H
#define SHARD_PLANNER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t n_layers;        /* N >= 1 */
    int32_t n_devices;       /* M >= 1 (throughput planning: M <= 16) */
    const double *t_comp;    /* [N][M] seconds, host pointer */
    const double *act_bytes; /* [N] */
    const double *req_bytes; /* [N] */
    const double *mem_bytes; /* [M] */
    const double *bandwidth; /* [M][M] bytes/s; entries with k == j are ignored */
} shard_plan_problem;

/* Sequential inference (Sec. 4.1): minimise the total time of one token,
 *   T = sum_i t_comp[i][dev(i)] + sum_{i>=1} comm(i-1, dev(i-1), dev(i)) + comm(N-1, dev(N-1), 0)
 * (Eq. 2 plus the return of the result to the source, which Eq. 6 adds for the last layer),
 * by the dynamic program of Eq. 6-8 / Algo. 1.  Without binding memory limits the result is
 * the exact optimum.  With them the program is the paper's heuristic: each table entry
 * carries the memory its own best path has used on every device, and a transition is
 * allowed only if layer i still fits (Eq. 5 along that path).
 * device_of_layer: host array [N] (out).  Returns 0, -1 on bad arguments, -2 when no
 * feasible assignment was found. */
int shard_plan_latency(const shard_plan_problem *p, int32_t *device_of_layer, double *t_total);

/* Pipeline-parallel inference (Sec. 4.2): every selected device gets ONE contiguous range
 * of layers; a stage's time is max(compute of its range, time to receive its input)
 * (Eq. 9); minimise the slowest stage (Eq. 10) by the dynamic program of Eq. 11-13 /
 * Algo. 2 over (layers placed, device set, last device).  Exact for this formulation,
 * memory limits included (Eq. 12).  with_return_hop != 0 also counts the transfer of the
 * last activation back to device 0 as a stage.
 * Returns 0, -1 on bad arguments (or M > 16), -2 when nothing fits. */
int shard_plan_throughput(const shard_plan_problem *p, int32_t with_return_hop,
                          int32_t *device_of_layer, double *t_slowest_stage);

#ifdef __cplusplus
}
#endif
#endif /* SHARD_PLANNER_H */
