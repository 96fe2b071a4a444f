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
 * feasible assignment was found, -3 when a host allocation failed. */
int shard_plan_latency(const shard_plan_problem *p, int32_t *device_of_layer, double *t_total);

/* Pipeline-parallel inference (Sec. 4.2): every selected device gets ONE contiguous range
 * of layers; a stage's time is max(compute of its range, time to receive its input)
 * (Eq. 9); minimise the slowest stage (Eq. 10) by the dynamic program of Eq. 11-13 /
 * Algo. 2 over (layers placed, device set, last device).  Exact for this formulation,
 * memory limits included (Eq. 12).  with_return_hop != 0 also counts the transfer of the
 * last activation back to device 0 as a stage.
 * Returns 0, -1 on bad arguments (or M > 16), -2 when nothing fits, -3 when a host
 * allocation or thread start failed. */
int shard_plan_throughput(const shard_plan_problem *p, int32_t with_return_hop,
                          int32_t *device_of_layer, double *t_slowest_stage);

/* From a plan to the pipeline it describes (Sec. 4.2): the devices of a throughput plan, in
 * layer order, are the stages; a stage's compute time is the sum of its layers' times on its
 * device (the t_comp term of Eq. 9), and the link between two consecutive stages carries the
 * output activation of the earlier stage's last layer, O_i / B_{k,j} (Eq. 1; the t_comm term of
 * Eq. 9); the generated token returns from the last stage's device to the first's over
 * O_{N-1} / B (zero when they are the same device).  These are the inputs of
 * shard_simulate_pipeline (shard_schedule.h).
 *   device_of_layer   [N]     a plan in which every device owns ONE contiguous range
 *   t_prefill, t_decode [N][M] seconds of layer i on device j in the prefill / in one decode
 *                             iteration (the two columns shard_profile measures)
 *   act_prefill, act_decode [N] bytes of layer i's output activation in the two phases
 *   bandwidth         [M][M]  bytes per second
 * Outputs (host arrays of N entries each, of which the first *n_stages are written):
 * stage_device, t_stage_prefill, t_stage_decode; c_prefill and c_decode hold *n_stages - 1
 * link times; *c_return the return hop.
 * Returns 0; -1 on bad arguments (NULL, sizes, a device index outside [0, M), a bandwidth
 * that is not positive on a link the plan uses); -2 when a device owns two separate ranges
 * (legal for the latency plan of Sec. 4.1, but not a pipeline). */
int shard_plan_to_stages(int32_t n_layers, int32_t n_devices, const int32_t *device_of_layer,
                         const double *t_prefill, const double *t_decode,
                         const double *act_prefill, const double *act_decode, const double *bandwidth,
                         int32_t *n_stages, int32_t *stage_device,
                         double *t_stage_prefill, double *t_stage_decode,
                         double *c_prefill, double *c_decode, double *c_return);

#ifdef __cplusplus
}
#endif
#endif /* SHARD_PLANNER_H */
