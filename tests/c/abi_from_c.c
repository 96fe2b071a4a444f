/* The boundary used from plain C99: the three headers compile with -pedantic, the library links,
 * error reporting works without a GPU, and a host-only entry point returns the closed form for
 * balanced stages without bubbles, (S - 1) t + MB (1 + n) t (hand-off times zero). */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "shard.h"
#include "shard_planner.h"
#include "shard_schedule.h"

int main(void) {
    const double t[3] = {2.0, 2.0, 2.0}, c[2] = {0.0, 0.0};
    shard_pipeline_problem p;
    double makespan = -1.0, busy[3] = {0.0, 0.0, 0.0};
    int s;
    memset(&p, 0, sizeof p);
    p.n_stages = 3; p.n_micro = 4; p.n_decode = 5;
    p.t_prefill = t; p.t_decode = t; p.c_prefill = c; p.c_decode = c; p.c_return = 0.0;
    if (shard_simulate_pipeline(&p, 1, &makespan, busy) != 0) { printf("simulate failed\n"); return 1; }
    if (fabs(makespan - ((3 - 1) * 2.0 + 4 * (1 + 5) * 2.0)) > 1e-12) { printf("makespan %g\n", makespan); return 2; }
    for (s = 0; s < 3; ++s)
        if (fabs(busy[s] - 4 * (1 + 5) * 2.0) > 1e-12) { printf("busy[%d] %g\n", s, busy[s]); return 3; }
    if (shard_simulate_pipeline(NULL, 1, &makespan, busy) != -1) { printf("NULL accepted\n"); return 4; }
    /* a call that must fail before it touches a GPU, and say why */
    if (shard_seq_alloc(NULL, NULL) != SHARD_E_INVAL) { printf("seq_alloc(NULL) accepted\n"); return 5; }
    if (shard_last_error() == NULL || strlen(shard_last_error()) == 0) { printf("no error text\n"); return 6; }
    printf("ok\n");
    return 0;
}
