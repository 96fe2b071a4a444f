// Event-driven simulation of EdgeShard's two pipeline execution strategies (Sec. 4.2
// "Pipeline Execution Optimization", Fig. 5).  See include/shard_schedule.h for the model.
#include "../../include/shard_schedule.h"

#include <cmath>
#include <cstddef>
#include <queue>
#include <vector>

namespace {

struct Task {
    double ready;
    int it, m;
};
struct Later {  // priority queue order: earliest ready first, then lower iteration, then lower m
    bool operator()(const Task& a, const Task& b) const {
        if (a.ready != b.ready) return a.ready > b.ready;
        if (a.it != b.it) return a.it > b.it;
        return a.m > b.m;
    }
};

bool good(double v) { return std::isfinite(v) && v >= 0.0; }

}  // namespace

static int simulate_impl(const shard_pipeline_problem* p, int32_t no_bubbles, double* makespan_s, double* busy_s) {
    if (!p || !makespan_s || p->n_stages < 1 || p->n_micro < 1 || p->n_decode < 0 || !p->t_prefill || !p->t_decode)
        return -1;
    const int S = p->n_stages, MB = p->n_micro, IT = 1 + p->n_decode;
    if (S > 1 && (!p->c_prefill || !p->c_decode)) return -1;
    if (!good(p->c_return)) return -1;
    for (int s = 0; s < S; ++s) {
        if (!good(p->t_prefill[s]) || !good(p->t_decode[s])) return -1;
        if (s + 1 < S && (!good(p->c_prefill[s]) || !good(p->c_decode[s]))) return -1;
    }
    std::vector<std::priority_queue<Task, std::vector<Task>, Later>> waiting(S);
    std::vector<double> free_at(S, 0.0), busy(S, 0.0);
    std::vector<double> back(static_cast<size_t>(IT) * MB, 0.0);  // when iteration i of m is back at the source
    std::vector<int> returned(IT, 0);                             // micro-batches of iteration i that are back
    for (int m = 0; m < MB; ++m) waiting[0].push(Task{0.0, 0, m});
    long remaining = static_cast<long>(S) * MB * IT;
    double makespan = 0.0;
    while (remaining > 0) {
        // the stage whose next task starts first (ties: lower stage)
        int best = -1;
        double best_start = 0.0;
        for (int s = 0; s < S; ++s) {
            if (waiting[s].empty()) continue;
            const double r = waiting[s].top().ready;
            const double st = r > free_at[s] ? r : free_at[s];
            if (best < 0 || st < best_start) { best = s; best_start = st; }
        }
        if (best < 0) return -1;  // cannot happen: some task is always waiting
        const int s = best;
        // among the tasks ready by the time the stage is free, the one that became ready first
        const Task t = waiting[s].top();
        waiting[s].pop();
        const double dur = t.it == 0 ? p->t_prefill[s] : p->t_decode[s];
        const double fin = best_start + dur;
        free_at[s] = fin;
        busy[s] += dur;
        --remaining;
        if (s + 1 < S) {
            const double c = t.it == 0 ? p->c_prefill[s] : p->c_decode[s];
            waiting[s + 1].push(Task{fin + c, t.it, t.m});
            continue;
        }
        const double home = fin + p->c_return;
        if (home > makespan) makespan = home;
        back[static_cast<size_t>(t.it) * MB + t.m] = home;
        returned[t.it] += 1;
        if (t.it + 1 >= IT) continue;
        if (no_bubbles) {
            waiting[0].push(Task{home, t.it + 1, t.m});
        } else if (returned[t.it] == MB) {  // the barrier: everyone enters the next iteration together
            double all = 0.0;
            for (int m = 0; m < MB; ++m) all = all > back[static_cast<size_t>(t.it) * MB + m] ? all : back[static_cast<size_t>(t.it) * MB + m];
            for (int m = 0; m < MB; ++m) waiting[0].push(Task{all, t.it + 1, m});
        }
    }
    *makespan_s = makespan;
    if (busy_s)
        for (int s = 0; s < S; ++s) busy_s[s] = busy[s];
    return 0;
}

// Nothing throws across the C boundary: a failed host allocation is -3.
extern "C" int shard_simulate_pipeline(const shard_pipeline_problem* p, int32_t no_bubbles, double* makespan_s,
                                       double* busy_s) {
    try {
        return simulate_impl(p, no_bubbles, makespan_s, busy_s);
    } catch (...) {
        return -3;
    }
}
