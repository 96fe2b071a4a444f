// EdgeShard's two dynamic programs (Sec. 4.1, Eq. 6-8 / Algo. 1; Sec. 4.2, Eq. 11-13 /
// Algo. 2) on the host.  See include/shard_planner.h for the model and the contract.
//
// Readings where the printed algorithms are loose:
//  - Eq. 6 lists its two cases under the min; they are the cases i < N-1 and i = N-1.
//  - Algo. 1 tests Mem_j against Req_i per layer and decrements Mem_j whenever an entry
//    improves, which depends on the visiting order.  Here every table entry carries the
//    memory its own best path has placed on each device, so Eq. 5 holds along the path
//    that is returned (a heuristic once memory binds, exact otherwise).
//  - Eq. 10 is written as a min over devices; it is the min over strategies of the
//    slowest stage.  Algo. 2 compares a candidate with g(i,S,k); it has to be compared
//    with the entry it would replace, g(m,S',j).
//  - Eq. 13 initialises only "one layer on device 0"; here device 0 may own any prefix
//    that fits, otherwise the single-device plan would be unreachable.
#include "../../include/shard_planner.h"

#include <cstddef>
#include <limits>
#include <thread>
#include <vector>

namespace {

const double INF = std::numeric_limits<double>::infinity();

struct View {
    const shard_plan_problem* p;
    int N, M;
    double comp(int i, int j) const { return p->t_comp[static_cast<size_t>(i) * M + j]; }
    double comm(int i, int k, int j) const {  // activation of layer i from device k to device j
        return k == j ? 0.0 : p->act_bytes[i] / p->bandwidth[static_cast<size_t>(k) * M + j];
    }
};

bool valid(const shard_plan_problem* p) {
    return p && p->n_layers >= 1 && p->n_devices >= 1 && p->t_comp && p->act_bytes && p->req_bytes &&
           p->mem_bytes && p->bandwidth;
}

}  // namespace

static int plan_latency_impl(const shard_plan_problem* p, int32_t* device_of_layer, double* t_total) {
    if (!valid(p) || !device_of_layer || !t_total) return -1;
    const View v{p, p->n_layers, p->n_devices};
    const int N = v.N, M = v.M;
    std::vector<double> dp(static_cast<size_t>(N) * M, INF);
    std::vector<int> choice(static_cast<size_t>(N) * M, -1);
    // used[i][j][d]: memory placed on device d by the best path that ends with layer i on j
    std::vector<double> used(static_cast<size_t>(N) * M * M, 0.0);
    auto U = [&](int i, int j) { return used.data() + (static_cast<size_t>(i) * M + j) * M; };

    if (p->req_bytes[0] > p->mem_bytes[0]) return -2;
    dp[0] = v.comp(0, 0);  // Eq. 7 (with N == 1 the result is already on the source)
    U(0, 0)[0] = p->req_bytes[0];
    for (int i = 1; i < N; ++i)
        for (int j = 0; j < M; ++j) {
            double best = INF;
            int arg = -1;
            for (int k = 0; k < M; ++k) {
                const double prev = dp[static_cast<size_t>(i - 1) * M + k];
                if (prev == INF) continue;
                if (U(i - 1, k)[j] + p->req_bytes[i] > p->mem_bytes[j]) continue;  // Eq. 5 along this path
                double t = prev + v.comp(i, j) + v.comm(i - 1, k, j);
                if (i == N - 1) t += v.comm(i, j, 0);  // the result returns to the source
                if (t < best) { best = t; arg = k; }
            }
            if (arg < 0) continue;
            dp[static_cast<size_t>(i) * M + j] = best;
            choice[static_cast<size_t>(i) * M + j] = arg;
            for (int d = 0; d < M; ++d) U(i, j)[d] = U(i - 1, arg)[d];
            U(i, j)[j] += p->req_bytes[i];
        }
    int last = -1;
    double best = INF;
    for (int j = 0; j < M; ++j)
        if (dp[static_cast<size_t>(N - 1) * M + j] < best) { best = dp[static_cast<size_t>(N - 1) * M + j]; last = j; }
    if (last < 0) return -2;
    for (int i = N - 1; i >= 0; --i) {
        device_of_layer[i] = last;
        last = i > 0 ? choice[static_cast<size_t>(i) * M + last] : 0;
    }
    *t_total = best;
    return 0;
}

static int plan_throughput_impl(const shard_plan_problem* p, int32_t with_return_hop, int32_t* device_of_layer,
                                double* t_slowest_stage) {
    if (!valid(p) || !device_of_layer || !t_slowest_stage || p->n_devices > 16) return -1;
    const View v{p, p->n_layers, p->n_devices};
    const int N = v.N, M = v.M;
    const size_t S = static_cast<size_t>(1) << M;
    // prefix sums of compute per device and of memory need
    std::vector<double> pc(static_cast<size_t>(N + 1) * M, 0.0), pr(N + 1, 0.0);
    for (int i = 0; i < N; ++i) {
        pr[i + 1] = pr[i] + p->req_bytes[i];
        for (int j = 0; j < M; ++j) pc[static_cast<size_t>(i + 1) * M + j] = pc[static_cast<size_t>(i) * M + j] + v.comp(i, j);
    }
    auto range_comp = [&](int lo, int hi, int j) {  // layers [lo, hi)
        return pc[static_cast<size_t>(hi) * M + j] - pc[static_cast<size_t>(lo) * M + j];
    };
    // g[c][set][k]: slowest stage so far when the first c layers are placed on the devices of
    // `set`, the last range on device k
    auto idx = [&](int c, size_t set, int k) { return (static_cast<size_t>(c) * S + set) * M + k; };
    std::vector<double> g(static_cast<size_t>(N + 1) * S * M, INF);
    struct Back { int c; int k; };
    std::vector<Back> back(g.size(), Back{-1, -1});
    for (int c = 1; c <= N; ++c)
        if (pr[c] <= p->mem_bytes[0]) g[idx(c, 1, 0)] = range_comp(0, c, 0);
    // Relaxations out of the states with c layers placed.  A state (c, set, k) only writes states
    // (c2 > c, set + {j}, j) with j outside set, so for one c different sets never write the same
    // entry: the sets are dealt out to host threads, each set's k loop stays in one thread, and
    // the result does not depend on the number of threads.
    auto relax = [&](int c, size_t set_lo, size_t set_hi) {
        for (size_t set = set_lo | 1; set < set_hi; set += 2)  // device 0 is always in the set
            for (int k = 0; k < M; ++k) {
                const double cur = g[idx(c, set, k)];
                if (cur == INF) continue;
                for (int j = 0; j < M; ++j) {
                    if (set >> j & 1) continue;
                    const double recv = v.comm(c - 1, k, j);
                    for (int c2 = c + 1; c2 <= N; ++c2) {
                        if (pr[c2] - pr[c] > p->mem_bytes[j]) break;  // Eq. 12
                        double t = cur;
                        if (recv > t) t = recv;
                        const double comp = range_comp(c, c2, j);
                        if (comp > t) t = comp;
                        const size_t to = idx(c2, set | (static_cast<size_t>(1) << j), j);
                        if (t < g[to]) { g[to] = t; back[to] = Back{c, k}; }
                    }
                }
            }
    };
    unsigned n_threads = std::thread::hardware_concurrency();
    if (n_threads > 16) n_threads = 16;
    if (n_threads < 1 || S < 4096) n_threads = 1;   // small problems: not worth a thread
    for (int c = 1; c < N; ++c) {
        if (n_threads == 1) { relax(c, 0, S); continue; }
        std::vector<std::thread> pool;
        const size_t chunk = (S / n_threads + 1) & ~static_cast<size_t>(1);   // even boundaries
        for (unsigned t = 0; t < n_threads; ++t) {
            const size_t lo = t * chunk, hi = t + 1 == n_threads ? S : (t + 1) * chunk;
            if (lo < S) pool.emplace_back(relax, c, lo, hi < S ? hi : S);
        }
        for (auto& th : pool) th.join();
    }
    double best = INF;
    size_t bset = 0;
    int bk = -1;
    for (size_t set = 1; set < S; set += 2)
        for (int k = 0; k < M; ++k) {
            double t = g[idx(N, set, k)];
            if (t == INF) continue;
            if (with_return_hop) {
                const double r = v.comm(N - 1, k, 0);
                if (r > t) t = r;
            }
            if (t < best) { best = t; bset = set; bk = k; }
        }
    if (bk < 0) return -2;
    int c = N;
    while (c > 0) {
        const Back b = back[idx(c, bset, bk)];
        const int lo = b.c < 0 ? 0 : b.c;
        for (int i = lo; i < c; ++i) device_of_layer[i] = bk;
        if (b.c < 0) break;
        bset &= ~(static_cast<size_t>(1) << bk);
        bk = b.k;
        c = b.c;
    }
    *t_slowest_stage = best;
    return 0;
}

// Nothing throws across the C boundary: a failed host allocation or thread start is -3.
extern "C" int shard_plan_latency(const shard_plan_problem* p, int32_t* device_of_layer, double* t_total) {
    try {
        return plan_latency_impl(p, device_of_layer, t_total);
    } catch (...) {
        return -3;
    }
}

extern "C" int shard_plan_throughput(const shard_plan_problem* p, int32_t with_return_hop, int32_t* device_of_layer,
                                     double* t_slowest_stage) {
    try {
        return plan_throughput_impl(p, with_return_hop, device_of_layer, t_slowest_stage);
    } catch (...) {
        return -3;
    }
}

extern "C" int shard_plan_to_stages(int32_t n_layers, int32_t n_devices, const int32_t* device_of_layer,
                                    const double* t_prefill, const double* t_decode, const double* act_prefill,
                                    const double* act_decode, const double* bandwidth, int32_t* n_stages,
                                    int32_t* stage_device, double* t_stage_prefill, double* t_stage_decode,
                                    double* c_prefill, double* c_decode, double* c_return) {
    if (n_layers < 1 || n_devices < 1 || !device_of_layer || !t_prefill || !t_decode || !act_prefill || !act_decode ||
        !bandwidth || !n_stages || !stage_device || !t_stage_prefill || !t_stage_decode || !c_prefill || !c_decode || !c_return)
        return -1;
    const int N = n_layers, M = n_devices;
    for (int i = 0; i < N; ++i)
        if (device_of_layer[i] < 0 || device_of_layer[i] >= M) return -1;
    auto link = [&](int k, int j) { return bandwidth[static_cast<size_t>(k) * M + j]; };
    int S = 0;
    for (int i = 0; i < N; ++i) {
        const int dev = device_of_layer[i];
        if (i == 0 || dev != device_of_layer[i - 1]) {
            for (int s = 0; s < S; ++s)
                if (stage_device[s] == dev) return -2;   // the device already closed a range
            if (S > 0) {                                 // Eq. 1 for the activation that crosses into the new stage
                const double bw = link(stage_device[S - 1], dev);
                if (!(bw > 0.0)) return -1;
                c_prefill[S - 1] = act_prefill[i - 1] / bw;
                c_decode[S - 1] = act_decode[i - 1] / bw;
            }
            stage_device[S] = dev;
            t_stage_prefill[S] = 0.0;
            t_stage_decode[S] = 0.0;
            ++S;
        }
        t_stage_prefill[S - 1] += t_prefill[static_cast<size_t>(i) * M + dev];   // the compute term of Eq. 9
        t_stage_decode[S - 1] += t_decode[static_cast<size_t>(i) * M + dev];
    }
    *c_return = 0.0;
    if (stage_device[S - 1] != stage_device[0]) {
        const double bw = link(stage_device[S - 1], stage_device[0]);
        if (!(bw > 0.0)) return -1;
        *c_return = act_decode[N - 1] / bw;
    }
    *n_stages = S;
    return 0;
}
