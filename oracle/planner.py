"""CPU oracle for EdgeShard's two placement problems: the optimisation problems as the
paper states them, solved by exhaustive enumeration.

TEST INFRASTRUCTURE ONLY (see oracle/llama_shard.py); shares no code with the library's
dynamic programs.

Sequential inference (Sec. 4.1): choose a device for every layer, layer 0 on device 0
(Eq. 4), the layers on a device within its memory (Eq. 5), minimising Eq. 2's
    T = sum_i t_comp[i][dev(i)] + sum_{i>=1} comm(i-1, dev(i-1), dev(i))
plus the return of the last activation to device 0 that Eq. 6 adds, with
    comm(i, k, j) = O_i / B[k][j] if k != j else 0                                (Eq. 1).
Pipeline-parallel inference (Sec. 4.2): every used device owns one contiguous range, the
first range on device 0; a stage costs max(compute of its range, receiving its input)
(Eq. 9); minimise the slowest stage (Eq. 10) subject to Eq. 12.

Pinned by tests/test_planner.py: hand-computed two-layer examples, single-device and
infinite / zero-bandwidth closed forms; stages_of by a hand-worked five-layer plan and by the
identity max(stage compute, incoming link) = stage_time_of.
"""
from __future__ import annotations

import itertools

import numpy as np


def comm(prob, i, k, j):
    return 0.0 if k == j else prob["act_bytes"][i] / prob["bandwidth"][k][j]


def latency_of(prob, dev):
    n = len(dev)
    t = sum(prob["t_comp"][i][dev[i]] for i in range(n))
    t += sum(comm(prob, i - 1, dev[i - 1], dev[i]) for i in range(1, n))
    return t + comm(prob, n - 1, dev[n - 1], 0)


def fits(prob, dev):
    used = np.zeros(len(prob["mem_bytes"]))
    for i, j in enumerate(dev):
        used[j] += prob["req_bytes"][i]
    return bool(np.all(used <= np.asarray(prob["mem_bytes"])))


def best_latency(prob):
    """(optimal T, one optimal assignment) over all M^(N-1) assignments."""
    n, m = len(prob["t_comp"]), len(prob["mem_bytes"])
    best, arg = np.inf, None
    for rest in itertools.product(range(m), repeat=n - 1):
        dev = (0,) + rest
        if not fits(prob, dev):
            continue
        t = latency_of(prob, dev)
        if t < best:
            best, arg = t, dev
    return best, arg


def stage_time_of(prob, dev, with_return_hop=False):
    """Slowest stage of a contiguous-range assignment (Eq. 9-10)."""
    n = len(dev)
    worst, i = 0.0, 0
    while i < n:
        j = dev[i]
        hi = i
        while hi < n and dev[hi] == j:
            hi += 1
        stage = sum(prob["t_comp"][l][j] for l in range(i, hi))
        if i > 0:
            stage = max(stage, comm(prob, i - 1, dev[i - 1], j))
        worst = max(worst, stage)
        i = hi
    if with_return_hop:
        worst = max(worst, comm(prob, n - 1, dev[n - 1], 0))
    return worst


def best_throughput(prob, with_return_hop=False):
    """(optimal slowest-stage time, assignment) over every ordered choice of distinct devices
    starting with device 0 and every way to cut the layers into that many ranges."""
    n, m = len(prob["t_comp"]), len(prob["mem_bytes"])
    best, arg = np.inf, None
    others = list(range(1, m))
    for stages in range(1, min(n, m) + 1):
        for tail in itertools.permutations(others, stages - 1):
            order = (0,) + tail
            for cuts in itertools.combinations(range(1, n), stages - 1):
                bounds = (0,) + cuts + (n,)
                dev = []
                for s in range(stages):
                    dev += [order[s]] * (bounds[s + 1] - bounds[s])
                if not fits(prob, dev):
                    continue
                t = stage_time_of(prob, dev, with_return_hop)
                if t < best:
                    best, arg = t, tuple(dev)
    return best, arg


def stages_of(dev, t_prefill, t_decode, act_prefill, act_decode, bandwidth):
    """The pipeline a contiguous-range plan describes (Sec. 4.2): per stage the sum of its
    layers' times on its device (the compute term of Eq. 9), per boundary the time O_i / B of
    the activation that crosses it (Eq. 1), and the return of the last activation to the first
    stage's device.  Written stage by stage from the definition: list the maximal runs of equal
    devices, then read each quantity off the run."""
    runs = []                                   # (device, first layer, one past the last layer)
    for i, d in enumerate(dev):
        if runs and runs[-1][0] == d:
            runs[-1] = (d, runs[-1][1], i + 1)
        else:
            runs.append((d, i, i + 1))
    devices = [r[0] for r in runs]
    if len(set(devices)) != len(devices):
        raise ValueError("a device owns two separate ranges")
    tp = [sum(t_prefill[l][d] for l in range(lo, hi)) for d, lo, hi in runs]
    td = [sum(t_decode[l][d] for l in range(lo, hi)) for d, lo, hi in runs]
    cp = [act_prefill[a[2] - 1] / bandwidth[a[0]][b[0]] for a, b in zip(runs[:-1], runs[1:])]
    cd = [act_decode[a[2] - 1] / bandwidth[a[0]][b[0]] for a, b in zip(runs[:-1], runs[1:])]
    last = len(dev) - 1
    c_ret = 0.0 if devices[-1] == devices[0] else act_decode[last] / bandwidth[devices[-1]][devices[0]]
    return dict(stages=devices, t_prefill=tp, t_decode=td, c_prefill=cp, c_decode=cd, c_return=c_ret)
