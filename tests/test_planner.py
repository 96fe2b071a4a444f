"""Planner (EdgeShard Sec. 4): pins for the brute-force oracle, then the library's dynamic
programs against it.  CPU only."""
import numpy as np
import pytest

from oracle import planner as orc


def problem(n, m, seed, mem=1e18, bw_scale=1.0):
    rng = np.random.default_rng(seed)
    bw = rng.uniform(0.5, 2.0, (m, m)) * bw_scale
    return dict(t_comp=rng.uniform(0.5, 3.0, (n, m)), act_bytes=rng.uniform(0.5, 2.0, n),
                req_bytes=rng.uniform(1.0, 2.0, n), mem_bytes=np.full(m, mem), bandwidth=bw)


# ---- the oracle itself: hand-computed and closed-form cases ------------------------------
def test_oracle_hand_computed_two_layers_two_devices():
    # layer times: device 0 is slow (4, 4), device 1 fast (1, 1); O = (6, 2); B = 2 both ways.
    prob = dict(t_comp=[[4.0, 1.0], [4.0, 1.0]], act_bytes=[6.0, 2.0], req_bytes=[1.0, 1.0],
                mem_bytes=[10.0, 10.0], bandwidth=[[1.0, 2.0], [2.0, 1.0]])
    # both local: 4 + 4 = 8.  layer 1 remote: 4 + 1 + 6/2 (send) + 2/2 (return) = 9.
    assert orc.latency_of(prob, (0, 0)) == 8.0
    assert orc.latency_of(prob, (0, 1)) == 9.0
    assert orc.best_latency(prob) == (8.0, (0, 0))
    # pipeline: one stage: 8.  two stages: max(4, max(1, 6/2)) = 4.
    assert orc.stage_time_of(prob, (0, 0)) == 8.0
    assert orc.stage_time_of(prob, (0, 1)) == 4.0
    assert orc.best_throughput(prob) == (4.0, (0, 1))
    assert orc.stage_time_of(prob, (0, 1), with_return_hop=True) == 4.0
    prob["act_bytes"] = [6.0, 20.0]     # an expensive return hop dominates when it is counted
    assert orc.stage_time_of(prob, (0, 1), with_return_hop=True) == 10.0
    assert orc.best_throughput(prob, with_return_hop=True) == (8.0, (0, 0))


def test_oracle_closed_forms():
    prob = problem(5, 3, 1)
    solo = dict(prob, t_comp=prob["t_comp"][:, :1], mem_bytes=prob["mem_bytes"][:1], bandwidth=prob["bandwidth"][:1, :1])
    assert orc.best_latency(solo)[0] == pytest.approx(prob["t_comp"][:, 0].sum())       # one device: sum of its times
    assert orc.best_throughput(solo)[0] == pytest.approx(prob["t_comp"][:, 0].sum())
    fast = problem(5, 3, 2, bw_scale=1e15)                                             # free links: fastest device per layer
    want = fast["t_comp"][0, 0] + fast["t_comp"][1:].min(axis=1).sum()
    assert orc.best_latency(fast)[0] == pytest.approx(want, rel=1e-9)
    slow = problem(5, 3, 3, bw_scale=1e-15)                                            # dead links: everything stays local
    assert orc.best_latency(slow)[1] == (0,) * 5
    assert orc.best_throughput(slow)[1] == (0,) * 5
    tight = problem(4, 2, 4, mem=4.0)                                                  # memory forces a split
    dev = orc.best_latency(tight)[1]
    assert orc.fits(tight, dev) and len(set(dev)) == 2


# ---- the library's dynamic programs against the enumeration ----------------------------------
@pytest.mark.parametrize("n,m,seed", [(2, 2, 0), (5, 3, 1), (6, 3, 2), (7, 2, 3), (4, 4, 4), (8, 3, 5)])
def test_latency_dp_is_optimal_when_memory_does_not_bind(lib, n, m, seed):
    for bw_scale in (0.05, 1.0, 50.0):
        prob = problem(n, m, seed, bw_scale=bw_scale)
        t, dev = lib.plan_latency(prob)
        want, _ = orc.best_latency(prob)
        assert t == pytest.approx(want, rel=1e-12)
        assert dev[0] == 0 and orc.latency_of(prob, dev) == pytest.approx(t, rel=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_latency_dp_with_binding_memory_is_feasible_and_consistent(lib, seed):
    prob = problem(6, 3, 10 + seed, mem=4.5)
    t, dev = lib.plan_latency(prob)
    assert orc.fits(prob, dev) and dev[0] == 0
    assert orc.latency_of(prob, dev) == pytest.approx(t, rel=1e-12)
    assert t >= orc.best_latency(prob)[0] - 1e-12          # a heuristic here: never better than the optimum


@pytest.mark.parametrize("n,m,seed,mem", [(3, 2, 0, 1e18), (6, 3, 1, 1e18), (7, 4, 2, 1e18), (8, 3, 3, 5.0),
                                          (6, 4, 4, 3.2), (8, 4, 5, 4.1)])
@pytest.mark.parametrize("hop", [False, True])
def test_throughput_dp_matches_enumeration(lib, n, m, seed, mem, hop):
    for bw_scale in (0.1, 1.0, 30.0):
        prob = problem(n, m, seed, mem=mem, bw_scale=bw_scale)
        want, _ = orc.best_throughput(prob, hop)
        if not np.isfinite(want):
            with pytest.raises(lib.ShardError):
                lib.plan_throughput(prob, hop)
            continue
        t, dev = lib.plan_throughput(prob, hop)
        assert t == pytest.approx(want, rel=1e-12)
        assert dev[0] == 0 and orc.fits(prob, dev)
        assert orc.stage_time_of(prob, dev, hop) == pytest.approx(t, rel=1e-12)
        # one contiguous range per device
        runs = [d for i, d in enumerate(dev) if i == 0 or dev[i - 1] != d]
        assert len(runs) == len(set(runs))


@pytest.mark.parametrize("seed", [11, 12])
def test_throughput_dp_on_many_devices_equals_the_problem_without_the_useless_ones(lib, seed):
    """13 devices (8192 subsets: the size from which the dynamic program deals the subsets out
    to host threads), nine of them without memory for a single layer: the optimum is that of
    the four usable devices alone, which the enumeration above covers, and the plan uses only
    those."""
    small = problem(9, 4, seed, mem=6.0, bw_scale=1.0)
    keep = [0, 5, 7, 12]                      # where the four usable devices sit in the big problem
    m = 13
    rng = np.random.default_rng(100 + seed)
    big = dict(t_comp=rng.uniform(0.01, 0.02, (9, m)),     # the useless devices would be much faster
               act_bytes=small["act_bytes"], req_bytes=small["req_bytes"],
               mem_bytes=np.zeros(m), bandwidth=rng.uniform(50.0, 60.0, (m, m)))
    for a, ka in enumerate(keep):
        big["t_comp"][:, ka] = small["t_comp"][:, a]
        big["mem_bytes"][ka] = small["mem_bytes"][a]
        for b, kb in enumerate(keep):
            big["bandwidth"][ka, kb] = small["bandwidth"][a, b]
    for hop in (False, True):
        want, _ = orc.best_throughput(small, hop)
        t_small, _ = lib.plan_throughput(small, hop)
        t_big, dev = lib.plan_throughput(big, hop)
        assert t_small == pytest.approx(want, rel=1e-12)
        assert t_big == pytest.approx(want, rel=1e-12)
        assert set(dev) <= set(keep) and dev[0] == 0


def test_paper_baselines_are_special_cases(lib):
    """Edge-Solo is the plan with one device; Cloud-Edge-Opt the plan with two; the planner
    over the full pool is never worse than either (Sec. 5.1 "Baselines", Sec. 5.2)."""
    prob = problem(8, 4, 7, bw_scale=0.5)
    sub = lambda k: dict(prob, t_comp=prob["t_comp"][:, :k], mem_bytes=prob["mem_bytes"][:k], bandwidth=prob["bandwidth"][:k, :k])
    solo, _ = lib.plan_latency(sub(1))
    two, _ = lib.plan_latency(sub(2))
    full, _ = lib.plan_latency(prob)
    assert solo == pytest.approx(prob["t_comp"][:, 0].sum())
    assert full <= two + 1e-12 <= solo + 2e-12
    # latency is monotone in bandwidth
    faster, _ = lib.plan_latency(dict(prob, bandwidth=prob["bandwidth"] * 4))
    assert faster <= full + 1e-12


def test_planner_rejects_bad_arguments(lib):
    prob = problem(3, 2, 0, mem=0.5)                       # nothing fits, not even layer 0
    with pytest.raises(lib.ShardError) as e:
        lib.plan_latency(prob)
    assert e.value.code == -2
    assert lib.load().shard_plan_latency(None, None, None) == -1
    assert lib.load().shard_plan_throughput(None, 0, None, None) == -1


# --------------------------------------------------------------------------------------
# From a plan to pipeline stages (the compute and link terms of Eq. 9, Eq. 1)
# --------------------------------------------------------------------------------------
def test_oracle_stages_hand_worked_five_layers():
    """Plan (0, 0, 2, 2, 1) over three devices, worked by hand:
    stage times are column sums over the runs, the two links carry the activations of layers
    1 and 3, the token returns from device 1 to device 0."""
    tp = [[1, 9, 9], [2, 9, 9], [9, 9, 3], [9, 9, 4], [9, 5, 9]]
    td = [[.1, 9, 9], [.2, 9, 9], [9, 9, .3], [9, 9, .4], [9, .5, 9]]
    ap, ad = [10, 20, 30, 40, 50], [1, 2, 3, 4, 5]
    bw = [[0, 7, 4], [5, 0, 7], [7, 8, 0]]
    st = orc.stages_of((0, 0, 2, 2, 1), tp, td, ap, ad, bw)
    assert st["stages"] == [0, 2, 1]
    assert st["t_prefill"] == [3, 7, 5]
    assert st["t_decode"] == pytest.approx([0.3, 0.7, 0.5])
    assert st["c_prefill"] == pytest.approx([20 / 4, 40 / 8])
    assert st["c_decode"] == pytest.approx([2 / 4, 4 / 8])
    assert st["c_return"] == pytest.approx(5 / 5)
    with pytest.raises(ValueError):
        orc.stages_of((0, 1, 0), tp[:3], td[:3], ap[:3], ad[:3], bw)


@pytest.mark.parametrize("seed", range(6))
def test_stages_agree_with_the_stage_time_of_eq9(lib, seed):
    """max over stages of max(compute, incoming link) read off the collapsed stages is Eq. 9-10's
    slowest stage, which the enumeration oracle computes directly from the plan; and the
    library's shard_plan_to_stages returns what the oracle's stages_of does."""
    rng = np.random.default_rng(100 + seed)
    N, M = int(rng.integers(3, 9)), int(rng.integers(2, 5))
    tdec = rng.uniform(0.1, 1.0, (N, M)); tpre = rng.uniform(1.0, 5.0, (N, M))
    act = rng.uniform(1.0, 4.0, N); bw = rng.uniform(2.0, 20.0, (M, M))
    prob = dict(t_comp=tdec, act_bytes=act, req_bytes=np.ones(N), mem_bytes=np.full(M, N / 2 + 0.5), bandwidth=bw)
    _, dev = lib.plan_throughput(prob)
    want = orc.stages_of(dev, tpre, tdec, 8 * act, act, bw)
    got = lib.stages_of_plan(dev, tpre, tdec, 8 * act, act, bw)
    assert got["stages"] == want["stages"]
    for k in ("t_prefill", "t_decode", "c_prefill", "c_decode"):
        assert got[k] == pytest.approx(want[k], rel=1e-12), k
    assert got["c_return"] == pytest.approx(want["c_return"], rel=1e-12)
    slowest = max(max(t, c) for t, c in zip(want["t_decode"], [0.0] + want["c_decode"]))
    assert slowest == pytest.approx(orc.stage_time_of(prob, dev))
    assert max(slowest, want["c_return"]) == pytest.approx(orc.stage_time_of(prob, dev, with_return_hop=True))


def test_plan_to_stages_rejects_what_is_not_a_pipeline(lib):
    tp = np.ones((3, 2)); act = np.ones(3); bw = np.ones((2, 2))
    with pytest.raises(lib.ShardError) as e:
        lib.stages_of_plan([0, 1, 0], tp, tp, act, act, bw)      # device 0 owns two ranges
    assert e.value.code == -2
    with pytest.raises(lib.ShardError) as e:
        lib.stages_of_plan([0, 2, 2], tp, tp, act, act, bw)      # device index outside [0, M)
    assert e.value.code == -1
    with pytest.raises(lib.ShardError) as e:
        lib.stages_of_plan([0, 1, 1], tp, tp, act, act, np.zeros((2, 2)))   # a used link without bandwidth
    assert e.value.code == -1
    one = lib.stages_of_plan([0, 0, 0], tp, 2 * tp, act, act, bw)
    assert one == dict(stages=[0], t_prefill=[3.0], t_decode=[6.0], c_prefill=[], c_decode=[], c_return=0.0)
