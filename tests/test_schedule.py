"""Pipeline execution strategies (EdgeShard Sec. 4.2 "Pipeline Execution Optimization",
Fig. 5): pins for the tick-by-tick oracle, then the library's event simulation against it.
CPU only."""
import numpy as np
import pytest

from oracle import schedule as orc


def case(S, seed, zero_comm=False):
    rng = np.random.default_rng(seed)
    tp = [int(v) for v in rng.integers(2, 9, S)]
    td = [int(v) for v in rng.integers(1, 5, S)]
    cp = [0 if zero_comm else int(v) for v in rng.integers(0, 4, max(0, S - 1))]
    cd = [0 if zero_comm else int(v) for v in rng.integers(0, 3, max(0, S - 1))]
    cr = 0 if zero_comm else int(rng.integers(0, 3))
    return tp, td, cp, cd, cr


# ---- the oracle: hand-worked timelines and closed forms -----------------------------------
def test_oracle_hand_worked_two_stages_two_microbatches():
    # stage times: prefill (3, 2), decode (1, 1); no transfer cost; one decode iteration.
    # No-bubbles, by hand:
    #   stage 0: P(m0) 0-3, P(m1) 3-6, G(m0) 6-7 (m0's prefill left stage 1 at 5), G(m1) 8-9
    #   stage 1: P(m0) 3-5, P(m1) 6-8, G(m0) 8-9 (stage 1 busy with P(m1) until 8), G(m1) 9-10
    args = ([3, 2], [1, 1], [0], [0], 0, 2, 1)
    assert orc.simulate_ticks(*args, no_bubbles=True)[0] == 10
    # Bubbles: nobody starts the decode iteration before both prefills are back (t = 8):
    #   stage 0: G(m0) 8-9, G(m1) 9-10;  stage 1: G(m0) 9-10, G(m1) 10-11
    assert orc.simulate_ticks(*args, no_bubbles=False)[0] == 11
    assert orc.bubbles_recurrence(*args) == 11
    # busy time is the same work either way
    assert orc.simulate_ticks(*args, no_bubbles=True)[1] == [3 + 3 + 1 + 1, 2 + 2 + 1 + 1]


def test_oracle_one_stage_has_no_pipeline():
    # a single device: both strategies do MB * (prefill + n * decode) of work back to back
    # (the paper's Cloud-Edge-Opt case that "selects local execution": equal throughput)
    for nb in (True, False):
        span, busy = orc.simulate_ticks([5], [2], [], [], 0, 3, 4, no_bubbles=nb)
        assert span == 3 * (5 + 4 * 2) and busy == [span]


def test_oracle_closed_forms_for_balanced_stages():
    S, MB, n, t = 3, 4, 5, 2
    eq = ([t] * S, [t] * S, [0] * (S - 1), [0] * (S - 1), 0, MB, n)
    # Bubbles: every iteration fills and drains the pipeline: (S + MB - 1) slots of t
    assert orc.simulate_ticks(*eq, no_bubbles=False)[0] == (1 + n) * (S + MB - 1) * t
    assert orc.bubbles_recurrence(*eq) == (1 + n) * (S + MB - 1) * t
    # No-bubbles with MB >= S: stage 0 never idles: (S - 1) * t to reach the last stage,
    # then one task per slot until all MB * (1 + n) are through
    assert orc.simulate_ticks(*eq, no_bubbles=True)[0] == (S - 1) * t + MB * (1 + n) * t


@pytest.mark.parametrize("seed", range(8))
def test_oracle_two_formulations_agree_and_no_bubbles_never_loses(seed):
    S = 1 + seed % 4
    tp, td, cp, cd, cr = case(S, seed)
    for MB, n in ((1, 3), (3, 2), (5, 4)):
        bub = orc.simulate_ticks(tp, td, cp, cd, cr, MB, n, no_bubbles=False)[0]
        assert bub == orc.bubbles_recurrence(tp, td, cp, cd, cr, MB, n)
        nob = orc.simulate_ticks(tp, td, cp, cd, cr, MB, n, no_bubbles=True)[0]
        assert nob <= bub                                     # Sec. 5.3: No-bubbles >= Bubbles in throughput
        # nothing beats the busiest stage's total work, nor one micro-batch's critical path
        work = max(MB * (tp[s] + n * td[s]) for s in range(S))
        path = sum(tp) + sum(cp) + cr + n * (sum(td) + sum(cd) + cr)
        assert nob >= max(work, path)


# ---- the library against the oracle -------------------------------------------------------------
@pytest.mark.parametrize("seed", range(12))
def test_library_matches_the_tick_simulation(lib, seed):
    S = 1 + seed % 5
    tp, td, cp, cd, cr = case(S, 100 + seed, zero_comm=(seed % 3 == 0))
    for MB, n in ((1, 0), (2, 1), (4, 3), (7, 5)):
        for nb in (False, True):
            want, want_busy = orc.simulate_ticks(tp, td, cp, cd, cr, MB, n, no_bubbles=nb)
            got, busy = lib.simulate_pipeline(tp, td, cp, cd, cr, MB, n, nb)
            assert got == pytest.approx(want, abs=1e-9), (S, MB, n, nb)
            assert busy == pytest.approx(want_busy, abs=1e-9)


def test_library_scales_times_and_rejects_bad_arguments(lib):
    tp, td, cp, cd, cr = case(3, 5)
    a, _ = lib.simulate_pipeline(tp, td, cp, cd, cr, 4, 6, True)
    k = 1e-3                                                 # seconds instead of ticks
    b, _ = lib.simulate_pipeline([v * k for v in tp], [v * k for v in td], [v * k for v in cp],
                                 [v * k for v in cd], cr * k, 4, 6, True)
    assert b == pytest.approx(a * k, rel=1e-12)
    with pytest.raises(lib.ShardError):
        lib.simulate_pipeline([1.0, -1.0], [1.0, 1.0], [0.0], [0.0], 0.0, 2, 2, True)
    with pytest.raises(lib.ShardError):
        lib.simulate_pipeline([1.0], [1.0], [], [], 0.0, 0, 2, True)
    assert lib.load().shard_simulate_pipeline(None, 1, None, None) == -1


def test_plan_to_stages_and_the_papers_direction(lib):
    """A throughput plan collapses into stages; on it No-bubbles is at least as fast as
    Bubbles, and a one-device plan shows no difference (Sec. 5.3, Fig. 10 discussion)."""
    rng = np.random.default_rng(3)
    N, M = 8, 3
    tpre = rng.uniform(2.0, 4.0, (N, M)); tdec = rng.uniform(0.1, 0.3, (N, M))
    bw = np.full((M, M), 50.0)
    prob = dict(t_comp=tdec, act_bytes=np.full(N, 1.0), req_bytes=np.ones(N), mem_bytes=np.full(M, 3.5), bandwidth=bw)
    _, dev = lib.plan_throughput(prob)
    st = lib.stages_of_plan(dev, tpre, tdec, np.full(N, 8.0), np.full(N, 1.0), bw)
    assert len(st["stages"]) >= 2 and len(st["c_prefill"]) == len(st["stages"]) - 1
    assert sum(st["t_decode"]) == pytest.approx(sum(tdec[i][d] for i, d in enumerate(dev)))
    args = (st["t_prefill"], st["t_decode"], st["c_prefill"], st["c_decode"], st["c_return"], 4, 16)
    nob, _ = lib.simulate_pipeline(*args, True)
    bub, _ = lib.simulate_pipeline(*args, False)
    assert nob < bub
    solo = lib.stages_of_plan([0] * N, tpre, tdec, np.full(N, 8.0), np.full(N, 1.0), bw)
    a1 = (solo["t_prefill"], solo["t_decode"], solo["c_prefill"], solo["c_decode"], solo["c_return"], 4, 16)
    assert lib.simulate_pipeline(*a1, True)[0] == pytest.approx(lib.simulate_pipeline(*a1, False)[0])
