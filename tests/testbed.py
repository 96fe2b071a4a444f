"""A planner problem shaped like the paper's testbed (Sec. 5.1 "Testbed", Table 3), built from
one measured (or stand-in) per-layer profile.  Test input construction only: none of the
planner's or the schedule's arithmetic lives here.

Devices: 12 Jetson AGX Orin (32 GB, 3.33 TFLOPS), 2 Jetson Orin NX (16 GB, 1.88 TFLOPS), one
RTX 3090 cloud server (24 GB, 36 TFLOPS); device 0, the source node, is an AGX Orin.  Links:
50 Mbps with a seeded spread of +-20 %, source <-> cloud 1 Mbps unless stated (Sec. 5.2).
A layer's time on a device is the profiled time scaled by the devices' TFLOPS ratio, with the
scale fixed so that the whole model on one AGX Orin takes the Edge-Solo latency the paper
reports for Llama2-7B (140.34 ms per token, Table 4) times the model's parameter ratio.
The N layers are the embedding, the decoder layers and the output layer (Sec. 4 "System
Model"); requests are 32 prompt tokens and 96 generated ones (Sec. 5.1 "Benchmarks").
"""
from __future__ import annotations

import numpy as np

TFLOPS = [3.33] * 12 + [1.88] * 2 + [36.0]
MEM_GB = [32.0] * 12 + [16.0] * 2 + [24.0]
CLOUD = 14
EDGE_SOLO_7B_S = 0.14034          # Table 4, Llama2-7B, Edge-Solo latency per token
VOCAB = 32000
PROMPT, GENERATED = 32, 96


def build(profile: dict, d_model: int, n_decoder_layers: int, params_ratio_to_7b: float, batch: int = 1,
          source_cloud_mbps: float = 1.0, seed: int = 0, devices=None) -> dict:
    """profile: one decoder layer's t_prefill_s, t_decode_s, weight_bytes, kv_bytes_per_token
    (what shard_profile returns for a layer).  Returns the planner problem for decode steps
    (t_comp = decode time, the paper's per-token latency) plus the prefill columns and the
    activation sizes of both phases, restricted to `devices` (default: all 15)."""
    devices = list(range(15)) if devices is None else list(devices)
    N = n_decoder_layers + 2
    # relative cost of the three layer kinds on one device: embedding ~ a lookup, output layer ~
    # vocab x d against a decoder layer's parameter count
    dec_params = profile["weight_bytes"]
    rel = np.array([1e-3] + [1.0] * n_decoder_layers + [VOCAB * d_model * 4.0 / dec_params])
    solo = EDGE_SOLO_7B_S * params_ratio_to_7b
    t_dec_agx = rel / rel.sum() * solo
    t_pre_agx = t_dec_agx * (profile["t_prefill_s"] / profile["t_decode_s"])
    speed = np.array([TFLOPS[j] / TFLOPS[0] for j in devices])
    t_dec = t_dec_agx[:, None] / speed[None, :]
    t_pre = t_pre_agx[:, None] / speed[None, :]
    act_dec = np.full(N, batch * d_model * 4.0)
    act_pre = np.full(N, batch * PROMPT * d_model * 4.0)
    ends = VOCAB * d_model * 4.0
    req = np.array([ends] + [profile["weight_bytes"] + profile["kv_bytes_per_token"] * (PROMPT + GENERATED) * batch]
                   * n_decoder_layers + [ends])
    mem = np.array([MEM_GB[j] * 1e9 for j in devices])
    rng = np.random.default_rng(seed)
    mbps = 50.0 * rng.uniform(0.8, 1.2, (15, 15))
    mbps = (mbps + mbps.T) / 2
    mbps[0, CLOUD] = mbps[CLOUD, 0] = source_cloud_mbps
    bw = mbps[np.ix_(devices, devices)] * 1e6 / 8.0
    return dict(t_comp=t_dec, t_prefill=t_pre, act_bytes=act_dec, act_prefill=act_pre, req_bytes=req, mem_bytes=mem,
                bandwidth=bw, n_layers=N)


def planner_view(tb: dict) -> dict:
    return {k: tb[k] for k in ("t_comp", "act_bytes", "req_bytes", "mem_bytes", "bandwidth")}


# A stand-in profile for CPU tests: one fp32 7B-shaped decoder layer as an MI355X times it
# (order of magnitude; only the ratio prefill / decode enters the table).
STAND_IN_7B = dict(t_prefill_s=2.6e-4, t_decode_s=1.4e-4, weight_bytes=202_383_360 * 4, kv_bytes_per_token=2 * 32 * 128 * 4)


def check_chain(lib, profile: dict) -> dict:
    """profile -> testbed tables -> both dynamic programs -> stages -> both schedules, with the
    relations the paper reports.  Returns a few figures for the caller to print."""
    import pytest

    def latency(tb):
        return lib.plan_latency(planner_view(tb))

    # ---- Llama2-7B-sized model: 34 layers -------------------------------------------------
    kw = dict(d_model=4096, n_decoder_layers=32, params_ratio_to_7b=1.0)
    full = build(profile, **kw)
    solo_tb = build(profile, devices=[0], **kw)
    two_tb = build(profile, devices=[0, CLOUD], **kw)
    t_solo, dev_solo = latency(solo_tb)
    assert dev_solo == [0] * 34 and t_solo == pytest.approx(EDGE_SOLO_7B_S, rel=1e-9)      # Edge-Solo is reachable
    t_two, dev_two = latency(two_tb)
    assert dev_two == [0] * 34 and t_two == pytest.approx(t_solo)                          # 1 Mbps: all local (Sec. 5.2)
    t_full, dev_full = latency(full)
    assert t_full <= t_two * (1 + 1e-12)                                                   # EdgeShard <= Cloud-Edge-Opt
    assert t_full < t_solo and len(set(dev_full)) >= 2                                     # and it does use the edge network
    used = np.zeros(15)
    for i, j in enumerate(dev_full):
        used[j] += full["req_bytes"][i]
    assert np.all(used <= full["mem_bytes"]) and dev_full[0] == 0                           # Eq. 5, Eq. 4
    # more source <-> cloud bandwidth never hurts, and from 10 Mbps on the cloud pays off (Sec. 5.3)
    prev = t_two
    for mbps in (10.0, 50.0):
        t, dev = latency(build(profile, devices=[0, CLOUD], source_cloud_mbps=mbps, **kw))
        assert t <= prev * (1 + 1e-12)
        prev = t
    assert prev < t_solo and 1 in dev
    # ---- throughput plan over the 15 devices, collapsed to stages, both schedules ---------
    batch = 8
    tput = build(profile, batch=batch, **kw)
    t_stage, dev_t = lib.plan_throughput(planner_view(tput))
    t_stage_two, dev_t2 = lib.plan_throughput(planner_view(build(profile, batch=batch, devices=[0, CLOUD], **kw)))
    assert t_stage <= t_stage_two * (1 + 1e-12)
    st = lib.stages_of_plan(dev_t, tput["t_prefill"], tput["t_comp"], tput["act_prefill"], tput["act_bytes"], tput["bandwidth"])
    assert len(st["stages"]) >= 2 and st["stages"][0] == 0
    slowest = max(max(t, c) for t, c in zip(st["t_decode"], [0.0] + st["c_decode"]))
    assert slowest == pytest.approx(t_stage, rel=1e-9)                                     # Eq. 9-10 read off the stages
    args = (st["t_prefill"], st["t_decode"], st["c_prefill"], st["c_decode"], st["c_return"], 4, GENERATED)
    nob, busy = lib.simulate_pipeline(*args, True)
    bub, _ = lib.simulate_pipeline(*args, False)
    assert nob <= bub * (1 + 1e-12) and nob < bub                                          # No-bubbles >= Bubbles (Sec. 5.3)
    assert busy == pytest.approx([4 * (tp + GENERATED * td) for tp, td in zip(st["t_prefill"], st["t_decode"])])
    one = lib.stages_of_plan(dev_t2, *[build(profile, batch=batch, devices=[0, CLOUD], **kw)[k] for k in
                                       ("t_prefill", "t_comp", "act_prefill", "act_bytes", "bandwidth")])
    if len(one["stages"]) == 1:                                                            # local execution: no pipeline
        a1 = (one["t_prefill"], one["t_decode"], one["c_prefill"], one["c_decode"], one["c_return"], 4, GENERATED)
        assert lib.simulate_pipeline(*a1, True)[0] == pytest.approx(lib.simulate_pipeline(*a1, False)[0])
    # ---- Llama2-70B-sized model: 82 layers, no single device and no edge-cloud pair holds it --
    kw70 = dict(d_model=8192, n_decoder_layers=80, params_ratio_to_7b=855_654_400 / 202_383_360)
    prof70 = dict(profile, weight_bytes=855_654_400 * 4, kv_bytes_per_token=2 * 8 * 128 * 4)
    for devs in ([0], [0, CLOUD]):
        with pytest.raises(lib.ShardError) as e:
            latency(build(prof70, devices=devs, **kw70))
        assert e.value.code == -2                                                          # OOM rows of Table 4
    big = build(prof70, **kw70)
    t70, dev70 = latency(big)
    used = np.zeros(15)
    for i, j in enumerate(dev70):
        used[j] += big["req_bytes"][i]
    assert np.all(used <= big["mem_bytes"]) and dev70[0] == 0 and len(dev70) == 82
    t70_stage, dev70_t = lib.plan_throughput(planner_view(big))
    st70 = lib.stages_of_plan(dev70_t, big["t_prefill"], big["t_comp"], big["act_prefill"], big["act_bytes"], big["bandwidth"])
    assert len(st70["stages"]) >= 9                                                        # 276 GB over devices of at most 32 GB
    a70 = (st70["t_prefill"], st70["t_decode"], st70["c_prefill"], st70["c_decode"], st70["c_return"], 4, 16)
    assert lib.simulate_pipeline(*a70, True)[0] < lib.simulate_pipeline(*a70, False)[0]
    return dict(t_solo=t_solo, t_edgeshard=t_full, devices_7b=sorted(set(dev_full)), stages_7b=st["stages"],
                no_bubbles_s=nob, bubbles_s=bub, t70=t70, stages_70b=len(st70["stages"]))
