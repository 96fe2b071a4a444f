"""The benchmark's algorithmic bytes and FLOPs against closed forms typed in by hand.

The achieved-bandwidth and TFLOP/s figures bench.py prints are algorithmic work divided by
measured time, so the work formulas are pinned here, without a GPU: matrix elements per layer
from the Llama 2 layer shapes (the same shapes whose totals reproduce the paper's Table 1 memory
column, see test_oracle_pins), the shard totals of the benchmark configurations, and the
roofline times they imply at 8 TB/s and at the MFMA peaks."""
import pytest

import bench
from paper_2405_14371_amd import synth

# matrix elements of one decoder layer: 2 d Hq dh + 2 d Hkv dh + 3 d F
LAYER_ELEMS = {"7b": 202_375_168, "13b": 317_194_240, "70b": 855_638_016}


@pytest.mark.parametrize("model,d,hq,hkv,F", [("7b", 4096, 32, 32, 11008), ("13b", 5120, 40, 40, 13824),
                                              ("70b", 8192, 64, 8, 28672)])
def test_layer_shapes_give_the_typed_element_counts(model, d, hq, hkv, F):
    cfg = synth.model_cfg(model)
    assert (cfg["d_model"], cfg["n_heads"], cfg["n_kv_heads"], cfg["ffn_dim"], cfg["head_dim"]) == (d, hq, hkv, F, 128)
    assert 2 * d * hq * 128 + 2 * d * hkv * 128 + 3 * d * F == LAYER_ELEMS[model]


def work(name):
    wl = bench.WORKLOADS[name]
    return wl, bench.algorithmic_work(synth.model_cfg(wl["model"]), wl)


def test_headline_workload_is_config_2():
    wl, w = work(bench.DEFAULT_WORKLOAD)
    assert (wl["model"], wl["layers"], wl["dtype"], wl["B"], wl["T"], wl["n_dec"]) == ("7b", 8, "f32", 1, 512, 128)
    # 8 layers x (202,375,168 matrix elements + 2 x 4096 gains) x 4 bytes
    assert w["weight_bytes"] == 8 * (202_375_168 + 8192) * 4 == 6_476_267_520
    # the four projections of one layer, per launch of the streaming kernel
    assert w["linear_bytes"] == {"qkv": 12288 * 4096 * 4, "o": 4096 * 4096 * 4, "gateup": 22016 * 4096 * 4,
                                 "down": 4096 * 11008 * 4}
    assert sum(w["linear_bytes"].values()) == 202_375_168 * 4
    # a decode step at 8 TB/s: weights + mean KV read (about 576 keys x 32 KB per layer and token) = 0.83 ms
    assert w["decode_bytes"] / 8e12 == pytest.approx(0.828e-3, rel=2e-3)
    # prefill: 2 x 512 x 8 x 202,375,168 for the projections + 2 x 32 x 128 x 512 x 513 x 8 for causal attention
    assert w["prefill_flops"] == pytest.approx(2 * 512 * 8 * 202_375_168 + 2 * 32 * 128 * 512 * 513 * 8, rel=1e-12)
    assert w["prefill_flops"] / 157.3e12 == pytest.approx(10.65e-3, rel=2e-3)


@pytest.mark.parametrize("name,weights,flops,decode_ms", [
    ("llama2-7b-32l-bf16-b1-p1024-d256", 12.95e9, 1.354e13, 1.695),
    ("llama2-13b-l0-19-bf16-8xb1-p256-d128", 12.69e9, 3.26e12, 1.602),
    ("llama2-70b-l0-19-bf16-b16-p512-d128", 34.23e9, 2.818e14, 4.373),
])
def test_other_configurations(name, weights, flops, decode_ms):
    wl, w = work(name)
    assert w["weight_bytes"] == pytest.approx(weights, rel=1e-3)
    assert w["prefill_flops"] == pytest.approx(flops, rel=2e-3)
    assert w["decode_bytes"] / 8e12 * 1e3 == pytest.approx(decode_ms, rel=3e-3)


def test_gemm_flops_are_two_per_multiply_add():
    wl, w = work("llama2-70b-l0-19-bf16-b16-p512-d128")
    M = wl["B"] * wl["T"]
    assert w["gemm_flops"]["gateup"] == 2.0 * M * 57344 * 8192
    assert w["gemm_flops"]["qkv"] == 2.0 * M * 10240 * 8192
    assert sum(w["gemm_flops"].values()) == 2.0 * M * LAYER_ELEMS["70b"]
