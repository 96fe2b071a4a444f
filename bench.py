#!/usr/bin/env python3
"""Benchmark of the shard forward pass on one MI355X.

One *step* is one pass of the whole hot path over one batch of synthetic input on the
headline workload: a Llama2-7B-shaped shard, layers 0-7 of 32,
fp32 weights, batch 1, a 512-token prefill followed by 128 decode steps.  Weights and all
inputs are resident in HBM before the timed region.  Prints one JSON line.

  value            decode tokens/s of the shard (tokens generated / time inside shard_decode)
  decode_gbps      algorithmic bytes of a decode step (weights once + KV read/write + the
                   boundary activations) / time, and its fraction of 8 TB/s
  prefill_tflops   algorithmic FLOPs of the prefill (projections + causal half of attention)
                   / time, and its fraction of the fp32 MFMA peak (157.3 TFLOP/s)
  roofline         the dominant kernel (the weight-streaming decode projection) from HIP
                   events attached to each of its dispatches (they read the kernel's own start
                   and end, as a profiler's kernel trace does), in one extra instrumented step
  cpu_baseline     the float64 CPU oracle timed on a bounded sample of the same workload
  also             the other benchmark configurations (7B 32 layers bf16; 13B eight micro-batches;
                   70B batch 16), one timed step each after one warm-up step, same fields
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}

WORKLOADS = {
    # name: model, layers, dtype, batch, prefill tokens, decode steps
    "llama2-7b-l0-7-fp32-b1-p512-d128": dict(model="7b", layers=8, dtype="f32", B=1, T=512, n_dec=128),
    "llama2-7b-32l-bf16-b1-p1024-d256": dict(model="7b", layers=32, dtype="bf16", B=1, T=1024, n_dec=256),
    "llama2-13b-l0-19-bf16-8xb1-p256-d128": dict(model="13b", layers=20, dtype="bf16", B=1, T=256, n_dec=128, micro=8),
    # the same eight sequences as one batch of 8: one pass over the weights serves all of them
    "llama2-13b-l0-19-bf16-b8-fused-p256-d128": dict(model="13b", layers=20, dtype="bf16", B=8, T=256, n_dec=128),
    "llama2-70b-l0-19-bf16-b16-p512-d128": dict(model="70b", layers=20, dtype="bf16", B=16, T=512, n_dec=128),
    # the paper's own request shape (Sec. 5.1: 32 input tokens, 96 generated) on the whole 7B stack
    "llama2-7b-32l-bf16-b1-p32-d96": dict(model="7b", layers=32, dtype="bf16", B=1, T=32, n_dec=96),
    "tiny-2l-fp32-b1-p32-d16": dict(model="tiny", layers=2, dtype="f32", B=1, T=32, n_dec=16),
}
DEFAULT_WORKLOAD = "llama2-7b-l0-7-fp32-b1-p512-d128"


def algorithmic_work(cfg, wl):
    """Bytes a decode step must move and FLOPs a prefill must do (weights once per step,
    the causal half of attention only)."""
    d, hq, hkv, dh, F = (cfg[k] for k in ("d_model", "n_heads", "n_kv_heads", "head_dim", "ffn_dim"))
    L, B, T, n_dec = wl["layers"], wl["B"], wl["T"], wl["n_dec"]
    e = 4 if wl["dtype"] == "f32" else 2
    mat = 2 * d * hq * dh + 2 * d * hkv * dh + 3 * d * F            # matrix elements per layer
    gains = 2 * d
    mean_ctx = T + (n_dec + 1) / 2.0                                 # keys read by an average step
    kv_tok = 2 * hkv * dh * e
    decode_bytes = L * (mat * e + gains * 4) + B * L * kv_tok * (mean_ctx + 1) + 2 * B * d * 4
    prefill_flops = 2.0 * B * T * L * mat + 2.0 * hq * dh * T * (T + 1) * L * B
    linear_bytes = {  # per launch of the streaming projection kernel, by projection
        "qkv": (hq + 2 * hkv) * dh * d * e, "o": d * hq * dh * e, "gateup": 2 * F * d * e, "down": d * F * e,
    }
    gemm_flops = {k: 2.0 * B * T * v / e for k, v in linear_bytes.items()}
    return dict(decode_bytes=decode_bytes, prefill_flops=prefill_flops, linear_bytes=linear_bytes,
                gemm_flops=gemm_flops, weight_bytes=L * (mat * e + gains * 4))


def cpu_baseline(cfg, wl, seed):
    """Time the oracle, as it stands, on a bounded sample of the workload (about 20-30 s of host
    work at the 7B shape): as many of the shard's layers as fit 16 GB of float64 copies (all 8 of
    the default workload, so nothing is extrapolated there), a 64-token prefill and 16 decode
    steps; per-layer times are scaled only if layers had to be left out."""
    from threadpoolctl import threadpool_info
    from oracle import llama_shard as orc
    from paper_2405_14371_amd import synth
    per_layer_f64 = orc.params_per_layer(cfg) * 8
    n_l = max(1, min(wl["layers"], int(16e9 // per_layer_f64)))
    t_pre, n_dec = min(64, wl["T"]), min(16, wl["n_dec"])
    layers = synth.shard_weights(cfg, seed, 0, n_l, wl["dtype"])
    o = orc.OracleShard(cfg, layers, keep_f64=True)
    del layers
    x = synth.hidden_states(cfg, seed, "prefill", 0, 0, 1, t_pre)[0].astype(np.float64)
    t0 = time.perf_counter()
    o.forward(0, x)
    t_prefill = time.perf_counter() - t0
    t0 = time.perf_counter()
    for s in range(n_dec):
        o.forward(0, synth.hidden_states(cfg, seed, "dec", s, 0, 1, 1)[0].astype(np.float64))
    t_dec = (time.perf_counter() - t0) / n_dec
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    scale = wl["layers"] / n_l
    return {
        "value": round(wl["B"] / (t_dec * scale), 4), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": f"{n_l} of {wl['layers']} layers of the workload, {t_pre}-token prefill + {n_dec} decode steps, batch 1"
                  + ("" if n_l == wl["layers"] else f"; per-layer times scaled to {wl['layers']} layers"),
        "prefill_tokens_per_s": round(t_pre / (t_prefill * scale), 3),
    }


ARITHMETIC = {   # what the path computes in (not a precision claim)
    "f32": "f32",
    "bf16": "f16 (bf16 weights converted once to IEEE half; f16 MFMA / FMA inputs, f32 accumulation and residual stream)",
}
# the other benchmark configurations that ride along on the default run, each with fewer steps
ALSO_DEFAULT = ("llama2-7b-32l-bf16-b1-p1024-d256", "llama2-13b-l0-19-bf16-8xb1-p256-d128",
                "llama2-70b-l0-19-bf16-b16-p512-d128")


def prefill_roof(cfg, wl, work):
    """The binding roof of ONE shard_prefill call of the workload: the larger of its MFMA time
    (algorithmic FLOPs at the dtype's peak) and its HBM time (every weight once, the boundary
    activations in and out, the KV cache written once) - a prefill of few rows (config 4's
    256-token micro-batches) is bandwidth-bound."""
    B, T, L = wl["B"], wl["T"], wl["layers"]
    e = 4 if wl["dtype"] == "f32" else 2
    kv_tok = 2 * cfg["n_kv_heads"] * cfg["head_dim"] * e
    t_mfma = work["prefill_flops"] / (MFMA_PEAK_TFLOPS[wl["dtype"]] * 1e12)
    t_hbm = (work["weight_bytes"] + 2 * B * T * cfg["d_model"] * 4 + B * T * L * kv_tok) / (HBM_PEAK_GBPS * 1e9)
    return ("mfma" if t_mfma >= t_hbm else "hbm"), max(t_mfma, t_hbm), t_mfma, t_hbm


def stored_traffic(lib, cfg, wl, workload, wd):
    """HBM bytes per launch of the dominant decode kernel from a stored rocprofv3 PMC summary
    (profiles/pmc_traffic.json), or None with the reason.  The entry names the kernel variants
    it was measured on; it is used only if this run launches exactly those."""
    d, hq, hkv, dh, F = (cfg[k] for k in ("d_model", "n_heads", "n_kv_heads", "head_dim", "ffn_dim"))
    shapes = (((hq + 2 * hkv) * dh, d), (d, hq * dh), (2 * F, d), (d, F))
    now = sorted({lib.variant_decode_linear(cfg, wd, wl["B"], n, k)[0] for n, k in shapes})
    try:
        with open(os.path.join(ROOT, "profiles", "pmc_traffic.json")) as fh:
            entry = json.load(fh)[workload]
    except (OSError, KeyError, ValueError):
        return None, "no stored PMC summary for this workload", now
    if sorted(entry.get("kernel_variants", [])) != now:
        return None, f"stored PMC summary ({entry.get('source')}) is for other kernel variants: stale", now
    return entry["traffic_bytes_per_launch"], f"stored: {entry.get('source')}", now


def measure(lib, torch, synth, workload, steps, warmup, seed, with_cpu_baseline):
    """Build the workload's shard, time `steps` steps after `warmup`, run one instrumented step,
    release everything.  Returns the fields of the JSON line for this workload."""
    wl = WORKLOADS[workload]
    cfg = synth.model_cfg(wl["model"])
    work = algorithmic_work(cfg, wl)
    wd = lib.SHARD_F32 if wl["dtype"] == "f32" else lib.SHARD_BF16
    B, T, n_dec, L = wl["B"], wl["T"], wl["n_dec"], wl["layers"]
    MB = wl.get("micro", 1)     # micro-batches driven round-robin through the shard (each of batch B)

    t0 = time.perf_counter()
    layers = [lib.pack_layers([synth.layer_weights(cfg, seed, li, wl["dtype"])], wd)[0] for li in range(L)]
    sh = lib.Shard(cfg, layers, 0, weight_dtype=wd, max_seqs=B * MB, max_seq_len=T + n_dec,
                   page_size=16, max_batch_tokens=B * T)
    del layers
    x_pre = torch.from_numpy(np.stack([np.concatenate(
        [synth.hidden_states(cfg, seed, "prefill", 0, mb * B + b, 1, T) for b in range(B)])
        for mb in range(MB)])).cuda()                         # [MB, B, T, d]
    x_dec = torch.from_numpy(np.stack([np.stack(
        [np.concatenate([synth.hidden_states(cfg, seed, "dec", s, mb * B + b, 1, 1) for b in range(B)])
         for mb in range(MB)]) for s in range(n_dec)])).cuda()   # [n_dec, MB, B, 1, d]
    y_pre = torch.empty_like(x_pre)
    y_dec = torch.empty_like(x_dec)
    setup_s = time.perf_counter() - t0

    stream = torch.cuda.current_stream()
    st = stream.cuda_stream
    ev = lambda: torch.cuda.Event(enable_timing=True)

    # micro-batches are independent sequences: their calls go round-robin over two streams, so
    # that one micro-batch's kernels fill the ramp and tail of the other's
    side = [torch.cuda.Stream() for _ in range(min(MB, 2))] if MB > 1 else []

    def one_step(timed):
        ids = [[sh.seq_alloc() for _ in range(B)] for _ in range(MB)]
        e0, e1, e2 = ev(), ev(), ev()
        e0.record(stream)
        for q in side:
            q.wait_stream(stream)
        for mb in range(MB):
            q = side[mb % len(side)].cuda_stream if side else st
            sh.prefill(ids[mb], T, x_pre[mb], y_pre[mb], q)
        for q in side:
            stream.wait_stream(q)
        e1.record(stream)
        for q in side:
            q.wait_stream(stream)
        for s in range(n_dec):
            for mb in range(MB):
                q = side[mb % len(side)].cuda_stream if side else st
                sh.decode(ids[mb], x_dec[s, mb], y_dec[s, mb], q)
        for q in side:
            stream.wait_stream(q)
        e2.record(stream)
        torch.cuda.synchronize()
        for group in ids:
            for i in group:
                sh.seq_free(i)
        return (e0.elapsed_time(e1) * 1e-3, e1.elapsed_time(e2) * 1e-3) if timed else None

    for _ in range(warmup):
        one_step(False)
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    times = [one_step(True) for _ in range(steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_wall0
    assert torch.isfinite(y_dec).all() and torch.isfinite(y_pre).all()
    assert not sh.overflow()

    t_pre = sum(t[0] for t in times)
    t_dec = sum(t[1] for t in times)
    dec_tok_s = MB * B * n_dec * steps / t_dec
    dec_gbps = work["decode_bytes"] * MB * n_dec * steps / t_dec / 1e9
    pre_tflops = work["prefill_flops"] * MB * steps / t_pre / 1e12

    # one more step with a HIP event pair on every dispatch, for the per-kernel roofline
    sh.timing_enable(True)
    one_step(False)
    kt = sh.timing_read()
    sh.timing_enable(False)
    proj = ("qkv", "o", "gateup", "down")
    # passes over a projection's weights: one per layer call and group of sequences the decode
    # kernels take at once (fp32: 8 rows; half: 8 rows up to 4 sequences, else 16)
    mfma_decode = wl["dtype"] != "f32" and B > 4
    calls_dec = L * n_dec * MB * (-(-B // 16) if mfma_decode else -(-B // 8))
    calls_pre = L * MB
    lin = {f: sum(kt["decode_" + k][f] for k in proj) for f in ("launches", "seconds")}
    lin_bytes = sum(work["linear_bytes"].values()) * calls_dec
    lin_gbps = lin_bytes / lin["seconds"] / 1e9
    traffic, traffic_note, variants = stored_traffic(lib, cfg, wl, workload, wd)
    n_lin = 4 * calls_dec                   # projection launches (the batched path's one cast of x_in per step not counted)
    roofline = {
        "kernel": ("decode_linear_mfma_kernel / decode_linear_dma_kernel" if mfma_decode else "decode_linear_kernel")
                  + " (weight-streaming projections of shard_decode)",
        "kernel_variants": variants,
        "bound": "hbm", "achieved": round(lin_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(lin_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_note,
        "launches": n_lin, "avg_launch_us": round(lin["seconds"] / n_lin * 1e6, 2),
        "algorithmic_bytes_per_launch": round(lin_bytes / n_lin),
    }
    gm = {f: sum(kt["prefill_" + k][f] for k in proj) for f in ("launches", "seconds")}
    gm_flops = sum(work["gemm_flops"].values()) * L * MB
    peak_tf = MFMA_PEAK_TFLOPS[wl["dtype"]]
    roofline_prefill = {
        "kernel": "gemm_dma_kernel (MFMA projections of shard_prefill)",
        "bound": "mfma", "achieved": round(gm_flops / gm["seconds"] / 1e12, 2), "peak": peak_tf, "unit": "TFLOP/s",
        "frac": round(gm_flops / gm["seconds"] / 1e12 / peak_tf, 4),
        # one projection = one GEMM launch, plus the short reduction launch where K is split
        "launches": 4 * calls_pre, "avg_launch_us": round(gm["seconds"] / (4 * calls_pre) * 1e6, 2),
    }
    kernel_seconds = {k: {"launches": v["launches"], "ms": round(v["seconds"] * 1e3, 3),
                          "avg_us": round(v["seconds"] / max(1, v["launches"]) * 1e6, 2)} for k, v in kt.items()}
    for k in proj:      # per-projection rates of the two engines
        kernel_seconds["decode_" + k]["gbps"] = round(
            work["linear_bytes"][k] * calls_dec / kt["decode_" + k]["seconds"] / 1e9, 1)
        kernel_seconds["prefill_" + k]["tflops"] = round(
            work["gemm_flops"][k] * calls_pre / kt["prefill_" + k]["seconds"] / 1e12, 2)
    sh.close()
    del sh, x_pre, x_dec, y_pre, y_dec
    torch.cuda.empty_cache()

    bound, t_roof, t_mfma, t_hbm = prefill_roof(cfg, wl, work)
    prefill_call_s = t_pre / (steps * MB)        # micro-batches overlap on two streams: the mean share of a call
    out = {
        "metric": "shard_decode_tokens_per_s",
        "value": round(dec_tok_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round((t_pre + t_dec) / steps * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": ARITHMETIC[wl["dtype"]], "data": "synthetic",
        "config": {"workload": workload, "layers": L, "batch": B, "micro_batches": MB, "decode_streams": max(1, len(side)),
                   "prefill_tokens": T,
                   "decode_steps": n_dec, "page_size": 16, "seed": seed, "weights": wl["dtype"]},
        "decode_ms_per_step": round(t_dec / (n_dec * MB * steps) * 1e3, 4),
        "decode_gbps": round(dec_gbps, 1), "decode_hbm_frac": round(dec_gbps / HBM_PEAK_GBPS, 4),
        "prefill_ms": round(t_pre / steps * 1e3, 3),
        "prefill_tokens_per_s": round(MB * B * T * steps / t_pre, 1),
        "prefill_tflops": round(pre_tflops, 2), "prefill_mfma_frac": round(pre_tflops / peak_tf, 4),
        # one prefill call against its binding roof, max(MFMA time, HBM time)
        "prefill_bound": {"bound": bound, "roof_ms_per_call": round(t_roof * 1e3, 4), "mfma_ms": round(t_mfma * 1e3, 4),
                          "hbm_ms": round(t_hbm * 1e3, 4), "measured_ms_per_call": round(prefill_call_s * 1e3, 4),
                          "frac": round(t_roof / prefill_call_s, 4)},
        "roofline": roofline, "roofline_prefill": roofline_prefill, "kernel_ms_instrumented_step": kernel_seconds,
        "wall_s_timed_region": round(wall, 3), "setup_s": round(setup_s, 1),
    }
    if with_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, wl, seed)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(WORKLOADS))
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads measured after the main one with one timed step each and reported in "
                         "the line's `also` array; 'none' for none; default: the other BASELINE configurations when the "
                         "main workload is the default one")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of a benchmark: copy a 1 GiB device tensor three times and exit - the known traffic "
                         "against which the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled")
    args = ap.parse_args()
    if args.calibrate_copy:
        import torch
        a = torch.ones(2 ** 28, device="cuda")          # 1 GiB of float32
        for _ in range(3):
            b = a.clone()                               # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 2 ** 30, "copy_bytes_written": 2 ** 30, "copies": 3, "checksum": float(b[12345])}))
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs one shard on ONE GPU; --gpus > 1 is not supported "
              "(a shard is a single device's share of the pipeline)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2405_14371_amd as pkg
    from paper_2405_14371_amd import synth
    lib = pkg.binding
    lib.load()
    torch.cuda.set_device(0)

    if args.also is None:
        also = ALSO_DEFAULT if args.workload == DEFAULT_WORKLOAD else ()
    else:
        also = tuple(w for w in args.also.split(",") if w and w != "none")
    for w in also:
        if w not in WORKLOADS:
            ap.error(f"unknown workload in --also: {w}")
    out = measure(lib, torch, synth, args.workload, args.steps, args.warmup, args.seed, not args.no_cpu_baseline)
    keep = ("value", "unit", "steps", "warmup", "ms_per_step", "dtype", "config", "decode_ms_per_step", "decode_gbps",
            "decode_hbm_frac", "prefill_ms", "prefill_tokens_per_s", "prefill_tflops", "prefill_mfma_frac", "prefill_bound",
            "roofline", "roofline_prefill", "setup_s")
    if also:
        out["also"] = []
        for w in also:
            r = measure(lib, torch, synth, w, 1, 1, args.seed, False)
            out["also"].append({k: r[k] for k in keep})
    print(json.dumps(out))


if __name__ == "__main__":
    main()
