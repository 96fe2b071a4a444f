#!/usr/bin/env python3
"""Write the stored expected values for the full-size parity tests.

Calls ONLY the CPU oracle (oracle/llama_shard.py) and the seeded input generator; nothing
here touches the GPU library.  For a workload (model shape, layer range, dtype, prefill
length T, decode steps n_dec, micro-batch index) it runs the oracle over all T + n_dec
tokens of one sequence and stores a sample of the output rows (one per 32-row band of the
prefill, every 8th decode step; float32) in tests/golden/<name>.npz, together with a
checksum of the inputs so that a drift of the input generator is noticed.

Two uses of identities the oracle's pins establish (tests/test_oracle_pins.py):
  * layers are streamed one at a time - shard [0,L) equals [0,1) then [1,2) ... on the
    handed-over activation (shard composition) - so a 70B-shaped range fits in host memory;
  * the n_dec decode inputs are fed as one n_dec-token chunk after the prefill, which
    equals n_dec single-token steps (prefill + decode = longer prefill).

usage: python tests/golden/make_golden.py c2            (a few minutes on 8 cores)
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import llama_shard as orc  # noqa: E402
from paper_2405_14371_amd import synth  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))

# name -> workload.  seqs: which (micro-)batch indices get an oracle run.
WORKLOADS = {
    "c2": dict(model="7b", layers=8, dtype="f32", T=512, n_dec=128, seqs=(0,), seed=0),
    "c3": dict(model="7b", layers=32, dtype="bf16", T=1024, n_dec=256, seqs=(0,), seed=0),
    "c4": dict(model="13b", layers=20, dtype="bf16", T=256, n_dec=128, seqs=(0, 7), seed=0),
    "c5": dict(model="70b", layers=20, dtype="bf16", T=512, n_dec=128, seqs=(0, 15), seed=0),
}


def sample_rows(T: int, n_dec: int):
    """Prefill: one row out of every band of 32 consecutive rows (the finest row tile any
    kernel uses), at an offset that changes from band to band so that over the bands every
    residue modulo 32 is hit, plus the first two and last two rows.  Decode: every 8th step,
    the second and the last."""
    pre = {0, 1, T - 2, T - 1} | {32 * i + (11 * i + 5) % 32 for i in range((T + 31) // 32)}
    dec = {1, n_dec - 1} | set(range(0, n_dec, 8))
    return sorted(pre & set(range(T))), sorted(dec & set(range(n_dec)))


def inputs(cfg, wl, seq):
    xp = synth.hidden_states(cfg, wl["seed"], "prefill", 0, seq, 1, wl["T"])[0]
    xd = np.concatenate([synth.hidden_states(cfg, wl["seed"], "dec", s, seq, 1, 1)[0] for s in range(wl["n_dec"])])
    return xp, xd


def checksum(a: np.ndarray) -> float:
    return float(np.sum(a.astype(np.float64) * np.cos(np.arange(a.size, dtype=np.float64)).reshape(a.shape)))


def main(name: str) -> None:
    wl = WORKLOADS[name]
    cfg = synth.model_cfg(wl["model"])
    pre_rows, dec_rows = sample_rows(wl["T"], wl["n_dec"])
    acts = {}
    sums = {}
    for seq in wl["seqs"]:
        xp, xd = inputs(cfg, wl, seq)
        sums[seq] = checksum(xp) + checksum(xd)
        acts[seq] = [xp.astype(np.float64), xd.astype(np.float64)]
    wsum = 0.0
    t0 = time.time()
    for layer in range(wl["layers"]):
        lw = synth.layer_weights(cfg, wl["seed"], layer, wl["dtype"])
        wsum += checksum(lw["wq"][:8]) + checksum(lw["w_down"][-8:])
        one = orc.OracleShard(cfg, [lw], keep_f64=True)
        for seq in wl["seqs"]:
            acts[seq] = [one.forward(seq, acts[seq][0]), one.forward(seq, acts[seq][1])]
        print(f"{name}: layer {layer + 1}/{wl['layers']} done, {time.time() - t0:.0f} s", flush=True)
    out = {"pre_rows": np.array(pre_rows), "dec_rows": np.array(dec_rows), "seqs": np.array(wl["seqs"]),
           "input_checksum": np.array([sums[s] for s in wl["seqs"]]), "weight_checksum": np.array(wsum)}
    for seq in wl["seqs"]:
        # float32 storage: its rounding (6e-8 relative) is far below both tolerances
        out[f"prefill_{seq}"] = acts[seq][0][pre_rows].astype(np.float32)
        out[f"decode_{seq}"] = acts[seq][1][dec_rows].astype(np.float32)
        # denominators of the two parity metrics, taken over the call's whole output tensor
        out[f"prefill_absmax_{seq}"] = np.array(np.abs(acts[seq][0]).max())
        out[f"decode_absmax_{seq}"] = np.abs(acts[seq][1]).max(axis=1)[dec_rows]
        out[f"prefill_rms_{seq}"] = np.array(np.sqrt(np.mean(acts[seq][0] ** 2)))
        out[f"decode_rms_{seq}"] = np.sqrt(np.mean(acts[seq][1] ** 2, axis=1))[dec_rows]
    np.savez(os.path.join(HERE, f"{name}.npz"), **out)
    print(f"wrote tests/golden/{name}.npz")


if __name__ == "__main__":
    for n in sys.argv[1:] or ["c2"]:
        main(n)
