"""Shared driver for the GPU parity tests: feed the same seeded inputs to libshard (through
the C-ABI binding) and to the CPU oracle, and compare with the parity metric."""
from __future__ import annotations

import numpy as np

from oracle import llama_shard as orc
from paper_2405_14371_amd import synth

TOL = {"f32": 1e-3, "bf16": 2e-2}     # max |y - y_ref| / max |y_ref| on hidden states


def torch_mod():
    import torch
    return torch


def make_layers(cfg, seed, n_layers, dtype="f32", gains=False, layer_lo=0):
    layers = synth.shard_weights(cfg, seed, layer_lo, layer_lo + n_layers, dtype)
    if gains:
        for i, lw in enumerate(layers):
            lw.update(synth.random_gains(cfg, seed, layer_lo + i))
    return layers


def gpu_shard(lib, cfg, layers, dtype="f32", layer_lo=0, **kv):
    wd = lib.SHARD_F32 if dtype == "f32" else lib.SHARD_BF16
    return lib.Shard(cfg, lib.pack_layers(layers, wd), layer_lo, weight_dtype=wd, **kv)


def to_dev(a):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def run_gpu(shard, seq_ids, chunks):
    """chunks: list of [B, T, d] float32 arrays; T == 1 chunks after the first go through
    shard_decode, everything else through shard_prefill.  Returns list of outputs."""
    torch = torch_mod()
    outs = []
    for i, x in enumerate(chunks):
        xd = to_dev(x)
        yd = torch.empty_like(xd)
        B, T, _ = x.shape
        st = torch.cuda.current_stream().cuda_stream
        if T == 1 and i > 0:
            shard.decode(seq_ids, xd, yd, st)
        else:
            shard.prefill(seq_ids, T, xd, yd, st)
        torch.cuda.synchronize()
        outs.append(yd.cpu().numpy())
    return outs


def run_oracle(cfg, layers, chunks):
    """Same chunks through the oracle, one sequence at a time."""
    o = orc.OracleShard(cfg, layers)
    outs = []
    for x in chunks:
        outs.append(np.stack([o.forward(b, x[b].astype(np.float64)) for b in range(x.shape[0])]))
    return outs


def assert_parity(got, want, tol, what=""):
    for i, (g, w) in enumerate(zip(got, want)):
        assert np.all(np.isfinite(g)), f"{what} chunk {i}: non-finite output"
        err = orc.max_rel_err(g, w)
        assert err <= tol, f"{what} chunk {i}: max rel err {err:.3e} > {tol:.1e}"
