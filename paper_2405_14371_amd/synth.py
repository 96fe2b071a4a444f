"""Seeded synthetic inputs for a Llama2-shaped shard: model shapes, weights, hidden states.

This module only *draws data*.  It contains none of the decoder layer's arithmetic and
imports nothing from the GPU binding or from the CPU oracle; tests and the benchmark hand
the arrays it returns, unchanged, to both sides.

The paper evaluates on Llama2-7B/13B/70B checkpoints with WikiText-2 prompts (Sec. 5.1,
"Benchmarks").  Neither is available here and a shard's interface is hidden states in,
hidden states out, so the stand-in is: every weight matrix i.i.d. N(0, 0.02^2), norm gains
1.0, hidden states i.i.d. N(0, 1), each tensor drawn from its own stream keyed by
(seed, layer, tensor) or (seed, phase, step, micro-batch) so any tensor can be regenerated
alone.  For bf16 configurations the values are rounded to bf16 once here
(round-to-nearest-even) and kept in float32 containers, so both sides see the same reals.
"""
from __future__ import annotations

import numpy as np

# Per-layer shapes.  7B/13B/70B are the public Llama 2 shapes the paper's Table 1 memory
# figures imply; "tiny" is the small parity configuration.
MODELS = {
    "tiny": dict(d_model=256, n_heads=4, n_kv_heads=4, head_dim=64, ffn_dim=688, n_layers=2),
    "7b": dict(d_model=4096, n_heads=32, n_kv_heads=32, head_dim=128, ffn_dim=11008, n_layers=32),
    "13b": dict(d_model=5120, n_heads=40, n_kv_heads=40, head_dim=128, ffn_dim=13824, n_layers=40),
    "70b": dict(d_model=8192, n_heads=64, n_kv_heads=8, head_dim=128, ffn_dim=28672, n_layers=80),
}
RMS_EPS = 1e-5
ROPE_THETA = 10000.0
WEIGHT_STD = 0.02

# Order is part of the stream key: never reorder.
WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")
GAIN_NAMES = ("g_attn", "g_ffn")
_PHASES = {"prefill": 0, "dec": 1, "aux": 2}


def model_cfg(name: str, **overrides) -> dict:
    """Shape dictionary of a named model plus eps/theta; `overrides` replace entries."""
    cfg = dict(MODELS[name])
    cfg.update(rms_eps=RMS_EPS, rope_theta=ROPE_THETA)
    cfg.update(overrides)
    return cfg


def weight_shapes(cfg: dict) -> dict:
    """[out, in] shape of every projection of one layer."""
    d, hq, hkv, dh, f = (cfg[k] for k in ("d_model", "n_heads", "n_kv_heads", "head_dim", "ffn_dim"))
    return {
        "wq": (hq * dh, d), "wk": (hkv * dh, d), "wv": (hkv * dh, d), "wo": (d, hq * dh),
        "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }


def _stream(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.SFC64(np.random.SeedSequence([int(k) for k in key])))


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    if np.any(u & np.uint32(0xFFFF)):
        raise ValueError("values are not bf16-representable; call round_to_bf16 first")
    return (u >> np.uint32(16)).astype(np.uint16)


def layer_weights(cfg: dict, seed: int, layer: int, dtype: str = "f32") -> dict:
    """All tensors of decoder layer `layer` as float32 arrays (bf16-rounded if dtype='bf16').
    Each matrix has its own stream, so they are drawn concurrently (numpy releases the GIL)."""
    if dtype not in ("f32", "bf16"):
        raise ValueError(dtype)
    from concurrent.futures import ThreadPoolExecutor

    def draw(item):
        idx, (name, shape) = item
        w = _stream(seed, 1, layer, idx).standard_normal(shape, dtype=np.float32)
        w *= np.float32(WEIGHT_STD)
        return name, (round_to_bf16(w) if dtype == "bf16" else w)

    with ThreadPoolExecutor(max_workers=7) as pool:
        out = dict(pool.map(draw, enumerate(weight_shapes(cfg).items())))
    for name in GAIN_NAMES:
        out[name] = np.ones(cfg["d_model"], dtype=np.float32)
    return out


def shard_weights(cfg: dict, seed: int, layer_lo: int, layer_hi: int, dtype: str = "f32") -> list:
    return [layer_weights(cfg, seed, layer, dtype) for layer in range(layer_lo, layer_hi)]


def ends_weights(cfg: dict, seed: int, vocab: int, dtype: str = "f32") -> dict:
    """Token embedding table and LM head [vocab, d_model] (N(0, 0.02^2), bf16-rounded if
    dtype='bf16') and a non-trivial final norm gain, as float32 arrays."""
    if dtype not in ("f32", "bf16"):
        raise ValueError(dtype)
    out = {}
    for idx, name in enumerate(("tok_embeddings", "lm_head")):
        w = _stream(seed, 4, idx).standard_normal((vocab, cfg["d_model"]), dtype=np.float32)
        w *= np.float32(WEIGHT_STD)
        out[name] = round_to_bf16(w) if dtype == "bf16" else w
    g = _stream(seed, 4, 2).standard_normal(cfg["d_model"], dtype=np.float32)
    out["g_final"] = np.float32(1.0) + np.float32(0.1) * g
    return out


def random_gains(cfg: dict, seed: int, layer: int) -> dict:
    """Non-trivial norm gains (1 + 0.1 N(0,1)) for tests that must see the gain multiply."""
    g = _stream(seed, 3, layer).standard_normal((2, cfg["d_model"]), dtype=np.float32)
    g = np.float32(1.0) + np.float32(0.1) * g
    return {"g_attn": g[0].copy(), "g_ffn": g[1].copy()}


def hidden_states(cfg: dict, seed: int, phase: str, step: int, micro_batch: int,
                  batch: int, tokens: int) -> np.ndarray:
    """N(0,1) hidden states [batch, tokens, d_model], float32.

    phase 'prefill' is the prompt's activations; phase 'dec' with step s is the fresh
    hidden state fed to decode step s (a shard has no sampler, so decode inputs are drawn).
    """
    g = _stream(seed, 2, _PHASES[phase], step, micro_batch)
    return g.standard_normal((batch, tokens, cfg["d_model"]), dtype=np.float32)
