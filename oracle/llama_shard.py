"""CPU oracle: the forward pass of a shard of Llama2 decoder layers, in float64.

TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP path is compared with; only
the tests, the smoke check and the benchmark's cpu_baseline leg may import it.  It shares
no code with the GPU library and imports nothing from it.

What it follows.  The paper (EdgeShard) treats a model as N layers, assigns a contiguous
range of them - a shard - to each device, pre-allocates a KV cache there, and passes the
range's output activations to the next device (Sec. 3, "Collaborative inference"; Sec. 4,
"System Model").  Inference has a prefill phase that consumes the whole prompt and an
autoregressive phase that consumes one token per iteration while re-using cached keys
and values (Sec. 2, "Generative LLM Inference").  Partitioning must not change the result
(full-precision inference, Sec. 5.1), so the oracle is simply the definition of the
stacked layers written out.  The paper never spells the layer out; it names Llama 2
(Sec. 5.1, "Benchmarks"), whose published decoder layer is, for one sequence:

    h  = rmsnorm(x; g_attn)                     r = 1/sqrt(mean_j x_j^2 + eps), h = x*r*g
    q,k,v = Wq h, Wk h, Wv h                    no biases; W is [out, in]
    q,k <- rope(q,k; position p)                pair (2i, 2i+1) of every head rotated by
                                                angle p * theta^(-2i/dh); v untouched
    cache[p] <- (k, v)
    o_head = softmax_{u<=p}(q_head . k_u / sqrt(dh)) applied to v_u     KV head = head // G
    x1 = x + Wo o
    h2 = rmsnorm(x1; g_ffn)
    y  = x1 + Wd ( silu(Wg h2) * (Wu h2) )      silu(z) = z / (1 + exp(-z))

Readings taken where nothing pins a convention: eps sits inside the square root; RoPE pairs
adjacent elements; the mask removes keys at later positions (no additive constant);
consecutive query heads share a KV head.  All arithmetic is float64; weights arrive as
float32 arrays (exactly representing fp32 or bf16 values) and are widened, never rounded.
Library routine used as a step: numpy's float64 matmul.  No tiling, fusion or paging: the
cache is a plain [position, kv_head, dh] array per layer and sequence.

The ends of a model (embed, logits, greedy) are at the bottom of the file.

The two error metrics (max_rel_err, max_rel_err_strict) are pinned by hand-computed values.

Parity status of this file: every function is pinned by tests/test_oracle_pins.py
(pure-Python brute force on tiny shapes, closed forms, invariants, independent library
routines).  Unpinned: agreement of the RoPE pairing convention with real Llama 2
checkpoints (none are available) - "parity unpinned" for that one convention.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """Rows of x scaled to unit root-mean-square (eps inside the root), then times gain."""
    x = np.asarray(x, F64)
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x * r * np.asarray(gain, F64)


def rope(u: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotate adjacent pairs of u [T, heads, dh]; token t sits at absolute positions[t]."""
    u = np.asarray(u, F64)
    dh = u.shape[-1]
    i = np.arange(dh // 2, dtype=F64)
    inv_freq = np.power(F64(theta), -2.0 * i / dh)                       # theta^(-2i/dh)
    phi = np.asarray(positions, F64)[:, None, None] * inv_freq[None, None, :]
    c, s = np.cos(phi), np.sin(phi)
    a, b = u[..., 0::2], u[..., 1::2]
    out = np.empty_like(u)
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


def silu(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, F64)
    return z / (1.0 + np.exp(-z))


def attention(q: np.ndarray, k_all: np.ndarray, v_all: np.ndarray, q_positions: np.ndarray) -> np.ndarray:
    """Causal softmax attention of T queries over C cached keys/values.

    q [T, Hq, dh]; k_all, v_all [C, Hkv, dh] hold cache positions 0..C-1; query t may see
    cache positions 0..q_positions[t] inclusive.  Returns [T, Hq, dh].
    """
    q, k_all, v_all = (np.asarray(a, F64) for a in (q, k_all, v_all))
    t_len, hq, dh = q.shape
    c_len, hkv, _ = k_all.shape
    group = hq // hkv
    key_pos = np.arange(c_len)
    visible = key_pos[None, :] <= np.asarray(q_positions)[:, None]       # [T, C]
    out = np.empty_like(q)
    for head in range(hq):
        kv = head // group
        s = (q[:, head, :] @ k_all[:, kv, :].T) / np.sqrt(F64(dh))        # [T, C]
        s = np.where(visible, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        w = np.exp(s)
        w = w / w.sum(axis=1, keepdims=True)
        out[:, head, :] = w @ v_all[:, kv, :]
    return out


class OracleShard:
    """Layers [layer_lo, layer_hi) with per-sequence KV caches.

    `layers` is a list (one entry per layer of the range, in order) of dicts holding
    wq, wk, wv, wo, w_gate, w_up, w_down as [out, in] arrays and g_attn, g_ffn as [d].
    With keep_f64 the widened copies stay resident (8 bytes per parameter); otherwise each
    matrix is widened when it is used.
    """

    def __init__(self, cfg: dict, layers: list, keep_f64: bool = False):
        self.cfg = dict(cfg)
        self.d = cfg["d_model"]
        self.hq, self.hkv, self.dh = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
        self.eps, self.theta = float(cfg["rms_eps"]), float(cfg["rope_theta"])
        if self.hq % self.hkv or self.dh % 2:
            raise ValueError("n_heads must be a multiple of n_kv_heads and head_dim even")
        self.layers = [
            {k: (np.asarray(v, F64) if keep_f64 else v) for k, v in lw.items()} for lw in layers
        ]
        self.cache = {}          # seq_id -> list over layers of (k [C,Hkv,dh], v [C,Hkv,dh])

    def n_cached(self, seq_id) -> int:
        c = self.cache.get(seq_id)
        return 0 if c is None else c[0][0].shape[0]

    def free(self, seq_id) -> None:
        self.cache.pop(seq_id, None)

    def forward(self, seq_id, x: np.ndarray) -> np.ndarray:
        """Append the T tokens x [T, d] to sequence seq_id and return the shard output [T, d].

        T > 1 on an empty sequence is prefill, T = 1 afterwards is a decode step; any T at
        any time is legal (the tokens take positions P..P+T-1, P = tokens already cached).
        """
        x = np.asarray(x, F64)
        t_len = x.shape[0]
        if seq_id not in self.cache:
            empty = lambda: np.zeros((0, self.hkv, self.dh), F64)
            self.cache[seq_id] = [(empty(), empty()) for _ in self.layers]
        p0 = self.n_cached(seq_id)
        positions = np.arange(p0, p0 + t_len)
        for li, w in enumerate(self.layers):
            x = self._layer(w, li, seq_id, x, positions)
        return x

    def _layer(self, w, li, seq_id, x, positions):
        t_len = x.shape[0]
        wide = lambda name: np.asarray(w[name], F64)
        h = rmsnorm(x, w["g_attn"], self.eps)
        q = (h @ wide("wq").T).reshape(t_len, self.hq, self.dh)
        k = (h @ wide("wk").T).reshape(t_len, self.hkv, self.dh)
        v = (h @ wide("wv").T).reshape(t_len, self.hkv, self.dh)
        q = rope(q, positions, self.theta)
        k = rope(k, positions, self.theta)
        k_old, v_old = self.cache[seq_id][li]
        k_all = np.concatenate([k_old, k], axis=0)
        v_all = np.concatenate([v_old, v], axis=0)
        self.cache[seq_id][li] = (k_all, v_all)
        o = attention(q, k_all, v_all, positions).reshape(t_len, self.hq * self.dh)
        x1 = x + o @ wide("wo").T
        h2 = rmsnorm(x1, w["g_ffn"], self.eps)
        f = silu(h2 @ wide("w_gate").T) * (h2 @ wide("w_up").T)
        return x1 + f @ wide("w_down").T


# ---- the ends of a model around its decoder layers (the "embedding layer" and "output layer"
# the paper counts among the N layers, Sec. 4 "System Model"; the first is pinned to the
# source node by Eq. 4).  Plain definitions of the Llama 2 ends: a table lookup, and the final
# RMSNorm followed by the output projection; greedy decoding takes the largest logit.
def embed(table: np.ndarray, token_ids) -> np.ndarray:
    """x[i, :] = table[token_ids[i], :] in float64."""
    return np.stack([np.asarray(table[int(t)], dtype=np.float64) for t in token_ids])


def logits(x: np.ndarray, g_final: np.ndarray, lm_head: np.ndarray, eps: float) -> np.ndarray:
    """logits[i, v] = sum_j lm_head[v, j] * rmsnorm(x[i]; g_final)[j], float64."""
    h = rmsnorm(np.asarray(x, dtype=np.float64), np.asarray(g_final, dtype=np.float64), eps)
    return h @ np.asarray(lm_head, dtype=np.float64).T


def greedy(lg: np.ndarray) -> np.ndarray:
    """Index of the largest logit of each row (the lowest index among equals)."""
    return np.array([int(np.argmax(row)) for row in lg], dtype=np.int64)


def params_per_layer(cfg: dict) -> int:
    """Parameter count of one decoder layer: the four attention and three FFN matrices
    plus the two gain vectors."""
    d, hq, hkv, dh, f = (cfg[k] for k in ("d_model", "n_heads", "n_kv_heads", "head_dim", "ffn_dim"))
    return 2 * d * hq * dh + 2 * d * hkv * dh + 3 * d * f + 2 * d


def max_rel_err(y: np.ndarray, y_ref: np.ndarray) -> float:
    """The parity metric: largest absolute deviation over the largest reference magnitude
    of the same tensor.  (Element-wise relative error is meaningless at the zero crossings
    of zero-mean data.)"""
    y, y_ref = np.asarray(y, F64), np.asarray(y_ref, F64)
    return float(np.max(np.abs(y - y_ref)) / np.max(np.abs(y_ref)))


def max_rel_err_strict(y: np.ndarray, y_ref: np.ndarray) -> float:
    """The stricter companion of max_rel_err: every element's deviation over its own
    reference magnitude, but never over less than the root-mean-square of the reference
    tensor (so that elements near a zero crossing are measured against the data's scale,
    not against themselves)."""
    y, y_ref = np.asarray(y, F64), np.asarray(y_ref, F64)
    rms = np.sqrt(np.mean(y_ref * y_ref))
    return float(np.max(np.abs(y - y_ref) / np.maximum(np.abs(y_ref), rms)))
