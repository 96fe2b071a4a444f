"""Pins for the CPU oracle (oracle/llama_shard.py): things the mathematics fixes, checked
without any GPU.  Each pin is chosen so that a plausible slip in the oracle (dropped term,
wrong sign or index, transposed operand, off-by-one mask) breaks at least one of them; the
last test plants such slips and checks that the pins notice."""
import math
import os

import numpy as np
import pytest

from oracle import llama_shard as orc
from paper_2405_14371_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_cfg(d=16, hq=4, hkv=2, dh=4, f=12, eps=1e-5, theta=10000.0):
    return dict(d_model=d, n_heads=hq, n_kv_heads=hkv, head_dim=dh, ffn_dim=f,
                rms_eps=eps, rope_theta=theta, n_layers=2)


def rand_layers(cfg, seed, n, std=0.3, gains=True):
    layers = []
    for li in range(n):
        rng = np.random.default_rng([seed, li])
        lw = {k: rng.normal(0, std, s) for k, s in synth.weight_shapes(cfg).items()}
        for g in synth.GAIN_NAMES:
            lw[g] = 1.0 + 0.2 * rng.normal(size=cfg["d_model"]) if gains else np.ones(cfg["d_model"])
        layers.append(lw)
    return layers


# --------------------------------------------------------------------------------------
# Brute force: the whole layer stack with scalar Python loops, written token by token and
# head by head from the layer's definition, with its own list-based cache.
# --------------------------------------------------------------------------------------
def brute_shard(cfg, layers, chunks):
    d, hq, hkv, dh, f = (cfg[k] for k in ("d_model", "n_heads", "n_kv_heads", "head_dim", "ffn_dim"))
    eps, theta = cfg["rms_eps"], cfg["rope_theta"]
    group = hq // hkv
    kcache = [[] for _ in layers]      # per layer: list over positions of [hkv][dh]
    vcache = [[] for _ in layers]

    def matvec(w, x):                  # w [out][in]
        return [sum(w[o][i] * x[i] for i in range(len(x))) for o in range(len(w))]

    def norm(x, g):
        ms = sum(v * v for v in x) / len(x)
        return [x[j] / math.sqrt(ms + eps) * g[j] for j in range(len(x))]

    def rot(vec, heads, pos):
        out = list(vec)
        for h in range(heads):
            for i in range(dh // 2):
                ang = pos * theta ** (-2.0 * i / dh)
                a, b = vec[h * dh + 2 * i], vec[h * dh + 2 * i + 1]
                out[h * dh + 2 * i] = a * math.cos(ang) - b * math.sin(ang)
                out[h * dh + 2 * i + 1] = a * math.sin(ang) + b * math.cos(ang)
        return out

    outputs = []
    pos = 0
    for chunk in chunks:
        for x in chunk:
            x = [float(v) for v in x]
            for li, w in enumerate(layers):
                W = {k: np.asarray(v).tolist() for k, v in w.items()}
                h = norm(x, W["g_attn"])
                q = rot(matvec(W["wq"], h), hq, pos)
                k = rot(matvec(W["wk"], h), hkv, pos)
                v = matvec(W["wv"], h)
                kcache[li].append(k)
                vcache[li].append(v)
                o = [0.0] * (hq * dh)
                for head in range(hq):
                    kv = head // group
                    scores = []
                    for u in range(pos + 1):
                        dot = sum(q[head * dh + e] * kcache[li][u][kv * dh + e] for e in range(dh))
                        scores.append(dot / math.sqrt(dh))
                    m = max(scores)
                    ex = [math.exp(s - m) for s in scores]
                    z = sum(ex)
                    for e in range(dh):
                        o[head * dh + e] = sum(ex[u] / z * vcache[li][u][kv * dh + e] for u in range(pos + 1))
                att = matvec(W["wo"], o)
                x1 = [x[j] + att[j] for j in range(d)]
                h2 = norm(x1, W["g_ffn"])
                gate, up = matvec(W["w_gate"], h2), matvec(W["w_up"], h2)
                ff = [gate[j] / (1.0 + math.exp(-gate[j])) * up[j] for j in range(f)]
                down = matvec(W["w_down"], ff)
                x = [x1[j] + down[j] for j in range(d)]
            outputs.append(x)
            pos += 1
    return np.array(outputs)


def run_oracle(cfg, layers, chunks, module=orc):
    sh = module.OracleShard(cfg, layers)
    return np.concatenate([sh.forward(0, np.asarray(c)) for c in chunks], axis=0)


BRUTE_CASES = [
    dict(cfg=small_cfg(), chunks=(5,)),                      # GQA 4/2, one prefill
    dict(cfg=small_cfg(hq=2, hkv=2, d=8, dh=4, f=6), chunks=(3, 1, 1)),   # MHA, prefill + 2 decodes
    dict(cfg=small_cfg(hq=4, hkv=1, dh=6, d=10, f=7), chunks=(2, 3, 1)),  # MQA, d != hq*dh, chunked
]


@pytest.mark.parametrize("case", BRUTE_CASES)
def test_whole_shard_matches_scalar_brute_force(case):
    cfg = case["cfg"]
    layers = rand_layers(cfg, 11, 2)
    rng = np.random.default_rng(5)
    chunks = [rng.normal(size=(t, cfg["d_model"])) for t in case["chunks"]]
    got = run_oracle(cfg, layers, chunks)
    want = brute_shard(cfg, layers, chunks)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-12)


def test_attention_matches_explicit_score_matrix():
    """T x C score matrix, explicit mask, naive softmax - no streaming, no max-subtraction."""
    rng = np.random.default_rng(0)
    t_len, c_len, hq, hkv, dh = 4, 7, 4, 2, 8
    q = rng.normal(size=(t_len, hq, dh))
    k = rng.normal(size=(c_len, hkv, dh))
    v = rng.normal(size=(c_len, hkv, dh))
    qpos = np.arange(c_len - t_len, c_len)
    got = orc.attention(q, k, v, qpos)
    for t in range(t_len):
        for h in range(hq):
            kv = h // (hq // hkv)
            e = [math.exp(float(q[t, h] @ k[u, kv]) / math.sqrt(dh)) if u <= qpos[t] else 0.0
                 for u in range(c_len)]
            want = sum(e[u] * v[u, kv] for u in range(c_len)) / sum(e)
            np.testing.assert_allclose(got[t, h], want, rtol=1e-12)


def test_attention_special_cases():
    rng = np.random.default_rng(1)
    v = rng.normal(size=(5, 1, 4))
    # one visible key: output is that key's value, whatever the scores are
    out = orc.attention(rng.normal(size=(1, 2, 4)), rng.normal(size=(5, 1, 4)), v, np.array([0]))
    np.testing.assert_allclose(out[0, 0], v[0, 0], rtol=1e-14)
    # all scores equal (q = 0): output is the mean of the visible values
    out = orc.attention(np.zeros((1, 2, 4)), rng.normal(size=(5, 1, 4)), v, np.array([3]))
    np.testing.assert_allclose(out[0, 1], v[:4, 0].mean(axis=0), rtol=1e-14)
    # a key far above the rest takes all the weight (softmax, not a linear average)
    k = np.zeros((3, 1, 4)); k[1, 0, 0] = 1000.0
    q = np.zeros((1, 1, 4)); q[0, 0, 0] = 1.0
    out = orc.attention(q, k, v[:3], np.array([2]))
    np.testing.assert_allclose(out[0, 0], v[1, 0], rtol=1e-12)


def test_attention_against_library_sdpa():
    """Independent routine: torch's float64 scaled_dot_product_attention (causal)."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    t_len, hq, dh = 9, 3, 16
    q, k, v = (rng.normal(size=(t_len, hq, dh)) for _ in range(3))
    got = orc.attention(q, k, v, np.arange(t_len))
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-10, atol=1e-12)


# --------------------------------------------------------------------------------------
# RoPE
# --------------------------------------------------------------------------------------
def test_rope_closed_forms():
    # dh = 2: the only pair turns by exactly `position` radians (theta^0 = 1).
    u = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    out = orc.rope(u, np.array([0.5, 2.0]), 10000.0)
    np.testing.assert_allclose(out[0, 0], [math.cos(0.5), math.sin(0.5)], rtol=1e-15)
    np.testing.assert_allclose(out[1, 0], [-math.sin(2.0), math.cos(2.0)], rtol=1e-15)
    # dh = 4, theta = 10000: pair 1 turns by position/100; pair 0 by position.
    u = np.array([[[1.0, 0.0, 1.0, 0.0]]])
    out = orc.rope(u, np.array([50.0 * math.pi]), 10000.0)        # pair 1: quarter turn
    np.testing.assert_allclose(out[0, 0, 2:], [0.0, 1.0], atol=1e-12)
    np.testing.assert_allclose(out[0, 0, :2], [1.0, 0.0], atol=1e-12)   # 25 full turns
    # dh = 8, theta = 16: angles position * 16^(-i/4) = position / 2^i
    u = np.zeros((1, 1, 8)); u[0, 0, 0::2] = 1.0
    out = orc.rope(u, np.array([3.0]), 16.0)
    for i in range(4):
        np.testing.assert_allclose(out[0, 0, 2 * i:2 * i + 2],
                                   [math.cos(3.0 / 2 ** i), math.sin(3.0 / 2 ** i)], rtol=1e-14)


def test_rope_invariants():
    rng = np.random.default_rng(3)
    u = rng.normal(size=(6, 3, 8))
    pos = np.array([0, 1, 5, 17, 300, 1279])
    out = orc.rope(u, pos, 10000.0)
    np.testing.assert_array_equal(out[0], u[0])                                     # p = 0: identity
    pair_norm = lambda a: a[..., 0::2] ** 2 + a[..., 1::2] ** 2
    np.testing.assert_allclose(pair_norm(out), pair_norm(u), rtol=1e-13)            # norm per pair
    # relative-position property: <R_m q, R_n k> = <R_{m-n} q, k>
    q, k = rng.normal(size=(1, 1, 8)), rng.normal(size=(1, 1, 8))
    for m, n in ((7, 3), (100, 99), (5, 5)):
        lhs = np.sum(orc.rope(q, [m], 10000.0) * orc.rope(k, [n], 10000.0))
        rhs = np.sum(orc.rope(q, [m - n], 10000.0) * k)
        assert abs(lhs - rhs) < 1e-12
    # composition: turning by m then n equals turning by m + n; inverse is the negative
    np.testing.assert_allclose(orc.rope(orc.rope(q, [4], 100.0), [9], 100.0),
                               orc.rope(q, [13], 100.0), rtol=1e-12)


# --------------------------------------------------------------------------------------
# RMSNorm, SiLU
# --------------------------------------------------------------------------------------
def test_rmsnorm_closed_forms():
    eps = 1e-5
    x = np.full((1, 8), 3.0)
    g = np.arange(1.0, 9.0)
    np.testing.assert_allclose(orc.rmsnorm(x, g, eps)[0], 3.0 / math.sqrt(9.0 + eps) * g, rtol=1e-15)
    # eps inside the root: with x = 0 the output is 0 (not NaN); with tiny x, eps dominates
    assert np.all(orc.rmsnorm(np.zeros((1, 4)), np.ones(4), eps) == 0.0)
    tiny = np.full((1, 4), 1e-10)
    np.testing.assert_allclose(orc.rmsnorm(tiny, np.ones(4), 1e-2)[0], 1e-10 / math.sqrt(1e-20 + 1e-2), rtol=1e-14)
    # x = (3, 4): mean square 12.5
    np.testing.assert_allclose(orc.rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0)[0],
                               [3 / math.sqrt(12.5), 8 / math.sqrt(12.5)], rtol=1e-15)


def test_rmsnorm_invariants_and_library():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(4)
    x = rng.normal(size=(5, 64)) * 3.0
    eps = 1e-5
    out = orc.rmsnorm(x, np.ones(64), eps)
    rms = np.sqrt(np.mean(out * out, axis=1))
    np.testing.assert_allclose(rms, 1.0 / np.sqrt(1.0 + eps / np.mean(x * x, axis=1)), rtol=1e-13)
    np.testing.assert_allclose(orc.rmsnorm(7.0 * x, np.ones(64), 0.0), orc.rmsnorm(x, np.ones(64), 0.0), rtol=1e-13)
    g = rng.normal(size=64)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps)
    np.testing.assert_allclose(orc.rmsnorm(x, g, eps), want.numpy(), rtol=1e-12)


def test_silu():
    torch = pytest.importorskip("torch")
    assert orc.silu(np.array([0.0]))[0] == 0.0
    z = np.linspace(-20, 20, 41)
    np.testing.assert_allclose(orc.silu(z) - orc.silu(-z), z, atol=1e-12)     # z*(s(z) + s(-z)) = z
    np.testing.assert_allclose(orc.silu(np.array([50.0])), [50.0], rtol=1e-15)
    np.testing.assert_allclose(orc.silu(np.array([1.0])), [1.0 / (1.0 + math.exp(-1.0))], rtol=1e-15)
    np.testing.assert_allclose(orc.silu(z), torch.nn.functional.silu(torch.from_numpy(z)).numpy(), rtol=1e-13)


# --------------------------------------------------------------------------------------
# Cache semantics, composition, GQA, degenerate layers, causality, batch independence
# --------------------------------------------------------------------------------------
def test_prefill_then_decode_equals_longer_prefill():
    cfg = small_cfg(d=32, hq=4, hkv=2, dh=8, f=40)
    layers = rand_layers(cfg, 21, 3)
    x = np.random.default_rng(6).normal(size=(12, 32))
    full = run_oracle(cfg, layers, [x])
    for split in ([8, 1, 1, 1, 1], [5, 7], [1] * 12):
        chunks, s = [], 0
        for t in split:
            chunks.append(x[s:s + t]); s += t
        np.testing.assert_allclose(run_oracle(cfg, layers, chunks), full, rtol=1e-11, atol=1e-12)


def test_shard_composition():
    """Layers [0,k) then [k,L) on the hand-off activation equals [0,L) (Sec. 3: a device's
    output activations are the next device's input)."""
    cfg = small_cfg(d=32, hq=4, hkv=4, dh=8, f=24)
    layers = rand_layers(cfg, 22, 4)
    rng = np.random.default_rng(7)
    chunks = [rng.normal(size=(6, 32)), rng.normal(size=(1, 32)), rng.normal(size=(1, 32))]
    whole = orc.OracleShard(cfg, layers)
    for k in (1, 2, 3):
        a, b = orc.OracleShard(cfg, layers[:k]), orc.OracleShard(cfg, layers[k:])
        w2 = orc.OracleShard(cfg, layers)
        for c in chunks:
            np.testing.assert_array_equal(b.forward(0, a.forward(0, c)), w2.forward(0, c))
    assert whole.n_cached(0) == 0


def test_gqa_equals_mha_with_repeated_kv_heads():
    cfg = small_cfg(d=24, hq=6, hkv=2, dh=4, f=16)
    layers = rand_layers(cfg, 23, 2)
    mha_cfg = dict(cfg, n_kv_heads=6)
    mha_layers = []
    for lw in layers:
        m = dict(lw)
        for name in ("wk", "wv"):
            blocks = lw[name].reshape(2, 4, 24)                      # [kv head, dh, d]
            m[name] = np.repeat(blocks, 3, axis=0).reshape(6 * 4, 24)   # heads 0,0,0,1,1,1
        mha_layers.append(m)
    x = np.random.default_rng(8).normal(size=(7, 24))
    np.testing.assert_allclose(run_oracle(cfg, layers, [x]), run_oracle(mha_cfg, mha_layers, [x]),
                               rtol=1e-12, atol=1e-13)


def test_degenerate_layers():
    cfg = small_cfg(d=16, hq=2, hkv=2, dh=8, f=10)
    layers = rand_layers(cfg, 24, 2)
    x = np.random.default_rng(9).normal(size=(4, 16))
    for lw in layers:
        lw["wo"] = np.zeros_like(lw["wo"]); lw["w_down"] = np.zeros_like(lw["w_down"])
    np.testing.assert_array_equal(run_oracle(cfg, layers, [x]), x)       # both branches off: identity
    # FFN off, single token: attention output is v itself, so y = x + Wo Wv rmsnorm(x)
    one = rand_layers(cfg, 25, 1)
    one[0]["w_down"] = np.zeros_like(one[0]["w_down"])
    h = x[:1] / np.sqrt(np.mean(x[:1] ** 2) + cfg["rms_eps"]) * one[0]["g_attn"]
    want = x[:1] + (h @ one[0]["wv"].T) @ one[0]["wo"].T
    np.testing.assert_allclose(run_oracle(cfg, one, [x[:1]]), want, rtol=1e-12)


def test_causality_and_batch_independence():
    cfg = small_cfg(d=16, hq=4, hkv=2, dh=4, f=12)
    layers = rand_layers(cfg, 26, 2)
    rng = np.random.default_rng(10)
    x = rng.normal(size=(8, 16))
    base = run_oracle(cfg, layers, [x])
    x2 = x.copy(); x2[5] += 1.0
    pert = run_oracle(cfg, layers, [x2])
    np.testing.assert_array_equal(pert[:5], base[:5])
    assert np.all(np.abs(pert[5:] - base[5:]).max(axis=1) > 1e-6)
    # two sequences interleaved in one shard do not see each other
    sh = orc.OracleShard(cfg, layers)
    other = rng.normal(size=(3, 16))
    a0 = sh.forward("a", x[:4]); sh.forward("b", other); a1 = sh.forward("a", x[4:])
    np.testing.assert_array_equal(np.concatenate([a0, a1]), run_oracle(cfg, layers, [x[:4], x[4:]]))


# --------------------------------------------------------------------------------------
# Shapes against the paper's printed memory figures (Table 1)
# --------------------------------------------------------------------------------------
def test_layer_shapes_reproduce_table1_memory():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table1_memory.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    vocab = 32000            # public Llama 2 vocabulary: embedding + output matrices
    for name, n_layers, printed_gb in rows:
        cfg = synth.model_cfg(name)
        assert cfg["n_layers"] == int(n_layers)
        shapes = synth.weight_shapes(cfg)
        assert orc.params_per_layer(cfg) == sum(a * b for a, b in shapes.values()) + 2 * cfg["d_model"]
        total = orc.params_per_layer(cfg) * cfg["n_layers"] + 2 * vocab * cfg["d_model"] + cfg["d_model"]
        gb = total * 4 / 1e9
        assert abs(gb - float(printed_gb)) / float(printed_gb) < 0.04, (name, gb)
    assert orc.params_per_layer(synth.model_cfg("7b")) == 202_383_360
    assert orc.params_per_layer(synth.model_cfg("13b")) == 317_204_480
    assert orc.params_per_layer(synth.model_cfg("70b")) == 855_654_400


def test_max_rel_err_metric():
    ref = np.array([1.0, -4.0, 0.0])
    assert orc.max_rel_err(ref, ref) == 0.0
    assert orc.max_rel_err(np.array([1.0, -4.0, 0.2]), ref) == pytest.approx(0.05)


def test_strict_rel_err_metric_hand_values():
    """ref = (3, -4, 0, 1): rms = sqrt(26/4) = 2.5495...  Deviations (0.3, 0, 0.5, 0.2) are
    measured against max(|ref|, rms) = (3, 4, rms, rms)."""
    ref = np.array([3.0, -4.0, 0.0, 1.0])
    rms = np.sqrt(26.0 / 4.0)
    got = orc.max_rel_err_strict(np.array([3.3, -4.0, 0.5, 1.2]), ref)
    assert got == pytest.approx(max(0.3 / 3.0, 0.5 / rms, 0.2 / rms))
    assert got == pytest.approx(0.5 / rms)
    assert orc.max_rel_err_strict(ref, ref) == 0.0
    # an error on a large element counts against that element, not against the rms
    assert orc.max_rel_err_strict(np.array([3.0, -4.4, 0.0, 1.0]), ref) == pytest.approx(0.1)
    # never looser than the primary metric
    y = ref + np.array([0.01, -0.02, 0.03, 0.0])
    assert orc.max_rel_err_strict(y, ref) >= orc.max_rel_err(y, ref)


# --------------------------------------------------------------------------------------
# Planted mistakes: each plausible slip must be caught by the brute-force pin.
# --------------------------------------------------------------------------------------
def _mutants():
    true_rope, true_rms, true_attn = orc.rope, orc.rmsnorm, orc.attention

    def rope_wrong_sign(u, positions, theta):
        return true_rope(u, -np.asarray(positions, float), theta)

    def rope_half_split(u, positions, theta):
        u = np.asarray(u, float); dh = u.shape[-1]
        perm = np.concatenate([np.arange(0, dh, 2), np.arange(1, dh, 2)])
        inv = np.argsort(perm)
        return true_rope(u[..., inv], positions, theta)[..., perm]

    def rms_eps_outside(x, gain, eps):
        x = np.asarray(x, float)
        return x / (np.sqrt(np.mean(x * x, axis=-1, keepdims=True)) + eps) * gain

    def rms_no_gain(x, gain, eps):
        return true_rms(x, np.ones_like(gain), eps)

    def attn_strict_mask(q, k, v, qpos):
        return true_attn(q, k, v, np.maximum(np.asarray(qpos) - 1, 0))

    def attn_no_scale(q, k, v, qpos):
        return true_attn(np.asarray(q) * math.sqrt(q.shape[-1]), k, v, qpos)

    def attn_interleaved_gqa(q, k, v, qpos):
        hq, hkv = q.shape[1], k.shape[1]
        idx = np.arange(hq) % hkv
        return true_attn(q, np.asarray(k)[:, idx], np.asarray(v)[:, idx], qpos)

    def silu_as_sigmoid(z):
        return 1.0 / (1.0 + np.exp(-np.asarray(z, float)))

    return {
        "rope": [rope_wrong_sign, rope_half_split],
        "rmsnorm": [rms_eps_outside, rms_no_gain],
        "attention": [attn_strict_mask, attn_no_scale, attn_interleaved_gqa],
        "silu": [silu_as_sigmoid],
    }


def test_planted_mistakes_are_caught(monkeypatch):
    cfg = small_cfg(eps=1e-2)           # a large eps so its placement matters
    layers = rand_layers(cfg, 11, 2)
    chunks = [np.random.default_rng(5).normal(size=(4, cfg["d_model"]))]
    want = brute_shard(cfg, layers, chunks)
    np.testing.assert_allclose(run_oracle(cfg, layers, chunks), want, rtol=1e-11, atol=1e-12)
    for name, muts in _mutants().items():
        original = getattr(orc, name)
        for mut in muts:
            monkeypatch.setattr(orc, name, mut)
            got = run_oracle(cfg, layers, chunks)
            assert np.max(np.abs(got - want)) > 1e-6, f"pin blind to {mut.__name__}"
            monkeypatch.setattr(orc, name, original)


# ---- the ends of a model (embedding, final norm + LM head, greedy choice) -------------------
def test_ends_embedding_is_a_one_hot_product_and_logits_match_torch_f64():
    import torch
    rng = np.random.default_rng(11)
    V, d = 37, 16
    table = rng.standard_normal((V, d)).astype(np.float32)
    ids = [0, 36, 5, 5, 20]
    onehot = np.zeros((len(ids), V)); onehot[np.arange(len(ids)), ids] = 1.0
    np.testing.assert_array_equal(orc.embed(table, ids), onehot @ table.astype(np.float64))
    x = rng.standard_normal((4, d)); g = 1.0 + 0.1 * rng.standard_normal(d); W = rng.standard_normal((V, d))
    want = torch.nn.functional.linear(
        torch.nn.functional.rms_norm(torch.from_numpy(x), (d,), torch.from_numpy(g), 1e-5), torch.from_numpy(W)).numpy()
    np.testing.assert_allclose(orc.logits(x, g, W, 1e-5), want, rtol=1e-12, atol=1e-12)


def test_ends_logits_closed_form_and_greedy_rule():
    d, V = 8, 5
    W = np.arange(V * d, dtype=np.float64).reshape(V, d)
    # a constant row c normalises to c / sqrt(c^2 + eps) in every element: logits are row sums times that
    c, eps = 3.0, 0.25
    lg = orc.logits(np.full((1, d), c), np.ones(d), W, eps)
    np.testing.assert_allclose(lg[0], W.sum(axis=1) * c / np.sqrt(c * c + eps), rtol=1e-14)
    # the gain multiplies after normalisation: doubling it doubles the logits
    np.testing.assert_allclose(orc.logits(np.full((1, d), c), 2 * np.ones(d), W, eps), 2 * lg, rtol=1e-14)
    assert list(orc.greedy(np.array([[1.0, 7.0, 7.0, 2.0], [-1.0, -3.0, -1.0, -5.0]]))) == [1, 0]
