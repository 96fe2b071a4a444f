"""The ends of a model on the GPU (embedding lookup, final RMSNorm + LM head, greedy choice)
against the oracle, and a whole token loop: embed -> shard -> logits -> argmax."""
import numpy as np
import pytest

from oracle import llama_shard as orc
from paper_2405_14371_amd import synth
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def make_ends(lib, cfg, vocab, dtype, seed=0, **kw):
    w = synth.ends_weights(cfg, seed, vocab, dtype)
    wd = lib.SHARD_F32 if dtype == "f32" else lib.SHARD_BF16
    pack = (lambda a: np.ascontiguousarray(a, dtype=np.float32)) if dtype == "f32" else synth.bf16_bits
    ends = lib.ShardEnds(cfg, vocab, tok_embeddings=pack(w["tok_embeddings"]), g_final=w["g_final"],
                         lm_head=pack(w["lm_head"]), weight_dtype=wd, **kw)
    return ends, w


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("vocab", [1000, 32000])
def test_embedding_logits_and_argmax(lib, dtype, vocab):
    torch = H.torch_mod()
    cfg = synth.model_cfg("tiny", d_model=512, n_heads=4, n_kv_heads=4, head_dim=128, ffn_dim=1024)
    ends, w = make_ends(lib, cfg, vocab, dtype, max_tokens=300)
    rng = np.random.default_rng(5)
    for n in (1, 7, 200):                         # by-value ids, and the staged copy above 128
        ids = [int(v) for v in rng.integers(0, vocab, n)]
        ids[0], ids[-1] = 0, vocab - 1
        x = torch.empty((n, cfg["d_model"]), dtype=torch.float32, device="cuda")
        ends.embed(ids, x)
        torch.cuda.synchronize()
        want = orc.embed(w["tok_embeddings"], ids)
        # fp32 tables are copied bit for bit; bf16 values convert to half exactly above 6.1e-5
        tol = 0.0 if dtype == "f32" else 3e-8
        assert np.max(np.abs(x.cpu().numpy().astype(np.float64) - want)) <= tol
    for n in (1, 3, 8, 13):                       # one pass, and two passes of up to 8 rows
        xin = (3.0 * rng.standard_normal((n, cfg["d_model"]))).astype(np.float32)
        lg = torch.empty((n, vocab), dtype=torch.float32, device="cuda")
        out = torch.empty((n,), dtype=torch.int32, device="cuda")
        ends.logits(torch.from_numpy(xin).cuda(), n, lg)
        ends.argmax(lg, n, out)
        torch.cuda.synchronize()
        got = lg.cpu().numpy().astype(np.float64)
        want = orc.logits(xin, w["g_final"], w["lm_head"], cfg["rms_eps"])
        assert orc.max_rel_err(got, want) <= H.TOL[dtype]
        # the choice is taken in the GPU's own precision: exact against its own logits ...
        np.testing.assert_array_equal(out.cpu().numpy(), orc.greedy(got))
        # ... and a valid choice for the oracle: its logit there is the maximum up to the tolerance
        top = want.max(axis=1)
        assert np.all(want[np.arange(n), out.cpu().numpy()] >= top - H.TOL[dtype] * np.abs(want).max())
    ends.close()


def test_argmax_ties_and_bad_arguments(lib):
    torch = H.torch_mod()
    cfg = synth.model_cfg("tiny")
    ends, _ = make_ends(lib, cfg, 300, "f32", max_tokens=4)
    lg = torch.full((3, 300), -1.0, dtype=torch.float32, device="cuda")
    lg[0, 299] = 5.0; lg[0, 17] = 5.0             # equal maxima: the lower index
    lg[1, 0] = float("nan"); lg[1, 123] = 0.5      # a NaN is never chosen
    out = torch.empty((3,), dtype=torch.int32, device="cuda")
    ends.argmax(lg, 3, out)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [17, 123, 0]
    x = torch.empty((4, cfg["d_model"]), dtype=torch.float32, device="cuda")
    for bad in ([300], [-1], [0, 1, 2, 3, 4]):
        with pytest.raises(lib.ShardError) as e:
            ends.embed(bad, x)
        assert e.value.code == lib.SHARD_E_INVAL
    only_embed = lib.ShardEnds(cfg, 300, tok_embeddings=np.zeros((300, cfg["d_model"]), np.float32))
    with pytest.raises(lib.ShardError) as e:
        only_embed.logits(x, 1, lg)
    assert e.value.code == lib.SHARD_E_STATE
    with pytest.raises(lib.ShardError):
        lib.ShardEnds(cfg, 300)                    # neither end
    only_embed.close(); ends.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_whole_token_loop_against_the_oracle(lib, dtype):
    """Prompt -> embedding -> two shards in sequence -> logits -> greedy token, repeated.
    Both sides are fed the ORACLE's token at every step (so one near-tie cannot derail the
    comparison); the GPU's choice must still be a maximum of the oracle's logits up to the
    tolerance, and its logits must match."""
    torch = H.torch_mod()
    cfg = synth.model_cfg("tiny", d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=688)
    vocab, L, split, T, steps = 777, 4, 1, 9, 6
    ends, w = make_ends(lib, cfg, vocab, dtype)
    wd = lib.SHARD_F32 if dtype == "f32" else lib.SHARD_BF16
    layers = synth.shard_weights(cfg, 3, 0, L, dtype)
    for i, lw in enumerate(layers):
        lw.update(synth.random_gains(cfg, 3, i))
    sh0 = lib.Shard(cfg, lib.pack_layers(layers[:split], wd), 0, weight_dtype=wd, max_seqs=1, max_seq_len=T + steps)
    sh1 = lib.Shard(cfg, lib.pack_layers(layers[split:], wd), split, weight_dtype=wd, max_seqs=1, max_seq_len=T + steps)
    o = orc.OracleShard(cfg, layers)
    s0, s1 = sh0.seq_alloc(), sh1.seq_alloc()
    prompt = [int(v) for v in np.random.default_rng(9).integers(0, vocab, T)]
    d = cfg["d_model"]
    x = torch.empty((T, d), dtype=torch.float32, device="cuda")
    lg = torch.empty((1, vocab), dtype=torch.float32, device="cuda")
    tok = torch.empty((1,), dtype=torch.int32, device="cuda")
    feed, n_in = prompt, T
    for step in range(steps + 1):
        xs = x[:n_in]
        ends.embed(feed, xs)
        if step == 0:
            sh0.prefill([s0], n_in, xs, xs); sh1.prefill([s1], n_in, xs, xs)
        else:
            sh0.decode([s0], xs, xs); sh1.decode([s1], xs, xs)
        ends.logits(xs[n_in - 1:], 1, lg)
        ends.argmax(lg, 1, tok)
        torch.cuda.synchronize()
        y = o.forward(0, orc.embed(w["tok_embeddings"], feed))
        want = orc.logits(y[-1:], w["g_final"], w["lm_head"], cfg["rms_eps"])
        assert orc.max_rel_err(lg.cpu().numpy().astype(np.float64), want) <= H.TOL[dtype], f"step {step}"
        choice = int(tok.cpu()[0])
        assert want[0, choice] >= want.max() - H.TOL[dtype] * np.abs(want).max()
        feed, n_in = [int(orc.greedy(want)[0])], 1
    sh0.close(); sh1.close(); ends.close()
