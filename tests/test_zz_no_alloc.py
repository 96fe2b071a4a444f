"""shard_decode_static - the decode entry point that allocates nothing (its intermediate buffers
live in an array inside the library's device image) - against shard_decode: same kernels, so
the outputs must be identical, on two calls in a row, the second with a smaller batch, for the
fp32 streaming path and for the 16-bit matrix-core path; and its refusals."""
import numpy as np
import pytest

from paper_2405_14371_amd import synth
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def two_shards(lib, cfg, dtype, seed, B, T, n_dec):
    layers = H.make_layers(cfg, seed, 2, dtype, gains=True)
    kv = dict(max_seqs=B, max_seq_len=T + n_dec, page_size=16, max_batch_tokens=B * T)
    return layers, H.gpu_shard(lib, cfg, layers, dtype, **kv), H.gpu_shard(lib, cfg, layers, dtype, **kv)


@pytest.mark.parametrize("dtype,B,cfgkw", [
    ("f32", 3, dict()),
    ("bf16", 2, dict()),
    ("bf16", 9, dict(d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=1024)),     # matrix-core projections
    ("f32", 4, dict(d_model=256, n_heads=8, n_kv_heads=2, head_dim=128, ffn_dim=512)),
])
def test_static_decode_equals_decode(lib, dtype, B, cfgkw):
    torch = H.torch_mod()
    cfg = synth.model_cfg("tiny", **cfgkw)
    T, n_dec, seed = 300, 3, 47          # 300 cached tokens: the attention context is cut into slices (partials in scratch)
    layers, ref, sta = two_shards(lib, cfg, dtype, seed, B, T, n_dec)
    ids_r = [ref.seq_alloc() for _ in range(B)]
    ids_s = [sta.seq_alloc() for _ in range(B)]
    xp = H.to_dev(np.concatenate([synth.hidden_states(cfg, seed, "prefill", 0, b, 1, T) for b in range(B)]))
    st = torch.cuda.current_stream().cuda_stream
    yp = torch.empty_like(xp)
    ref.prefill(ids_r, T, xp, yp, st)
    sta.prefill(ids_s, T, xp, torch.empty_like(xp), st)
    want_p = H.run_oracle(cfg, layers, [xp.cpu().numpy()])[0]
    torch.cuda.synchronize()
    H.assert_parity([yp.cpu().numpy()], [want_p], dtype, "prefill")
    o = H.orc.OracleShard(cfg, layers)
    for b in range(B):
        o.forward(b, xp[b].cpu().numpy().astype(np.float64))
    # step 0: all B sequences; step 1: a smaller batch (the first B - 1 ... at least 1); step 2: all again
    for step, nb in enumerate((B, max(1, B - 1), B)):
        x = H.to_dev(np.concatenate([synth.hidden_states(cfg, seed, "dec", step, b, 1, 1) for b in range(nb)]))
        y_r, y_s = torch.empty_like(x), torch.full_like(x, float("nan"))
        ref.decode(ids_r[:nb], x, y_r, st)
        sta.decode_static(ids_s[:nb], x, y_s, st)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(y_s.cpu().numpy(), y_r.cpu().numpy())
        want = np.stack([o.forward(b, x[b].cpu().numpy().astype(np.float64)) for b in range(nb)])
        H.assert_parity([y_s.cpu().numpy()], [want], dtype, f"static decode step {step}")
    assert [sta.seq_len(i) for i in ids_s] == [ref.seq_len(i) for i in ids_r]
    ref.close(); sta.close()


def test_static_decode_refuses_what_does_not_fit_and_timing(lib):
    torch = H.torch_mod()
    # the SwiGLU output of 64 sequences alone, 64 x 40960 floats = 10 MB, is more than the 8 MB array
    cfg = synth.model_cfg("tiny", ffn_dim=40960)
    layers = H.make_layers(cfg, 49, 1)
    sh = H.gpu_shard(lib, cfg, layers, max_seqs=64, max_seq_len=4, page_size=4, max_batch_tokens=64)
    ids = [sh.seq_alloc() for _ in range(64)]
    x = H.to_dev(np.concatenate([synth.hidden_states(cfg, 49, "prefill", 0, b, 1, 1) for b in range(64)]))
    y = torch.empty_like(x)
    sh.prefill(ids, 1, x, y)
    with pytest.raises(lib.ShardError) as e:
        sh.decode_static(ids, x, y)
    assert e.value.code == lib.SHARD_E_INVAL and str(lib.SHARD_STATIC_SCRATCH_BYTES) in str(e.value)
    assert all(sh.seq_len(i) == 1 for i in ids)
    sh.decode_static(ids[:8], x[:8], y[:8])               # 8 sequences fit
    sh.timing_enable(True)
    with pytest.raises(lib.ShardError) as e:
        sh.decode_static(ids[:1], x[:1], y[:1])
    assert e.value.code == lib.SHARD_E_STATE
    sh.timing_enable(False)
    torch.cuda.synchronize()
    assert sh.seq_len(ids[0]) == 2 and sh.seq_len(ids[9]) == 1
    sh.close()
