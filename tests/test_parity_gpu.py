"""GPU parity: libshard (HIP, through the C-ABI) against the float64 CPU oracle on the same
seeded inputs, element by element, with max|y - y_ref| / max|y_ref| <= 1e-3 (fp32) or
2e-2 (bf16) and the element-wise metric with an rms floor <= 4e-3 / 8e-2, checked after every
prefill chunk and after every decode step."""
import numpy as np
import pytest

from paper_2405_14371_amd import synth
from tests import gpu_harness as H
from tests import gpu_shapes as S

pytestmark = pytest.mark.gpu


def chunks_for(cfg, seed, B, T, n_dec):
    out = [np.concatenate([synth.hidden_states(cfg, seed, "prefill", 0, b, 1, T) for b in range(B)])]
    for s in range(n_dec):
        out.append(np.concatenate([synth.hidden_states(cfg, seed, "dec", s, b, 1, 1) for b in range(B)]))
    return out


def run_case(lib, cfg, n_layers, dtype, B, T, n_dec, seed=0, gains=False, page_size=16, max_seq_len=None):
    """Prefill chunk(s) of T tokens (an int or a tuple of chunk lengths) and n_dec decode steps
    through the library and through the oracle; every output tensor compared."""
    Ts = (T,) if isinstance(T, int) else tuple(T)
    layers = H.make_layers(cfg, seed, n_layers, dtype, gains)
    sh = H.gpu_shard(lib, cfg, layers, dtype, max_seqs=B, max_seq_len=max_seq_len or (sum(Ts) + n_dec),
                     page_size=page_size, max_batch_tokens=B * max(Ts))
    ids = [sh.seq_alloc() for _ in range(B)]
    chunks = [np.concatenate([synth.hidden_states(cfg, seed, "prefill", k, b, 1, t) for b in range(B)]) for k, t in enumerate(Ts)]
    chunks += [np.concatenate([synth.hidden_states(cfg, seed, "dec", s, b, 1, 1) for b in range(B)]) for s in range(n_dec)]
    got = H.run_gpu(sh, ids, chunks, n_prefill=len(Ts))
    want = H.run_oracle(cfg, layers, chunks)
    H.assert_parity(got, want, dtype, f"{dtype} B{B} T{Ts}")
    for i in ids:
        assert sh.seq_len(i) == sum(Ts) + n_dec
    assert not sh.overflow()
    sh.close()
    return got, want


@pytest.mark.parametrize("case", S.CASES, ids=lambda c: c.id)
def test_parity_with_the_oracle(lib, case):
    """Every registered shape (tests/gpu_shapes.py says why each is there): all rows of every
    prefill chunk and every decode step against the float64 oracle, both error metrics."""
    c = case
    run_case(lib, c.cfg, c.n_layers, c.dtype, c.B, c.prefill, c.n_dec, seed=c.seed, gains=c.gains, page_size=c.page,
             max_seq_len=c.max_seq_len or None)


def test_one_more_than_the_largest_batch_is_refused(lib):
    """SHARD_MAX_BATCH + 1 sequences in one call are refused before anything is launched."""
    cfg = synth.model_cfg("tiny", d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=1024)
    layers = H.make_layers(cfg, 73, 1, "f32")
    sh = H.gpu_shard(lib, cfg, layers, "f32", max_seqs=65, max_seq_len=8, page_size=4, max_batch_tokens=65)
    ids = [sh.seq_alloc() for _ in range(65)]
    x = H.to_dev(np.zeros((65, 1, cfg["d_model"]), np.float32))
    with pytest.raises(lib.ShardError) as e:
        sh.prefill(ids, 1, x, x.clone())
    assert e.value.code == lib.SHARD_E_INVAL
    assert all(sh.seq_len(i) == 0 for i in ids)
    sh.close()


def test_batched_half_precision_paths_are_deterministic(lib):
    """Two shards from the same weights, the same calls: bit-identical outputs through the
    split-K prefill projections, the matrix-core decode projections (register and LDS-ring
    variants) and grouped-query attention, whose partial results all meet in a fixed order."""
    cfg = synth.model_cfg("tiny", d_model=2304, n_heads=16, n_kv_heads=4, head_dim=128, ffn_dim=2368)
    layers = H.make_layers(cfg, 83, 1, "bf16", True)
    chunks = chunks_for(cfg, 83, 6, 40, 3)
    outs = []
    for _ in range(2):
        sh = H.gpu_shard(lib, cfg, layers, "bf16", max_seqs=6, max_seq_len=48, page_size=16, max_batch_tokens=240)
        outs.append(H.run_gpu(sh, [sh.seq_alloc() for _ in range(6)], chunks))
        sh.close()
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a, b)


def test_chunked_prefill_and_ragged_decode_batch(lib):
    """Two sequences prefilled separately to different lengths (one of them in two chunks),
    then decoded together: positions and lengths differ inside one decode call."""
    cfg = synth.model_cfg("tiny")
    layers = H.make_layers(cfg, 11, 2, gains=True)
    sh = H.gpu_shard(lib, cfg, layers, max_seqs=2, max_seq_len=64, page_size=4, max_batch_tokens=64)
    a, b = sh.seq_alloc(), sh.seq_alloc()
    xa = synth.hidden_states(cfg, 11, "prefill", 0, 0, 1, 33)
    xb = synth.hidden_states(cfg, 11, "prefill", 0, 1, 1, 9)
    ga = H.run_gpu(sh, [a], [xa[:, :20], xa[:, 20:]])
    gb = H.run_gpu(sh, [b], [xb])
    dec = [np.concatenate([synth.hidden_states(cfg, 11, "dec", s, m, 1, 1) for m in range(2)]) for s in range(3)]
    torch = H.torch_mod()
    gd = []
    for x in dec:
        xd = H.to_dev(x); yd = torch.empty_like(xd)
        sh.decode([a, b], xd, yd, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        gd.append(yd.cpu().numpy())
    o = H.orc.OracleShard(cfg, layers)
    wa = o.forward("a", xa[0].astype(np.float64))
    wb = o.forward("b", xb[0].astype(np.float64))
    H.assert_parity([np.concatenate(ga, axis=1)[0]], [wa], 1e-3, "chunked prefill")
    H.assert_parity([gb[0][0]], [wb], 1e-3, "second sequence")
    for s, x in enumerate(dec):
        w = np.stack([o.forward("a", x[0].astype(np.float64)), o.forward("b", x[1].astype(np.float64))])
        H.assert_parity([gd[s]], [w], 1e-3, f"ragged decode {s}")
    assert sh.seq_len(a) == 36 and sh.seq_len(b) == 12
    sh.close()


def test_shard_composition_is_exact_on_gpu(lib):
    """Layers [0,1) then [1,2) on the handed-over activation give bit-identical results to
    [0,2): the hand-off is fp32 and the kernels are deterministic."""
    cfg = synth.model_cfg("tiny")
    layers = H.make_layers(cfg, 13, 2)
    chunks = chunks_for(cfg, 13, 1, 24, 3)
    kv = dict(max_seqs=1, max_seq_len=32, page_size=8)
    whole = H.gpu_shard(lib, cfg, layers, **kv)
    first = H.gpu_shard(lib, cfg, layers[:1], layer_lo=0, **kv)
    second = H.gpu_shard(lib, cfg, layers[1:], layer_lo=1, **kv)
    w = H.run_gpu(whole, [whole.seq_alloc()], chunks)
    mid = H.run_gpu(first, [first.seq_alloc()], chunks)
    two = H.run_gpu(second, [second.seq_alloc()], mid)
    for x, y in zip(w, two):
        np.testing.assert_array_equal(x, y)
    again = H.gpu_shard(lib, cfg, layers, **kv)
    for x, y in zip(w, H.run_gpu(again, [again.seq_alloc()], chunks)):
        np.testing.assert_array_equal(x, y)          # run-to-run determinism
    for s in (whole, first, second, again):
        s.close()


def test_decode_after_prefill_matches_longer_prefill_on_gpu(lib):
    """prefill(T) + decode(1) against prefill(T+1): two different kernel paths, same maths."""
    cfg = synth.model_cfg("tiny")
    layers = H.make_layers(cfg, 17, 2)
    x = synth.hidden_states(cfg, 17, "prefill", 0, 0, 1, 41)
    kv = dict(max_seqs=1, max_seq_len=48, page_size=16)
    a = H.gpu_shard(lib, cfg, layers, **kv)
    b = H.gpu_shard(lib, cfg, layers, **kv)
    ya = H.run_gpu(a, [a.seq_alloc()], [x[:, :40], x[:, 40:]])
    yb = H.run_gpu(b, [b.seq_alloc()], [x])
    err = H.orc.max_rel_err(ya[1][0, 0], yb[0][0, 40])
    assert err < 2e-5, err
    np.testing.assert_allclose(ya[0][0], yb[0][0, :40], rtol=0, atol=1e-5 * np.abs(yb[0]).max())
    a.close(); b.close()


def test_output_may_alias_input_and_freed_pages_are_reused(lib):
    cfg = synth.model_cfg("tiny")
    layers = H.make_layers(cfg, 19, 2)
    torch = H.torch_mod()
    sh = H.gpu_shard(lib, cfg, layers, max_seqs=2, max_seq_len=40, page_size=4)
    x = synth.hidden_states(cfg, 19, "prefill", 0, 0, 1, 30)
    want = H.run_oracle(cfg, layers, [x])[0]
    st = torch.cuda.current_stream().cuda_stream
    for _ in range(3):                     # slot and pages are recycled each round
        sid = sh.seq_alloc()
        junk = sh.seq_alloc()
        buf = H.to_dev(x)
        sh.prefill([sid], 30, buf, buf, st)          # in place
        torch.cuda.synchronize()
        H.assert_parity([buf.cpu().numpy()], [want], 1e-3, "aliased")
        sh.seq_free(junk); sh.seq_free(sid)
    sh.close()


def test_runtime_errors_leave_state_unchanged(lib):
    cfg = synth.model_cfg("tiny")
    layers = H.make_layers(cfg, 23, 1)
    torch = H.torch_mod()
    sh = H.gpu_shard(lib, cfg, layers, max_seqs=2, max_seq_len=16, page_size=4, max_batch_tokens=16)
    x = H.to_dev(synth.hidden_states(cfg, 23, "prefill", 0, 0, 1, 16))
    y = torch.empty_like(x)
    a = sh.seq_alloc()

    def expect(code, fn, *args):
        with pytest.raises(lib.ShardError) as e:
            fn(*args)
        assert e.value.code == code, e.value

    expect(lib.SHARD_E_STATE, sh.decode, [a], x, y)                 # decode on an empty sequence
    expect(lib.SHARD_E_STATE, sh.prefill, [a, a], 2, x, y)          # duplicate id
    expect(lib.SHARD_E_STATE, sh.prefill, [1], 2, x, y)             # slot 1 not live
    expect(lib.SHARD_E_KV_FULL, sh.prefill, [a], 17, x, y)          # longer than max_seq_len...
    expect(lib.SHARD_E_INVAL, sh.prefill, [a], 0, x, y)                # no tokens
    expect(lib.SHARD_E_INVAL, sh.prefill, [], 4, x, y)                 # no sequences
    expect(lib.SHARD_E_INVAL, sh.decode, [], x, y)
    expect(lib.SHARD_E_INVAL, sh.prefill, [a], 4, None, y)
    assert sh.seq_len(a) == 0
    sh.prefill([a], 12, x, y)
    expect(lib.SHARD_E_KV_FULL, sh.prefill, [a], 5, x, y)           # 12 + 5 > 16
    assert sh.seq_len(a) == 12
    b = sh.seq_alloc()
    expect(lib.SHARD_E_KV_FULL, sh.seq_alloc)
    sh.seq_free(b)
    expect(lib.SHARD_E_STATE, sh.seq_free, b)
    torch.cuda.synchronize()
    sh.close()


def test_create_rejects_16_bit_weights_outside_the_range_of_half(lib):
    """bf16 matrices live on the device as IEEE half with the RMSNorm gains folded in: a weight
    above 65504, or a weight whose product with its gain is, makes shard_create fail."""
    cfg = synth.model_cfg("tiny")

    def create(mutate):
        layers = H.make_layers(cfg, 29, 1, "bf16")
        mutate(layers[0])
        with pytest.raises(lib.ShardError) as e:
            H.gpu_shard(lib, cfg, layers, "bf16", max_seqs=1, max_seq_len=16, page_size=4)
        assert e.value.code == lib.SHARD_E_INVAL and "65504" in str(e.value), e.value

    def big_weight(lw):
        w = lw["w_down"].copy()
        w.flat[5] = 65536.0           # exact in bf16, above half's largest finite value
        lw["w_down"] = w

    def big_gain(lw):
        g = lw["g_ffn"].copy()
        g[7] = 1e7                    # times weights of about 0.02
        lw["g_ffn"] = g

    create(big_weight)
    create(big_gain)
    ok = H.gpu_shard(lib, cfg, H.make_layers(cfg, 29, 1, "bf16"), "bf16", max_seqs=1, max_seq_len=16, page_size=4)
    ok.close()


def test_profile_and_kernel_timing(lib):
    cfg = synth.model_cfg("tiny")
    layers = H.make_layers(cfg, 29, 2)
    sh = H.gpu_shard(lib, cfg, layers, max_seqs=1, max_seq_len=64)
    prof = sh.profile(B=1, T_prefill=32, n_decode=4, iters=2)
    assert len(prof) == 2
    for p in prof:
        assert 0 < p["t_decode_s"] < 1.0 and 0 < p["t_prefill_s"] < 1.0
        assert p["t_avg_s"] == pytest.approx((p["t_prefill_s"] + 4 * p["t_decode_s"]) / 5)
        assert p["act_bytes_prefill"] == 32 * 256 * 4 and p["act_bytes_decode"] == 256 * 4
        assert p["weight_bytes"] == H.orc.params_per_layer(cfg) * 4
        assert p["kv_bytes_per_token"] == 2 * 4 * 64 * 4
    torch = H.torch_mod()
    sid = sh.seq_alloc()
    x = H.to_dev(synth.hidden_states(cfg, 29, "prefill", 0, 0, 1, 8)); y = torch.empty_like(x)
    sh.timing_enable(True)
    sh.prefill([sid], 8, x, y)
    sh.decode([sid], x[:, :1].contiguous(), y[:, :1].contiguous())
    t = sh.timing_read()
    for k in lib.KERNEL_CLASSES:
        assert t[k]["launches"] == (4 if k == "prefill_norm" else 2), (k, t[k])
    assert all(v["seconds"] > 0 for k, v in t.items() if v["launches"])
    sh.timing_enable(False)
    sh.close()


def test_profile_layer_times_add_up_to_the_calls(lib):
    """Six layers of one shape (7B width, so that a layer's kernels outweigh the launch gaps):
    the per-layer times of shard_profile add up to what HIP events around the same calls read,
    within 20 %, and layers of equal shape time alike (25 %)."""
    torch = H.torch_mod()
    cfg = synth.model_cfg("tiny", d_model=2048, n_heads=16, n_kv_heads=16, head_dim=128, ffn_dim=5504)
    L, T, n_dec = 6, 256, 8
    layers = H.make_layers(cfg, 31, 1) * L            # the same weights six times: the shape is what matters
    sh = H.gpu_shard(lib, cfg, layers, max_seqs=2, max_seq_len=T + n_dec, max_batch_tokens=T)
    prof = sh.profile(B=1, T_prefill=T, n_decode=n_dec, iters=3)
    t_pre = [p["t_prefill_s"] for p in prof]
    t_dec = [p["t_decode_s"] for p in prof]
    # the same calls under the caller's own events (best of three, after a warm-up)
    x = H.to_dev(synth.hidden_states(cfg, 31, "prefill", 0, 0, 1, T)); y = torch.empty_like(x)
    xd = H.to_dev(synth.hidden_states(cfg, 31, "dec", 0, 0, 1, 1)); yd = torch.empty_like(xd)
    st = torch.cuda.current_stream()
    best_pre, best_dec = 1e9, 1e9
    for it in range(4):
        sid = sh.seq_alloc()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record(st)
        sh.prefill([sid], T, x, y, st.cuda_stream)
        e[1].record(st)
        for _ in range(n_dec):
            sh.decode([sid], xd, yd, st.cuda_stream)
        e[2].record(st)
        torch.cuda.synchronize()
        sh.seq_free(sid)
        if it:
            best_pre = min(best_pre, e[0].elapsed_time(e[1]) * 1e-3)
            best_dec = min(best_dec, e[1].elapsed_time(e[2]) * 1e-3 / n_dec)
    assert sum(t_pre) == pytest.approx(best_pre, rel=0.20), (t_pre, best_pre)
    assert sum(t_dec) == pytest.approx(best_dec, rel=0.20), (t_dec, best_dec)
    # layers of one shape: every layer within 25 % of the median (layer 0 reads x_in, the others x_out)
    for ts in (t_pre, t_dec):
        med = sorted(ts)[len(ts) // 2]
        assert all(abs(t - med) <= 0.25 * med for t in ts), ts
    sh.close()


def test_measured_profile_feeds_the_planner_and_the_schedule(lib):
    """The chain the paper describes (Sec. 3: profile, then schedule, then collaborative
    inference): shard_profile of one fp32 7B-shaped layer -> the 15-device testbed table of
    Sec. 5.1 -> both dynamic programs at N = 34 and N = 82 -> stages -> both pipeline schedules,
    with the relations the paper reports (tests/testbed.py states them)."""
    from tests import testbed
    cfg = synth.model_cfg("7b")
    layers = H.make_layers(cfg, 43, 1)
    sh = H.gpu_shard(lib, cfg, layers, max_seqs=1, max_seq_len=testbed.PROMPT + 8, max_batch_tokens=testbed.PROMPT)
    prof = sh.profile(B=1, T_prefill=testbed.PROMPT, n_decode=8, iters=2)[0]
    sh.close()
    assert prof["weight_bytes"] == H.orc.params_per_layer(cfg) * 4 and prof["t_prefill_s"] > 0 and prof["t_decode_s"] > 0
    out = testbed.check_chain(lib, prof)
    print(f"measured layer: prefill {prof['t_prefill_s'] * 1e6:.0f} us, decode {prof['t_decode_s'] * 1e6:.0f} us; {out}")


def test_half_range_overflow_is_flagged_and_refuses_further_calls(lib):
    """16-bit path: a value beyond 65504 rounded to half raises the shard's sticky flag, and the
    next call is refused with SHARD_E_RANGE before anything is launched.  Two producers: the half
    copy of the residual stream of a batched decode step (x_in itself out of range), and the
    SwiGLU output of a prefill (weights of ordinary size times a large gate/up pair)."""
    torch = H.torch_mod()
    cfg = synth.model_cfg("tiny", d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=1024)
    layers = H.make_layers(cfg, 35, 1, "bf16")
    sh = H.gpu_shard(lib, cfg, layers, "bf16", max_seqs=6, max_seq_len=16, page_size=4, max_batch_tokens=48)
    ids = [sh.seq_alloc() for _ in range(6)]
    x = H.to_dev(np.concatenate([synth.hidden_states(cfg, 35, "prefill", 0, b, 1, 8) for b in range(6)]))
    y = torch.empty_like(x)
    sh.prefill(ids, 8, x, y)
    torch.cuda.synchronize()
    assert not sh.overflow()
    big = torch.full((6, 1, cfg["d_model"]), 1.0e5, device="cuda")       # 1e5 > 65504
    sh.decode(ids, big, torch.empty_like(big))
    torch.cuda.synchronize()
    assert sh.overflow()
    with pytest.raises(lib.ShardError) as e:
        sh.decode(ids, x[:, :1].contiguous(), y[:, :1].contiguous())
    assert e.value.code == lib.SHARD_E_RANGE and "65504" in str(e.value)
    assert all(sh.seq_len(i) == 9 for i in ids)                          # the refused call added nothing
    assert sh.overflow(clear=True) and not sh.overflow()
    for i in ids:
        sh.seq_free(i)
    a = sh.seq_alloc()
    sh.prefill([a], 8, x[:1], y[:1])                                     # the shard works again
    torch.cuda.synchronize()
    assert not sh.overflow()
    sh.close()
    # SwiGLU output: gate and up of about 25 * sqrt(512) ~ 570 each -> products beyond 65504
    hot = H.make_layers(cfg, 37, 1, "bf16")
    for name in ("w_gate", "w_up"):
        hot[0][name] = synth.round_to_bf16(hot[0][name] * np.float32(25.0 / 0.02))
    sh = H.gpu_shard(lib, cfg, hot, "bf16", max_seqs=1, max_seq_len=16, page_size=4, max_batch_tokens=8)
    a = sh.seq_alloc()
    sh.prefill([a], 8, x[:1], y[:1])
    torch.cuda.synchronize()
    assert sh.overflow()
    sh.close()
    # fp32 shards have no such limit
    sh = H.gpu_shard(lib, cfg, H.make_layers(cfg, 35, 1), "f32", max_seqs=6, max_seq_len=16, page_size=4, max_batch_tokens=48)
    ids = [sh.seq_alloc() for _ in range(6)]
    sh.prefill(ids, 1, big, torch.empty_like(big))
    torch.cuda.synchronize()
    assert not sh.overflow()
    sh.close()


def test_a_failed_launch_check_rolls_the_call_back(lib):
    """The library's final check of a call fails (forced from the host through the test hook
    of shard_introspect.h; every kernel still runs normally): the call returns SHARD_E_HIP, the
    sequences keep their lengths, the pages it reserved are free again - the cache can still
    take a full-length prefill - and the same call succeeds once the failure is gone."""
    torch = H.torch_mod()
    cfg = synth.model_cfg("tiny")
    layers = H.make_layers(cfg, 39, 1)
    sh = H.gpu_shard(lib, cfg, layers, max_seqs=2, max_seq_len=32, page_size=4, max_batch_tokens=64)
    a, b = sh.seq_alloc(), sh.seq_alloc()
    x = H.to_dev(np.concatenate([synth.hidden_states(cfg, 39, "prefill", 0, s, 1, 32) for s in range(2)]))
    y = torch.empty_like(x)
    sh.prefill([a], 5, x[:1, :5].contiguous(), y[:1, :5].contiguous())
    torch.cuda.synchronize()
    lib.inject_launch_error(True)
    try:
        with pytest.raises(lib.ShardError) as e:
            sh.prefill([a, b], 20, x[:, :20].contiguous(), y[:, :20].contiguous())
        assert e.value.code == lib.SHARD_E_HIP and "LDS" in str(e.value)
        with pytest.raises(lib.ShardError) as e:
            sh.decode([a], x[:1, :1].contiguous(), y[:1, :1].contiguous())
        assert e.value.code == lib.SHARD_E_HIP
        with pytest.raises(lib.ShardError):
            H.gpu_shard(lib, cfg, layers, max_seqs=1, max_seq_len=8)
    finally:
        lib.inject_launch_error(False)
    torch.cuda.synchronize()
    assert sh.seq_len(a) == 5 and sh.seq_len(b) == 0
    # every page is available again: b takes the whole 32 tokens, a grows to 32 as well
    sh.prefill([b], 32, x[1:2], y[1:2])
    sh.prefill([a], 27, x[:1, 5:].contiguous(), y[:1, 5:].contiguous())
    torch.cuda.synchronize()
    assert sh.seq_len(a) == 32 and sh.seq_len(b) == 32
    want = H.run_oracle(cfg, layers, [x[1:2].cpu().numpy()])[0]
    H.assert_parity([y[1:2].cpu().numpy()], [want], "f32", "prefill after the rolled-back call")
    sh.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_micro_batches_on_several_streams(lib, dtype):
    """Six sequences driven like pipeline micro-batches: prefills on one stream, then decode
    steps round-robin over five streams - one more than the shard has workspace sets, so a
    set changes hands (the library orders that with events) - while a late prefill of a
    seventh sequence runs next to them.  Every output against the oracle."""
    torch = H.torch_mod()
    cfg = synth.model_cfg("tiny", d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=688)
    n_seq, T, n_dec, seed = 6, 40, 5, 31
    layers = H.make_layers(cfg, seed, 2, dtype, gains=True)
    sh = H.gpu_shard(lib, cfg, layers, dtype, max_seqs=n_seq + 1, max_seq_len=T + n_dec, page_size=16, max_batch_tokens=T)
    ids = [sh.seq_alloc() for _ in range(n_seq + 1)]
    main = torch.cuda.current_stream()
    streams = [torch.cuda.Stream() for _ in range(5)]
    xp = [H.to_dev(synth.hidden_states(cfg, seed, "prefill", 0, b, 1, T)) for b in range(n_seq + 1)]
    xd = [[H.to_dev(synth.hidden_states(cfg, seed, "dec", s, b, 1, 1)) for b in range(n_seq)] for s in range(n_dec)]
    yp = [torch.empty_like(x) for x in xp]
    yd = [[torch.empty_like(x) for x in row] for row in xd]
    for b in range(n_seq):
        sh.prefill([ids[b]], T, xp[b], yp[b], main.cuda_stream)
    for q in streams:
        q.wait_stream(main)
    for s in range(n_dec):
        for b in range(n_seq):
            q = streams[(b + s) % len(streams)]
            if s > 0:                       # this sequence's previous step ran on another stream
                q.wait_stream(streams[(b + s - 1) % len(streams)])
            sh.decode([ids[b]], xd[s][b], yd[s][b], q.cuda_stream)
        if s == 1:                           # a prefill in the middle of the decode traffic
            sh.prefill([ids[n_seq]], T, xp[n_seq], yp[n_seq], main.cuda_stream)
    torch.cuda.synchronize()
    o = H.orc.OracleShard(cfg, layers)
    for b in range(n_seq + 1):
        want = o.forward(b, xp[b].cpu().numpy()[0].astype(np.float64))
        assert H.orc.max_rel_err(yp[b].cpu().numpy()[0], want) <= H.TOL[dtype], f"prefill of sequence {b}"
    for s in range(n_dec):
        for b in range(n_seq):
            want = o.forward(b, xd[s][b].cpu().numpy()[0].astype(np.float64))
            assert H.orc.max_rel_err(yd[s][b].cpu().numpy()[0], want) <= H.TOL[dtype], f"step {s} of sequence {b}"
    sh.close()
