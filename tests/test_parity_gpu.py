"""GPU parity: libshard (HIP, through the C-ABI) against the float64 CPU oracle on the same
seeded inputs, element by element, with max|y - y_ref| / max|y_ref| <= 1e-3 (fp32) or
2e-2 (bf16), checked after the prefill and after every decode step."""
import numpy as np
import pytest

from paper_2405_14371_amd import synth
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def chunks_for(cfg, seed, B, T, n_dec):
    out = [np.concatenate([synth.hidden_states(cfg, seed, "prefill", 0, b, 1, T) for b in range(B)])]
    for s in range(n_dec):
        out.append(np.concatenate([synth.hidden_states(cfg, seed, "dec", s, b, 1, 1) for b in range(B)]))
    return out


def run_case(lib, cfg, n_layers, dtype, B, T, n_dec, seed=0, gains=False, page_size=16, max_seq_len=None):
    layers = H.make_layers(cfg, seed, n_layers, dtype, gains)
    sh = H.gpu_shard(lib, cfg, layers, dtype, max_seqs=B, max_seq_len=max_seq_len or (T + n_dec),
                     page_size=page_size, max_batch_tokens=B * T)
    ids = [sh.seq_alloc() for _ in range(B)]
    chunks = chunks_for(cfg, seed, B, T, n_dec)
    got = H.run_gpu(sh, ids, chunks)
    want = H.run_oracle(cfg, layers, chunks)
    H.assert_parity(got, want, H.TOL[dtype], f"{dtype} B{B} T{T}")
    for i in ids:
        assert sh.seq_len(i) == T + n_dec
    sh.close()
    return got, want


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tiny_config_prefill_32_decode_16(lib, dtype):
    """The tiny configuration: 2 layers, d 256, 4 heads x 64, FFN 688, batch 1, 32 + 16."""
    run_case(lib, synth.model_cfg("tiny"), 2, dtype, B=1, T=32, n_dec=16)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_sizes_random_gains_small_pages(lib, dtype):
    """T and context lengths that are not multiples of any tile, gains != 1, 3-token pages."""
    run_case(lib, synth.model_cfg("tiny"), 2, dtype, B=2, T=37, n_dec=5, seed=3, gains=True, page_size=3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_grouped_query_attention(lib, dtype):
    cfg = synth.model_cfg("tiny", n_heads=8, n_kv_heads=2, head_dim=32, ffn_dim=344)
    run_case(lib, cfg, 2, dtype, B=3, T=45, n_dec=4, seed=5, gains=True, page_size=16)


def test_single_token_prefill_and_page_size_one(lib):
    run_case(lib, synth.model_cfg("tiny"), 1, "f32", B=1, T=1, n_dec=3, page_size=1)


def test_head_dim_128_and_wide_batch_decode(lib):
    """dh = 128 (the Llama2 head size) and a decode batch of 16 (two passes of 8 rows)."""
    cfg = synth.model_cfg("tiny", d_model=512, n_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=1024)
    run_case(lib, cfg, 2, "f32", B=16, T=20, n_dec=3, seed=7)


@pytest.mark.parametrize("B", [5, 8, 9, 16, 17, 40])
def test_bf16_batches_above_4_decode_on_matrix_cores(lib, B):
    """bf16 decode batches of more than 4 rows take the MFMA projection kernels, one pass over
    the weights per group of up to 16 sequences (17 and 40: a ragged last group); GQA, random
    gains, ragged page use."""
    cfg = synth.model_cfg("tiny", d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=1024)
    run_case(lib, cfg, 2, "bf16", B=B, T=19, n_dec=4, seed=21, gains=True, page_size=16)


@pytest.mark.parametrize("ffn", [2240, 5120, 7424, 8960, 11520, 13440, 15360, 20480])
def test_matrix_core_decode_rows_per_workgroup(lib, ffn):
    """The MFMA decode projections give every workgroup N / 256 rows (rounded up to even, at
    most 128, else two rounds): gate/up widths that come out as 18, 40, 58, 70, 90, 106, 120
    and 2 x 80 rows, i.e. 2..8 row tiles with and without a partial last tile."""
    cfg = synth.model_cfg("tiny", d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=ffn)
    run_case(lib, cfg, 1, "bf16", B=6, T=8, n_dec=2, seed=33, gains=True)


@pytest.mark.parametrize("ffn,B", [(2304, 6), (5120, 5), (7680, 16), (5120, 19)])
def test_matrix_core_decode_weights_through_lds_ring(lib, ffn, B):
    """Inner dimensions of 2048 and more (multiples of 256, not a power of two: d_model 2304 and
    the FFN widths) with at most 64 rows per workgroup: the batched decode projections stream
    their weights through an LDS ring of direct loads (the O projection, K = 2048, does not);
    16, 18, 40 and 60 rows per workgroup (1 to 4 row tiles, with partial tiles), a down
    projection whose 9 k-steps barely exceed the ring, batches of 5..19."""
    cfg = synth.model_cfg("tiny", d_model=2304, n_heads=16, n_kv_heads=4, head_dim=128, ffn_dim=ffn)
    run_case(lib, cfg, 1, "bf16", B=B, T=4, n_dec=2, seed=61, gains=True)


@pytest.mark.parametrize("hq,hkv,B,T,page", [(8, 2, 1, 37, 16), (8, 1, 6, 150, 16), (8, 1, 2, 300, 3),
                                             (16, 1, 3, 70, 16), (12, 2, 5, 33, 16), (16, 2, 1, 1, 1),
                                             (8, 2, 1, 1100, 16), (16, 1, 2, 1030, 16)])
def test_grouped_query_decode_attention_on_matrix_cores(lib, hq, hkv, B, T, page):
    """Half cache, dh = 128 and 4..16 query heads per KV head: the decode attention kernel that
    puts the heads of a group on the MFMA's second dimension (groups of 4, 8, 16 and 6 heads;
    contexts of one token, within one 16-token tile, over several tiles in one 16-wave workgroup,
    and past 1024 tokens, where the context is cut into slices that a second kernel merges;
    3-token and 1-token pages)."""
    cfg = synth.model_cfg("tiny", d_model=256, n_heads=hq, n_kv_heads=hkv, head_dim=128, ffn_dim=512)
    run_case(lib, cfg, 2, "bf16", B=B, T=T, n_dec=5, seed=41, gains=True, page_size=page)


@pytest.mark.parametrize("B,T", [(2, 37), (1, 200), (3, 128)])
def test_half_prefill_projections_split_k(lib, B, T):
    """Few output tiles and a long inner dimension: the half-precision O and down projections of
    the prefill run as 3 or 4 K slices whose partial sums a second kernel adds in slice order
    (O: K = 2048 = 32 k-steps in 4 slices; down: K = 2368 = 37 k-steps, which 4 slices do not
    divide evenly)."""
    cfg = synth.model_cfg("tiny", d_model=256, n_heads=16, n_kv_heads=4, head_dim=128, ffn_dim=2368)
    run_case(lib, cfg, 2, "bf16", B=B, T=T, n_dec=2, seed=57, gains=True)


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


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_largest_batch_of_64_sequences(lib, dtype):
    """SHARD_MAX_BATCH sequences in one call (fp32: eight passes of 8 rows; bf16: four groups
    of 16 on the matrix cores), and one more is refused before anything is launched."""
    cfg = synth.model_cfg("tiny", d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=1024)
    run_case(lib, cfg, 1, dtype, B=64, T=3, n_dec=2, seed=73, gains=True)
    layers = H.make_layers(cfg, 73, 1, dtype)
    sh = H.gpu_shard(lib, cfg, layers, dtype, max_seqs=65, max_seq_len=8, page_size=4, max_batch_tokens=65)
    ids = [sh.seq_alloc() for _ in range(65)]
    x = H.to_dev(np.zeros((65, 1, cfg["d_model"]), np.float32))
    with pytest.raises(lib.ShardError) as e:
        sh.prefill(ids, 1, x, x.clone())
    assert e.value.code == lib.SHARD_E_INVAL
    assert all(sh.seq_len(i) == 0 for i in ids)
    sh.close()


def test_fp32_prefill_two_k_slices(lib):
    """512 tokens against a model width of 2304: the O and down projections (K = 2048) have 144
    tiles of 128 x 64, at most one per compute unit, and run as two K slices plus the ordered
    reduction."""
    cfg = synth.model_cfg("tiny", d_model=2304, n_heads=16, n_kv_heads=4, head_dim=128, ffn_dim=2048)
    run_case(lib, cfg, 1, "f32", B=1, T=512, n_dec=1, seed=89, gains=True)


def test_fp32_prefill_with_192_row_weight_tiles(lib):
    """512 tokens against 12288 QKV rows and 22016 gate/up rows (a ragged last tile): the shapes
    for which the fp32 prefill GEMM takes its 192 x 64 and 192 x 128 tiles, with a short inner
    dimension so that the oracle stays quick."""
    cfg = synth.model_cfg("tiny", d_model=64, n_heads=32, n_kv_heads=32, head_dim=128, ffn_dim=11008)
    run_case(lib, cfg, 1, "f32", B=1, T=512, n_dec=1, seed=79, gains=True)


def test_sixteen_thousand_tokens_in_one_token_pages(lib):
    """A context of 16,500 tokens in pages of one token: the block-table row is longer than the
    prefill attention kernel's LDS copy (it falls back to the kernel that reads pages from global
    memory) and a decode slice spans more pages than its LDS page cache holds."""
    run_case(lib, synth.model_cfg("tiny"), 1, "f32", B=1, T=16500, n_dec=2, seed=71, page_size=1)


def test_long_context_spans_many_key_tiles_and_splits(lib):
    cfg = synth.model_cfg("tiny")
    run_case(lib, cfg, 1, "f32", B=1, T=300, n_dec=3, seed=9)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_llama2_7b_width_two_layers(lib, dtype):
    """Full 7B layer shapes (d 4096, 32 x 128, FFN 11008): several GEMM tiles per dimension,
    a ragged row count, and decode steps through the streaming kernels."""
    run_case(lib, synth.model_cfg("7b"), 2, dtype, B=1, T=72, n_dec=4, seed=1)


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


def _sweep_cases():
    """Seeded shapes chosen to land on every tile variant and tail of the prefill kernels:
    query blocks of 128 with ragged ends, key blocks of 32, contexts that start above zero,
    head sizes 64 and 128 (LDS-staged attention) and 32 (per-wave attention), K multiples and
    non-multiples of the direct-to-LDS k-step, page sizes that divide nothing."""
    rng = np.random.default_rng(2024)
    cases = []
    for i in range(10):
        dh = int(rng.choice([32, 64, 128]))
        hkv = int(rng.choice([1, 2, 4]))
        hq = hkv * int(rng.choice([1, 2, 4]))
        d = int(rng.choice([128, 192, 256, 320]))
        ffn = int(rng.choice([344, 512, 688, 1000]))
        cases.append(dict(dtype="f32" if i % 2 == 0 else "bf16", d_model=d, n_heads=hq, n_kv_heads=hkv, head_dim=dh,
                          ffn_dim=ffn, B=int(rng.integers(1, 4)), T0=int(rng.integers(1, 200)),
                          T1=int(rng.integers(1, 300)), n_dec=2, page=int(rng.choice([1, 5, 16, 64])), seed=100 + i))
    cases.append(dict(dtype="f32", d_model=256, n_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=688, B=2, T0=130, T1=259,
                      n_dec=2, page=16, seed=120))
    cases.append(dict(dtype="bf16", d_model=512, n_heads=8, n_kv_heads=1, head_dim=128, ffn_dim=1000, B=1, T0=1, T1=385,
                      n_dec=2, page=1, seed=121))
    return cases


@pytest.mark.parametrize("case", _sweep_cases(), ids=lambda c: f"{c['dtype']}-d{c['d_model']}-h{c['n_heads']}x{c['head_dim']}-kv{c['n_kv_heads']}-T{c['T0']}+{c['T1']}-p{c['page']}")
def test_seeded_shape_sweep_two_prefill_chunks_then_decode(lib, case):
    c = case
    cfg = synth.model_cfg("tiny", d_model=c["d_model"], n_heads=c["n_heads"], n_kv_heads=c["n_kv_heads"],
                          head_dim=c["head_dim"], ffn_dim=c["ffn_dim"])
    B, T0, T1 = c["B"], c["T0"], c["T1"]
    layers = H.make_layers(cfg, c["seed"], 2, c["dtype"], gains=True)
    sh = H.gpu_shard(lib, cfg, layers, c["dtype"], max_seqs=B, max_seq_len=T0 + T1 + c["n_dec"],
                     page_size=c["page"], max_batch_tokens=B * max(T0, T1))
    ids = [sh.seq_alloc() for _ in range(B)]
    chunks = [np.concatenate([synth.hidden_states(cfg, c["seed"], "prefill", k, b, 1, T) for b in range(B)])
              for k, T in enumerate((T0, T1))]
    chunks += [np.concatenate([synth.hidden_states(cfg, c["seed"], "dec", s, b, 1, 1) for b in range(B)])
               for s in range(c["n_dec"])]
    # the second chunk is a prefill on a non-empty cache (its first chunk may even be one token)
    torch = H.torch_mod()
    got = []
    st = torch.cuda.current_stream().cuda_stream
    for k, x in enumerate(chunks):
        xd = H.to_dev(x); yd = torch.empty_like(xd)
        if k < 2:
            sh.prefill(ids, x.shape[1], xd, yd, st)
        else:
            sh.decode(ids, xd, yd, st)
        torch.cuda.synchronize()
        got.append(yd.cpu().numpy())
    want = H.run_oracle(cfg, layers, chunks)
    H.assert_parity(got, want, H.TOL[c["dtype"]], str(c))
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
