"""CPU-only checks of the C-ABI: the library loads, exports every symbol include/shard.h
declares, and rejects bad arguments before it touches a GPU."""
import ctypes as C
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(shard_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    syms = declared_symbols()
    for name in ("shard_create", "shard_destroy", "shard_prefill", "shard_decode", "shard_profile"):
        assert name in syms


def test_library_exports_every_declared_symbol(lib):
    handle = lib.load()
    for name in declared_symbols():
        assert hasattr(handle, name), f"libshard.so does not export {name}"
    assert sorted(lib.EXPORTS) == declared_symbols()


def test_binding_struct_layout_matches_header(lib):
    # 9 x 4-byte fields; 4 x int32; 9 pointers; 3 doubles + 4 uint64
    assert C.sizeof(lib.ModelCfg) == 36
    assert C.sizeof(lib.KvCfg) == 16
    assert C.sizeof(lib.LayerWeights) == 9 * C.sizeof(C.c_void_p)
    assert C.sizeof(lib.LayerProfile) == 56


def _create(lib, mc, kc, lo=0, hi=1, weights=None):
    h = C.c_void_p()
    rc = lib.load().shard_create(C.byref(h), C.byref(mc) if mc else None, C.byref(kc) if kc else None,
                                 lo, hi, weights, 0)
    assert not h.value
    return rc, lib.last_error()


GOOD = dict(d_model=256, n_heads=4, n_kv_heads=4, head_dim=64, ffn_dim=688, rms_eps=1e-5,
            rope_theta=1e4, weight_dtype=0, act_dtype=0)


@pytest.mark.parametrize("field,value,needle", [
    ("head_dim", 48, "head_dim"),
    ("n_kv_heads", 3, "n_kv_heads"),
    ("d_model", 252, "multiples of 8"),
    ("ffn_dim", 0, "positive"),
    ("weight_dtype", 7, "weight_dtype"),
    ("act_dtype", 1, "act_dtype"),
    ("rope_theta", 0.0, "rope_theta"),
])
def test_create_rejects_bad_model(lib, field, value, needle):
    mc = lib.ModelCfg(**dict(GOOD, **{field: value}))
    rc, msg = _create(lib, mc, lib.KvCfg(1, 64, 16, 0))
    assert rc == lib.SHARD_E_INVAL and needle in msg


def test_create_rejects_bad_ranges_and_nulls(lib):
    mc, kc = lib.ModelCfg(**GOOD), lib.KvCfg(1, 64, 16, 0)
    assert _create(lib, mc, kc, 2, 2)[0] == lib.SHARD_E_INVAL
    assert _create(lib, mc, kc, -1, 2)[0] == lib.SHARD_E_INVAL
    assert _create(lib, None, kc)[0] == lib.SHARD_E_INVAL
    assert _create(lib, mc, lib.KvCfg(0, 64, 16, 0))[0] == lib.SHARD_E_INVAL
    assert _create(lib, mc, lib.KvCfg(1, 64, 0, 0))[0] == lib.SHARD_E_INVAL
    rc, msg = _create(lib, mc, kc, 0, 1, None)
    assert rc == lib.SHARD_E_INVAL and "null weights" in msg
    w = (lib.LayerWeights * 1)()          # all-null tensors
    rc, msg = _create(lib, mc, kc, 0, 1, w)
    assert rc == lib.SHARD_E_INVAL and "null tensor" in msg


def test_page_index_by_multiply_high_is_exact():
    """The kernels find a token's page as mulhi(u, ceil(2^32 / page)); that equals u // page
    for every position the library admits (u * page < 2^32, enforced at create)."""
    import random
    rng = random.Random(7)
    for page in list(range(2, 70)) + [127, 128, 129, 1000, 4096, 65535, 65536]:
        magic = ((1 << 32) + page - 1) // page
        assert magic < (1 << 32)
        lim = (1 << 32) // page
        us = [0, 1, page - 1, page, page + 1] + [lim - 1 - i for i in range(min(lim, 500))]
        us += [rng.randrange(lim) for _ in range(500)] + [k * page - 1 for k in range(1, 40) if k * page - 1 < lim]
        for u in us:
            assert (u * magic) >> 32 == u // page, (u, page)


def test_create_rejects_positions_beyond_the_page_index_range(lib):
    mc = lib.ModelCfg(**GOOD)
    rc, msg = _create(lib, mc, lib.KvCfg(1, 1 << 30, 16, 0))
    assert rc == lib.SHARD_E_INVAL and "2^32" in msg


def test_null_handles_are_errors_not_crashes(lib):
    h = lib.load()
    ids = (C.c_int32 * 1)(0)
    assert h.shard_destroy(None) == lib.SHARD_OK
    assert h.shard_seq_alloc(None, None) == lib.SHARD_E_INVAL
    assert h.shard_seq_free(None, 0) == lib.SHARD_E_INVAL
    assert h.shard_seq_len(None, 0) == lib.SHARD_E_INVAL
    assert h.shard_prefill(None, ids, 1, 1, None, None, None) == lib.SHARD_E_INVAL
    assert h.shard_decode(None, ids, 1, None, None, None) == lib.SHARD_E_INVAL
    assert h.shard_profile(None, 1, 1, 1, 1, None) == lib.SHARD_E_INVAL
    assert h.shard_timing_enable(None, 1) == lib.SHARD_E_INVAL


def test_synth_is_deterministic_and_bf16_rounding_is_rne():
    import numpy as np
    from paper_2405_14371_amd import synth
    cfg = synth.model_cfg("tiny")
    a = synth.layer_weights(cfg, 0, 1)["wq"]
    b = synth.layer_weights(cfg, 0, 1)["wq"]
    assert a.shape == (256, 256) and np.array_equal(a, b)
    assert not np.array_equal(a, synth.layer_weights(cfg, 0, 0)["wq"])
    assert abs(float(a.std()) - 0.02) < 1e-3
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -9, -(1.0 + 3 * 2 ** -9)], dtype=np.float32)
    # ties go to the even mantissa; others to nearest
    np.testing.assert_array_equal(synth.round_to_bf16(x),
                                  np.array([1.0, 1.0, 1.0 + 2 ** -6, 1.0, -(1.0 + 2 ** -7)], dtype=np.float32))
    assert synth.bf16_bits(np.array([1.0], dtype=np.float32))[0] == 0x3F80
    with pytest.raises(ValueError):
        synth.bf16_bits(np.array([1.0 + 2 ** -20], dtype=np.float32))


def test_boundary_from_plain_c(lib, tmp_path):
    """tests/c/abi_from_c.c: strict C99 against the three headers, linked with libshard.so; it
    checks a host-only entry point against a closed form and the error path without a GPU."""
    lib.load()
    libdir = os.path.dirname(lib.LIB_PATH)
    exe = str(tmp_path / "abi_from_c")
    cc = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                         os.path.join(ROOT, "tests", "c", "abi_from_c.c"), "-o", exe, "-L", libdir, "-lshard", "-lm",
                         "-Wl,-rpath," + libdir], capture_output=True, text=True)
    assert cc.returncode == 0, cc.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert run.returncode == 0 and run.stdout.strip() == "ok", (run.returncode, run.stdout, run.stderr)
