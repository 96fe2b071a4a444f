"""CPU only: which kernel variant every launch of every GPU parity case takes, asked of the
library's own selection code (include/shard_introspect.h), and that the cases leave no entry
of the variant tables unreached.  A variant nobody launches is a variant nobody compared with
the oracle."""
import pytest

from tests import gpu_shapes as S


def launches_of(lib, case):
    """(family, variant name) of every projection launch the case causes."""
    wd = lib.SHARD_F32 if case.dtype == "f32" else lib.SHARD_BF16
    out = set()
    for T in case.prefill:
        for _, N, K, resid in S.projections(case.cfg):
            name, _ = lib.variant_prefill_gemm(wd, case.B * T, N, K, resid)
            out.add(("prefill", name))
    if case.n_dec:
        for _, N, K, _ in S.projections(case.cfg):
            name, rows_per_pass, _ = lib.variant_decode_linear(case.cfg, wd, case.B, N, K)
            out.add(("decode", name))
            tail = case.B % rows_per_pass
            if tail:                    # the ragged last pass carries fewer rows
                if "mfma" in name:
                    out.add(("decode", name))
                else:
                    out.add(("decode", lib.variant_decode_linear(case.cfg, wd, tail, N, K)[0]))
    return out


def test_every_variant_in_the_tables_is_reached_by_a_parity_case(lib):
    reached = set()
    by_variant = {}
    for case in S.CASES + S.FULLSIZE:
        for fam, name in launches_of(lib, case):
            reached.add(name)
            by_variant.setdefault(name, []).append(case.name)
    tables = sum((lib.variant_names(f) for f in (lib.FAMILY_PREFILL_GEMM, lib.FAMILY_DECODE_STREAM, lib.FAMILY_DECODE_MFMA)), [])
    assert len(tables) == len(set(tables)) >= 30
    missing = [n for n in tables if n not in reached]
    assert not missing, f"variants no parity case launches: {missing}"
    # and the small cases alone (every row and step compared) reach all but the tiles only a
    # full-size shape can select
    small = set()
    for case in S.CASES:
        small |= {name for _, name in launches_of(lib, case)}
    only_fullsize = [n for n in tables if n not in small]
    assert only_fullsize == [], f"variants reached only at full size (sampled rows): {only_fullsize}"


@pytest.mark.parametrize("name,proj,want", [
    ("c2", "qkv", "f32 dma 192x64"), ("c2", "gateup", "f32 dma 192x128"), ("c2", "o", "f32 dma 128x128 split-k"),
    ("c3", "qkv", "f16 dma 192x256"), ("c3", "gateup", "f16 dma 192x256"), ("c3", "down", "f16 dma 128x128"),
    ("c5", "gateup", "f16 dma 256x256"),
])
def test_benchmark_shapes_land_on_the_variants_tuned_for_them(lib, name, proj, want):
    case = next(c for c in S.FULLSIZE if c.name == name)
    wd = lib.SHARD_F32 if case.dtype == "f32" else lib.SHARD_BF16
    N, K, resid = next((n, k, r) for p, n, k, r in S.projections(case.cfg) if p == proj)
    assert lib.variant_prefill_gemm(wd, case.B * case.prefill[0], N, K, resid)[0] == want


def test_decode_route_and_rows_per_workgroup(lib):
    """The 70B gate/up projection at batch 16 runs on the matrix cores with 112 rows per
    workgroup (57344 rows over two rounds of 256 workgroups); a batch of 4 streams."""
    c5 = next(c for c in S.FULLSIZE if c.name == "c5")
    name, rpp, rows = lib.variant_decode_linear(c5.cfg, lib.SHARD_BF16, 16, 2 * c5.cfg["ffn_dim"], c5.cfg["d_model"])
    assert name == "f16 mfma reg 7 tiles" and rpp == 16 and rows == 112
    name, rpp, rows = lib.variant_decode_linear(c5.cfg, lib.SHARD_BF16, 4, 2 * c5.cfg["ffn_dim"], c5.cfg["d_model"])
    assert name.startswith("f16 stream nb4") and rpp == 4
    assert lib.load().shard_variant_prefill_gemm(5, 1, 1, 1, 0, None) == -1
    assert lib.load().shard_variant_name(9, 0) is None


def test_fullsize_registry_mirrors_the_golden_workloads():
    from tests.golden import make_golden as G
    from paper_2405_14371_amd import synth
    for name, wl in G.WORKLOADS.items():
        c = next(c for c in S.FULLSIZE if c.name == name)
        assert c.cfg == synth.model_cfg(wl["model"]) and c.n_layers == wl["layers"] and c.dtype == wl["dtype"]
        assert c.prefill == (wl["T"],) and c.n_dec == wl["n_dec"]
        assert len(wl["seqs"]) <= c.B * c.micro


def test_golden_rows_cover_every_32_row_band_and_every_8th_step():
    from tests.golden import make_golden as G
    for wl in G.WORKLOADS.values():
        pre, dec = G.sample_rows(wl["T"], wl["n_dec"])
        assert {r // 32 for r in pre} == set(range((wl["T"] + 31) // 32))
        assert {r % 32 for r in pre} == set(range(32)) or wl["T"] < 1024
        assert set(range(0, wl["n_dec"], 8)) <= set(dec) and wl["n_dec"] - 1 in dec
