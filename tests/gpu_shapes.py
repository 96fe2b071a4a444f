"""Every shape the GPU parity tests run, in one place.

tests/test_parity_gpu.py parametrises its oracle-parity test over CASES, and
tests/test_fullsize_gpu.py runs FULLSIZE; tests/test_variant_coverage.py (CPU only) asks
the library which kernel variant each launch of each case takes and fails when a variant in
the library's tables is reached by none of them.  No arithmetic of the method lives here.
"""
from __future__ import annotations

from dataclasses import dataclass, field

from paper_2405_14371_amd import synth


@dataclass(frozen=True)
class Case:
    name: str
    why: str
    cfg: dict
    dtype: str                 # "f32" | "bf16"
    B: int
    prefill: tuple             # prefill chunk lengths, in call order
    n_dec: int
    n_layers: int = 2
    seed: int = 0
    gains: bool = False
    page: int = 16
    max_seq_len: int = 0       # 0 = exactly what the case needs
    micro: int = 1             # > 1: that many independent sequences driven one call each (B = 1 per call)

    @property
    def id(self) -> str:
        return self.name


def tiny(**kw):
    return synth.model_cfg("tiny", **kw)


CASES = [
    Case("tiny-f32", "the tiny configuration: 2 layers, d 256, 4 heads x 64, FFN 688, batch 1, 32 + 16",
         tiny(), "f32", 1, (32,), 16),
    Case("tiny-bf16", "the same with bf16 weights and a half cache", tiny(), "bf16", 1, (32,), 16),
    Case("ragged-f32", "T and contexts that are multiples of no tile, gains != 1, 3-token pages",
         tiny(), "f32", 2, (37,), 5, seed=3, gains=True, page=3),
    Case("ragged-bf16", "the same in bf16", tiny(), "bf16", 2, (37,), 5, seed=3, gains=True, page=3),
    Case("gqa-f32", "grouped-query attention, head_dim 32, FFN 344",
         tiny(n_heads=8, n_kv_heads=2, head_dim=32, ffn_dim=344), "f32", 3, (45,), 4, seed=5, gains=True),
    Case("gqa-bf16", "the same in bf16", tiny(n_heads=8, n_kv_heads=2, head_dim=32, ffn_dim=344), "bf16", 3, (45,), 4,
         seed=5, gains=True),
    Case("one-token-prefill-page-1", "a prefill of one token, pages of one token", tiny(), "f32", 1, (1,), 3, n_layers=1, page=1),
    Case("dh128-batch16-f32", "dh = 128 and a decode batch of 16 (two passes of 8 rows)",
         tiny(d_model=512, n_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=1024), "f32", 16, (20,), 3, seed=7),
]
# bf16 decode batches above 4 rows: matrix-core projections, one pass per group of up to 16 sequences
# (17 and 40: a ragged last group); GQA, random gains
CASES += [Case(f"bf16-mfma-decode-B{B}", "bf16 batch > 4 on the matrix cores",
               tiny(d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=1024), "bf16", B, (19,), 4, seed=21, gains=True)
          for B in (5, 8, 9, 16, 17, 40)]
# bf16 batches above 4 whose widths are NOT multiples of 64: no matrix-core route, the streaming
# kernel carries 8 half-weight rows per pass (and a second, ragged pass at B = 11)
CASES += [Case(f"bf16-stream-8rows-ffn344-B{B}", "bf16 batch > 4, FFN 344: streaming kernel with 8 rows per pass",
               tiny(n_heads=8, n_kv_heads=2, head_dim=32, ffn_dim=344), "bf16", B, (21,), 3, seed=25, gains=True)
          for B in (5, 8, 11)]
CASES += [Case("bf16-stream-8rows-d200-B5", "bf16 batch of 5, d_model 200 (not a multiple of 64)",
               tiny(d_model=200, n_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=512), "bf16", 5, (18,), 3, seed=27, gains=True)]
# rows per workgroup of the matrix-core decode projections: N / 256 rounded up to even, at most 128,
# else two rounds: gate/up widths that come out as 18, 40, 58, 70, 90, 106, 120 and 2 x 80 rows
CASES += [Case(f"bf16-mfma-rows-ffn{ffn}", "2..8 row tiles per workgroup, with and without a partial last tile",
               tiny(d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=ffn), "bf16", 6, (8,), 2, n_layers=1, seed=33, gains=True)
          for ffn in (2240, 5120, 7424, 8960, 11520, 13440, 15360, 20480)]
# inner dimensions of 2048 and more (multiples of 256, not powers of two) with at most 64 rows per
# workgroup: weights through the LDS ring (1 to 4 row tiles, partial tiles, 9 k-steps barely past the ring)
CASES += [Case(f"bf16-mfma-ldsring-ffn{ffn}-B{B}", "batched decode projections through the LDS ring",
               tiny(d_model=2304, n_heads=16, n_kv_heads=4, head_dim=128, ffn_dim=ffn), "bf16", B, (4,), 2, n_layers=1, seed=61,
               gains=True)
          for ffn, B in ((2304, 6), (5120, 5), (7680, 16), (5120, 19))]
# half cache, dh 128, 4..16 query heads per KV head: grouped-query decode attention on the matrix cores
CASES += [Case(f"bf16-gqa-attn-h{hq}kv{hkv}-B{B}-T{T}-p{page}", "groups of 4, 6, 8, 16 heads; one token to past 1024 tokens",
               tiny(d_model=256, n_heads=hq, n_kv_heads=hkv, head_dim=128, ffn_dim=512), "bf16", B, (T,), 5, seed=41, gains=True,
               page=page)
          for hq, hkv, B, T, page in ((8, 2, 1, 37, 16), (8, 1, 6, 150, 16), (8, 1, 2, 300, 3), (16, 1, 3, 70, 16),
                                      (12, 2, 5, 33, 16), (16, 2, 1, 1, 1), (8, 2, 1, 1100, 16), (16, 1, 2, 1030, 16))]
# few output tiles and a long inner dimension: half O / down prefill projections as 3 or 4 K slices
CASES += [Case(f"bf16-prefill-splitk-B{B}-T{T}", "K = 2048 in 4 slices; K = 2368 = 37 k-steps, not divisible by 4",
               tiny(d_model=256, n_heads=16, n_kv_heads=4, head_dim=128, ffn_dim=2368), "bf16", B, (T,), 2, seed=57, gains=True)
          for B, T in ((2, 37), (1, 200), (3, 128))]
CASES += [
    Case("bf16-prefill-splitk-128x128-tiles", "256 tokens x 4096 features back to d_model: 64 tiles of 128 x 128, K = 2048 and 2368 in 4 slices",
         tiny(d_model=4096, n_heads=16, n_kv_heads=2, head_dim=128, ffn_dim=2368), "bf16", 1, (256,), 1, n_layers=1, seed=107, gains=True),
    Case("batch64-f32", "SHARD_MAX_BATCH sequences in one call, fp32: eight passes of 8 rows",
         tiny(d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=1024), "f32", 64, (3,), 2, n_layers=1, seed=73, gains=True),
    Case("batch64-bf16", "the same in bf16: four groups of 16 on the matrix cores",
         tiny(d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, ffn_dim=1024), "bf16", 64, (3,), 2, n_layers=1, seed=73, gains=True),
    Case("f32-prefill-two-k-slices", "512 tokens, width 2304: O and down have 144 tiles of 128 x 64 -> two K slices",
         tiny(d_model=2304, n_heads=16, n_kv_heads=4, head_dim=128, ffn_dim=2048), "f32", 1, (512,), 1, n_layers=1, seed=89, gains=True),
    Case("f32-prefill-192-row-tiles", "512 tokens x 12288 QKV rows and 22016 gate/up rows: the 192 x 64 and 192 x 128 tiles",
         tiny(d_model=64, n_heads=32, n_kv_heads=32, head_dim=128, ffn_dim=11008), "f32", 1, (512,), 1, n_layers=1, seed=79, gains=True),
    Case("16500-tokens-page-1", "block-table row longer than the prefill attention's LDS copy; a decode slice over more "
         "pages than its LDS cache", tiny(), "f32", 1, (16500,), 2, n_layers=1, seed=71, page=1),
    Case("d-model-8448-bf16", "rows wider than 8192 elements: the two-pass RMSNorm of the prefill",
         tiny(d_model=8448, n_heads=2, n_kv_heads=1, head_dim=64, ffn_dim=128), "bf16", 2, (5,), 2, n_layers=1, seed=109, gains=True),
    Case("300-tokens", "many key tiles and context splits", tiny(), "f32", 1, (300,), 3, n_layers=1, seed=9),
    Case("7b-width-f32", "full 7B layer shapes, a ragged row count, streaming decode", synth.model_cfg("7b"), "f32", 1, (72,), 4, seed=1),
    Case("7b-width-bf16", "the same in bf16", synth.model_cfg("7b"), "bf16", 1, (72,), 4, seed=1),
    # tile variants of the half GEMM that only large M x N reach; the inner dimension is kept short
    Case("bf16-prefill-192x256-tiles", "1024 tokens x (12288 QKV, 22016 gate/up) rows: 256 and 460 tiles of 192 x 256",
         tiny(d_model=128, n_heads=32, n_kv_heads=32, head_dim=128, ffn_dim=11008), "bf16", 1, (1024,), 1, n_layers=1, seed=91, gains=True),
    Case("bf16-prefill-384x128-tiles", "1152 tokens x 10240 QKV rows: 243 tiles of 384 x 128 (270 of 192 x 256 would need a second round)",
         tiny(d_model=128, n_heads=64, n_kv_heads=8, head_dim=128, ffn_dim=1024), "bf16", 1, (1152,), 1, n_layers=1, seed=103, gains=True),
    Case("bf16-prefill-2560-rows", "2 x 1280 tokens: the 256 x 256 tiles, row bands of 8 tiles and a second band",
         tiny(d_model=128, n_heads=16, n_kv_heads=16, head_dim=128, ffn_dim=5504), "bf16", 2, (1280,), 1, n_layers=1, seed=93, gains=True),
    Case("bf16-prefill-k-not-64", "inner dimensions 200 and 344: the register-staged half GEMM",
         tiny(d_model=200, n_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=344), "bf16", 2, (150,), 2, seed=95, gains=True),
    Case("f32-prefill-k-not-16", "inner dimensions 200 and 344 (multiples of 8 only): the register-staged fp32 GEMM",
         tiny(d_model=200, n_heads=4, n_kv_heads=2, head_dim=64, ffn_dim=344), "f32", 2, (150,), 2, seed=97, gains=True),
    Case("f32-prefill-reg-128x128", "2048 rows x 4096 / 5120 features with inner dimension 200: the large register-staged tiles",
         tiny(d_model=200, n_heads=24, n_kv_heads=4, head_dim=128, ffn_dim=2560), "f32", 2, (1024,), 1, n_layers=1, seed=101, gains=True),
    Case("bf16-prefill-reg-128x128", "the same in bf16: 512 tiles take the k-step-64 variant, 640 tiles the k-step-32 one",
         tiny(d_model=200, n_heads=24, n_kv_heads=4, head_dim=128, ffn_dim=2560), "bf16", 2, (1024,), 1, n_layers=1, seed=101, gains=True),
    Case("f32-prefill-k16-not-32", "inner dimension 240 (a multiple of 16, not 32)",
         tiny(d_model=240, n_heads=4, n_kv_heads=4, head_dim=64, ffn_dim=1008), "f32", 1, (300,), 1, n_layers=1, seed=99, gains=True),
]


def _sweep():
    """Seeded shapes: query blocks of 128 with ragged ends, key blocks of 32, contexts that start
    above zero (two prefill chunks), head sizes 64 / 128 (LDS-staged attention) and 32 (per-wave),
    K multiples and non-multiples of the direct-to-LDS k-step, page sizes that divide nothing."""
    import numpy as np
    rng = np.random.default_rng(2024)
    out = []
    for i in range(10):
        dh = int(rng.choice([32, 64, 128]))
        hkv = int(rng.choice([1, 2, 4]))
        hq = hkv * int(rng.choice([1, 2, 4]))
        d = int(rng.choice([128, 192, 256, 320]))
        ffn = int(rng.choice([344, 512, 688, 1000]))
        dtype = "f32" if i % 2 == 0 else "bf16"
        B, T0, T1 = int(rng.integers(1, 4)), int(rng.integers(1, 200)), int(rng.integers(1, 300))
        page = int(rng.choice([1, 5, 16, 64]))
        out.append(Case(f"sweep-{dtype}-d{d}-h{hq}x{dh}-kv{hkv}-T{T0}+{T1}-p{page}", "seeded sweep, two prefill chunks then decode",
                        tiny(d_model=d, n_heads=hq, n_kv_heads=hkv, head_dim=dh, ffn_dim=ffn), dtype, B, (T0, T1), 2,
                        seed=100 + i, gains=True, page=page))
    out.append(Case("sweep-f32-d256-h4x128-kv2-T130+259-p16", "seeded sweep", tiny(d_model=256, n_heads=4, n_kv_heads=2, head_dim=128, ffn_dim=688),
                    "f32", 2, (130, 259), 2, seed=120, gains=True))
    out.append(Case("sweep-bf16-d512-h8x128-kv1-T1+385-p1", "seeded sweep", tiny(d_model=512, n_heads=8, n_kv_heads=1, head_dim=128, ffn_dim=1000),
                    "bf16", 1, (1, 385), 2, seed=121, gains=True, page=1))
    return out


CASES += _sweep()

# the benchmark configurations at full size (stored oracle rows: tests/golden/)
FULLSIZE = [
    Case("c2", "7B layers 0-7, fp32, batch 1, 512 + 128", synth.model_cfg("7b"), "f32", 1, (512,), 128, n_layers=8),
    Case("c3", "7B, 32 layers, bf16, batch 1, 1024 + 256", synth.model_cfg("7b"), "bf16", 1, (1024,), 256, n_layers=32),
    Case("c4", "13B layers 0-19, bf16, eight micro-batches of one sequence, 256 + 128", synth.model_cfg("13b"), "bf16", 1, (256,), 128,
         n_layers=20, micro=8),
    Case("c4-fused", "the same eight sequences as one batch", synth.model_cfg("13b"), "bf16", 8, (256,), 128, n_layers=20),
    Case("c5", "70B layers 0-19, GQA, bf16, batch 16, 512 + 128", synth.model_cfg("70b"), "bf16", 16, (512,), 128, n_layers=20),
]


def projections(cfg: dict):
    """(name, N, K, residual epilogue) of the four projections of a layer."""
    d, hq, hkv, dh, f = (cfg[k] for k in ("d_model", "n_heads", "n_kv_heads", "head_dim", "ffn_dim"))
    return (("qkv", (hq + 2 * hkv) * dh, d, False), ("o", d, hq * dh, True), ("gateup", 2 * f, d, False), ("down", d, f, True))
