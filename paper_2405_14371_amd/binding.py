"""ctypes binding of libshard.so: the same entry points as include/shard.h, argument
marshalling only.  PyTorch supplies device buffers and streams; every step of the layer
runs in the library's HIP kernels.  There is no fallback: a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libshard.so")

SHARD_OK, SHARD_E_INVAL, SHARD_E_NOMEM, SHARD_E_KV_FULL, SHARD_E_STATE, SHARD_E_HIP, SHARD_E_RANGE = 0, -1, -2, -3, -4, -5, -6
SHARD_STATIC_SCRATCH_BYTES = 8 << 20
SHARD_F32, SHARD_BF16 = 0, 1
SHARD_MAX_BATCH = 64
KERNEL_CLASSES = ("decode_qkv", "decode_attn", "decode_o", "decode_gateup", "decode_down", "prefill_norm",
                  "prefill_qkv", "prefill_attn", "prefill_o", "prefill_gateup", "prefill_down")
K_COUNT = len(KERNEL_CLASSES)

class PlanProblem(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_devices", C.c_int32), ("t_comp", C.POINTER(C.c_double)),
                ("act_bytes", C.POINTER(C.c_double)), ("req_bytes", C.POINTER(C.c_double)),
                ("mem_bytes", C.POINTER(C.c_double)), ("bandwidth", C.POINTER(C.c_double))]


class PipelineProblem(C.Structure):
    _fields_ = [("n_stages", C.c_int32), ("n_micro", C.c_int32), ("n_decode", C.c_int32),
                ("t_prefill", C.POINTER(C.c_double)), ("t_decode", C.POINTER(C.c_double)),
                ("c_prefill", C.POINTER(C.c_double)), ("c_decode", C.POINTER(C.c_double)),
                ("c_return", C.c_double)]


EXPORTS = (
    "shard_create", "shard_destroy", "shard_seq_alloc", "shard_seq_free", "shard_seq_len",
    "shard_prefill", "shard_decode", "shard_decode_static", "shard_overflow", "shard_profile",
    "shard_timing_enable", "shard_timing_read",
    "shard_last_error", "shard_plan_latency", "shard_plan_throughput", "shard_plan_to_stages", "shard_simulate_pipeline",
    "shard_ends_create", "shard_ends_destroy", "shard_ends_embed", "shard_ends_logits", "shard_ends_argmax",
    "shard_variant_name", "shard_variant_prefill_gemm", "shard_variant_decode_linear", "shard_test_inject_launch_error",
)
FAMILY_PREFILL_GEMM, FAMILY_DECODE_STREAM, FAMILY_DECODE_MFMA = 0, 1, 2


class ModelCfg(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn_dim", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("weight_dtype", C.c_int32), ("act_dtype", C.c_int32)]


class KvCfg(C.Structure):
    _fields_ = [("max_seqs", C.c_int32), ("max_seq_len", C.c_int32), ("page_size", C.c_int32),
                ("max_batch_tokens", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "g_attn", "g_ffn")]


class LayerProfile(C.Structure):
    _fields_ = [("t_prefill_s", C.c_double), ("t_decode_s", C.c_double), ("t_avg_s", C.c_double),
                ("act_bytes_prefill", C.c_uint64), ("act_bytes_decode", C.c_uint64),
                ("weight_bytes", C.c_uint64), ("kv_bytes_per_token", C.c_uint64)]


class ShardError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libshard error {code}: {message}")
        self.code = code


_lib = None


def load():
    """Load libshard.so (built in-tree by build.py) and declare its signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2405_14371_amd.build` "
                           "(or __graft_entry__.build()) first; there is no CPU fallback")
    # PyTorch ships its own HIP runtime under the same soname as the system one; it must
    # be the first (and only) copy in the process, or torch finds no device afterwards.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32 = C.c_void_p, C.c_int32
    lib.shard_create.argtypes = [C.POINTER(vp), C.POINTER(ModelCfg), C.POINTER(KvCfg), i32, i32,
                                 C.POINTER(LayerWeights), i32]
    lib.shard_destroy.argtypes = [vp]
    lib.shard_seq_alloc.argtypes = [vp, C.POINTER(i32)]
    lib.shard_seq_free.argtypes = [vp, i32]
    lib.shard_seq_len.argtypes = [vp, i32]
    lib.shard_prefill.argtypes = [vp, C.POINTER(i32), i32, i32, vp, vp, vp]
    lib.shard_decode.argtypes = [vp, C.POINTER(i32), i32, vp, vp, vp]
    lib.shard_decode_static.argtypes = [vp, C.POINTER(i32), i32, vp, vp, vp]
    lib.shard_overflow.argtypes = [vp, i32, C.POINTER(i32)]
    lib.shard_profile.argtypes = [vp, i32, i32, i32, i32, C.POINTER(LayerProfile)]
    lib.shard_timing_enable.argtypes = [vp, i32]
    lib.shard_timing_read.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    lib.shard_plan_latency.argtypes = [C.POINTER(PlanProblem), C.POINTER(i32), C.POINTER(C.c_double)]
    lib.shard_plan_throughput.argtypes = [C.POINTER(PlanProblem), i32, C.POINTER(i32), C.POINTER(C.c_double)]
    dp = C.POINTER(C.c_double)
    lib.shard_plan_to_stages.argtypes = [i32, i32, C.POINTER(i32), dp, dp, dp, dp, dp, C.POINTER(i32), C.POINTER(i32),
                                         dp, dp, dp, dp, dp]
    lib.shard_simulate_pipeline.argtypes = [C.POINTER(PipelineProblem), i32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.shard_ends_create.argtypes = [C.POINTER(vp), C.POINTER(ModelCfg), i32, i32, vp, vp, vp, i32]
    lib.shard_ends_destroy.argtypes = [vp]
    lib.shard_ends_embed.argtypes = [vp, C.POINTER(i32), i32, vp, vp]
    lib.shard_ends_logits.argtypes = [vp, vp, i32, vp, vp]
    lib.shard_ends_argmax.argtypes = [vp, vp, i32, vp, vp]
    lib.shard_variant_name.argtypes = [i32, i32]
    lib.shard_variant_name.restype = C.c_char_p
    lib.shard_variant_prefill_gemm.argtypes = [i32, i32, i32, i32, i32, C.POINTER(i32)]
    lib.shard_variant_decode_linear.argtypes = [C.POINTER(ModelCfg), i32, i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    lib.shard_test_inject_launch_error.argtypes = [i32]
    lib.shard_test_inject_launch_error.restype = None
    lib.shard_last_error.argtypes = []
    lib.shard_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("shard_last_error", "shard_variant_name", "shard_test_inject_launch_error"):
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def last_error() -> str:
    return load().shard_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise ShardError(rc, last_error())
    return rc


def _ptr(t) -> int:
    """Raw pointer of a torch tensor, a numpy array or an int."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _ids(seq_ids):
    arr = (C.c_int32 * len(seq_ids))(*[int(i) for i in seq_ids])
    return arr, len(seq_ids)


def model_cfg(cfg: dict, weight_dtype: int) -> ModelCfg:
    return ModelCfg(cfg["d_model"], cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["ffn_dim"],
                    cfg["rms_eps"], cfg["rope_theta"], weight_dtype, SHARD_F32)


class Shard:
    """One shard on the current device.  `layers` is a list of dicts of host numpy arrays
    (float32 for SHARD_F32, uint16 bf16 bit patterns for SHARD_BF16; gains float32) or of
    torch device tensors of the matching element size (on_device=True)."""

    def __init__(self, cfg: dict, layers: list, layer_lo: int = 0, *, weight_dtype: int = SHARD_F32,
                 max_seqs: int = 1, max_seq_len: int = 2048, page_size: int = 16,
                 max_batch_tokens: int = 0, on_device: bool = False):
        self._h = C.c_void_p()
        self.cfg = dict(cfg)
        self.n_layers = len(layers)
        lib = load()
        mc = model_cfg(cfg, weight_dtype)
        kc = KvCfg(max_seqs, max_seq_len, page_size, max_batch_tokens)
        arr = (LayerWeights * max(1, len(layers)))()
        keep = []
        for i, lw in enumerate(layers):
            for name, _ in LayerWeights._fields_:
                t = lw[name]
                if isinstance(t, np.ndarray):
                    want = np.float32 if (name.startswith("g_") or weight_dtype == SHARD_F32) else np.uint16
                    if t.dtype != want:
                        raise TypeError(f"{name}: expected {want.__name__}, got {t.dtype}")
                    t = np.ascontiguousarray(t)
                keep.append(t)
                setattr(arr[i], name, _ptr(t))
        _check(lib.shard_create(C.byref(self._h), C.byref(mc), C.byref(kc), layer_lo, layer_lo + len(layers),
                                arr, 1 if on_device else 0))

    def close(self):
        if self._h:
            _check(load().shard_destroy(self._h))
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def seq_alloc(self) -> int:
        out = C.c_int32(-1)
        _check(load().shard_seq_alloc(self._h, C.byref(out)))
        return out.value

    def seq_free(self, seq_id: int) -> None:
        _check(load().shard_seq_free(self._h, seq_id))

    def seq_len(self, seq_id: int) -> int:
        return _check(load().shard_seq_len(self._h, seq_id))

    def prefill(self, seq_ids, T: int, x_in, x_out, stream: int = 0) -> None:
        ids, n = _ids(seq_ids)
        _check(load().shard_prefill(self._h, ids, n, T, _ptr(x_in), _ptr(x_out), stream))

    def decode(self, seq_ids, x_in, x_out, stream: int = 0) -> None:
        ids, n = _ids(seq_ids)
        _check(load().shard_decode(self._h, ids, n, _ptr(x_in), _ptr(x_out), stream))

    def decode_static(self, seq_ids, x_in, x_out, stream: int = 0) -> None:
        ids, n = _ids(seq_ids)
        _check(load().shard_decode_static(self._h, ids, n, _ptr(x_in), _ptr(x_out), stream))

    def overflow(self, clear: bool = False) -> bool:
        out = C.c_int32(0)
        _check(load().shard_overflow(self._h, 1 if clear else 0, C.byref(out)))
        return bool(out.value)

    def profile(self, B: int, T_prefill: int, n_decode: int, iters: int = 3) -> list:
        out = (LayerProfile * self.n_layers)()
        _check(load().shard_profile(self._h, B, T_prefill, n_decode, iters, out))
        return [{f: getattr(p, f) for f, _ in LayerProfile._fields_} for p in out]

    def timing_enable(self, on: bool = True) -> None:
        _check(load().shard_timing_enable(self._h, 1 if on else 0))

    def timing_read(self) -> dict:
        n = (C.c_int64 * K_COUNT)()
        s = (C.c_double * K_COUNT)()
        _check(load().shard_timing_read(self._h, n, s))
        return {KERNEL_CLASSES[k]: {"launches": n[k], "seconds": s[k]} for k in range(K_COUNT)}


class ShardEnds:
    """Embedding table and/or final norm + LM head on the current device (host numpy arrays:
    float32 for SHARD_F32, uint16 bf16 bit patterns for SHARD_BF16; g_final float32)."""

    def __init__(self, cfg: dict, vocab: int, *, tok_embeddings=None, g_final=None, lm_head=None,
                 weight_dtype: int = SHARD_F32, max_tokens: int = 4096):
        self._h = C.c_void_p()
        self.vocab = vocab
        mc = model_cfg(cfg, weight_dtype)
        keep = [None if t is None else np.ascontiguousarray(t) for t in (tok_embeddings, g_final, lm_head)]
        _check(load().shard_ends_create(C.byref(self._h), C.byref(mc), vocab, max_tokens,
                                        _ptr(keep[0]), _ptr(keep[1]), _ptr(keep[2]), 0))

    def close(self):
        if self._h:
            _check(load().shard_ends_destroy(self._h))
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def embed(self, token_ids, x_out, stream: int = 0) -> None:
        ids, n = _ids(token_ids)
        _check(load().shard_ends_embed(self._h, ids, n, _ptr(x_out), stream))

    def logits(self, x, n: int, logits_out, stream: int = 0) -> None:
        _check(load().shard_ends_logits(self._h, _ptr(x), n, _ptr(logits_out), stream))

    def argmax(self, logits, n: int, ids_out, stream: int = 0) -> None:
        _check(load().shard_ends_argmax(self._h, _ptr(logits), n, _ptr(ids_out), stream))


def pack_layers(layers: list, weight_dtype: int) -> list:
    """float32 host arrays from synth -> the element type the library expects."""
    from .synth import bf16_bits
    out = []
    for lw in layers:
        d = {}
        for k, v in lw.items():
            if k.startswith("g_") or weight_dtype == SHARD_F32:
                d[k] = np.ascontiguousarray(v, dtype=np.float32)
            else:
                d[k] = bf16_bits(v)
        out.append(d)
    return out


def variant_names(family: int) -> list:
    """All variant names of a family, in table order."""
    out, i = [], 0
    while True:
        name = load().shard_variant_name(family, i)
        if name is None:
            return out
        out.append(name.decode())
        i += 1


def variant_prefill_gemm(weight_dtype: int, M: int, N: int, K: int, residual_epilogue: bool):
    """shard_variant_prefill_gemm: (variant name, K slices)."""
    ks = C.c_int32(0)
    i = _check(load().shard_variant_prefill_gemm(weight_dtype, M, N, K, 1 if residual_epilogue else 0, C.byref(ks)))
    return load().shard_variant_name(FAMILY_PREFILL_GEMM, i).decode(), ks.value


def variant_decode_linear(cfg: dict, weight_dtype: int, B: int, N: int, K: int):
    """shard_variant_decode_linear: (variant name, rows per pass, weight rows per workgroup)."""
    mc = model_cfg(cfg, weight_dtype)
    fam, rpp, rows = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    i = _check(load().shard_variant_decode_linear(C.byref(mc), B, N, K, C.byref(fam), C.byref(rpp), C.byref(rows)))
    return load().shard_variant_name(fam.value, i).decode(), rpp.value, rows.value


def inject_launch_error(on: bool) -> None:
    load().shard_test_inject_launch_error(1 if on else 0)


def _plan_problem(prob: dict):
    dbl = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    arrs = [dbl(prob[k]) for k in ("t_comp", "act_bytes", "req_bytes", "mem_bytes", "bandwidth")]
    n, m = arrs[0].shape
    ptr = lambda a: a.ctypes.data_as(C.POINTER(C.c_double))
    return PlanProblem(n, m, *[ptr(a) for a in arrs]), arrs, n


def plan_latency(prob: dict):
    """shard_plan_latency: returns (total time of one token, device of each layer)."""
    pp, keep, n = _plan_problem(prob)
    dev = (C.c_int32 * n)()
    t = C.c_double()
    rc = load().shard_plan_latency(C.byref(pp), dev, C.byref(t))
    if rc:
        raise ShardError(rc, "no feasible placement" if rc == -2 else "bad planner arguments")
    return t.value, list(dev)


def plan_throughput(prob: dict, with_return_hop: bool = False):
    """shard_plan_throughput: returns (slowest stage time, device of each layer)."""
    pp, keep, n = _plan_problem(prob)
    dev = (C.c_int32 * n)()
    t = C.c_double()
    rc = load().shard_plan_throughput(C.byref(pp), 1 if with_return_hop else 0, dev, C.byref(t))
    if rc:
        raise ShardError(rc, "no feasible placement" if rc == -2 else "bad planner arguments")
    return t.value, list(dev)


def simulate_pipeline(t_prefill, t_decode, c_prefill, c_decode, c_return, n_micro, n_decode, no_bubbles):
    """shard_simulate_pipeline: returns (makespan in seconds, busy seconds per stage)."""
    dbl = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    tp, td, cp, cd = dbl(t_prefill), dbl(t_decode), dbl(c_prefill), dbl(c_decode)
    S = len(tp)
    ptr = lambda a: a.ctypes.data_as(C.POINTER(C.c_double)) if len(a) else None
    pp = PipelineProblem(S, n_micro, n_decode, ptr(tp), ptr(td), ptr(cp), ptr(cd), float(c_return))
    span = C.c_double()
    busy = (C.c_double * max(1, S))()
    rc = load().shard_simulate_pipeline(C.byref(pp), 1 if no_bubbles else 0, C.byref(span), busy)
    if rc:
        raise ShardError(rc, "bad pipeline problem")
    return span.value, list(busy)[:S]


def stages_of_plan(device_of_layer, t_prefill_layer, t_decode_layer, act_bytes_prefill, act_bytes_decode, bandwidth):
    """shard_plan_to_stages: collapse a throughput plan (one contiguous layer range per device)
    into the per-stage and per-link times shard_simulate_pipeline takes.  Per-layer times are
    [N][M] (layer, device), activation sizes [N], bandwidth [M][M] in bytes per second."""
    dbl = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    ptr = lambda a: a.ctypes.data_as(C.POINTER(C.c_double))
    tp, td, ap, ad, bw = (dbl(a) for a in (t_prefill_layer, t_decode_layer, act_bytes_prefill, act_bytes_decode, bandwidth))
    n, m = tp.shape
    dev = (C.c_int32 * n)(*[int(d) for d in device_of_layer])
    n_stages = C.c_int32(0)
    stage_dev = (C.c_int32 * n)()
    out = [np.zeros(n, dtype=np.float64) for _ in range(4)]
    c_ret = C.c_double(0.0)
    rc = load().shard_plan_to_stages(n, m, dev, ptr(tp), ptr(td), ptr(ap), ptr(ad), ptr(bw), C.byref(n_stages), stage_dev,
                                     ptr(out[0]), ptr(out[1]), ptr(out[2]), ptr(out[3]), C.byref(c_ret))
    if rc:
        raise ShardError(rc, "a device owns two separate layer ranges" if rc == -2 else "bad plan arguments")
    S = n_stages.value
    return dict(stages=list(stage_dev)[:S], t_prefill=out[0][:S].tolist(), t_decode=out[1][:S].tolist(),
                c_prefill=out[2][:S - 1].tolist(), c_decode=out[3][:S - 1].tolist(), c_return=c_ret.value)
