"""ctypes binding of include/taskkv.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

F32, BF16 = 0, 1
PACK_SELECTIVE, PACK_NO_CACHE, PACK_COMPRESSED = 0, 1, 2
CHUNK_TOKENS = 512

EXPORTED_SYMBOLS = [
    "taskkv_create", "taskkv_destroy", "taskkv_strerror", "taskkv_workspace_bytes",
    "taskkv_cache_tokens", "taskkv_hetero_head_count", "taskkv_middle_budget", "taskkv_separate",
    "taskkv_compress", "taskkv_decode_attn", "taskkv_cache_export", "taskkv_last_async_error",
    "taskkv_profile_enable", "taskkv_profile_read", "taskkv_set_screening", "taskkv_set_stream_skew",
    "taskkv_set_stats_engine", "taskkv_stack_rebase", "taskkv_decode_attn_layers",
    "taskkv_decode_attn_static", "taskkv_layer_plan",
]


class TaskKVError(RuntimeError):
    pass


class LayerCfg(C.Structure):
    """Mirror of taskkv_layer_cfg."""
    _fields_ = [(n, C.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "ctx_len", "obs_window", "top_t", "n_sink",
        "n_recent", "n_middle", "n_hetero", "add_centre_head", "pool_kernel", "pack_mode", "dtype")] + [
        ("softmax_scale", C.c_float)]

    def __init__(self, **kw):
        super().__init__()
        self.pool_kernel = 1
        self.obs_window = 32
        self.top_t = 256
        for k, v in kw.items():
            if k not in dict(self._fields_):
                raise TypeError(f"unknown cfg field {k}")
            setattr(self, k, v)


def library_path() -> str:
    """In-tree libtaskkv.so, or the file named by TASKKV_LIBRARY."""
    return os.environ.get("TASKKV_LIBRARY") or os.path.join(
        os.path.dirname(os.path.abspath(__file__)), "libtaskkv.so")


_LIB = None


def load_library():
    """dlopen the in-tree libtaskkv.so; raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise TaskKVError(f"{path} is missing: build it first "
                          "(python -c 'import __graft_entry__ as g; g.build()'); there is no fallback")
    lib = C.CDLL(path)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    cfgp = C.POINTER(LayerCfg)
    lib.taskkv_create.argtypes = [C.POINTER(vp), C.c_int, sz]
    lib.taskkv_create.restype = C.c_int
    lib.taskkv_destroy.argtypes = [vp]
    lib.taskkv_destroy.restype = None
    lib.taskkv_strerror.argtypes = [C.c_int]
    lib.taskkv_strerror.restype = C.c_char_p
    lib.taskkv_workspace_bytes.argtypes = [cfgp, i32]
    lib.taskkv_workspace_bytes.restype = sz
    lib.taskkv_cache_tokens.argtypes = [cfgp, i32]
    lib.taskkv_cache_tokens.restype = i64
    lib.taskkv_hetero_head_count.argtypes = [i32, C.c_double, i32, i32, i32]
    lib.taskkv_hetero_head_count.restype = i32
    lib.taskkv_middle_budget.argtypes = [i64, i32, i32, i32, i32, i32]
    lib.taskkv_middle_budget.restype = i32
    lib.taskkv_layer_plan.argtypes = [i32, C.c_double, i32, i32, C.c_double, i32, i32, i32, C.POINTER(i32),
                                      C.POINTER(i32)]
    lib.taskkv_layer_plan.restype = C.c_int
    lib.taskkv_separate.argtypes = [vp, cfgp] + [vp] * 8
    lib.taskkv_separate.restype = C.c_int
    lib.taskkv_compress.argtypes = [vp, cfgp, vp, vp, vp, vp, vp, vp, i64, i32, vp, vp, vp, vp]
    lib.taskkv_compress.restype = C.c_int
    lib.taskkv_decode_attn.argtypes = [vp, cfgp, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp]
    lib.taskkv_decode_attn.restype = C.c_int
    lib.taskkv_stack_rebase.argtypes = [vp, i32, i32, vp, C.POINTER(i64), vp, vp]
    lib.taskkv_stack_rebase.restype = C.c_int
    lib.taskkv_decode_attn_layers.argtypes = [vp, cfgp, i32, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp]
    lib.taskkv_decode_attn_layers.restype = C.c_int
    lib.taskkv_decode_attn_static.argtypes = [cfgp, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp, vp]
    lib.taskkv_decode_attn_static.restype = C.c_int
    lib.taskkv_cache_export.argtypes = [vp, cfgp, vp, vp, i64, vp, vp, vp, vp]
    lib.taskkv_cache_export.restype = C.c_int
    lib.taskkv_last_async_error.argtypes = [vp, vp]
    lib.taskkv_last_async_error.restype = C.c_int
    lib.taskkv_set_screening.argtypes = [vp, C.c_int]
    lib.taskkv_set_screening.restype = C.c_int
    lib.taskkv_set_stats_engine.argtypes = [vp, C.c_int]
    lib.taskkv_set_stats_engine.restype = C.c_int
    lib.taskkv_set_stream_skew.argtypes = [vp, C.c_int]
    lib.taskkv_set_stream_skew.restype = C.c_int
    lib.taskkv_profile_enable.argtypes = [vp, C.c_int]
    lib.taskkv_profile_enable.restype = C.c_int
    lib.taskkv_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.taskkv_profile_read.restype = C.c_int
    _LIB = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise TaskKVError(f"{what}: {load_library().taskkv_strerror(rc).decode()} ({rc})")


def _ptr(t, dtype=None, allow_none=False):
    """Device pointer of a contiguous CUDA/HIP torch tensor."""
    if t is None:
        if allow_none:
            return None
        raise TaskKVError("tensor argument is None")
    if not t.is_cuda or not t.is_contiguous():
        raise TaskKVError("tensor arguments must be contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise TaskKVError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _elem(cfg: LayerCfg):
    import torch
    return torch.float32 if cfg.dtype == F32 else torch.bfloat16


def taskkv_strerror(status: int) -> str:
    return load_library().taskkv_strerror(status).decode()


def taskkv_create(device_id: int, workspace_bytes: int) -> C.c_void_p:
    ctx = C.c_void_p()
    _check(load_library().taskkv_create(C.byref(ctx), device_id, workspace_bytes), "taskkv_create")
    return ctx


def taskkv_destroy(ctx) -> None:
    load_library().taskkv_destroy(ctx)


def taskkv_workspace_bytes(cfg: LayerCfg, reserve_decode_tokens: int) -> int:
    n = load_library().taskkv_workspace_bytes(C.byref(cfg), reserve_decode_tokens)
    if n == 0:
        raise TaskKVError("taskkv_workspace_bytes: invalid cfg")
    return n


def taskkv_cache_tokens(cfg: LayerCfg, reserve_decode_tokens: int) -> int:
    n = load_library().taskkv_cache_tokens(C.byref(cfg), reserve_decode_tokens)
    if n < 0:
        raise TaskKVError("taskkv_cache_tokens: invalid cfg")
    return n


def taskkv_hetero_head_count(n_heads, beta, m_top, layer, n_layers) -> int:
    return load_library().taskkv_hetero_head_count(n_heads, beta, m_top, layer, n_layers)


def taskkv_middle_budget(layer_budget_tokens, ctx_len, n_heads, n_hetero, n_sink, n_recent) -> int:
    return load_library().taskkv_middle_budget(layer_budget_tokens, ctx_len, n_heads, n_hetero, n_sink,
                                               n_recent)


def taskkv_layer_plan(n_heads, beta, m_top, n_layers, budget_frac, ctx_len, n_sink, n_recent):
    """[(n_hetero, n_middle)] of every layer of a stack under one budget (Eq. 16-17)."""
    f, k = (C.c_int32 * n_layers)(), (C.c_int32 * n_layers)()
    _check(load_library().taskkv_layer_plan(n_heads, beta, m_top, n_layers, budget_frac, ctx_len, n_sink,
                                            n_recent, f, k), "taskkv_layer_plan")
    return list(zip(list(f), list(k)))


def taskkv_separate(ctx, cfg, q_win, k, v, scores, sem_vec, dist, hetero_mask, stream=None) -> None:
    import torch
    e = _elem(cfg)
    _check(load_library().taskkv_separate(
        ctx, C.byref(cfg), _ptr(q_win, e), _ptr(k, e), _ptr(v, e), _ptr(scores, torch.float64),
        _ptr(sem_vec, torch.float64), _ptr(dist, torch.float64), _ptr(hetero_mask, torch.uint8),
        _stream(stream)), "taskkv_separate")


def taskkv_compress(ctx, cfg, k, v, scores, hetero_mask, k_cache, v_cache, capacity_tokens,
                    reserve_decode_tokens, offsets, lens, kept_idx, stream=None) -> None:
    import torch
    e = _elem(cfg)
    _check(load_library().taskkv_compress(
        ctx, C.byref(cfg), _ptr(k, e), _ptr(v, e), _ptr(scores, torch.float64),
        _ptr(hetero_mask, torch.uint8), _ptr(k_cache, e), _ptr(v_cache, e), capacity_tokens,
        reserve_decode_tokens, _ptr(offsets, torch.int64), _ptr(lens, torch.int32),
        _ptr(kept_idx, torch.int32, allow_none=True), _stream(stream)), "taskkv_compress")


def taskkv_decode_attn(ctx, cfg, q, k_new, v_new, k_cache, v_cache, capacity_tokens, offsets, lens, out,
                       stream=None) -> None:
    import torch
    e = _elem(cfg)
    _check(load_library().taskkv_decode_attn(
        ctx, C.byref(cfg), _ptr(q, e), _ptr(k_new, e, allow_none=True), _ptr(v_new, e, allow_none=True),
        _ptr(k_cache, e), _ptr(v_cache, e), capacity_tokens, _ptr(offsets, torch.int64),
        _ptr(lens, torch.int32), _ptr(out, torch.float32), _stream(stream)), "taskkv_decode_attn")


def taskkv_decode_attn_static(cfg, q, k_new, v_new, k_cache, v_cache, capacity_tokens, offsets, lens, out,
                              async_flag=None, stream=None) -> None:
    """taskkv_decode_attn without a ctx: scratch memory is the library's own fixed device array."""
    import torch
    e = _elem(cfg)
    _check(load_library().taskkv_decode_attn_static(
        C.byref(cfg), _ptr(q, e), _ptr(k_new, e, allow_none=True), _ptr(v_new, e, allow_none=True),
        _ptr(k_cache, e), _ptr(v_cache, e), capacity_tokens, _ptr(offsets, torch.int64),
        _ptr(lens, torch.int32), _ptr(out, torch.float32), _ptr(async_flag, torch.int32, allow_none=True),
        _stream(stream)), "taskkv_decode_attn_static")


def taskkv_stack_rebase(ctx, n_layers, units_per_layer, layer_offsets, layer_capacity_tokens, stacked_offsets,
                        stream=None) -> None:
    import torch
    caps = (C.c_int64 * n_layers)(*[int(c) for c in layer_capacity_tokens])
    _check(load_library().taskkv_stack_rebase(
        ctx, n_layers, units_per_layer, _ptr(layer_offsets, torch.int64), caps,
        _ptr(stacked_offsets, torch.int64), _stream(stream)), "taskkv_stack_rebase")


def taskkv_decode_attn_layers(ctx, cfg, n_layers, q, k_new, v_new, k_cache, v_cache, capacity_tokens, offsets,
                              lens, out, stream=None) -> None:
    import torch
    e = _elem(cfg)
    _check(load_library().taskkv_decode_attn_layers(
        ctx, C.byref(cfg), n_layers, _ptr(q, e), _ptr(k_new, e, allow_none=True),
        _ptr(v_new, e, allow_none=True), _ptr(k_cache, e), _ptr(v_cache, e), capacity_tokens,
        _ptr(offsets, torch.int64), _ptr(lens, torch.int32), _ptr(out, torch.float32), _stream(stream)),
        "taskkv_decode_attn_layers")


def taskkv_cache_export(ctx, cfg, k_cache, v_cache, capacity_tokens, offsets, k_rows, v_rows,
                        stream=None) -> None:
    import torch
    e = _elem(cfg)
    _check(load_library().taskkv_cache_export(
        ctx, C.byref(cfg), _ptr(k_cache, e), _ptr(v_cache, e), capacity_tokens,
        _ptr(offsets, torch.int64), _ptr(k_rows, e), _ptr(v_rows, e), _stream(stream)),
        "taskkv_cache_export")


def taskkv_last_async_error(ctx, stream=None) -> int:
    rc = load_library().taskkv_last_async_error(ctx, _stream(stream))
    if rc < 0:
        _check(rc, "taskkv_last_async_error")
    return rc


def taskkv_set_screening(ctx, mode: int) -> None:
    """0 = never, 1 = automatic (default), 2 = whenever the inputs allow."""
    _check(load_library().taskkv_set_screening(ctx, int(mode)), "taskkv_set_screening")


def taskkv_set_stats_engine(ctx, engine: int) -> None:
    """Row statistics of bf16 inputs: 1 = int8 digits (default), 0 = fp64 matrix instruction."""
    _check(load_library().taskkv_set_stats_engine(ctx, int(engine)), "taskkv_set_stats_engine")


def taskkv_set_stream_skew(ctx, skew: int) -> None:
    """Share (in 1/1024ths) that decode attention moves from waves on odd XCDs to even ones; 0 = equal."""
    _check(load_library().taskkv_set_stream_skew(ctx, int(skew)), "taskkv_set_stream_skew")


def taskkv_profile_enable(ctx, on) -> None:
    """0 / False = off, 1 / True = time the decode attention kernel, 2 = the separator's row-statistics kernel."""
    _check(load_library().taskkv_profile_enable(ctx, int(on)), "taskkv_profile_enable")


def taskkv_profile_read(ctx):
    """(total milliseconds, launches) of the profiled kernel since the last read."""
    ms, n = C.c_double(), C.c_int64()
    _check(load_library().taskkv_profile_read(ctx, C.byref(ms), C.byref(n)), "taskkv_profile_read")
    return ms.value, n.value
