"""ctypes binding of libarkv's C ABI (include/arkv.h): argument marshalling only.

Functions have the names of the C entry points.  Device tensors are torch tensors (bf16 / fp32,
contiguous, on the GPU); the binding passes their data pointers and the current torch stream.
There is no fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ARKV_LIBRARY") or os.path.join(_HERE, "libarkv.so")

OK, EINVAL, ESTATE, ENOMEM, EHIP, EUNSUPPORTED, ESCRATCH = 0, -1, -2, -3, -4, -5, -6
STATE_ORIGINAL, STATE_QUANTIZED, STATE_EVICTED = 0, 1, 2

EXPORTED = [
    "arkv_config_default", "arkv_cache_create", "arkv_cache_destroy", "arkv_cache_reset",
    "arkv_prefill_stats", "arkv_prefill_stats_lse", "arkv_prefill_attention", "arkv_oq_ratio", "arkv_budget_counts", "arkv_prefill_commit",
    "arkv_decode_step", "arkv_decode_step_static", "arkv_decode_step_layers", "arkv_cache_counters", "arkv_cache_export",
    "arkv_debug_last_tailor_scores", "arkv_debug_last_out_f32", "arkv_debug_prefill_attention_f32", "arkv_cache_progress",
    "arkv_debug_time_attend", "arkv_debug_attend_time", "arkv_debug_set_launch_shape", "arkv_debug_split_range", "arkv_debug_phase_trace",
    "arkv_strerror",
    "arkv_last_hip_error",
]


class arkv_config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
        ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("capacity_tokens", C.c_int32),
        ("window", C.c_int32), ("alpha", C.c_float), ("gamma", C.c_float), ("tau", C.c_float * 3),
        ("quant_bits", C.c_int32), ("group_size", C.c_int32), ("tailor_policy", C.c_int32),
        ("budget_mode", C.c_int32),
    ]


class ArkvError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = f"{where}: {strerror(code)} ({code})"
        if code == EHIP:
            msg += ": " + last_hip_error()
        super().__init__(msg)


_lib = None


def load():
    """Loads libarkv.so once.  Raises if it has not been built (python -m paper_2603_08727_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build(); "
                           "there is no CPU fallback for the HIP path")
    lib = C.CDLL(LIB_PATH)
    vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
    P = C.POINTER
    sig = {
        "arkv_config_default": (C.c_int, [P(arkv_config)]),
        "arkv_cache_create": (C.c_int, [P(arkv_config), P(vp)]),
        "arkv_cache_destroy": (C.c_int, [vp]),
        "arkv_cache_reset": (C.c_int, [vp, i32]),
        "arkv_prefill_stats": (C.c_int, [vp, i32, vp, vp, i32, f32, vp, vp]),
        "arkv_prefill_stats_lse": (C.c_int, [vp, i32, vp, vp, i32, f32, vp, vp, vp]),
        "arkv_oq_ratio": (C.c_int, [vp, i32, i32, vp, vp]),
        "arkv_budget_counts": (C.c_int, [P(arkv_config), f32, P(i32), P(i32), P(i32)]),
        "arkv_prefill_commit": (C.c_int, [vp, i32, vp, vp, i32, vp, vp]),
        "arkv_decode_step": (C.c_int, [vp, i32, vp, vp, vp, f32, vp, vp]),
        "arkv_decode_step_static": (C.c_int, [vp, i32, vp, vp, vp, f32, vp, vp]),
        "arkv_decode_step_layers": (C.c_int, [vp, i32, i32, vp, vp, vp, vp, vp, vp]),
        "arkv_cache_counters": (C.c_int, [vp, i32, vp, vp, vp, vp]),
        "arkv_cache_export": (C.c_int, [vp, i32, i32] + [vp] * 13),
        "arkv_debug_last_tailor_scores": (C.c_int, [vp, i32, i32, vp, vp, vp]),
        "arkv_debug_last_out_f32": (C.c_int, [vp, i32, vp]),
        "arkv_debug_prefill_attention_f32": (C.c_int, [vp, vp]),
        "arkv_cache_progress": (C.c_int, [vp, i32, P(i32), P(i32), P(i32)]),
        "arkv_debug_set_launch_shape": (C.c_int, [vp, i32, i32, i32]),
        "arkv_debug_time_attend": (C.c_int, [vp, i32]),
        "arkv_debug_attend_time": (C.c_int, [vp, P(C.c_double), P(C.c_int64)]),
        "arkv_debug_phase_trace": (C.c_int, [i32, vp, i32]),
        "arkv_strerror": (C.c_char_p, [C.c_int]),
        "arkv_last_hip_error": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().arkv_strerror(code).decode()


def last_hip_error() -> str:
    return load().arkv_last_hip_error().decode()


def _check(code, where):
    if code != OK:
        raise ArkvError(code, where)


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _dev_ptr(t, dtype=None):
    import torch
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous GPU tensors"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


# ---- entry points, same names as the C ABI ---------------------------------------------------

def arkv_config_default(**overrides) -> arkv_config:
    cfg = arkv_config()
    _check(load().arkv_config_default(C.byref(cfg)), "arkv_config_default")
    for k, v in overrides.items():
        if k == "tau":
            cfg.tau = (C.c_float * 3)(*v)
        else:
            setattr(cfg, k, v)
    return cfg


def arkv_cache_create(cfg: arkv_config):
    h = C.c_void_p()
    _check(load().arkv_cache_create(C.byref(cfg), C.byref(h)), "arkv_cache_create")
    return h


def arkv_cache_destroy(cache):
    _check(load().arkv_cache_destroy(cache), "arkv_cache_destroy")


def arkv_cache_reset(cache, layer=-1):
    _check(load().arkv_cache_reset(cache, layer), "arkv_cache_reset")


def arkv_prefill_stats(cache, layer, q_win, k, T, softmax_scale, stats):
    import torch
    _check(load().arkv_prefill_stats(cache, layer, _dev_ptr(q_win, torch.bfloat16), _dev_ptr(k, torch.bfloat16),
                                     T, softmax_scale, _dev_ptr(stats, torch.float32), _stream()),
           "arkv_prefill_stats")


def arkv_prefill_stats_lse(cache, layer, q_win, k, T, softmax_scale, lse, stats):
    import torch
    _check(load().arkv_prefill_stats_lse(cache, layer, _dev_ptr(q_win, torch.bfloat16), _dev_ptr(k, torch.bfloat16),
                                         T, softmax_scale, _dev_ptr(lse, torch.float32),
                                         _dev_ptr(stats, torch.float32), _stream()),
           "arkv_prefill_stats_lse")


def arkv_prefill_attention(cache, layer, q, k, v, T_q, T, softmax_scale, out, stats=None):
    import torch
    lib = load()
    lib.arkv_prefill_attention.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                           C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.arkv_prefill_attention.restype = C.c_int
    _check(lib.arkv_prefill_attention(cache, layer, _dev_ptr(q, torch.bfloat16), _dev_ptr(k, torch.bfloat16),
                                      _dev_ptr(v, torch.bfloat16), T_q, T, softmax_scale,
                                      _dev_ptr(out, torch.bfloat16),
                                      None if stats is None else _dev_ptr(stats, torch.float32), _stream()),
           "arkv_prefill_attention")


def arkv_oq_ratio(stats: np.ndarray, tau) -> np.ndarray:
    stats = np.ascontiguousarray(stats, dtype=np.float32)
    L, B, three = stats.shape
    assert three == 3
    rho = np.empty((L, B), dtype=np.float32)
    t = np.asarray(tau, dtype=np.float32)
    _check(load().arkv_oq_ratio(_np_ptr(stats), L, B, _np_ptr(t), _np_ptr(rho)), "arkv_oq_ratio")
    return rho


def arkv_budget_counts(cfg: arkv_config, rho: float):
    a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load().arkv_budget_counts(C.byref(cfg), rho, C.byref(a), C.byref(b), C.byref(c)), "arkv_budget_counts")
    return a.value, b.value, c.value


def arkv_prefill_commit(cache, layer, k, v, T, rho):
    import torch
    rho = np.ascontiguousarray(rho, dtype=np.float32)
    _check(load().arkv_prefill_commit(cache, layer, _dev_ptr(k, torch.bfloat16), _dev_ptr(v, torch.bfloat16), T,
                                      _np_ptr(rho), _stream()), "arkv_prefill_commit")


def arkv_decode_step(cache, layer, q, k_new, v_new, softmax_scale, out):
    import torch
    bf = torch.bfloat16
    _check(load().arkv_decode_step(cache, layer, _dev_ptr(q, bf), _dev_ptr(k_new, bf), _dev_ptr(v_new, bf),
                                   softmax_scale, _dev_ptr(out, bf), _stream()), "arkv_decode_step")


def arkv_decode_step_static(cache, layer, q, k_new, v_new, softmax_scale, out):
    import torch
    bf = torch.bfloat16
    _check(load().arkv_decode_step_static(cache, layer, _dev_ptr(q, bf), _dev_ptr(k_new, bf), _dev_ptr(v_new, bf),
                                          softmax_scale, _dev_ptr(out, bf), _stream()), "arkv_decode_step_static")


def arkv_decode_step_layers(cache, layer_begin, n, q, k_new, v_new, softmax_scale, out):
    import torch
    bf = torch.bfloat16
    sc = np.ascontiguousarray(softmax_scale, dtype=np.float32)
    assert sc.shape == (n,)
    _check(load().arkv_decode_step_layers(cache, layer_begin, n, _dev_ptr(q, bf), _dev_ptr(k_new, bf),
                                          _dev_ptr(v_new, bf), _np_ptr(sc), _dev_ptr(out, bf), _stream()),
           "arkv_decode_step_layers")


def arkv_cache_counters(cache, layer, n_units):
    no = np.empty(n_units, dtype=np.int32); nq = np.empty(n_units, dtype=np.int32)
    ne = np.empty(n_units, dtype=np.int32); lb = np.empty(n_units, dtype=np.int64)
    _check(load().arkv_cache_counters(cache, layer, _np_ptr(no), _np_ptr(nq), _np_ptr(ne), _np_ptr(lb)),
           "arkv_cache_counters")
    return no, nq, ne, lb


def arkv_cache_progress(cache, layer):
    a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load().arkv_cache_progress(cache, layer, C.byref(a), C.byref(b), C.byref(c)), "arkv_cache_progress")
    return a.value, b.value, c.value


def arkv_cache_export(cache, layer, cfg: arkv_config, rows=True, codes=True):
    """Returns a dict of NumPy arrays, tokens of every unit sorted by position (see arkv.h)."""
    U = cfg.batch * cfg.n_kv_heads
    d = cfg.head_dim
    # token mode: at most N live tokens; byte mode: N bf16 rows' worth of bytes can hold more packed tokens
    MT = cfg.capacity_tokens + (arkv_budget_counts(cfg, 0.0)[2] if cfg.budget_mode == 1 else 0)
    CB, NG = d * cfg.quant_bits // 8, (1 if cfg.quant_bits == 8 else d // 32)
    out = dict(
        n_live=np.zeros(U, np.int32), pos=np.full((U, MT), -1, np.int32), state=np.full((U, MT), 255, np.uint8),
        s1=np.zeros((U, MT), np.float32), s2=np.zeros((U, MT), np.float32),
        rows_k=np.zeros((U, MT, d), np.uint16) if rows else None,
        rows_v=np.zeros((U, MT, d), np.uint16) if rows else None,
        codes_k=np.zeros((U, MT, CB), np.uint8) if codes else None,
        codes_v=np.zeros((U, MT, CB), np.uint8) if codes else None,
        scale_k=np.zeros((U, MT, NG), np.uint16) if codes else None,
        zero_k=np.zeros((U, MT, NG), np.uint16) if codes else None,
        scale_v=np.zeros((U, MT, NG), np.uint16) if codes else None,
        zero_v=np.zeros((U, MT, NG), np.uint16) if codes else None,
    )
    order = ["n_live", "pos", "state", "s1", "s2", "rows_k", "rows_v", "codes_k", "codes_v",
             "scale_k", "zero_k", "scale_v", "zero_v"]
    _check(load().arkv_cache_export(cache, layer, MT, *[_np_ptr(out[k]) for k in order]), "arkv_cache_export")
    return out


def arkv_debug_last_tailor_scores(cache, layer, n_units, max_tokens):
    cnt = np.empty(n_units, np.int32)
    pos = np.empty((n_units, max_tokens), np.int32)
    sc = np.empty((n_units, max_tokens), np.float32)
    _check(load().arkv_debug_last_tailor_scores(cache, layer, max_tokens, _np_ptr(cnt), _np_ptr(pos), _np_ptr(sc)),
           "arkv_debug_last_tailor_scores")
    return cnt, pos, sc


def arkv_debug_last_out_f32(cache, layer, shape):
    out = np.empty(shape, np.float32)
    _check(load().arkv_debug_last_out_f32(cache, layer, _np_ptr(out)), "arkv_debug_last_out_f32")
    return out


def arkv_debug_prefill_attention_f32(cache, out_f32=None):
    """out_f32: GPU fp32 tensor that later arkv_prefill_attention calls also fill, or None to switch it off."""
    import torch
    _check(load().arkv_debug_prefill_attention_f32(cache, None if out_f32 is None else _dev_ptr(out_f32, torch.float32)),
           "arkv_debug_prefill_attention_f32")


def arkv_debug_set_launch_shape(cache, wg_target=0, packed_weight=0, prefill_chunk=0):
    _check(load().arkv_debug_set_launch_shape(cache, wg_target, packed_weight, prefill_chunk),
           "arkv_debug_set_launch_shape")


def arkv_debug_time_attend(cache, enable: bool):
    _check(load().arkv_debug_time_attend(cache, 1 if enable else 0), "arkv_debug_time_attend")


def arkv_debug_attend_time(cache):
    ms, n = C.c_double(), C.c_int64()
    _check(load().arkv_debug_attend_time(cache, C.byref(ms), C.byref(n)), "arkv_debug_attend_time")
    return ms.value, n.value


def arkv_debug_phase_trace(which: int, n_rows: int = 1):
    """In-kernel timestamps of the latest launches (profiling builds only; ARKV_EUNSUPPORTED otherwise):
    a uint64 array [n_rows][8] for which = 0 (decode phases) or 1 (merge phases), [4] for which = 2."""
    import numpy as np
    buf = np.zeros((max(n_rows, 1), 8), dtype=np.uint64)
    _check(load().arkv_debug_phase_trace(which, buf.ctypes.data_as(C.c_void_p), n_rows), "arkv_debug_phase_trace")
    return buf.reshape(-1)[:4] if which == 2 else buf


MEASURE_LIB_PATH = os.environ.get("ARKV_MEASURE_LIBRARY") or os.path.join(_HERE, "libarkv_measure.so")
MEASURE_EXPORTED = ["arkv_measure_stream_read"]
_mlib = None


def load_measure():
    """libarkv_measure.so (include/arkv_measure.h): bandwidth measurement kernels, separate from the product."""
    global _mlib
    if _mlib is None:
        if not os.path.exists(MEASURE_LIB_PATH):
            raise RuntimeError(f"{MEASURE_LIB_PATH} is missing: build it with `python -m paper_2603_08727_amd.build`")
        _mlib = C.CDLL(MEASURE_LIB_PATH)
        _mlib.arkv_measure_stream_read.restype = C.c_int
        _mlib.arkv_measure_stream_read.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_int32, C.c_int32, C.c_void_p,
                                                   C.POINTER(C.c_float)]
    return _mlib


def arkv_measure_stream_read(buf, bytes_per_launch: int, launches: int, pattern: int = 0) -> float:
    """Average microseconds per launch of a plain streaming read over the GPU tensor `buf`
    (pattern 0: coalesced; 1: the attention kernel's key-operand layout; 2: plain copy, buf is modified)."""
    us = C.c_float()
    nbytes = buf.numel() * buf.element_size()
    rc = load_measure().arkv_measure_stream_read(_dev_ptr(buf), nbytes, bytes_per_launch, launches, pattern, _stream(),
                                                 C.byref(us))
    if rc != 0:
        raise RuntimeError(f"arkv_measure_stream_read failed with code {rc}")
    return us.value


def arkv_debug_split_range(n_original, n_quantized, packed_weight, n_splits, split):
    r = (C.c_int32 * 4)()
    lib = load()
    lib.arkv_debug_split_range.argtypes = [C.c_int32] * 5 + [C.POINTER(C.c_int32)]
    lib.arkv_debug_split_range.restype = C.c_int
    _check(lib.arkv_debug_split_range(n_original, n_quantized, packed_weight, n_splits, split, r), "arkv_debug_split_range")
    return tuple(r)
