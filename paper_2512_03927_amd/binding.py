"""ctypes binding over libodmoe.so: same names as include/odmoe.h, argument marshalling only.

Every step of the path runs in the library's HIP kernels.  There is no CPU
fallback: if the shared library is missing, loading raises.  PyTorch is used by
callers for device memory and streams; tensors are passed here as raw pointers.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libodmoe.so")

ODMOE_OK, ODMOE_EINVAL, ODMOE_ENOMEM, ODMOE_EHIP, ODMOE_ESTATE, ODMOE_EBUSY = 0, -1, -2, -3, -4, -5
ODMOE_F32, ODMOE_BF16 = 0, 1
ODMOE_Q_NONE, ODMOE_Q_INT8_ROW, ODMOE_Q_INT4_G64, ODMOE_Q_F16 = 0, 1, 2, 3
ODMOE_MAX_TOPK = 8
ODMOE_MAX_EXPERTS = 1024

# every symbol include/odmoe.h and include/odmoe_measure.h declare
EXPORTS = (
    "odmoe_layer_init", "odmoe_layer_destroy", "odmoe_route_topk", "odmoe_expert_load_async",
    "odmoe_expert_evict", "odmoe_expert_ffn", "odmoe_expert_ffn_static", "odmoe_decode_step", "odmoe_pinned_alloc",
    "odmoe_pinned_free", "odmoe_slot_pool_bytes", "odmoe_last_error", "odmoe_version", "odmoe_probe_hbm",
    "odmoe_time_decode_kernels", "odmoe_time_expert_loads", "odmoe_load_window_ms", "odmoe_slot_groups",
    "odmoe_expert_bytes", "odmoe_quantize", "odmoe_quantize_expert", "odmoe_sep_emulate",
)


class odmoe_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("hidden", "ffn", "n_experts", "top_k", "n_layers", "n_slots", "dtype", "glue", "expert_quant")]


class odmoe_stats(C.Structure):
    _fields_ = [("t_route_ms", C.c_float), ("t_load_ms", C.c_float), ("t_ffn_up_ms", C.c_float),
                ("t_ffn_down_ms", C.c_float), ("t_glue_ms", C.c_float), ("t_step_ms", C.c_float),
                ("h2d_bytes", C.c_uint64), ("loads", C.c_uint64), ("reloads", C.c_uint64),
                ("hint_hits", C.c_uint64)]


class OdmoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"odmoe status {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Load libodmoe.so (once).  torch is imported first so that the library binds to the
    HIP runtime already in the process (the one that owns torch's streams and allocations)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2512_03927_amd.build` "
            "(there is no fallback path)")
    import torch  # noqa: F401  (loads libamdhip64 before our library needs it)
    L = C.CDLL(LIB_PATH, mode=C.RTLD_GLOBAL)
    vp, i32, u64 = C.c_void_p, C.c_int32, C.c_uint64
    L.odmoe_layer_init.argtypes = [C.POINTER(odmoe_config), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                   vp, vp, C.POINTER(vp)]
    L.odmoe_layer_destroy.argtypes = [vp]
    L.odmoe_route_topk.argtypes = [vp, i32, vp, i32, vp, vp]
    L.odmoe_expert_load_async.argtypes = [vp, i32, i32, C.POINTER(i32)]
    L.odmoe_expert_evict.argtypes = [vp, i32, i32]
    L.odmoe_expert_ffn.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp, i32]
    L.odmoe_decode_step.argtypes = [vp, vp, vp, vp, vp, C.POINTER(odmoe_stats)]
    L.odmoe_expert_ffn_static.argtypes = [C.POINTER(odmoe_config), vp, vp, vp, vp, i32, vp, vp]
    L.odmoe_expert_bytes.argtypes = [C.POINTER(odmoe_config)]
    L.odmoe_expert_bytes.restype = u64
    L.odmoe_quantize.argtypes = [vp, i32, C.c_int64, C.c_int64, i32, vp, vp, vp, vp]
    L.odmoe_quantize_expert.argtypes = [C.POINTER(odmoe_config), i32, vp, vp, vp]
    L.odmoe_sep_emulate.argtypes = [vp, vp, vp, i32, i32, C.POINTER(C.c_float), vp, C.POINTER(C.c_float),
                                    C.POINTER(C.c_float)]
    L.odmoe_pinned_alloc.argtypes = [u64, C.POINTER(vp)]
    L.odmoe_pinned_free.argtypes = [vp]
    L.odmoe_probe_hbm.argtypes = [vp, vp, u64, i32, vp]
    L.odmoe_time_decode_kernels.argtypes = [vp, i32, vp, i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_float),
                                            C.POINTER(C.c_float)]
    L.odmoe_time_expert_loads.argtypes = [vp, i32, C.POINTER(C.c_float)]
    L.odmoe_load_window_ms.argtypes = [i32, C.c_double, C.c_double]
    L.odmoe_load_window_ms.restype = C.c_double
    L.odmoe_slot_groups.argtypes = [vp]
    L.odmoe_slot_groups.restype = i32
    L.odmoe_slot_pool_bytes.argtypes = [vp]
    L.odmoe_slot_pool_bytes.restype = u64
    L.odmoe_last_error.restype = C.c_char_p
    L.odmoe_version.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("odmoe_slot_pool_bytes", "odmoe_last_error", "odmoe_version", "odmoe_load_window_ms",
                        "odmoe_slot_groups", "odmoe_expert_bytes"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != ODMOE_OK:
        raise OdmoeError(rc, (lib().odmoe_last_error() or b"").decode())


def _ptr(t) -> Optional[int]:
    """Raw address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    if hasattr(t, "ctypes"):
        return t.ctypes.data
    raise TypeError(type(t))


def _ptr_array(items: Optional[Sequence]) -> Optional[C.Array]:
    if items is None:
        return None
    arr = (C.c_void_p * len(items))()
    for i, it in enumerate(items):
        arr[i] = _ptr(it)
    return arr


def odmoe_last_error() -> str:
    return (lib().odmoe_last_error() or b"").decode()


def odmoe_version() -> str:
    return lib().odmoe_version().decode()


def odmoe_layer_init(cfg: odmoe_config, router_w: Sequence, router_b: Optional[Sequence],
                     expert_w: Sequence, compute_stream: Optional[int] = None,
                     copy_stream: Optional[int] = None) -> int:
    """Returns the opaque handle (an address).  Lists hold tensors or raw addresses."""
    out = C.c_void_p()
    rw, rb, ew = _ptr_array(router_w), _ptr_array(router_b), _ptr_array(expert_w)
    _check(lib().odmoe_layer_init(C.byref(cfg), rw, rb, ew, compute_stream, copy_stream, C.byref(out)))
    return out.value


def odmoe_layer_destroy(h: Optional[int]) -> None:
    _check(lib().odmoe_layer_destroy(h))


def odmoe_route_topk(h: int, layer: int, x_dev, n_tokens: int, idx_dev, gate_dev) -> None:
    _check(lib().odmoe_route_topk(h, layer, _ptr(x_dev), n_tokens, _ptr(idx_dev), _ptr(gate_dev)))


def odmoe_expert_load_async(h: int, layer: int, expert: int) -> int:
    slot = C.c_int32(-1)
    _check(lib().odmoe_expert_load_async(h, layer, expert, C.byref(slot)))
    return slot.value


def odmoe_expert_evict(h: int, layer: int, expert: int) -> None:
    _check(lib().odmoe_expert_evict(h, layer, expert))


def odmoe_expert_ffn(h: int, layer: int, idx_dev, gate_dev, idx_host, x_dev, n_tokens: int, y_dev,
                     evict_after: int = 1) -> None:
    _check(lib().odmoe_expert_ffn(h, layer, _ptr(idx_dev), _ptr(gate_dev), _ptr(idx_host), _ptr(x_dev),
                                  n_tokens, _ptr(y_dev), evict_after))


def odmoe_expert_ffn_static(cfg: odmoe_config, expert_table_dev, idx_dev, gate_dev, x_dev, n_tokens: int, y_dev,
                            stream: Optional[int] = None) -> None:
    _check(lib().odmoe_expert_ffn_static(C.byref(cfg), _ptr(expert_table_dev), _ptr(idx_dev), _ptr(gate_dev),
                                         _ptr(x_dev), n_tokens, _ptr(y_dev), stream))


def odmoe_decode_step(h: int, x_dev, y_dev, predicted_idx_host=None, idx_out_host=None,
                      stats: Optional[odmoe_stats] = None) -> None:
    _check(lib().odmoe_decode_step(h, _ptr(x_dev), _ptr(y_dev), _ptr(predicted_idx_host),
                                   _ptr(idx_out_host), C.byref(stats) if stats is not None else None))


def odmoe_expert_bytes(cfg: odmoe_config) -> int:
    return int(lib().odmoe_expert_bytes(C.byref(cfg)))


def odmoe_quantize(w_dev, dtype: int, rows: int, cols: int, kind: int, code_dev=None, scale_dev=None,
                   dequant_dev=None, stream: Optional[int] = None) -> None:
    _check(lib().odmoe_quantize(_ptr(w_dev), dtype, rows, cols, kind, _ptr(code_dev), _ptr(scale_dev),
                                _ptr(dequant_dev), stream))


def odmoe_quantize_expert(cfg: odmoe_config, kind: int, expert_dev, dst_dev, stream: Optional[int] = None) -> None:
    _check(lib().odmoe_quantize_expert(C.byref(cfg), kind, _ptr(expert_dev), _ptr(dst_dev), stream))


def odmoe_sep_emulate(main: int, shadow: int, x0_dev, n_iter: int, aligned: bool, x_final_dev=None):
    """(recall per iteration: list of float, shadow_ms, main_ms)."""
    rec = (C.c_float * max(1, n_iter))()
    sm, mm = C.c_float(), C.c_float()
    _check(lib().odmoe_sep_emulate(main, shadow, _ptr(x0_dev), n_iter, 1 if aligned else 0, rec, _ptr(x_final_dev),
                                   C.byref(sm), C.byref(mm)))
    return [float(rec[i]) for i in range(n_iter)], sm.value, mm.value


def odmoe_pinned_alloc(nbytes: int) -> int:
    out = C.c_void_p()
    _check(lib().odmoe_pinned_alloc(nbytes, C.byref(out)))
    return out.value


def odmoe_pinned_free(host: Optional[int]) -> None:
    _check(lib().odmoe_pinned_free(host))


def odmoe_probe_hbm(dst_dev, src_dev, nbytes: int, mode: int, stream: Optional[int] = None) -> None:
    _check(lib().odmoe_probe_hbm(_ptr(dst_dev), _ptr(src_dev), nbytes, mode, stream))


def odmoe_time_decode_kernels(h: int, layer: int, x_dev, n_tokens: int, reps: int = 1):
    """(route_us, ffn_up_us, ffn_down_us): average kernel durations from HIP events."""
    r, u, d = C.c_float(), C.c_float(), C.c_float()
    _check(lib().odmoe_time_decode_kernels(h, layer, _ptr(x_dev), n_tokens, reps, C.byref(r), C.byref(u),
                                           C.byref(d)))
    return r.value, u.value, d.value


def odmoe_time_expert_loads(h: int, n_tokens: int) -> float:
    """Wall-clock ms per token of the expert copies of n_tokens decode tokens, no kernels."""
    ms = C.c_float()
    _check(lib().odmoe_time_expert_loads(h, n_tokens, C.byref(ms)))
    return ms.value


def odmoe_load_window_ms(n_groups: int, t_main_ms: float, t_worker_ms: float) -> float:
    return float(lib().odmoe_load_window_ms(n_groups, t_main_ms, t_worker_ms))


def odmoe_slot_groups(h: int) -> int:
    return int(lib().odmoe_slot_groups(h))


def odmoe_slot_pool_bytes(h: int) -> int:
    return int(lib().odmoe_slot_pool_bytes(h))
