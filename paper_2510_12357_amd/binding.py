"""ctypes front end of ``libmobile_moe.so`` -- argument marshalling only.

Every function has the name and argument order of its C entry point in
``include/mobile_moe.h``; tensors are torch tensors (device memory and streams are all that
torch is used for) and are passed down as raw pointers.  Nothing is computed in Python, and
there is no fallback: if the HIP library is missing, loading fails with an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

from .workloads import LayerConfig

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmobile_moe.so")

MOE_BF16, MOE_FP32, MOE_BF16_W8, MOE_BF16_MXFP4 = 0, 1, 2, 3
MOE_FETCH_DEMAND, MOE_FETCH_PREFETCH = 0, 1
MOE_MAX_SHARED = 4
MOE_OK = 0
ERRORS = {-1: "MOE_E_BADARG", -2: "MOE_E_SHAPE", -3: "MOE_E_UNSUPPORTED", -4: "MOE_E_HIP",
          -5: "MOE_E_CACHE_FULL", -6: "MOE_E_WORKSPACE"}

EXPORTS = ("moe_last_error", "moe_device_info", "moe_profile_enable", "moe_profile_read", "moe_profile_plain_read", "moe_route", "moe_token_confidence",
           "moe_dispatch_workspace_bytes", "moe_dispatch", "moe_dispatch_from", "moe_combine_add",
           "moe_expert_ffn_workspace_bytes", "moe_expert_blob_bytes",
           "moe_shared_out_slabs", "moe_layer_decode_workspace_bytes", "moe_layer_decode_init",
           "moe_layer_decode_status", "moe_layer_decode", "moe_expert_ffn", "moe_expert_ffn_static", "moe_expert_ffn_static_max_bytes",
           "moe_combine", "moe_cache_create", "moe_cache_destroy",
           "moe_cache_expert_table", "expert_cache_fetch", "moe_expert_ffn_cached", "moe_cache_snapshot", "moe_cache_sync",
           "moe_cache_set_prefetch_limit", "moe_cache_emulate_link", "moe_prefetcher_create", "moe_prefetcher_destroy",
           "moe_prefetcher_set_in_flight_limit", "moe_prefetcher_set_yield_to_demand", "moe_prefetcher_predict", "moe_prefetcher_predicted",
           "moe_prefetcher_advance")


class MoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{ERRORS.get(code, code)}: {msg}")
        self.code = code


class moe_config(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("H", ctypes.c_int32), ("E", ctypes.c_int32),
                ("I", ctypes.c_int32), ("k_big", ctypes.c_int32), ("k_little", ctypes.c_int32),
                ("n_shared", ctypes.c_int32), ("shared_I", ctypes.c_int32 * MOE_MAX_SHARED),
                ("dtype", ctypes.c_int32), ("renorm", ctypes.c_int32), ("gamma", ctypes.c_float)]


class moe_fetch_stats(ctypes.Structure):
    _fields_ = [("hits", ctypes.c_int32), ("misses", ctypes.c_int32), ("dropped", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("bytes_h2d", ctypes.c_uint64)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the HIP library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           "`python -m paper_2510_12357_amd.build` (hipcc, gfx950)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    cfgp = ctypes.POINTER(moe_config)
    lib.moe_last_error.restype = ctypes.c_char_p
    lib.moe_last_error.argtypes = []
    lib.moe_device_info.argtypes = [ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.moe_profile_enable.argtypes = [ctypes.c_int]
    lib.moe_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int64),
                                     ctypes.POINTER(ctypes.c_double)]
    lib.moe_profile_plain_read.argtypes = [vp, sz, vp, vp]
    lib.moe_route.argtypes = [cfgp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp, vp, vp, vp]
    lib.moe_token_confidence.argtypes = [vp, i32, i32, vp, vp]
    lib.moe_dispatch_workspace_bytes.argtypes = [cfgp]
    lib.moe_dispatch_workspace_bytes.restype = sz
    lib.moe_dispatch.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_dispatch_from.argtypes = [cfgp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.moe_combine_add.argtypes = [cfgp, vp, vp, vp, vp, i32, vp, vp]
    lib.moe_expert_ffn_workspace_bytes.argtypes = [cfgp]
    lib.moe_expert_ffn_workspace_bytes.restype = sz
    lib.moe_expert_blob_bytes.argtypes = [cfgp, i32]
    lib.moe_expert_blob_bytes.restype = sz
    lib.moe_shared_out_slabs.argtypes = [cfgp]
    lib.moe_shared_out_slabs.restype = i32
    lib.moe_expert_ffn.argtypes = [cfgp, vp, vp, vp, vp, ctypes.POINTER(vp), ctypes.c_int,
                                   ctypes.c_int, vp, vp, vp, sz, vp]
    lib.moe_layer_decode_workspace_bytes.argtypes = [cfgp]
    lib.moe_layer_decode_workspace_bytes.restype = sz
    lib.moe_layer_decode_init.argtypes = [vp, sz, vp]
    lib.moe_layer_decode_init.restype = ctypes.c_int
    lib.moe_layer_decode_status.argtypes = [vp, ctypes.POINTER(i32)]
    lib.moe_layer_decode_status.restype = ctypes.c_int
    lib.moe_layer_decode.argtypes = [cfgp, vp, vp, vp, vp, vp, ctypes.POINTER(vp), vp, ctypes.c_int] + [vp] * 11 + [
        vp, sz, vp]
    lib.moe_layer_decode.restype = ctypes.c_int
    lib.moe_expert_ffn_static.argtypes = [cfgp, vp, vp, vp, vp, ctypes.POINTER(vp), ctypes.c_int,
                                          ctypes.c_int, vp, vp, vp]
    lib.moe_expert_ffn_static.restype = ctypes.c_int
    lib.moe_expert_ffn_static_max_bytes.argtypes = []
    lib.moe_expert_ffn_static_max_bytes.restype = sz
    lib.moe_combine.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp]
    lib.moe_cache_create.argtypes = [i32, sz, i32, vp, vp]
    lib.moe_cache_create.restype = vp
    lib.moe_cache_destroy.argtypes = [vp]
    lib.moe_cache_destroy.restype = None
    lib.moe_cache_expert_table.argtypes = [vp]
    lib.moe_cache_expert_table.restype = vp
    lib.expert_cache_fetch.argtypes = [vp, ctypes.POINTER(i32), i32, i32, ctypes.POINTER(i32),
                                       ctypes.POINTER(moe_fetch_stats), vp]
    lib.moe_expert_ffn_cached.argtypes = [cfgp, vp, vp, vp, vp, ctypes.POINTER(vp), vp, vp, vp, sz,
                                          ctypes.POINTER(moe_fetch_stats), ctypes.POINTER(i32), vp]
    lib.moe_cache_snapshot.argtypes = [vp, ctypes.POINTER(i32)]
    lib.moe_cache_sync.argtypes = [vp]
    lib.moe_cache_set_prefetch_limit.argtypes = [vp, i32]
    lib.moe_cache_emulate_link.argtypes = [vp, ctypes.c_double]
    lib.moe_prefetcher_create.argtypes = [i32, ctypes.POINTER(vp), i32]
    lib.moe_prefetcher_create.restype = vp
    lib.moe_prefetcher_destroy.argtypes = [vp]
    lib.moe_prefetcher_destroy.restype = None
    lib.moe_prefetcher_set_in_flight_limit.argtypes = [vp, i32]
    lib.moe_prefetcher_set_yield_to_demand.argtypes = [vp, i32]
    lib.moe_prefetcher_predict.argtypes = [vp, ctypes.POINTER(vp), i32, ctypes.POINTER(i32), i32, vp]
    lib.moe_prefetcher_predicted.argtypes = [vp, i32, ctypes.POINTER(i32)]
    lib.moe_prefetcher_advance.argtypes = [vp, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32),
                                           ctypes.POINTER(moe_fetch_stats), vp]
    for name in ("moe_prefetcher_set_in_flight_limit", "moe_prefetcher_set_yield_to_demand", "moe_prefetcher_predict", "moe_prefetcher_predicted",
                 "moe_prefetcher_advance"):
        getattr(lib, name).restype = ctypes.c_int
    for name in ("moe_device_info", "moe_profile_enable", "moe_profile_read", "moe_profile_plain_read", "moe_route", "moe_token_confidence", "moe_dispatch",
                 "moe_dispatch_from", "moe_combine_add",
                 "moe_expert_ffn", "moe_combine", "expert_cache_fetch", "moe_expert_ffn_cached", "moe_cache_snapshot",
                 "moe_cache_sync", "moe_cache_set_prefetch_limit", "moe_cache_emulate_link"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != MOE_OK:
        raise MoeError(rc, load_library().moe_last_error().decode())


def make_config(cfg: LayerConfig, T: Optional[int] = None) -> moe_config:
    c = moe_config()
    c.T = cfg.T if T is None else T
    c.H, c.E, c.I, c.k_big, c.k_little = cfg.H, cfg.E, cfg.I, cfg.k_big, cfg.k_little
    c.n_shared = len(cfg.shared_I)
    for i, v in enumerate(cfg.shared_I):
        c.shared_I[i] = v
    c.dtype = {"bf16": MOE_BF16, "fp32": MOE_FP32, "bf16w8": MOE_BF16_W8, "bf16mx4": MOE_BF16_MXFP4}[cfg.dtype]
    c.renorm = int(cfg.renorm)
    c.gamma = cfg.gamma
    return c


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous(), "tensors passed to the C ABI must be dense"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


# ------------------------------------------------------------------------------ entry points
def moe_last_error() -> str:
    return load_library().moe_last_error().decode()


def moe_device_info():
    n_cu, is950 = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load_library().moe_device_info(ctypes.byref(n_cu), ctypes.byref(is950)))
    return n_cu.value, bool(is950.value)


PROFILE_KINDS = ("router_gemm", "route_topk", "dispatch", "ffn_gate_up", "ffn_down", "combine",
                 "token_confidence", "decode_step")


def moe_profile_enable(on: bool) -> None:
    _check(load_library().moe_profile_enable(int(bool(on))))


def moe_profile_plain_read(buf, sink) -> None:
    """One plain streaming read of the tensor `buf` on the current stream (measurement aid)."""
    _check(load_library().moe_profile_plain_read(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), _stream(None)))


def moe_profile_read(kind: int):
    """-> (launch sites recorded, summed duration in ms) of one kernel kind"""
    n, ms = ctypes.c_int64(0), ctypes.c_double(0.0)
    _check(load_library().moe_profile_read(kind, ctypes.byref(n), ctypes.byref(ms)))
    return n.value, ms.value


def moe_route(cfg: moe_config, x, Wg, gate_bias, conf, logits, logits_given, topk_idx, topk_w,
              important, k_t, stream=None) -> None:
    _check(load_library().moe_route(ctypes.byref(cfg), _ptr(x), _ptr(Wg), _ptr(gate_bias), _ptr(conf),
                                    _ptr(logits), int(bool(logits_given)), _ptr(topk_idx),
                                    _ptr(topk_w), _ptr(important), _ptr(k_t), _stream(stream)))


def moe_token_confidence(lm_logits, T: int, V: int, conf, stream=None) -> None:
    _check(load_library().moe_token_confidence(_ptr(lm_logits), T, V, _ptr(conf), _stream(stream)))


def moe_dispatch_workspace_bytes(cfg: moe_config) -> int:
    return int(load_library().moe_dispatch_workspace_bytes(ctypes.byref(cfg)))


def moe_dispatch(cfg: moe_config, topk_idx, k_t, expert_offsets, sorted_token, sorted_rank,
                 inv_pos, ws, ws_bytes: int, stream=None) -> None:
    _check(load_library().moe_dispatch(ctypes.byref(cfg), _ptr(topk_idx), _ptr(k_t),
                                       _ptr(expert_offsets), _ptr(sorted_token), _ptr(sorted_rank),
                                       _ptr(inv_pos), _ptr(ws), ws_bytes, _stream(stream)))


def moe_dispatch_from(cfg: moe_config, topk_idx, k_t, j_lo: int, expert_offsets, sorted_token, sorted_rank,
                      inv_pos, ws, ws_bytes: int, stream=None) -> None:
    _check(load_library().moe_dispatch_from(ctypes.byref(cfg), _ptr(topk_idx), _ptr(k_t), int(j_lo),
                                            _ptr(expert_offsets), _ptr(sorted_token), _ptr(sorted_rank),
                                            _ptr(inv_pos), _ptr(ws), ws_bytes, _stream(stream)))


def moe_combine_add(cfg: moe_config, y, topk_w, inv_pos, k_t, j_lo: int, out, stream=None) -> None:
    _check(load_library().moe_combine_add(ctypes.byref(cfg), _ptr(y), _ptr(topk_w), _ptr(inv_pos), _ptr(k_t),
                                          int(j_lo), _ptr(out), _stream(stream)))


def moe_expert_ffn_workspace_bytes(cfg: moe_config) -> int:
    return int(load_library().moe_expert_ffn_workspace_bytes(ctypes.byref(cfg)))


def moe_expert_blob_bytes(cfg: moe_config, I: int) -> int:
    return int(load_library().moe_expert_blob_bytes(ctypes.byref(cfg), I))


def moe_shared_out_slabs(cfg: moe_config) -> int:
    return int(load_library().moe_shared_out_slabs(ctypes.byref(cfg)))


def moe_expert_ffn(cfg: moe_config, x, expert_offsets, sorted_token, expert_w, shared_w: Sequence,
                   run_routed, run_shared, y, shared_out, ws, ws_bytes: int, stream=None) -> None:
    """expert_w: device int64 tensor [E] of blob addresses, or a raw device address (int);
    shared_w: sequence of device tensors (their addresses form the host pointer array)."""
    sw = (ctypes.c_void_p * max(1, len(shared_w)))(*[t.data_ptr() for t in shared_w])
    ew = ctypes.c_void_p(expert_w) if isinstance(expert_w, int) else _ptr(expert_w)
    _check(load_library().moe_expert_ffn(ctypes.byref(cfg), _ptr(x), _ptr(expert_offsets),
                                         _ptr(sorted_token), ew, sw, int(bool(run_routed)),
                                         int(bool(run_shared)), _ptr(y), _ptr(shared_out), _ptr(ws),
                                         ws_bytes, _stream(stream)))


def moe_layer_decode_workspace_bytes(cfg: moe_config) -> int:
    return int(load_library().moe_layer_decode_workspace_bytes(ctypes.byref(cfg)))


def moe_layer_decode_init(ws, ws_bytes: int, stream=None) -> None:
    _check(load_library().moe_layer_decode_init(_ptr(ws), ws_bytes, _stream(stream)))


def moe_layer_decode_status(ws) -> int:
    """-> number of waits inside the kernel that have ever given up on this workspace (synchronises)"""
    n = ctypes.c_int32(0)
    _check(load_library().moe_layer_decode_status(_ptr(ws), ctypes.byref(n)))
    return n.value


def moe_layer_decode(cfg: moe_config, x, Wg, gate_bias, conf, expert_w, shared_w: Sequence, logits, logits_given,
                     topk_idx, topk_w, important, k_t, expert_offsets, sorted_token, sorted_rank, inv_pos, y,
                     shared_out, out, ws, ws_bytes: int, stream=None) -> None:
    sw = (ctypes.c_void_p * max(1, len(shared_w)))(*[t.data_ptr() for t in shared_w])
    ew = ctypes.c_void_p(expert_w) if isinstance(expert_w, int) else _ptr(expert_w)
    _check(load_library().moe_layer_decode(ctypes.byref(cfg), _ptr(x), _ptr(Wg), _ptr(gate_bias), _ptr(conf), ew, sw,
                                           _ptr(logits), int(bool(logits_given)), _ptr(topk_idx), _ptr(topk_w),
                                           _ptr(important), _ptr(k_t), _ptr(expert_offsets), _ptr(sorted_token),
                                           _ptr(sorted_rank), _ptr(inv_pos), _ptr(y), _ptr(shared_out), _ptr(out),
                                           _ptr(ws), ws_bytes, _stream(stream)))


def moe_expert_ffn_static_max_bytes() -> int:
    return int(load_library().moe_expert_ffn_static_max_bytes())


def moe_expert_ffn_static(cfg: moe_config, x, expert_offsets, sorted_token, expert_w, shared_w: Sequence,
                          run_routed, run_shared, y, shared_out, stream=None) -> None:
    """moe_expert_ffn without a workspace argument (the library's built-in scratch buffer)."""
    sw = (ctypes.c_void_p * max(1, len(shared_w)))(*[t.data_ptr() for t in shared_w])
    ew = ctypes.c_void_p(expert_w) if isinstance(expert_w, int) else _ptr(expert_w)
    _check(load_library().moe_expert_ffn_static(ctypes.byref(cfg), _ptr(x), _ptr(expert_offsets),
                                                _ptr(sorted_token), ew, sw, int(bool(run_routed)),
                                                int(bool(run_shared)), _ptr(y), _ptr(shared_out),
                                                _stream(stream)))


def moe_combine(cfg: moe_config, y, topk_w, inv_pos, k_t, shared_out, out, stream=None) -> None:
    _check(load_library().moe_combine(ctypes.byref(cfg), _ptr(y), _ptr(topk_w), _ptr(inv_pos),
                                      _ptr(k_t), _ptr(shared_out), _ptr(out), _stream(stream)))


def moe_cache_create(E: int, blob_bytes: int, n_slots: int, host_blobs: torch.Tensor,
                     device_slots: torch.Tensor) -> int:
    assert host_blobs.is_pinned(), "host arena must be pinned memory"
    h = load_library().moe_cache_create(E, blob_bytes, n_slots, _ptr(host_blobs), _ptr(device_slots))
    if not h:
        raise MoeError(-1, moe_last_error())
    return h


def moe_cache_destroy(cache: int) -> None:
    load_library().moe_cache_destroy(ctypes.c_void_p(cache))


def moe_cache_expert_table(cache: int) -> int:
    return int(load_library().moe_cache_expert_table(ctypes.c_void_p(cache)))


def expert_cache_fetch(cache: int, expert_ids: Sequence[int], mode: int, stream=None):
    """-> (slot_of list, moe_fetch_stats)"""
    n = len(expert_ids)
    ids = (ctypes.c_int32 * max(1, n))(*expert_ids)
    slots = (ctypes.c_int32 * max(1, n))()
    st = moe_fetch_stats()
    _check(load_library().expert_cache_fetch(ctypes.c_void_p(cache), ids, n, mode, slots,
                                             ctypes.byref(st), _stream(stream)))
    return list(slots[:n]), st


def moe_expert_ffn_cached(cfg: moe_config, cache: int, x, expert_offsets, sorted_token, shared_w: Sequence,
                          y, shared_out, ws, ws_bytes: int, stream=None):
    """-> (summed moe_fetch_stats, number of waves)"""
    sw = (ctypes.c_void_p * max(1, len(shared_w)))(*[t.data_ptr() for t in shared_w])
    st, nw = moe_fetch_stats(), ctypes.c_int32(0)
    _check(load_library().moe_expert_ffn_cached(ctypes.byref(cfg), ctypes.c_void_p(cache), _ptr(x),
                                                _ptr(expert_offsets), _ptr(sorted_token), sw, _ptr(y),
                                                _ptr(shared_out), _ptr(ws), ws_bytes, ctypes.byref(st),
                                                ctypes.byref(nw), _stream(stream)))
    return st, nw.value


def moe_cache_snapshot(cache: int, n_slots: int):
    out = (ctypes.c_int32 * n_slots)()
    rc = load_library().moe_cache_snapshot(ctypes.c_void_p(cache), out)
    if rc < 0:
        _check(rc)
    return list(out)


def moe_cache_sync(cache: int) -> None:
    _check(load_library().moe_cache_sync(ctypes.c_void_p(cache)))


def moe_cache_set_prefetch_limit(cache: int, max_copies_per_call: int) -> None:
    _check(load_library().moe_cache_set_prefetch_limit(ctypes.c_void_p(cache), int(max_copies_per_call)))


def moe_cache_emulate_link(cache: int, gb_per_s: float) -> None:
    _check(load_library().moe_cache_emulate_link(ctypes.c_void_p(cache), float(gb_per_s)))


def moe_prefetcher_create(caches: Sequence[int], k_big: int) -> int:
    arr = (ctypes.c_void_p * max(1, len(caches)))(*caches)
    h = load_library().moe_prefetcher_create(len(caches), arr, int(k_big))
    if not h:
        raise MoeError(-1, moe_last_error())
    return int(h)


def moe_prefetcher_destroy(p: int) -> None:
    load_library().moe_prefetcher_destroy(ctypes.c_void_p(p))


def moe_prefetcher_set_in_flight_limit(p: int, max_copies_in_flight: int) -> None:
    _check(load_library().moe_prefetcher_set_in_flight_limit(ctypes.c_void_p(p), int(max_copies_in_flight)))


def moe_prefetcher_set_yield_to_demand(p: int, on: bool) -> None:
    _check(load_library().moe_prefetcher_set_yield_to_demand(ctypes.c_void_p(p), 1 if on else 0))


def moe_prefetcher_predict(p: int, layer_logits: Sequence, T: int, rejected: Sequence[int], stream=None) -> None:
    """layer_logits: one device tensor [T, E] fp32 per layer."""
    ptrs = (ctypes.c_void_p * max(1, len(layer_logits)))(*[t.data_ptr() for t in layer_logits])
    n = len(rejected)
    rej = (ctypes.c_int32 * max(1, n))(*rejected)
    _check(load_library().moe_prefetcher_predict(ctypes.c_void_p(p), ptrs, int(T), rej, n, _stream(stream)))


def moe_prefetcher_predicted(p: int, layer: int, n_experts: int):
    out = (ctypes.c_int32 * n_experts)()
    rc = load_library().moe_prefetcher_predicted(ctypes.c_void_p(p), int(layer), out)
    if rc < 0:
        _check(rc)
    return list(out[:rc])


def moe_prefetcher_advance(p: int, layer: int, distance: int, n_layers: int, stream=None):
    """-> [(layer, limit the request ran under, moe_fetch_stats), ...] of the requests made"""
    ls, lim = (ctypes.c_int32 * n_layers)(), (ctypes.c_int32 * n_layers)()
    st = (moe_fetch_stats * n_layers)()
    rc = load_library().moe_prefetcher_advance(ctypes.c_void_p(p), int(layer), int(distance), ls, lim, st,
                                               _stream(stream))
    if rc < 0:
        _check(rc)
    return [(int(ls[i]), int(lim[i]), st[i]) for i in range(rc)]


# ------------------------------------------------------------------------------ plumbing helpers
def torch_dtype(cfg: LayerConfig):
    return torch.float32 if cfg.dtype == "fp32" else torch.bfloat16


def to_device(a, cfg: LayerConfig, device="cuda") -> torch.Tensor:
    """Uploads a stored host tensor (float32, or uint16 holding bf16 bits) without changing bits."""
    import numpy as np
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


class StepBuffers:
    """Device buffers of one layer step (allocation only; the step itself is the C calls)."""

    def __init__(self, cfg: LayerConfig, T: Optional[int] = None, device="cuda"):
        T = cfg.T if T is None else T
        self.cfg, self.T = cfg, T
        self.c = make_config(cfg, T)
        K, E, H = cfg.k_big, cfg.E, cfg.H
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.logits = torch.empty((T, E), **f32)
        self.topk_idx = torch.empty((T, K), **i32)
        self.topk_w = torch.empty((T, K), **f32)
        self.important = torch.empty((T,), dtype=torch.uint8, device=device)
        self.k_t = torch.empty((T,), **i32)
        self.expert_offsets = torch.empty((E + 1,), **i32)
        self.sorted_token = torch.empty((T * K,), **i32)
        self.sorted_rank = torch.empty((T * K,), **i32)
        self.inv_pos = torch.empty((T, K), **i32)
        self.y = torch.zeros((T * K, H), **f32)
        ns = moe_shared_out_slabs(self.c)
        self.shared_out = torch.zeros((ns, T, H), **f32) if ns > 0 else None
        self.out = torch.empty((T, H), dtype=torch_dtype(cfg), device=device)
        self.dws_bytes = moe_dispatch_workspace_bytes(self.c)
        self.dws = torch.empty((self.dws_bytes,), dtype=torch.uint8, device=device)
        self.fws_bytes = moe_expert_ffn_workspace_bytes(self.c)
        self.fws = torch.empty((self.fws_bytes,), dtype=torch.uint8, device=device)
        self.ev_in, self.ev_shared = torch.cuda.Event(), torch.cuda.Event()
        # workspace of moe_layer_decode (steps of at most 64 tokens, bf16 activations), cleared once
        self.lws_bytes = moe_layer_decode_workspace_bytes(self.c) if 0 < T <= 64 and cfg.dtype in ("bf16", "bf16w8") else 0
        self.lws = None
        if self.lws_bytes:
            self.lws = torch.empty((self.lws_bytes,), dtype=torch.uint8, device=device)
            moe_layer_decode_init(self.lws, self.lws_bytes)


def layer_step(b: StepBuffers, x, Wg, gate_bias, conf, expert_table, shared_w, logits_given=False,
               stream=None, side_stream=None) -> torch.Tensor:
    """One step of the layer with all experts resident: the C calls back to back on `stream`.

    With `side_stream` (a second torch stream of default priority) the shared experts, which do not
    depend on the router, are enqueued there first and run under the router, selection and dispatch
    kernels; the combine waits for them.  Only stream plumbing is added; the calls are the same."""
    overlap = side_stream is not None and b.shared_out is not None
    if overlap:
        main = stream if stream is not None else torch.cuda.current_stream()
        b.ev_in.record(main)                     # x is ready; the previous combine has read shared_out
        side_stream.wait_event(b.ev_in)
        moe_expert_ffn(b.c, x, b.expert_offsets, b.sorted_token, None, shared_w, False, True, b.y,
                       b.shared_out, b.fws, b.fws_bytes, side_stream)
        b.ev_shared.record(side_stream)
    moe_route(b.c, x, Wg, gate_bias, conf, b.logits, logits_given, b.topk_idx, b.topk_w, b.important,
              b.k_t, stream)
    moe_dispatch(b.c, b.topk_idx, b.k_t, b.expert_offsets, b.sorted_token, b.sorted_rank, b.inv_pos,
                 b.dws, b.dws_bytes, stream)
    moe_expert_ffn(b.c, x, b.expert_offsets, b.sorted_token, expert_table, shared_w, True, not overlap, b.y,
                   b.shared_out, b.fws, b.fws_bytes, stream)
    if overlap:
        main.wait_event(b.ev_shared)
    moe_combine(b.c, b.y, b.topk_w, b.inv_pos, b.k_t, b.shared_out, b.out, stream)
    return b.out


def layer_decode_step(b: StepBuffers, x, Wg, gate_bias, conf, expert_table, shared_w, logits_given=False,
                      stream=None) -> torch.Tensor:
    """One decode step (at most 64 tokens) of the layer in one launch: a single C call."""
    moe_layer_decode(b.c, x, Wg, gate_bias, conf, expert_table, shared_w, b.logits, logits_given, b.topk_idx,
                     b.topk_w, b.important, b.k_t, b.expert_offsets, b.sorted_token, b.sorted_rank, b.inv_pos, b.y,
                     b.shared_out, b.out, b.lws, b.lws_bytes, stream)
    return b.out


def fallback_step(b: StepBuffers, x, conf, expert_table, stream=None) -> torch.Tensor:
    """Second pass of Alg. 1 on the buffers of a little pass (layer_step with a confidence above gamma
    for every token, which leaves the router logits in b.logits and the little output in b.out): the
    tokens rejected by `conf` get the experts of ranks k_little .. k_big-1 added.  Four C calls."""
    kl = int(b.c.k_little)
    moe_route(b.c, x, None, None, conf, b.logits, True, b.topk_idx, b.topk_w, b.important, b.k_t, stream)
    moe_dispatch_from(b.c, b.topk_idx, b.k_t, kl, b.expert_offsets, b.sorted_token, b.sorted_rank, b.inv_pos,
                      b.dws, b.dws_bytes, stream)
    moe_expert_ffn(b.c, x, b.expert_offsets, b.sorted_token, expert_table, (), True, False, b.y,
                   b.shared_out, b.fws, b.fws_bytes, stream)
    moe_combine_add(b.c, b.y, b.topk_w, b.inv_pos, b.k_t, kl, b.out, stream)
    return b.out


def layer_step_cached(b: StepBuffers, x, Wg, gate_bias, conf, cache: int, shared_w, stream=None):
    """One step of the layer whose routed experts live in pinned host memory behind `cache`
    (Sec. II-B): router and dispatch as in layer_step, then the execution stage through the cache
    (the host waits once for the router's decision).  -> (b.out, summed fetch statistics, waves)."""
    moe_route(b.c, x, Wg, gate_bias, conf, b.logits, False, b.topk_idx, b.topk_w, b.important, b.k_t, stream)
    moe_dispatch(b.c, b.topk_idx, b.k_t, b.expert_offsets, b.sorted_token, b.sorted_rank, b.inv_pos,
                 b.dws, b.dws_bytes, stream)
    st, waves = moe_expert_ffn_cached(b.c, cache, x, b.expert_offsets, b.sorted_token, shared_w, b.y,
                                      b.shared_out, b.fws, b.fws_bytes, stream)
    moe_combine(b.c, b.y, b.topk_w, b.inv_pos, b.k_t, b.shared_out, b.out, stream)
    return b.out, st, waves
