"""Thin binding of libstalloc.so (include/stalloc.h): argument marshalling only.

Every step of the planning path runs inside the HIP library; PyTorch is used for
device memory and streams.  There is no CPU fallback: if the library has not been
built (`python paper_2507_16274_amd/build.py`) importing the entry points fails.

Tensors are CUDA/HIP tensors on the current device.  Byte quantities are int64
tensors holding the library's uint64 bit patterns (all values stay below 2^63);
timestamps, orders and indices are int32 tensors holding uint32 values below 2^31.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

import torch  # loaded first so that the HIP runtime already in the process is shared

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libstalloc.so")

STATUS = {0: "STALLOC_OK", 1: "STALLOC_ERR_INVALID_ARG", 2: "STALLOC_ERR_BAD_TRACE", 3: "STALLOC_ERR_OVERFLOW",
          4: "STALLOC_ERR_NOMEM", 5: "STALLOC_ERR_DEVICE", 6: "STALLOC_ERR_BAD_ORDER", 7: "STALLOC_ERR_BAD_WINDOW",
          8: "STALLOC_ERR_BAD_LAYER", 9: "STALLOC_ERR_TOO_LARGE"}
STATIC_MAX_T_END = 524288        # STALLOC_STATIC_MAX_T_END of include/stalloc.h
EXPORTS = ("stalloc_plan", "stalloc_validate", "stalloc_lower_bound", "stalloc_lower_bound_static",
           "stalloc_reusable_space",
           "stalloc_memory_layers", "stalloc_expand_layers", "stalloc_tmp", "stalloc_make_orders",
           "stalloc_status_string", "stalloc_plan_lds_capacity", "stalloc_plan_report", "stalloc_probe",
           "stalloc_fuse_groups", "stalloc_plan_sized")
KERNELS = {0: "none", 1: "bitmap", 2: "list_lds", 3: "list_memory", 4: "long_list"}


class StallocError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {STATUS.get(code, code)}")
        self.code = code


class _Trace(ctypes.Structure):
    _fields_ = [("n", ctypes.c_uint32), ("t_end", ctypes.c_uint32), ("size", ctypes.c_void_p),
                ("t_alloc", ctypes.c_void_p), ("t_free", ctypes.c_void_p)]


class _PlanInfo(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_uint32), ("granule_log2", ctypes.c_uint32), ("granules", ctypes.c_uint64),
                ("plans_64bit", ctypes.c_uint32), ("lifetime_threshold", ctypes.c_uint32),
                ("long_requests", ctypes.c_uint32), ("address_bits", ctypes.c_uint32),
                ("large_size", ctypes.c_uint64), ("large_requests", ctypes.c_uint32), ("list_entry_bytes", ctypes.c_uint32)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_2507_16274_amd/build.py` "
                          "(hipcc, gfx950); there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, u32 = ctypes.c_void_p, ctypes.c_uint32
    szp = ctypes.POINTER(ctypes.c_size_t)
    tp = ctypes.POINTER(_Trace)
    lib.stalloc_plan.argtypes = [tp, vp, u32, vp, vp, vp, vp, vp, vp, szp, vp]
    lib.stalloc_plan_sized.argtypes = [tp, vp, u32, vp, vp, vp, vp, vp, ctypes.c_uint64, ctypes.c_uint64, vp, szp, vp]
    lib.stalloc_validate.argtypes = [tp, vp, u32, vp, vp, vp, vp, szp, vp]
    lib.stalloc_lower_bound.argtypes = [tp, vp, vp, vp, vp, szp, vp]
    lib.stalloc_lower_bound_static.argtypes = [tp, vp, vp, vp, vp]
    lib.stalloc_reusable_space.argtypes = [tp, vp, vp, u32, u32, vp, vp, vp, vp, vp, szp, vp]
    lib.stalloc_memory_layers.argtypes = [tp, vp, vp, vp, vp, vp, vp, vp, szp, vp]
    lib.stalloc_expand_layers.argtypes = [u32, u32, vp, vp, u32, vp, vp, vp]
    lib.stalloc_tmp.argtypes = [tp, vp, u32, vp, vp, vp, szp, vp]
    lib.stalloc_make_orders.argtypes = [tp, u32, u32, ctypes.c_uint64, vp, vp, vp, szp, vp]
    lib.stalloc_fuse_groups.argtypes = [tp, vp, vp, vp, u32, u32, u32, vp, vp, vp, vp, vp, vp, szp, vp]
    for name in ("stalloc_plan", "stalloc_validate", "stalloc_lower_bound", "stalloc_lower_bound_static",
                 "stalloc_reusable_space", "stalloc_memory_layers", "stalloc_expand_layers", "stalloc_tmp",
                 "stalloc_make_orders", "stalloc_fuse_groups", "stalloc_plan_sized"):
        getattr(lib, name).restype = ctypes.c_int
    lib.stalloc_plan_report.argtypes = [vp, ctypes.POINTER(_PlanInfo), vp]
    lib.stalloc_plan_report.restype = ctypes.c_int
    lib.stalloc_probe.argtypes = [u32, vp, ctypes.c_size_t, u32, ctypes.POINTER(ctypes.c_uint64), vp]
    lib.stalloc_probe.restype = ctypes.c_int
    lib.stalloc_status_string.argtypes = [ctypes.c_int]
    lib.stalloc_status_string.restype = ctypes.c_char_p
    lib.stalloc_plan_lds_capacity.argtypes = []
    lib.stalloc_plan_lds_capacity.restype = ctypes.c_uint32
    return lib


lib = _load()


def _dev(t: Optional[torch.Tensor], dtype: torch.dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous {dtype} tensor on the GPU")
    return t.data_ptr()


def _trace(size: torch.Tensor, t_alloc: torch.Tensor, t_free: torch.Tensor, t_end: int) -> _Trace:
    n = size.numel()
    if t_alloc.numel() != n or t_free.numel() != n:
        raise ValueError("size, t_alloc and t_free must have the same length")
    return _Trace(n, int(t_end), _dev(size, torch.int64, "size"), _dev(t_alloc, torch.int32, "t_alloc"),
                  _dev(t_free, torch.int32, "t_free"))


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    return (stream or torch.cuda.current_stream()).cuda_stream


def _workspace(nbytes: int, device, cache: Optional[Dict]) -> torch.Tensor:
    if cache is not None:
        ws = cache.get("ws")
        if ws is None or ws.numel() < nbytes:
            ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
            cache["ws"] = ws
        return ws
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise StallocError(rc, where)


def stalloc_plan(size, t_alloc, t_free, t_end: int, orders, *, want_offsets: bool = True,
                 want_best_offsets: bool = True, stream=None, workspace_cache: Optional[Dict] = None,
                 out: Optional[Dict] = None) -> Dict[str, torch.Tensor]:
    """Enqueue stalloc_plan; returns the (asynchronously filled) output tensors.

    orders: int32 [P][n].  Outputs: offsets int64 [P][n] (None unless want_offsets),
    peaks int64 [P], best_offsets int64 [n] (None unless want_best_offsets),
    best_plan int32 [1], status int32 [1].  `out` may carry preallocated outputs.
    """
    return _plan(lib.stalloc_plan, "stalloc_plan", (), size, t_alloc, t_free, t_end, orders, want_offsets, want_best_offsets,
                 stream, workspace_cache, out)


def stalloc_plan_sized(size, t_alloc, t_free, t_end: int, orders, largest_size: int, granule: int, *,
                       want_offsets: bool = True, want_best_offsets: bool = True, stream=None,
                       workspace_cache: Optional[Dict] = None, out: Optional[Dict] = None) -> Dict[str, torch.Tensor]:
    """stalloc_plan for a caller that knows an upper bound of its sizes and a power of two dividing them all."""
    return _plan(lib.stalloc_plan_sized, "stalloc_plan_sized", (int(largest_size), int(granule)), size, t_alloc, t_free, t_end,
                 orders, want_offsets, want_best_offsets, stream, workspace_cache, out)


def _plan(fn, name, extra, size, t_alloc, t_free, t_end, orders, want_offsets, want_best_offsets, stream, workspace_cache, out):
    tr = _trace(size, t_alloc, t_free, t_end)
    if orders.dim() != 2 or orders.shape[1] != tr.n:
        raise ValueError("orders must be [P][n]")
    P, n, dev = orders.shape[0], tr.n, size.device
    out = dict(out) if out else {}
    if want_offsets and out.get("offsets") is None:
        out["offsets"] = torch.empty((P, n), dtype=torch.int64, device=dev)
    if not want_offsets:
        out["offsets"] = None
    if out.get("peaks") is None:
        out["peaks"] = torch.empty(P, dtype=torch.int64, device=dev)
    if want_best_offsets and out.get("best_offsets") is None:
        out["best_offsets"] = torch.empty(n, dtype=torch.int64, device=dev)
    if not want_best_offsets:
        out["best_offsets"] = None
    if out.get("best_plan") is None:
        out["best_plan"] = torch.empty(1, dtype=torch.int32, device=dev)
    if out.get("status") is None:
        out["status"] = torch.empty(1, dtype=torch.int32, device=dev)
    args = (ctypes.byref(tr), _dev(orders, torch.int32, "orders"), P,
            _dev(out["offsets"], torch.int64, "offsets"), _dev(out["peaks"], torch.int64, "peaks"),
            _dev(out["best_offsets"], torch.int64, "best_offsets"),
            _dev(out["best_plan"], torch.int32, "best_plan"), _dev(out["status"], torch.int32, "status")) + tuple(extra)
    need = ctypes.c_size_t(0)
    _check(fn(*args, None, ctypes.byref(need), None), name + "(workspace query)")
    ws = _workspace(need.value, dev, workspace_cache)
    have = ctypes.c_size_t(ws.numel())
    _check(fn(*args, ws.data_ptr(), ctypes.byref(have), _stream(stream)), name)
    out["workspace"] = ws
    out["workspace_bytes"] = need.value
    return out


def stalloc_plan_report(plan: Dict[str, torch.Tensor], *, stream=None) -> Dict[str, int]:
    """What the stalloc_plan call that produced `plan` did (synchronises): kernel name, address granule, ..."""
    info = _PlanInfo()
    _check(lib.stalloc_plan_report(plan["workspace"].data_ptr(), ctypes.byref(info), _stream(stream)), "stalloc_plan_report")
    return {"kernel": KERNELS.get(info.kernel, str(info.kernel)), "granule_log2": info.granule_log2,
            "granules": info.granules, "plans_64bit": info.plans_64bit,
            "lifetime_threshold": info.lifetime_threshold, "long_requests": info.long_requests,
            "address_bits": info.address_bits, "large_size": info.large_size, "large_requests": info.large_requests,
            "list_entry_bytes": info.list_entry_bytes}


def stalloc_probe(what: int, buffer: torch.Tensor, iters: int = 0, *, stream=None) -> int:
    """Enqueue one probe kernel (0 copy, 1 LDS read, 2 integer ALU) on `buffer` (uint8); returns its work."""
    done = ctypes.c_uint64(0)
    _check(lib.stalloc_probe(int(what), _dev(buffer, torch.uint8, "buffer"), buffer.numel(), int(iters),
                             ctypes.byref(done), _stream(stream)), "stalloc_probe")
    return int(done.value)


def stalloc_validate(size, t_alloc, t_free, t_end: int, offsets, *, stream=None,
                     workspace_cache: Optional[Dict] = None) -> Dict[str, torch.Tensor]:
    """offsets int64 [P][n] -> conflicts int64 [P], first_pair int32 [P][2] (-1, -1 when valid)."""
    tr = _trace(size, t_alloc, t_free, t_end)
    if offsets.dim() != 2 or offsets.shape[1] != tr.n:
        raise ValueError("offsets must be [P][n]")
    P, dev = offsets.shape[0], size.device
    out = {"conflicts": torch.empty(P, dtype=torch.int64, device=dev),
           "first_pair": torch.empty((P, 2), dtype=torch.int32, device=dev),
           "status": torch.empty(1, dtype=torch.int32, device=dev)}
    args = (ctypes.byref(tr), _dev(offsets, torch.int64, "offsets"), P, out["conflicts"].data_ptr(),
            out["first_pair"].data_ptr(), out["status"].data_ptr())
    need = ctypes.c_size_t(0)
    _check(lib.stalloc_validate(*args, None, ctypes.byref(need), None), "stalloc_validate(workspace query)")
    ws = _workspace(need.value, dev, workspace_cache)
    have = ctypes.c_size_t(ws.numel())
    _check(lib.stalloc_validate(*args, ws.data_ptr(), ctypes.byref(have), _stream(stream)), "stalloc_validate")
    out["workspace"] = ws
    return out


def stalloc_lower_bound(size, t_alloc, t_free, t_end: int, *, stream=None,
                        workspace_cache: Optional[Dict] = None) -> Dict[str, torch.Tensor]:
    """-> lower_bound int64 [1], t_at_max int32 [1], status int32 [1]."""
    tr = _trace(size, t_alloc, t_free, t_end)
    dev = size.device
    out = {"lower_bound": torch.empty(1, dtype=torch.int64, device=dev),
           "t_at_max": torch.empty(1, dtype=torch.int32, device=dev),
           "status": torch.empty(1, dtype=torch.int32, device=dev)}
    args = (ctypes.byref(tr), out["lower_bound"].data_ptr(), out["t_at_max"].data_ptr(), out["status"].data_ptr())
    need = ctypes.c_size_t(0)
    _check(lib.stalloc_lower_bound(*args, None, ctypes.byref(need), None), "stalloc_lower_bound(workspace query)")
    ws = _workspace(need.value, dev, workspace_cache)
    have = ctypes.c_size_t(ws.numel())
    _check(lib.stalloc_lower_bound(*args, ws.data_ptr(), ctypes.byref(have), _stream(stream)), "stalloc_lower_bound")
    out["workspace"] = ws
    return out


def stalloc_lower_bound_static(size, t_alloc, t_free, t_end: int, *, out: Dict[str, torch.Tensor],
                               stream=None) -> Dict[str, torch.Tensor]:
    """stalloc_lower_bound without a workspace; `out` carries the preallocated outputs
    (lower_bound int64 [1], t_at_max int32 [1], status int32 [1]), so nothing is allocated here either."""
    tr = _trace(size, t_alloc, t_free, t_end)
    _check(lib.stalloc_lower_bound_static(ctypes.byref(tr), _dev(out["lower_bound"], torch.int64, "lower_bound"),
                                          _dev(out["t_at_max"], torch.int32, "t_at_max"),
                                          _dev(out["status"], torch.int32, "status"), _stream(stream)),
           "stalloc_lower_bound_static")
    return out


def stalloc_reusable_space(size, t_alloc, t_free, t_end: int, offsets, windows, max_ranges: int, *, stream=None,
                           workspace_cache: Optional[Dict] = None) -> Dict[str, torch.Tensor]:
    """offsets int64 [n], windows int32 [k][2] -> ranges int64 [k][max_ranges][2], counts int32 [k],
    idle_bytes int64 [k], status int32 [1]."""
    tr = _trace(size, t_alloc, t_free, t_end)
    if offsets.dim() != 1 or offsets.numel() != tr.n:
        raise ValueError("offsets must be [n]")
    if windows.dim() != 2 or windows.shape[1] != 2:
        raise ValueError("windows must be [k][2]")
    k, dev = windows.shape[0], size.device
    out = {"ranges": torch.empty((k, max_ranges, 2), dtype=torch.int64, device=dev) if max_ranges else None,
           "counts": torch.empty(k, dtype=torch.int32, device=dev),
           "idle_bytes": torch.empty(k, dtype=torch.int64, device=dev),
           "status": torch.empty(1, dtype=torch.int32, device=dev)}
    args = (ctypes.byref(tr), _dev(offsets, torch.int64, "offsets"), _dev(windows, torch.int32, "windows"), k,
            int(max_ranges), out["ranges"].data_ptr() if max_ranges else None, out["counts"].data_ptr(),
            out["idle_bytes"].data_ptr(), out["status"].data_ptr())
    need = ctypes.c_size_t(0)
    _check(lib.stalloc_reusable_space(*args, None, ctypes.byref(need), None), "stalloc_reusable_space(workspace query)")
    ws = _workspace(need.value, dev, workspace_cache)
    have = ctypes.c_size_t(ws.numel())
    _check(lib.stalloc_reusable_space(*args, ws.data_ptr(), ctypes.byref(have), _stream(stream)), "stalloc_reusable_space")
    out["workspace"] = ws
    return out


def check_status(out: Dict[str, torch.Tensor], where: str = "stalloc") -> None:
    """Synchronising read of the device status word; raises StallocError when non-zero."""
    code = int(out["status"].item())
    if code != 0:
        raise StallocError(code, where)


def trace_to_device(trace, device="cuda"):
    """numpy trace (size uint64, t_alloc/t_free uint32) -> (size, t_alloc, t_free) device tensors."""
    import numpy as np
    size = torch.from_numpy(np.ascontiguousarray(trace.size).view(np.int64)).to(device)
    ta = torch.from_numpy(np.ascontiguousarray(trace.t_alloc).view(np.int32)).to(device)
    tf = torch.from_numpy(np.ascontiguousarray(trace.t_free).view(np.int32)).to(device)
    return size, ta, tf


def stalloc_memory_layers(size, t_alloc, t_free, t_end: int, *, stream=None,
                          workspace_cache: Optional[Dict] = None) -> Dict[str, torch.Tensor]:
    """-> layer_of int32 [n], n_layers int32 [1], layer_size int64 [n], layer_t_alloc / layer_t_free int32 [n]
    (the first n_layers entries are written), status int32 [1]."""
    tr = _trace(size, t_alloc, t_free, t_end)
    dev, n = size.device, tr.n
    out = {"layer_of": torch.empty(n, dtype=torch.int32, device=dev),
           "n_layers": torch.empty(1, dtype=torch.int32, device=dev),
           "layer_size": torch.empty(n, dtype=torch.int64, device=dev),
           "layer_t_alloc": torch.empty(n, dtype=torch.int32, device=dev),
           "layer_t_free": torch.empty(n, dtype=torch.int32, device=dev),
           "status": torch.empty(1, dtype=torch.int32, device=dev)}
    args = (ctypes.byref(tr), out["layer_of"].data_ptr(), out["n_layers"].data_ptr(), out["layer_size"].data_ptr(),
            out["layer_t_alloc"].data_ptr(), out["layer_t_free"].data_ptr(), out["status"].data_ptr())
    need = ctypes.c_size_t(0)
    _check(lib.stalloc_memory_layers(*args, None, ctypes.byref(need), None), "stalloc_memory_layers(workspace query)")
    ws = _workspace(need.value, dev, workspace_cache)
    have = ctypes.c_size_t(ws.numel())
    _check(lib.stalloc_memory_layers(*args, ws.data_ptr(), ctypes.byref(have), _stream(stream)), "stalloc_memory_layers")
    out["workspace"] = ws
    return out


def stalloc_expand_layers(layer_of, layer_offsets, *, stream=None) -> Dict[str, torch.Tensor]:
    """layer_of int32 [n], layer_offsets int64 [P][n_layers] -> offsets int64 [P][n], status int32 [1]."""
    if layer_of.dim() != 1 or layer_offsets.dim() != 2:
        raise ValueError("layer_of must be [n] and layer_offsets [P][n_layers]")
    n, (P, n_layers), dev = layer_of.numel(), layer_offsets.shape, layer_of.device
    out = {"offsets": torch.empty((P, n), dtype=torch.int64, device=dev),
           "status": torch.empty(1, dtype=torch.int32, device=dev)}
    _check(lib.stalloc_expand_layers(n, P, _dev(layer_of, torch.int32, "layer_of"),
                                     _dev(layer_offsets, torch.int64, "layer_offsets"), n_layers,
                                     out["offsets"].data_ptr(), out["status"].data_ptr(), _stream(stream)),
           "stalloc_expand_layers")
    return out


def stalloc_tmp(size, t_alloc, t_free, t_end: int, extents, *, stream=None,
                workspace_cache: Optional[Dict] = None) -> Dict[str, torch.Tensor]:
    """extents int64 [P] (`peaks` of stalloc_plan) -> tmp float64 [P], status int32 [1]."""
    tr = _trace(size, t_alloc, t_free, t_end)
    if extents.dim() != 1:
        raise ValueError("extents must be [P]")
    P, dev = extents.numel(), size.device
    out = {"tmp": torch.empty(P, dtype=torch.float64, device=dev),
           "status": torch.empty(1, dtype=torch.int32, device=dev)}
    args = (ctypes.byref(tr), _dev(extents, torch.int64, "extents"), P, out["tmp"].data_ptr(), out["status"].data_ptr())
    need = ctypes.c_size_t(0)
    _check(lib.stalloc_tmp(*args, None, ctypes.byref(need), None), "stalloc_tmp(workspace query)")
    ws = _workspace(need.value, dev, workspace_cache)
    have = ctypes.c_size_t(ws.numel())
    _check(lib.stalloc_tmp(*args, ws.data_ptr(), ctypes.byref(have), _stream(stream)), "stalloc_tmp")
    out["workspace"] = ws
    return out


def stalloc_fuse_groups(size, t_alloc, t_free, t_end: int, members, pair_begin, count1, largest_pair: int, *,
                        stream=None, workspace_cache: Optional[Dict] = None) -> Dict[str, torch.Tensor]:
    """members int32 [m], pair_begin int32 [k+1], count1 int32 [k], largest_pair = the largest pair's size ->
    order int32 [m], addr int64 [m], extents int64 [k][3], accepted int32 [k], status int32 [1]."""
    tr = _trace(size, t_alloc, t_free, t_end)
    k, m, dev = count1.numel(), members.numel(), size.device
    if pair_begin.numel() != k + 1:
        raise ValueError("pair_begin must hold k + 1 entries")
    out = {"order": torch.empty(m, dtype=torch.int32, device=dev), "addr": torch.empty(m, dtype=torch.int64, device=dev),
           "extents": torch.empty((k, 3), dtype=torch.int64, device=dev),
           "accepted": torch.empty(k, dtype=torch.int32, device=dev),
           "status": torch.empty(1, dtype=torch.int32, device=dev)}
    args = (ctypes.byref(tr), _dev(members, torch.int32, "members"), _dev(pair_begin, torch.int32, "pair_begin"),
            _dev(count1, torch.int32, "count1"), k, m, int(largest_pair), out["order"].data_ptr(), out["addr"].data_ptr(),
            out["extents"].data_ptr(), out["accepted"].data_ptr(), out["status"].data_ptr())
    need = ctypes.c_size_t(0)
    _check(lib.stalloc_fuse_groups(*args, None, ctypes.byref(need), None), "stalloc_fuse_groups(workspace query)")
    ws = _workspace(need.value, dev, workspace_cache)
    have = ctypes.c_size_t(ws.numel())
    _check(lib.stalloc_fuse_groups(*args, ws.data_ptr(), ctypes.byref(have), _stream(stream)), "stalloc_fuse_groups")
    out["workspace"] = ws
    return out


def stalloc_make_orders(size, t_alloc, t_free, t_end: int, P: int, *, seed: int = 1000, first_plan: int = 0,
                        stream=None, workspace_cache: Optional[Dict] = None) -> Dict[str, torch.Tensor]:
    """-> orders int32 [P][n] (rows first_plan .. first_plan + P - 1), status int32 [1]."""
    tr = _trace(size, t_alloc, t_free, t_end)
    dev = size.device
    out = {"orders": torch.empty((P, tr.n), dtype=torch.int32, device=dev),
           "status": torch.empty(1, dtype=torch.int32, device=dev)}
    args = (ctypes.byref(tr), int(first_plan), int(P), int(seed), out["orders"].data_ptr(), out["status"].data_ptr())
    need = ctypes.c_size_t(0)
    _check(lib.stalloc_make_orders(*args, None, ctypes.byref(need), None), "stalloc_make_orders(workspace query)")
    ws = _workspace(need.value, dev, workspace_cache)
    have = ctypes.c_size_t(ws.numel())
    _check(lib.stalloc_make_orders(*args, ws.data_ptr(), ctypes.byref(have), _stream(stream)), "stalloc_make_orders")
    out["workspace"] = ws
    return out
