"""Thin ctypes binding of libkvl.so: argument marshalling only.

Every step of the load path runs inside the library's HIP kernels and host
code; this module turns Python objects (NumPy block tables, torch tensors used
as raw device or pinned-host memory, torch streams) into the pointers and sizes
of the C ABI declared in include/kvl.h, and checks buffer sizes that the C side
cannot know.  There is no fallback: if the library is missing and cannot be
built, importing fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch  # first: the library must bind to the HIP runtime torch has loaded

from . import build as _build

KVL_MAX_PLANES = 4
KVL_OK, KVL_EINVAL, KVL_ERANGE, KVL_EALIAS, KVL_ESPACE, KVL_EHIP, KVL_ENOMEM = 0, -1, -2, -3, -4, -5, -6
KVL_ENOSYS = -7
KVL_GATHER, KVL_SCATTER, KVL_HOST_ONLY, KVL_NO_MERGE = 1, 2, 4, 8
KVL_TOKENS_APPEND, KVL_TOKENS_ALL = 16, 32
KVL_NO_POINTER_CHECKS = 64
KVL_CALLER_SYNCS = 128


class KvlError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        msg = f"{what}: {_lib.kvl_strerror(code).decode()} ({code})"
        if code == KVL_EHIP:
            msg += f" [hip {_lib.kvl_last_hip_error()}: {_lib.kvl_last_hip_error_string().decode()}]"
        super().__init__(msg)


class kvl_layout_t(C.Structure):
    _fields_ = [("n_layers", C.c_uint32), ("block_tokens", C.c_uint32), ("n_planes", C.c_uint32),
                ("row_bytes", C.c_uint32 * KVL_MAX_PLANES), ("pool_blocks", C.c_uint64)]


class kvl_request_t(C.Structure):
    _fields_ = [("hit_tokens", C.c_uint32), ("append_tokens", C.c_uint32), ("n_blocks", C.c_uint32),
                ("block_table", C.POINTER(C.c_int32))]


class kvl_unit_t(C.Structure):
    _fields_ = [("pool_row", C.c_uint32), ("xfer_row", C.c_uint32), ("n_rows", C.c_uint32),
                ("block_index", C.c_uint32)]


class kvl_tuning_t(C.Structure):
    _fields_ = [("unit_bytes", C.c_uint32), ("block_threads", C.c_uint32), ("variant", C.c_uint32),
                ("max_groups", C.c_uint32)]


class kvl_ceiling_t(C.Structure):
    _fields_ = [("mode", C.c_uint32), ("block_bytes", C.c_uint32), ("hopping_side", C.c_uint32),
                ("skew_bytes", C.c_uint32), ("hop_blocks_log2", C.c_uint32)]


class kvl_chunk_t(C.Structure):
    _fields_ = [("plane", C.c_uint32), ("unit_begin", C.c_uint32), ("unit_end", C.c_uint32),
                ("reserved", C.c_uint32), ("host_offset", C.c_uint64), ("bytes", C.c_uint64)]


class kvl_probe_t(C.Structure):
    _fields_ = [("plane", C.c_uint32), ("reserved", C.c_uint32), ("byte_offset", C.c_uint64)]


HOST_FILL_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64)
COMPUTE_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p), C.c_void_p)


class kvl_stream_cfg_t(C.Structure):
    _fields_ = [("n_layers", C.c_uint32), ("n_host_slots", C.c_uint32),
                ("host_layers", C.POINTER(C.c_void_p)),
                ("n_dev_slots", C.c_uint32),
                ("dev_slot_planes", C.POINTER(C.c_void_p)),
                ("dev_staging", C.c_void_p), ("staging_bytes", C.c_uint64), ("chunk_bytes", C.c_uint64),
                ("compute_us", C.c_uint32), ("n_probes", C.c_uint32),
                ("probes", C.POINTER(kvl_probe_t)), ("probe_out", C.c_void_p),
                ("snapshot_planes", C.POINTER(C.c_void_p)),
                ("host_fill", HOST_FILL_FN), ("host_fill_user", C.c_void_p),
                ("copy_stream", C.c_void_p), ("kernel_stream", C.c_void_p), ("compute_stream", C.c_void_p),
                ("full_blocks", C.c_void_p), ("full_blocks_bytes", C.c_uint64),
                ("compute", COMPUTE_FN), ("compute_user", C.c_void_p),
                ("out_plan", C.c_void_p), ("n_out_host_slots", C.c_uint32),
                ("out_host_layers", C.POINTER(C.c_void_p)), ("out_staging", C.c_void_p),
                ("out_staging_bytes", C.c_uint64), ("out_chunk_bytes", C.c_uint64),
                ("host_drain", HOST_FILL_FN), ("host_drain_user", C.c_void_p)]


class kvl_stream_stats_t(C.Structure):
    _fields_ = [("total_ms", C.c_double), ("h2d_bytes", C.c_double), ("link_gbps", C.c_double),
                ("exposed_ms", C.c_double), ("t_loaded", C.POINTER(C.c_float)),
                ("t_compute_begin", C.POINTER(C.c_float)), ("t_compute_end", C.POINTER(C.c_float)),
                ("t_out_done", C.POINTER(C.c_float)), ("d2h_bytes", C.c_double), ("out_gbps", C.c_double)]


# every symbol include/kvl.h declares, with its C signature
_PLAN_P = C.c_void_p
_SIGNATURES = {
    "kvl_plan": (C.c_int, [C.POINTER(kvl_layout_t), C.POINTER(kvl_request_t), C.c_uint32, C.c_uint32,
                           C.POINTER(_PLAN_P)]),
    "kvl_plan_tuned": (C.c_int, [C.POINTER(kvl_layout_t), C.POINTER(kvl_request_t), C.c_uint32, C.c_uint32,
                                 C.POINTER(kvl_tuning_t), C.POINTER(_PLAN_P)]),
    "kvl_plan_destroy": (None, [_PLAN_P]),
    "kvl_release_cached_memory": (None, []),
    "kvl_plan_pair": (C.c_int, [_PLAN_P, _PLAN_P, C.POINTER(_PLAN_P)]),
    "kvl_move_layer": (C.c_int, [_PLAN_P, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_void_p]),
    "kvl_plan_set_tuning": (C.c_int, [_PLAN_P, C.POINTER(kvl_tuning_t)]),
    "kvl_plan_payload_bytes": (C.c_int, [_PLAN_P, C.POINTER(C.c_uint64)]),
    "kvl_plan_hit_tokens": (C.c_int, [_PLAN_P, C.POINTER(C.c_uint64)]),
    "kvl_plan_n_units": (C.c_int, [_PLAN_P, C.POINTER(C.c_uint64)]),
    "kvl_plan_get_units": (C.c_int, [_PLAN_P, C.POINTER(kvl_unit_t), C.c_uint64, C.POINTER(C.c_uint64)]),
    "kvl_plan_get_chunks": (C.c_int, [_PLAN_P, C.c_uint64, C.POINTER(kvl_chunk_t), C.c_uint64,
                                      C.POINTER(C.c_uint64)]),
    "kvl_pack_layer": (C.c_int, [_PLAN_P, C.POINTER(C.c_void_p), C.c_void_p, C.c_uint64, C.c_void_p]),
    "kvl_unpack_layer": (C.c_int, [_PLAN_P, C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p), C.c_void_p]),
    "kvl_unpack_layer_noalloc": (C.c_int, [C.POINTER(kvl_layout_t), C.POINTER(kvl_request_t), C.c_uint32, C.c_uint32,
                                           C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p), C.c_void_p]),
    "kvl_h2d_unpack_layer": (C.c_int, [_PLAN_P, C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64,
                                       C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p]),
    "kvl_plan_fullblock_geometry": (C.c_int, [_PLAN_P, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]),
    "kvl_fullblocks_to_pool_layer": (C.c_int, [_PLAN_P, C.c_void_p, C.c_uint64, C.c_uint32,
                                               C.POINTER(C.c_void_p), C.c_void_p]),
    "kvl_pool_to_fullblocks_layer": (C.c_int, [_PLAN_P, C.POINTER(C.c_void_p), C.c_uint32, C.c_void_p,
                                               C.c_uint64, C.c_void_p]),
    "kvl_d2h_fullblocks_layer": (C.c_int, [_PLAN_P, C.POINTER(C.c_void_p), C.c_uint32, C.c_void_p, C.c_uint64,
                                           C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]),
    "kvl_d2h_pack_layer": (C.c_int, [_PLAN_P, C.POINTER(C.c_void_p), C.c_void_p, C.c_uint64, C.c_uint64,
                                     C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]),
    "kvl_h2d_fullblocks_layer": (C.c_int, [_PLAN_P, C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p, C.c_uint64,
                                           C.c_uint64, C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p]),
    "kvl_plan_set_lane_cu_mask": (C.c_int, [_PLAN_P, C.POINTER(C.c_uint32), C.c_uint32]),
    "kvl_h2d_blockwise_layer": (C.c_int, [_PLAN_P, C.c_void_p, C.POINTER(C.c_void_p), C.c_void_p,
                                          C.POINTER(C.c_uint64)]),
    "kvl_h2d_blockwise_batched_layer": (C.c_int, [_PLAN_P, C.c_void_p, C.POINTER(C.c_void_p), C.c_void_p,
                                                  C.POINTER(C.c_uint64)]),
    "kvl_stream_layers": (C.c_int, [_PLAN_P, C.POINTER(kvl_stream_cfg_t), C.POINTER(kvl_stream_stats_t)]),
    "kvl_measure_h2d_peak": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p,
                                       C.POINTER(C.c_double)]),
    "kvl_copy_linear": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]),
    "kvl_check_buffer": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int]),
    "kvl_ceiling_kernel": (C.c_int, [C.POINTER(kvl_ceiling_t), C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64,
                                     C.c_uint64, C.c_void_p, C.c_void_p]),
    "kvl_strerror": (C.c_char_p, [C.c_int]),
    "kvl_last_hip_error": (C.c_int, []),
    "kvl_last_hip_error_string": (C.c_char_p, []),
    "kvl_variant_name": (C.c_char_p, [C.c_uint32]),
    "kvl_version": (C.c_char_p, []),
}


def _load() -> C.CDLL:
    path = _build.LIB
    if not os.path.exists(path):
        _build.build()          # nothing built yet: build once, in-tree
    lib = C.CDLL(path)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)  # AttributeError if the library lacks a declared symbol
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()
LIB_PATH = _build.LIB


def _check(rc: int, what: str) -> None:
    if rc != KVL_OK:
        raise KvlError(rc, what)


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _nbytes(t: torch.Tensor) -> int:
    return t.numel() * t.element_size()


def _dev(t: torch.Tensor, what: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{what}: need a contiguous device tensor")
    return t.data_ptr()


class Plan:
    """Owner of a kvl_plan_t*."""

    def __init__(self, handle: int, layout: kvl_layout_t, flags: int):
        self._h = C.c_void_p(handle)
        self.layout = layout
        self.flags = flags

    def destroy(self) -> None:
        if self._h:
            _lib.kvl_plan_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()
        return False

    @property
    def handle(self) -> C.c_void_p:
        if not self._h:
            raise ValueError("plan destroyed")
        return self._h

    @property
    def n_planes(self) -> int:
        return int(self.layout.n_planes)

    def plane_bytes(self, p: int) -> int:
        return int(self.layout.pool_blocks) * int(self.layout.block_tokens) * int(self.layout.row_bytes[p])

    @property
    def payload_bytes(self) -> int:
        v = C.c_uint64()
        _check(_lib.kvl_plan_payload_bytes(self.handle, C.byref(v)), "kvl_plan_payload_bytes")
        return int(v.value)

    @property
    def hit_tokens(self) -> int:
        v = C.c_uint64()
        _check(_lib.kvl_plan_hit_tokens(self.handle, C.byref(v)), "kvl_plan_hit_tokens")
        return int(v.value)

    @property
    def n_units(self) -> int:
        v = C.c_uint64()
        _check(_lib.kvl_plan_n_units(self.handle, C.byref(v)), "kvl_plan_n_units")
        return int(v.value)

    def units(self) -> np.ndarray:
        """Descriptors as an (n, 4) uint32 array: pool_row, xfer_row, n_rows, block_index."""
        n = self.n_units
        out = np.zeros((n, 4), dtype=np.uint32)
        got = C.c_uint64()
        _check(_lib.kvl_plan_get_units(self.handle, out.ctypes.data_as(C.POINTER(kvl_unit_t)), n,
                                       C.byref(got)), "kvl_plan_get_units")
        return out

    def chunks(self, chunk_bytes: int) -> List[dict]:
        n = C.c_uint64()
        _check(_lib.kvl_plan_get_chunks(self.handle, chunk_bytes, None, 0, C.byref(n)), "kvl_plan_get_chunks")
        arr = (kvl_chunk_t * max(1, n.value))()
        _check(_lib.kvl_plan_get_chunks(self.handle, chunk_bytes, arr, n.value, C.byref(n)),
               "kvl_plan_get_chunks")
        return [dict(plane=c.plane, unit_begin=c.unit_begin, unit_end=c.unit_end,
                     host_offset=c.host_offset, bytes=c.bytes) for c in arr[:n.value]]

    def fullblock_geometry(self):
        """(bytes of one Full Block, Full Blocks a buffer of this plan's ranges holds)."""
        a, b = C.c_uint64(), C.c_uint64()
        _check(_lib.kvl_plan_fullblock_geometry(self.handle, C.byref(a), C.byref(b)), "kvl_plan_fullblock_geometry")
        return int(a.value), int(b.value)

    def set_lane_cu_mask(self, enabled_cus: Optional[Sequence[int]]) -> None:
        """Confine the host-buffer path's scatter kernels to the given compute units (None: no mask)."""
        if not enabled_cus:
            _check(_lib.kvl_plan_set_lane_cu_mask(self.handle, None, 0), "kvl_plan_set_lane_cu_mask")
            return
        words = max(enabled_cus) // 32 + 1
        arr = (C.c_uint32 * words)()
        for cu in enabled_cus:
            arr[cu // 32] |= 1 << (cu % 32)
        _check(_lib.kvl_plan_set_lane_cu_mask(self.handle, arr, words), "kvl_plan_set_lane_cu_mask")

    def set_tuning(self, block_threads: int = 0, variant: int = 0, max_groups: int = 0) -> None:
        t = kvl_tuning_t(0, block_threads, variant, max_groups)
        _check(_lib.kvl_plan_set_tuning(self.handle, C.byref(t)), "kvl_plan_set_tuning")


def make_layout(n_layers: int, block_tokens: int, row_bytes: Sequence[int], pool_blocks: int) -> kvl_layout_t:
    if len(row_bytes) > KVL_MAX_PLANES:
        raise ValueError("too many planes")
    lay = kvl_layout_t()
    lay.n_layers, lay.block_tokens, lay.n_planes, lay.pool_blocks = n_layers, block_tokens, len(row_bytes), pool_blocks
    for i, r in enumerate(row_bytes):
        lay.row_bytes[i] = int(r)
    return lay


def _requests(hit, app, tables: Sequence[np.ndarray]):
    """(kvl_request_t array, n, arrays to keep alive while it is in use)"""
    hit = np.asarray(hit, dtype=np.uint32)
    app = np.asarray(app, dtype=np.uint32)
    n = int(hit.shape[0])
    if len(tables) != n or app.shape[0] != n:
        raise ValueError("hit, app and tables must have one entry per request")
    keep = [np.ascontiguousarray(np.asarray(t, dtype=np.int32)) for t in tables]
    reqs = (kvl_request_t * max(1, n))()
    for r in range(n):
        reqs[r].hit_tokens = int(hit[r])
        reqs[r].append_tokens = int(app[r])
        reqs[r].n_blocks = int(keep[r].size)
        reqs[r].block_table = keep[r].ctypes.data_as(C.POINTER(C.c_int32)) if keep[r].size else None
    return reqs, n, keep


def kvl_plan(layout: kvl_layout_t, hit, app, tables: Sequence[np.ndarray], flags: int,
             unit_bytes: int = 0, block_threads: int = 0, variant: int = 0, max_groups: int = 0) -> Plan:
    """kvl_plan / kvl_plan_tuned: block tables -> copy descriptors (host; device upload unless HOST_ONLY)."""
    reqs, n, _keep = _requests(hit, app, tables)
    out = C.c_void_p()
    if unit_bytes or block_threads or variant or max_groups:
        t = kvl_tuning_t(unit_bytes, block_threads, variant, max_groups)
        rc = _lib.kvl_plan_tuned(C.byref(layout), reqs, n, flags, C.byref(t), C.byref(out))
    else:
        rc = _lib.kvl_plan(C.byref(layout), reqs, n, flags, C.byref(out))
    _check(rc, "kvl_plan")
    return Plan(out.value, layout, flags)


def _plane_ptrs(plan: Plan, planes: Sequence[torch.Tensor], what: str):
    if len(planes) != plan.n_planes:
        raise ValueError(f"{what}: expected {plan.n_planes} planes")
    arr = (C.c_void_p * plan.n_planes)()
    for p, t in enumerate(planes):
        arr[p] = _dev(t, what)
        if _nbytes(t) < plan.plane_bytes(p):
            raise ValueError(f"{what}: plane {p} holds {_nbytes(t)} bytes, pool needs {plan.plane_bytes(p)}")
    return arr


def kvl_pack_layer(plan: Plan, pool_planes: Sequence[torch.Tensor], xfer: torch.Tensor, stream=None) -> None:
    """xfer: a device tensor, or a pinned host tensor (the kernel then writes it over the host link)."""
    arr = _plane_ptrs(plan, pool_planes, "kvl_pack_layer pool")
    if isinstance(xfer, torch.Tensor) and not xfer.is_cuda:
        ptr = _pinned(xfer, "xfer", 0)
    else:
        ptr = _dev(xfer, "xfer")
    _check(_lib.kvl_pack_layer(plan.handle, arr, ptr, _nbytes(xfer), _stream_handle(stream)),
           "kvl_pack_layer")


def kvl_plan_pair(gather: Plan, scatter: Plan) -> Plan:
    """Join a gather plan and a scatter plan into one pool-to-pool plan for kvl_move_layer."""
    out = C.c_void_p()
    _check(_lib.kvl_plan_pair(gather.handle, scatter.handle, C.byref(out)), "kvl_plan_pair")
    p = Plan(out.value, gather.layout, gather.flags)
    p.dst_layout = scatter.layout
    return p


def kvl_move_layer(paired: Plan, src_pool_planes: Sequence[torch.Tensor],
                   dst_pool_planes: Sequence[torch.Tensor], stream=None) -> None:
    src = _plane_ptrs(paired, src_pool_planes, "kvl_move_layer source pool")
    dl = paired.dst_layout
    if len(dst_pool_planes) != paired.n_planes:
        raise ValueError("kvl_move_layer: wrong number of destination planes")
    dst = (C.c_void_p * paired.n_planes)()
    for p, t in enumerate(dst_pool_planes):
        need = int(dl.pool_blocks) * int(dl.block_tokens) * int(dl.row_bytes[p])
        if _nbytes(t) < need:
            raise ValueError(f"kvl_move_layer: destination plane {p} holds {_nbytes(t)} bytes, pool needs {need}")
        dst[p] = _dev(t, "kvl_move_layer destination pool")
    _check(_lib.kvl_move_layer(paired.handle, src, dst, _stream_handle(stream)), "kvl_move_layer")


def kvl_unpack_layer(plan: Plan, xfer: torch.Tensor, pool_planes: Sequence[torch.Tensor], stream=None) -> None:
    """xfer: a device tensor, or a pinned host tensor (the kernel then reads it over the host link)."""
    arr = _plane_ptrs(plan, pool_planes, "kvl_unpack_layer pool")
    if isinstance(xfer, torch.Tensor) and not xfer.is_cuda:
        ptr = _pinned(xfer, "xfer", 0)
    else:
        ptr = _dev(xfer, "xfer")
    _check(_lib.kvl_unpack_layer(plan.handle, ptr, _nbytes(xfer), arr, _stream_handle(stream)),
           "kvl_unpack_layer")


KVL_NOALLOC_MAX_UNITS = 524288


def kvl_unpack_layer_noalloc(layout: kvl_layout_t, hit, app, tables: Sequence[np.ndarray], flags: int,
                             xfer: torch.Tensor, pool_planes: Sequence[torch.Tensor], stream=None) -> None:
    """The scatter of kvl_plan + kvl_unpack_layer in one call that allocates nothing on the device."""
    reqs, n, _keep = _requests(hit, app, tables)
    if len(pool_planes) != int(layout.n_planes):
        raise ValueError(f"kvl_unpack_layer_noalloc: expected {int(layout.n_planes)} planes")
    arr = (C.c_void_p * int(layout.n_planes))()
    for p, t in enumerate(pool_planes):
        need = int(layout.pool_blocks) * int(layout.block_tokens) * int(layout.row_bytes[p])
        if _nbytes(t) < need:
            raise ValueError(f"kvl_unpack_layer_noalloc: plane {p} holds {_nbytes(t)} bytes, pool needs {need}")
        arr[p] = _dev(t, "kvl_unpack_layer_noalloc pool")
    ptr = _pinned(xfer, "xfer", 0) if (isinstance(xfer, torch.Tensor) and not xfer.is_cuda) else _dev(xfer, "xfer")
    _check(_lib.kvl_unpack_layer_noalloc(C.byref(layout), reqs, n, flags, ptr, _nbytes(xfer), arr,
                                         _stream_handle(stream)), "kvl_unpack_layer_noalloc")


KVL_CEILING_COPY, KVL_CEILING_READ, KVL_CEILING_WRITE = 0, 1, 2


def kvl_ceiling_kernel(mode: int, src: torch.Tensor, dst: torch.Tensor, nbytes: int, block_bytes: int = 0,
                       hopping_side: int = 0, skew_bytes: int = 0, hop_blocks_log2: int = 0,
                       block_table: Optional[torch.Tensor] = None, stream=None) -> None:
    """One launch of a reference stream (see kvl_ceiling_kernel in kvl.h); the caller times it."""
    c = kvl_ceiling_t(mode, block_bytes, hopping_side, skew_bytes, hop_blocks_log2)
    if block_table is not None and (block_table.dtype != torch.int32 or not block_table.is_cuda):
        raise TypeError("block_table: need an int32 device tensor")
    _check(_lib.kvl_ceiling_kernel(C.byref(c), _dev(src, "src"), _nbytes(src), _dev(dst, "dst"), _nbytes(dst), nbytes,
                                   _dev(block_table, "block_table") if block_table is not None else None,
                                   _stream_handle(stream)), "kvl_ceiling_kernel")


def _pinned(t: torch.Tensor, what: str, need: int) -> int:
    if not isinstance(t, torch.Tensor) or t.is_cuda or not t.is_pinned() or not t.is_contiguous():
        raise TypeError(f"{what}: need a contiguous pinned host tensor")
    if _nbytes(t) < need:
        raise ValueError(f"{what}: holds {_nbytes(t)} bytes, payload is {need}")
    return t.data_ptr()


def kvl_h2d_unpack_layer(plan: Plan, pinned_host_xfer: torch.Tensor, dev_staging: torch.Tensor,
                         chunk_bytes: int, pool_planes: Sequence[torch.Tensor],
                         copy_stream, kernel_stream) -> None:
    arr = _plane_ptrs(plan, pool_planes, "kvl_h2d_unpack_layer pool")
    host = _pinned(pinned_host_xfer, "pinned_host_xfer", plan.payload_bytes)
    stage = _dev(dev_staging, "staging") if dev_staging is not None else None
    stage_bytes = _nbytes(dev_staging) if dev_staging is not None else 0
    _check(_lib.kvl_h2d_unpack_layer(plan.handle, host, stage, stage_bytes,
                                     chunk_bytes, arr, _stream_handle(copy_stream),
                                     _stream_handle(kernel_stream)), "kvl_h2d_unpack_layer")


def _dev_or_pinned(t: torch.Tensor, what: str) -> int:
    if isinstance(t, torch.Tensor) and not t.is_cuda:
        return _pinned(t, what, 0)
    return _dev(t, what)


def kvl_fullblocks_to_pool_layer(plan: Plan, full_blocks: torch.Tensor, layer: int,
                                 pool_planes: Sequence[torch.Tensor], stream=None) -> None:
    """full_blocks: a device tensor or a pinned host tensor holding the plan's Full Blocks."""
    arr = _plane_ptrs(plan, pool_planes, "kvl_fullblocks_to_pool_layer pool")
    _check(_lib.kvl_fullblocks_to_pool_layer(plan.handle, _dev_or_pinned(full_blocks, "full_blocks"),
                                             _nbytes(full_blocks), layer, arr, _stream_handle(stream)),
           "kvl_fullblocks_to_pool_layer")


def kvl_d2h_fullblocks_layer(plan: Plan, pool_planes: Sequence[torch.Tensor], layer: int,
                             dev_staging: torch.Tensor, chunk_bytes: int, full_blocks: torch.Tensor,
                             kernel_stream, copy_stream) -> None:
    """Staged persist of one layer: converting kernels into dev_staging, runtime copies into the Full Blocks."""
    arr = _plane_ptrs(plan, pool_planes, "kvl_d2h_fullblocks_layer pool")
    _check(_lib.kvl_d2h_fullblocks_layer(plan.handle, arr, layer, _dev(dev_staging, "staging"),
                                         _nbytes(dev_staging), chunk_bytes,
                                         _dev_or_pinned(full_blocks, "full_blocks"), _nbytes(full_blocks),
                                         _stream_handle(kernel_stream), _stream_handle(copy_stream)),
           "kvl_d2h_fullblocks_layer")


def kvl_d2h_pack_layer(plan: Plan, pool_planes: Sequence[torch.Tensor], dev_staging: torch.Tensor,
                       chunk_bytes: int, pinned_host_xfer: torch.Tensor, kernel_stream, copy_stream) -> None:
    """Staged gather into a pinned host tensor: pack kernels into dev_staging, copy engine to the host."""
    arr = _plane_ptrs(plan, pool_planes, "kvl_d2h_pack_layer pool")
    _check(_lib.kvl_d2h_pack_layer(plan.handle, arr, _dev(dev_staging, "staging"), _nbytes(dev_staging),
                                   chunk_bytes, _pinned(pinned_host_xfer, "pinned_host_xfer", 0),
                                   _nbytes(pinned_host_xfer), _stream_handle(kernel_stream),
                                   _stream_handle(copy_stream)), "kvl_d2h_pack_layer")


def kvl_h2d_fullblocks_layer(plan: Plan, full_blocks: torch.Tensor, layer: int, dev_staging: torch.Tensor,
                             chunk_bytes: int, pool_planes: Sequence[torch.Tensor], copy_stream,
                             kernel_stream) -> None:
    """Staged Full-Block load of one layer: strided copies into dev_staging, converting kernels from there."""
    arr = _plane_ptrs(plan, pool_planes, "kvl_h2d_fullblocks_layer pool")
    _check(_lib.kvl_h2d_fullblocks_layer(plan.handle, _dev_or_pinned(full_blocks, "full_blocks"),
                                         _nbytes(full_blocks), layer, _dev(dev_staging, "staging"),
                                         _nbytes(dev_staging), chunk_bytes, arr, _stream_handle(copy_stream),
                                         _stream_handle(kernel_stream)), "kvl_h2d_fullblocks_layer")


def kvl_pool_to_fullblocks_layer(plan: Plan, pool_planes: Sequence[torch.Tensor], layer: int,
                                 full_blocks: torch.Tensor, stream=None) -> None:
    arr = _plane_ptrs(plan, pool_planes, "kvl_pool_to_fullblocks_layer pool")
    _check(_lib.kvl_pool_to_fullblocks_layer(plan.handle, arr, layer, _dev_or_pinned(full_blocks, "full_blocks"),
                                             _nbytes(full_blocks), _stream_handle(stream)),
           "kvl_pool_to_fullblocks_layer")


def kvl_h2d_blockwise_layer(plan: Plan, pinned_host_xfer: torch.Tensor, pool_planes: Sequence[torch.Tensor],
                            stream=None) -> int:
    """One hipMemcpyAsync per descriptor and plane (a measurement aid); returns the number of copies."""
    arr = _plane_ptrs(plan, pool_planes, "kvl_h2d_blockwise_layer pool")
    host = _pinned(pinned_host_xfer, "pinned_host_xfer", plan.payload_bytes)
    n = C.c_uint64()
    _check(_lib.kvl_h2d_blockwise_layer(plan.handle, host, arr, _stream_handle(stream), C.byref(n)),
           "kvl_h2d_blockwise_layer")
    return int(n.value)


def kvl_h2d_blockwise_batched_layer(plan: Plan, pinned_host_xfer: torch.Tensor,
                                    pool_planes: Sequence[torch.Tensor], stream=None) -> int:
    """The same copies in one hipMemcpyBatchAsync; raises KvlError(KVL_ENOSYS) if the runtime lacks it."""
    arr = _plane_ptrs(plan, pool_planes, "kvl_h2d_blockwise_batched_layer pool")
    host = _pinned(pinned_host_xfer, "pinned_host_xfer", plan.payload_bytes)
    n = C.c_uint64()
    _check(_lib.kvl_h2d_blockwise_batched_layer(plan.handle, host, arr, _stream_handle(stream), C.byref(n)),
           "kvl_h2d_blockwise_batched_layer")
    return int(n.value)


def kvl_stream_layers(plan: Plan, host_layers: Sequence[torch.Tensor],
                      dev_slots: Sequence[Sequence[torch.Tensor]], dev_staging: torch.Tensor,
                      chunk_bytes: int, compute_us: int, copy_stream, kernel_stream, compute_stream,
                      n_layers: int = 0, probes: Optional[Sequence[tuple]] = None,
                      probe_out: Optional[torch.Tensor] = None,
                      snapshots: Optional[Sequence[Sequence[torch.Tensor]]] = None,
                      host_fill=None, per_layer_times: bool = False,
                      full_blocks: Optional[torch.Tensor] = None, compute=None,
                      out_plan: Optional[Plan] = None, out_host_layers: Optional[Sequence[torch.Tensor]] = None,
                      out_staging: Optional[torch.Tensor] = None, out_chunk_bytes: int = 0,
                      host_drain=None) -> dict:
    """kvl_stream_layers; returns the stats as a dict.  host_fill(layer, slot_index) is an
    optional Python callable run where the storage read of that layer would deliver.
    compute(layer, slot_index, stream_handle) is an optional Python callable that enqueues
    the caller's own work for that layer on the compute stream (given as a raw handle; wrap
    it in torch.cuda.ExternalStream to use it from torch) in place of the synthetic kernel.
    out_plan (a gather plan over the same pool geometry) with out_host_layers (pinned tensors)
    adds the outflow: after each layer's compute its slot is gathered into a host buffer, staged
    through out_staging (out_chunk_bytes != 0) or written by the kernel itself;
    host_drain(layer, slot_index) is called when a layer has arrived in its buffer.
    With full_blocks (device or pinned host tensor) the layers are loaded from the storage
    layout instead; host_layers, dev_staging and chunk_bytes may then be None / 0."""
    L = n_layers or int(plan.layout.n_layers)
    P = plan.n_planes
    cfg = kvl_stream_cfg_t()
    cfg.n_layers = L
    need = plan.payload_bytes
    host_layers = host_layers or []
    H = len(host_layers)
    hl = (C.c_void_p * max(1, H))()
    for i, t in enumerate(host_layers):
        hl[i] = _pinned(t, f"host_layers[{i}]", need)
    cfg.n_host_slots, cfg.host_layers = H, hl
    if full_blocks is not None:
        cfg.full_blocks = _dev_or_pinned(full_blocks, "full_blocks")
        cfg.full_blocks_bytes = _nbytes(full_blocks)
    S = len(dev_slots)
    sp = (C.c_void_p * max(1, S * P))()
    for s, planes in enumerate(dev_slots):
        arr = _plane_ptrs(plan, planes, f"dev_slots[{s}]")
        for p in range(P):
            sp[s * P + p] = arr[p]
    cfg.n_dev_slots, cfg.dev_slot_planes = S, sp
    if dev_staging is not None:
        cfg.dev_staging = _dev(dev_staging, "staging")
        cfg.staging_bytes = _nbytes(dev_staging)
    cfg.chunk_bytes, cfg.compute_us = chunk_bytes, compute_us
    keep = []
    if probes:
        pa = (kvl_probe_t * len(probes))()
        for i, (plane, off) in enumerate(probes):
            pa[i].plane, pa[i].byte_offset = plane, off
        if probe_out is None or _nbytes(probe_out) < L * len(probes) * 16:
            raise ValueError("probe_out too small")
        cfg.n_probes, cfg.probes, cfg.probe_out = len(probes), pa, _dev(probe_out, "probe_out")
        keep.append(pa)
    if snapshots is not None:
        if len(snapshots) != L:
            raise ValueError("need one snapshot (or None) per layer")
        sn = (C.c_void_p * (L * P))()
        for l, planes in enumerate(snapshots):
            if planes is None:
                continue
            for p in range(P):
                if _nbytes(planes[p]) < plan.plane_bytes(p):
                    raise ValueError("snapshot plane too small")
                sn[l * P + p] = _dev(planes[p], "snapshot")
        cfg.snapshot_planes = sn
        keep.append(sn)
    if host_fill is not None:
        def _tramp(_user, layer, _slot_ptr, _bytes):
            try:
                host_fill(int(layer), int(layer) % H)
                return 0
            except Exception:  # surfaces as KVL_EINVAL from the call
                import traceback
                traceback.print_exc()
                return 1
        cb = HOST_FILL_FN(_tramp)
        cfg.host_fill = cb
        keep.append(cb)
    if compute is not None:
        def _ctramp(_user, layer, _planes, stream_ptr):
            try:
                compute(int(layer), int(layer) % S, int(stream_ptr or 0))
                return 0
            except Exception:  # surfaces as KVL_EINVAL from the call
                import traceback
                traceback.print_exc()
                return 1
        ccb = COMPUTE_FN(_ctramp)
        cfg.compute = ccb
        keep.append(ccb)
    if out_plan is not None:
        out_host_layers = list(out_host_layers or [])
        Ho = len(out_host_layers)
        oh = (C.c_void_p * max(1, Ho))()
        for i, t in enumerate(out_host_layers):
            oh[i] = _pinned(t, f"out_host_layers[{i}]", out_plan.payload_bytes)
        cfg.out_plan, cfg.n_out_host_slots, cfg.out_host_layers = out_plan.handle, Ho, oh
        keep.append(oh)
        if out_staging is not None:
            cfg.out_staging = _dev(out_staging, "out_staging")
            cfg.out_staging_bytes = _nbytes(out_staging)
        cfg.out_chunk_bytes = out_chunk_bytes
        if host_drain is not None:
            def _dtramp(_user, layer, _slot_ptr, _bytes):
                try:
                    host_drain(int(layer), int(layer) % Ho)
                    return 0
                except Exception:  # surfaces as KVL_EINVAL from the call
                    import traceback
                    traceback.print_exc()
                    return 1
            dcb = HOST_FILL_FN(_dtramp)
            cfg.host_drain = dcb
            keep.append(dcb)
    cfg.copy_stream = _stream_handle(copy_stream)
    cfg.kernel_stream = _stream_handle(kernel_stream)
    cfg.compute_stream = _stream_handle(compute_stream)
    st = kvl_stream_stats_t()
    times = None
    if per_layer_times:
        times = np.zeros((4, L), dtype=np.float32)
        fp = C.POINTER(C.c_float)
        st.t_loaded = times[0].ctypes.data_as(fp)
        st.t_compute_begin = times[1].ctypes.data_as(fp)
        st.t_compute_end = times[2].ctypes.data_as(fp)
        st.t_out_done = times[3].ctypes.data_as(fp)
    _check(_lib.kvl_stream_layers(plan.handle, C.byref(cfg), C.byref(st)), "kvl_stream_layers")
    out = dict(total_ms=st.total_ms, h2d_bytes=st.h2d_bytes, link_gbps=st.link_gbps, exposed_ms=st.exposed_ms,
               d2h_bytes=st.d2h_bytes, out_gbps=st.out_gbps)
    if times is not None:
        out.update(t_loaded=times[0], t_compute_begin=times[1], t_compute_end=times[2], t_out_done=times[3])
    return out


def kvl_measure_h2d_peak(pinned_host: torch.Tensor, dev: torch.Tensor, reps: int = 5, stream=None) -> float:
    n = min(_nbytes(pinned_host), _nbytes(dev))
    g = C.c_double()
    _check(_lib.kvl_measure_h2d_peak(_pinned(pinned_host, "pinned_host", 0), _dev(dev, "dev"), n, reps,
                                     _stream_handle(stream), C.byref(g)), "kvl_measure_h2d_peak")
    return float(g.value)


def kvl_copy_linear(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    n = _nbytes(src)
    if _nbytes(dst) < n:
        raise ValueError("dst smaller than src")
    _check(_lib.kvl_copy_linear(_dev(src, "src"), _dev(dst, "dst"), n, _stream_handle(stream)), "kvl_copy_linear")


def kvl_check_buffer(ptr: int, nbytes: int, allow_host: bool = False) -> int:
    """The library's own buffer check on a raw address; returns a KVL_* code."""
    return int(_lib.kvl_check_buffer(ptr, nbytes, int(allow_host)))


def kvl_release_cached_memory() -> None:
    _lib.kvl_release_cached_memory()


def kvl_strerror(code: int) -> str:
    return _lib.kvl_strerror(code).decode()


def kvl_variant_name(v: int) -> Optional[str]:
    s = _lib.kvl_variant_name(v)
    return s.decode() if s else None


def kvl_version() -> str:
    return _lib.kvl_version().decode()
