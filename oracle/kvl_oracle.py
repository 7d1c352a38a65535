"""ctypes binding of the C oracle (kvl_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this.  It never touches the HIP library and the HIP library never touches it.

The C file holds the definitions; this file adds only the per-layer compositions
(stream_layers, stream_layers_fullblocks) and the sharding of requests over host
threads.  Pins (tests/test_oracle_pins.py): both compositions are checked against
per-layer tags, with expected slot contents written out from the layout's defining
sentence (Appendix A.5) by NumPy reshapes, for several numbers of resident slots and
host buffers, and against each other on ragged ranges; mistakes planted in copies of
this file (wrong slot, wrong layer, H and S swapped, a lost request in the sharding)
must each trip a pin.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from typing import Iterator, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvl_oracle.c")
_LIB = os.path.join(_HERE, "libkvl_oracle.so")

OK, E_ARG, E_TABLE, E_BLOCK, E_DUP = 0, -1, -2, -3, -4

_lib = None


def build(force: bool = False) -> str:
    """Compile kvl_oracle.c with gcc into libkvl_oracle.so beside it."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-fPIC",
                               "-shared", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _bind(path: str):
    lib = C.CDLL(path)
    u32p, i32pp, u8pp = C.POINTER(C.c_uint32), C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_void_p)
    lib.kvo_total_hit_tokens.restype = C.c_uint64
    lib.kvo_total_hit_tokens.argtypes = [C.c_uint32, u32p]
    lib.kvo_payload_bytes.restype = C.c_uint64
    lib.kvo_payload_bytes.argtypes = [C.c_uint32, u32p, C.c_uint32, u32p]
    lib.kvo_check.restype = C.c_int
    lib.kvo_check.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, u32p, u32p, u32p, i32pp, C.c_int]
    lib.kvo_pack.restype = C.c_int
    lib.kvo_pack.argtypes = [C.c_uint32, C.c_uint32, u32p, C.c_uint32, u32p, i32pp,
                             u8pp, C.c_void_p, C.c_uint32, C.c_uint32]
    lib.kvo_unpack.restype = C.c_int
    lib.kvo_unpack.argtypes = [C.c_uint32, C.c_uint32, u32p, C.c_uint32, u32p, i32pp,
                               C.c_void_p, u8pp, C.c_uint32, C.c_uint32]
    u32p_n = C.POINTER(C.c_uint32)
    lib.kvo_pack_range.restype = C.c_int
    lib.kvo_pack_range.argtypes = [C.c_uint32, C.c_uint32, u32p, C.c_uint32, u32p_n, u32p, i32pp,
                                   u8pp, C.c_void_p, C.c_uint32, C.c_uint32]
    lib.kvo_unpack_range.restype = C.c_int
    lib.kvo_unpack_range.argtypes = [C.c_uint32, C.c_uint32, u32p, C.c_uint32, u32p_n, u32p, i32pp,
                                     C.c_void_p, u8pp, C.c_uint32, C.c_uint32]
    lib.kvo_check_range_scatter.restype = C.c_int
    lib.kvo_check_range_scatter.argtypes = [C.c_uint32, C.c_uint64, C.c_uint32, u32p_n, u32p, i32pp]
    lib.kvo_fullblock_bytes.restype = C.c_uint64
    lib.kvo_fullblock_bytes.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, u32p]
    lib.kvo_fullblock_count.restype = C.c_uint64
    lib.kvo_fullblock_count.argtypes = [C.c_uint32, C.c_uint32, u32p_n, u32p]
    for fn in (lib.kvo_fullblocks_to_pool, lib.kvo_pool_to_fullblocks):
        fn.restype = C.c_int
    lib.kvo_fullblocks_to_pool.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, u32p, C.c_uint32, u32p_n, u32p,
                                           i32pp, C.c_uint32, C.c_void_p, u8pp]
    lib.kvo_pool_to_fullblocks.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, u32p, C.c_uint32, u32p_n, u32p,
                                           i32pp, C.c_uint32, u8pp, C.c_void_p]
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


class use_library:
    """Context manager for tests that plant a mistake in a copy of the C source:
    route every call through another build of the oracle, then restore."""

    def __init__(self, path: str):
        self.path = path

    def __enter__(self):
        global _lib
        self.saved = _load()
        _lib = _bind(self.path)
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = self.saved
        return False


def _u32(a) -> Tuple[np.ndarray, "C._Pointer"]:
    arr = np.ascontiguousarray(np.asarray(a, dtype=np.uint32))
    return arr, arr.ctypes.data_as(C.POINTER(C.c_uint32))


def _tables(tables: Sequence[np.ndarray]):
    keep = [np.ascontiguousarray(np.asarray(t, dtype=np.int32)) for t in tables]
    arr = (C.POINTER(C.c_int32) * max(1, len(keep)))()
    for i, t in enumerate(keep):
        arr[i] = t.ctypes.data_as(C.POINTER(C.c_int32)) if t.size else None
    return keep, arr


def _planes(planes: Sequence[np.ndarray], writable: bool):
    for p in planes:
        if p.dtype != np.uint8 or not p.flags["C_CONTIGUOUS"]:
            raise TypeError("pool planes must be contiguous uint8 arrays")
        if writable and not p.flags["WRITEABLE"]:
            raise TypeError("pool plane is read-only")
    arr = (C.c_void_p * max(1, len(planes)))()
    for i, p in enumerate(planes):
        arr[i] = p.ctypes.data
    return arr


def total_hit_tokens(hit) -> int:
    h, hp = _u32(hit)
    return int(_load().kvo_total_hit_tokens(h.size, hp))


def payload_bytes(hit, row_bytes) -> int:
    """Bytes of one layer's transfer buffer (all planes)."""
    h, hp = _u32(hit)
    rb, rbp = _u32(row_bytes)
    return int(_load().kvo_payload_bytes(h.size, hp, rb.size, rbp))


def check(block_tokens: int, pool_blocks: int, hit, app, tables, scatter: bool) -> int:
    h, hp = _u32(hit)
    a, ap = _u32(app)
    keep, tp = _tables(tables)
    ln, lp = _u32([t.size for t in keep])
    return int(_load().kvo_check(block_tokens, pool_blocks, h.size, hp, ap, lp, tp, int(scatter)))


def _ranges(n_req: int, threads: int) -> List[Tuple[int, int]]:
    threads = max(1, min(threads, n_req))
    cuts = np.linspace(0, n_req, threads + 1).astype(int)
    return [(int(cuts[i]), int(cuts[i + 1])) for i in range(threads) if cuts[i] < cuts[i + 1]]


def pack(block_tokens: int, row_bytes, hit, tables, pool_planes: Sequence[np.ndarray],
         xfer: Optional[np.ndarray] = None, threads: int = 1) -> np.ndarray:
    """Gather the hit rows of every request into a dense transfer buffer."""
    lib = _load()
    h, hp = _u32(hit)
    rb, rbp = _u32(row_bytes)
    keep, tp = _tables(tables)
    pp = _planes(pool_planes, writable=False)
    n = payload_bytes(h, rb)
    if xfer is None:
        xfer = np.empty(n, dtype=np.uint8)
    if xfer.dtype != np.uint8 or xfer.size < n or not xfer.flags["C_CONTIGUOUS"]:
        raise ValueError("transfer buffer too small or not contiguous uint8")

    def run(rng):
        rc = lib.kvo_pack(block_tokens, rb.size, rbp, h.size, hp, tp, pp,
                          xfer.ctypes.data, rng[0], rng[1])
        if rc != OK:
            raise RuntimeError(f"kvo_pack failed: {rc}")

    ranges = _ranges(h.size, threads) if h.size else []
    if len(ranges) <= 1:
        run((0, h.size))
    else:
        with ThreadPoolExecutor(len(ranges)) as ex:
            list(ex.map(run, ranges))
    return xfer


def unpack(block_tokens: int, row_bytes, hit, tables, xfer: np.ndarray,
           pool_planes: Sequence[np.ndarray], threads: int = 1) -> None:
    """Scatter a dense transfer buffer into the hit rows of a paged pool, in place."""
    lib = _load()
    h, hp = _u32(hit)
    rb, rbp = _u32(row_bytes)
    keep, tp = _tables(tables)
    pp = _planes(pool_planes, writable=True)
    n = payload_bytes(h, rb)
    if xfer.dtype != np.uint8 or xfer.size < n or not xfer.flags["C_CONTIGUOUS"]:
        raise ValueError("transfer buffer too small or not contiguous uint8")

    def run(rng):
        rc = lib.kvo_unpack(block_tokens, rb.size, rbp, h.size, hp, tp,
                            xfer.ctypes.data, pp, rng[0], rng[1])
        if rc != OK:
            raise RuntimeError(f"kvo_unpack failed: {rc}")

    ranges = _ranges(h.size, threads) if h.size else []
    if len(ranges) <= 1:
        run((0, h.size))
    else:
        with ThreadPoolExecutor(len(ranges)) as ex:
            list(ex.map(run, ranges))


def pack_range(block_tokens: int, row_bytes, first, count, tables, pool_planes: Sequence[np.ndarray],
               xfer: Optional[np.ndarray] = None, threads: int = 1) -> np.ndarray:
    """Gather token rows [first_r, first_r + count_r) of every request (first=None: zeros)."""
    lib = _load()
    c, cp = _u32(count)
    f, fp = _u32(first) if first is not None else (None, None)
    rb, rbp = _u32(row_bytes)
    keep, tp = _tables(tables)
    pp = _planes(pool_planes, writable=False)
    n = payload_bytes(c, rb)
    if xfer is None:
        xfer = np.empty(n, dtype=np.uint8)
    if xfer.dtype != np.uint8 or xfer.size < n or not xfer.flags["C_CONTIGUOUS"]:
        raise ValueError("transfer buffer too small or not contiguous uint8")

    def run(rng):
        rc = lib.kvo_pack_range(block_tokens, rb.size, rbp, c.size, fp, cp, tp, pp,
                                xfer.ctypes.data, rng[0], rng[1])
        if rc != OK:
            raise RuntimeError(f"kvo_pack_range failed: {rc}")

    ranges = _ranges(c.size, threads) if c.size else []
    if len(ranges) <= 1:
        run((0, c.size))
    else:
        with ThreadPoolExecutor(len(ranges)) as ex:
            list(ex.map(run, ranges))
    return xfer


def unpack_range(block_tokens: int, row_bytes, first, count, tables, xfer: np.ndarray,
                 pool_planes: Sequence[np.ndarray], threads: int = 1) -> None:
    """Scatter a transfer buffer into token rows [first_r, first_r + count_r), in place."""
    lib = _load()
    c, cp = _u32(count)
    f, fp = _u32(first) if first is not None else (None, None)
    rb, rbp = _u32(row_bytes)
    keep, tp = _tables(tables)
    pp = _planes(pool_planes, writable=True)
    n = payload_bytes(c, rb)
    if xfer.dtype != np.uint8 or xfer.size < n or not xfer.flags["C_CONTIGUOUS"]:
        raise ValueError("transfer buffer too small or not contiguous uint8")

    def run(rng):
        rc = lib.kvo_unpack_range(block_tokens, rb.size, rbp, c.size, fp, cp, tp,
                                  xfer.ctypes.data, pp, rng[0], rng[1])
        if rc != OK:
            raise RuntimeError(f"kvo_unpack_range failed: {rc}")

    ranges = _ranges(c.size, threads) if c.size else []
    if len(ranges) <= 1:
        run((0, c.size))
    else:
        with ThreadPoolExecutor(len(ranges)) as ex:
            list(ex.map(run, ranges))


def check_range_scatter(block_tokens: int, pool_blocks: int, first, count, tables) -> int:
    c, cp = _u32(count)
    f, fp = _u32(first) if first is not None else (None, None)
    keep, tp = _tables(tables)
    return int(_load().kvo_check_range_scatter(block_tokens, pool_blocks, c.size, fp, cp, tp))


def fullblock_bytes(block_tokens: int, n_layers: int, row_bytes) -> int:
    rb, rbp = _u32(row_bytes)
    return int(_load().kvo_fullblock_bytes(block_tokens, n_layers, rb.size, rbp))


def fullblock_count(block_tokens: int, first, count) -> int:
    c, cp = _u32(count)
    f, fp = _u32(first) if first is not None else (None, None)
    return int(_load().kvo_fullblock_count(block_tokens, c.size, fp, cp))


def fullblocks_to_pool(block_tokens: int, n_layers: int, row_bytes, first, count, tables, layer: int,
                       blocks: np.ndarray, pool_planes: Sequence[np.ndarray]) -> None:
    """Load layer `layer` of the ranges' rows from a buffer of Full Blocks into a paged pool."""
    c, cp = _u32(count)
    f, fp = _u32(first) if first is not None else (None, None)
    rb, rbp = _u32(row_bytes)
    keep, tp = _tables(tables)
    pp = _planes(pool_planes, writable=True)
    need = fullblock_count(block_tokens, first, count) * fullblock_bytes(block_tokens, n_layers, rb)
    if blocks.dtype != np.uint8 or blocks.size < need or not blocks.flags["C_CONTIGUOUS"]:
        raise ValueError("Full-Block buffer too small or not contiguous uint8")
    rc = _load().kvo_fullblocks_to_pool(block_tokens, n_layers, rb.size, rbp, c.size, fp, cp, tp, layer,
                                        blocks.ctypes.data, pp)
    if rc != OK:
        raise RuntimeError(f"kvo_fullblocks_to_pool failed: {rc}")


def pool_to_fullblocks(block_tokens: int, n_layers: int, row_bytes, first, count, tables, layer: int,
                       pool_planes: Sequence[np.ndarray], blocks: np.ndarray) -> None:
    """Store layer `layer` of the ranges' rows from a paged pool into a buffer of Full Blocks."""
    c, cp = _u32(count)
    f, fp = _u32(first) if first is not None else (None, None)
    rb, rbp = _u32(row_bytes)
    keep, tp = _tables(tables)
    pp = _planes(pool_planes, writable=False)
    need = fullblock_count(block_tokens, first, count) * fullblock_bytes(block_tokens, n_layers, rb)
    if blocks.dtype != np.uint8 or blocks.size < need or not blocks.flags["C_CONTIGUOUS"] \
            or not blocks.flags["WRITEABLE"]:
        raise ValueError("Full-Block buffer too small, read-only or not contiguous uint8")
    rc = _load().kvo_pool_to_fullblocks(block_tokens, n_layers, rb.size, rbp, c.size, fp, cp, tp, layer,
                                        pp, blocks.ctypes.data)
    if rc != OK:
        raise RuntimeError(f"kvo_pool_to_fullblocks failed: {rc}")


def stream_layers(block_tokens: int, row_bytes, hit, tables, host_layers: Sequence[np.ndarray],
                  n_layers: int, dev_slots: Sequence[Sequence[np.ndarray]]
                  ) -> Iterator[Tuple[int, int, Sequence[np.ndarray]]]:
    """Layer-wise load (Section 4.1: the hit cache of layer l is brought into
    the prefill engine's memory before layer l is computed, layer after layer).

    Layer l's transfer buffer is ``host_layers[l mod H]``; it is unpacked into
    destination slot ``l mod S``.  Yields ``(l, slot, planes)``: the slot's
    contents as the compute of layer l must see them.
    """
    H, S = len(host_layers), len(dev_slots)
    for l in range(n_layers):
        s = l % S
        unpack(block_tokens, row_bytes, hit, tables, host_layers[l % H], dev_slots[s])
        yield l, s, dev_slots[s]


def stream_layers_fullblocks(block_tokens: int, n_layers: int, row_bytes, first, count, tables,
                             blocks: np.ndarray, dev_slots: Sequence[Sequence[np.ndarray]], run_layers: int = 0
                             ) -> Iterator[Tuple[int, int, Sequence[np.ndarray]]]:
    """The same layer-wise load with the storage layout as its source: layer l is taken
    from layer l of a buffer of Full Blocks into destination slot l mod S."""
    S = len(dev_slots)
    for l in range(run_layers or n_layers):
        s = l % S
        fullblocks_to_pool(block_tokens, n_layers, row_bytes, first, count, tables, l, blocks, dev_slots[s])
        yield l, s, dev_slots[s]
