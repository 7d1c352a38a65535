"""ctypes binding of the scheduling functions declared in include/kvl_sched.h."""
from __future__ import annotations

import ctypes as C
from typing import List, Sequence, Tuple

import numpy as np

from . import binding as _b


class kvl_pd_range_t(C.Structure):
    _fields_ = [("lo", C.c_double), ("hi", C.c_double), ("hi_de_read", C.c_double),
                ("hi_de_write", C.c_double), ("hi_dram", C.c_double), ("feasible", C.c_int)]


_u64p = C.POINTER(C.c_uint64)
_i32p = C.POINTER(C.c_int32)
SIGNATURES = {
    "kvl_pd_range": (C.c_int, [C.c_double, C.c_double, C.c_double, C.c_double, C.POINTER(kvl_pd_range_t)]),
    "kvl_sched_pe_fetch": (C.c_int, [_u64p, _u64p, C.c_uint32, _u64p, C.c_uint32, C.c_uint64, C.c_uint64,
                                     _i32p, C.POINTER(C.c_uint32)]),
    "kvl_sched_de_groups": (C.c_int, [_u64p, C.c_uint32, _u64p, C.c_uint32, _i32p]),
    "kvl_sched_de_fetch": (C.c_int, [_u64p, _u64p, _u64p, C.c_uint32, _u64p, C.c_uint32, _i32p,
                                     C.POINTER(C.c_uint32), C.POINTER(C.c_double)]),
    "kvl_sched_read_side": (C.c_int, [C.c_uint64, C.c_uint64]),
}
_lib = _b._lib
for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(_lib, _name)
    _fn.restype, _fn.argtypes = _res, _args


def _u64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint64))


def _p(a: np.ndarray):
    return a.ctypes.data_as(_u64p)


def kvl_pd_range(g: float, s: float, mem_bw: float, storage_bw: float) -> dict:
    r = kvl_pd_range_t()
    _b._check(_lib.kvl_pd_range(g, s, mem_bw, storage_bw, C.byref(r)), "kvl_pd_range")
    return dict(lo=r.lo, hi=r.hi, hi_de_read=r.hi_de_read, hi_de_write=r.hi_de_write, hi_dram=r.hi_dram,
                feasible=bool(r.feasible))


def kvl_sched_pe_fetch(tok, read_q, req_tokens, alpha: int, beta: int) -> Tuple[List[int], np.ndarray]:
    """Returns (engine per request or -1, updated tok)."""
    t, q, r = _u64(tok).copy(), _u64(read_q), _u64(req_tokens)
    out = np.full(r.size, -1, dtype=np.int32)
    n = C.c_uint32()
    _b._check(_lib.kvl_sched_pe_fetch(_p(t), _p(q), t.size, _p(r), r.size, alpha, beta,
                                      out.ctypes.data_as(_i32p), C.byref(n)), "kvl_sched_pe_fetch")
    assert n.value == int((out >= 0).sum())
    return out.tolist(), t


def kvl_sched_de_groups(group_tok, req_len) -> Tuple[List[int], np.ndarray]:
    g, r = _u64(group_tok).copy(), _u64(req_len)
    out = np.full(r.size, -1, dtype=np.int32)
    _b._check(_lib.kvl_sched_de_groups(_p(g), g.size, _p(r), r.size, out.ctypes.data_as(_i32p)),
              "kvl_sched_de_groups")
    return out.tolist(), g


def kvl_sched_de_fetch(tok, seq, free_hbm, req_len):
    """Returns (engine per request or -1, Z, updated tok, seq, free_hbm)."""
    t, s, f, r = _u64(tok).copy(), _u64(seq).copy(), _u64(free_hbm).copy(), _u64(req_len)
    out = np.full(r.size, -1, dtype=np.int32)
    n, z = C.c_uint32(), C.c_double()
    _b._check(_lib.kvl_sched_de_fetch(_p(t), _p(s), _p(f), t.size, _p(r), r.size, out.ctypes.data_as(_i32p),
                                      C.byref(n), C.byref(z)), "kvl_sched_de_fetch")
    return out.tolist(), float(z.value), t, s, f


def kvl_sched_read_side(read_q_pe: int, read_q_de: int) -> int:
    return int(_lib.kvl_sched_read_side(read_q_pe, read_q_de))
