"""ctypes marshalling for libmtpp.so (include/mtpp.h): max-throughput slicing of a topological order.  Host only."""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmtpp.so")
EXPORTS = ("mtpp_kahn_order", "mtpp_block_cost", "mtpp_slice_order")
_lib = None


class MtppError(RuntimeError):
    pass


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MtppError("libmtpp.so is not built: run `python -m paper_2407_19775_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        i32, f64, vp = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        L.mtpp_kahn_order.argtypes = [i32, i32, vp, vp, vp]
        L.mtpp_block_cost.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp, i32, i32, f64, f64, vp]
        L.mtpp_slice_order.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp, i32, f64, f64, vp, vp, vp]
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise MtppError({-1: "invalid argument", -2: "not acyclic, or not a topological order"}.get(status, "status %d" % status))


def _edges(edges):
    e = np.asarray(list(edges), dtype=np.int32).reshape(-1, 2)
    return np.ascontiguousarray(e[:, 0]), np.ascontiguousarray(e[:, 1])


def _ptr(a):
    return a.ctypes.data if a is not None and a.size else None


def kahn_order(n, edges):
    u, v = _edges(edges)
    out = np.empty(n, np.int32)
    _check(lib().mtpp_kahn_order(n, u.size, _ptr(u), _ptr(v), out.ctypes.data))
    return out


def block_cost(n, edges, work, sizeparam, sizeout, order, first, last, B, M):
    u, v = _edges(edges)
    w, sp, so = (np.ascontiguousarray(a, dtype=np.float64) for a in (work, sizeparam, sizeout))
    o = np.ascontiguousarray(order, dtype=np.int32)
    cost = ctypes.c_double()
    _check(lib().mtpp_block_cost(n, u.size, _ptr(u), _ptr(v), w.ctypes.data, sp.ctypes.data, so.ctypes.data,
                                 o.ctypes.data, first, last, B, M, ctypes.addressof(cost)))
    return cost.value


def slice_order(n, edges, work, sizeparam, sizeout, k, B, M, order=None):
    """-> (bottleneck cost, block ends: positions in the order after each block's last operation)."""
    u, v = _edges(edges)
    w, sp, so = (np.ascontiguousarray(a, dtype=np.float64) for a in (work, sizeparam, sizeout))
    o = np.ascontiguousarray(order, dtype=np.int32) if order is not None else None
    cost, blocks = ctypes.c_double(), ctypes.c_int32()
    ends = np.zeros(max(k, 1), np.int32)
    _check(lib().mtpp_slice_order(n, u.size, _ptr(u), _ptr(v), w.ctypes.data, sp.ctypes.data, so.ctypes.data,
                                  o.ctypes.data if o is not None else None, k, B, M, ctypes.addressof(cost),
                                  ctypes.addressof(blocks), ends.ctypes.data))
    return cost.value, ends[:blocks.value].copy()
