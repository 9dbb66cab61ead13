"""ctypes face of the CPU oracle (oracle.cpp).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module; the
HIP library and its Python binding never do.  Arrays are numpy, host memory.
"""
import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

F_OVERFLOW, F_NONFINITE, F_EXHAUSTED = 1, 2, 4


class _Result(C.Structure):
    _fields_ = [("nnz", C.c_uint32), ("rounds", C.c_uint32), ("count", C.c_uint32 * 4),
                ("flags", C.c_uint32), ("thres_f32", C.c_float), ("mean", C.c_double),
                ("std", C.c_double), ("z", C.c_double), ("thres0", C.c_double),
                ("thres", C.c_double), ("topk_key", C.c_uint32), ("topk_ties_taken", C.c_uint32)]


@dataclass
class Result:
    nnz: int
    rounds: int
    count: tuple
    flags: int
    thres_f32: np.float32
    mean: float
    std: float
    z: float
    thres0: float
    thres: float
    topk_key: int
    topk_ties_taken: int

    @staticmethod
    def of(r: _Result) -> "Result":
        return Result(r.nnz, r.rounds, tuple(r.count), r.flags, np.float32(r.thres_f32), r.mean,
                      r.std, r.z, r.thres0, r.thres, r.topk_key, r.topk_ties_taken)


_lib = None


def lib():
    global _lib
    if _lib is None:
        # ORACLE_LIBRARY names another build of oracle.cpp to load instead: the mutation check of
        # the pins (tests/test_oracle_mutants.py) runs the pins against deliberately broken copies
        L = C.CDLL(os.environ.get("ORACLE_LIBRARY") or _build.ensure_built())
        fp, up, ip = C.POINTER(C.c_float), C.POINTER(C.c_uint32), C.POINTER(C.c_int64)
        L.oracle_accumulate.argtypes = [C.c_int64, fp, fp, fp]
        L.oracle_accumulate.restype = None
        L.oracle_moments.argtypes = [C.c_int64, fp, C.c_int32, C.POINTER(C.c_double),
                                     C.POINTER(C.c_double)]
        L.oracle_moments.restype = None
        L.oracle_norm_isf.argtypes = [C.c_double]
        L.oracle_norm_isf.restype = C.c_double
        L.oracle_sqnorm.argtypes = [C.c_int64, fp]
        L.oracle_sqnorm.restype = C.c_double
        L.oracle_topk.argtypes = [C.c_int64, C.c_int64, fp, up, fp, fp, C.POINTER(_Result)]
        L.oracle_gaussiank.argtypes = [C.c_int64, C.c_int64, fp, C.c_int64, C.c_double, C.c_int32,
                                       up, fp, fp, C.POINTER(_Result)]
        L.oracle_randk_dense.argtypes = [C.c_int64, C.c_int64, fp, up, fp]
        L.oracle_dgck.argtypes = [C.c_int64, C.c_int64, fp, C.c_int32, C.c_uint64, up, fp, fp,
                                  C.POINTER(_Result), up]
        L.oracle_scatter_add.argtypes = [C.c_int64, C.c_int32, up, fp, C.c_int64, up, C.c_float, fp]
        L.oracle_segmented.argtypes = [C.c_int32, ip, ip, C.c_int32, fp, ip, C.c_double, C.c_int32,
                                       up, fp, fp, C.POINTER(_Result)]
        _lib = L
    return _lib


def _f(a):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _u(a):
    assert a.dtype == np.uint32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_uint32))


def _i(a):
    assert a.dtype == np.int64 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_int64))


def accumulate(g: np.ndarray, eps: np.ndarray, out: np.ndarray = None) -> np.ndarray:
    acc = np.empty_like(g) if out is None else out
    lib().oracle_accumulate(g.size, _f(g), _f(eps), _f(acc))
    return acc


def moments(acc: np.ndarray, ddof: int = 1):
    m, s = C.c_double(), C.c_double()
    lib().oracle_moments(acc.size, _f(acc), ddof, C.byref(m), C.byref(s))
    return m.value, s.value


def norm_isf(q: float) -> float:
    return lib().oracle_norm_isf(q)


def sqnorm(x: np.ndarray) -> float:
    return lib().oracle_sqnorm(x.size, _f(x))


def topk(acc: np.ndarray, k: int, eps_out: np.ndarray = None, idx: np.ndarray = None,
         val: np.ndarray = None):
    """-> (idx[k] ascending, val[k], eps_out[d], Result); the optional arrays are reused as
    output storage (idx/val need at least k entries)."""
    idx = np.empty(max(k, 1), np.uint32) if idx is None else idx
    val = np.empty(max(k, 1), np.float32) if val is None else val
    eps = np.empty_like(acc) if eps_out is None else eps_out
    r = _Result()
    rc = lib().oracle_topk(acc.size, k, _f(acc), _u(idx), _f(val), _f(eps), C.byref(r))
    if rc != 0:
        raise ValueError("oracle_topk: invalid arguments")
    return idx[:r.nnz], val[:r.nnz], eps, Result.of(r)


def gaussiank(acc: np.ndarray, k: int, cap: int = None, tail_div: float = 2.0, ddof: int = 1,
              eps_out: np.ndarray = None, idx: np.ndarray = None, val: np.ndarray = None):
    """-> (idx[nnz] ascending, val[nnz], eps_out[d], Result); the optional arrays are reused as
    output storage (idx/val need at least cap entries)."""
    cap = acc.size if cap is None else cap
    idx = np.empty(max(cap, 1), np.uint32) if idx is None else idx
    val = np.empty(max(cap, 1), np.float32) if val is None else val
    eps = np.empty_like(acc) if eps_out is None else eps_out
    r = _Result()
    rc = lib().oracle_gaussiank(acc.size, k, _f(acc), cap, tail_div, ddof, _u(idx), _f(val),
                                _f(eps), C.byref(r))
    if rc != 0:
        raise ValueError("oracle_gaussiank: invalid arguments")
    return idx[:r.nnz], val[:r.nnz], eps, Result.of(r)


def dgck(acc: np.ndarray, k: int, sample_stride: int = 100, seed: int = 0,
         eps_out: np.ndarray = None, idx: np.ndarray = None, val: np.ndarray = None,
         want_positions: bool = False):
    """-> (idx[nnz] ascending, val[nnz], eps_out[d], Result[, sample positions]); nnz <= k."""
    idx = np.empty(max(k, 1), np.uint32) if idx is None else idx
    val = np.empty(max(k, 1), np.float32) if val is None else val
    eps = np.empty_like(acc) if eps_out is None else eps_out
    m = -(-acc.size // sample_stride) if sample_stride >= 1 else 1
    pos = np.empty(m, np.uint32) if want_positions else None
    r = _Result()
    rc = lib().oracle_dgck(acc.size, k, _f(acc), sample_stride, seed, _u(idx), _f(val), _f(eps),
                           C.byref(r), _u(pos) if want_positions else None)
    if rc != 0:
        raise ValueError("oracle_dgck: invalid arguments")
    out = (idx[:r.nnz], val[:r.nnz], eps, Result.of(r))
    return out + (pos,) if want_positions else out


def randk_dense(acc: np.ndarray, chosen: np.ndarray) -> np.ndarray:
    out = np.empty_like(acc)
    rc = lib().oracle_randk_dense(acc.size, chosen.size, _f(acc), _u(chosen), _f(out))
    if rc != 0:
        raise ValueError("oracle_randk_dense: invalid arguments")
    return out


def segmented(acc: np.ndarray, seg_off: np.ndarray, seg_k: np.ndarray, mode: int,
              out_off: np.ndarray, tail_div: float = 2.0, ddof: int = 1,
              eps_out: np.ndarray = None):
    """-> (idx[out_off[-1]], val[...], eps_out[d], [Result]*L); segment l's pairs occupy
    idx[out_off[l] : out_off[l] + results[l].nnz]."""
    L = seg_k.size
    idx = np.zeros(max(int(out_off[-1]), 1), np.uint32)
    val = np.zeros(max(int(out_off[-1]), 1), np.float32)
    eps = np.empty_like(acc) if eps_out is None else eps_out
    res = (_Result * L)()
    rc = lib().oracle_segmented(L, _i(seg_off), _i(seg_k), mode, _f(acc), _i(out_off), tail_div,
                                ddof, _u(idx), _f(val), _f(eps), res)
    if rc != 0:
        raise ValueError("oracle_segmented: invalid arguments")
    return idx, val, eps, [Result.of(res[l]) for l in range(L)]


def scatter_add(d: int, idx: np.ndarray, val: np.ndarray, nnz: np.ndarray, scale: float = 1.0,
                out: np.ndarray = None) -> np.ndarray:
    """idx, val: [P, stride] (uint32, float32); nnz: uint32[P] -> dense float32[d]."""
    assert idx.ndim == 2 and idx.shape == val.shape and nnz.shape == (idx.shape[0],)
    dense = np.empty(d, np.float32) if out is None else out
    rc = lib().oracle_scatter_add(d, idx.shape[0], _u(idx.reshape(-1)), _f(val.reshape(-1)),
                                  idx.shape[1], _u(nnz), scale, _f(dense))
    if rc != 0:
        raise ValueError("oracle_scatter_add: invalid arguments")
    return dense
