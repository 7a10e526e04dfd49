"""ctypes front end of the C data-path oracle (datapath.c).  TEST INFRASTRUCTURE ONLY.

Operates on NumPy fp32 / uint32 host arrays.  `merged_gradient_path` strings the
steps together in the paper's order: for every group (communication order), pack
each worker's layers into its layer buffer (Algorithm 2), all-reduce arithmetic
(Eq. 2), scatter back, then optionally the weight update (Algorithm 2's
W = W - eta*grad, with momentum).
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import numpy as np

from .build import build_oracle

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build_oracle(force=False))
        _lib.oracle_pack.argtypes = [C.POINTER(C.c_void_p), C.POINTER(C.c_uint64),
                                     C.POINTER(C.c_int32), C.c_int32, C.c_void_p, C.c_int32]
        _lib.oracle_pack.restype = None
        _lib.oracle_reduce.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_uint64,
                                       C.c_void_p, C.c_int32]
        _lib.oracle_reduce.restype = None
        _lib.oracle_unpack.argtypes = [C.c_void_p, C.POINTER(C.c_uint64),
                                       C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_void_p), C.c_int32]
        _lib.oracle_unpack.restype = None
        _lib.oracle_sgd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64,
                                    C.c_float, C.c_float, C.c_int32]
        _lib.oracle_sgd.restype = None
        _lib.oracle_max_threads.restype = C.c_int32
    return _lib


def max_threads() -> int:
    return int(lib().oracle_max_threads())


def _ptrs(arrs: Sequence[np.ndarray]):
    return (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def _check(a: np.ndarray, dtypes) -> None:
    assert a.dtype in dtypes and a.flags["C_CONTIGUOUS"], (a.dtype, a.flags)


def pack(layers: Sequence[np.ndarray], group_layers: Sequence[int], threads: int = 1) -> np.ndarray:
    """Layer buffer of one worker for one group; layers[l] is 0-based layer l (4-byte items)."""
    for a in layers:
        _check(a, (np.float32, np.uint32))
    p = np.array([a.size for a in layers], dtype=np.uint64)
    gl = np.asarray(group_layers, dtype=np.int32)
    total = int(sum(int(p[l]) for l in gl))
    merged = np.empty(total, dtype=layers[0].dtype)
    lib().oracle_pack(_ptrs(layers), p.ctypes.data_as(C.POINTER(C.c_uint64)),
                      gl.ctypes.data_as(C.POINTER(C.c_int32)), len(gl), merged.ctypes.data, threads)
    return merged


def reduce(buffers: Sequence[np.ndarray], threads: int = 1) -> np.ndarray:
    """(1/N) * sum of the N workers' buffers, workers added in order 0..N-1 in fp32."""
    for a in buffers:
        _check(a, (np.float32,))
        assert a.size == buffers[0].size
    out = np.empty_like(buffers[0])
    lib().oracle_reduce(_ptrs(buffers), len(buffers), buffers[0].size, out.ctypes.data, threads)
    return out


def unpack(merged: np.ndarray, out_layers: Sequence[np.ndarray], group_layers: Sequence[int],
           threads: int = 1) -> None:
    """Scatter `merged` into out_layers[l] for l in the group (in place)."""
    _check(merged, (np.float32, np.uint32))
    for a in out_layers:
        _check(a, (merged.dtype,))
    p = np.array([a.size for a in out_layers], dtype=np.uint64)
    gl = np.asarray(group_layers, dtype=np.int32)
    assert merged.size == sum(int(p[l]) for l in gl)
    lib().oracle_unpack(merged.ctypes.data, p.ctypes.data_as(C.POINTER(C.c_uint64)),
                        gl.ctypes.data_as(C.POINTER(C.c_int32)), len(gl), _ptrs(out_layers), threads)


def sgd(w: np.ndarray, v: np.ndarray, g: np.ndarray, lr: float, mu: float, threads: int = 1) -> None:
    """In place: v = mu*v + g ; w = w - lr*v."""
    for a in (w, v, g):
        _check(a, (np.float32,))
        assert a.size == w.size
    lib().oracle_sgd(w.ctypes.data, v.ctypes.data, g.ctypes.data, w.size,
                     np.float32(lr), np.float32(mu), threads)


def merged_gradient_path(grads: Sequence[Sequence[np.ndarray]], groups: Sequence[Sequence[int]],
                         w: Optional[List[np.ndarray]] = None, v: Optional[List[np.ndarray]] = None,
                         lr: float = 0.0, mu: float = 0.0, threads: int = 1) -> List[np.ndarray]:
    """Whole path.  grads[g][l]; groups = lists of 0-based layers, arrival order.

    Returns the averaged per-layer gradients; updates w, v in place when given.
    """
    L = len(grads[0])
    avg = [np.empty_like(grads[0][l]) for l in range(L)]
    for grp in groups:
        buffers = [pack(grads[g], grp, threads) for g in range(len(grads))]
        reduced = reduce(buffers, threads)
        unpack(reduced, avg, grp, threads)
        if w is not None:
            for l in grp:
                sgd(w[l], v[l], avg[l], lr, mu, threads)
    return avg
