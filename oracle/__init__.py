"""ROBE-Z CPU oracle: ctypes front end for ``robe_oracle.c``.

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``; never by the product package.
It shares nothing with the HIP path: its own C source, its own argument
layout (eight coefficients in a flat tuple), NumPy arrays in and out.

The arithmetic is in the C file; each function there cites the passage of the
paper (arXiv 2108.02191, Section 3) that it writes out.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "robe_oracle.c")
_LIB = os.path.join(_HERE, "librobe_oracle.so")

P_DEFAULT = 2**31 - 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP on, FMA contraction off)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u64, i64, u32, i32 = ctypes.c_uint64, ctypes.c_int64, ctypes.c_uint32, ctypes.c_int32
        vp = ctypes.c_void_p
        L.oracle_splitmix64_next.restype = u64
        L.oracle_splitmix64_next.argtypes = [ctypes.POINTER(u64)]
        L.oracle_init_hash.restype = None
        L.oracle_init_hash.argtypes = [u64, u64, vp]
        L.oracle_h.restype = u64
        L.oracle_h.argtypes = [vp, u64, u64, u64, u64, u64]
        L.oracle_g.restype = ctypes.c_int
        L.oracle_g.argtypes = [vp, u64, ctypes.c_int, u64, u64, u64]
        L.oracle_idx.restype = u64
        L.oracle_idx.argtypes = [vp, u64, u64, u32, u32, u64, u64, u64]
        L.oracle_offsets.restype = None
        L.oracle_offsets.argtypes = [vp, u64, u64, u32, u32, vp, i64, i32, vp]
        L.oracle_signs.restype = None
        L.oracle_signs.argtypes = [vp, u64, u32, ctypes.c_int, vp, i64, i32, vp]
        L.oracle_forward.restype = None
        L.oracle_forward.argtypes = [vp, u64, u64, u32, u32, ctypes.c_int, vp, vp, vp, i64, i32, vp, ctypes.c_int]
        L.oracle_backward.restype = None
        L.oracle_backward.argtypes = [vp, u64, u64, u32, u32, ctypes.c_int, vp, vp, vp, i64, i32, vp, vp, ctypes.c_int]
        L.oracle_forward_mixed.restype = None
        L.oracle_forward_mixed.argtypes = [vp, u64, u64, vp, u32, ctypes.c_int, vp, vp, vp, i64, i32, vp]
        L.oracle_backward_mixed.restype = None
        L.oracle_backward_mixed.argtypes = [vp, u64, u64, vp, u32, ctypes.c_int, vp, vp, vp, i64, i32, vp, vp]
        L.oracle_array_to_bf16.restype = None
        L.oracle_array_to_bf16.argtypes = [vp, vp, u64]
        L.oracle_forward_bf16.restype = None
        L.oracle_forward_bf16.argtypes = [vp, u64, u64, u32, u32, ctypes.c_int, vp, vp, vp, i64, i32, vp]
        L.oracle_adagrad.restype = None
        L.oracle_adagrad.argtypes = [vp, vp, vp, u64, ctypes.c_double, ctypes.c_double, ctypes.c_int]
        L.oracle_sgd.restype = None
        L.oracle_sgd.argtypes = [vp, vp, u64, ctypes.c_double, ctypes.c_int]
        L.oracle_max_threads.restype = ctypes.c_int
        L.oracle_max_threads.argtypes = []
        _lib = L
    return _lib


@dataclass(frozen=True)
class Hash:
    """Parameters of one ROBE-Z instance: array length m, embedding size d,
    block size Z, sign on/off, prime P and (A_h,B_h,C_h,D_h,A_g,B_g,C_g,D_g)."""
    m: int
    d: int
    Z: int
    use_sign: int
    P: int
    coef: Tuple[int, ...]

    def _c(self):
        return (ctypes.c_uint64 * 8)(*self.coef)


def splitmix64_stream(seed: int, n: int):
    L = _load()
    st = ctypes.c_uint64(seed)
    return [int(L.oracle_splitmix64_next(ctypes.byref(st))) for _ in range(n)]


def init_hash(seed: int, m: int, d: int, Z: int, use_sign: int, P: int = P_DEFAULT) -> Hash:
    if m < 1 or d < 1 or Z < 1 or Z > m or (d % Z if Z <= d else Z % d):
        raise ValueError("need m >= 1, Z >= 1, Z | d or d | Z, Z <= m")
    L = _load()
    c = (ctypes.c_uint64 * 8)()
    L.oracle_init_hash(seed, P, c)
    return Hash(m, d, Z, int(bool(use_sign)), P, tuple(int(v) for v in c))


def h(H: Hash, e: int, x: int, c: int) -> int:
    return int(_load().oracle_h(H._c(), H.P, H.m, e, x & (2**64 - 1), c))


def g(H: Hash, e: int, x: int, i: int) -> int:
    return int(_load().oracle_g(H._c(), H.P, H.use_sign, e, x & (2**64 - 1), i))


def idx(H: Hash, e: int, x: int, i: int) -> int:
    return int(_load().oracle_idx(H._c(), H.P, H.m, H.d, H.Z, e, x & (2**64 - 1), i))


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def offsets(H: Hash, indices, F: int) -> np.ndarray:
    ind = _i64(indices).ravel()
    out = np.empty((ind.size, max(1, H.d // H.Z)), dtype=np.int64)
    _load().oracle_offsets(H._c(), H.P, H.m, H.d, H.Z, _ptr(ind), ind.size, F, _ptr(out))
    return out


def signs(H: Hash, indices, F: int) -> np.ndarray:
    ind = _i64(indices).ravel()
    out = np.empty((ind.size, H.d), dtype=np.int8)
    _load().oracle_signs(H._c(), H.P, H.d, H.use_sign, _ptr(ind), ind.size, F, _ptr(out))
    return out


def _check_bags(ind: np.ndarray, off: Optional[np.ndarray], rows: int):
    if off is None:
        if ind.size != rows:
            raise ValueError("single-hot: indices must hold batch*F ids")
    else:
        if off.size != rows + 1 or off[0] != 0 or off[-1] != ind.size or np.any(np.diff(off) < 0):
            raise ValueError("bad CSR offsets")


def forward(H: Hash, array, indices, bag_offsets, batch: int, F: int, threads: int = 1) -> np.ndarray:
    arr = _f32(array)
    assert arr.size == H.m
    ind = _i64(indices).ravel()
    off = None if bag_offsets is None else _i64(bag_offsets)
    _check_bags(ind, off, batch * F)
    out = np.empty((batch, F, H.d), dtype=np.float32)
    _load().oracle_forward(H._c(), H.P, H.m, H.d, H.Z, H.use_sign, _ptr(arr), _ptr(ind), _ptr(off),
                           batch, F, _ptr(out), threads)
    return out


def backward(H: Hash, grad_out, indices, bag_offsets, batch: int, F: int, threads: int = 1,
             want_abs: bool = True):
    """Returns (grad_array float64[m], abs_sum float64[m] or None), both from zero."""
    go = _f32(grad_out)
    assert go.size == batch * F * H.d
    ind = _i64(indices).ravel()
    off = None if bag_offsets is None else _i64(bag_offsets)
    _check_bags(ind, off, batch * F)
    ga = np.zeros(H.m, dtype=np.float64)
    ab = np.zeros(H.m, dtype=np.float64) if want_abs else None
    _load().oracle_backward(H._c(), H.P, H.m, H.d, H.Z, H.use_sign, _ptr(go), _ptr(ind), _ptr(off),
                            batch, F, _ptr(ga), _ptr(ab), threads)
    return ga, ab


def _check_dims(H: Hash, dims) -> np.ndarray:
    dm = np.ascontiguousarray(dims, dtype=np.uint32).ravel()
    for d in dm.tolist():
        if d < 1 or not (d % H.Z == 0 or H.Z % d == 0):
            raise ValueError("every table dimension must be a multiple or a divisor of Z")
    return dm


def forward_mixed(H: Hash, dims, array, indices, bag_offsets, batch: int) -> np.ndarray:
    """Tables of different dimensions (H.d is not used): returns float32[batch, sum(dims)]."""
    dm = _check_dims(H, dims)
    F = dm.size
    arr = _f32(array)
    assert arr.size == H.m
    ind = _i64(indices).ravel()
    off = None if bag_offsets is None else _i64(bag_offsets)
    _check_bags(ind, off, batch * F)
    out = np.empty((batch, int(dm.sum())), dtype=np.float32)
    _load().oracle_forward_mixed(H._c(), H.P, H.m, _ptr(dm), H.Z, H.use_sign, _ptr(arr), _ptr(ind), _ptr(off),
                                 batch, F, _ptr(out))
    return out


def backward_mixed(H: Hash, dims, grad_out, indices, bag_offsets, batch: int):
    """Returns (grad_array float64[m], abs_sum float64[m]), both from zero."""
    dm = _check_dims(H, dims)
    F = dm.size
    go = _f32(grad_out)
    assert go.size == batch * int(dm.sum())
    ind = _i64(indices).ravel()
    off = None if bag_offsets is None else _i64(bag_offsets)
    _check_bags(ind, off, batch * F)
    ga = np.zeros(H.m, dtype=np.float64)
    ab = np.zeros(H.m, dtype=np.float64)
    _load().oracle_backward_mixed(H._c(), H.P, H.m, _ptr(dm), H.Z, H.use_sign, _ptr(go), _ptr(ind), _ptr(off),
                                  batch, F, _ptr(ga), _ptr(ab))
    return ga, ab


def to_bf16(array) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even."""
    arr = _f32(array).ravel()
    out = np.empty(arr.size, dtype=np.uint16)
    _load().oracle_array_to_bf16(_ptr(arr), _ptr(out), arr.size)
    return out


def forward_bf16(H: Hash, array_bf16, indices, bag_offsets, batch: int, F: int) -> np.ndarray:
    """Forward on an array of bfloat16 bit patterns (uint16[m]); output float32[batch, F, d]."""
    arr = np.ascontiguousarray(array_bf16, dtype=np.uint16).ravel()
    assert arr.size == H.m
    ind = _i64(indices).ravel()
    off = None if bag_offsets is None else _i64(bag_offsets)
    _check_bags(ind, off, batch * F)
    out = np.empty((batch, F, H.d), dtype=np.float32)
    _load().oracle_forward_bf16(H._c(), H.P, H.m, H.d, H.Z, H.use_sign, _ptr(arr), _ptr(ind), _ptr(off),
                                batch, F, _ptr(out))
    return out


def adagrad(array: np.ndarray, state: np.ndarray, grad: np.ndarray, lr: float, eps: float,
            threads: int = 1) -> None:
    """In place on three contiguous float32 arrays of equal length; grad is zeroed."""
    for a in (array, state, grad):
        assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"] and a.size == array.size
    _load().oracle_adagrad(_ptr(array), _ptr(state), _ptr(grad), array.size, lr, eps, threads)


def sgd(array: np.ndarray, grad: np.ndarray, lr: float, threads: int = 1) -> None:
    """In place on two contiguous float32 arrays of equal length; grad is zeroed."""
    for a in (array, grad):
        assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"] and a.size == array.size
    _load().oracle_sgd(_ptr(array), _ptr(grad), array.size, lr, threads)


def max_threads() -> int:
    return int(_load().oracle_max_threads())
