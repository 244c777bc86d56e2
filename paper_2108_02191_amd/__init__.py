"""ROBE-Z embedding lookup for MI355X (gfx950): thin Python binding of ``librobe.so``.

The functions here have the names and semantics of the C ABI in
``include/robe.h`` (arXiv 2108.02191, Section 3: Eq. 4/5 forward, Eq. 3
backward, Eq. 2 sign hash).  They only marshal arguments: every step of the
path runs in the HIP kernels of the library.  PyTorch supplies device memory
and the current stream, nothing else.  There is no CPU fallback: if the
library is not built, importing a function's result fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # loads the HIP runtime the library binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librobe.so")

ROBE_OK, ROBE_EINVAL, ROBE_EHIP = 0, -1, -2
ROBE_PRIME = 2**31 - 1


class RobeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"robe error {code}: {msg}")
        self.code = code


class RobeHash(ctypes.Structure):
    """Mirror of ``robe_hash_t``."""
    _fields_ = [("m", ctypes.c_uint64), ("d", ctypes.c_uint32), ("Z", ctypes.c_uint32),
                ("use_sign", ctypes.c_uint32), ("P", ctypes.c_uint32),
                ("Ah", ctypes.c_uint32), ("Bh", ctypes.c_uint32), ("Ch", ctypes.c_uint32), ("Dh", ctypes.c_uint32),
                ("Ag", ctypes.c_uint32), ("Bg", ctypes.c_uint32), ("Cg", ctypes.c_uint32), ("Dg", ctypes.c_uint32)]

    @property
    def coef(self):
        return (self.Ah, self.Bh, self.Ch, self.Dh, self.Ag, self.Bg, self.Cg, self.Dg)

    @property
    def chunks(self) -> int:
        return max(1, self.d // self.Z)


class RobeOptions(ctypes.Structure):
    """Mirror of ``robe_options_t``: per-call choices, all-zero = the library's defaults."""
    _fields_ = [("reproducible", ctypes.c_int32), ("backward_route", ctypes.c_int32), ("fused_route", ctypes.c_int32),
                ("fwd_elems", ctypes.c_int32), ("fwd_strided", ctypes.c_int32),
                ("bwd_elems", ctypes.c_int32), ("bwd_strided", ctypes.c_int32),
                ("tile_lookups", ctypes.c_int32), ("row_order", ctypes.c_int32), ("tile_combine", ctypes.c_int32),
                ("region_shift", ctypes.c_int32), ("key_bits", ctypes.c_int32), ("region_records", ctypes.c_int32),
                ("probe_kernel", ctypes.c_int32), ("reserved", ctypes.c_int32 * 2),
                ("probe_begin", ctypes.c_void_p), ("probe_end", ctypes.c_void_p)]


ROUTE_AUTO, ROUTE_DIRECT, ROUTE_COMBINE, ROUTE_REGIONS, ROUTE_TWO_STEP = 0, 1, 2, 3, 4
ROWS_AUTO, ROWS_MEMORY, ROWS_BY_TABLE, ROWS_BY_TABLE_ALWAYS = 0, 1, 2, 3
PROBE_NONE, PROBE_COMBINE, PROBE_REDUCE, PROBE_SORT = 0, 1, 2, 3

EXPORTS = ("robe_init_hash", "robe_offsets", "robe_forward", "robe_workspace_bytes", "robe_backward",
           "robe_adagrad_update", "robe_sgd_update", "robe_fused_workspace_bytes", "robe_backward_adagrad", "robe_backward_sgd",
           "robe_forward_mixed", "robe_mixed_workspace_bytes", "robe_backward_mixed", "robe_fused_mixed_workspace_bytes",
           "robe_backward_adagrad_mixed", "robe_array_to_bf16", "robe_forward_bf16",
           "robe_sort_workspace_bytes", "robe_sort_pairs", "robe_noalloc_max_workspace_bytes", "robe_backward_noalloc",
           "robe_last_error")

_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (``python -m paper_2108_02191_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2108_02191_amd.build` "
                              "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        HP = ctypes.POINTER(RobeHash)
        vp, i64, i32, u64, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint32
        L.robe_init_hash.restype = ctypes.c_int
        L.robe_init_hash.argtypes = [u64, u64, u32, u32, ctypes.c_int, HP]
        L.robe_offsets.restype = ctypes.c_int
        L.robe_offsets.argtypes = [HP, vp, i64, i32, vp, vp, vp]
        OP = ctypes.POINTER(RobeOptions)
        szp = ctypes.POINTER(ctypes.c_size_t)
        L.robe_forward.restype = ctypes.c_int
        L.robe_forward.argtypes = [HP, vp, vp, vp, i64, i64, i32, vp, OP, vp]
        L.robe_workspace_bytes.restype = ctypes.c_int
        L.robe_workspace_bytes.argtypes = [HP, i64, i32, i64, OP, szp]
        L.robe_backward.restype = ctypes.c_int
        L.robe_backward.argtypes = [HP, vp, vp, vp, i64, i64, i32, vp, vp, ctypes.c_size_t, OP, vp]
        L.robe_noalloc_max_workspace_bytes.restype = ctypes.c_size_t
        L.robe_noalloc_max_workspace_bytes.argtypes = []
        L.robe_backward_noalloc.restype = ctypes.c_int
        L.robe_backward_noalloc.argtypes = [HP, vp, vp, vp, i64, i64, i32, vp, OP, vp]
        L.robe_adagrad_update.restype = ctypes.c_int
        L.robe_adagrad_update.argtypes = [HP, vp, vp, vp, ctypes.c_float, ctypes.c_float, vp]
        L.robe_sgd_update.restype = ctypes.c_int
        L.robe_sgd_update.argtypes = [HP, vp, vp, ctypes.c_float, vp]
        L.robe_fused_workspace_bytes.restype = ctypes.c_int
        L.robe_fused_workspace_bytes.argtypes = [HP, i64, i32, i64, OP, szp]
        L.robe_backward_adagrad.restype = ctypes.c_int
        L.robe_backward_adagrad.argtypes = [HP, vp, vp, vp, i64, i64, i32, vp, vp, ctypes.c_float, ctypes.c_float,
                                            vp, ctypes.c_size_t, OP, vp]
        L.robe_backward_sgd.restype = ctypes.c_int
        L.robe_backward_sgd.argtypes = [HP, vp, vp, vp, i64, i64, i32, vp, ctypes.c_float, vp, ctypes.c_size_t, OP, vp]
        L.robe_forward_mixed.restype = ctypes.c_int
        L.robe_forward_mixed.argtypes = [HP, vp, vp, vp, vp, i64, i64, i32, vp, OP, vp]
        L.robe_mixed_workspace_bytes.restype = ctypes.c_int
        L.robe_mixed_workspace_bytes.argtypes = [HP, vp, i64, i32, i64, OP, szp]
        L.robe_backward_mixed.restype = ctypes.c_int
        L.robe_backward_mixed.argtypes = [HP, vp, vp, vp, vp, i64, i64, i32, vp, vp, ctypes.c_size_t, OP, vp]
        L.robe_fused_mixed_workspace_bytes.restype = ctypes.c_int
        L.robe_fused_mixed_workspace_bytes.argtypes = [HP, vp, i64, i32, i64, OP, szp]
        L.robe_backward_adagrad_mixed.restype = ctypes.c_int
        L.robe_backward_adagrad_mixed.argtypes = [HP, vp, vp, vp, vp, i64, i64, i32, vp, vp, ctypes.c_float, ctypes.c_float,
                                                  vp, ctypes.c_size_t, OP, vp]
        L.robe_array_to_bf16.restype = ctypes.c_int
        L.robe_array_to_bf16.argtypes = [vp, vp, u64, vp]
        L.robe_forward_bf16.restype = ctypes.c_int
        L.robe_forward_bf16.argtypes = [HP, vp, vp, vp, i64, i64, i32, vp, OP, vp]
        L.robe_sort_workspace_bytes.restype = ctypes.c_size_t
        L.robe_sort_workspace_bytes.argtypes = [u64]
        L.robe_sort_pairs.restype = ctypes.c_int
        L.robe_sort_pairs.argtypes = [vp, vp, vp, vp, u64, u32, u32, vp, ctypes.c_size_t,
                                      ctypes.POINTER(ctypes.c_int), vp]
        L.robe_last_error.restype = ctypes.c_char_p
        L.robe_last_error.argtypes = []
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != ROBE_OK:
        raise RobeError(rc, lib().robe_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: Optional[torch.Tensor], dtype: torch.dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: need a contiguous {dtype} tensor on the GPU")
    return t.data_ptr()


def robe_init_hash(seed: int, m: int, d: int, Z: int, use_sign: int) -> RobeHash:
    h = RobeHash()
    _check(lib().robe_init_hash(seed & (2**64 - 1), m, d, Z, int(bool(use_sign)), ctypes.byref(h)))
    return h


def robe_offsets(h: RobeHash, indices: torch.Tensor, n_features: int, want_signs: bool = False):
    """Testing aid: chunk offsets int64[n, d/Z] (and element signs int8[n, d])."""
    n = indices.numel()
    off = torch.empty((n, h.chunks), dtype=torch.int64, device=indices.device)
    sg = torch.empty((n, h.d), dtype=torch.int8, device=indices.device) if want_signs else None
    _check(lib().robe_offsets(ctypes.byref(h), _dev(indices, torch.int64, "indices"), n, n_features,
                              off.data_ptr(), None if sg is None else sg.data_ptr(), _stream()))
    return (off, sg) if want_signs else off


def _opt(options: Optional[RobeOptions]):
    return None if options is None else ctypes.byref(options)


def options(**fields) -> RobeOptions:
    """A ``robe_options_t`` with the given fields set and every other field at its default (0)."""
    o = RobeOptions()
    for k, v in fields.items():
        if k not in {f[0] for f in RobeOptions._fields_} or k == "reserved":
            raise TypeError(f"robe_options_t has no field {k!r}")
        setattr(o, k, v if k in ("probe_begin", "probe_end") else int(v))
    return o


def robe_forward(h: RobeHash, array: torch.Tensor, indices: torch.Tensor, offsets: Optional[torch.Tensor],
                 batch: int, n_features: int, out: Optional[torch.Tensor] = None,
                 options: Optional[RobeOptions] = None) -> torch.Tensor:
    if array.numel() != h.m:
        raise ValueError("array length differs from hash.m")
    if offsets is not None and offsets.numel() != batch * n_features + 1:
        raise ValueError("offsets must hold batch*n_features + 1 entries")
    if out is None:
        out = torch.empty((batch, n_features, h.d), dtype=torch.float32, device=array.device)
    elif out.numel() != batch * n_features * h.d:
        raise ValueError("out has the wrong size")
    _check(lib().robe_forward(ctypes.byref(h), _dev(array, torch.float32, "array"),
                              _dev(indices, torch.int64, "indices"), _dev(offsets, torch.int64, "offsets"),
                              indices.numel(), batch, n_features, _dev(out, torch.float32, "out"), _opt(options), _stream()))
    return out


def robe_workspace_bytes(h: RobeHash, batch: int, n_features: int, n_indices: int,
                         options: Optional[RobeOptions] = None) -> int:
    need = ctypes.c_size_t(0)
    _check(lib().robe_workspace_bytes(ctypes.byref(h), batch, n_features, n_indices, _opt(options), ctypes.byref(need)))
    return int(need.value)


def _workspace(workspace: Optional[torch.Tensor], need: int, device):
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    ws_ptr = None if workspace is None else workspace.data_ptr()
    ws_len = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return workspace, ws_ptr, ws_len


def robe_backward(h: RobeHash, grad_out: torch.Tensor, indices: torch.Tensor, offsets: Optional[torch.Tensor],
                  batch: int, n_features: int, grad_array: torch.Tensor,
                  workspace: Optional[torch.Tensor] = None, options: Optional[RobeOptions] = None) -> torch.Tensor:
    """grad_array += scatter of grad_out (in place); returns grad_array."""
    if grad_array.numel() != h.m:
        raise ValueError("grad_array length differs from hash.m")
    if grad_out.numel() != batch * n_features * h.d:
        raise ValueError("grad_out has the wrong size")
    if offsets is not None and offsets.numel() != batch * n_features + 1:
        raise ValueError("offsets must hold batch*n_features + 1 entries")
    need = robe_workspace_bytes(h, batch, n_features, indices.numel(), options) if workspace is None else 0
    workspace, ws_ptr, ws_len = _workspace(workspace, need, grad_array.device)
    _check(lib().robe_backward(ctypes.byref(h), _dev(grad_out, torch.float32, "grad_out"),
                               _dev(indices, torch.int64, "indices"), _dev(offsets, torch.int64, "offsets"),
                               indices.numel(), batch, n_features, _dev(grad_array, torch.float32, "grad_array"),
                               ws_ptr, ws_len, _opt(options), _stream()))
    return grad_array


def robe_backward_noalloc(h: RobeHash, grad_out: torch.Tensor, indices: torch.Tensor, offsets: Optional[torch.Tensor],
                          batch: int, n_features: int, grad_array: torch.Tensor,
                          options: Optional[RobeOptions] = None) -> torch.Tensor:
    """robe_backward on the library's built-in workspace: nothing is allocated, here or in the library."""
    if grad_array.numel() != h.m:
        raise ValueError("grad_array length differs from hash.m")
    if grad_out.numel() != batch * n_features * h.d:
        raise ValueError("grad_out has the wrong size")
    if offsets is not None and offsets.numel() != batch * n_features + 1:
        raise ValueError("offsets must hold batch*n_features + 1 entries")
    _check(lib().robe_backward_noalloc(ctypes.byref(h), _dev(grad_out, torch.float32, "grad_out"),
                                       _dev(indices, torch.int64, "indices"), _dev(offsets, torch.int64, "offsets"),
                                       indices.numel(), batch, n_features, _dev(grad_array, torch.float32, "grad_array"),
                                       _opt(options), _stream()))
    return grad_array


def robe_adagrad_update(h: RobeHash, array: torch.Tensor, state: torch.Tensor, grad_array: torch.Tensor,
                        lr: float, eps: float) -> None:
    for t, name in ((array, "array"), (state, "state"), (grad_array, "grad_array")):
        if t.numel() != h.m:
            raise ValueError(f"{name} length differs from hash.m")
    _check(lib().robe_adagrad_update(ctypes.byref(h), _dev(array, torch.float32, "array"),
                                     _dev(state, torch.float32, "state"),
                                     _dev(grad_array, torch.float32, "grad_array"), lr, eps, _stream()))


def robe_sgd_update(h: RobeHash, array: torch.Tensor, grad_array: torch.Tensor, lr: float) -> None:
    for t, name in ((array, "array"), (grad_array, "grad_array")):
        if t.numel() != h.m:
            raise ValueError(f"{name} length differs from hash.m")
    _check(lib().robe_sgd_update(ctypes.byref(h), _dev(array, torch.float32, "array"),
                                 _dev(grad_array, torch.float32, "grad_array"), lr, _stream()))


def robe_fused_workspace_bytes(h: RobeHash, batch: int, n_features: int, n_indices: int,
                               options: Optional[RobeOptions] = None) -> int:
    need = ctypes.c_size_t(0)
    _check(lib().robe_fused_workspace_bytes(ctypes.byref(h), batch, n_features, n_indices, _opt(options), ctypes.byref(need)))
    return int(need.value)


def robe_backward_adagrad(h: RobeHash, grad_out: torch.Tensor, indices: torch.Tensor, offsets: Optional[torch.Tensor],
                          batch: int, n_features: int, array: torch.Tensor, state: torch.Tensor,
                          lr: float, eps: float, workspace: Optional[torch.Tensor] = None,
                          options: Optional[RobeOptions] = None) -> None:
    """Backward scatter-add and Adagrad update in one call (array and state updated in place)."""
    for t, name in ((array, "array"), (state, "state")):
        if t.numel() != h.m:
            raise ValueError(f"{name} length differs from hash.m")
    if grad_out.numel() != batch * n_features * h.d:
        raise ValueError("grad_out has the wrong size")
    if offsets is not None and offsets.numel() != batch * n_features + 1:
        raise ValueError("offsets must hold batch*n_features + 1 entries")
    need = robe_fused_workspace_bytes(h, batch, n_features, indices.numel(), options) if workspace is None else 0
    workspace, ws_ptr, ws_len = _workspace(workspace, need, array.device)
    _check(lib().robe_backward_adagrad(ctypes.byref(h), _dev(grad_out, torch.float32, "grad_out"),
                                       _dev(indices, torch.int64, "indices"), _dev(offsets, torch.int64, "offsets"),
                                       indices.numel(), batch, n_features, _dev(array, torch.float32, "array"),
                                       _dev(state, torch.float32, "state"), lr, eps, ws_ptr, ws_len, _opt(options), _stream()))


def robe_backward_sgd(h: RobeHash, grad_out: torch.Tensor, indices: torch.Tensor, offsets: Optional[torch.Tensor],
                      batch: int, n_features: int, array: torch.Tensor, lr: float,
                      workspace: Optional[torch.Tensor] = None, options: Optional[RobeOptions] = None) -> None:
    """Backward scatter-add and SGD update in one call (array updated in place)."""
    if array.numel() != h.m:
        raise ValueError("array length differs from hash.m")
    if grad_out.numel() != batch * n_features * h.d:
        raise ValueError("grad_out has the wrong size")
    if offsets is not None and offsets.numel() != batch * n_features + 1:
        raise ValueError("offsets must hold batch*n_features + 1 entries")
    need = robe_fused_workspace_bytes(h, batch, n_features, indices.numel(), options) if workspace is None else 0
    workspace, ws_ptr, ws_len = _workspace(workspace, need, array.device)
    _check(lib().robe_backward_sgd(ctypes.byref(h), _dev(grad_out, torch.float32, "grad_out"),
                                   _dev(indices, torch.int64, "indices"), _dev(offsets, torch.int64, "offsets"),
                                   indices.numel(), batch, n_features, _dev(array, torch.float32, "array"),
                                   lr, ws_ptr, ws_len, _opt(options), _stream()))


def _dims_array(dims):
    arr = (ctypes.c_uint32 * len(dims))(*[int(d) for d in dims])
    return arr


def robe_forward_mixed(h: RobeHash, dims, array: torch.Tensor, indices: torch.Tensor,
                       offsets: Optional[torch.Tensor], batch: int, out: Optional[torch.Tensor] = None,
                       options: Optional[RobeOptions] = None) -> torch.Tensor:
    """Forward for tables of different dimensions: returns float32[batch, sum(dims)]."""
    F, D = len(dims), int(sum(dims))
    if array.numel() != h.m:
        raise ValueError("array length differs from hash.m")
    if offsets is not None and offsets.numel() != batch * F + 1:
        raise ValueError("offsets must hold batch*n_features + 1 entries")
    if out is None:
        out = torch.empty((batch, D), dtype=torch.float32, device=array.device)
    elif out.numel() != batch * D:
        raise ValueError("out has the wrong size")
    da = _dims_array(dims)
    _check(lib().robe_forward_mixed(ctypes.byref(h), ctypes.cast(da, ctypes.c_void_p), _dev(array, torch.float32, "array"),
                                    _dev(indices, torch.int64, "indices"), _dev(offsets, torch.int64, "offsets"),
                                    indices.numel(), batch, F, _dev(out, torch.float32, "out"), _opt(options), _stream()))
    return out


def robe_mixed_workspace_bytes(h: RobeHash, dims, batch: int, n_indices: int, options: Optional[RobeOptions] = None) -> int:
    need = ctypes.c_size_t(0)
    da = _dims_array(dims)
    _check(lib().robe_mixed_workspace_bytes(ctypes.byref(h), ctypes.cast(da, ctypes.c_void_p), batch, len(dims), n_indices,
                                            _opt(options), ctypes.byref(need)))
    return int(need.value)


def robe_backward_mixed(h: RobeHash, dims, grad_out: torch.Tensor, indices: torch.Tensor,
                        offsets: Optional[torch.Tensor], batch: int, grad_array: torch.Tensor,
                        workspace: Optional[torch.Tensor] = None, options: Optional[RobeOptions] = None) -> None:
    """Backward for tables of different dimensions (accumulates onto grad_array)."""
    F, D = len(dims), int(sum(dims))
    if grad_array.numel() != h.m:
        raise ValueError("grad_array length differs from hash.m")
    if grad_out.numel() != batch * D:
        raise ValueError("grad_out has the wrong size")
    if offsets is not None and offsets.numel() != batch * F + 1:
        raise ValueError("offsets must hold batch*n_features + 1 entries")
    need = robe_mixed_workspace_bytes(h, dims, batch, indices.numel(), options) if workspace is None else 0
    workspace, ws_ptr, ws_len = _workspace(workspace, need, grad_array.device)
    da = _dims_array(dims)
    _check(lib().robe_backward_mixed(ctypes.byref(h), ctypes.cast(da, ctypes.c_void_p), _dev(grad_out, torch.float32, "grad_out"),
                                     _dev(indices, torch.int64, "indices"), _dev(offsets, torch.int64, "offsets"),
                                     indices.numel(), batch, F, _dev(grad_array, torch.float32, "grad_array"),
                                     ws_ptr, ws_len, _opt(options), _stream()))


def robe_fused_mixed_workspace_bytes(h: RobeHash, dims, batch: int, n_indices: int,
                                     options: Optional[RobeOptions] = None) -> int:
    need = ctypes.c_size_t(0)
    da = _dims_array(dims)
    _check(lib().robe_fused_mixed_workspace_bytes(ctypes.byref(h), ctypes.cast(da, ctypes.c_void_p), batch, len(dims), n_indices,
                                                  _opt(options), ctypes.byref(need)))
    return int(need.value)


def robe_backward_adagrad_mixed(h: RobeHash, dims, grad_out: torch.Tensor, indices: torch.Tensor,
                                offsets: Optional[torch.Tensor], batch: int, array: torch.Tensor, state: torch.Tensor,
                                lr: float, eps: float, workspace: Optional[torch.Tensor] = None,
                                options: Optional[RobeOptions] = None) -> None:
    """Backward and Adagrad in one call for tables of different dimensions (array and state in place)."""
    F, D = len(dims), int(sum(dims))
    if array.numel() != h.m or state.numel() != h.m:
        raise ValueError("array / state length differs from hash.m")
    if grad_out.numel() != batch * D:
        raise ValueError("grad_out has the wrong size")
    if offsets is not None and offsets.numel() != batch * F + 1:
        raise ValueError("offsets must hold batch*n_features + 1 entries")
    need = robe_fused_mixed_workspace_bytes(h, dims, batch, indices.numel(), options) if workspace is None else 0
    workspace, ws_ptr, ws_len = _workspace(workspace, need, array.device)
    da = _dims_array(dims)
    _check(lib().robe_backward_adagrad_mixed(ctypes.byref(h), ctypes.cast(da, ctypes.c_void_p),
                                             _dev(grad_out, torch.float32, "grad_out"), _dev(indices, torch.int64, "indices"),
                                             _dev(offsets, torch.int64, "offsets"), indices.numel(), batch, F,
                                             _dev(array, torch.float32, "array"), _dev(state, torch.float32, "state"),
                                             lr, eps, ws_ptr, ws_len, _opt(options), _stream()))


def robe_array_to_bf16(array: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """float32 device array -> bfloat16 bit patterns (int16 tensor of the same length)."""
    if out is None:
        out = torch.empty(array.numel(), dtype=torch.int16, device=array.device)
    elif out.numel() != array.numel():
        raise ValueError("out has the wrong size")
    _check(lib().robe_array_to_bf16(_dev(array, torch.float32, "array"), _dev(out, torch.int16, "out"),
                                    array.numel(), _stream()))
    return out


def robe_forward_bf16(h: RobeHash, array_bf16: torch.Tensor, indices: torch.Tensor, offsets: Optional[torch.Tensor],
                      batch: int, n_features: int, out: Optional[torch.Tensor] = None,
                      options: Optional[RobeOptions] = None) -> torch.Tensor:
    """robe_forward on an array of bfloat16 bit patterns (int16 tensor of length m)."""
    if array_bf16.numel() != h.m:
        raise ValueError("array length differs from hash.m")
    if offsets is not None and offsets.numel() != batch * n_features + 1:
        raise ValueError("offsets must hold batch*n_features + 1 entries")
    if out is None:
        out = torch.empty((batch, n_features, h.d), dtype=torch.float32, device=array_bf16.device)
    elif out.numel() != batch * n_features * h.d:
        raise ValueError("out has the wrong size")
    _check(lib().robe_forward_bf16(ctypes.byref(h), _dev(array_bf16, torch.int16, "array"),
                                   _dev(indices, torch.int64, "indices"), _dev(offsets, torch.int64, "offsets"),
                                   indices.numel(), batch, n_features, _dev(out, torch.float32, "out"), _opt(options), _stream()))
    return out


def robe_sort_pairs(keys: torch.Tensor, vals: torch.Tensor, lo_bit: int, hi_bit: int):
    """Stable sort of (key, value) pairs (int32 tensors holding 32-bit patterns) by key bits [lo_bit, hi_bit).
    The inputs are overwritten; returns the sorted (keys, vals)."""
    n = keys.numel()
    if vals.numel() != n:
        raise ValueError("keys and vals differ in length")
    kb, vb = torch.empty_like(keys), torch.empty_like(vals)
    need = int(lib().robe_sort_workspace_bytes(n))
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device=keys.device)
    in_b = ctypes.c_int(0)
    _check(lib().robe_sort_pairs(_dev(keys, torch.int32, "keys"), _dev(vals, torch.int32, "vals"),
                                 _dev(kb, torch.int32, "keys_b"), _dev(vb, torch.int32, "vals_b"), n, lo_bit, hi_bit,
                                 ws.data_ptr(), need, ctypes.byref(in_b), _stream()))
    return (kb, vb) if in_b.value else (keys, vals)
