"""ctypes binding of libfsdp_flat: argument marshalling only.

Every function here has the name and argument order of the C entry point it
wraps (include/fsdp_flat.h).  Tensors are checked (device, dtype, contiguity,
size) and reduced to raw device addresses; all work happens in the library's
HIP kernels.  There is no CPU fallback: if the library is not built, loading
fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

FSDP_F32 = 0
FSDP_BF16 = 1
FSDP_F16 = 2
FSDP_WALK_AUTO = 0
FSDP_WALK_WIDE = 1
FSDP_WALK_DEEP = 2
FSDP_WALK_HALF = 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfsdp_flat.so")

_STATUS = {
    0: "ok", -1: "invalid argument", -2: "null pointer", -3: "size overflows int64",
    -4: "host allocation failed", -5: "bad dtype", -6: "rank or parameter index out of range",
    -7: "HIP launch error",
}


class FsdpError(RuntimeError):
    def __init__(self, fn: str, status: int, hip_error: int = 0):
        self.status = status
        self.hip_error = hip_error
        msg = f"{fn} failed: {status} ({_STATUS.get(status, 'unknown')})"
        if status == -7:
            msg += f", hipError_t={hip_error}"
        super().__init__(msg)


def library_path() -> str:
    return _LIB_PATH


_lib = None

_i32, _i64, _f32, _vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p
_pp = ctypes.POINTER(ctypes.c_void_p)

_SIGNATURES = {
    "fsdp_layout_init": [ctypes.POINTER(_i64), ctypes.POINTER(_i32), _i32, _i32, ctypes.POINTER(_vp)],
    "fsdp_layout_init_ex": [ctypes.POINTER(_i64), ctypes.POINTER(_i32), _i32, _i32, _i32, ctypes.POINTER(_vp)],
    "fsdp_layout_info": [_vp, ctypes.POINTER(_i64), ctypes.POINTER(_i64), ctypes.POINTER(_i64),
                         ctypes.POINTER(_i64), ctypes.POINTER(_i32), ctypes.POINTER(_i32)],
    "fsdp_layout_param": [_vp, _i32, ctypes.POINTER(_i64), ctypes.POINTER(_i64)],
    "fsdp_view_ptr": [_vp, _vp, ctypes.c_int, _i32, ctypes.POINTER(_vp)],
    "fsdp_default_divide_factors": [_i32, ctypes.POINTER(_f32), ctypes.POINTER(_f32)],
    "fsdp_flatten_shard": [_vp, _pp, _pp, _vp],
    "fsdp_unshard": [_vp, _pp, _vp, ctypes.c_int, _vp],
    "fsdp_reduce_scatter_local": [_vp, _pp, ctypes.c_int, _i32, _f32, _f32, _vp, _vp],
    "fsdp_shard_adam_step": [_vp, _vp, _vp, _vp, _vp, _i64, _f32, _f32, _f32, _f32, _vp],
    "fsdp_reduce_scatter_adam_fused": [_vp, _pp, ctypes.c_int, _i32, _f32, _f32, _vp, _vp, _vp, _vp, _i64,
                                       _f32, _f32, _f32, _f32, _vp, _vp],
    "fsdp_reduce_scatter_adam_prefetch_unshard": [_vp, _pp, ctypes.c_int, _i32, _f32, _f32, _vp, _vp, _vp, _vp, _i64,
                                                  _f32, _f32, _f32, _f32, _vp, _vp, _pp, _vp, ctypes.c_int, _vp],
    "fsdp_reduce_scatter_hybrid": [_vp, _pp, ctypes.c_int, _i32, _i32, _f32, _f32, _vp, _vp],
    "fsdp_reduce_scatter_hybrid_adam_fused": [_vp, _pp, ctypes.c_int, _i32, _i32, _f32, _f32, _vp, _vp, _vp, _vp, _i64,
                                              _f32, _f32, _f32, _f32, _vp, _vp],
    "fsdp_reduce_scatter_accumulate": [_vp, _pp, ctypes.c_int, _i32, _f32, _f32, _vp, _vp],
    "fsdp_reduce_scatter_accumulate_adam_fused": [_vp, _pp, ctypes.c_int, _i32, _f32, _f32, _vp, _vp, _vp, _vp, _i64,
                                                  _f32, _f32, _f32, _f32, _vp, _vp],
    "fsdp_grad_accumulate": [_vp, _vp, _vp, ctypes.c_int, _vp],
    "fsdp_cast_shard": [_vp, _vp, _vp, ctypes.c_int, _vp],
    "fsdp_reduce_scatter_unscale": [_vp, _pp, ctypes.c_int, _i32, _f32, _f32, _f32, _vp, _vp, _vp],
    "fsdp_found_inf_combine": [_pp, _i32, _vp],
    "fsdp_shard_adam_step_guarded": [_vp, _vp, _vp, _vp, _vp, _i64, _f32, _f32, _f32, _f32, _vp, _vp],
    "fsdp_grad_scaler_update": [_vp, _vp, _vp, _f32, _f32, _i32, _vp],
    "fsdp_unshard_lp": [_vp, _pp, _vp, _vp],
    "fsdp_batch_create": [ctypes.POINTER(_vp)],
    "fsdp_batch_clear": [_vp],
    "fsdp_batch_add_unshard": [_vp, _vp, _pp, _vp, ctypes.c_int],
    "fsdp_batch_add_unshard_lp": [_vp, _vp, _pp, _vp],
    "fsdp_batch_add_reduce_scatter_adam": [_vp, _vp, _pp, ctypes.c_int, _i32, _f32, _f32, _vp, _vp, _vp, _vp,
                                           _f32, _f32, _f32, _f32, _vp],
    "fsdp_batch_launch": [_vp, _i64, _vp],
    "fsdp_batch_launch_count": [_vp, ctypes.POINTER(_i32)],
    "fsdp_batch_launch_info": [_vp, _i32, ctypes.POINTER(_i32), ctypes.POINTER(_i32), ctypes.POINTER(_i32),
                               ctypes.POINTER(_i64)],
    "fsdp_last_hip_error": [],
}


def lib() -> ctypes.CDLL:
    """Load libfsdp_flat.so (built in-tree by paper_2304_11277_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is not built; run `python -m paper_2304_11277_amd.build` "
                "(there is no fallback path)")
        l = ctypes.CDLL(_LIB_PATH)
        for name, argtypes in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.argtypes = argtypes
            fn.restype = ctypes.c_int
        l.fsdp_layout_destroy.argtypes = [_vp]
        l.fsdp_layout_destroy.restype = None
        l.fsdp_batch_destroy.argtypes = [_vp]
        l.fsdp_batch_destroy.restype = None
        l.fsdp_status_string.argtypes = [ctypes.c_int]
        l.fsdp_status_string.restype = ctypes.c_char_p
        l.fsdp_kernel_name.argtypes = [_i32]
        l.fsdp_kernel_name.restype = ctypes.c_char_p
        _lib = l
    return _lib


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise FsdpError(fn, status, lib().fsdp_last_hip_error() if status == -7 else 0)


class PtrArray:
    """A host array of device addresses, marshalled once and reusable across
    calls (keeps the tensors alive).  The tensors are checked here (device
    tensors of one device and one dtype, contiguous) and their dtype and sizes
    recorded, so that every call that takes the array can compare them with
    what its layout needs before anything is launched.  `allow_empty` admits
    zero-element entries (a null address, never dereferenced)."""

    def __init__(self, tensors: Sequence[torch.Tensor], allow_empty: bool = False, _device_check: bool = True):
        self.tensors = list(tensors)
        self.dtype = None
        self.device = None
        self.numels: List[int] = []
        # False only in CPU tests of the checks below; such an array is refused by every call
        self.device_checked = bool(_device_check)
        addrs = []
        for i, t in enumerate(self.tensors):
            if not isinstance(t, torch.Tensor):
                raise TypeError(f"PtrArray[{i}]: expected a tensor, got {type(t).__name__}")
            self.numels.append(t.numel())
            if t.numel() == 0 and allow_empty:
                addrs.append(0)
                continue
            if _device_check and not t.is_cuda:
                raise TypeError(f"PtrArray[{i}]: expected a device tensor, got one on {t.device}")
            if not t.is_contiguous():
                raise ValueError(f"PtrArray[{i}]: must be contiguous")
            if self.dtype is None:
                self.dtype, self.device = t.dtype, t.device
            elif t.dtype != self.dtype:
                raise TypeError(f"PtrArray[{i}]: {t.dtype} in a table of {self.dtype}")
            elif t.device != self.device:
                raise ValueError(f"PtrArray[{i}]: on {t.device} in a table on {self.device}")
            addrs.append(t.data_ptr())
        self.array = (ctypes.c_void_p * max(1, len(addrs)))(*addrs)
        self.n = len(addrs)


def _stream_handle(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def _dev_tensor(t: torch.Tensor, dtype, min_numel: int, what: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what}: expected a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: must be contiguous")
    if t.numel() < min_numel:
        raise ValueError(f"{what}: needs at least {min_numel} elements, has {t.numel()}")
    return t.data_ptr()


def _ptr_table(ts, dtype, min_numel, n_expected: int, what: str, allow_empty=False) -> PtrArray:
    """Checked pointer table: `ts` is a sequence of tensors or a PtrArray built
    earlier; either way every entry must be a contiguous device tensor of
    `dtype` with at least min_numel (one number, or one per entry) elements."""
    tab = ts if isinstance(ts, PtrArray) else PtrArray(list(ts), allow_empty=allow_empty)
    if tab.n != n_expected:
        raise ValueError(f"{what}: expected {n_expected} entries, got {tab.n}")
    if not tab.device_checked:
        raise TypeError(f"{what}: built without the device check")
    for i, have in enumerate(tab.numels):
        need = min_numel[i] if isinstance(min_numel, (list, tuple)) else min_numel
        if allow_empty and need == 0:
            continue
        if have < need:
            raise ValueError(f"{what}[{i}]: needs at least {need} elements, has {have}")
        if have == 0:
            raise ValueError(f"{what}[{i}]: empty tensor where {need} elements are read or written")
    if tab.dtype is not None and tab.dtype != dtype:
        raise TypeError(f"{what}: expected {dtype}, got {tab.dtype}")
    return tab


class Layout:
    """Owner of a fsdp_layout_t handle (the FlatParamHandle's bookkeeping,
    Sec. 4.2): offsets, N, S, P, pad."""

    def __init__(self, handle: int, shapes: Sequence[Tuple[int, ...]]):
        self._h = ctypes.c_void_p(handle)
        self.shapes = [tuple(int(d) for d in s) for s in shapes]
        N, P, S, pad = _i64(), _i64(), _i64(), _i64()
        p, W = _i32(), _i32()
        _check("fsdp_layout_info", lib().fsdp_layout_info(self._h, ctypes.byref(N), ctypes.byref(P), ctypes.byref(S),
                                                         ctypes.byref(pad), ctypes.byref(p), ctypes.byref(W)))
        self.numel, self.padded, self.shard, self.pad = N.value, P.value, S.value, pad.value
        self.num_params, self.world_size = p.value, W.value
        self.offsets: List[int] = []
        self.numels: List[int] = []
        for i in range(self.num_params):
            o, n = _i64(), _i64()
            _check("fsdp_layout_param", lib().fsdp_layout_param(self._h, i, ctypes.byref(o), ctypes.byref(n)))
            self.offsets.append(o.value)
            self.numels.append(n.value)

    @property
    def handle(self) -> ctypes.c_void_p:
        if self._h is None:
            raise ValueError("layout was destroyed")
        return self._h

    def close(self) -> None:
        if self._h is not None:
            lib().fsdp_layout_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def fsdp_layout_init(shapes: Sequence[Sequence[int]], world_size: int, reduce_walk: Optional[int] = None) -> Layout:
    """fsdp_layout_init, or fsdp_layout_init_ex when a rank-walk hint
    (FSDP_WALK_AUTO / _WIDE / _DEEP / _HALF) is given."""
    shapes = [tuple(int(d) for d in s) for s in shapes]
    flat = [d for s in shapes for d in s]
    dims = (_i64 * max(1, len(flat)))(*flat)
    ndims = (_i32 * max(1, len(shapes)))(*[len(s) for s in shapes])
    out = _vp()
    if reduce_walk is None:
        _check("fsdp_layout_init", lib().fsdp_layout_init(dims, ndims, len(shapes), int(world_size), ctypes.byref(out)))
    else:
        _check("fsdp_layout_init_ex", lib().fsdp_layout_init_ex(dims, ndims, len(shapes), int(world_size),
                                                                int(reduce_walk), ctypes.byref(out)))
    return Layout(out.value, shapes)


fsdp_layout_init_ex = fsdp_layout_init


def fsdp_default_divide_factors(world_size: int) -> Tuple[float, float]:
    pre, post = _f32(), _f32()
    _check("fsdp_default_divide_factors",
           lib().fsdp_default_divide_factors(int(world_size), ctypes.byref(pre), ctypes.byref(post)))
    return pre.value, post.value


_DTYPES = {torch.float32: FSDP_F32, torch.bfloat16: FSDP_BF16, torch.float16: FSDP_F16}


def _flat_dtype(t: torch.Tensor) -> int:
    try:
        return _DTYPES[t.dtype]
    except KeyError:
        raise TypeError(f"unsupported dtype {t.dtype}") from None


def fsdp_view_ptr(layout: Layout, flat_base: torch.Tensor, i: int) -> int:
    """Device address of parameter i inside the unsharded flat buffer."""
    out = _vp()
    _check("fsdp_view_ptr", lib().fsdp_view_ptr(layout.handle, _vp(flat_base.data_ptr()), _flat_dtype(flat_base),
                                                int(i), ctypes.byref(out)))
    return out.value or 0


def fsdp_views(layout: Layout, flat: torch.Tensor) -> List[torch.Tensor]:
    """Zero-copy per-parameter tensors over the unsharded flat buffer
    (Sec. 3.2.3); their addresses are the ones fsdp_view_ptr returns."""
    views = []
    for i, shp in enumerate(layout.shapes):
        v = flat[layout.offsets[i]:layout.offsets[i] + layout.numels[i]].view(shp)
        if v.numel() and v.data_ptr() != fsdp_view_ptr(layout, flat, i):
            raise AssertionError("view address mismatch")
        views.append(v)
    return views


def fsdp_flatten_shard(layout: Layout, param_ptrs, shard_ptrs, stream=None) -> None:
    params = _ptr_table(param_ptrs, torch.float32, layout.numels, layout.num_params, "param_ptrs", allow_empty=True)
    shards = _ptr_table(shard_ptrs, torch.float32, layout.shard, layout.world_size, "shard_ptrs")
    _check("fsdp_flatten_shard", lib().fsdp_flatten_shard(layout.handle, params.array, shards.array,
                                                         _stream_handle(stream)))


def fsdp_unshard(layout: Layout, shard_ptrs, flat_out: torch.Tensor, stream=None) -> None:
    shards = _ptr_table(shard_ptrs, torch.float32, layout.shard, layout.world_size, "shard_ptrs")
    dt = _flat_dtype(flat_out)
    _dev_tensor(flat_out, flat_out.dtype, layout.padded, "flat_out")
    _check("fsdp_unshard", lib().fsdp_unshard(layout.handle, shards.array, _vp(flat_out.data_ptr()), dt,
                                              _stream_handle(stream)))


def _grad_table(layout: Layout, grad_ptrs, num_groups: int = 1) -> Tuple[PtrArray, int]:
    tab = grad_ptrs if isinstance(grad_ptrs, PtrArray) else PtrArray(list(grad_ptrs))
    gdt = tab.dtype
    if gdt not in _DTYPES:
        raise TypeError(f"grad dtype {gdt} not supported")
    tab = _ptr_table(tab, gdt, layout.padded, layout.world_size * num_groups, "grad_ptrs")
    return tab, _DTYPES[gdt]


def fsdp_reduce_scatter_local(layout: Layout, grad_ptrs, rank: int, pre_div: float, post_div: float,
                              grad_shard_out: torch.Tensor, stream=None) -> None:
    tab, gdt = _grad_table(layout, grad_ptrs)
    _dev_tensor(grad_shard_out, torch.float32, layout.shard, "grad_shard_out")
    _check("fsdp_reduce_scatter_local",
           lib().fsdp_reduce_scatter_local(layout.handle, tab.array, gdt, int(rank), float(pre_div), float(post_div),
                                           _vp(grad_shard_out.data_ptr()), _stream_handle(stream)))


def fsdp_shard_adam_step(layout: Layout, p_shard, g_shard, exp_avg, exp_avg_sq, step: int, lr: float, beta1: float,
                         beta2: float, eps: float, stream=None) -> None:
    S = layout.shard
    ptrs = [_dev_tensor(t, torch.float32, S, n) for t, n in
            ((p_shard, "p_shard"), (g_shard, "g_shard"), (exp_avg, "exp_avg"), (exp_avg_sq, "exp_avg_sq"))]
    _check("fsdp_shard_adam_step",
           lib().fsdp_shard_adam_step(layout.handle, *[_vp(x) for x in ptrs], int(step), float(lr), float(beta1),
                                      float(beta2), float(eps), _stream_handle(stream)))


def fsdp_reduce_scatter_adam_fused(layout: Layout, grad_ptrs, rank: int, pre_div: float, post_div: float,
                                   grad_shard_out: Optional[torch.Tensor], p_shard, exp_avg, exp_avg_sq, step: int,
                                   lr: float, beta1: float, beta2: float, eps: float,
                                   p_lp_out: Optional[torch.Tensor] = None, stream=None) -> None:
    tab, gdt = _grad_table(layout, grad_ptrs)
    S = layout.shard
    g_out = _dev_tensor(grad_shard_out, torch.float32, S, "grad_shard_out") if grad_shard_out is not None else None
    lp = _dev_tensor(p_lp_out, torch.bfloat16, S, "p_lp_out") if p_lp_out is not None else None
    ptrs = [_dev_tensor(t, torch.float32, S, n) for t, n in
            ((p_shard, "p_shard"), (exp_avg, "exp_avg"), (exp_avg_sq, "exp_avg_sq"))]
    _check("fsdp_reduce_scatter_adam_fused",
           lib().fsdp_reduce_scatter_adam_fused(layout.handle, tab.array, gdt, int(rank), float(pre_div),
                                                float(post_div), _vp(g_out), *[_vp(x) for x in ptrs], int(step),
                                                float(lr), float(beta1), float(beta2), float(eps), _vp(lp),
                                                _stream_handle(stream)))


def fsdp_reduce_scatter_adam_prefetch_unshard(layout: Layout, grad_ptrs, rank: int, pre_div: float, post_div: float,
                                              grad_shard_out: Optional[torch.Tensor], p_shard, exp_avg, exp_avg_sq,
                                              step: int, lr: float, beta1: float, beta2: float, eps: float,
                                              p_lp_out: Optional[torch.Tensor], next_layout: Layout, next_shard_ptrs,
                                              next_flat_out: torch.Tensor, stream=None) -> None:
    tab, gdt = _grad_table(layout, grad_ptrs)
    S = layout.shard
    g_out = _dev_tensor(grad_shard_out, torch.float32, S, "grad_shard_out") if grad_shard_out is not None else None
    lp = _dev_tensor(p_lp_out, torch.bfloat16, S, "p_lp_out") if p_lp_out is not None else None
    ptrs = [_dev_tensor(t, torch.float32, S, n) for t, n in
            ((p_shard, "p_shard"), (exp_avg, "exp_avg"), (exp_avg_sq, "exp_avg_sq"))]
    shards = _ptr_table(next_shard_ptrs, torch.float32, next_layout.shard, next_layout.world_size, "next_shard_ptrs")
    dt = _flat_dtype(next_flat_out)
    _dev_tensor(next_flat_out, next_flat_out.dtype, next_layout.padded, "next_flat_out")
    _check("fsdp_reduce_scatter_adam_prefetch_unshard",
           lib().fsdp_reduce_scatter_adam_prefetch_unshard(
               layout.handle, tab.array, gdt, int(rank), float(pre_div), float(post_div), _vp(g_out),
               *[_vp(x) for x in ptrs], int(step), float(lr), float(beta1), float(beta2), float(eps), _vp(lp),
               next_layout.handle, shards.array, _vp(next_flat_out.data_ptr()), dt, _stream_handle(stream)))


def fsdp_reduce_scatter_hybrid(layout: Layout, grad_ptrs, num_groups: int, rank: int, pre_div: float,
                               post_div: float, grad_shard_out: torch.Tensor, stream=None) -> None:
    tab, gdt = _grad_table(layout, grad_ptrs, num_groups)
    _dev_tensor(grad_shard_out, torch.float32, layout.shard, "grad_shard_out")
    _check("fsdp_reduce_scatter_hybrid",
           lib().fsdp_reduce_scatter_hybrid(layout.handle, tab.array, gdt, int(num_groups), int(rank), float(pre_div),
                                            float(post_div), _vp(grad_shard_out.data_ptr()), _stream_handle(stream)))


def fsdp_reduce_scatter_hybrid_adam_fused(layout: Layout, grad_ptrs, num_groups: int, rank: int, pre_div: float,
                                          post_div: float, grad_shard_out: Optional[torch.Tensor], p_shard, exp_avg,
                                          exp_avg_sq, step: int, lr: float, beta1: float, beta2: float, eps: float,
                                          p_lp_out: Optional[torch.Tensor] = None, stream=None) -> None:
    tab, gdt = _grad_table(layout, grad_ptrs, num_groups)
    S = layout.shard
    g_out = _dev_tensor(grad_shard_out, torch.float32, S, "grad_shard_out") if grad_shard_out is not None else None
    lp = _dev_tensor(p_lp_out, torch.bfloat16, S, "p_lp_out") if p_lp_out is not None else None
    ptrs = [_dev_tensor(t, torch.float32, S, n) for t, n in
            ((p_shard, "p_shard"), (exp_avg, "exp_avg"), (exp_avg_sq, "exp_avg_sq"))]
    _check("fsdp_reduce_scatter_hybrid_adam_fused",
           lib().fsdp_reduce_scatter_hybrid_adam_fused(layout.handle, tab.array, gdt, int(num_groups), int(rank),
                                                       float(pre_div), float(post_div), _vp(g_out),
                                                       *[_vp(x) for x in ptrs], int(step), float(lr), float(beta1),
                                                       float(beta2), float(eps), _vp(lp), _stream_handle(stream)))


def fsdp_reduce_scatter_accumulate(layout: Layout, grad_ptrs, rank: int, pre_div: float, post_div: float,
                                   grad_shard_acc: torch.Tensor, stream=None) -> None:
    tab, gdt = _grad_table(layout, grad_ptrs)
    _dev_tensor(grad_shard_acc, torch.float32, layout.shard, "grad_shard_acc")
    _check("fsdp_reduce_scatter_accumulate",
           lib().fsdp_reduce_scatter_accumulate(layout.handle, tab.array, gdt, int(rank), float(pre_div),
                                                float(post_div), _vp(grad_shard_acc.data_ptr()),
                                                _stream_handle(stream)))


def fsdp_reduce_scatter_accumulate_adam_fused(layout: Layout, grad_ptrs, rank: int, pre_div: float, post_div: float,
                                              grad_shard_acc: torch.Tensor, p_shard, exp_avg, exp_avg_sq, step: int,
                                              lr: float, beta1: float, beta2: float, eps: float,
                                              p_lp_out: Optional[torch.Tensor] = None, stream=None) -> None:
    tab, gdt = _grad_table(layout, grad_ptrs)
    S = layout.shard
    acc = _dev_tensor(grad_shard_acc, torch.float32, S, "grad_shard_acc")
    lp = _dev_tensor(p_lp_out, torch.bfloat16, S, "p_lp_out") if p_lp_out is not None else None
    ptrs = [_dev_tensor(t, torch.float32, S, n) for t, n in
            ((p_shard, "p_shard"), (exp_avg, "exp_avg"), (exp_avg_sq, "exp_avg_sq"))]
    _check("fsdp_reduce_scatter_accumulate_adam_fused",
           lib().fsdp_reduce_scatter_accumulate_adam_fused(layout.handle, tab.array, gdt, int(rank), float(pre_div),
                                                           float(post_div), _vp(acc), *[_vp(x) for x in ptrs],
                                                           int(step), float(lr), float(beta1), float(beta2),
                                                           float(eps), _vp(lp), _stream_handle(stream)))


def fsdp_grad_accumulate(layout: Layout, grad_acc: torch.Tensor, grad_add: torch.Tensor, stream=None) -> None:
    _dev_tensor(grad_acc, torch.float32, layout.padded, "grad_acc")
    dt = _flat_dtype(grad_add)
    _dev_tensor(grad_add, grad_add.dtype, layout.padded, "grad_add")
    _check("fsdp_grad_accumulate",
           lib().fsdp_grad_accumulate(layout.handle, _vp(grad_acc.data_ptr()), _vp(grad_add.data_ptr()), dt,
                                      _stream_handle(stream)))


def fsdp_cast_shard(layout: Layout, shard: torch.Tensor, lp_shard_out: torch.Tensor, stream=None) -> None:
    _dev_tensor(shard, torch.float32, layout.shard, "shard")
    if lp_shard_out.dtype not in (torch.bfloat16, torch.float16):
        raise TypeError("lp_shard_out must be bfloat16 or float16")
    _dev_tensor(lp_shard_out, lp_shard_out.dtype, layout.shard, "lp_shard_out")
    _check("fsdp_cast_shard", lib().fsdp_cast_shard(layout.handle, _vp(shard.data_ptr()),
                                                   _vp(lp_shard_out.data_ptr()), _flat_dtype(lp_shard_out),
                                                   _stream_handle(stream)))


def fsdp_unshard_lp(layout: Layout, lp_shard_ptrs, flat_out: torch.Tensor, stream=None) -> None:
    if flat_out.dtype not in (torch.bfloat16, torch.float16):
        raise TypeError("flat_out must be bfloat16 or float16")
    shards = _ptr_table(lp_shard_ptrs, flat_out.dtype, layout.shard, layout.world_size, "lp_shard_ptrs")
    _dev_tensor(flat_out, flat_out.dtype, layout.padded, "flat_out")
    _check("fsdp_unshard_lp", lib().fsdp_unshard_lp(layout.handle, shards.array, _vp(flat_out.data_ptr()),
                                                   _stream_handle(stream)))


def fsdp_reduce_scatter_unscale(layout: Layout, grad_ptrs, rank: int, pre_div: float, post_div: float,
                                inv_scale: float, grad_shard_out: torch.Tensor, found_inf: torch.Tensor,
                                stream=None) -> None:
    tab, gdt = _grad_table(layout, grad_ptrs)
    _dev_tensor(grad_shard_out, torch.float32, layout.shard, "grad_shard_out")
    _dev_tensor(found_inf, torch.float32, 1, "found_inf")
    _check("fsdp_reduce_scatter_unscale",
           lib().fsdp_reduce_scatter_unscale(layout.handle, tab.array, gdt, int(rank), float(pre_div), float(post_div),
                                             float(inv_scale), _vp(grad_shard_out.data_ptr()),
                                             _vp(found_inf.data_ptr()), _stream_handle(stream)))


def fsdp_found_inf_combine(found_inf_ptrs, stream=None) -> None:
    flags = list(found_inf_ptrs)
    for i, f in enumerate(flags):
        _dev_tensor(f, torch.float32, 1, f"found_inf_ptrs[{i}]")
    tab = PtrArray(flags)
    _check("fsdp_found_inf_combine", lib().fsdp_found_inf_combine(tab.array, len(flags), _stream_handle(stream)))


def fsdp_shard_adam_step_guarded(layout: Layout, p_shard, g_shard, exp_avg, exp_avg_sq, step: int, lr: float,
                                 beta1: float, beta2: float, eps: float, found_inf: torch.Tensor, stream=None) -> None:
    S = layout.shard
    ptrs = [_dev_tensor(t, torch.float32, S, n) for t, n in
            ((p_shard, "p_shard"), (g_shard, "g_shard"), (exp_avg, "exp_avg"), (exp_avg_sq, "exp_avg_sq"))]
    _dev_tensor(found_inf, torch.float32, 1, "found_inf")
    _check("fsdp_shard_adam_step_guarded",
           lib().fsdp_shard_adam_step_guarded(layout.handle, *[_vp(x) for x in ptrs], int(step), float(lr),
                                              float(beta1), float(beta2), float(eps), _vp(found_inf.data_ptr()),
                                              _stream_handle(stream)))


def fsdp_grad_scaler_update(scale: torch.Tensor, growth_tracker: torch.Tensor, found_inf: torch.Tensor,
                            growth_factor: float = 2.0, backoff_factor: float = 0.5, growth_interval: int = 2000,
                            stream=None) -> None:
    _dev_tensor(scale, torch.float32, 1, "scale")
    _dev_tensor(growth_tracker, torch.int32, 1, "growth_tracker")
    _dev_tensor(found_inf, torch.float32, 1, "found_inf")
    _check("fsdp_grad_scaler_update",
           lib().fsdp_grad_scaler_update(_vp(scale.data_ptr()), _vp(growth_tracker.data_ptr()),
                                         _vp(found_inf.data_ptr()), float(growth_factor), float(backoff_factor),
                                         int(growth_interval), _stream_handle(stream)))


class Batch:
    """Owner of a fsdp_batch_t: independent operations issued in few launches.
    Keeps the tensors and layouts it was given alive."""

    def __init__(self):
        h = _vp()
        _check("fsdp_batch_create", lib().fsdp_batch_create(ctypes.byref(h)))
        self._h = h
        self._keep = []

    def clear(self) -> None:
        _check("fsdp_batch_clear", lib().fsdp_batch_clear(self._h))
        self._keep = []

    def add_unshard(self, layout: Layout, shard_ptrs, flat_out: torch.Tensor) -> None:
        shards = _ptr_table(shard_ptrs, torch.float32, layout.shard, layout.world_size, "shard_ptrs")
        dt = _flat_dtype(flat_out)
        _dev_tensor(flat_out, flat_out.dtype, layout.padded, "flat_out")
        _check("fsdp_batch_add_unshard",
               lib().fsdp_batch_add_unshard(self._h, layout.handle, shards.array, _vp(flat_out.data_ptr()), dt))
        self._keep += [layout, shards, flat_out]

    def add_unshard_lp(self, layout: Layout, lp_shard_ptrs, flat_out: torch.Tensor) -> None:
        if flat_out.dtype not in (torch.bfloat16, torch.float16):
            raise TypeError("flat_out must be bfloat16 or float16")
        shards = _ptr_table(lp_shard_ptrs, flat_out.dtype, layout.shard, layout.world_size, "lp_shard_ptrs")
        _dev_tensor(flat_out, flat_out.dtype, layout.padded, "flat_out")
        _check("fsdp_batch_add_unshard_lp",
               lib().fsdp_batch_add_unshard_lp(self._h, layout.handle, shards.array, _vp(flat_out.data_ptr())))
        self._keep += [layout, shards, flat_out]

    def add_reduce_scatter_adam(self, layout: Layout, grad_ptrs, rank: int, pre_div: float, post_div: float,
                                grad_shard_out: Optional[torch.Tensor], p_shard, exp_avg, exp_avg_sq, lr: float,
                                beta1: float, beta2: float, eps: float,
                                p_lp_out: Optional[torch.Tensor] = None) -> None:
        tab, gdt = _grad_table(layout, grad_ptrs)
        S = layout.shard
        g_out = _dev_tensor(grad_shard_out, torch.float32, S, "grad_shard_out") if grad_shard_out is not None else None
        lp = _dev_tensor(p_lp_out, torch.bfloat16, S, "p_lp_out") if p_lp_out is not None else None
        ptrs = [_dev_tensor(t, torch.float32, S, n) for t, n in
                ((p_shard, "p_shard"), (exp_avg, "exp_avg"), (exp_avg_sq, "exp_avg_sq"))]
        _check("fsdp_batch_add_reduce_scatter_adam",
               lib().fsdp_batch_add_reduce_scatter_adam(self._h, layout.handle, tab.array, gdt, int(rank),
                                                        float(pre_div), float(post_div), _vp(g_out),
                                                        *[_vp(x) for x in ptrs], float(lr), float(beta1),
                                                        float(beta2), float(eps), _vp(lp)))
        self._keep += [layout, tab, grad_shard_out, p_shard, exp_avg, exp_avg_sq, p_lp_out]

    def launch(self, step: int, stream=None) -> None:
        _check("fsdp_batch_launch", lib().fsdp_batch_launch(self._h, int(step), _stream_handle(stream)))

    def launches(self) -> List[dict]:
        """fsdp_batch_launch_count / _info: the kernel launches one launch() call issues."""
        n = _i32()
        _check("fsdp_batch_launch_count", lib().fsdp_batch_launch_count(self._h, ctypes.byref(n)))
        out = []
        for i in range(n.value):
            k, nu, ns, wg = _i32(), _i32(), _i32(), _i64()
            _check("fsdp_batch_launch_info", lib().fsdp_batch_launch_info(self._h, i, ctypes.byref(k), ctypes.byref(nu),
                                                                         ctypes.byref(ns), ctypes.byref(wg)))
            out.append({"kernel": lib().fsdp_kernel_name(k.value).decode(), "updates": nu.value, "unshards": ns.value,
                        "workgroups": wg.value})
        return out

    def close(self) -> None:
        if self._h is not None:
            lib().fsdp_batch_destroy(self._h)
            self._h = None
            self._keep = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
