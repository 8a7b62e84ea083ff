"""CPU oracle for the FlatParameter data path (arXiv 2304.11277).

TEST INFRASTRUCTURE ONLY.  Importers: tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg.  The product package never imports this, and this
package never imports the product.

All arithmetic lives in fsdp_oracle.c (plain C, one loop per definition).  This
file only builds that C file with gcc, loads it with ctypes and marshals numpy
arrays.  bf16 data is carried as numpy uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fsdp_oracle.c")
_LIB = os.path.join(_HERE, "libfsdp_oracle.so")

CFLAGS = ["-O2", "-std=gnu99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (about a second)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_bf16_rne.restype = ctypes.c_uint16
        _lib.orc_bf16_rne.argtypes = [ctypes.c_uint32]
        _lib.orc_num_threads.restype = ctypes.c_int
        _configure(_lib)
    return _lib


def _configure(l) -> None:
    """restype / argtypes of the functions that do not return int."""
    l.orc_bf16_rne.restype = ctypes.c_uint16
    l.orc_bf16_rne.argtypes = [ctypes.c_uint32]
    l.orc_f16_rne.restype = ctypes.c_uint16
    l.orc_f16_rne.argtypes = [ctypes.c_uint32]
    l.orc_unscale_check.restype = ctypes.c_float
    l.orc_found_inf_combine.restype = ctypes.c_float


_c_i64 = ctypes.c_int64
_c_i32 = ctypes.c_int32
_c_f32 = ctypes.c_float
_vp = ctypes.c_void_p


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32, a.dtype
    return a


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _ptr_array(arrs: Sequence[np.ndarray]):
    return (_vp * len(arrs))(*[_ptr(a) for a in arrs])


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    lib().orc_set_num_threads(ctypes.c_int(int(n)))


# ---------------------------------------------------------------- layout

def layout(shapes: Sequence[Sequence[int]], W: int):
    """Returns (off[p+1], N, S, P, pad).  Sec. 3.2.1."""
    p = len(shapes)
    flat_dims = [int(d) for s in shapes for d in s]
    dims = (_c_i64 * max(1, len(flat_dims)))(*flat_dims)
    ndims = (_c_i32 * max(1, p))(*[len(s) for s in shapes])
    off = (_c_i64 * (p + 1))()
    S, P, pad = _c_i64(), _c_i64(), _c_i64()
    rc = lib().orc_layout(dims, ndims, _c_i32(p), _c_i32(W), off,
                          ctypes.byref(S), ctypes.byref(P), ctypes.byref(pad))
    if rc != 0:
        raise ValueError("orc_layout: invalid argument")
    off = [int(x) for x in off]
    return off, off[-1], int(S.value), int(P.value), int(pad.value)


def flatten_pad(params: Sequence[np.ndarray], P: int) -> np.ndarray:
    """Concatenate the flattened (row-major) parameters and zero-pad to P."""
    ps = [_f32(np.asarray(a).reshape(-1)) for a in params]
    numel = (_c_i64 * len(ps))(*[a.size for a in ps])
    flat = np.empty(P, dtype=np.float32)
    lib().orc_flatten_pad(_ptr_array(ps), numel, _c_i32(len(ps)), _c_i64(P), _vp(_ptr(flat)))
    return flat


def chunk(flat: np.ndarray, S: int, w: int) -> np.ndarray:
    flat = _f32(flat)
    out = np.empty(S, dtype=np.float32)
    lib().orc_chunk(_vp(_ptr(flat)), _c_i64(S), _c_i32(w), _vp(_ptr(out)))
    return out


def flatten_shard(params: Sequence[np.ndarray], W: int) -> Tuple[List[np.ndarray], tuple]:
    """layout + flatten_pad + chunk for every rank."""
    off, N, S, P, pad = layout([tuple(np.asarray(a).shape) for a in params], W)
    flat = flatten_pad(params, P)
    return [chunk(flat, S, w) for w in range(W)], (off, N, S, P, pad)


# ------------------------------------------------------------------ cast

def bf16_rne_scalar(bits: int) -> int:
    return int(lib().orc_bf16_rne(ctypes.c_uint32(bits & 0xFFFFFFFF)))


def cast_bf16(x: np.ndarray) -> np.ndarray:
    shape = np.shape(x)
    x = _f32(x)
    y = np.empty(shape, dtype=np.uint16)
    lib().orc_cast_bf16(_vp(_ptr(x)), _c_i64(x.size), _vp(_ptr(y)))
    return y


def cast_bf16_bits(first: int, count: int) -> np.ndarray:
    y = np.empty(count, dtype=np.uint16)
    lib().orc_cast_bf16_bits(ctypes.c_uint32(first), _c_i64(count), _vp(_ptr(y)))
    return y


# --------------------------------------------------------------- unshard

def unshard_bf16(shards: Sequence[np.ndarray]) -> np.ndarray:
    sh = [_f32(s) for s in shards]
    S = sh[0].size
    assert all(s.size == S for s in sh)
    out = np.empty(S * len(sh), dtype=np.uint16)
    lib().orc_unshard_bf16(_ptr_array(sh), _c_i32(len(sh)), _c_i64(S), _vp(_ptr(out)))
    return out


def unshard_f32(shards: Sequence[np.ndarray]) -> np.ndarray:
    sh = [_f32(s) for s in shards]
    S = sh[0].size
    assert all(s.size == S for s in sh)
    out = np.empty(S * len(sh), dtype=np.float32)
    lib().orc_unshard_f32(_ptr_array(sh), _c_i32(len(sh)), _c_i64(S), _vp(_ptr(out)))
    return out


def gather_lp(lp_shards: Sequence[np.ndarray]) -> np.ndarray:
    """AllGather of the ranks' bf16 shards (uint16 bit patterns) into the flat buffer."""
    sh = [_u16(s) for s in lp_shards]
    S = sh[0].size
    assert all(s.size == S for s in sh)
    out = np.empty(S * len(sh), dtype=np.uint16)
    lib().orc_gather_lp(_ptr_array(sh), _c_i32(len(sh)), _c_i64(S), _vp(_ptr(out)))
    return out


def views(flat: np.ndarray, off: Sequence[int], shapes: Sequence[Sequence[int]]) -> List[np.ndarray]:
    """Per-parameter views into the unsharded flat buffer (Sec. 3.2.3): zero
    copy, view_i = flat[off_i : off_i + n_i] reshaped."""
    return [flat[off[i]:off[i + 1]].reshape(tuple(shapes[i])) for i in range(len(shapes))]


# -------------------------------------------------------- reduce-scatter

def _is_bf16(arrs) -> bool:
    dt = arrs[0].dtype
    assert all(a.dtype == dt for a in arrs)
    if dt == np.uint16:
        return True
    assert dt == np.float32, dt
    return False


def reduce_slices(slices: Sequence[np.ndarray], pre: float, post: float) -> np.ndarray:
    """slices[w] = rank w's gradient elements [r*S, (r+1)*S)."""
    sl = [np.ascontiguousarray(s) for s in slices]
    S = sl[0].size
    assert all(s.size == S for s in sl)
    out = np.empty(S, dtype=np.float32)
    fn = lib().orc_reduce_slices_bf16 if _is_bf16(sl) else lib().orc_reduce_slices_f32
    fn(_ptr_array(sl), _c_i32(len(sl)), _c_i64(S), _c_f32(pre), _c_f32(post), _vp(_ptr(out)))
    return out


def reduce_scatter(gradbufs: Sequence[np.ndarray], r: int, pre: float, post: float) -> np.ndarray:
    """gradbufs[w] = rank w's whole unsharded gradient buffer (P elements)."""
    gb = [np.ascontiguousarray(g) for g in gradbufs]
    W = len(gb)
    P = gb[0].size
    assert all(g.size == P for g in gb) and P % W == 0 and 0 <= r < W
    S = P // W
    out = np.empty(S, dtype=np.float32)
    fn = lib().orc_reduce_scatter_bf16 if _is_bf16(gb) else lib().orc_reduce_scatter_f32
    fn(_ptr_array(gb), _c_i32(W), _c_i64(S), _c_i32(r), _c_f32(pre), _c_f32(post), _vp(_ptr(out)))
    return out


def reduce_full_f32(gradbufs: Sequence[np.ndarray], pre: float, post: float) -> np.ndarray:
    gb = [_f32(g) for g in gradbufs]
    P = gb[0].size
    out = np.empty(P, dtype=np.float32)
    lib().orc_reduce_full_f32(_ptr_array(gb), _c_i32(len(gb)), _c_i64(P), _c_f32(pre), _c_f32(post),
                              _vp(_ptr(out)))
    return out


def reduce_slices_hybrid(slices: Sequence[np.ndarray], G: int, F: int, pre: float, post: float) -> np.ndarray:
    """Two-level reduction of Sec. 3.2.2: slices[i*F + l] = slice of local rank
    l in sharded group i; inner sums per group, outer sum over the groups."""
    sl = [np.ascontiguousarray(s) for s in slices]
    assert len(sl) == G * F
    S = sl[0].size
    assert all(s.size == S for s in sl)
    out = np.empty(S, dtype=np.float32)
    fn = lib().orc_reduce_slices_hybrid_bf16 if _is_bf16(sl) else lib().orc_reduce_slices_hybrid_f32
    fn(_ptr_array(sl), _c_i32(G), _c_i32(F), _c_i64(S), _c_f32(pre), _c_f32(post), _vp(_ptr(out)))
    return out


def accumulate(acc: np.ndarray, add: np.ndarray) -> np.ndarray:
    """Gradient accumulation (Sec. 3.3.4): returns acc + add in binary32;
    add may be float32 or bf16 bit patterns (uint16)."""
    acc = _f32(acc).copy()
    add = np.ascontiguousarray(add)
    assert add.size == acc.size
    if add.dtype == np.uint16:
        lib().orc_accumulate_bf16(_vp(_ptr(acc)), _vp(_ptr(add)), _c_i64(acc.size))
    else:
        assert add.dtype == np.float32
        lib().orc_accumulate_f32(_vp(_ptr(acc)), _vp(_ptr(add)), _c_i64(acc.size))
    return acc


# ------------------------------------------------- fp16 and gradient scaler

def f16_rne_scalar(bits: int) -> int:
    return int(lib().orc_f16_rne(ctypes.c_uint32(bits & 0xFFFFFFFF)))


def cast_f16(x: np.ndarray) -> np.ndarray:
    shape = np.shape(x)
    x = _f32(x)
    y = np.empty(shape, dtype=np.uint16)
    lib().orc_cast_f16(_vp(_ptr(x)), _c_i64(x.size), _vp(_ptr(y)))
    return y


def cast_f16_bits(first: int, count: int) -> np.ndarray:
    y = np.empty(count, dtype=np.uint16)
    lib().orc_cast_f16_bits(ctypes.c_uint32(first), _c_i64(count), _vp(_ptr(y)))
    return y


def upcast_f16(h: np.ndarray) -> np.ndarray:
    h = _u16(h)
    y = np.empty(h.shape, dtype=np.float32)
    lib().orc_upcast_f16(_vp(_ptr(h)), _c_i64(h.size), _vp(_ptr(y)))
    return y


def unshard_f16(shards: Sequence[np.ndarray]) -> np.ndarray:
    sh = [_f32(s) for s in shards]
    S = sh[0].size
    out = np.empty(S * len(sh), dtype=np.uint16)
    lib().orc_unshard_f16(_ptr_array(sh), _c_i32(len(sh)), _c_i64(S), _vp(_ptr(out)))
    return out


def reduce_slices_f16(slices: Sequence[np.ndarray], pre: float, post: float) -> np.ndarray:
    """slices hold binary16 bit patterns (uint16)."""
    sl = [_u16(s) for s in slices]
    S = sl[0].size
    out = np.empty(S, dtype=np.float32)
    lib().orc_reduce_slices_f16(_ptr_array(sl), _c_i32(len(sl)), _c_i64(S), _c_f32(pre), _c_f32(post), _vp(_ptr(out)))
    return out


def unscale_check(g: np.ndarray, inv_scale: float):
    """Returns (g * inv_scale, found_inf of this shard)."""
    g = _f32(g).copy()
    found = lib().orc_unscale_check(_vp(_ptr(g)), _c_i64(g.size), _c_f32(inv_scale))
    return g, float(found)


def found_inf_combine(flags: Sequence[float]) -> float:
    a = np.asarray(flags, dtype=np.float32)
    return float(lib().orc_found_inf_combine(_vp(_ptr(a)), _c_i32(a.size)))


def scaler_update(scale: float, growth_tracker: int, found_inf: float, growth: float = 2.0, backoff: float = 0.5,
                  growth_interval: int = 2000):
    s = _c_f32(scale)
    t = _c_i32(growth_tracker)
    lib().orc_scaler_update(ctypes.byref(s), ctypes.byref(t), _c_f32(found_inf), _c_f32(growth), _c_f32(backoff),
                            _c_i32(growth_interval))
    return float(s.value), int(t.value)


# ------------------------------------------------------------------ Adam

def adam_f32(p, g, m, v, t: int, lr: float, beta1: float, beta2: float, eps: float):
    """Returns new (p, m, v); inputs are not modified."""
    p, m, v = _f32(p).copy(), _f32(m).copy(), _f32(v).copy()
    g = _f32(g)
    S = p.size
    assert g.size == S and m.size == S and v.size == S and t >= 1
    lib().orc_adam_f32(_vp(_ptr(p)), _vp(_ptr(g)), _vp(_ptr(m)), _vp(_ptr(v)), _c_i64(S), _c_i64(t),
                       _c_f32(lr), _c_f32(beta1), _c_f32(beta2), _c_f32(eps))
    return p, m, v


def adam_f64(p, g, m, v, t: int, lr: float, beta1: float, beta2: float, eps: float):
    p, g, m, v = _f32(p), _f32(g), _f32(m), _f32(v)
    S = p.size
    po, mo, vo = (np.empty(S, dtype=np.float64) for _ in range(3))
    lib().orc_adam_f64(_vp(_ptr(p)), _vp(_ptr(g)), _vp(_ptr(m)), _vp(_ptr(v)), _c_i64(S), _c_i64(t),
                       _c_f32(lr), _c_f32(beta1), _c_f32(beta2), _c_f32(eps),
                       _vp(_ptr(po)), _vp(_ptr(mo)), _vp(_ptr(vo)))
    return po, mo, vo
