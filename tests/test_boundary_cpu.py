"""Host-side tests of the C ABI: the library loads, exports every symbol the
header declares, plans layouts like the oracle does, and turns every invalid
argument into an error code before anything is launched.  No GPU needed."""
import ctypes
import os
import re

import pytest

import oracle
import workloads
from paper_2304_11277_amd import build as fbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    fbuild.build_lib(force=False)
    import paper_2304_11277_amd as f
    return f


def test_header_symbols_are_exported(L):
    hdr = open(os.path.join(ROOT, "include", "fsdp_flat.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(fsdp_[a-z_0-9]+)\s*\(", hdr))
    assert {"fsdp_layout_init", "fsdp_flatten_shard", "fsdp_unshard", "fsdp_reduce_scatter_local",
            "fsdp_shard_adam_step"} <= names
    raw = ctypes.CDLL(L.library_path())
    for n in sorted(names):
        assert hasattr(raw, n), n


def test_binding_names_match_c_names(L):
    for n in ("fsdp_layout_init", "fsdp_flatten_shard", "fsdp_unshard", "fsdp_reduce_scatter_local",
              "fsdp_shard_adam_step", "fsdp_reduce_scatter_adam_fused", "fsdp_view_ptr",
              "fsdp_default_divide_factors"):
        assert callable(getattr(L, n))


def test_layout_matches_oracle_on_configs_and_ragged(L):
    cases = [(workloads.config(i).units[j].shapes, workloads.config(i).world_size)
             for i in range(workloads.NUM_CONFIGS) for j in workloads.config(i).distinct_units]
    cases += [(workloads.ragged_unit().shapes, W) for W in (1, 2, 3, 7, 8, 12, 64, 100)]
    cases += [(((3, 4), (3,)), 16)]
    for shapes, W in cases:
        lay = L.fsdp_layout_init(shapes, W)
        off, N, S, P, pad = oracle.layout(shapes, W)
        assert (lay.numel, lay.shard, lay.padded, lay.pad) == (N, S, P, pad)
        assert lay.offsets == off[:-1]
        assert lay.numels == [off[i + 1] - off[i] for i in range(len(shapes))]
        assert (lay.num_params, lay.world_size) == (len(shapes), W)
        lay.close()


def test_fig3_worked_example_through_the_abi(L):
    lay = L.fsdp_layout_init([(3, 4), (3,)], 16)
    assert (lay.numel, lay.shard, lay.padded, lay.pad) == (15, 1, 16, 1)


def test_default_divide_factors(L):
    expect = {1: (1, 1), 2: (2, 1), 3: (1, 3), 6: (2, 3), 8: (4, 2), 12: (4, 3), 16: (4, 4), 64: (8, 8),
              128: (16, 8), 7: (1, 7)}
    for W, (pre, post) in expect.items():
        assert L.fsdp_default_divide_factors(W) == (float(pre), float(post))
        assert pre * post == W


# ---- error codes, straight through ctypes -------------------------------

OK, INVALID, NULL, OVERFLOW, OOM, BAD_DTYPE, RANK_RANGE, HIP = 0, -1, -2, -3, -4, -5, -6, -7


def _init(raw, shapes, W):
    flat = [d for s in shapes for d in s]
    dims = (ctypes.c_int64 * max(1, len(flat)))(*flat)
    nd = (ctypes.c_int32 * max(1, len(shapes)))(*[len(s) for s in shapes])
    out = ctypes.c_void_p()
    rc = raw.fsdp_layout_init(dims, nd, len(shapes), W, ctypes.byref(out))
    return rc, out


def test_layout_init_errors(L):
    raw = L.lib()
    assert _init(raw, [(2, 3)], 0)[0] == INVALID
    assert _init(raw, [(2, 3)], -4)[0] == INVALID
    assert _init(raw, [], 4)[0] == INVALID
    assert _init(raw, [(2, -3)], 4)[0] == INVALID
    assert _init(raw, [(0, 5), (0,)], 4)[0] == INVALID            # N == 0
    assert _init(raw, [(2 ** 40, 2 ** 40)], 4)[0] == OVERFLOW     # numel past int64
    assert _init(raw, [(2 ** 62,), (2 ** 62,)], 4)[0] == OVERFLOW  # sum past int64
    assert _init(raw, [(2 ** 61,)], 4)[0] == OVERFLOW             # 4 * P past int64
    assert _init(raw, [(0, 2 ** 62, 2 ** 62), (3,)], 4)[0] == OK  # a zero dim is numel 0, not an overflow
    nd = (ctypes.c_int32 * 1)(1)
    out = ctypes.c_void_p()
    assert raw.fsdp_layout_init(None, nd, 1, 2, ctypes.byref(out)) == NULL
    dims = (ctypes.c_int64 * 1)(5)
    assert raw.fsdp_layout_init(dims, None, 1, 2, ctypes.byref(out)) == NULL
    assert raw.fsdp_layout_init(dims, nd, 1, 2, None) == NULL
    nd[0] = -1
    assert raw.fsdp_layout_init(dims, nd, 1, 2, ctypes.byref(out)) == INVALID
    raw.fsdp_layout_destroy(None)                                   # no-op


def test_query_errors(L):
    raw = L.lib()
    rc, h = _init(raw, [(4, 3), (3,)], 4)
    assert rc == OK
    n = ctypes.c_int64()
    assert raw.fsdp_layout_info(None, None, None, None, None, None, None) == NULL
    assert raw.fsdp_layout_info(h, ctypes.byref(n), None, None, None, None, None) == OK and n.value == 15
    assert raw.fsdp_layout_param(h, 2, None, None) == RANK_RANGE
    assert raw.fsdp_layout_param(h, -1, None, None) == RANK_RANGE
    assert raw.fsdp_layout_param(None, 0, None, None) == NULL
    out = ctypes.c_void_p()
    base = ctypes.c_void_p(0x1000)
    assert raw.fsdp_view_ptr(h, base, 1, 1, ctypes.byref(out)) == OK and out.value == 0x1000 + 12 * 2
    assert raw.fsdp_view_ptr(h, base, 0, 1, ctypes.byref(out)) == OK and out.value == 0x1000 + 12 * 4
    assert raw.fsdp_view_ptr(h, base, 2, 1, ctypes.byref(out)) == OK and out.value == 0x1000 + 12 * 2
    assert raw.fsdp_view_ptr(h, base, 3, 1, ctypes.byref(out)) == BAD_DTYPE
    assert raw.fsdp_view_ptr(h, base, 0, 5, ctypes.byref(out)) == RANK_RANGE
    assert raw.fsdp_view_ptr(h, None, 0, 0, ctypes.byref(out)) == NULL
    assert raw.fsdp_view_ptr(h, base, 0, 0, None) == NULL
    pre, post = ctypes.c_float(), ctypes.c_float()
    assert raw.fsdp_default_divide_factors(0, ctypes.byref(pre), ctypes.byref(post)) == INVALID
    assert raw.fsdp_default_divide_factors(8, None, ctypes.byref(post)) == NULL
    raw.fsdp_layout_destroy(h)


def _table(vals):
    return (ctypes.c_void_p * len(vals))(*vals)


def test_compute_entry_points_reject_bad_arguments_before_launch(L):
    """Fake (never dereferenced) device addresses: every call must fail in host
    validation, so nothing reaches a device."""
    raw = L.lib()
    rc, h = _init(raw, [(4, 3), (3,)], 4)
    assert rc == OK
    good4 = _table([0x10000 + 64 * i for i in range(4)])
    good2 = _table([0x20000, 0x20100])
    with_null = _table([0x10000, None, 0x10080, 0x100C0])
    odd = _table([0x10000, 0x10042, 0x10080, 0x100C0])   # 2-byte aligned only
    buf = ctypes.c_void_p(0x30000)
    st = None
    # flatten
    assert raw.fsdp_flatten_shard(None, good2, good4, st) == NULL
    assert raw.fsdp_flatten_shard(h, None, good4, st) == NULL
    assert raw.fsdp_flatten_shard(h, good2, None, st) == NULL
    assert raw.fsdp_flatten_shard(h, _table([0x20000, None]), good4, st) == NULL
    assert raw.fsdp_flatten_shard(h, good2, with_null, st) == NULL
    assert raw.fsdp_flatten_shard(h, _table([0x20002, 0x20100]), good4, st) == INVALID
    assert raw.fsdp_flatten_shard(h, good2, odd, st) == INVALID
    # unshard
    assert raw.fsdp_unshard(None, good4, buf, 1, st) == NULL
    assert raw.fsdp_unshard(h, None, buf, 1, st) == NULL
    assert raw.fsdp_unshard(h, good4, None, 1, st) == NULL
    assert raw.fsdp_unshard(h, with_null, buf, 1, st) == NULL
    assert raw.fsdp_unshard(h, good4, buf, 3, st) == BAD_DTYPE
    assert raw.fsdp_unshard(h, good4, buf, -1, st) == BAD_DTYPE
    assert raw.fsdp_unshard(h, odd, buf, 1, st) == INVALID
    assert raw.fsdp_unshard(h, good4, ctypes.c_void_p(0x30001), 1, st) == INVALID
    assert raw.fsdp_unshard(h, good4, ctypes.c_void_p(0x30002), 0, st) == INVALID
    # reduce-scatter
    f = ctypes.c_float
    assert raw.fsdp_reduce_scatter_local(None, good4, 0, 0, f(2), f(2), buf, st) == NULL
    assert raw.fsdp_reduce_scatter_local(h, None, 0, 0, f(2), f(2), buf, st) == NULL
    assert raw.fsdp_reduce_scatter_local(h, good4, 0, 0, f(2), f(2), None, st) == NULL
    assert raw.fsdp_reduce_scatter_local(h, with_null, 0, 0, f(2), f(2), buf, st) == NULL
    assert raw.fsdp_reduce_scatter_local(h, good4, 7, 0, f(2), f(2), buf, st) == BAD_DTYPE
    assert raw.fsdp_reduce_scatter_local(h, good4, 0, 4, f(2), f(2), buf, st) == RANK_RANGE
    assert raw.fsdp_reduce_scatter_local(h, good4, 0, -1, f(2), f(2), buf, st) == RANK_RANGE
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        assert raw.fsdp_reduce_scatter_local(h, good4, 0, 0, f(bad), f(2), buf, st) == INVALID
        assert raw.fsdp_reduce_scatter_local(h, good4, 0, 0, f(2), f(bad), buf, st) == INVALID
    assert raw.fsdp_reduce_scatter_local(h, odd, 0, 0, f(2), f(2), buf, st) == INVALID     # fp32 needs 4 B
    assert raw.fsdp_reduce_scatter_local(h, _table([0x10001, 0x10040, 0x10080, 0x100C0]), 1, 0, f(2), f(2), buf,
                                         st) == INVALID
    # adam
    p, g, m, v = (ctypes.c_void_p(0x40000 + 0x100 * i) for i in range(4))
    i64 = ctypes.c_int64
    ok_h = (f(1e-4), f(0.9), f(0.999), f(1e-8))
    assert raw.fsdp_shard_adam_step(None, p, g, m, v, i64(1), *ok_h, st) == NULL
    for k in range(4):
        a = [p, g, m, v]
        a[k] = None
        assert raw.fsdp_shard_adam_step(h, *a, i64(1), *ok_h, st) == NULL
    assert raw.fsdp_shard_adam_step(h, p, g, m, v, i64(0), *ok_h, st) == INVALID
    assert raw.fsdp_shard_adam_step(h, p, g, m, v, i64(1), f(float("nan")), f(0.9), f(0.999), f(1e-8), st) == INVALID
    assert raw.fsdp_shard_adam_step(h, p, g, m, v, i64(1), f(1e-4), f(1.0), f(0.999), f(1e-8), st) == INVALID
    assert raw.fsdp_shard_adam_step(h, p, g, m, v, i64(1), f(1e-4), f(0.9), f(-0.1), f(1e-8), st) == INVALID
    assert raw.fsdp_shard_adam_step(h, p, g, m, v, i64(1), f(1e-4), f(0.9), f(0.999), f(-1e-8), st) == INVALID
    assert raw.fsdp_shard_adam_step(h, ctypes.c_void_p(0x40002), g, m, v, i64(1), *ok_h, st) == INVALID
    # fused
    assert raw.fsdp_reduce_scatter_adam_fused(h, good4, 0, 9, f(2), f(2), None, p, m, v, i64(1), *ok_h, None,
                                              st) == RANK_RANGE
    assert raw.fsdp_reduce_scatter_adam_fused(h, good4, 0, 0, f(2), f(2), None, None, m, v, i64(1), *ok_h, None,
                                              st) == NULL
    assert raw.fsdp_reduce_scatter_adam_fused(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(0), *ok_h, None,
                                              st) == INVALID
    assert raw.fsdp_reduce_scatter_adam_fused(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(1), *ok_h,
                                              ctypes.c_void_p(0x50001), st) == INVALID
    # one-launch prefetch form: both halves are validated before anything is launched
    rc, hn = _init(raw, [(64,)], 4)
    assert rc == OK
    pf = raw.fsdp_reduce_scatter_adam_prefetch_unshard
    assert pf(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(1), *ok_h, None, None, good4, buf, 1, st) == NULL
    assert pf(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(1), *ok_h, None, hn, None, buf, 1, st) == NULL
    assert pf(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(1), *ok_h, None, hn, good4, None, 1, st) == NULL
    assert pf(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(1), *ok_h, None, hn, with_null, buf, 1, st) == NULL
    assert pf(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(1), *ok_h, None, hn, good4, buf, 4, st) == BAD_DTYPE
    assert pf(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(1), *ok_h, None, hn, odd, buf, 1, st) == INVALID
    assert pf(h, good4, 0, 4, f(2), f(2), None, p, m, v, i64(1), *ok_h, None, hn, good4, buf, 1, st) == RANK_RANGE
    assert pf(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(0), *ok_h, None, hn, good4, buf, 1, st) == INVALID
    raw.fsdp_layout_destroy(hn)
    # hybrid sharding and gradient accumulation
    good8 = _table([0x10000 + 64 * i for i in range(8)])
    hy = raw.fsdp_reduce_scatter_hybrid
    assert hy(h, good8, 0, 2, 0, f(2), f(4), None, st) == NULL
    assert hy(h, None, 0, 2, 0, f(2), f(4), buf, st) == NULL
    assert hy(h, good8, 0, 0, 0, f(2), f(4), buf, st) == INVALID
    assert hy(h, good8, 0, 2, 4, f(2), f(4), buf, st) == RANK_RANGE
    assert hy(h, good8, 5, 2, 0, f(2), f(4), buf, st) == BAD_DTYPE
    assert hy(h, _table([0x10000 + 64 * i for i in range(7)] + [None]), 0, 2, 0, f(2), f(4), buf, st) == NULL
    many68 = _table([0x10000 + 64 * i for i in range(68)])
    # more ranks than one launch takes are split between sharded groups; a group larger than a launch cannot be
    rc65, h65 = _init(raw, [(4, 3), (3,)], 65)
    assert rc65 == OK
    many130 = _table([0x10000 + 64 * i for i in range(130)])
    assert hy(h65, many130, 0, 2, 0, f(2), f(65), buf, st) == INVALID        # sharded groups of 65 ranks
    assert raw.fsdp_reduce_scatter_accumulate(h65, many130, 0, 0, f(5), f(13), buf, st) == INVALID   # 65 ranks, one launch only
    raw.fsdp_layout_destroy(h65)
    hf = raw.fsdp_reduce_scatter_hybrid_adam_fused
    assert hf(h, good8, 0, 2, 0, f(2), f(4), None, None, m, v, i64(1), *ok_h, None, st) == NULL
    assert hf(h, None, 0, 2, 0, f(2), f(4), None, p, m, v, i64(1), *ok_h, None, st) == NULL
    assert hf(h, good8, 0, 0, 0, f(2), f(4), None, p, m, v, i64(1), *ok_h, None, st) == INVALID
    assert hf(h, good8, 0, 2, 4, f(2), f(4), None, p, m, v, i64(1), *ok_h, None, st) == RANK_RANGE
    assert hf(h, good8, 0, 2, 0, f(2), f(4), None, p, m, v, i64(0), *ok_h, None, st) == INVALID
    assert hf(h, good8, 9, 2, 0, f(2), f(4), None, p, m, v, i64(1), *ok_h, None, st) == BAD_DTYPE
    assert hf(h, many68, 0, 17, 0, f(2), f(34), None, p, m, v, i64(1), *ok_h, None, st) == NULL   # 68 ranks: the shard carries the sum
    ra = raw.fsdp_reduce_scatter_accumulate
    assert ra(h, good4, 0, 0, f(2), f(2), None, st) == NULL
    assert ra(h, good4, 0, 9, f(2), f(2), buf, st) == RANK_RANGE
    assert ra(h, good4, 0, 0, f(0), f(2), buf, st) == INVALID
    raf = raw.fsdp_reduce_scatter_accumulate_adam_fused
    assert raf(h, good4, 0, 0, f(2), f(2), None, p, m, v, i64(1), *ok_h, None, st) == NULL     # the accumulator is required
    assert raf(h, good4, 0, 0, f(2), f(2), buf, p, None, v, i64(1), *ok_h, None, st) == NULL
    assert raf(h, good4, 0, 4, f(2), f(2), buf, p, m, v, i64(1), *ok_h, None, st) == RANK_RANGE
    assert raf(h, good4, 0, 0, f(2), f(2), buf, p, m, v, i64(0), *ok_h, None, st) == INVALID
    assert raf(h, good4, 0, 0, f(2), f(2), buf, p, m, v, i64(1), f(1e-4), f(1.0), f(0.999), f(1e-8), None, st) == INVALID
    assert raw.fsdp_cast_shard(None, buf, buf, 1, st) == NULL
    assert raw.fsdp_cast_shard(h, None, buf, 1, st) == NULL
    assert raw.fsdp_cast_shard(h, buf, None, 2, st) == NULL
    assert raw.fsdp_cast_shard(h, buf, buf, 0, st) == BAD_DTYPE
    assert raw.fsdp_cast_shard(h, buf, buf, 3, st) == BAD_DTYPE
    assert raw.fsdp_cast_shard(h, ctypes.c_void_p(0x30002), buf, 1, st) == INVALID
    assert raw.fsdp_cast_shard(h, buf, ctypes.c_void_p(0x30001), 2, st) == INVALID
    # gradient scaler
    flag = ctypes.c_void_p(0x60000)
    us = raw.fsdp_reduce_scatter_unscale
    assert us(h, good4, 2, 0, f(2), f(2), f(0.5), buf, None, st) == NULL
    assert us(h, good4, 2, 0, f(2), f(2), f(0.5), None, flag, st) == NULL
    assert us(h, good4, 2, 0, f(2), f(2), f(0.0), buf, flag, st) == INVALID
    assert us(h, good4, 2, 0, f(2), f(2), f(float("inf")), buf, flag, st) == INVALID
    assert us(h, good4, 3, 0, f(2), f(2), f(0.5), buf, flag, st) == BAD_DTYPE
    assert us(h, good4, 2, 0, f(2), f(2), f(0.5), buf, ctypes.c_void_p(0x60002), st) == INVALID
    assert raw.fsdp_found_inf_combine(None, 4, st) == NULL
    assert raw.fsdp_found_inf_combine(good4, 0, st) == INVALID
    assert raw.fsdp_found_inf_combine(_table([0x10000 + 64 * i for i in range(66)] + [None, 0x20000]), 68, st) == NULL
    assert raw.fsdp_found_inf_combine(_table([0x10000 + 64 * i for i in range(66)] + [0x20002]), 67, st) == INVALID
    assert raw.fsdp_found_inf_combine(many68, -1, st) == INVALID
    assert raw.fsdp_found_inf_combine(with_null, 4, st) == NULL
    assert raw.fsdp_shard_adam_step_guarded(h, p, g, m, v, i64(1), *ok_h, None, st) == NULL
    assert raw.fsdp_shard_adam_step_guarded(h, p, g, m, v, i64(0), *ok_h, flag, st) == INVALID
    gsu = raw.fsdp_grad_scaler_update
    i32p = ctypes.c_void_p(0x61000)
    assert gsu(None, i32p, flag, f(2), f(0.5), 2000, st) == NULL
    assert gsu(flag, None, flag, f(2), f(0.5), 2000, st) == NULL
    assert gsu(flag, i32p, None, f(2), f(0.5), 2000, st) == NULL
    assert gsu(flag, i32p, flag, f(1.0), f(0.5), 2000, st) == INVALID
    assert gsu(flag, i32p, flag, f(2.0), f(1.0), 2000, st) == INVALID
    assert gsu(flag, i32p, flag, f(2.0), f(0.5), 0, st) == INVALID
    assert raw.fsdp_unshard_lp(None, good4, buf, st) == NULL
    assert raw.fsdp_unshard_lp(h, None, buf, st) == NULL
    assert raw.fsdp_unshard_lp(h, good4, None, st) == NULL
    assert raw.fsdp_unshard_lp(h, with_null, buf, st) == NULL
    assert raw.fsdp_unshard_lp(h, _table([0x10000, 0x10041, 0x10080, 0x100C0]), buf, st) == INVALID
    # batches
    bh = ctypes.c_void_p()
    assert raw.fsdp_batch_create(None) == NULL
    assert raw.fsdp_batch_create(ctypes.byref(bh)) == OK
    assert raw.fsdp_batch_clear(None) == NULL
    assert raw.fsdp_batch_add_unshard(None, h, good4, buf, 1) == NULL
    assert raw.fsdp_batch_add_unshard(bh, None, good4, buf, 1) == NULL
    assert raw.fsdp_batch_add_unshard(bh, h, with_null, buf, 1) == NULL
    assert raw.fsdp_batch_add_unshard(bh, h, good4, buf, 7) == BAD_DTYPE
    assert raw.fsdp_batch_add_unshard(bh, h, odd, buf, 1) == INVALID
    add_r = raw.fsdp_batch_add_reduce_scatter_adam
    assert add_r(bh, h, good4, 0, 9, f(2), f(2), None, p, m, v, *ok_h, None) == RANK_RANGE
    assert add_r(bh, h, good4, 0, 0, f(2), f(2), None, None, m, v, *ok_h, None) == NULL
    assert add_r(bh, h, good4, 0, 0, f(0), f(2), None, p, m, v, *ok_h, None) == INVALID
    assert add_r(bh, h, good4, 0, 0, f(2), f(2), None, p, m, v, f(1e-4), f(1.5), f(0.999), f(1e-8), None) == INVALID
    assert raw.fsdp_batch_launch(None, i64(1), st) == NULL
    assert raw.fsdp_batch_launch(bh, i64(0), st) == INVALID
    assert raw.fsdp_batch_launch(bh, i64(1), st) == OK          # an empty batch launches nothing
    raw.fsdp_batch_destroy(bh)
    raw.fsdp_batch_destroy(None)
    ga = raw.fsdp_grad_accumulate
    assert ga(None, buf, buf, 0, st) == NULL
    assert ga(h, None, buf, 0, st) == NULL
    assert ga(h, buf, None, 0, st) == NULL
    assert ga(h, buf, buf, 3, st) == BAD_DTYPE
    assert ga(h, ctypes.c_void_p(0x30002), buf, 0, st) == INVALID
    assert ga(h, buf, ctypes.c_void_p(0x30001), 1, st) == INVALID
    raw.fsdp_layout_destroy(h)
    # W > 64 needs the gradient shard buffer to carry partial sums
    rc, h2 = _init(raw, [(1000,)], 65)
    assert rc == OK
    many = _table([0x10000 + 64 * i for i in range(65)])
    assert raw.fsdp_reduce_scatter_adam_fused(h2, many, 0, 0, f(1), f(65), None, p, m, v, i64(1), *ok_h, None,
                                              st) == NULL
    raw.fsdp_layout_destroy(h2)


def test_binding_rejects_host_tensors(L):
    import torch
    lay = L.fsdp_layout_init([(4, 3), (3,)], 4)
    cpu = [torch.zeros(4) for _ in range(4)]
    with pytest.raises(TypeError):
        L.fsdp_unshard(lay, cpu, torch.zeros(16, dtype=torch.bfloat16))
    assert L.lib().fsdp_status_string(-6) == b"rank or parameter index out of range"


def test_layout_init_ex_takes_only_the_rank_walks_it_knows(L):
    for walk in (L.FSDP_WALK_AUTO, L.FSDP_WALK_WIDE, L.FSDP_WALK_DEEP, L.FSDP_WALK_HALF):
        lay = L.fsdp_layout_init([(4, 3), (3,)], 16, reduce_walk=walk)
        assert (lay.numel, lay.shard, lay.padded, lay.pad) == (15, 1, 16, 1)
    for bad in (-1, 4, 99):
        with pytest.raises(L.FsdpError) as e:
            L.fsdp_layout_init([(4, 3)], 2, reduce_walk=bad)
        assert e.value.status == INVALID


def test_library_exports_no_process_wide_setter(L):
    """The library keeps no process-wide tuning state: the rank walk is an option of each layout."""
    with pytest.raises(AttributeError):
        L.lib().fsdp_set_reduce_walk


def test_pointer_tables_are_checked_before_any_launch(L):
    """A table built ahead of time is held to the same checks as a list of
    tensors: device, one dtype, contiguity at construction; the count, the
    dtype the call expects and the sizes its layout needs at every call."""
    import torch
    with pytest.raises(TypeError):
        L.PtrArray([torch.zeros(8)])                                     # host memory
    with pytest.raises(TypeError):
        L.PtrArray([1.0, 2.0])
    # the remaining checks, on host tensors that stand in for device ones (such a table can never be launched)
    def tab(ts, **kw):
        return L.PtrArray(ts, _device_check=False, **kw)
    with pytest.raises(TypeError):
        tab([torch.zeros(8), torch.zeros(8, dtype=torch.bfloat16)])      # mixed dtypes
    with pytest.raises(ValueError):
        tab([torch.zeros(4, 4).t()])                                     # not contiguous
    lay = L.fsdp_layout_init([(4, 3), (3,)], 4)                          # N 15, S 4, P 16
    flat = torch.zeros(16, dtype=torch.bfloat16)
    good = tab([torch.zeros(4) for _ in range(4)])
    assert good.dtype == torch.float32 and good.numels == [4, 4, 4, 4] and not good.device_checked
    from paper_2304_11277_amd import binding
    with pytest.raises(TypeError, match="device check"):
        binding._ptr_table(good, torch.float32, lay.shard, 4, "shard_ptrs")
    good.device_checked = True                                           # look at the checks behind that one
    assert binding._ptr_table(good, torch.float32, lay.shard, 4, "shard_ptrs") is good
    with pytest.raises(ValueError, match="expected 4 entries"):
        binding._ptr_table(tab([torch.zeros(4)] * 3), torch.float32, lay.shard, 4, "shard_ptrs")
    short = tab([torch.zeros(4), torch.zeros(3), torch.zeros(4), torch.zeros(4)])
    short.device_checked = True
    with pytest.raises(ValueError, match=r"shard_ptrs\[1\]: needs at least 4"):
        binding._ptr_table(short, torch.float32, lay.shard, 4, "shard_ptrs")
    wrong = tab([torch.zeros(4, dtype=torch.float16)] * 4)
    wrong.device_checked = True
    with pytest.raises(TypeError, match="expected torch.float32"):
        binding._ptr_table(wrong, torch.float32, lay.shard, 4, "shard_ptrs")
    # gradient tables: the dtype comes from the table, the size must cover the padded flat buffer
    g_short = tab([torch.zeros(15)] * 4)
    g_short.device_checked = True
    with pytest.raises(ValueError, match="needs at least 16"):
        binding._grad_table(lay, g_short)
    g_int = tab([torch.zeros(16, dtype=torch.int32)] * 4)
    g_int.device_checked = True
    with pytest.raises(TypeError, match="not supported"):
        binding._grad_table(lay, g_int)
    # through a public entry point: the unchecked table is refused before the library is called
    with pytest.raises(TypeError):
        L.fsdp_unshard(lay, good.__class__([torch.zeros(4) for _ in range(4)], _device_check=False), flat)


def _plan(raw, b):
    n = ctypes.c_int32()
    assert raw.fsdp_batch_launch_count(b, ctypes.byref(n)) == OK
    out = []
    for i in range(n.value):
        k, nu, ns, wg = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int64()
        assert raw.fsdp_batch_launch_info(b, i, ctypes.byref(k), ctypes.byref(nu), ctypes.byref(ns), ctypes.byref(wg)) == OK
        out.append((raw.fsdp_kernel_name(k.value).decode(), nu.value, ns.value, wg.value))
    assert raw.fsdp_batch_launch_info(b, n.value, None, None, None, None) == -6
    return out


def test_batches_are_planned_while_they_are_recorded(L):
    """The grouping rules of fsdp_batch_*, read back through
    fsdp_batch_launch_count / _info with fake device addresses (nothing is
    launched): which operations share a grid and which kernel each launch is."""
    raw = L.lib()
    f, i64 = ctypes.c_float, ctypes.c_int64
    hyper = (f(1e-4), f(0.9), f(0.999), f(1e-8))
    addr = [0x100000]

    def table(n):
        vals = [addr[0] + 0x1000 * j for j in range(n)]
        addr[0] += 0x1000 * n
        return _table(vals)

    def add_update(b, h, W, dt=0, rank=0):
        p, m, v, g = (ctypes.c_void_p(addr[0] + 0x100 * j) for j in range(4))
        addr[0] += 0x1000
        return raw.fsdp_batch_add_reduce_scatter_adam(b, h, table(W), dt, rank, f(4.0), f(W / 4.0), g, p, m, v, *hyper, None)

    def add_unshard(b, h, W, dt=1):
        return raw.fsdp_batch_add_unshard(b, h, table(W), ctypes.c_void_p(0x7000000), dt)

    b = ctypes.c_void_p()
    assert raw.fsdp_batch_create(ctypes.byref(b)) == OK
    assert _plan(raw, b) == []
    # a GPT-2-small block over 8 ranks: six updates and six unshards share one grid, a seventh update opens another
    rc, small = _init(raw, workloads.config(0).units[0].shapes, 8)
    S = 885984
    for _ in range(6):
        assert add_update(b, small, 8) == OK and add_unshard(b, small, 8) == OK
    assert _plan(raw, b) == [("batch_kernel", 6, 6, 6 * (S // 4 // 256 + 1) + 6 * 8 * (S // 8 // 256 + 1))]
    assert add_update(b, small, 8) == OK
    assert [p[:3] for p in _plan(raw, b)] == [("batch_kernel", 6, 6), ("reduce_kernel", 1, 0)]    # alone in its grid
    # another gradient dtype cannot join the open grid; an fp32 unshard goes through its own kernel
    assert add_update(b, small, 8, dt=1) == OK
    assert add_unshard(b, small, 8, dt=0) == OK
    assert [p[:3] for p in _plan(raw, b)][2:] == [("reduce_kernel", 1, 0), ("unshard_f32_kernel", 0, 1)]
    assert raw.fsdp_batch_clear(b) == OK and _plan(raw, b) == []
    # 65 ranks: each operation is split over two launches of its own kernel
    rc, wide = _init(raw, [(100000,)], 65)
    assert add_update(b, wide, 65) == OK and add_unshard(b, wide, 65) == OK
    assert [p[0] for p in _plan(raw, b)] == ["reduce_kernel", "reduce_kernel", "unshard_lp_kernel", "unshard_lp_kernel"]
    assert _plan(raw, b)[3][3] == 1 * (100000 // 65 // 8 // 256 + 1)          # the second unshard launch carries one rank
    raw.fsdp_batch_clear(b)
    # 64 ranks fit one grid (the pointer pool holds 64 + 64)
    rc, w64 = _init(raw, [(100000,)], 64)
    assert add_update(b, w64, 64, dt=1) == OK and add_unshard(b, w64, 64) == OK
    assert [p[:3] for p in _plan(raw, b)] == [("batch_kernel", 1, 1)]
    raw.fsdp_batch_clear(b)
    # the 1.3B block, fp32 gradients: a large update pairs with a large unshard
    rc, mid = _init(raw, workloads.config(2).units[0].shapes, 12)
    assert add_update(b, mid, 12) == OK and add_unshard(b, mid, 12) == OK
    assert [p[:3] for p in _plan(raw, b)] == [("batch_kernel", 1, 1)]
    raw.fsdp_batch_clear(b)
    # the GPT-3-175B block, bf16 gradients: no pairing; the lone update takes the stand-alone kernel and, with 16
    # ranks, its half-chunk walk (single-wave workgroups of 256 elements); the lone unshard of aligned shards goes
    # out as single-wave workgroups too
    rc, big = _init(raw, workloads.config(4).units[0].shapes, 16)
    S = 113256192
    assert add_update(b, big, 16, dt=1) == OK and add_unshard(b, big, 16) == OK
    assert _plan(raw, b) == [("reduce_kernel", 1, 0, -(-(S // 4 + 1) // 64)),
                             ("unshard_lp_light_kernel", 0, 1, 16 * (-(-(S // 4 + 1) // 64)))]
    raw.fsdp_batch_clear(b)
    # a lone unshard whose loads would not be 16-byte aligned keeps the kernel that realigns through LDS
    assert raw.fsdp_batch_add_unshard(b, big, _table([0x9000004 + 0x1000 * j for j in range(16)]), ctypes.c_void_p(0x7000000), 1) == OK
    assert _plan(raw, b) == [("unshard_lp_kernel", 0, 1, 16 * (S // 8 // 256 + 1))]
    raw.fsdp_batch_clear(b)
    # the library's own choice of walk for a lone large update (measured rules): the Llama-7B block over 64 ranks
    # takes the deep walk (386 workgroups of 1024 chunks), a 16 M-element shard over 8 ranks with 16-bit gradients
    # the half-chunk walk
    rc, llama = _init(raw, workloads.config(3).units[0].shapes, 64)
    S3 = 3162240
    assert add_update(b, llama, 64, dt=1) == OK
    assert _plan(raw, b) == [("reduce_kernel", 1, 0, -(-(S3 // 8 + 1) // 1024))]
    raw.fsdp_batch_clear(b)
    rc, w8 = _init(raw, [(8 * 16000000,)], 8)
    assert add_update(b, w8, 8, dt=1) == OK
    assert _plan(raw, b) == [("reduce_kernel", 1, 0, -(-(16000000 // 4 + 1) // 64))]
    raw.fsdp_batch_clear(b)
    rc, w8m = _init(raw, [(8 * 2000000,)], 8)       # 80 MB of update, alone in its grid: the stand-alone kernel, in the
    assert add_update(b, w8m, 8, dt=1) == OK        # half-chunk walk with 16-bit gradients, in the deep one with fp32 ones
    assert _plan(raw, b) == [("reduce_kernel", 1, 0, -(-(2000000 // 4 + 1) // 64))]
    raw.fsdp_batch_clear(b)
    assert add_update(b, w8m, 8, dt=0) == OK
    assert _plan(raw, b) == [("reduce_kernel", 1, 0, -(-(2000000 // 4 + 1) // 1024))]     # 489 deep workgroups, 8 ranks
    raw.fsdp_batch_clear(b)
    raw.fsdp_layout_destroy(w8m)
    rc, w8s = _init(raw, [(8 * 8000000,)], 8)       # fp32 gradients, 8 M elements: below the fp32 rule's 12 Mi, wide walk
    assert add_update(b, w8s, 8, dt=0) == OK
    assert _plan(raw, b) == [("reduce_kernel", 1, 0, -(-(8000000 // 4 + 1) // 256))]
    raw.fsdp_batch_clear(b)
    raw.fsdp_layout_destroy(w8s)
    raw.fsdp_layout_destroy(llama)
    raw.fsdp_layout_destroy(w8)
    # ... unless its layout asks for the wide walk
    hw = ctypes.c_void_p()
    shapes = workloads.config(4).units[0].shapes
    flat = [d for s in shapes for d in s]
    assert raw.fsdp_layout_init_ex((ctypes.c_int64 * len(flat))(*flat), (ctypes.c_int32 * len(shapes))(*[len(s) for s in shapes]),
                                   len(shapes), 16, L.FSDP_WALK_WIDE, ctypes.byref(hw)) == OK
    assert add_update(b, hw, 16, dt=1) == OK
    assert _plan(raw, b) == [("reduce_kernel", 1, 0, -(-(S // 8 + 1) // 256))]
    assert raw.fsdp_kernel_name(99) is None
    assert raw.fsdp_batch_launch_count(None, None) == NULL
    raw.fsdp_batch_destroy(b)
    for h in (small, wide, w64, mid, big, hw):
        raw.fsdp_layout_destroy(h)
