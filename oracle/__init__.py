"""ctypes front-end of the CPU oracle (``pv_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py``.  It never imports the HIP
package and the HIP package never imports it.

All arrays are numpy; 16-bit float data travels as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpv_oracle.so")
_lib = None

DTYPES = {"f16": 0, "bf16": 1}


class PoolDesc(ctypes.Structure):
    _fields_ = [("num_pages", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP).  Returns the library path."""
    srcs = [os.path.join(_HERE, "pv_oracle.c"), os.path.join(_HERE, "pv_oracle_attend.inc")]
    if not force and os.path.exists(_LIB_PATH) and \
            all(os.path.getmtime(_LIB_PATH) >= os.path.getmtime(s) for s in srcs):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra",
           "-o", _LIB_PATH, srcs[0], "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    _lib = _bind(ctypes.CDLL(_LIB_PATH))
    return _lib


def _bind(lib):
    """Declare the argument types of an oracle library (also used by the tests that load
    deliberately broken builds of it)."""
    i32p = ctypes.POINTER(ctypes.c_int32)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    f64p = ctypes.POINTER(ctypes.c_double)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    dp = ctypes.POINTER(PoolDesc)
    lib.pvo_k_index.restype = ctypes.c_int64
    lib.pvo_k_index.argtypes = [dp] + [ctypes.c_int64] * 4
    lib.pvo_v_index.restype = ctypes.c_int64
    lib.pvo_v_index.argtypes = [dp] + [ctypes.c_int64] * 4
    lib.pvo_widen16.restype = ctypes.c_double
    lib.pvo_widen16.argtypes = [ctypes.c_uint16, ctypes.c_int32]
    lib.pvo_kv_append.restype = ctypes.c_int
    lib.pvo_kv_append.argtypes = [dp, u16p, u16p, i32p, ctypes.c_int32, i32p, i32p, i32p,
                                  ctypes.c_int32, u16p, u16p]
    lib.pvo_gather_kv.restype = ctypes.c_int
    lib.pvo_gather_kv.argtypes = [dp, u16p, u16p, i32p, ctypes.c_int32, ctypes.c_int32,
                                  ctypes.c_int32, f64p, f64p]
    lib.pvo_attn.restype = ctypes.c_int
    lib.pvo_attn.argtypes = [dp, ctypes.c_int32, u16p, u16p, u16p, i32p, ctypes.c_int32, i32p,
                             i32p, i32p, ctypes.c_int32, ctypes.c_double, u8p, ctypes.c_int32,
                             ctypes.c_int32, f64p, ctypes.c_int32, ctypes.c_int32, f64p, i32p]
    lib.pvo_cost.restype = ctypes.c_double
    lib.pvo_cost.argtypes = [i32p, f64p, ctypes.c_int32, ctypes.c_double, ctypes.c_int32]
    lib.pvo_retention_order.restype = ctypes.c_int
    lib.pvo_retention_order.argtypes = [f64p, f64p, ctypes.c_int32, i32p]
    f32p = ctypes.POINTER(ctypes.c_float)
    lib.pvo_rope_table.restype = ctypes.c_int
    lib.pvo_rope_table.argtypes = [ctypes.c_double, ctypes.c_int32, ctypes.c_int32, f32p]
    lib.pvo_rope.restype = ctypes.c_int
    lib.pvo_rope.argtypes = [u16p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, i32p, f32p,
                             ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, f64p]
    lib.pvo_round16.restype = ctypes.c_int
    lib.pvo_round16.argtypes = [f64p, ctypes.c_int64, ctypes.c_int32, u16p]
    lib.pvo_pages_gather.restype = ctypes.c_int
    lib.pvo_pages_gather.argtypes = [dp, u16p, u16p, i32p, ctypes.c_int32, u16p]
    lib.pvo_pages_scatter.restype = ctypes.c_int
    lib.pvo_pages_scatter.argtypes = [dp, u16p, i32p, ctypes.c_int32, u16p, u16p]
    return lib


def _desc(num_pages, page_size, num_kv_heads, head_dim, dtype) -> PoolDesc:
    return PoolDesc(int(num_pages), int(page_size), int(num_kv_heads), int(head_dim),
                    DTYPES[dtype])


def _p(a: Optional[np.ndarray], ctype):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc} "
                           "(1 bad argument, 2 page index out of range, 3 out of memory)")


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact value of 16-bit patterns as float64 (element-wise, via the C routine)."""
    lib = _load()
    flat = np.ascontiguousarray(bits, dtype=np.uint16).ravel()
    out = np.empty(flat.shape, dtype=np.float64)
    code = DTYPES[dtype]
    for i, b in enumerate(flat):
        out[i] = lib.pvo_widen16(int(b), code)
    return out.reshape(np.shape(bits))


def k_index(pool: Tuple[int, int, int, int, str], page, head, slot, d) -> int:
    return int(_load().pvo_k_index(ctypes.byref(_desc(*pool)), page, head, slot, d))


def v_index(pool: Tuple[int, int, int, int, str], page, head, slot, d) -> int:
    return int(_load().pvo_v_index(ctypes.byref(_desc(*pool)), page, head, slot, d))


def kv_append(pool, k_new, v_new, page_table, slot_offsets, q_lens, q_start, k_pages, v_pages):
    """Scatter new rows into the pools IN PLACE (uint16 arrays)."""
    lib = _load()
    desc = _desc(*pool)
    page_table = _i32(page_table)
    assert page_table.ndim == 2
    k_new = np.ascontiguousarray(k_new, dtype=np.uint16)
    v_new = np.ascontiguousarray(v_new, dtype=np.uint16)
    assert k_pages.dtype == np.uint16 and k_pages.flags.c_contiguous
    assert v_pages.dtype == np.uint16 and v_pages.flags.c_contiguous
    so, ql, qs = _i32(slot_offsets), _i32(q_lens), _i32(q_start)
    rc = lib.pvo_kv_append(ctypes.byref(desc), _p(k_new, ctypes.c_uint16),
                           _p(v_new, ctypes.c_uint16), _p(page_table, ctypes.c_int32),
                           page_table.shape[1], _p(so, ctypes.c_int32), _p(ql, ctypes.c_int32),
                           _p(qs, ctypes.c_int32), len(ql), _p(k_pages, ctypes.c_uint16),
                           _p(v_pages, ctypes.c_uint16))
    _check(rc, "kv_append")


def gather_kv(pool, k_pages, v_pages, page_row, length, head):
    """Contiguous [length, D] float64 K and V of one request / KV head."""
    lib = _load()
    desc = _desc(*pool)
    D = pool[3]
    page_row = _i32(page_row)
    k = np.empty((length, D), dtype=np.float64)
    v = np.empty((length, D), dtype=np.float64)
    rc = lib.pvo_gather_kv(ctypes.byref(desc), _p(k_pages, ctypes.c_uint16),
                           _p(v_pages, ctypes.c_uint16), _p(page_row, ctypes.c_int32),
                           len(page_row), int(length), int(head), _p(k, ctypes.c_double),
                           _p(v, ctypes.c_double))
    _check(rc, "gather_kv")
    return k, v


def attn(pool, num_q_heads, q, k_pages, v_pages, page_table, ctx_lens, q_lens, q_start, scale,
         unit_mask=None, precision="f64", num_threads=0, probs_of=None):
    """Causal paged attention of the whole batch.

    Returns ``out`` ([total_q, Hq, D] float64, NaN where a unit was not
    selected), and additionally the probability rows of ``probs_of=(req, head)``
    when given.  ``info['threads']`` reports the OpenMP team size.
    """
    lib = _load()
    desc = _desc(*pool)
    D = pool[3]
    page_table = _i32(page_table)
    cl, ql, qs = _i32(ctx_lens), _i32(q_lens), _i32(q_start)
    total_q = int(ql.sum())
    q = np.ascontiguousarray(q, dtype=np.uint16)
    assert q.size == total_q * num_q_heads * D
    out = np.full((total_q, num_q_heads, D), np.nan, dtype=np.float64)
    mask = None
    if unit_mask is not None:
        mask = np.ascontiguousarray(unit_mask, dtype=np.uint8).ravel()
        assert mask.size == len(ql) * pool[2]
    probs = None
    pr, ph = -1, -1
    if probs_of is not None:
        pr, ph = probs_of
        probs = np.zeros((int(ql[pr]), int(cl[pr] + ql[pr])), dtype=np.float64)
    threads = ctypes.c_int32(0)
    rc = lib.pvo_attn(ctypes.byref(desc), int(num_q_heads), _p(q, ctypes.c_uint16),
                      _p(k_pages, ctypes.c_uint16), _p(v_pages, ctypes.c_uint16),
                      _p(page_table, ctypes.c_int32), page_table.shape[1],
                      _p(cl, ctypes.c_int32), _p(ql, ctypes.c_int32), _p(qs, ctypes.c_int32),
                      len(ql), float(scale), _p(mask, ctypes.c_uint8),
                      {"f64": 0, "f32": 1}[precision], int(num_threads),
                      _p(out, ctypes.c_double), int(pr), int(ph), _p(probs, ctypes.c_double),
                      ctypes.byref(threads))
    _check(rc, "attn")
    info = {"threads": int(threads.value)}
    if probs_of is not None:
        return out, probs, info
    return out, info


def pages_gather(pool, k_pages, v_pages, page_ids):
    """Staging image [n, 2, page_elems] (uint16) of the listed pages: K image then V image."""
    lib = _load()
    desc = _desc(*pool)
    ids = _i32(page_ids)
    page_elems = pool[2] * pool[1] * pool[3]
    staging = np.zeros((len(ids), 2, page_elems), dtype=np.uint16)
    rc = lib.pvo_pages_gather(ctypes.byref(desc), _p(k_pages, ctypes.c_uint16),
                              _p(v_pages, ctypes.c_uint16), _p(ids, ctypes.c_int32), len(ids),
                              _p(staging, ctypes.c_uint16))
    _check(rc, "pages_gather")
    return staging


def pages_scatter(pool, staging, page_ids, k_pages, v_pages):
    """Write a staging image back into the listed pages of the pools IN PLACE."""
    lib = _load()
    desc = _desc(*pool)
    ids = _i32(page_ids)
    staging = np.ascontiguousarray(staging, dtype=np.uint16)
    assert k_pages.dtype == np.uint16 and k_pages.flags.c_contiguous
    assert v_pages.dtype == np.uint16 and v_pages.flags.c_contiguous
    rc = lib.pvo_pages_scatter(ctypes.byref(desc), _p(staging, ctypes.c_uint16),
                               _p(ids, ctypes.c_int32), len(ids), _p(k_pages, ctypes.c_uint16),
                               _p(v_pages, ctypes.c_uint16))
    _check(rc, "pages_scatter")


def cost(ctx_points, attn_cost, c_other, l) -> float:
    """Cost(l) = interpolated attention cost + c (eviction policy's recomputation cost)."""
    lib = _load()
    pts = _i32(ctx_points)
    ys = np.ascontiguousarray(attn_cost, dtype=np.float64)
    return float(lib.pvo_cost(_p(pts, ctypes.c_int32), _p(ys, ctypes.c_double), len(pts),
                              float(c_other), int(l)))


def retention_order(cost_values, idle_time) -> np.ndarray:
    """Chunk indices in eviction order: ascending V = cost / idle_time."""
    lib = _load()
    c = np.ascontiguousarray(cost_values, dtype=np.float64)
    t = np.ascontiguousarray(idle_time, dtype=np.float64)
    assert c.shape == t.shape and c.ndim == 1
    order = np.zeros(len(c), dtype=np.int32)
    _check(lib.pvo_retention_order(_p(c, ctypes.c_double), _p(t, ctypes.c_double), len(c),
                                   _p(order, ctypes.c_int32)), "retention_order")
    return order


ROPE_STYLES = {"interleaved": 0, "half": 1}


def rope_table(base: float, head_dim: int, max_pos: int) -> np.ndarray:
    """float32 [max_pos, head_dim]: D/2 cosines then D/2 sines of t * base^(-2i/D)."""
    out = np.zeros((max_pos, head_dim), dtype=np.float32)
    _check(_load().pvo_rope_table(float(base), int(head_dim), int(max_pos),
                                  _p(out, ctypes.c_float)), "pvo_rope_table")
    return out


def rope(x_bits: np.ndarray, positions, table: np.ndarray, style: str, dtype: str) -> np.ndarray:
    """Rotary embedding of x [rows, heads, D] (16-bit patterns) at positions [rows]; float64,
    not rounded."""
    x = np.ascontiguousarray(x_bits, dtype=np.uint16)
    rows, heads, D = x.shape
    pos = _i32(positions)
    tab = np.ascontiguousarray(table, dtype=np.float32)
    assert pos.shape == (rows,) and tab.ndim == 2 and tab.shape[1] == D
    out = np.zeros((rows, heads, D), dtype=np.float64)
    _check(_load().pvo_rope(_p(x, ctypes.c_uint16), rows, heads, D, _p(pos, ctypes.c_int32),
                            _p(tab, ctypes.c_float), tab.shape[0], ROPE_STYLES[style],
                            DTYPES[dtype], _p(out, ctypes.c_double)), "pvo_rope")
    return out


def round16(values: np.ndarray, dtype: str) -> np.ndarray:
    """Nearest 16-bit value (ties to even) of every float64 in `values`, as bit patterns."""
    v = np.ascontiguousarray(values, dtype=np.float64)
    out = np.zeros(v.shape, dtype=np.uint16)
    _check(_load().pvo_round16(_p(v, ctypes.c_double), v.size, DTYPES[dtype],
                               _p(out, ctypes.c_uint16)), "pvo_round16")
    return out
