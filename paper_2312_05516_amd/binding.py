"""ctypes binding of libpv.so: argument marshalling only.

Every function has the name of the C entry point it calls (see ``include/pv.h``).  Device arrays
are passed as torch tensors (or raw integer addresses); host length arrays as anything numpy can
turn into int32.  PyTorch is used for device memory and the current stream, nothing else: every
step of the path runs in the library's HIP kernels.  There is no CPU fallback: if the library has
not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
# torch is imported BEFORE libpv.so is loaded on purpose: the PyTorch wheel carries its own HIP
# runtime, and a process must end up with exactly one.  Loaded first, torch's runtime also
# satisfies libpv.so's dependency, so device pointers and streams made by torch are valid inside
# the library's launches.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpv.so")

PV_OK = 0
STATUS_NAMES = {0: "PV_OK", 1: "PV_ERR_INVALID_ARG", 2: "PV_ERR_UNSUPPORTED",
                3: "PV_ERR_OUT_OF_RANGE", 4: "PV_ERR_WORKSPACE", 5: "PV_ERR_HIP"}
DTYPES = {"f16": 0, "bf16": 1}

EXPORTS = [
    "pv_status_string", "pv_pool_bytes", "pv_pool_k_offset", "pv_pool_v_offset",
    "pv_plan_create", "pv_plan_destroy", "pv_plan_upload", "pv_plan_upload_to",
    "pv_plan_device_bytes", "pv_plan_owns_device_memory", "pv_plan_total_q", "pv_plan_q_start",
    "pv_plan_workspace_bytes", "pv_plan_num_work_items", "pv_plan_work_item",
    "pv_plan_check_page_table", "pv_plan_enable_timing", "pv_plan_kernel_ms",
    "pv_kv_append_planned", "pv_multi_token_paged_attn_planned",
    "pv_kv_append", "pv_multi_token_paged_attn", "pv_attn_workspace_bytes",
    "pv_pages_gather", "pv_pages_scatter", "pv_cost_model", "pv_retention_order",
    "pv_rope_kv_append_planned", "pv_rope_table",
    "pv_multi_token_paged_attn_noalloc", "pv_static_scratch_bytes",
]


class PvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({status_string(status)})")


class PoolDesc(ctypes.Structure):
    _fields_ = [("num_pages", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -m paper_2312_05516_amd.build or "
        "__graft_entry__.build()).  There is no fallback path.")

_lib = ctypes.CDLL(LIB_PATH)

_i32p = ctypes.POINTER(ctypes.c_int32)
_descp = ctypes.POINTER(PoolDesc)
_vp = ctypes.c_void_p

_lib.pv_status_string.restype = ctypes.c_char_p
_lib.pv_status_string.argtypes = [ctypes.c_int]
_lib.pv_pool_bytes.restype = ctypes.c_size_t
_lib.pv_pool_bytes.argtypes = [_descp]
for _n in ("pv_pool_k_offset", "pv_pool_v_offset"):
    getattr(_lib, _n).restype = ctypes.c_int64
    getattr(_lib, _n).argtypes = [_descp] + [ctypes.c_int32] * 4
_lib.pv_plan_create.restype = ctypes.c_int
_lib.pv_plan_create.argtypes = [_descp, ctypes.c_int32, _i32p, _i32p, ctypes.c_int32,
                                ctypes.c_int32, ctypes.POINTER(_vp)]
_lib.pv_plan_destroy.restype = None
_lib.pv_plan_destroy.argtypes = [_vp]
_lib.pv_plan_upload.restype = ctypes.c_int
_lib.pv_plan_upload.argtypes = [_vp]
_lib.pv_plan_upload_to.restype = ctypes.c_int
_lib.pv_plan_upload_to.argtypes = [_vp, _vp, ctypes.c_size_t, _vp]
_lib.pv_plan_device_bytes.restype = ctypes.c_size_t
_lib.pv_plan_device_bytes.argtypes = [_vp]
_lib.pv_plan_owns_device_memory.restype = ctypes.c_int32
_lib.pv_plan_owns_device_memory.argtypes = [_vp]
_lib.pv_plan_total_q.restype = ctypes.c_int32
_lib.pv_plan_total_q.argtypes = [_vp]
_lib.pv_plan_q_start.restype = _i32p
_lib.pv_plan_q_start.argtypes = [_vp]
_lib.pv_plan_workspace_bytes.restype = ctypes.c_size_t
_lib.pv_plan_workspace_bytes.argtypes = [_vp]
_lib.pv_plan_num_work_items.restype = ctypes.c_int32
_lib.pv_plan_num_work_items.argtypes = [_vp, ctypes.c_int32]
_lib.pv_plan_work_item.restype = ctypes.c_int
_lib.pv_plan_work_item.argtypes = [_vp, ctypes.c_int32, ctypes.c_int32, _i32p]
_lib.pv_plan_check_page_table.restype = ctypes.c_int
_lib.pv_plan_check_page_table.argtypes = [_vp, _i32p, ctypes.c_int32]
_lib.pv_plan_enable_timing.restype = ctypes.c_int
_lib.pv_plan_enable_timing.argtypes = [_vp, ctypes.c_int32]
_lib.pv_plan_kernel_ms.restype = ctypes.c_int
_lib.pv_plan_kernel_ms.argtypes = [_vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_float)]
_lib.pv_kv_append_planned.restype = ctypes.c_int
_lib.pv_kv_append_planned.argtypes = [_vp] * 7
_lib.pv_multi_token_paged_attn_planned.restype = ctypes.c_int
_lib.pv_multi_token_paged_attn_planned.argtypes = [_vp, _vp, _vp, _vp, _vp, ctypes.c_float, _vp,
                                                   _vp, ctypes.c_size_t, _vp]
_lib.pv_multi_token_paged_attn_noalloc.restype = ctypes.c_int
_lib.pv_multi_token_paged_attn_noalloc.argtypes = [_vp, _vp, _vp, _vp, _vp, ctypes.c_float, _vp, _vp]
_lib.pv_static_scratch_bytes.restype = ctypes.c_size_t
_lib.pv_static_scratch_bytes.argtypes = []
_lib.pv_kv_append.restype = ctypes.c_int
_lib.pv_kv_append.argtypes = [_descp, _vp, _vp, _vp, ctypes.c_int32, _i32p, _i32p, _i32p,
                              ctypes.c_int32, ctypes.c_int32, _vp, _vp, _vp]
_lib.pv_multi_token_paged_attn.restype = ctypes.c_int
_lib.pv_multi_token_paged_attn.argtypes = [_descp, ctypes.c_int32, _vp, _vp, _vp, _vp,
                                           ctypes.c_int32, _i32p, _i32p, _i32p, ctypes.c_int32,
                                           ctypes.c_int32, ctypes.c_float, _vp, _vp,
                                           ctypes.c_size_t, _vp]
_lib.pv_pages_gather.restype = ctypes.c_int
_lib.pv_pages_gather.argtypes = [_descp, _vp, _vp, _vp, ctypes.c_int32, _vp, _vp]
_lib.pv_pages_scatter.restype = ctypes.c_int
_lib.pv_pages_scatter.argtypes = [_descp, _vp, _vp, ctypes.c_int32, _vp, _vp, _vp]
_f64p = ctypes.POINTER(ctypes.c_double)
_lib.pv_cost_model.restype = ctypes.c_double
_lib.pv_cost_model.argtypes = [_i32p, _f64p, ctypes.c_int32, ctypes.c_double, ctypes.c_int32]
_lib.pv_retention_order.restype = ctypes.c_int
_lib.pv_retention_order.argtypes = [_f64p, _f64p, ctypes.c_int32, _i32p]
_lib.pv_rope_kv_append_planned.restype = ctypes.c_int
_lib.pv_rope_kv_append_planned.argtypes = [_vp] * 6 + [ctypes.c_int32, ctypes.c_int32] + [_vp] * 4
_lib.pv_rope_table.restype = ctypes.c_int
_lib.pv_rope_table.argtypes = [ctypes.c_double, ctypes.c_int32, ctypes.c_int32,
                               ctypes.POINTER(ctypes.c_float)]
_lib.pv_attn_workspace_bytes.restype = ctypes.c_size_t
_lib.pv_attn_workspace_bytes.argtypes = [_descp] + [ctypes.c_int32] * 4


# ------------------------------------------------------------------ marshalling helpers
def _ptr(x) -> Optional[int]:
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        if not x.is_contiguous():
            raise ValueError("tensor arguments must be contiguous")
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        if not x.flags.c_contiguous:
            raise ValueError("array arguments must be contiguous")
        return x.ctypes.data
    raise TypeError(f"cannot take the address of {type(x)}")


def _host_i32(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _i32(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_i32p)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _nbytes(x) -> int:
    if x is None:
        return 0
    if hasattr(x, "element_size"):
        return x.numel() * x.element_size()
    return int(x.nbytes)


def pool_desc(num_pages: int, num_kv_heads: int, head_dim: int, dtype: str,
              page_size: int = 16) -> PoolDesc:
    return PoolDesc(int(num_pages), int(page_size), int(num_kv_heads), int(head_dim),
                    DTYPES[dtype] if isinstance(dtype, str) else int(dtype))


def _check(status: int, where: str):
    if status != PV_OK:
        raise PvError(status, where)


# ------------------------------------------------------------------ entry points
def status_string(status: int) -> str:
    return _lib.pv_status_string(int(status)).decode()


def pool_bytes(desc: PoolDesc) -> int:
    return int(_lib.pv_pool_bytes(ctypes.byref(desc)))


def pool_k_offset(desc: PoolDesc, page: int, head: int, slot: int, d: int) -> int:
    return int(_lib.pv_pool_k_offset(ctypes.byref(desc), page, head, slot, d))


def pool_v_offset(desc: PoolDesc, page: int, head: int, slot: int, d: int) -> int:
    return int(_lib.pv_pool_v_offset(ctypes.byref(desc), page, head, slot, d))


class Plan:
    """Owner of a ``pv_plan*``."""

    def __init__(self, handle: int, desc: PoolDesc, num_q_heads: int, num_reqs: int):
        self._h = handle
        self.desc = desc
        self.num_q_heads = num_q_heads
        self.num_reqs = num_reqs

    @property
    def handle(self) -> int:
        if not self._h:
            raise ValueError("plan already destroyed")
        return self._h

    def destroy(self):
        if self._h:
            _lib.pv_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def plan_create(desc: PoolDesc, num_q_heads: int, ctx_lens, q_lens,
                max_pages_per_req: int) -> Plan:
    cl, ql = _host_i32(ctx_lens), _host_i32(q_lens)
    if cl.shape != ql.shape or cl.ndim != 1:
        raise ValueError("ctx_lens and q_lens must be 1-D and of equal length")
    h = _vp()
    _check(_lib.pv_plan_create(ctypes.byref(desc), int(num_q_heads), _i32(cl), _i32(ql), len(cl),
                               int(max_pages_per_req), ctypes.byref(h)), "pv_plan_create")
    return Plan(h.value, desc, int(num_q_heads), len(cl))


def plan_destroy(plan: Plan):
    plan.destroy()


def plan_upload(plan: Plan):
    _check(_lib.pv_plan_upload(plan.handle), "pv_plan_upload")


def plan_upload_to(plan: Plan, device_buf, stream=None):
    """device_buf: a CUDA tensor (256-byte aligned) of at least plan_device_bytes(plan) bytes that
    the caller keeps alive while the plan is in use."""
    _check(_lib.pv_plan_upload_to(plan.handle, _ptr(device_buf), _nbytes(device_buf),
                                  _stream(stream)), "pv_plan_upload_to")


def plan_device_bytes(plan: Plan) -> int:
    return int(_lib.pv_plan_device_bytes(plan.handle))


def plan_owns_device_memory(plan: Plan) -> bool:
    return bool(_lib.pv_plan_owns_device_memory(plan.handle))


def plan_total_q(plan: Plan) -> int:
    return int(_lib.pv_plan_total_q(plan.handle))


def plan_q_start(plan: Plan) -> np.ndarray:
    p = _lib.pv_plan_q_start(plan.handle)
    if plan.num_reqs == 0:
        return np.zeros(0, dtype=np.int32)
    return np.ctypeslib.as_array(p, shape=(plan.num_reqs,)).copy()


def plan_workspace_bytes(plan: Plan) -> int:
    return int(_lib.pv_plan_workspace_bytes(plan.handle))


def plan_num_work_items(plan: Plan, kind: int) -> int:
    return int(_lib.pv_plan_num_work_items(plan.handle, int(kind)))


def plan_work_item(plan: Plan, kind: int, index: int) -> np.ndarray:
    out = np.zeros(8, dtype=np.int32)
    _check(_lib.pv_plan_work_item(plan.handle, int(kind), int(index), _i32(out)),
           "pv_plan_work_item")
    return out


def plan_check_page_table(plan: Plan, page_table_host, check_append_unique: bool = True) -> int:
    """Returns the status code (does not raise): the caller decides what a bad table means."""
    pt = _host_i32(page_table_host)
    return int(_lib.pv_plan_check_page_table(plan.handle, _i32(pt), int(check_append_unique)))


def plan_enable_timing(plan: Plan, enable: bool = True):
    _check(_lib.pv_plan_enable_timing(plan.handle, int(enable)), "pv_plan_enable_timing")


def plan_kernel_ms(plan: Plan, kind: int) -> float:
    ms = ctypes.c_float(-1.0)
    _check(_lib.pv_plan_kernel_ms(plan.handle, int(kind), ctypes.byref(ms)), "pv_plan_kernel_ms")
    return float(ms.value)


def kv_append_planned(plan: Plan, k_new, v_new, page_table, k_pages, v_pages, stream=None):
    _check(_lib.pv_kv_append_planned(plan.handle, _ptr(k_new), _ptr(v_new), _ptr(page_table),
                                     _ptr(k_pages), _ptr(v_pages), _stream(stream)),
           "pv_kv_append_planned")


ROPE_STYLES = {"interleaved": 0, "half": 1}


def rope_table(base: float, head_dim: int, max_pos: int) -> np.ndarray:
    """Host float32 [max_pos, head_dim]: D/2 cosines then D/2 sines per position."""
    out = np.zeros((int(max_pos), int(head_dim)), dtype=np.float32)
    _check(_lib.pv_rope_table(float(base), int(head_dim), int(max_pos),
                              out.ctypes.data_as(ctypes.POINTER(ctypes.c_float))), "pv_rope_table")
    return out


def rope_kv_append_planned(plan: Plan, q_in, q_out, k_new, v_new, cos_sin, style, page_table,
                           k_pages, v_pages, stream=None):
    """cos_sin: device float32 [max_pos, D] (contiguous); style: "interleaved" | "half" | 0 | 1."""
    st = ROPE_STYLES[style] if isinstance(style, str) else int(style)
    _check(_lib.pv_rope_kv_append_planned(plan.handle, _ptr(q_in), _ptr(q_out), _ptr(k_new),
                                          _ptr(v_new), _ptr(cos_sin), int(cos_sin.shape[0]), st,
                                          _ptr(page_table), _ptr(k_pages), _ptr(v_pages),
                                          _stream(stream)), "pv_rope_kv_append_planned")


def multi_token_paged_attn_planned(plan: Plan, q, k_pages, v_pages, page_table, scale: float, out,
                                   workspace=None, stream=None):
    _check(_lib.pv_multi_token_paged_attn_planned(
        plan.handle, _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(page_table), float(scale),
        _ptr(out), _ptr(workspace), _nbytes(workspace), _stream(stream)),
        "pv_multi_token_paged_attn_planned")


def multi_token_paged_attn_noalloc(plan: Plan, q, k_pages, v_pages, page_table, scale: float, out,
                                   stream=None):
    _check(_lib.pv_multi_token_paged_attn_noalloc(
        plan.handle, _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(page_table), float(scale),
        _ptr(out), _stream(stream)), "pv_multi_token_paged_attn_noalloc")


def static_scratch_bytes() -> int:
    return int(_lib.pv_static_scratch_bytes())


def kv_append(desc: PoolDesc, k_new, v_new, page_table, max_pages_per_req: int, slot_offsets,
              q_lens, q_start, k_pages, v_pages, stream=None, total_q: Optional[int] = None):
    so, ql, qs = _host_i32(slot_offsets), _host_i32(q_lens), _host_i32(q_start)
    tq = int(ql.sum()) if total_q is None else int(total_q)
    _check(_lib.pv_kv_append(ctypes.byref(desc), _ptr(k_new), _ptr(v_new), _ptr(page_table),
                             int(max_pages_per_req), _i32(so), _i32(ql), _i32(qs), len(ql), tq,
                             _ptr(k_pages), _ptr(v_pages), _stream(stream)), "pv_kv_append")


def multi_token_paged_attn(desc: PoolDesc, num_q_heads: int, q, k_pages, v_pages, page_table,
                           max_pages_per_req: int, ctx_lens, q_lens, q_start, scale: float, out,
                           workspace=None, stream=None, total_q: Optional[int] = None):
    cl, ql, qs = _host_i32(ctx_lens), _host_i32(q_lens), _host_i32(q_start)
    tq = int(ql.sum()) if total_q is None else int(total_q)
    _check(_lib.pv_multi_token_paged_attn(
        ctypes.byref(desc), int(num_q_heads), _ptr(q), _ptr(k_pages), _ptr(v_pages),
        _ptr(page_table), int(max_pages_per_req), _i32(cl), _i32(ql), _i32(qs), len(ql), tq,
        float(scale), _ptr(out), _ptr(workspace), _nbytes(workspace), _stream(stream)),
        "pv_multi_token_paged_attn")


def attn_workspace_bytes(desc: PoolDesc, num_q_heads: int, num_reqs: int, total_q: int,
                         max_kv_len: int) -> int:
    return int(_lib.pv_attn_workspace_bytes(ctypes.byref(desc), int(num_q_heads), int(num_reqs),
                                            int(total_q), int(max_kv_len)))


def pages_gather(desc: PoolDesc, k_pages, v_pages, page_ids, n: int, staging, stream=None):
    _check(_lib.pv_pages_gather(ctypes.byref(desc), _ptr(k_pages), _ptr(v_pages), _ptr(page_ids),
                                int(n), _ptr(staging), _stream(stream)), "pv_pages_gather")


def pages_scatter(desc: PoolDesc, staging, page_ids, n: int, k_pages, v_pages, stream=None):
    _check(_lib.pv_pages_scatter(ctypes.byref(desc), _ptr(staging), _ptr(page_ids), int(n),
                                 _ptr(k_pages), _ptr(v_pages), _stream(stream)),
           "pv_pages_scatter")


def cost_model(ctx_points, attn_cost, c_other: float, l: int) -> float:
    pts = _host_i32(ctx_points)
    ys = np.ascontiguousarray(attn_cost, dtype=np.float64)
    return float(_lib.pv_cost_model(_i32(pts), ys.ctypes.data_as(_f64p), len(pts), float(c_other),
                                    int(l)))


def retention_order(cost, idle_time) -> np.ndarray:
    c = np.ascontiguousarray(cost, dtype=np.float64)
    t = np.ascontiguousarray(idle_time, dtype=np.float64)
    if c.shape != t.shape or c.ndim != 1:
        raise ValueError("cost and idle_time must be 1-D and of equal length")
    order = np.zeros(len(c), dtype=np.int32)
    _check(_lib.pv_retention_order(c.ctypes.data_as(_f64p), t.ctypes.data_as(_f64p), len(c),
                                   _i32(order)), "pv_retention_order")
    return order
