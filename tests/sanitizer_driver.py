"""Runs the CPU-side code of the repository inside AddressSanitizer / UndefinedBehaviorSanitizer builds.

Started by test_sanitizers.py in a subprocess (the sanitizer runtime has to be preloaded into the
interpreter).  argv: <sanitized oracle library> <sanitized host-plan library>.
"""
import ctypes
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, HERE)

import helpers as H  # noqa: E402
import oracle  # noqa: E402
from paper_2312_05516_amd import workloads as wl  # noqa: E402


def check_oracle(path: str):
    oracle._lib = oracle._bind(ctypes.CDLL(path))  # every oracle.* call below runs the sanitized build
    shapes = [([37, 100], [5, 12], 4, 4, 64, "f16"), ([0, 16, 31, 33], [7, 1, 33, 31], 4, 2, 64, "bf16"),
              ([200, 0, 77], [40, 130, 1], 8, 1, 128, "bf16"), ([10, 10], [0, 3], 2, 2, 64, "f16")]
    for ctx, qn, hq, hkv, d, dt in shapes:
        b = wl.custom(ctx, qn, num_q_heads=hq, num_kv_heads=hkv, head_dim=d, dtype=dt, seed=41)
        case = H.make_case(b, fill="nan")
        kp, vp = case.k_pool0.copy(), case.v_pool0.copy()
        oracle.kv_append(H.pool_tuple(b), case.k_new, case.v_new, b.page_table, b.ctx_lens, b.q_lens,
                         b.q_start, kp, vp)
        assert np.array_equal(kp, case.k_pool1) and np.array_equal(vp, case.v_pool1)
        out, _ = oracle.attn(H.pool_tuple(b), hq, case.q, kp, vp, b.page_table, b.ctx_lens, b.q_lens,
                             b.q_start, b.scale)
        assert np.abs(out - H.dense_causal_attention(case)).max() < 1e-9
        used = b.page_table[b.page_table >= 0].astype(np.int32)
        st = oracle.pages_gather(H.pool_tuple(b), kp, vp, used)
        k2, v2 = np.zeros_like(kp), np.zeros_like(vp)
        oracle.pages_scatter(H.pool_tuple(b), st, used, k2, v2)
    pts = [32, 64, 128, 256]
    ys = [1.0, 1.5, 2.5, 4.5]
    assert abs(oracle.cost(pts, ys, 0.5, 96) - 2.5) < 1e-12
    assert oracle.retention_order([3.0, 1.0, 2.0], [1.0, 1.0, 1.0]).tolist() == [1, 2, 0]
    table = oracle.rope_table(10000.0, 64, 50)
    x = wl.as_u16(wl.random_values((6, 2, 64), "bf16", 3))
    for style in ("interleaved", "half"):
        oracle.rope(x, np.arange(6) + 40, table, style, "bf16")
    oracle.round16(np.linspace(-70000, 70000, 1001), "f16")
    print("oracle under sanitizers: ok", flush=True)


class PoolDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("num_pages", "page_size", "num_kv_heads", "head_dim", "dtype")]


def check_plan(path: str):
    lib = ctypes.CDLL(path)
    i32p = ctypes.POINTER(ctypes.c_int32)
    vp = ctypes.c_void_p
    lib.pv_plan_create.restype = ctypes.c_int
    lib.pv_plan_create.argtypes = [ctypes.POINTER(PoolDesc), ctypes.c_int32, i32p, i32p, ctypes.c_int32,
                                   ctypes.c_int32, ctypes.POINTER(vp)]
    lib.pv_plan_destroy.argtypes = [vp]
    lib.pv_plan_num_work_items.restype = ctypes.c_int32
    lib.pv_plan_num_work_items.argtypes = [vp, ctypes.c_int32]
    lib.pv_plan_work_item.restype = ctypes.c_int
    lib.pv_plan_work_item.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, i32p]
    lib.pv_plan_check_page_table.restype = ctypes.c_int
    lib.pv_plan_check_page_table.argtypes = [vp, i32p, ctypes.c_int32]
    lib.pv_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.pv_plan_workspace_bytes.argtypes = [vp]
    lib.pv_plan_device_bytes.restype = ctypes.c_size_t
    lib.pv_plan_device_bytes.argtypes = [vp]
    lib.pv_cost_model.restype = ctypes.c_double
    lib.pv_cost_model.argtypes = [i32p, ctypes.POINTER(ctypes.c_double), ctypes.c_int32, ctypes.c_double,
                                  ctypes.c_int32]
    lib.pv_retention_order.restype = ctypes.c_int
    lib.pv_retention_order.argtypes = [ctypes.POINTER(ctypes.c_double)] * 2 + [ctypes.c_int32, i32p]
    lib.pv_rope_table.restype = ctypes.c_int
    lib.pv_rope_table.argtypes = [ctypes.c_double, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_float)]

    def i32(a):
        a = np.ascontiguousarray(a, dtype=np.int32)
        return a, a.ctypes.data_as(i32p)

    def plan_rows(desc, hq, ctx, qn, max_pages):
        """Creates a plan, walks every work item, returns rows covered per kind."""
        h = vp()
        c, cp = i32(ctx)
        q, qp = i32(qn)
        rc = lib.pv_plan_create(ctypes.byref(desc), hq, cp, qp, len(c), max_pages, ctypes.byref(h))
        if rc != 0:
            return rc, None
        rows = {}
        item = np.zeros(8, dtype=np.int32)
        for kind in (0, 1, 2, 3):
            n = lib.pv_plan_num_work_items(h, kind)
            tot = 0
            for i in range(n):
                assert lib.pv_plan_work_item(h, kind, i, item.ctypes.data_as(i32p)) == 0
                if kind != 2 and item[6] == 0:  # count every row once, not once per KV part
                    tot += int(item[3])
            rows[kind] = (n, tot)
        assert lib.pv_plan_work_item(h, 0, 1 << 30, item.ctypes.data_as(i32p)) != 0
        assert lib.pv_plan_device_bytes(h) % 256 == 0
        lib.pv_plan_workspace_bytes(h)
        return 0, (h, rows)

    for name in wl.CONFIG_ORDER:
        b = wl.CONFIGS[name]()
        desc = PoolDesc(b.num_pages, 16, b.num_kv_heads, b.head_dim, 0 if b.dtype == "f16" else 1)
        rc, res = plan_rows(desc, b.num_q_heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
        assert rc == 0
        h, rows = res
        G = b.num_q_heads // b.num_kv_heads
        assert rows[0][1] + rows[1][1] + rows[3][1] == int(b.q_lens.sum()) * G * b.num_kv_heads, (name, rows)
        t, tp = i32(b.page_table)
        assert lib.pv_plan_check_page_table(h, tp, 1) == 0
        t2 = t.copy()
        t2[0, 0] = b.num_pages  # out of the pool
        assert lib.pv_plan_check_page_table(h, t2.ctypes.data_as(i32p), 0) == 3
        lib.pv_plan_destroy(h)
    desc = PoolDesc(1 << 16, 16, 8, 128, 1)
    for ctx, qn, hq in [([50000], [1], 64), ([300] * 200 + [60000], [1] * 201, 8), ([120000], [128], 64),
                        ([], [], 8), ([0, 5], [0, 300], 8)]:
        rc, res = plan_rows(desc, hq, ctx, qn, 8192)
        assert rc == 0, (ctx[:3], rc)
        lib.pv_plan_destroy(res[0])
    for ctx, qn, hq, mp in [([-1], [1], 8, 4), ([60], [5], 8, 4), ([1], [1], 6, 4), ([2 ** 31 - 10], [100], 8, 4)]:
        rc, _ = plan_rows(desc, hq, ctx, qn, mp)
        assert rc != 0
    pts, ptp = i32([32, 64, 128, 256])
    ys = np.array([1.0, 1.5, 2.5, 4.5])
    f64p = ctypes.POINTER(ctypes.c_double)
    for l, want in [(96, 2.5), (16, 1.25), (512, 9.0)]:
        assert abs(lib.pv_cost_model(ptp, ys.ctypes.data_as(f64p), 4, 0.5, l) - want) < 1e-12
    cost = np.array([3.0, 1.0, 2.0])
    idle = np.ones(3)
    order = np.zeros(3, dtype=np.int32)
    assert lib.pv_retention_order(cost.ctypes.data_as(f64p), idle.ctypes.data_as(f64p), 3,
                                  order.ctypes.data_as(i32p)) == 0 and order.tolist() == [1, 2, 0]
    tab = np.zeros((50, 64), dtype=np.float32)
    assert lib.pv_rope_table(10000.0, 64, 50, tab.ctypes.data_as(ctypes.POINTER(ctypes.c_float))) == 0
    print("host plan under sanitizers: ok", flush=True)


if __name__ == "__main__":
    check_oracle(sys.argv[1])
    check_plan(sys.argv[2])
