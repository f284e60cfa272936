"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what the header
declares, and its pure-host entry points (plan construction, validation, pool offsets) behave."""
import os
import re

import numpy as np
import pytest

from paper_2312_05516_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pv():
    from paper_2312_05516_amd import binding
    return binding


def test_every_declared_symbol_is_exported(pv):
    import ctypes
    text = open(os.path.join(ROOT, "include", "pv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(pv_[a-z0-9_]+)\s*\(", text))
    assert declared == set(pv.EXPORTS), declared ^ set(pv.EXPORTS)
    lib = ctypes.CDLL(pv.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(pv):
    names = {pv.status_string(i) for i in range(6)}
    assert len(names) == 6 and "ok" in names


def test_pool_bytes_and_offsets(pv):
    desc = pv.pool_desc(5, 3, 64, "f16")
    assert pv.pool_bytes(desc) == 5 * 3 * 16 * 64 * 2
    assert pv.pool_bytes(pv.pool_desc(5, 3, 64, "f16", page_size=32)) == 0
    ids = np.arange(5 * 3 * 16 * 64)
    kv = ids.reshape(5, 3, 8, 16, 8)
    vv = ids.reshape(5, 3, 2, 64, 8)
    rng = np.random.default_rng(0)
    for _ in range(300):
        p, h, s, d = rng.integers(5), rng.integers(3), rng.integers(16), rng.integers(64)
        assert pv.pool_k_offset(desc, p, h, s, d) == kv[p, h, d // 8, s, d % 8]
        assert pv.pool_v_offset(desc, p, h, s, d) == vv[p, h, s // 8, d, s % 8]
    assert pv.pool_k_offset(desc, 5, 0, 0, 0) == -1
    assert pv.pool_v_offset(desc, 0, 0, 16, 0) == -1


def _items(pv, plan, kind):
    return [pv.plan_work_item(plan, kind, i) for i in range(pv.plan_num_work_items(plan, kind))]


@pytest.mark.parametrize("name", ["tiny", "mha13b", "gqa70b", "decode_heavy", "long_history"])
def test_plan_covers_every_row_exactly_once(pv, name, monkeypatch):
    monkeypatch.setenv("PV_TILE_MIN_KEYS", "2048")
    b = wl.CONFIGS[name]()
    desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
    plan = pv.plan_create(desc, b.num_q_heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
    assert pv.plan_total_q(plan) == b.total_q
    assert np.array_equal(pv.plan_q_start(plan), b.q_start)
    G = b.num_q_heads // b.num_kv_heads
    # for every (req, kv head, row): the KV parts that contain it must tile [0, causal limit)
    cover = {}
    for kind in (0, 1, 3):
        for it in _items(pv, plan, kind):
            req, hk, rb, rc, k0, k1, si, sc = (int(x) for x in it)
            assert 0 < rc <= {0: 16, 1: 128, 3: 256}[kind]
            if kind == 3:  # the 256-row kernel only takes full tiles of long units, head size 128
                assert rc == 256 and rb % 256 == 0 and b.head_dim == 128
                assert b.ctx_lens[req] + b.q_lens[req] >= 2048
            assert k0 % 32 == 0 and k0 < k1
            last_tok = (rb + rc - 1) // G
            assert k1 <= b.ctx_lens[req] + last_tok + 1
            for row in range(rb, rb + rc):
                cover.setdefault((req, hk, row), []).append((k0, k1, si, sc))
    n_rows = 0
    for r in range(b.num_reqs):
        for hk in range(b.num_kv_heads):
            for row in range(int(b.q_lens[r]) * G):
                parts = sorted(cover[(r, hk, row)])
                n_rows += 1
                assert parts[0][0] == 0
                for a, c in zip(parts, parts[1:]):
                    assert a[1] == c[0]
                # the union must reach at least this row's own causal limit
                assert parts[-1][1] >= b.ctx_lens[r] + row // G + 1
                assert [p[2] for p in parts] == list(range(len(parts)))
                assert all(p[3] == len(parts) for p in parts)
    assert n_rows == len(cover)
    # split bookkeeping: workspace is exactly the partial rows
    slots = sum(int(it[3]) * int(it[7]) for it in _items(pv, plan, 2))
    assert pv.plan_workspace_bytes(plan) == slots * (b.head_dim + 2) * 4
    plan.destroy()


def test_plan_orders_items_longest_first_per_xcd(pv, monkeypatch):
    """Workgroup i goes to XCD i % 8: every XCD sees its items longest first, and the tiles of one
    (request, KV head) sit on one XCD."""
    b = wl.decode_heavy()
    desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
    plan = pv.plan_create(desc, b.num_q_heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
    lens = [int(it[5] - it[4]) for it in _items(pv, plan, 0)]
    assert len(lens) == 256 * 40
    for x in range(8):
        q = lens[x::8]
        assert q == sorted(q, reverse=True)
    plan.destroy()
    b = wl.long_history()
    monkeypatch.setenv("PV_TILE_MIN_KEYS", "2048")
    desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
    plan = pv.plan_create(desc, b.num_q_heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
    assert pv.plan_num_work_items(plan, 1) == 0
    items = _items(pv, plan, 3)
    assert len(items) == 8 * 8 * 16
    home = {}
    for i, it in enumerate(items):
        home.setdefault((int(it[0]), int(it[1])), set()).add(i % 8)
    assert all(len(v) == 1 for v in home.values())
    plan.destroy()


def test_plan_splits_long_single_request(pv):
    desc = pv.pool_desc(4096, 8, 128, "bf16")
    plan = pv.plan_create(desc, 64, [50000], [1], 4096)
    items = _items(pv, plan, 0)
    assert len(items) > 8 and all(int(it[7]) > 1 for it in items)
    assert pv.plan_num_work_items(plan, 2) == 8
    assert pv.plan_workspace_bytes(plan) > 0
    plan.destroy()


def test_plan_sends_small_units_to_the_matrix_core_kernel_unless_they_are_many(pv):
    """A mixed batch is one attention launch as long as its small units (generation steps) sum to at
    most 90 K steps of 32 keys over all KV heads; beyond that they keep the bandwidth-oriented
    kernel.  A batch without prompt work never uses the matrix-core kernel."""
    desc = pv.pool_desc(1 << 17, 4, 128, "f16")
    # a 200-token prompt next to two generation steps: 2 x 32 steps x 4 heads
    plan = pv.plan_create(desc, 4, [1000, 1000, 1000], [200, 1, 1], 128)
    assert pv.plan_num_work_items(plan, 0) == 0
    rows = sorted(int(it[3]) for it in _items(pv, plan, 1))
    assert rows[0] == 1 and rows[-1] == 128
    plan.destroy()
    # the same prompt next to 100 generation steps over 8000 cached tokens: 100 K steps
    plan = pv.plan_create(desc, 4, [1000] + [8000] * 100, [200] + [1] * 100, 512)
    assert pv.plan_num_work_items(plan, 0) > 0 and pv.plan_num_work_items(plan, 1) > 0
    assert all(int(it[3]) > 32 for it in _items(pv, plan, 1))
    plan.destroy()
    # 80 of them: 80 K steps, still one launch
    plan = pv.plan_create(desc, 4, [1000] + [8000] * 80, [200] + [1] * 80, 512)
    assert pv.plan_num_work_items(plan, 0) == 0
    plan.destroy()
    plan = pv.plan_create(desc, 4, [8000] * 3, [1] * 3, 512)
    assert pv.plan_num_work_items(plan, 1) == 0
    plan.destroy()


def test_plan_cuts_outliers_of_a_long_list(pv):
    """More than split_target items, one of them far longer than the rest: only that one is cut."""
    desc = pv.pool_desc(1 << 16, 8, 128, "bf16")
    ctx = [300] * 200 + [60000]
    plan = pv.plan_create(desc, 8, ctx, [1] * 201, 4096)
    items = _items(pv, plan, 0)
    assert len(items) > 201 * 8
    for it in items:
        assert (int(it[7]) > 1) == (int(it[0]) == 200)
    longest = max(int(it[5] - it[4]) for it in items)
    assert longest < 60000 // 4
    assert pv.plan_num_work_items(plan, 2) == 8
    plan.destroy()


def test_rope_table_matches_the_definition(pv, oracle):
    """The library's host table generator against the oracle's (independent code, same formula):
    equal up to one unit in the last place of a float."""
    for base, D, n in [(10000.0, 128, 300), (500000.0, 64, 77)]:
        got = pv.rope_table(base, D, n)
        want = oracle.rope_table(base, D, n)
        assert got.shape == (n, D)
        assert np.abs(got.view(np.int32).astype(np.int64) - want.view(np.int32)).max() <= 1
    assert pv.rope_table(10000.0, 64, 0).shape == (0, 64)
    for bad in [(0.0, 64, 4), (-2.0, 64, 4), (10000.0, 63, 4)]:
        with pytest.raises(pv.PvError) as e:
            pv.rope_table(*bad)
        assert e.value.status == 1


def test_plan_rejects_bad_arguments(pv):
    good = pv.pool_desc(64, 4, 64, "f16")
    with pytest.raises(pv.PvError) as e:
        pv.plan_create(pv.pool_desc(64, 4, 96, "f16"), 4, [1], [1], 4)
    assert e.value.status == 2
    with pytest.raises(pv.PvError) as e:
        pv.plan_create(pv.pool_desc(64, 4, 64, "f16", page_size=32), 4, [1], [1], 4)
    assert e.value.status == 2
    with pytest.raises(pv.PvError) as e:
        pv.plan_create(good, 6, [1], [1], 4)  # 6 query heads over 4 KV heads
    assert e.value.status == 1
    with pytest.raises(pv.PvError) as e:
        pv.plan_create(good, 4, [-1], [1], 4)
    assert e.value.status == 1
    with pytest.raises(pv.PvError) as e:
        pv.plan_create(good, 4, [60], [5], 4)  # 65 tokens need 5 pages, the table has 4
    assert e.value.status == 3
    # empty batches and empty requests are fine
    p = pv.plan_create(good, 4, [], [], 4)
    assert pv.plan_total_q(p) == 0 and pv.plan_num_work_items(p, 0) == 0
    p.destroy()
    p = pv.plan_create(good, 4, [10, 3], [0, 2], 4)
    assert pv.plan_total_q(p) == 2 and pv.plan_q_start(p).tolist() == [0, 0]
    p.destroy()


def test_page_table_check(pv):
    b = wl.custom([20, 5], [3, 4], num_q_heads=4, num_kv_heads=2, head_dim=64, seed=3)
    desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
    plan = pv.plan_create(desc, 4, b.ctx_lens, b.q_lens, b.max_pages_per_req)
    assert pv.plan_check_page_table(plan, b.page_table) == 0
    bad = b.page_table.copy()
    bad[0, 1] = b.num_pages
    assert pv.plan_check_page_table(plan, bad) == 3
    bad = b.page_table.copy()
    bad[1, 0] = -1
    assert pv.plan_check_page_table(plan, bad) == 3
    shared = b.page_table.copy()
    shared[1, 0] = shared[0, 1]  # request 1 would append into request 0's second page
    assert pv.plan_check_page_table(plan, shared, check_append_unique=False) == 0
    assert pv.plan_check_page_table(plan, shared, check_append_unique=True) == 1
    plan.destroy()


def test_planned_launch_refuses_a_plan_whose_lists_are_on_no_device(pv):
    """A *_planned launch never allocates or copies: without pv_plan_upload / pv_plan_upload_to it
    returns an error before it touches the GPU (so this runs without one)."""
    desc = pv.pool_desc(64, 4, 64, "f16")
    plan = pv.plan_create(desc, 4, [10, 3], [2, 1], 4)
    assert pv.plan_device_bytes(plan) >= 256 and pv.plan_device_bytes(plan) % 256 == 0
    assert not pv.plan_owns_device_memory(plan)
    fake = 0x1000  # aligned, never dereferenced
    with pytest.raises(pv.PvError) as e:
        pv.multi_token_paged_attn_planned(plan, fake, fake, fake, fake, 0.125, fake, None, stream=0)
    assert e.value.status == 1
    with pytest.raises(pv.PvError) as e:
        pv.kv_append_planned(plan, fake, fake, fake, fake, fake, stream=0)
    assert e.value.status == 1
    with pytest.raises(pv.PvError) as e:  # misaligned q
        pv.multi_token_paged_attn_planned(plan, fake + 2, fake, fake, fake, 0.125, fake, None, stream=0)
    assert e.value.status == 1
    plan.destroy()


def test_workspace_bound_covers_plans(pv):
    for name in ["tiny", "mha13b", "gqa70b", "decode_heavy"]:
        b = wl.CONFIGS[name]()
        desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
        plan = pv.plan_create(desc, b.num_q_heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
        bound = pv.attn_workspace_bytes(desc, b.num_q_heads, b.num_reqs, b.total_q,
                                        int(b.kv_lens.max()))
        assert bound >= (pv.plan_workspace_bytes(plan) + 255) // 256 * 256 + pv.plan_device_bytes(plan)
        plan.destroy()
    # shapes that make the plan split: one long request alone, an outlier in a long list, a
    # mixed batch routed to one kernel, seeded random mixes
    rng = np.random.default_rng(23)
    shapes = [([50000], [1], 64, 8), ([300] * 200 + [60000], [1] * 201, 8, 8),
              ([40000, 100, 7000], [200, 1, 1], 8, 2), ([20000], [64], 2, 1)]
    for _ in range(20):
        n = int(rng.integers(1, 40))
        shapes.append((rng.integers(0, 30000, n).tolist(),
                       rng.choice([0, 1, 1, 1, 5, 40, 300], n).tolist(),
                       int(rng.choice([8, 16])), int(rng.choice([1, 2, 8]))))
    for ctx, qn, hq, hkv in shapes:
        desc = pv.pool_desc(1 << 16, hkv, 128, "bf16")
        plan = pv.plan_create(desc, hq, ctx, qn, 4096)
        kv_max = max([c + q for c, q in zip(ctx, qn)] + [0])
        bound = pv.attn_workspace_bytes(desc, hq, len(ctx), int(sum(qn)), kv_max)
        need = (pv.plan_workspace_bytes(plan) + 255) // 256 * 256 + pv.plan_device_bytes(plan)
        assert bound >= need, (ctx[:4], qn[:4], hq, hkv)
        plan.destroy()


def test_cost_model_and_retention_order_match_the_oracle(pv, oracle):
    """Pure host entry points: parity with the oracle is exact for the order, and to rounding for
    the interpolation."""
    pts = [32, 64, 128, 256, 512, 1024, 2048]
    rng = np.random.default_rng(5)
    ys = np.cumsum(rng.uniform(0.1, 2.0, size=len(pts)))
    for l in [1, 16, 32, 33, 64, 100, 128, 1000, 1024, 2047, 2048, 5000]:
        assert np.isclose(pv.cost_model(pts, ys, 0.7, l), oracle.cost(pts, ys, 0.7, l),
                          rtol=1e-13, atol=0)
    assert pv.cost_model([], [], 0.7, 5) == 0.7 and pv.cost_model([8], [2.0], 0.5, 99) == 2.5
    c = rng.uniform(1, 10, size=200)
    t = rng.uniform(1, 600, size=200)
    assert np.array_equal(pv.retention_order(c, t), oracle.retention_order(c, t))
    c[10:20] = c[10]
    t[10:20] = t[10]  # ties
    assert np.array_equal(pv.retention_order(c, t), oracle.retention_order(c, t))
    with pytest.raises(pv.PvError):
        pv.retention_order([1.0, 2.0], [3.0, 0.0])
    assert len(pv.retention_order([], [])) == 0


def test_plan_sends_a_batch_of_long_multi_token_units_to_the_256_row_kernel(pv, monkeypatch):
    """Units of at least 256 rows go to the 256-row kernel from 8192 keys up; from 1536 keys up
    when nearly all of the batch qualifies and the plan has no reason to cut the items.  A limit
    set by hand switches the batch rule off."""
    from paper_2312_05516_amd import workloads as wl
    monkeypatch.delenv("PV_TILE_MIN_KEYS", raising=False)
    kw = dict(num_q_heads=64, num_kv_heads=8, head_dim=128, dtype="bf16", seed=5)

    def counts(b):
        desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
        plan = pv.plan_create(desc, b.num_q_heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
        n = [pv.plan_num_work_items(plan, k) for k in (0, 1, 2, 3)]
        plan.destroy()
        return n

    uniform = wl.custom([1024] * 16, [512] * 16, **kw)          # 1536 keys, 16 tiles x 8 heads each
    assert counts(uniform) == [0, 0, 0, 2048]
    short = wl.custom([600] * 16, [512] * 16, **kw)              # 1112 keys: below the batch limit
    assert counts(short)[3] == 0
    few = wl.custom([2048] * 4, [512] * 4, **kw)                 # 512 items: the plan would cut them
    assert counts(few)[3] == 0
    mixed = wl.custom([2048] * 16 + [3000] * 40, [512] * 16 + [1] * 40, **kw)
    assert counts(mixed)[3] == 2048 and counts(mixed)[1] > 0     # a few generation steps: still
    half = wl.custom([2048] * 16 + [30000] * 40, [512] * 16 + [16] * 40, **kw)
    assert counts(half)[3] == 0                                  # most pairs elsewhere: not
    outlier = wl.custom([1024] * 15 + [20000], [512] * 16, **kw)
    n = counts(outlier)
    assert n[3] > 0 and n[1] > 0                                 # only the long unit qualifies
    for name in ("mha13b", "gqa70b"):
        assert counts(wl.CONFIGS[name]())[3] == 0
    assert counts(wl.CONFIGS["long_history"]())[3] == 1024
    monkeypatch.setenv("PV_TILE_MIN_KEYS", "8192")
    assert counts(uniform)[3] == 0
