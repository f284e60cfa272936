"""Parity of the 256-row matrix-core kernel (long multi-token units) with the CPU oracle.

The plan sends the full 256-row tiles of a (request, KV head) unit to that kernel when the unit
has at least 256 rows and at least 2048 keys (head size 128); the rest of the unit keeps the
128-row kernel.  Every case here checks that such items exist, then compares the whole output
with the oracle element by element (5e-3 fp16 / 2e-2 bf16) and the pools bit for bit.
"""
import numpy as np
import pytest

import helpers as H
from paper_2312_05516_amd import workloads as wl
from test_gpu_parity import check_case

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _route_long_units_to_the_256_row_kernel(monkeypatch):
    monkeypatch.setenv("PV_TILE_MIN_KEYS", "2048")


def _tile_items(b):
    from paper_2312_05516_amd import binding as pv
    desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
    plan = pv.plan_create(desc, b.num_q_heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
    items = [pv.plan_work_item(plan, 3, i) for i in range(pv.plan_num_work_items(plan, 3))]
    rest = pv.plan_num_work_items(plan, 0) + pv.plan_num_work_items(plan, 1)
    plan.destroy()
    return items, rest


SHAPES = [
    # ctx_lens, q_lens, Hq, Hkv, dtype: what the case is for
    ([2100], [40], 8, 1, "bf16"),            # one tile + a 64-row rest, KV range split into parts
    ([2003, 2500], [300, 77], 4, 4, "f16"),  # G = 1: a tile spans 256 tokens, long masked tail
    ([0], [2100], 2, 2, "f16"),              # prefill from an empty cache: mostly boundary blocks
    ([4096 - 64, 3000, 17], [64, 33, 5], 16, 2, "bf16"),  # ends on a page boundary; mixed batch
    ([5000, 2049, 2047], [32, 32, 32], 8, 1, "bf16"),     # exactly one tile each / just below
    ([9000], [100], 8, 2, "f16"),            # odd tail rows, two KV heads
]


@pytest.mark.parametrize("shape", SHAPES, ids=[f"t{i}" for i in range(len(SHAPES))])
def test_tile256_shapes(oracle, shape):
    ctx, qn, hq, hkv, dt = shape
    b = wl.custom(ctx, qn, num_q_heads=hq, num_kv_heads=hkv, head_dim=128, dtype=dt, seed=57)
    items, _ = _tile_items(b)
    assert items and all(int(it[3]) == 256 for it in items)
    check_case(oracle, H.make_case(b, fill="nan"))


def test_tile256_unsplit_items_and_short_ranges(oracle, monkeypatch):
    """With the length threshold lowered the kernel also gets items of one to a few 32-key blocks
    (fewer than its copy pipeline is deep), and with a high split target... none are cut."""
    monkeypatch.setenv("PV_TILE_MIN_KEYS", "1")
    for ctx, qn, hq, hkv in [([0, 5, 31, 100], [32, 32, 64, 40], 8, 1),
                             ([0, 150], [256, 300], 2, 2)]:
        b = wl.custom(ctx, qn, num_q_heads=hq, num_kv_heads=hkv, head_dim=128, dtype="bf16", seed=61)
        items, _ = _tile_items(b)
        assert items and min(int(it[5] - it[4]) for it in items) <= 256
        check_case(oracle, H.make_case(b, fill="nan"))


def test_tile256_many_items_without_split(oracle, monkeypatch):
    """Enough items that the plan leaves them whole (no partial results, direct output)."""
    monkeypatch.setenv("PV_SPLIT_TARGET", "4")
    b = wl.custom([2300, 2100], [64, 32], num_q_heads=16, num_kv_heads=2, head_dim=128,
                  dtype="bf16", seed=63)
    items, _ = _tile_items(b)
    assert len(items) == 2 * (2 + 1) and all(int(it[7]) == 1 for it in items)
    check_case(oracle, H.make_case(b, fill="nan"))


def test_tile256_large_scale_and_page_permutation(oracle):
    """Scores far apart (scale 3) exercise the reference-maximum updates; permuting the physical
    pages must not change a single output bit."""
    b = wl.custom([2200], [48], num_q_heads=8, num_kv_heads=1, head_dim=128, dtype="f16", seed=67)
    case = H.make_case(b, fill="nan")
    got, _, _ = H.gpu_run(case, scale=3.0)
    from test_gpu_parity import oracle_out
    want = oracle_out(oracle, case, scale=3.0)
    err = np.abs(H.bits_to_f64(got, b.dtype) - want).max()
    print(f"scale 3: max abs err {err:.3e}", flush=True)
    assert err <= H.TOL[b.dtype]
    rng = np.random.default_rng(5)
    perm = rng.permutation(b.num_pages)  # new physical place of each page
    elems = b.num_kv_heads * b.page_size * b.head_dim
    kp = np.empty_like(case.k_pool0)
    vp = np.empty_like(case.v_pool0)
    kp.reshape(b.num_pages, elems)[perm] = case.k_pool0.reshape(b.num_pages, elems)
    vp.reshape(b.num_pages, elems)[perm] = case.v_pool0.reshape(b.num_pages, elems)
    table = np.where(b.page_table >= 0, perm[np.maximum(b.page_table, 0)], -1).astype(np.int32)
    base, _, _ = H.gpu_run(case)
    moved, _, _ = H.gpu_run(case, page_table=table, pools=(kp, vp))
    assert np.array_equal(base, moved)


@pytest.mark.parametrize("scale", [-0.125, 0.0, 0.2, 0.5])
def test_tile256_scales_on_both_sides_of_the_prescaling_limit(oracle, scale):
    """|scale*log2(e)| <= 0.25 takes the instantiation with pre-multiplied queries (negative
    scales included: the sign travels with the queries; zero gives uniform weights), larger scales
    the one that scales in fp32."""
    b = wl.custom([2100, 2300], [40, 32], num_q_heads=8, num_kv_heads=1, head_dim=128,
                  dtype="bf16", seed=71, value_std=0.5)
    items, _ = _tile_items(b)
    assert items
    case = H.make_case(b, fill="nan")
    got, _, _ = H.gpu_run(case, scale=scale)
    from test_gpu_parity import oracle_out
    want = oracle_out(oracle, case, scale=scale)
    got = H.bits_to_f64(got, b.dtype)
    assert np.isfinite(got).all()
    err = np.abs(got - want).max()
    print(f"scale {scale}: max abs err {err:.3e}", flush=True)
    assert err <= H.TOL[b.dtype]


def test_tile256_range_longer_than_the_page_id_staging_is_cut(oracle, monkeypatch):
    """An item's page ids are staged in LDS, 8192 at most: a KV range of 140 K keys (8750 pages)
    is cut in two even when the plan would otherwise leave it whole (split target 1), and the
    parts are merged."""
    monkeypatch.setenv("PV_SPLIT_TARGET", "1")
    b = wl.custom([140000 - 32], [32], num_q_heads=8, num_kv_heads=1, head_dim=128, dtype="bf16",
                  seed=73)
    items, _ = _tile_items(b)
    assert items and all(int(it[5] - it[4]) <= 8192 * 16 for it in items)
    assert len(items) == 2 and all(int(it[7]) == 2 for it in items)
    check_case(oracle, H.make_case(b, fill="nan"))


def test_tile256_batch_of_medium_ranges_without_a_limit_set_by_hand(oracle, monkeypatch):
    """With no limit in the environment, a batch whose work is nearly all in long multi-token
    units goes to the 256-row kernel from 1536 keys up (here with the list length that counts as
    long enough lowered to the size of the test)."""
    monkeypatch.delenv("PV_TILE_MIN_KEYS")
    monkeypatch.setenv("PV_SPLIT_TARGET", "16")
    b = wl.custom([1500, 1700, 1600, 1900, 30], [64, 64, 96, 64, 1], num_q_heads=16,
                  num_kv_heads=2, head_dim=128, dtype="bf16", seed=79)
    items, rest = _tile_items(b)
    assert len(items) == 2 * (2 + 2 + 3 + 2) and rest > 0
    check_case(oracle, H.make_case(b, fill="nan"))


@pytest.mark.parametrize("idx", range(10))
def test_tile256_random_batches(oracle, idx, monkeypatch):
    """Seeded random batches with the length threshold of the 256-row kernel at its lowest, so
    that every unit of at least 256 rows has tiles there: ranges of a few blocks up to a hundred,
    cut and whole, causal boundaries at every offset inside a block, rests for the other kernels,
    group sizes 1 to 16, both dtypes, small and large scales."""
    monkeypatch.setenv("PV_TILE_MIN_KEYS", "1")
    rng = np.random.default_rng(900 + idx)
    group = int(rng.choice([1, 2, 4, 8, 16]))
    hkv = int(rng.choice([1, 2]))
    reqs = int(rng.integers(1, 5))
    ctx = [int(rng.integers(0, 3200)) for _ in range(reqs)]
    # at least one request with 256 rows or more, the others anything from a generation step up
    qn = [int(rng.integers(1, max(2, 700 // group))) for _ in range(reqs)]
    qn[0] = int(rng.integers((256 + group - 1) // group, (256 + group - 1) // group + 600 // group + 1))
    if idx % 3 == 0:
        monkeypatch.setenv("PV_SPLIT_TARGET", "4")  # whole ranges
    b = wl.custom(ctx, qn, num_q_heads=group * hkv, num_kv_heads=hkv, head_dim=128,
                  dtype="bf16" if idx % 2 else "f16", seed=910 + idx,
                  value_std=0.5 if idx % 4 == 1 else 1.0)
    items, _ = _tile_items(b)
    assert items
    print(f"random {idx}: G={group} Hkv={hkv} ctx={ctx} q={qn}: {len(items)} items of the 256-row "
          f"kernel, ranges {min(int(i[5] - i[4]) for i in items)}..{max(int(i[5] - i[4]) for i in items)}",
          flush=True)
    scale = None if idx % 4 else 0.3  # every fourth: the instantiation that scales in fp32
    case = H.make_case(b, fill="nan")
    if scale is None:
        check_case(oracle, case)
    else:
        got, _, _ = H.gpu_run(case, scale=scale)
        from test_gpu_parity import oracle_out
        want = oracle_out(oracle, case, scale=scale)
        err = np.abs(H.bits_to_f64(got, b.dtype) - want).max()
        print(f"  scale {scale}: max abs err {err:.3e}", flush=True)
        assert err <= H.TOL[b.dtype]
