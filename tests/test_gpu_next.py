"""GPU tests of the two adjacent rows that otherwise only exist as bench modes.

* The kernel figure of the paper (Section 6.4: batch of requests with a few query tokens each over
  a context sweep, KV at non-contiguous places) restated with this library's own variants:
  the paged call, the same call on a contiguous copy of the pages made with the library's page
  gather/scatter ("copy-out"), and one call per query token ("multi-round").  All three must give
  the oracle's result, and the copy-out variant the paged call's result bit for bit.
* The recomputation-cost profile of the eviction policy (Section 4.3.1): the attention time of a
  32-token chunk measured with the library at power-of-two context sizes, fed to pv_cost_model
  (against the oracle's interpolation on the same numbers) and pv_retention_order (against the
  oracle's order).
"""
import numpy as np
import pytest

import helpers as H
from paper_2312_05516_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _attend(pv, torch, desc, b, q, kp, vp, table_h, ctx_lens=None, q_lens=None):
    ctx_lens = b.ctx_lens if ctx_lens is None else ctx_lens
    q_lens = b.q_lens if q_lens is None else q_lens
    table = torch.from_numpy(np.ascontiguousarray(table_h, dtype=np.int32)).cuda()
    plan = pv.plan_create(desc, b.num_q_heads, ctx_lens, q_lens, b.max_pages_per_req)
    lists = torch.empty(pv.plan_device_bytes(plan), dtype=torch.uint8, device="cuda")
    pv.plan_upload_to(plan, lists)
    ws = torch.empty(max(pv.plan_workspace_bytes(plan), 256), dtype=torch.uint8, device="cuda")
    out = torch.full((int(np.sum(q_lens)), b.num_q_heads, b.head_dim), float("nan"), dtype=q.dtype,
                     device="cuda")
    pv.multi_token_paged_attn_planned(plan, q, kp, vp, table, b.scale, out, ws)
    torch.cuda.synchronize()
    plan.destroy()
    return out


@pytest.mark.parametrize("ctx", [40, 700, 3000])
def test_kernel_figure_variants_agree_with_the_oracle(oracle, ctx):
    import torch
    from paper_2312_05516_amd import binding as pv
    R, n = 6, 8
    b = wl.custom([ctx + 3 * r for r in range(R)], [n] * R, num_q_heads=4, num_kv_heads=4,
                  head_dim=128, dtype="f16", seed=81 + ctx)
    case = H.make_case(b, fill="nan")
    print(f"kernel-figure shape: {R} requests x {n} query tokens over ~{ctx} cached, "
          f"4 heads x 128, fp16, {b.num_pages} pages", flush=True)
    desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
    kp, vp = H.to_dev_bits(case.k_pool1, b.dtype), H.to_dev_bits(case.v_pool1, b.dtype)
    q = H.to_dev_bits(case.q, b.dtype)
    want, _ = oracle.attn(H.pool_tuple(b), b.num_q_heads, case.q, case.k_pool1, case.v_pool1,
                          b.page_table, b.ctx_lens, b.q_lens, b.q_start, b.scale)
    tol = H.TOL[b.dtype]

    # paged: pages at random places
    paged = _attend(pv, torch, desc, b, q, kp, vp, b.page_table)
    err = np.abs(H.bits_to_f64(H.from_dev_bits(paged), b.dtype) - want).max()
    print(f"  paged       max abs err {err:.3e}", flush=True)
    assert err <= tol

    # copy-out: gather the used pages, scatter them to consecutive pages of a second pool pair,
    # then the same call with the identity table
    used = b.page_table[b.page_table >= 0].astype(np.int32)
    ids = torch.from_numpy(used).cuda()
    page_elems = b.num_kv_heads * b.page_size * b.head_dim
    staging = torch.empty((len(used), 2, page_elems), dtype=torch.int16, device="cuda")
    pv.pages_gather(desc, kp, vp, ids, len(used), staging)
    kc = torch.full_like(kp, float("nan"))
    vc = torch.full_like(vp, float("nan"))
    home = torch.arange(len(used), dtype=torch.int32, device="cuda")
    pv.pages_scatter(desc, staging, home, len(used), kc, vc)
    ident = np.full_like(b.page_table, -1)
    at = 0
    for r in range(R):
        npg = int((b.page_table[r] >= 0).sum())
        ident[r, :npg] = np.arange(at, at + npg)
        at += npg
    copied = _attend(pv, torch, desc, b, q, kc, vc, ident)
    assert np.array_equal(H.from_dev_bits(copied), H.from_dev_bits(paged)), \
        "contiguous copy gives other bits than the paged call"

    # multi-round: one call per query token; round i sees the first i+1 new tokens
    rounds = np.zeros_like(H.from_dev_bits(paged))
    for i in range(n):
        qi = q[i::n].contiguous()
        oi = _attend(pv, torch, desc, b, qi, kp, vp, b.page_table, ctx_lens=b.ctx_lens + i,
                     q_lens=np.ones_like(b.q_lens))
        rounds[i::n] = H.from_dev_bits(oi)
    err = np.abs(H.bits_to_f64(rounds, b.dtype) - want).max()
    print(f"  multi-round max abs err {err:.3e}", flush=True)
    assert err <= tol
    # against the paged call: both are within tol of the oracle; they take different kernels
    # (eight rows per item vs one), so bits may differ, values not by more than rounding
    assert np.abs(H.bits_to_f64(rounds, b.dtype)
                  - H.bits_to_f64(H.from_dev_bits(paged), b.dtype)).max() <= tol


def _chunk_cost_ms(pv, torch, l: int, heads: int = 8, reps: int = 20) -> float:
    """Attention time of one 32-token chunk whose context, itself included, is l tokens."""
    b = wl.custom([l - 32], [32], num_q_heads=heads, num_kv_heads=heads, head_dim=128,
                  dtype="f16", seed=l, name=f"chunk_l{l}")
    page_elems = heads * 16 * 128
    kp = wl.random_values((b.num_pages, page_elems), b.dtype, 1, 1.0, "cuda")
    vp = wl.random_values((b.num_pages, page_elems), b.dtype, 2, 1.0, "cuda")
    q = wl.random_values((32, heads, 128), b.dtype, 3, 1.0, "cuda")
    out = torch.empty_like(q)
    table = torch.from_numpy(b.page_table).cuda()
    desc = pv.pool_desc(b.num_pages, heads, 128, b.dtype)
    plan = pv.plan_create(desc, heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
    pv.plan_upload(plan)
    ws = torch.empty(max(pv.plan_workspace_bytes(plan), 256), dtype=torch.uint8, device="cuda")
    for _ in range(3):
        pv.multi_token_paged_attn_planned(plan, q, kp, vp, table, b.scale, out, ws)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(reps):
        pv.multi_token_paged_attn_planned(plan, q, kp, vp, table, b.scale, out, ws)
    stop.record()
    torch.cuda.synchronize()
    plan.destroy()
    return start.elapsed_time(stop) / reps


def test_cost_profile_measured_with_the_kernel_feeds_the_cost_model(oracle):
    import torch
    from paper_2312_05516_amd import binding as pv
    points = [2048, 4096, 8192, 16384, 32768]
    costs = [_chunk_cost_ms(pv, torch, l) for l in points]
    print("Cost_attention(l) of a 32-token chunk, ms: "
          + ", ".join(f"l={l}: {c:.4f}" for l, c in zip(points, costs)), flush=True)
    assert all(np.isfinite(c) and c > 0 for c in costs)
    # the cost grows with the context once the call is no longer launch-bound: each doubling of l
    # may not make the call cheaper (10 % slack for timer noise), and 16 times the context costs
    # clearly more
    for a, c in zip(costs, costs[1:]):
        assert c >= 0.9 * a, (points, costs)
    assert costs[-1] > 1.5 * costs[0], (points, costs)
    # the library's interpolation of this profile against the oracle's, on and between the points
    # and beyond both ends
    c_other = 0.05
    for l in [32, 1000, 2048, 3000, 4096, 6000, 12000, 16384, 24000, 32768, 50000]:
        got = pv.cost_model(points, costs, c_other, l)
        want = oracle.cost(points, costs, c_other, l)
        assert np.isclose(got, want, rtol=1e-12, atol=0), (l, got, want)
    at_points = [pv.cost_model(points, costs, 0.0, l) for l in points]
    assert np.allclose(at_points, costs, rtol=1e-12)
    # retention order of 300 chunks with these costs: ascending Cost(l) / T, ties keep the index
    rng = np.random.default_rng(11)
    ls = rng.integers(32, 40000, size=300)
    chunk_cost = np.array([pv.cost_model(points, costs, c_other, int(l)) for l in ls])
    idle = rng.uniform(1.0, 600.0, size=300)
    idle[50:60] = idle[50]
    chunk_cost[50:60] = chunk_cost[50]
    order = pv.retention_order(chunk_cost, idle)
    assert np.array_equal(order, oracle.retention_order(chunk_cost, idle))
    v = chunk_cost[order] / idle[order]
    assert np.all(np.diff(v) >= 0)


def test_cost_model_and_retention_order_match_the_oracle_on_fixed_numbers(oracle):
    """The host-only parity check of the two entry points, here so that it also runs where the
    GPU tests run."""
    from paper_2312_05516_amd import binding as pv
    pts = [32, 64, 128, 256, 512, 1024, 2048]
    rng = np.random.default_rng(5)
    ys = np.cumsum(rng.uniform(0.1, 2.0, size=len(pts)))
    for l in [1, 16, 32, 33, 64, 100, 128, 1000, 1024, 2047, 2048, 5000]:
        assert np.isclose(pv.cost_model(pts, ys, 0.7, l), oracle.cost(pts, ys, 0.7, l),
                          rtol=1e-13, atol=0)
    c = rng.uniform(1, 10, size=200)
    t = rng.uniform(1, 600, size=200)
    assert np.array_equal(pv.retention_order(c, t), oracle.retention_order(c, t))
