"""The launch that allocates nothing (static device scratch array) against the planned launch.

Two calls in a row through the C ABI, the second with a smaller batch, each compared bit for bit
with pv_multi_token_paged_attn_planned on the same inputs (same kernels, same work lists: the
outputs must be identical) and, for the first, with the oracle within the attention tolerance.
Batches are chosen so that the KV ranges are split: the partial results then go through the
scratch array too, not only the work lists.
"""
import numpy as np
import pytest

import helpers as H
from paper_2312_05516_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _run_both(case):
    import torch
    from paper_2312_05516_amd import binding as pv
    b = case.batch
    desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
    kp, vp = H.to_dev_bits(case.k_pool1, b.dtype), H.to_dev_bits(case.v_pool1, b.dtype)
    table = torch.from_numpy(np.ascontiguousarray(b.page_table, dtype=np.int32)).cuda()
    q = H.to_dev_bits(case.q, b.dtype)
    plan = pv.plan_create(desc, b.num_q_heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
    need = (pv.plan_device_bytes(plan) + 255) // 256 * 256 + pv.plan_workspace_bytes(plan)
    assert need <= pv.static_scratch_bytes()
    out_a = torch.full((b.total_q, b.num_q_heads, b.head_dim), float("nan"),
                       dtype=q.dtype, device="cuda")
    out_b = out_a.clone()
    # the new entry point first, on a plan that was never uploaded
    print(f"noalloc call: ctx={b.ctx_lens.tolist()} q={b.q_lens.tolist()} {b.dtype} "
          f"lists+partials {need} bytes, combine items {pv.plan_num_work_items(plan, 2)}", flush=True)
    pv.multi_token_paged_attn_noalloc(plan, q, kp, vp, table, b.scale, out_a)
    torch.cuda.synchronize()
    assert not pv.plan_owns_device_memory(plan)
    # the existing entry point on the same plan
    lists = torch.empty(pv.plan_device_bytes(plan), dtype=torch.uint8, device="cuda")
    pv.plan_upload_to(plan, lists)
    ws = torch.empty(max(pv.plan_workspace_bytes(plan), 256), dtype=torch.uint8, device="cuda")
    pv.multi_token_paged_attn_planned(plan, q, kp, vp, table, b.scale, out_b, ws)
    torch.cuda.synchronize()
    splits = pv.plan_num_work_items(plan, 2)
    plan.destroy()
    return H.from_dev_bits(out_a), H.from_dev_bits(out_b), splits


def test_noalloc_entry_point_matches_the_planned_one_twice_in_a_row(oracle):
    big = wl.custom([5000, 40, 900], [20, 33, 1], num_q_heads=8, num_kv_heads=2, head_dim=128,
                    dtype="bf16", seed=71)
    small = wl.custom([700], [3], num_q_heads=8, num_kv_heads=2, head_dim=128, dtype="bf16", seed=72)
    for i, b in enumerate((big, small)):
        case = H.make_case(b, fill="nan")
        got, ref, splits = _run_both(case)
        assert splits > 0, "the case is meant to use partial results in the scratch array"
        assert np.array_equal(got, ref), f"call {i}: outputs differ from the planned launch"
        want, _ = oracle.attn(H.pool_tuple(b), b.num_q_heads, case.q, case.k_pool1, case.v_pool1,
                              b.page_table, b.ctx_lens, b.q_lens, b.q_start, b.scale)
        err = np.abs(H.bits_to_f64(got, b.dtype) - want).max()
        print(f"  call {i}: identical to the planned launch; max abs err vs oracle {err:.3e}", flush=True)
        assert err <= H.TOL[b.dtype]


def test_noalloc_entry_point_rejects_a_batch_beyond_the_array():
    import torch
    from paper_2312_05516_amd import binding as pv
    # one long request alone: its KV range is cut into many parts of 128 rows x 130 floats each
    desc = pv.pool_desc(8192, 8, 128, "bf16")
    plan = pv.plan_create(desc, 64, [120000], [128], 8192)
    need = (pv.plan_device_bytes(plan) + 255) // 256 * 256 + pv.plan_workspace_bytes(plan)
    assert need > pv.static_scratch_bytes()
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(pv.PvError) as e:
        pv.multi_token_paged_attn_noalloc(plan, dummy, dummy, dummy, dummy, 0.1, dummy)
    assert e.value.status == 4  # PV_ERR_WORKSPACE: nothing was launched
    plan.destroy()
