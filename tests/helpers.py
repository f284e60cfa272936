"""Test-side utilities: building host inputs for a batch and a dense brute force.

Everything here is numpy written for the tests; it calls neither the oracle nor
the HIP library, so it can serve as an independent pin for both.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

from paper_2312_05516_amd import workloads as wl


def f16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


def bits_to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    return f16_bits_to_f64(bits) if dtype == "f16" else bf16_bits_to_f64(bits)


def f64_to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the 16-bit type (round-to-nearest-even) and return bit patterns."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float64)).to(
        torch.float16 if dtype == "f16" else torch.bfloat16)
    return wl.as_u16(t).reshape(np.shape(x))


def pool_tuple(b: wl.Batch):
    return (b.num_pages, b.page_size, b.num_kv_heads, b.head_dim, b.dtype)


def k_view(b: wl.Batch, pool: np.ndarray) -> np.ndarray:
    """K pool as [page, head, d//8, slot, d%8] (the documented layout as a reshape)."""
    return pool.reshape(b.num_pages, b.num_kv_heads, b.head_dim // 8, b.page_size, 8)


def v_view(b: wl.Batch, pool: np.ndarray) -> np.ndarray:
    """V pool as [page, head, slot//8, d, slot%8]."""
    return pool.reshape(b.num_pages, b.num_kv_heads, b.page_size // 8, b.head_dim, 8)


def put_token(b: wl.Batch, kp: np.ndarray, vp: np.ndarray, page: int, slot: int,
              k_row: np.ndarray, v_row: np.ndarray):
    """Store one token ([Hkv, D] bit patterns) using the reshape views."""
    kv, vv = k_view(b, kp), v_view(b, vp)
    kv[page, :, :, slot, :] = k_row.reshape(b.num_kv_heads, b.head_dim // 8, 8)
    vv[page, :, slot // 8, :, slot % 8] = v_row


@dataclass
class Case:
    batch: wl.Batch
    q: np.ndarray  # [N, Hq, D] u16
    k_full: List[np.ndarray]  # per request [L, Hkv, D] u16
    v_full: List[np.ndarray]
    k_new: np.ndarray  # [N, Hkv, D] u16
    v_new: np.ndarray
    k_pool0: np.ndarray  # pools holding only the past tokens (before append), flat u16
    v_pool0: np.ndarray
    k_pool1: np.ndarray  # pools after the new tokens were stored (numpy placement)
    v_pool1: np.ndarray


def make_case(b: wl.Batch, fill: str = "nan", value_seed=None, k_full=None, v_full=None,
              q=None) -> Case:
    """Draw all values of a batch on the host (or take the given per-request [L, Hkv, D] rows and
    queries) and lay the pools out with numpy."""
    seed = b.seed if value_seed is None else value_seed
    Hq, Hkv, D, P = b.num_q_heads, b.num_kv_heads, b.head_dim, b.page_size
    N = b.total_q
    if q is None:
        q = wl.as_u16(wl.random_values((N, Hq, D), b.dtype, seed * 7 + 1, b.value_std))
    given = k_full is not None
    if not given:
        k_full, v_full = [], []
    for r in range(0 if given else b.num_reqs):
        L = int(b.kv_lens[r])
        k_full.append(wl.as_u16(wl.random_values((L, Hkv, D), b.dtype, seed * 7 + 100 + 2 * r,
                                                 b.value_std)))
        v_full.append(wl.as_u16(wl.random_values((L, Hkv, D), b.dtype, seed * 7 + 101 + 2 * r,
                                                 b.value_std)))
    elems = wl.pool_elems(b)
    if fill == "nan":
        kp = np.full(elems, wl.nan_pattern(b.dtype), dtype=np.uint16)
        vp = np.full(elems, wl.nan_pattern(b.dtype), dtype=np.uint16)
    elif fill == "random":
        kp = wl.as_u16(wl.random_values((elems,), b.dtype, seed * 7 + 3, b.value_std)).copy()
        vp = wl.as_u16(wl.random_values((elems,), b.dtype, seed * 7 + 4, b.value_std)).copy()
    else:
        kp = np.zeros(elems, dtype=np.uint16)
        vp = np.zeros(elems, dtype=np.uint16)
    k_new = np.zeros((N, Hkv, D), dtype=np.uint16)
    v_new = np.zeros((N, Hkv, D), dtype=np.uint16)
    for r in range(b.num_reqs):
        c, n = int(b.ctx_lens[r]), int(b.q_lens[r])
        for t in range(c):
            put_token(b, kp, vp, int(b.page_table[r, t // P]), t % P, k_full[r][t], v_full[r][t])
        s = int(b.q_start[r])
        k_new[s:s + n] = k_full[r][c:c + n]
        v_new[s:s + n] = v_full[r][c:c + n]
    kp1, vp1 = kp.copy(), vp.copy()
    for r in range(b.num_reqs):
        c, n = int(b.ctx_lens[r]), int(b.q_lens[r])
        for t in range(c, c + n):
            put_token(b, kp1, vp1, int(b.page_table[r, t // P]), t % P, k_full[r][t],
                      v_full[r][t])
    return Case(b, q, k_full, v_full, k_new, v_new, kp, vp, kp1, vp1)


def dense_causal_attention(case: Case, scale=None) -> np.ndarray:
    """Brute force: full L x L causal attention on the contiguous history + new tokens of every
    request in float64, keeping the last n rows.  Queries of the history rows are irrelevant and
    set to zero.  Returns [N, Hq, D] float64."""
    b = case.batch
    Hq, Hkv, D = b.num_q_heads, b.num_kv_heads, b.head_dim
    G = Hq // Hkv
    scale = b.scale if scale is None else scale
    out = np.zeros((b.total_q, Hq, D), dtype=np.float64)
    for r in range(b.num_reqs):
        c, n = int(b.ctx_lens[r]), int(b.q_lens[r])
        L = c + n
        s0 = int(b.q_start[r])
        K = bits_to_f64(case.k_full[r], b.dtype)  # [L, Hkv, D]
        V = bits_to_f64(case.v_full[r], b.dtype)
        Qn = bits_to_f64(case.q[s0:s0 + n], b.dtype)  # [n, Hq, D]
        for hq in range(Hq):
            hk = hq // G
            Qfull = np.zeros((L, D))
            Qfull[c:] = Qn[:, hq]
            A = (Qfull @ K[:, hk].T) * scale  # [L, L]
            mask = np.triu(np.ones((L, L), dtype=bool), k=1)
            A = np.where(mask, -np.inf, A)
            A = A - A.max(axis=1, keepdims=True)
            Pm = np.exp(A)
            Pm = Pm / Pm.sum(axis=1, keepdims=True)
            O = Pm @ V[:, hk]
            out[s0:s0 + n, hq] = O[c:]
    return out


# ---------------------------------------------------------------------------------------------
# GPU side: run a Case through the C-ABI library (imports torch / the binding lazily)
# ---------------------------------------------------------------------------------------------
def _torch_dtype(dtype: str):
    import torch
    return torch.float16 if dtype == "f16" else torch.bfloat16


def to_dev_bits(bits: np.ndarray, dtype: str):
    """uint16 bit patterns -> CUDA tensor of the 16-bit float type (same bits)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(_torch_dtype(dtype))


def from_dev_bits(t) -> np.ndarray:
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def gpu_run(case: Case, scale=None, page_table=None, pools=None, do_append=True, one_shot=False,
            k_new=None, v_new=None):
    """append + attention through libpv.  Returns (out_bits [N,Hq,D] u16, k_pool u16, v_pool u16)."""
    import torch
    from paper_2312_05516_amd import binding as pv
    b = case.batch
    desc = pv.pool_desc(b.num_pages, b.num_kv_heads, b.head_dim, b.dtype)
    kp0, vp0 = pools if pools is not None else (case.k_pool0, case.v_pool0)
    kp, vp = to_dev_bits(kp0, b.dtype), to_dev_bits(vp0, b.dtype)
    table_h = b.page_table if page_table is None else page_table
    table = torch.from_numpy(np.ascontiguousarray(table_h, dtype=np.int32)).cuda()
    q = to_dev_bits(case.q, b.dtype)
    kn = to_dev_bits(case.k_new if k_new is None else k_new, b.dtype)
    vn = to_dev_bits(case.v_new if v_new is None else v_new, b.dtype)
    out = torch.full((b.total_q, b.num_q_heads, b.head_dim), float("nan"),
                     dtype=_torch_dtype(b.dtype), device="cuda")
    sc = b.scale if scale is None else scale
    if one_shot:
        if do_append:
            pv.kv_append(desc, kn, vn, table, b.max_pages_per_req, b.ctx_lens, b.q_lens, b.q_start,
                         kp, vp)
        nbytes = pv.attn_workspace_bytes(desc, b.num_q_heads, b.num_reqs, b.total_q,
                                         int(b.kv_lens.max()) if b.num_reqs else 0)
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        pv.multi_token_paged_attn(desc, b.num_q_heads, q, kp, vp, table, b.max_pages_per_req,
                                  b.ctx_lens, b.q_lens, b.q_start, sc, out, ws)
    else:
        plan = pv.plan_create(desc, b.num_q_heads, b.ctx_lens, b.q_lens, b.max_pages_per_req)
        assert np.array_equal(pv.plan_q_start(plan), b.q_start)
        # the plan's lists go into a buffer of ours: the library allocates no device memory at all
        lists = torch.empty(pv.plan_device_bytes(plan), dtype=torch.uint8, device="cuda")
        pv.plan_upload_to(plan, lists)
        assert not pv.plan_owns_device_memory(plan)
        ws = torch.empty(max(pv.plan_workspace_bytes(plan), 256), dtype=torch.uint8, device="cuda")
        if do_append:
            pv.kv_append_planned(plan, kn, vn, table, kp, vp)
        pv.multi_token_paged_attn_planned(plan, q, kp, vp, table, sc, out, ws)
        torch.cuda.synchronize()
        plan.destroy()
    torch.cuda.synchronize()
    return from_dev_bits(out), from_dev_bits(kp).ravel(), from_dev_bits(vp).ravel()


TOL = {"f16": 5e-3, "bf16": 2e-2}
