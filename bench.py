#!/usr/bin/env python3
"""Benchmark of the multi-token paged attention hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch, as one transformer layer would run
it: KV append of the batch's new tokens, then multi-token paged attention (whichever of the
three attention kernels and the split-KV merge the batch needs).  The per-batch plan (prefix sums, work lists) is built once on
the CPU and reused by every step, as the paper does across layers (Section 6.4); its cost is
reported separately.  Every step uses the next of several independent KV pools ("layers") so the
data comes from HBM, not from a cache warmed by the previous step.

Prints ONE JSON line.  The headline workload is the largest single-GPU configuration
(long_history); `other_workloads` carries the same record for the other configurations.  Per
workload: the timed loop (--steps after --warmup), a `sustained` loop of at least 0.5 s with
median and minimum per step, the `roofline` of the dominant attention kernel from the library's
own per-kernel events, and `cpu_baseline`, the CPU oracle timed on a stated sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = 2500.0  # dense fp16 / bf16
KERNEL_NAMES = {0: "attn_narrow_kernel", 1: "attn_wide_kernel", 2: "attn_combine_kernel",
                3: "kv_append_kernel", 4: "attn_tile256_kernel"}
# timing kind of an attention kernel -> kind of its work items in the plan
ITEM_KIND = {0: 0, 1: 1, 4: 3}
OTHER_WORKLOADS = "decode_heavy,gqa70b,mha13b"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="long_history",
                    help="tiny | mha13b | gqa70b | long_history | decode_heavy | micro_c<ctx>")
    ap.add_argument("--layers", type=int, default=0, help="independent KV pools cycled through "
                    "(0 = pick: at least four, two for pools of 4 GiB of KV and more, enough to "
                    "exceed 1 GiB of KV, at most 8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="target CPU time of the oracle sample of the headline workload (the other "
                    "workloads get a third of it each)")
    ap.add_argument("--sustained-seconds", type=float, default=0.5,
                    help="minimum timed wall time of the second, per-step-timed loop whose median "
                    "and minimum are reported under 'sustained' (at least 50 steps)")
    ap.add_argument("--microbench", action="store_true",
                    help="instead of the step benchmark, time the attention call on the shape of the "
                    "paper's kernel figure (32 requests x 8 query tokens, context sweep) against our "
                    "own contiguous, copy-out and one-token-per-round variants")
    ap.add_argument("--cost-profile", action="store_true",
                    help="instead of the step benchmark, measure the attention cost of one 32-token "
                    "chunk at power-of-two context sizes (the profile the paper's eviction policy "
                    "interpolates) and check the library's interpolation at the midpoints")
    ap.add_argument("--swap", action="store_true",
                    help="instead of the step benchmark, time page gather / scatter (tier swapping) "
                    "through device staging and through pinned host memory")
    ap.add_argument("--rope", action="store_true",
                    help="time the fused rotary-embedding + KV-append call next to the plain "
                    "append on the mixed and decode configurations")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every step eagerly instead of replaying one captured HIP graph "
                    "per KV pool (the step of a small batch is otherwise bound by host launch time)")
    ap.add_argument("--serial-kernels", action="store_true",
                    help="keep the library's per-kernel event timing on in every step and launch "
                    "eagerly: for rocprofv3 runs whose per-kernel averages are compared with "
                    "the bench line's kernel_ms")
    ap.add_argument("--calibration-copy-gib", type=float, default=0.0,
                    help="also run plain device-to-device copies of this many GiB (untimed): the "
                    "known-size kernel that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--extra", default=OTHER_WORKLOADS,
                    help="comma list of further workloads to time briefly and report under "
                    "'other_workloads' ('none' for none)")
    return ap.parse_args()


def make_batch(name: str):
    from paper_2312_05516_amd import workloads as wl
    if name.startswith("micro_c"):
        return wl.microbench(int(name[len("micro_c"):]))
    return wl.CONFIGS[name]()


class DeviceBatch:
    """Device tensors of one workload: L pools, q, new K/V, page table, plan, workspace."""

    def __init__(self, b, layers: int, serial: bool = False, use_graph: bool = True):
        import torch
        from paper_2312_05516_amd import binding as pv
        from paper_2312_05516_amd import workloads as wl
        self.b, self.pv, self.torch = b, pv, torch
        dev = "cuda"
        Hq, Hkv, D = b.num_q_heads, b.num_kv_heads, b.head_dim
        page_elems = Hkv * b.page_size * D
        pool_bytes = 2 * b.num_pages * page_elems * 2  # K + V
        if layers <= 0:
            # at least four independent pools unless one pool alone is far beyond every cache
            # (the chip's last-level cache is 256 MB): every step then reads its KV from HBM
            few = 2 if b.kv_bytes() >= (4 << 30) else 4
            layers = int(min(8, max(few, np.ceil((1 << 30) / max(b.kv_bytes(), 1)))))
            free, _ = torch.cuda.mem_get_info()
            layers = int(max(1, min(layers, (free * 0.6) // pool_bytes)))
        self.layers = layers
        self.kp = [wl.random_values((b.num_pages, page_elems), b.dtype, b.seed * 13 + 2 * i, 1.0, dev)
                   for i in range(layers)]
        self.vp = [wl.random_values((b.num_pages, page_elems), b.dtype, b.seed * 13 + 2 * i + 1, 1.0,
                                    dev) for i in range(layers)]
        self.q = wl.random_values((b.total_q, Hq, D), b.dtype, b.seed * 13 + 101, 1.0, dev)
        self.kn = wl.random_values((b.total_q, Hkv, D), b.dtype, b.seed * 13 + 102, 1.0, dev)
        self.vn = wl.random_values((b.total_q, Hkv, D), b.dtype, b.seed * 13 + 103, 1.0, dev)
        self.out = torch.empty((b.total_q, Hq, D), dtype=self.q.dtype, device=dev)
        self.table = torch.from_numpy(b.page_table).to(dev)
        self.desc = pv.pool_desc(b.num_pages, Hkv, D, b.dtype)
        t0 = time.perf_counter()
        self.plan = pv.plan_create(self.desc, Hq, b.ctx_lens, b.q_lens, b.max_pages_per_req)
        self.plan_ms = (time.perf_counter() - t0) * 1e3
        pv.plan_upload(self.plan)
        self.serial = serial
        if serial:
            pv.plan_enable_timing(self.plan, True)
        self.ws = torch.empty(max(pv.plan_workspace_bytes(self.plan), 256), dtype=torch.uint8,
                              device=dev)
        self.items = {k: pv.plan_num_work_items(self.plan, k) for k in (0, 1, 2, 3)}
        torch.cuda.synchronize()
        self.graphs = None
        if use_graph and not serial:
            # one eager pass first (loads the kernels, uploads the plan), then capture the step of
            # every pool once; the library's launches go to torch's current (capturing) stream
            for l in range(self.layers):
                self.step(l)
            torch.cuda.synchronize()
            self.graphs = []
            cap = torch.cuda.Stream()
            for l in range(self.layers):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=cap):
                    self.step(l)
                self.graphs.append(g)
            torch.cuda.synchronize()

    def step(self, i: int):
        pv, l = self.pv, i % self.layers
        pv.kv_append_planned(self.plan, self.kn, self.vn, self.table, self.kp[l], self.vp[l])
        pv.multi_token_paged_attn_planned(self.plan, self.q, self.kp[l], self.vp[l], self.table,
                                          self.b.scale, self.out, self.ws)

    def run_step(self, i: int):
        if self.graphs is not None:
            self.graphs[i % self.layers].replay()
        else:
            self.step(i)

    def time_steps(self, steps: int, warmup: int) -> float:
        torch = self.torch
        for i in range(warmup):
            self.run_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.run_step(warmup + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def sustained(self, min_seconds: float, min_steps: int = 50) -> dict:
        """A second loop, long enough for the chip to settle at its power limit: at least
        `min_steps` steps and `min_seconds` of timed wall time, every step bracketed by its own
        pair of events on the launch stream; median, minimum and mean per step."""
        torch = self.torch
        for i in range(10):
            self.run_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(5):
            self.run_step(i)
        torch.cuda.synchronize()
        est = max((time.perf_counter() - t0) / 5, 1e-6)
        n = int(max(min_steps, min(20000, np.ceil(min_seconds / est))))
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        t0 = time.perf_counter()
        ev[0].record()
        for i in range(n):
            self.run_step(i)
            ev[i + 1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(n)])
        return {"steps": n, "wall_seconds": round(wall, 3), "median_ms": round(float(np.median(ms)), 5),
                "min_ms": round(float(ms.min()), 5), "mean_ms": round(float(ms.mean()), 5),
                "tflops_at_median": round(self.b.flops() / float(np.median(ms)) / 1e9, 2),
                "kv_gbps_at_median": round(self.b.kv_bytes() / float(np.median(ms)) / 1e6, 1)}

    def kernel_times(self, samples: int, burst: int = 8) -> dict:
        """Average duration of each kernel (HIP events recorded by the library on the launch
        stream around every kernel).  The plan keeps one pair of events per kernel, so a sample is
        the last step of a burst of back-to-back steps: the kernels are measured in the same
        busy state as in the timed loop, not after an idle gap."""
        pv = self.pv
        pv.plan_enable_timing(self.plan, True)
        acc = {k: [] for k in KERNEL_NAMES}
        for s in range(samples):
            for i in range(burst):
                self.step(s * burst + i)
            for k in KERNEL_NAMES:
                ms = pv.plan_kernel_ms(self.plan, k)
                if ms >= 0:
                    acc[k].append(ms)
        pv.plan_enable_timing(self.plan, self.serial)
        return {k: float(np.mean(v)) for k, v in acc.items() if v}

    def kernel_share(self, kind: int):
        """Algorithmic flops and bytes of the work items of attention kernel `kind`: causal
        (row, key) pairs inside the items' KV ranges counted exactly; every (request, KV head)
        K/V range the kernel streams counted once, plus its rows of q and out and the page ids."""
        pv, b = self.pv, self.b
        n = self.items[ITEM_KIND[kind]]
        if n == 0:
            return 0, 0
        it = np.stack([pv.plan_work_item(self.plan, ITEM_KIND[kind], i) for i in range(n)]).astype(np.int64)
        req, hk, rb, rc, k0, k1 = (it[:, j] for j in range(6))
        G = b.num_q_heads // b.num_kv_heads
        ctx = b.ctx_lens[req].astype(np.int64)
        pairs = 0
        for j in range(int(rc.max())):  # j-th row of every item that has one
            m = rc > j
            lim = np.minimum(k1[m], ctx[m] + (rb[m] + j) // G + 1)
            pairs += int(np.maximum(lim - k0[m], 0).sum())
        flops = 4 * b.head_dim * pairs
        # K/V streamed: per (request, KV head) the union of the items' ranges = [min k0, max k1)
        unit = req * b.num_kv_heads + hk
        lo = np.full(b.num_reqs * b.num_kv_heads, np.iinfo(np.int64).max)
        hi = np.zeros(b.num_reqs * b.num_kv_heads, dtype=np.int64)
        np.minimum.at(lo, unit, k0)
        np.maximum.at(hi, unit, k1)
        span = np.maximum(hi - np.minimum(lo, hi), 0)
        kv = int(2 * span.sum() * b.head_dim * 2)
        first = it[:, 6] == 0  # rows are counted once per item set, not once per KV part
        qo = int(2 * rc[first].sum() * b.head_dim * 2)
        pt = int(4 * np.ceil(span / b.page_size).sum())
        return flops, kv + qo + pt

    def close(self):
        self.plan.destroy()
        del self.kp, self.vp


def recorded_traffic(workload: str, kernel: str):
    """HBM bytes per launch measured earlier with rocprofv3 --pmc (profiles/traffic.txt), or None.
    Not measured in this run: the line says so in `traffic_source`."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 6 and f[0] == workload and f[1] == kernel:
                return int((float(f[2]) * float(f[4]) + float(f[3]) * float(f[5])) * 1024)
    except OSError:
        pass
    return None


def roofline_for(db: DeviceBatch, ktimes: dict) -> dict:
    attn = {k: v for k, v in ktimes.items() if k in ITEM_KIND}
    if not attn:
        return None
    kind = max(attn, key=attn.get)
    flops, nbytes = db.kernel_share(kind)
    t = attn[kind] * 1e-3
    t_hbm = nbytes / (HBM_PEAK_GBPS * 1e9)
    t_mfma = flops / (MFMA_PEAK_TFLOPS * 1e12)
    traffic = recorded_traffic(db.b.name, KERNEL_NAMES[kind])
    common = {"traffic": traffic,
              "traffic_source": None if traffic is None else
              "recorded earlier with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/traffic.txt), "
              "not measured in this run",
              "kernel": KERNEL_NAMES[kind], "kernel_ms": round(attn[kind], 5),
              "algorithmic_bytes": nbytes, "algorithmic_flops": flops}
    if t_hbm >= t_mfma:
        ach = nbytes / t / 1e9
        return {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBPS, 4), **common}
    ach = flops / t / 1e12
    return {"bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(ach / MFMA_PEAK_TFLOPS, 4), **common}


def _oracle_sample(db: DeviceBatch, budget_flops: float, threads: int):
    """Run the oracle on a stratified sample of (request, KV head) units worth about budget_flops.
    Returns (flops done, seconds, units, how they were picked, threads used)."""
    import torch
    import oracle
    b = db.b
    Hq, Hkv, D = b.num_q_heads, b.num_kv_heads, b.head_dim
    G = Hq // Hkv
    c = b.ctx_lens.astype(np.int64)
    n = b.q_lens.astype(np.int64)
    unit_flops = 4 * D * G * (n * c + n * (n + 1) // 2)  # per (request, KV head)
    # stratified sample: the (request, KV head) units sorted by cost, every k-th of them (KV head
    # order by a seeded draw), k such that the sample fits the budget; at least one unit
    rng = np.random.default_rng(b.seed + 99)
    live = [r for r in np.argsort(unit_flops, kind="stable") if n[r] > 0]
    all_units = [(int(r), int(h)) for r in live for h in rng.permutation(Hkv)]
    all_units.sort(key=lambda rh: (int(unit_flops[rh[0]]), rh[0]))
    total_all = sum(int(unit_flops[r]) for r, _ in all_units)
    stride = max(1, int(np.ceil(total_all / max(budget_flops, 1.0))))
    page_bytes = 2 * Hkv * b.page_size * D * 2  # K and V image of one page, all KV heads

    def host_bytes(units):
        return sum(int(np.ceil(b.kv_lens[r] / b.page_size)) * page_bytes for r in {r for r, _ in units})

    picked = all_units[stride // 2::stride] or all_units[:1]
    how = f"every {stride}-th unit in order of cost"
    if host_bytes(picked) > 4e9 and len(picked) > 1:
        # the sampled requests' pages are copied to the host; a request's pages hold all its KV
        # heads, so where that copy would pass 4 GB take whole requests instead: every k-th request
        # in order of cost with all its KV heads
        k = max(1, int(np.ceil(stride / Hkv)))
        while True:
            picked = [(int(r), h) for r in live[k // 2::k] for h in range(Hkv)]
            if host_bytes(picked) <= 4e9 or len(picked) <= Hkv:
                break
            k += max(1, k // 4)
        how = f"all KV heads of every {k}-th request in order of cost (host copy kept under 4 GB)"
    mask = np.zeros((b.num_reqs, Hkv), dtype=np.uint8)
    total = 0
    for r, h in picked:
        mask[r, h] = 1
        total += int(unit_flops[r])
    reqs = [r for r in range(b.num_reqs) if mask[r].any()]
    # compact host copy of the sampled requests' pages (layer 0 pools, after the append)
    pages, remap = [], {}
    sub_table = np.full((len(reqs), b.max_pages_per_req), -1, dtype=np.int32)
    for i, r in enumerate(reqs):
        for lp in range(int((b.kv_lens[r] + b.page_size - 1) // b.page_size)):
            p = int(b.page_table[r, lp])
            if p not in remap:
                remap[p] = len(pages)
                pages.append(p)
            sub_table[i, lp] = remap[p]
    idx = torch.tensor(pages, dtype=torch.long, device="cuda")

    def bits(t):
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)

    sub_k = bits(db.kp[0].index_select(0, idx)).ravel()
    sub_v = bits(db.vp[0].index_select(0, idx)).ravel()
    rows = np.concatenate([np.arange(b.q_start[r], b.q_start[r] + b.q_lens[r]) for r in reqs])
    q_s = bits(db.q.index_select(0, torch.from_numpy(rows.astype(np.int64)).cuda()))
    ql = b.q_lens[reqs]
    qs = np.concatenate([[0], np.cumsum(ql)[:-1]]).astype(np.int32)
    pool = (len(pages), b.page_size, Hkv, D, b.dtype)
    t0 = time.perf_counter()
    _, info = oracle.attn(pool, Hq, q_s, sub_k, sub_v, sub_table, b.ctx_lens[reqs], ql, qs, b.scale,
                          unit_mask=mask[reqs], num_threads=threads)
    dt = time.perf_counter() - t0
    return total, dt, int(mask.sum()), how, info["threads"]


def cpu_baseline(db: DeviceBatch, target_seconds: float) -> dict:
    """Time the CPU oracle (fp64, as it stands) on a bounded sample of (request, KV head) units of
    the same workload, on the host cores of this machine.  A small pilot sample measures how fast the
    oracle is on this workload (generation batches are memory-bound on the CPU too); the reported
    sample is then sized for about target_seconds."""
    import oracle
    b = db.b
    oracle.build()
    threads = len(os.sched_getaffinity(0))
    threads = int(os.environ.get("OMP_NUM_THREADS", threads) or threads)
    # assumed oracle speed, for sizing the sample only: ~4 GFLOP/s per thread in fp64.  Batches of
    # generation steps (a few rows per unit) are memory-bound on the CPU too: there a pilot sample
    # (a twentieth of the time) measures the speed first.
    speed = 4e9 * threads
    live = b.q_lens > 0
    rows_per_unit = float(b.q_lens[live].mean()) * b.num_q_heads / b.num_kv_heads if live.any() else 0
    if rows_per_unit < 16:
        done, dt, _, _, _ = _oracle_sample(db, target_seconds / 20 * speed, threads)
        speed = done / max(dt, 1e-6)
    total, dt, units, how, used = _oracle_sample(db, target_seconds * speed, threads)
    return {"value": round(total / dt / 1e12, 6), "unit": "TFLOP/s", "cores": used,
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"{units} of {b.num_reqs * b.num_kv_heads} (request, KV head) units of "
                      f"{b.name} ({how}), {total / 1e9:.2f} "
                      f"GFLOP, fp64 C oracle with OpenMP, attention only"}


def run_workload(name: str, steps: int, warmup: int, layers: int, with_cpu: bool,
                 cpu_seconds: float, serial: bool = False, use_graph: bool = True,
                 sustained_seconds: float = 0.5) -> dict:
    b = make_batch(name)
    db = DeviceBatch(b, layers, serial, use_graph)
    ms = db.time_steps(steps, warmup)
    sustained = db.sustained(sustained_seconds) if sustained_seconds > 0 else None
    ktimes = db.kernel_times(30)
    roof = roofline_for(db, ktimes)
    res = {
        "workload": name,
        "dtype": b.dtype,
        "ms_per_step": round(ms, 5),
        "tflops": round(b.flops() / (ms * 1e-3) / 1e12, 3),
        "kv_gbps": round(b.kv_bytes() / (ms * 1e-3) / 1e9, 1),
        "algorithmic_gbps": round(b.algorithmic_bytes() / (ms * 1e-3) / 1e9, 1),
        "steps": steps,
        "warmup": warmup,
        "sustained": sustained,
        "kernel_ms": {KERNEL_NAMES[k]: round(v, 5) for k, v in ktimes.items()},
        "roofline": roof,
        "plan_ms": round(db.plan_ms, 3),
        "layers": db.layers,
        "launch": "hipgraph" if db.graphs is not None else "eager",
        "items": {"narrow": db.items[0], "wide": db.items[1], "tile256": db.items[3],
                  "combine": db.items[2]},
        "batch": {"requests": b.num_reqs, "new_tokens": b.total_q,
                  "kv_tokens": int(b.kv_lens.sum()), "flops": b.flops(), "kv_bytes": b.kv_bytes()},
    }
    if with_cpu:
        res["cpu_baseline"] = cpu_baseline(db, cpu_seconds)
    db.close()
    return res


def microbench(ctx_list=(128, 512, 2048, 8192, 16384), reps: int = 30) -> list:
    """Shape of the paper's Section 6.4 figure (batch 32, query size 8, 40 heads, head size 128,
    fp16; attention operator only), all four variants built from THIS library's kernel:
      paged      - KV pages at random places in the pool (what the library is for);
      contiguous - the same call with every request's pages consecutive ("ideal" layout);
      copy_out   - first gather the scattered pages into a consecutive region (device copy), then
                   the contiguous call (the paper's CopyOut+Attention straw-man);
      multi_round- eight calls of one query token each (the paper's multi-round straw-man)."""
    import torch
    from paper_2312_05516_amd import binding as pv
    from paper_2312_05516_amd import workloads as wl
    rows = []
    for ctx in ctx_list:
        b = wl.microbench(ctx)
        bi = wl.microbench(ctx, identity_pages=True)
        Hq, Hkv, D = b.num_q_heads, b.num_kv_heads, b.head_dim
        page_elems = Hkv * b.page_size * D
        kp = wl.random_values((b.num_pages, page_elems), b.dtype, 1, 1.0, "cuda")
        vp = wl.random_values((b.num_pages, page_elems), b.dtype, 2, 1.0, "cuda")
        q = wl.random_values((b.total_q, Hq, D), b.dtype, 3, 1.0, "cuda")
        out = torch.empty_like(q)
        desc = pv.pool_desc(b.num_pages, Hkv, D, b.dtype)

        def timed(fn):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / reps

        def attn_call(batch, table):
            plan = pv.plan_create(desc, Hq, batch.ctx_lens, batch.q_lens, batch.max_pages_per_req)
            pv.plan_upload(plan)
            ws = torch.empty(max(pv.plan_workspace_bytes(plan), 256), dtype=torch.uint8,
                             device="cuda")
            return plan, ws, (lambda: pv.multi_token_paged_attn_planned(
                plan, q, kp, vp, table, batch.scale, out, ws))

        t_rand = torch.from_numpy(b.page_table).cuda()
        t_id = torch.from_numpy(bi.page_table).cuda()
        plan_r, ws_r, call_r = attn_call(b, t_rand)
        plan_i, ws_i, call_i = attn_call(bi, t_id)
        used = torch.from_numpy(b.page_table[b.page_table >= 0].astype(np.int64)).cuda()
        kc, vc = torch.empty_like(kp), torch.empty_like(vp)

        def copy_out():
            n = used.numel()
            torch.index_select(kp, 0, used, out=kc[:n])
            torch.index_select(vp, 0, used, out=vc[:n])
            pv.multi_token_paged_attn_planned(plan_i, q, kc, vc, t_id, bi.scale, out, ws_i)

        rounds = []
        n = int(b.q_lens[0])
        for i in range(n):
            pl = pv.plan_create(desc, Hq, b.ctx_lens + i, np.ones_like(b.q_lens),
                                b.max_pages_per_req)
            pv.plan_upload(pl)
            wsr = torch.empty(max(pv.plan_workspace_bytes(pl), 256), dtype=torch.uint8,
                              device="cuda")
            qi = q[i::n].contiguous()
            rounds.append((pl, wsr, qi, torch.empty_like(qi)))

        def multi_round():
            for pl, wsr, qi, oi in rounds:
                pv.multi_token_paged_attn_planned(pl, qi, kp, vp, t_rand, b.scale, oi, wsr)

        res = {"ctx": ctx, "paged_ms": round(timed(call_r), 5),
               "contiguous_ms": round(timed(call_i), 5), "copy_out_ms": round(timed(copy_out), 5),
               "multi_round_ms": round(timed(multi_round), 5),
               "kv_GB": round(b.kv_bytes() / 1e9, 4)}
        res["paged_kv_GBps"] = round(b.kv_bytes() / res["paged_ms"] / 1e6, 1)
        rows.append(res)
        torch.cuda.synchronize()
        for pl in [plan_r, plan_i] + [r[0] for r in rounds]:
            pl.destroy()
        del kp, vp, kc, vc
    return rows


def cost_profile(reps: int = 50) -> dict:
    """Cost_attention(l) of the eviction policy (paper Section 4.3.1): attention time of one
    32-token chunk whose context (itself included) is l tokens, 40 heads x head size 128, fp16, at
    powers of two; then the library's interpolated cost at the midpoints next to a measurement."""
    import torch
    from paper_2312_05516_amd import binding as pv
    from paper_2312_05516_amd import workloads as wl

    def measure(l: int) -> float:
        b = wl.custom([l - 32], [32], num_q_heads=40, num_kv_heads=40, head_dim=128, dtype="f16",
                      seed=l, name=f"chunk_l{l}")
        page_elems = 40 * 16 * 128
        kp = wl.random_values((b.num_pages, page_elems), b.dtype, 1, 1.0, "cuda")
        vp = wl.random_values((b.num_pages, page_elems), b.dtype, 2, 1.0, "cuda")
        q = wl.random_values((32, 40, 128), b.dtype, 3, 1.0, "cuda")
        out = torch.empty_like(q)
        table = torch.from_numpy(b.page_table).cuda()
        desc = pv.pool_desc(b.num_pages, 40, 128, b.dtype)
        plan = pv.plan_create(desc, 40, b.ctx_lens, b.q_lens, b.max_pages_per_req)
        pv.plan_upload(plan)
        ws = torch.empty(max(pv.plan_workspace_bytes(plan), 256), dtype=torch.uint8, device="cuda")
        for _ in range(5):
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

    points = [2 ** k for k in range(5, 16)]  # 32 .. 32768
    costs = [measure(l) for l in points]
    checks = []
    for l in (48, 3000, 24000):
        checks.append({"l": l, "interpolated_ms": round(pv.cost_model(points, costs, 0.0, l), 5),
                       "measured_ms": round(measure(l), 5)})
    return {"ctx_points": points, "attn_cost_ms": [round(c, 5) for c in costs],
            "interpolation_checks": checks}


def swap_bench(reps: int = 20) -> dict:
    """Page gather / scatter of 32-token chunks (two pages) picked at random from a pool shaped like
    the decode-heavy configuration (40 KV heads, head size 128, fp16: 160 KiB per K page)."""
    import torch
    from paper_2312_05516_amd import binding as pv
    from paper_2312_05516_amd import workloads as wl
    Hkv, D, dtype = 40, 128, "f16"
    num_pages, n = 16384, 4096  # 2.7 GB of K+V in the pool, 1.3 GB moved per call
    page_elems = Hkv * 16 * D
    desc = pv.pool_desc(num_pages, Hkv, D, dtype)
    kp = wl.random_values((num_pages, page_elems), dtype, 1, 1.0, "cuda")
    vp = wl.random_values((num_pages, page_elems), dtype, 2, 1.0, "cuda")
    rng = np.random.default_rng(7)
    chunks = rng.permutation(num_pages // 2)[:n // 2]
    ids = torch.from_numpy(np.stack([2 * chunks, 2 * chunks + 1], 1).ravel().astype(np.int32)).cuda()
    moved = 2 * n * page_elems * 2  # K and V bytes per call
    dev = torch.empty((n, 2, page_elems), dtype=torch.int16, device="cuda")
    host = torch.empty((n, 2, page_elems), dtype=torch.int16).pin_memory()

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    t = {"gather_device": timed(lambda: pv.pages_gather(desc, kp, vp, ids, n, dev)),
         "scatter_device": timed(lambda: pv.pages_scatter(desc, dev, ids, n, kp, vp)),
         "gather_pinned_host": timed(lambda: pv.pages_gather(desc, kp, vp, ids, n, host)),
         "scatter_pinned_host": timed(lambda: pv.pages_scatter(desc, host, ids, n, kp, vp))}
    res = {"pages": n, "bytes_moved": moved}
    for k, v in t.items():
        res[k + "_ms"] = round(v * 1e3, 4)
        res[k + "_GBps"] = round(moved / v / 1e9, 1)
    # device staging reads and writes HBM: 2 x moved bytes against 8 TB/s
    res["roofline_device"] = {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBPS,
                              "achieved": round(2 * moved / t["gather_device"] / 1e9, 1),
                              "frac": round(2 * moved / t["gather_device"] / 1e9 / HBM_PEAK_GBPS, 4)}
    return res


def rope_bench(reps: int = 50) -> list:
    """Fused rotary embedding + KV append (one launch: rotate Q, rotate and store K, store V) next to
    the plain append, per configuration.  Bytes per call: K, V rows read and written, Q rows read
    and written, one table row (D floats) per new token."""
    import torch
    from paper_2312_05516_amd import binding as pv
    res = []
    for name in ("mha13b", "gqa70b", "decode_heavy"):
        b = make_batch(name)
        db = DeviceBatch(b, 2, serial=False, use_graph=False)
        table = torch.from_numpy(pv.rope_table(10000.0, b.head_dim, int(b.kv_lens.max()))).cuda()
        q_out = torch.empty_like(db.q)

        def timed(fn):
            for i in range(5):
                fn(i)
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev[0].record()
            for i in range(reps):
                fn(i)
            ev[1].record()
            torch.cuda.synchronize()
            return ev[0].elapsed_time(ev[1]) / reps

        L = db.layers
        t_plain = timed(lambda i: pv.kv_append_planned(db.plan, db.kn, db.vn, db.table,
                                                       db.kp[i % L], db.vp[i % L]))
        out = {"workload": name, "new_tokens": int(b.total_q), "append_ms": round(t_plain, 5)}
        for style in ("interleaved", "half"):
            t = timed(lambda i: pv.rope_kv_append_planned(db.plan, db.q, q_out, db.kn, db.vn,
                                                          table, style, db.table, db.kp[i % L],
                                                          db.vp[i % L]))
            nbytes = b.total_q * b.head_dim * (2 * 2 * 2 * b.num_kv_heads + 2 * 2 * b.num_q_heads + 4)
            out[f"rope_append_{style}_ms"] = round(t, 5)
            out[f"rope_append_{style}_GBps"] = round(nbytes / t / 1e6, 1)
            out["bytes"] = int(nbytes)
        best = min(out["rope_append_interleaved_ms"], out["rope_append_half_ms"])
        out["roofline"] = {"bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBPS,
                           "achieved": round(out["bytes"] / best / 1e6, 1),
                           "frac": round(out["bytes"] / best / 1e6 / HBM_PEAK_GBPS, 4),
                           "kernel": "rope_append_kernel"}
        res.append(out)
        db.close()
    return res


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the attention shards "
              "by KV head or by request with no exchange). Run with --gpus 1.",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    if args.microbench:
        print(json.dumps({"metric": "attention call time on the paper's kernel-figure shape "
                          "(32 requests x 8 query tokens, 40 heads, head size 128, fp16)",
                          "unit": "ms", "n_gpus": 1, "data": "synthetic",
                          "microbench": microbench()}))
        return
    if args.cost_profile:
        print(json.dumps({"metric": "attention cost of one 32-token chunk vs context size "
                          "(40 heads, head size 128, fp16)", "unit": "ms", "n_gpus": 1,
                          "data": "synthetic", "cost_profile": cost_profile()}))
        return
    if args.rope:
        print(json.dumps({"metric": "fused rotary embedding + KV append, ms per call "
                          "(back-to-back calls on one stream)", "unit": "ms", "n_gpus": 1,
                          "data": "synthetic", "peak_GBps": HBM_PEAK_GBPS, "rope": rope_bench()}))
        return
    if args.swap:
        print(json.dumps({"metric": "page gather/scatter for tier swapping (chunks of two 16-token "
                          "pages, 40 KV heads x head size 128, fp16)", "unit": "GB/s", "n_gpus": 1,
                          "data": "synthetic", "swap": swap_bench()}))
        return
    if args.calibration_copy_gib > 0:
        n = int(args.calibration_copy_gib * (1 << 30)) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    with_cpu = not args.no_cpu_baseline
    main_res = run_workload(args.workload, args.steps, args.warmup, args.layers, with_cpu,
                            args.cpu_seconds, args.serial_kernels, not args.no_graph,
                            args.sustained_seconds)
    b = make_batch(args.workload)
    others = []
    for name in [x for x in args.extra.split(",") if x and x != "none" and x != args.workload]:
        # the same number of steps and warm-up steps as the headline, bounded to ~0.5 s per loop
        r = run_workload(name, args.steps, args.warmup, 0, with_cpu, args.cpu_seconds / 3, False,
                         not args.no_graph, args.sustained_seconds)
        others.append({k: r[k] for k in ("workload", "dtype", "ms_per_step", "tflops", "kv_gbps",
                                         "steps", "warmup", "sustained", "kernel_ms", "roofline",
                                         "items", "plan_ms") if k in r}
                      | ({"cpu_baseline": r["cpu_baseline"]} if "cpu_baseline" in r else {}))
    line = {
        "metric": "multi-token paged attn TFLOP/s + effective KV GB/s (1 MI355X, % roofline)",
        "value": main_res["tflops"],
        "unit": "TFLOP/s",
        "effective_kv_GBps": main_res["kv_gbps"],
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": b.dtype,
        "data": "synthetic",
        "config": {"workload": args.workload, "requests": b.num_reqs, "num_q_heads": b.num_q_heads,
                   "num_kv_heads": b.num_kv_heads, "head_dim": b.head_dim,
                   "page_size": b.page_size, "new_tokens": b.total_q,
                   "kv_tokens": int(b.kv_lens.sum()), "layers_cycled": main_res["layers"],
                   "step": "kv_append + multi_token_paged_attn (plan built once, reused)",
                   "launch": main_res["launch"]},
        "roofline": main_res["roofline"],
        "cpu_baseline": main_res.get("cpu_baseline"),
        "sustained": main_res["sustained"],
        "kernel_ms": main_res["kernel_ms"],
        "plan_ms": main_res["plan_ms"],
        "items": main_res["items"],
    }
    if others:
        line["other_workloads"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
