"""The pins must be able to fail: each plausible mistake planted in a copy of the oracle's source
(on the CPU, never in the product) has to be caught by the brute-force / layout / append checks."""
import ctypes
import os
import shutil
import subprocess

import numpy as np
import pytest

import helpers as H
from paper_2312_05516_amd import workloads as wl

ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")

MUTANTS = [
    # (name, file, text to find, replacement)
    ("causal limit one short", "pv_oracle_attend.inc", "const int64_t visible = c + i + 1;",
     "const int64_t visible = c + i;"),
    ("causal limit one long", "pv_oracle_attend.inc", "const int64_t visible = c + i + 1;",
     "const int64_t visible = (c + i + 2 < L) ? c + i + 2 : L;"),
    ("scale dropped", "pv_oracle_attend.inc", "s[t] = dot * (PVO_REAL)scale;", "s[t] = dot;"),
    ("softmax not normalised", "pv_oracle_attend.inc", "s[t] = s[t] / denom;", "s[t] = s[t];"),
    ("K used in place of V", "pv_oracle_attend.inc", "acc[d] += s[t] * (PVO_REAL)V[t * D + d];",
     "acc[d] += s[t] * (PVO_REAL)K[t * D + d];"),
    ("interleaved GQA mapping", "pv_oracle.c", "const int64_t hq = hk * G + g;",
     "const int64_t hq = g * Hkv + hk;"),
    ("K layout: slot and chunk swapped", "pv_oracle.c",
     "return (((page * H + head) * (D / 8) + d / 8) * P + slot) * 8 + d % 8;",
     "return (((page * H + head) * P + slot) * (D / 8) + d / 8) * 8 + d % 8;"),
    ("V layout: row-major", "pv_oracle.c",
     "return (((page * H + head) * (P / 8) + slot / 8) * D + d) * 8 + slot % 8;",
     "return ((page * H + head) * P + slot) * D + d;"),
    ("append reads the wrong row", "pv_oracle.c", "const int64_t row = (int64_t)q_start[r] + j;",
     "const int64_t row = (int64_t)q_start[r];"),
    ("page index not taken from the table", "pv_oracle.c",
     "const int64_t page = page_row[lp];", "const int64_t page = lp;"),
    ("half exponent bias", "pv_oracle.c", "(int)expo - 25);", "(int)expo - 24);"),
    ("bf16 shift", "pv_oracle.c", "uint32_t u = (uint32_t)b << 16;", "uint32_t u = (uint32_t)b << 15;"),
]


def _build_mutant(tmp_path, file, find, repl):
    for f in ("pv_oracle.c", "pv_oracle_attend.inc"):
        shutil.copy(os.path.join(ORACLE_DIR, f), tmp_path / f)
    src = (tmp_path / file).read_text()
    assert src.count(find) == 1, f"mutation target not unique: {find}"
    (tmp_path / file).write_text(src.replace(find, repl))
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", str(so),
                    str(tmp_path / "pv_oracle.c"), "-lm"], check=True)
    return str(so)


def _pins_hold(oracle) -> bool:
    """A compact version of the pins: layout vs reshape, append vs numpy placement, brute force."""
    try:
        for (ctx, qn, hq, hkv, d, dt) in [([37, 20], [5, 12], 4, 2, 64, "f16"),
                                           ([0, 31], [33, 1], 4, 4, 64, "bf16")]:
            b = wl.custom(ctx, qn, num_q_heads=hq, num_kv_heads=hkv, head_dim=d, dtype=dt, seed=19)
            case = H.make_case(b, fill="nan")
            kp, vp = case.k_pool0.copy(), case.v_pool0.copy()
            oracle.kv_append(H.pool_tuple(b), case.k_new, case.v_new, b.page_table, b.ctx_lens,
                             b.q_lens, b.q_start, kp, vp)
            if not (np.array_equal(kp, case.k_pool1) and np.array_equal(vp, case.v_pool1)):
                return False
            got, _ = oracle.attn(H.pool_tuple(b), hq, case.q, case.k_pool1, case.v_pool1,
                                 b.page_table, b.ctx_lens, b.q_lens, b.q_start, b.scale)
            want = H.dense_causal_attention(case)
            if not np.isfinite(got).all() or np.abs(got - want).max() > 1e-9:
                return False
        return True
    except RuntimeError:
        return False  # the mutant made the oracle reject its input: also a caught mistake


def test_unmutated_oracle_passes_the_compact_pins(oracle):
    assert _pins_hold(oracle)


@pytest.mark.parametrize("mutant", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(oracle, tmp_path, mutant):
    _, file, find, repl = mutant
    so = _build_mutant(tmp_path, file, find, repl)
    saved = oracle._lib
    try:
        oracle._lib = oracle._bind(ctypes.CDLL(so))
        assert not _pins_hold(oracle), "the pins did not notice this mistake"
    finally:
        oracle._lib = saved
