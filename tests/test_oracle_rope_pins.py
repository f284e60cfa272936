"""Pins for the oracle's rotary-embedding step (the producer in front of the append): closed forms,
the complex-multiplication form of the published transform, invariants, and numpy / torch rounding
for the 16-bit conversion.  Each planted mistake at the end must break at least one of them."""
import os
import shutil
import subprocess
import ctypes

import numpy as np
import pytest

import helpers as H

ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")


def _rand_bits(rng, shape, dtype, scale=1.0):
    return H.f64_to_bits(rng.standard_normal(shape) * scale, dtype)


def _pins(oracle) -> list:
    """Returns the list of failed pin names (empty = all hold)."""
    bad = []
    rng = np.random.default_rng(7)
    D, heads, rows = 16, 3, 9
    base = 10000.0
    tab = oracle.rope_table(base, D, 64)

    # table: first frequency is 1 rad per position, last is base^-(D-2)/D; cos first, sin second
    t = np.arange(64, dtype=np.float64)
    if not (np.array_equal(tab[:, 0], np.cos(t).astype(np.float32)) and
            np.array_equal(tab[:, D // 2], np.sin(t).astype(np.float32))):
        bad.append("table frequency 0")
    th_last = base ** (-(D - 2) / D)
    if not (np.abs(tab[:, D // 2 - 1] - np.cos(t * th_last)).max() < 1e-7 and
            np.abs(tab[:, D - 1] - np.sin(t * th_last)).max() < 1e-7):
        bad.append("table last frequency")
    th = base ** (-2.0 * np.arange(D // 2) / D)
    if np.abs(tab[:, :D // 2] - np.cos(np.outer(t, th))).max() > 1e-7:
        bad.append("table frequencies")

    for dtype in ("f16", "bf16"):
        x = _rand_bits(rng, (rows, heads, D), dtype)
        xv = H.bits_to_f64(x, dtype)
        pos = rng.integers(0, 64, rows).astype(np.int32)
        pos[0] = 0
        c = tab[pos][:, None, :D // 2].astype(np.float64)
        s = tab[pos][:, None, D // 2:].astype(np.float64)

        # interleaved pairing = multiplication of (x[2i] + i x[2i+1]) by exp(i t theta_i)
        got = oracle.rope(x, pos, tab, "interleaved", dtype)
        z = (xv[..., 0::2] + 1j * xv[..., 1::2]) * (c + 1j * s)
        want = np.empty_like(xv)
        want[..., 0::2], want[..., 1::2] = z.real, z.imag
        if np.abs(got - want).max() > 1e-12:
            bad.append(f"interleaved complex form {dtype}")
        # half-split pairing = x cos + rotate_half(x) sin with rotate_half(x) = (-x2, x1)
        got_h = oracle.rope(x, pos, tab, "half", dtype)
        x1, x2 = xv[..., :D // 2], xv[..., D // 2:]
        want_h = np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)
        if np.abs(got_h - want_h).max() > 1e-12:
            bad.append(f"half-split form {dtype}")
        # position 0 is the identity
        if not (np.array_equal(got[0], xv[0]) and np.array_equal(got_h[0], xv[0])):
            bad.append(f"position 0 {dtype}")
        # a rotation keeps the length of every pair (table entries are rounded to float: 1e-6)
        n_in = xv[..., 0::2] ** 2 + xv[..., 1::2] ** 2
        n_out = got[..., 0::2] ** 2 + got[..., 1::2] ** 2
        if np.abs(n_in - n_out).max() > 1e-5:
            bad.append(f"pair norm {dtype}")

    # quarter turn (cos 0, sin 1) from a hand-made table: (a, b) -> (-b, a) in both pairings
    quarter = np.zeros((1, D), dtype=np.float32)
    quarter[0, D // 2:] = 1.0
    x = _rand_bits(rng, (2, 1, D), "f16")
    xv = H.bits_to_f64(x, "f16")
    z0 = np.zeros(2, dtype=np.int32)
    g = oracle.rope(x, z0, quarter, "interleaved", "f16")
    if not (np.array_equal(g[..., 0::2], -xv[..., 1::2]) and np.array_equal(g[..., 1::2], xv[..., 0::2])):
        bad.append("quarter turn interleaved")
    g = oracle.rope(x, z0, quarter, "half", "f16")
    if not (np.array_equal(g[..., :D // 2], -xv[..., D // 2:]) and np.array_equal(g[..., D // 2:], xv[..., :D // 2])):
        bad.append("quarter turn half")

    # the point of the transform: <R(t1) q, R(t2) k> depends on t2 - t1 only
    q = _rand_bits(rng, (1, 1, D), "f16")
    k = _rand_bits(rng, (1, 1, D), "f16")
    for style in ("interleaved", "half"):
        dots = []
        for shift in (0, 5, 17):
            rq = oracle.rope(q, np.array([3 + shift], np.int32), tab, style, "f16")
            rk = oracle.rope(k, np.array([11 + shift], np.int32), tab, style, "f16")
            dots.append(float((rq * rk).sum()))
        if max(dots) - min(dots) > 1e-5:
            bad.append(f"relative position {style}")
        # and differs when the distance differs
        rq = oracle.rope(q, np.array([3], np.int32), tab, style, "f16")
        rk = oracle.rope(k, np.array([12], np.int32), tab, style, "f16")
        if abs(float((rq * rk).sum()) - dots[0]) < 1e-6:
            bad.append(f"relative position is not constant {style}")
    return bad


def _rounding_pins(oracle) -> list:
    bad = []
    rng = np.random.default_rng(11)
    v = np.concatenate([rng.standard_normal(4000), rng.standard_normal(2000) * 1e-6,
                        rng.standard_normal(2000) * 3e4, [0.0, -0.0, np.inf, -np.inf, 65504.0,
                        65519.99, 65520.0, -65520.0, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -24,
                        2.5 * 2.0 ** -24, 2.0 ** -14, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11,
                        2047.5, 2048.5]])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    if not np.array_equal(oracle.round16(v, "f16"), want):
        bad.append("f16 rounding vs numpy")
    import torch
    v32 = v.astype(np.float32)  # exact floats, so torch's float -> bfloat16 is a single rounding
    want_b = torch.from_numpy(v32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    if not np.array_equal(oracle.round16(v32.astype(np.float64), "bf16"), want_b):
        bad.append("bf16 rounding vs torch")
    # ties to even, written out: 1 + 2^-8 is halfway between bf16 1.0 and 1.0078125 -> 1.0;
    # 1 + 3*2^-8 is halfway between 1.0078125 (odd) and 1.015625 (even) -> 1.015625
    got = oracle.round16(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]), "bf16")
    if list(got) != [0x3F80, 0x3F82]:
        bad.append("bf16 ties")
    # widening what was rounded gives the same bits back (all 65536 patterns, NaNs aside)
    allb = np.arange(65536, dtype=np.uint16)
    for dt in ("f16", "bf16"):
        val = oracle.widen(allb, dt)
        ok = ~np.isnan(val)
        if not np.array_equal(oracle.round16(val[ok], dt), allb[ok]):
            bad.append(f"round trip {dt}")
    return bad


def test_rope_pins_hold(oracle):
    assert _pins(oracle) == []


def test_round16_pins_hold(oracle):
    assert _rounding_pins(oracle) == []


MUTANTS = [
    ("sign of the sine term", "dst[ia] = a * c - b * s;", "dst[ia] = a * c + b * s;"),
    ("second output uses the wrong operand", "dst[ib] = b * c + a * s;", "dst[ib] = a * c + b * s;"),
    ("pairings swapped", "const int32_t ia = style == 0 ? 2 * i : i;",
     "const int32_t ia = style == 1 ? 2 * i : i;"),
    ("sine read from the cosine half", "s = (double)cs[D / 2 + i];", "s = (double)cs[i];"),
    ("frequency exponent", "pow(base, -2.0 * (double)i / (double)D)", "pow(base, -(double)i / (double)D)"),
    ("table halves swapped", "table[t * D + i] = (float)cos((double)t * theta);",
     "table[t * D + i] = (float)sin((double)t * theta);"),
    ("position row", "table + (int64_t)pos[r] * D;", "table + (int64_t)r * D;"),
    ("rounding truncates", "double n = nearbyint(a / quantum);", "double n = floor(a / quantum);"),
    ("subnormal quantum", "if (ex < emin) ex = emin;", "if (ex < emin - 1) ex = emin - 1;"),
    ("overflow threshold", "if (ex > emax) return (uint16_t)(sign | inf);",
     "if (ex > emax + 1) return (uint16_t)(sign | inf);"),
]


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistakes_are_caught(tmp_path, name, find, repl):
    import oracle as O
    for f in ("pv_oracle.c", "pv_oracle_attend.inc"):
        shutil.copy(os.path.join(ORACLE_DIR, f), tmp_path / f)
    src = (tmp_path / "pv_oracle.c").read_text()
    assert src.count(find) == 1, f"mutation target not unique: {find}"
    (tmp_path / "pv_oracle.c").write_text(src.replace(find, repl))
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", str(so),
                    str(tmp_path / "pv_oracle.c"), "-lm"], check=True)
    saved = O._lib
    try:
        O._lib = O._bind(ctypes.CDLL(str(so)))
        try:
            failed = _pins(O) + _rounding_pins(O)
        except RuntimeError:
            failed = ["oracle rejected its input"]
    finally:
        O._lib = saved
    assert failed, f"mutant '{name}' survived every pin"
