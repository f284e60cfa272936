"""Pins for the CPU oracle: everything here runs without a GPU and without the HIP library.

Each test ties the oracle to something other than itself: the pool layout as a numpy
reshape, a dense float64 brute force over history + new tokens, torch's CPU
scaled_dot_product_attention, scipy's softmax for the 1-token case, closed forms
(prefix means, exact rational softmax weights), and invariants of the method
(page permutation, GQA = repeated MHA, sub-requests, chunked prefill).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import helpers as H
from paper_2312_05516_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_oracle(oracle, case, pools=None, precision="f64", scale=None, **kw):
    b = case.batch
    kp, vp = pools if pools is not None else (case.k_pool1, case.v_pool1)
    return oracle.attn(H.pool_tuple(b), b.num_q_heads, case.q, kp, vp, b.page_table, b.ctx_lens,
                       b.q_lens, b.q_start, b.scale if scale is None else scale,
                       precision=precision, **kw)


SMALL_SHAPES = [
    # ctx, q, Hq, Hkv, D, dtype
    ([37, 100], [5, 12], 4, 4, 64, "f16"),
    ([0, 16, 31], [7, 1, 33], 4, 2, 64, "bf16"),
    ([5, 0, 48, 15], [1, 1, 16, 17], 8, 2, 128, "f16"),
    ([63], [2], 2, 1, 128, "bf16"),
]


# ---------------------------------------------------------------- layout
def test_pool_index_matches_reshape_layout(oracle):
    b = wl.custom([20], [3], num_q_heads=6, num_kv_heads=3, head_dim=64, pool_pages=5)
    pool = H.pool_tuple(b)
    elems = wl.pool_elems(b)
    ids = np.arange(elems, dtype=np.int64)
    kv = ids.reshape(b.num_pages, b.num_kv_heads, b.head_dim // 8, b.page_size, 8)
    vv = ids.reshape(b.num_pages, b.num_kv_heads, b.page_size // 8, b.head_dim, 8)
    rng = np.random.default_rng(0)
    for _ in range(500):
        p, h = rng.integers(b.num_pages), rng.integers(b.num_kv_heads)
        s, d = rng.integers(b.page_size), rng.integers(b.head_dim)
        assert oracle.k_index(pool, p, h, s, d) == kv[p, h, d // 8, s, d % 8]
        assert oracle.v_index(pool, p, h, s, d) == vv[p, h, s // 8, d, s % 8]
    # both maps are bijections onto the pool
    all_k = {oracle.k_index(pool, p, h, s, d) for p in range(b.num_pages)
             for h in range(b.num_kv_heads) for s in range(b.page_size) for d in range(0, 64, 7)}
    assert len(all_k) == b.num_pages * b.num_kv_heads * b.page_size * len(range(0, 64, 7))


def test_widening_is_exact(oracle):
    bits = np.arange(0, 65536, 37, dtype=np.uint16)
    bits = np.concatenate([bits, np.array([0, 1, 0x3FF, 0x400, 0x7BFF, 0x7C00, 0x8000, 0xFBFF,
                                           0xFC00, 0x3C00, 0x7F80, 0xFF80], dtype=np.uint16)])
    for dt in ("f16", "bf16"):
        got = oracle.widen(bits, dt)
        want = H.bits_to_f64(bits, dt)
        assert np.array_equal(got, want, equal_nan=True)


# ---------------------------------------------------------------- whole result
@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_matches_dense_brute_force(oracle, shape):
    ctx, qn, hq, hkv, d, dt = shape
    b = wl.custom(ctx, qn, num_q_heads=hq, num_kv_heads=hkv, head_dim=d, dtype=dt, seed=11)
    case = H.make_case(b)
    want = H.dense_causal_attention(case)
    got, _ = run_oracle(oracle, case)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() < 1e-12
    got32, _ = run_oracle(oracle, case, precision="f32")
    assert np.abs(got32 - want).max() < 2e-5


def test_tiny_config_matches_brute_force(oracle):
    case = H.make_case(wl.tiny())
    assert case.batch.ctx_lens.tolist() == [37, 100] and case.batch.q_lens.tolist() == [5, 12]
    got, _ = run_oracle(oracle, case)
    assert np.abs(got - H.dense_causal_attention(case)).max() < 1e-12


def test_matches_torch_cpu_sdpa(oracle):
    import torch
    import torch.nn.functional as F
    b = wl.custom([21, 64], [9, 3], num_q_heads=4, num_kv_heads=2, head_dim=64, dtype="f16",
                  seed=5)
    case = H.make_case(b)
    got, _ = run_oracle(oracle, case)
    G = b.num_q_heads // b.num_kv_heads
    for r in range(b.num_reqs):
        c, n, s0 = int(b.ctx_lens[r]), int(b.q_lens[r]), int(b.q_start[r])
        K = torch.from_numpy(H.bits_to_f64(case.k_full[r], b.dtype)).float()
        V = torch.from_numpy(H.bits_to_f64(case.v_full[r], b.dtype)).float()
        Q = torch.from_numpy(H.bits_to_f64(case.q[s0:s0 + n], b.dtype)).float()
        K = K.permute(1, 0, 2).repeat_interleave(G, dim=0)  # [Hq, L, D]
        V = V.permute(1, 0, 2).repeat_interleave(G, dim=0)
        Qh = Q.permute(1, 0, 2)  # [Hq, n, D]
        allow = torch.arange(c + n)[None, :] <= (c + torch.arange(n))[:, None]
        O = F.scaled_dot_product_attention(Qh[None], K[None], V[None], attn_mask=allow[None, None],
                                           scale=b.scale)[0]
        ref = O.permute(1, 0, 2).double().numpy()
        assert np.abs(got[s0:s0 + n] - ref).max() < 5e-6


def test_single_token_is_plain_decode_attention(oracle):
    from scipy.special import softmax
    b = wl.custom([50, 1, 0], [1, 1, 1], num_q_heads=2, num_kv_heads=2, head_dim=64, seed=3)
    case = H.make_case(b)
    got, _ = run_oracle(oracle, case)
    for r in range(b.num_reqs):
        K = H.bits_to_f64(case.k_full[r], b.dtype)
        V = H.bits_to_f64(case.v_full[r], b.dtype)
        qv = H.bits_to_f64(case.q[int(b.q_start[r])], b.dtype)
        for h in range(2):
            w = softmax(K[:, h] @ qv[h] * b.scale)  # no mask at all: every cached token + itself
            assert np.abs(got[int(b.q_start[r]), h] - w @ V[:, h]).max() < 1e-12


# ---------------------------------------------------------------- softmax rows
def test_probability_rows(oracle):
    b = wl.custom([19, 40], [6, 4], num_q_heads=4, num_kv_heads=2, head_dim=64, seed=9)
    case = H.make_case(b)
    for (r, hq) in [(0, 0), (1, 3)]:
        _, probs, _ = run_oracle(oracle, case, probs_of=(r, hq))
        c, n = int(b.ctx_lens[r]), int(b.q_lens[r])
        assert probs.shape == (n, c + n)
        assert np.abs(probs.sum(axis=1) - 1.0).max() < 1e-12
        for i in range(n):
            assert np.count_nonzero(probs[i]) == c + i + 1
            assert (probs[i, c + i + 1:] == 0).all()


# ---------------------------------------------------------------- closed forms
def test_zero_query_gives_prefix_means(oracle):
    b = wl.custom([13, 0], [6, 5], num_q_heads=2, num_kv_heads=1, head_dim=64, seed=2)
    case = H.make_case(b)
    case.q[:] = 0
    got, _ = run_oracle(oracle, case)
    for r in range(b.num_reqs):
        c, n, s0 = int(b.ctx_lens[r]), int(b.q_lens[r]), int(b.q_start[r])
        V = H.bits_to_f64(case.v_full[r], b.dtype)[:, 0]
        for i in range(n):
            mean = V[:c + i + 1].mean(axis=0)
            assert np.abs(got[s0 + i, 0] - mean).max() < 1e-12
            assert np.abs(got[s0 + i, 1] - mean).max() < 1e-12
            if c + i + 2 <= c + n:  # a mask shifted by one position would give this instead
                shifted = V[:c + i + 2].mean(axis=0)
                assert np.abs(got[s0 + i, 0] - shifted).max() > 1e-4


def test_equal_value_rows_give_that_row(oracle):
    b = wl.custom([30], [4], num_q_heads=2, num_kv_heads=2, head_dim=64, seed=4)
    case = H.make_case(b)
    P = b.page_size
    row = case.v_full[0][0].copy()
    vp = case.v_pool1.copy()
    for t in range(int(b.kv_lens[0])):
        H.put_token(b, case.k_pool1, vp, int(b.page_table[0, t // P]), t % P, case.k_full[0][t], row)
    got, _ = run_oracle(oracle, case, pools=(case.k_pool1, vp))
    want = H.bits_to_f64(row, b.dtype)
    assert np.abs(got - want[None]).max() < 1e-12


def test_exact_rational_softmax_weights(oracle):
    """scores are integers * ln 2, so the weights are exact ratios of powers of two."""
    D, c, n = 64, 5, 3
    b = wl.custom([c], [n], num_q_heads=1, num_kv_heads=1, head_dim=D, seed=1)
    case = H.make_case(b)
    L = c + n
    ks = [3, -1, 0, 2, 1, -2, 4, 0]  # integer score of every position
    vs = [Fraction(k, 4) for k in (1, -3, 8, 5, -7, 2, 6, -4)]  # V[t, 0]; V[t, 1] = t
    K = np.zeros((L, 1, D))
    V = np.zeros((L, 1, D))
    K[:, 0, 0] = ks
    V[:, 0, 0] = [float(v) for v in vs]
    V[:, 0, 1] = np.arange(L)
    Q = np.zeros((n, 1, D))
    Q[:, 0, 0] = 1.0
    kp = np.zeros(wl.pool_elems(b), dtype=np.uint16)
    vp = np.zeros(wl.pool_elems(b), dtype=np.uint16)
    kb, vb = H.f64_to_bits(K, "f16"), H.f64_to_bits(V, "f16")
    for t in range(L):
        H.put_token(b, kp, vp, int(b.page_table[0, t // 16]), t % 16, kb[t], vb[t])
    got, _ = oracle.attn(H.pool_tuple(b), 1, H.f64_to_bits(Q, "f16"), kp, vp, b.page_table,
                         b.ctx_lens, b.q_lens, b.q_start, float(np.log(2.0)))
    for i in range(n):
        vis = c + i + 1
        wsum = sum(Fraction(2) ** k for k in ks[:vis])
        o0 = sum(Fraction(2) ** k * v for k, v in zip(ks[:vis], vs[:vis])) / wsum
        o1 = sum(Fraction(2) ** k * t for t, k in enumerate(ks[:vis])) / wsum
        assert abs(got[i, 0, 0] - float(o0)) < 1e-13
        assert abs(got[i, 0, 1] - float(o1)) < 1e-13
        assert np.abs(got[i, 0, 2:]).max() == 0.0


def test_one_hot_scores_read_the_right_slot(oracle):
    """V[t, 0] = t and a query aligned with exactly one key: the output names that position."""
    D = 64
    ctx, n = 45, 20  # spans pages 0..4, new tokens start mid-page
    b = wl.custom([ctx], [n], num_q_heads=1, num_kv_heads=1, head_dim=D, seed=8)
    L = ctx + n
    rng = np.random.default_rng(0)
    K = np.where(rng.random((L, 1, D)) < 0.5, -1.0, 1.0)  # +-1 keys: |<k_a,k_b>| << D for a != b
    V = np.zeros((L, 1, D))
    V[:, 0, 0] = np.arange(L)
    kp = np.zeros(wl.pool_elems(b), dtype=np.uint16)
    vp = np.zeros(wl.pool_elems(b), dtype=np.uint16)
    kb, vb = H.f64_to_bits(K, "f16"), H.f64_to_bits(V, "f16")
    for t in range(L):
        H.put_token(b, kp, vp, int(b.page_table[0, t // 16]), t % 16, kb[t], vb[t])
    for target in [0, 15, 16, 31, ctx - 1, ctx, ctx + 1, 47, 48, L - 1]:
        Q = np.repeat(K[target][None], n, axis=0)  # every new token asks for `target`
        got, _ = oracle.attn(H.pool_tuple(b), 1, H.f64_to_bits(Q, "f16"), kp, vp, b.page_table,
                             b.ctx_lens, b.q_lens, b.q_start, 1.0)
        for i in range(n):
            if target <= ctx + i:  # visible: weight e^64 against at most e^~30
                assert abs(got[i, 0, 0] - target) < 1e-6, (target, i)
            else:  # not yet visible: the answer must be some earlier position
                assert got[i, 0, 0] <= ctx + i + 1e-9


# ---------------------------------------------------------------- invariants
def test_page_permutation_invariance_is_bit_exact(oracle):
    b = wl.custom([37, 100, 3], [5, 12, 1], num_q_heads=4, num_kv_heads=2, head_dim=64, seed=21)
    case = H.make_case(b, fill="random")
    base, _ = run_oracle(oracle, case)
    rng = np.random.default_rng(99)
    for _ in range(3):
        perm = rng.permutation(b.num_pages)  # old page p moves to perm[p]
        page_elems = b.num_kv_heads * b.page_size * b.head_dim
        kp = np.empty_like(case.k_pool1).reshape(b.num_pages, page_elems)
        vp = np.empty_like(case.v_pool1).reshape(b.num_pages, page_elems)
        kp[perm] = case.k_pool1.reshape(b.num_pages, page_elems)
        vp[perm] = case.v_pool1.reshape(b.num_pages, page_elems)
        table = np.where(b.page_table >= 0, perm[np.maximum(b.page_table, 0)], -1).astype(np.int32)
        got, _ = oracle.attn(H.pool_tuple(b), b.num_q_heads, case.q, kp.ravel(), vp.ravel(), table,
                             b.ctx_lens, b.q_lens, b.q_start, b.scale)
        assert np.array_equal(got, base)


def test_paper_figure_page_lists(oracle):
    """The two page lists the paper prints: a decode request on chunks 3,1 and a prefill
    request on chunks 0,4,5,2,7 of an 8-chunk pool."""
    lists, pool_pages = {}, None
    with open(os.path.join(GOLDEN, "paper_page_example.txt")) as f:
        for line in f:
            tok = line.split()
            if not tok or tok[0].startswith("#"):
                continue
            if tok[0] == "pool_pages":
                pool_pages = int(tok[1])
            elif tok[0] == "request":
                lists[int(tok[1])] = [int(x) for x in tok[3:]]
    assert pool_pages == 8 and lists == {0: [3, 1], 1: [0, 4, 5, 2, 7]}
    # request 0: 27 cached + 1 new token (2 pages); request 1: 0 cached + 70 new tokens (5 pages)
    b = wl.custom([27, 0], [1, 70], num_q_heads=2, num_kv_heads=2, head_dim=64, pool_pages=8)
    b.page_table[:] = -1
    b.page_table[0, :2] = lists[0]
    b.page_table[1, :5] = lists[1]
    case = H.make_case(b)
    got, _ = run_oracle(oracle, case)
    assert np.abs(got - H.dense_causal_attention(case)).max() < 1e-12
    # page 6 belongs to nobody: it must still hold the fill pattern after the oracle's own append
    kp, vp = case.k_pool0.copy(), case.v_pool0.copy()
    oracle.kv_append(H.pool_tuple(b), case.k_new, case.v_new, b.page_table, b.ctx_lens, b.q_lens,
                     b.q_start, kp, vp)
    assert (H.k_view(b, kp)[6] == wl.nan_pattern(b.dtype)).all()
    assert np.array_equal(kp, case.k_pool1) and np.array_equal(vp, case.v_pool1)


def test_gqa_equals_mha_with_repeated_kv_heads(oracle):
    G, Hkv, D = 4, 2, 64
    bg = wl.custom([33, 7], [9, 1], num_q_heads=G * Hkv, num_kv_heads=Hkv, head_dim=D, seed=13)
    cg = H.make_case(bg)
    got, _ = run_oracle(oracle, cg)
    bm = wl.custom([33, 7], [9, 1], num_q_heads=G * Hkv, num_kv_heads=G * Hkv, head_dim=D, seed=13)
    assert np.array_equal(bm.page_table, bg.page_table)

    def mha_result(order):
        kp = np.zeros(wl.pool_elems(bm), dtype=np.uint16)
        vp = np.zeros(wl.pool_elems(bm), dtype=np.uint16)
        for r in range(bm.num_reqs):
            for t in range(int(bm.kv_lens[r])):
                H.put_token(bm, kp, vp, int(bm.page_table[r, t // 16]), t % 16,
                            cg.k_full[r][t][order], cg.v_full[r][t][order])
        out, _ = oracle.attn(H.pool_tuple(bm), bm.num_q_heads, cg.q, kp, vp, bm.page_table,
                             bm.ctx_lens, bm.q_lens, bm.q_start, bm.scale)
        return out

    consecutive = np.repeat(np.arange(Hkv), G)  # 0 0 0 0 1 1 1 1
    interleaved = np.tile(np.arange(Hkv), G)  # 0 1 0 1 0 1 0 1
    assert np.abs(mha_result(consecutive) - got).max() < 1e-13
    assert np.abs(mha_result(interleaved) - got).max() > 1e-3


def test_sub_requests_share_pages(oracle):
    """Section 4.3.4: a recomputed prefix attending to itself plus the new prompt attending to
    everything, as two batch entries on the same pages, equal one full prefill."""
    L, n_drop, n_new = 75, 22, 9
    full = wl.custom([0], [L], num_q_heads=4, num_kv_heads=2, head_dim=64, seed=17)
    cf = H.make_case(full)
    ref, _ = run_oracle(oracle, cf)
    sub = wl.custom([0, L - n_new], [n_drop, n_new], num_q_heads=4, num_kv_heads=2, head_dim=64,
                    seed=17, pool_pages=full.num_pages)
    sub.page_table = np.full((2, full.page_table.shape[1]), -1, dtype=np.int32)
    sub.page_table[0, :(n_drop + 15) // 16] = full.page_table[0, :(n_drop + 15) // 16]
    sub.page_table[1] = full.page_table[0]
    q = np.concatenate([cf.q[:n_drop], cf.q[L - n_new:]])
    got, _ = oracle.attn(H.pool_tuple(sub), 4, q, cf.k_pool1, cf.v_pool1, sub.page_table,
                         sub.ctx_lens, sub.q_lens, sub.q_start, sub.scale)
    assert np.abs(got[:n_drop] - ref[:n_drop]).max() < 1e-13
    assert np.abs(got[n_drop:] - ref[L - n_new:]).max() < 1e-13


def test_chunked_prefill_is_consistent(oracle):
    c, n, n1 = 20, 30, 11
    b = wl.custom([c], [n], num_q_heads=2, num_kv_heads=2, head_dim=64, seed=23)
    case = H.make_case(b)
    ref, _ = run_oracle(oracle, case)
    pool = H.pool_tuple(b)
    kp, vp = case.k_pool0.copy(), case.v_pool0.copy()
    outs = []
    for (cc, nn, lo) in [(c, n1, 0), (c + n1, n - n1, n1)]:
        oracle.kv_append(pool, case.k_new[lo:lo + nn], case.v_new[lo:lo + nn], b.page_table, [cc],
                         [nn], [0], kp, vp)
        o, _ = oracle.attn(pool, 2, case.q[lo:lo + nn], kp, vp, b.page_table, [cc], [nn], [0],
                           b.scale)
        outs.append(o)
    assert np.abs(np.concatenate(outs) - ref).max() < 1e-13


# ---------------------------------------------------------------- append
def test_append_is_an_exact_scatter(oracle):
    b = wl.custom([37, 0, 16, 15], [5, 40, 1, 2], num_q_heads=4, num_kv_heads=2, head_dim=64,
                  seed=29, dtype="bf16")
    case = H.make_case(b)
    N, Hkv, D = b.total_q, b.num_kv_heads, b.head_dim
    # unique bit patterns per element (K and V disjoint)
    k_new = (np.arange(N * Hkv * D, dtype=np.uint32) % 30000 + 1).astype(np.uint16).reshape(N, Hkv, D)
    v_new = (np.arange(N * Hkv * D, dtype=np.uint32) % 30000 + 30001).astype(np.uint16).reshape(N, Hkv, D)
    kp, vp = case.k_pool0.copy(), case.v_pool0.copy()
    oracle.kv_append(H.pool_tuple(b), k_new, v_new, b.page_table, b.ctx_lens, b.q_lens, b.q_start,
                     kp, vp)
    want_k, want_v = case.k_pool0.copy(), case.v_pool0.copy()
    for r in range(b.num_reqs):
        for j in range(int(b.q_lens[r])):
            t = int(b.ctx_lens[r]) + j
            H.put_token(b, want_k, want_v, int(b.page_table[r, t // 16]), t % 16,
                        k_new[int(b.q_start[r]) + j], v_new[int(b.q_start[r]) + j])
    assert np.array_equal(kp, want_k) and np.array_equal(vp, want_v)
    changed = np.count_nonzero(kp != case.k_pool0)
    assert changed == N * Hkv * D  # exactly the addressed slots, nothing else
    kp2, vp2 = kp.copy(), vp.copy()
    oracle.kv_append(H.pool_tuple(b), k_new, v_new, b.page_table, b.ctx_lens, b.q_lens, b.q_start,
                     kp2, vp2)
    assert np.array_equal(kp2, kp) and np.array_equal(vp2, vp)


def test_append_rejects_bad_pages(oracle):
    b = wl.custom([10], [3], num_q_heads=2, num_kv_heads=2, head_dim=64, seed=1)
    case = H.make_case(b)
    table = b.page_table.copy()
    table[0, 0] = b.num_pages
    with pytest.raises(RuntimeError):
        oracle.kv_append(H.pool_tuple(b), case.k_new, case.v_new, table, b.ctx_lens, b.q_lens,
                         b.q_start, case.k_pool0.copy(), case.v_pool0.copy())
    with pytest.raises(RuntimeError):
        oracle.attn(H.pool_tuple(b), 2, case.q, case.k_pool1, case.v_pool1, table, b.ctx_lens,
                    b.q_lens, b.q_start, b.scale)


def test_garbage_slots_are_never_read(oracle):
    """Slots past the end of the last page hold NaN in these pools; the result must be finite."""
    b = wl.custom([3, 17], [2, 1], num_q_heads=2, num_kv_heads=2, head_dim=64, seed=31)
    case = H.make_case(b, fill="nan")
    got, _ = run_oracle(oracle, case)
    assert np.isfinite(got).all()


def test_unit_mask_selects_units(oracle):
    b = wl.custom([9, 12], [3, 2], num_q_heads=4, num_kv_heads=2, head_dim=64, seed=37)
    case = H.make_case(b)
    full, _ = run_oracle(oracle, case)
    mask = np.array([[0, 1], [1, 0]], dtype=np.uint8)
    part, _ = run_oracle(oracle, case, unit_mask=mask)
    assert np.isnan(part[0:3, 0:2]).all() and np.isnan(part[3:5, 2:4]).all()
    assert np.array_equal(part[0:3, 2:4], full[0:3, 2:4])
    assert np.array_equal(part[3:5, 0:2], full[3:5, 0:2])


# ---------------------------------------------------------------- tier swapping (page copies)
def test_page_gather_scatter_are_plain_copies(oracle):
    b = wl.custom([100, 30], [5, 2], num_q_heads=4, num_kv_heads=2, head_dim=64, seed=41)
    case = H.make_case(b, fill="random")
    pool = H.pool_tuple(b)
    page_elems = b.num_kv_heads * b.page_size * b.head_dim
    kp = case.k_pool1.reshape(b.num_pages, page_elems)
    vp = case.v_pool1.reshape(b.num_pages, page_elems)
    rng = np.random.default_rng(3)
    ids = rng.permutation(b.num_pages)[:7].astype(np.int32)
    st = oracle.pages_gather(pool, case.k_pool1, case.v_pool1, ids)
    assert st.shape == (7, 2, page_elems)
    assert np.array_equal(st[:, 0], kp[ids]) and np.array_equal(st[:, 1], vp[ids])  # numpy indexing
    # scatter into other pages of a fresh pool: listed pages take the image, the rest is untouched
    k2 = np.full_like(case.k_pool1, 0x1234)
    v2 = np.full_like(case.v_pool1, 0x4321)
    dst = rng.permutation(b.num_pages)[:7].astype(np.int32)
    oracle.pages_scatter(pool, st, dst, k2, v2)
    k2r, v2r = k2.reshape(b.num_pages, page_elems), v2.reshape(b.num_pages, page_elems)
    assert np.array_equal(k2r[dst], kp[ids]) and np.array_equal(v2r[dst], vp[ids])
    rest = np.setdiff1d(np.arange(b.num_pages), dst)
    assert (k2r[rest] == 0x1234).all() and (v2r[rest] == 0x4321).all()
    # swap out + swap in to new places + remapped table = same attention result, bit for bit
    base, _ = run_oracle(oracle, case)
    used = np.unique(b.page_table[b.page_table >= 0])
    new_home = rng.permutation(b.num_pages)[:len(used)].astype(np.int32)
    st = oracle.pages_gather(pool, case.k_pool1, case.v_pool1, used.astype(np.int32))
    k3 = np.zeros_like(case.k_pool1)
    v3 = np.zeros_like(case.v_pool1)
    oracle.pages_scatter(pool, st, new_home, k3, v3)
    remap = np.full(b.num_pages, -1, dtype=np.int32)
    remap[used] = new_home
    table = np.where(b.page_table >= 0, remap[np.maximum(b.page_table, 0)], -1).astype(np.int32)
    got, _ = oracle.attn(pool, b.num_q_heads, case.q, k3, v3, table, b.ctx_lens, b.q_lens,
                         b.q_start, b.scale)
    assert np.array_equal(got, base)
    with pytest.raises(RuntimeError):
        oracle.pages_gather(pool, case.k_pool1, case.v_pool1, [b.num_pages])


# ---------------------------------------------------------------- eviction cost model
def test_cost_interpolation_and_retention_order(oracle):
    pts = [32, 64, 128, 256, 512]
    ys = [1.0, 1.5, 2.5, 4.5, 8.5]
    for p, y in zip(pts, ys):  # profiled points are reproduced exactly (+ c)
        assert oracle.cost(pts, ys, 0.25, p) == y + 0.25
    assert oracle.cost(pts, ys, 0.0, 96) == 2.0  # midway between 64 and 128
    assert oracle.cost(pts, ys, 0.0, 192) == 3.5
    assert np.isclose(oracle.cost(pts, ys, 0.0, np.interp(1, [0, 1], [300, 300])),
                      np.interp(300, pts, ys))  # numpy's piecewise-linear interpolation
    assert np.isclose(oracle.cost(pts, ys, 0.0, 1024), 8.5 + (8.5 - 4.5) * 2)  # last segment extended
    assert np.isclose(oracle.cost(pts, ys, 0.0, 16), 1.0 - 0.25)  # first segment extended
    rng = np.random.default_rng(0)
    c = rng.uniform(1, 10, size=50)
    t = rng.uniform(1, 600, size=50)
    order = oracle.retention_order(c, t)
    assert np.array_equal(order, np.argsort(c / t, kind="stable"))
    # same idle time: cheaper (earlier, shorter-context) chunks go first; same cost: older first
    assert oracle.retention_order([3, 1, 2], [5, 5, 5]).tolist() == [1, 2, 0]
    assert oracle.retention_order([2, 2, 2], [10, 300, 60]).tolist() == [1, 2, 0]
    with pytest.raises(RuntimeError):
        oracle.retention_order([1.0], [0.0])
