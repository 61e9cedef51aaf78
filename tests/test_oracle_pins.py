"""Pins of the CPU oracle against things other than itself: closed forms that follow from
the paper's equations, hand-evaluated Alg. 1, library routines (torch softmax / SDPA on
CPU), and the pure-loop brute force.  No GPU."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import brute
from oracle import vlcache_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_case(seed, Hq=4, Hkv=2, tau=5, m=23, d=8, spread=1.0):
    r = np.random.default_rng(seed)
    q = r.standard_normal((Hq, tau, d)) * spread
    k = r.standard_normal((Hkv, m, d))
    v = r.standard_normal((Hkv, m, d))
    return q, k, v


# ---------------------------------------------------------------- softmax / scores

def test_rows_sum_to_one_and_mass_is_tau():
    q, k, _ = rand_case(1, Hq=6, Hkv=2, tau=7, m=40)
    A, s, M, Z = O.post_vision_attention(q, k, 0.3)
    valid = O.causal_valid(40, 7)
    assert np.all(A[:, ~valid] == 0.0)
    np.testing.assert_allclose(A.sum(axis=2), 1.0, rtol=0, atol=1e-14)
    psi_kv, psi_h, _, _ = O.score(q, k, 0.3)
    np.testing.assert_allclose(psi_h.sum(axis=1), 7.0, atol=1e-12)
    np.testing.assert_allclose(psi_kv.sum(axis=1), 3 * 7.0, atol=1e-12)


def test_region_size_formula_vs_count():
    for m, tau in [(1, 1), (5, 5), (12, 4), (512, 32), (2944, 32), (100, 1)]:
        assert O.region_size(m, tau) == int(O.causal_valid(m, tau).sum())
    # values derived in the shape table from tau(m-tau)+tau(tau+1)/2
    assert O.region_size(512, 32) == 15888
    assert O.region_size(2944, 32) == 93712
    assert O.region_size(10368, 64) == 661536
    assert O.region_size(32768, 64) == 2095136


def test_equal_logits_give_harmonic_scores_golden():
    with open(os.path.join(GOLD, "harmonic_scores.txt")) as f:
        lines = [ln for ln in f if not ln.startswith("#")]
    want = np.array([float(Fraction(x)) for x in lines[0].split()])
    m, tau, d = 12, 4, 3
    q = np.zeros((2, tau, d))
    k = np.random.default_rng(0).standard_normal((1, m, d))
    psi_kv, psi_h, M, Z = O.score(q, k, 1.0)
    np.testing.assert_allclose(psi_h[0], want, rtol=1e-14)
    np.testing.assert_allclose(psi_kv[0], 2 * want, rtol=1e-14)   # two query heads in the group
    np.testing.assert_allclose(Z[0], [9, 10, 11, 12])
    nnz, gamma = O.sparsity(q, k, 1.0, 0.01)
    assert list(nnz) == [O.region_size(m, tau)] * 2 and np.all(gamma == 0.0)


def test_scores_vs_torch_softmax_and_sdpa():
    q, k, _ = rand_case(3, Hq=4, Hkv=2, tau=6, m=31, d=16)
    scale = 0.21
    psi_kv, psi_h, _, _ = O.score(q, k, scale)
    tq, tk = torch.from_numpy(q), torch.from_numpy(k)
    mask = torch.from_numpy(O.causal_valid(31, 6))
    # library softmax on masked logits
    s = torch.einsum("hid,hjd->hij", tq, tk.repeat_interleave(2, dim=0)) * scale
    A = torch.softmax(s.masked_fill(~mask, float("-inf")), dim=-1)
    np.testing.assert_allclose(psi_h, A.sum(1).numpy(), rtol=1e-12)
    # library attention with V = identity returns the attention matrix itself
    eye = torch.eye(31, dtype=torch.float64)[None, None].expand(1, 2, 31, 31)
    A2 = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk[None], eye, attn_mask=mask, scale=scale, enable_gqa=True)[0]
    np.testing.assert_allclose(psi_kv, A2.sum(1).reshape(2, 2, 31).sum(1).numpy(), rtol=1e-10)


def test_gqa_head_mapping_is_consecutive():
    # query heads 0,1 -> kv head 0; 2,3 -> kv head 1: make kv head 1 all zeros -> uniform rows
    q, k, _ = rand_case(4, Hq=4, Hkv=2, tau=3, m=10, d=4)
    k[1] = 0.0
    _, psi_h, _, Z = O.score(q, k, 1.0)
    np.testing.assert_allclose(Z[2:], [[8, 9, 10]] * 2)
    assert not np.allclose(Z[:2], [[8, 9, 10]] * 2)


# ---------------------------------------------------------------- ThresholdFilter sparsity

def test_one_dominant_key_per_row():
    m, tau = 30, 6
    q = np.ones((2, tau, 1))
    k = np.zeros((1, m, 1))
    k[0, 3, 0] = 50.0
    nnz, gamma = O.sparsity(q, k, 1.0, 0.01)
    assert list(nnz) == [tau, tau]
    np.testing.assert_allclose(gamma, 1 - tau / O.region_size(m, tau))


def test_two_level_logits_count():
    m, tau = 40, 8
    r = np.random.default_rng(5)
    level = np.where(r.random(m) < 0.3, 0.0, -10.0)
    level[0] = 0.0                     # every row sees at least one top-level key
    q = np.ones((1, tau, 1))
    k = level.reshape(1, m, 1)
    want = sum(int((level[: m - tau + i + 1] == 0.0).sum()) for i in range(tau))
    nnz, _ = O.sparsity(q, k, 1.0, 0.01)      # -10 < ln 0.01 = -4.6 < 0
    assert int(nnz[0]) == want
    # p small enough keeps everything
    nnz_all, g_all = O.sparsity(q, k, 1.0, 1e-5)
    assert int(nnz_all[0]) == O.region_size(m, tau) and g_all[0] == 0.0


def test_threshold_boundary_is_inclusive():
    # logits 0, ln p and the next double below ln p: s - M = ln p exactly for the second key (kept),
    # one ulp less for the third (filtered); one ulp above is kept as well
    lnp = math.log(0.01)
    below, above = np.nextafter(lnp, -np.inf), np.nextafter(lnp, np.inf)
    q = np.ones((1, 1, 1))
    nnz, _ = O.sparsity(q, np.array([0.0, lnp, below]).reshape(1, 3, 1), 1.0, 0.01)
    assert int(nnz[0]) == 2
    nnz, _ = O.sparsity(q, np.array([0.0, above, below, below]).reshape(1, 4, 1), 1.0, 0.01)
    assert int(nnz[0]) == 2
    # the decision is taken in double precision: a gap of 1e-12 (far below fp32 resolution) decides
    nnz, _ = O.sparsity(q, np.array([0.0, lnp - 1e-12, lnp + 1e-12]).reshape(1, 3, 1), 1.0, 0.01)
    assert int(nnz[0]) == 2


def test_logit_form_equals_literal_filter():
    # Eq. 1 on attention scores (brute, literal) == logit-domain test, away from the boundary
    for seed in range(5):
        q, k, _ = rand_case(10 + seed, Hq=2, Hkv=1, tau=4, m=17, d=4, spread=3.0)
        nnz_b, gam_b = brute.sparsity_literal(q.tolist(), k.tolist(), 0.5, 0.01)
        nnz, gam, margin, _ = O.sparsity(q, k, 0.5, 0.01, want_margin=True)
        assert margin.min() > 1e-6
        assert list(nnz) == nnz_b
        np.testing.assert_allclose(gam, gam_b, rtol=1e-13)
    assert 0 < gam[0] < 1


# ---------------------------------------------------------------- allocation

def test_alloc_golden_float():
    with open(os.path.join(GOLD, "alloc_two_layer.txt")) as f:
        rows = [ln.split() for ln in f if not ln.startswith("#")]
    for alpha, L, g1, g2, b1, b2 in rows:
        gam = np.array([[float(Fraction(g1))] * 3, [float(Fraction(g2))] * 3])
        beta = O.allocate_float(gam, float(alpha))
        np.testing.assert_allclose(beta, [float(Fraction(b1)), float(Fraction(b2))], rtol=1e-12)
        assert brute.budgets_literal(gam.tolist(), float(alpha)) == pytest.approx(list(beta), rel=1e-12)


def test_alloc_integer_worked_examples():
    # gamma' = (0.5, 0.9) with region size 1000 and one head: nnz = (500, 100); m = 3000, alpha = 0.1
    k, beta = O.allocate(np.array([[500], [100]]), 3000, 1, 10)
    assert list(k) == [500, 100]                       # beta = (1/6, 1/30)
    np.testing.assert_allclose(beta, [1 / 6, 1 / 30])
    # gamma' = (0, 0.999): lower clip binds on layer 2 (k_min = ceil(0.01 m) = 10)
    k, _ = O.allocate(np.array([[1000], [1]]), 1000, 1, 10)
    assert list(k) == [200, 10]
    # upper clip: alpha = 1 and one dense layer
    k, _ = O.allocate(np.array([[900], [100]]), 1000, 1, 1)
    assert list(k) == [1000, 200]
    # equal sparsity, odd budget: 2 layers, m = 101, alpha = 1/2 -> 101 tokens, quotas 50 + 50, the token
    # left over goes to the layer with the larger remainder, and among equal remainders to the lower layer
    k, _ = O.allocate(np.array([[7], [7]]), 101, 1, 2)
    assert list(k) == [51, 50]
    # three layers in proportion 1 : 2 : 4 of 70 tokens: exact quotas 10, 20, 40, nothing left over
    k, _ = O.allocate(np.array([[3], [6], [12]]), 100, 7, 30)
    assert list(k) == [10, 20, 40]
    # remainders decide before layer order: n = (1, 1, 2), 10 tokens -> quotas 2.5, 2.5, 5 -> floors 2, 2, 5 and
    # one token left, equal remainders on layers 0 and 1 -> layer 0
    k, _ = O.allocate(np.array([[1], [1], [2]]), 100, 1, 30)
    assert list(k) == [3, 2, 5]


def test_alloc_invariants_random():
    r = np.random.default_rng(7)
    for _ in range(200):
        L, H, m = int(r.integers(1, 40)), int(r.integers(1, 9)), int(r.integers(50, 5000))
        nnz = r.integers(1, 10 ** int(r.integers(1, 8)), size=(L, H))
        an, ad = int(r.integers(1, 30)), 100
        k, beta = O.allocate(nnz, m, an, ad)
        lo = O.k_min(m)
        assert np.all(k >= lo) and np.all(k <= m)
        n = nnz.sum(1)
        quota = n * ((an * L * m) // ad) / n.sum()
        unclipped = (quota >= lo) & (quota <= m)
        if unclipped.all():
            assert int(k.sum()) == (an * L * m) // ad
        assert np.all(np.abs(k[unclipped] - quota[unclipped]) < 1.0)
        # monotone in the layer's count
        order = np.argsort(n, kind="stable")
        strictly = np.diff(n[order]) > 0               # equal counts may differ by the tie-break token
        assert np.all(np.diff(k[order])[strictly] >= 0)
        # agrees with the printed float formula to within one token where no clip binds
        D = 10 ** 9
        beta_f = O.allocate_float(1.0 - nnz / D, an / ad)
        free = unclipped & (beta_f > 0.01) & (beta_f < 1.0)
        assert np.all(np.abs(beta_f[free] * m - k[free]) <= 1.0 + 1e-9)


def test_alloc_equal_sparsity_gives_alpha():
    k, beta = O.allocate(np.full((8, 4), 1234), 1000, 1, 10)
    assert list(k) == [100] * 8 and np.allclose(beta, 0.1)
    k, _ = O.allocate(np.full((3, 2), 5), 101, 1, 10)      # B_tot = 30 -> 10 each
    assert list(k) == [10, 10, 10]
    k, _ = O.allocate(np.full((3, 2), 5), 105, 1, 10)      # B_tot = 31: the extra token goes to the lowest layer
    assert list(k) == [11, 10, 10]


def test_k_min():
    assert [O.k_min(m) for m in (1, 99, 100, 101, 512, 2944, 10368, 32768)] == [1, 1, 1, 2, 6, 30, 104, 328]


# ---------------------------------------------------------------- TopK + gather

def test_topk_equals_full_sort():
    r = np.random.default_rng(11)
    for _ in range(50):
        m = int(r.integers(1, 60))
        psi = np.round(r.random(m), 1) if r.random() < 0.5 else r.random(m)   # with and without ties
        k = int(r.integers(1, m + 1))
        got = O.topk(psi, k)
        assert list(got) == brute.topk_sorted(psi.tolist(), k)
        ref = np.sort(np.lexsort((np.arange(m), -psi))[:k])
        assert list(got) == list(ref)
    assert list(O.topk(np.array([3.0, 1.0, 2.0]), 3)) == [0, 1, 2]
    assert list(O.topk(np.array([3.0, 9.0, 2.0]), 1)) == [1]
    assert list(O.topk(np.array([1.0, 1.0, 1.0, 1.0]), 2)) == [0, 1]


def test_topk_recent_window():
    psi = np.array([5.0, 1.0, 4.0, 0.0, 0.1, 0.2])
    assert list(O.topk(psi, 4, n_recent=2)) == [0, 2, 4, 5]
    assert list(O.topk(psi, 2, n_recent=2)) == [4, 5]
    assert list(O.topk(psi, 3, n_recent=0)) == [0, 1, 2]


def test_recent_window_as_a_fraction_of_the_budget():
    # Sec. 5 fixes the recent window at 10 % of the budget: 10 % of 294 tokens is 29.4 -> 29 whole tokens
    assert O.recent_count(294, 1, 10) == 29
    assert O.recent_count(9, 1, 10) == 0 and O.recent_count(10, 1, 10) == 1
    assert O.recent_count(77, 1, 1) == 77 and O.recent_count(77, 0, 5) == 0
    # never more than the budget, monotone in the budget
    r = np.random.default_rng(0)
    for _ in range(200):
        k, den = int(r.integers(1, 5000)), int(r.integers(1, 50))
        num = int(r.integers(0, den + 1))
        c = O.recent_count(k, num, den)
        assert 0 <= c <= k and c <= O.recent_count(k + 1, num, den)
        assert c * den <= k * num < (c + 1) * den
    # with the window in force the kept set is the last c positions plus the best of the rest (brute force)
    psi = r.random(40)
    k = 20
    c = O.recent_count(k, 1, 10)
    want = sorted(list(range(40 - c, 40)) + sorted(range(40 - c), key=lambda j: (-psi[j], j))[: k - c])
    assert list(O.topk(psi, k, c)) == want
    with pytest.raises(ValueError):
        O.recent_count(5, 3, 2)


def test_decode_query_attention_is_a_library_softmax_summed_over_the_group():
    r = np.random.default_rng(8)
    Hq, Hkv, m, d = 6, 2, 37, 16
    q, k = r.standard_normal((Hq, d)), r.standard_normal((Hkv, m, d))
    a = O.decode_query_attention(q, k, 0.3)
    want = np.zeros((Hkv, m))
    for h in range(Hq):
        want[h // 3] += torch.softmax(torch.from_numpy(k[h // 3] @ q[h] * 0.3), dim=0).numpy()
    np.testing.assert_allclose(a, want, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(a.sum(1), 3.0, rtol=1e-12)
    # the same numbers as the window scoring with a one-row window placed after the prompt's last key:
    # row 0 of a tau = 1 window sees every key (Alg. 1 region i + m - tau >= j)
    psi, *_ = O.score(q[:, None, :], k, 0.3)
    np.testing.assert_allclose(a, psi, rtol=1e-12)


def test_cache_hit_rate_definition():
    r = np.random.default_rng(9)
    m, k = 60, 15
    star = r.random(m)
    best = O.topk(star, k)
    assert O.cache_hit_rate(star, best, k) == (k, 1.0)                       # the optimal policy hits everything
    rest = np.setdiff1d(np.arange(m), best)[:k]
    assert O.cache_hit_rate(star, rest, k) == (0, 0.0)                       # a disjoint set hits nothing
    assert O.cache_hit_rate(star, np.arange(m), m) == (m, 1.0)               # full budget
    for _ in range(50):                                                      # brute-force set intersection
        kept = r.choice(m, size=k, replace=False)
        order = sorted(range(m), key=lambda j: (-star[j], j))[:k]
        hits = len(set(order) & set(kept.tolist()))
        assert O.cache_hit_rate(star, kept, k) == (hits, hits / k)
    # the denominator is |S*| = k (Def. 3.1), not the size of the preserved set: a policy that keeps twice as
    # many positions, all of S* among them, scores 1
    assert O.cache_hit_rate(star, np.concatenate([best, rest]), k) == (k, 1.0)
    assert O.cache_hit_rate(star, best[:5], k) == (5, 5 / k)
    # ties at the cut go to the lower position
    tied = np.array([1.0, 0.5, 0.5, 0.5, 0.0])
    assert O.cache_hit_rate(tied, np.array([0, 1]), 2) == (2, 1.0)
    assert O.cache_hit_rate(tied, np.array([0, 3]), 2) == (1, 0.5)


def test_e4m3_table_and_row_quantiser():
    # the format table against a library's float8 type, the quantiser against that library's conversion
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    mine = O.e4m3_values()
    assert np.array_equal(np.isnan(lib), np.isnan(mine)) and np.array_equal(lib[~np.isnan(lib)], mine[~np.isnan(mine)])
    assert mine[0x38] == 1.0 and mine[0x7E] == 448.0 and mine[0x01] == 2.0 ** -9 and mine[0x08] == 2.0 ** -6
    r = np.random.default_rng(12)
    x = (r.standard_normal((200, 128)) * 10.0 ** r.uniform(-3, 3, size=(200, 1))).astype(np.float32)
    x[3] = 0.0                                                                  # an all-zero row
    code, scale = O.quantize_e4m3_rows(x)
    assert scale.dtype == np.float32 and scale[3] == 1.0 and np.all(code[3] == 0)
    np.testing.assert_array_equal(scale[np.arange(200) != 3], (np.abs(x).max(1) / np.float32(448.0))[np.arange(200) != 3])
    y = np.clip((x / scale[:, None]).astype(np.float32), -448, 448)
    want = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(code, want)
    # the largest element of a row maps to +-448, the error is at most half a step of the local binade
    xh = O.dequantize_e4m3_rows(code, scale)
    assert np.all(np.abs(mine[code]).max(1)[np.arange(200) != 3] == 448.0)
    step = np.maximum(2.0 ** np.floor(np.log2(np.maximum(np.abs(y), 2.0 ** -6))) / 8.0, 2.0 ** -9)
    assert np.all(np.abs(xh - x) <= (0.5 * step + 1e-6) * scale[:, None] * 1.0001)
    # halfway cases go to the even code; quantising a dequantised row changes nothing
    c2, s2 = O.quantize_e4m3_rows(np.array([[448.0, 1.0625, 1.1875, 2.0 ** -10 * 1.0, 0.0]], dtype=np.float32))
    assert s2[0] == 1.0 and c2[0].tolist() == [0x7E, 0x38, 0x3A, 0x00, 0x00]
    c3, s3 = O.quantize_e4m3_rows(xh.astype(np.float32))
    np.testing.assert_array_equal(O.dequantize_e4m3_rows(c3, s3), xh)


def test_compact_is_a_gather():
    _, k, v = rand_case(2, m=19)
    idx = np.array([0, 3, 4, 18])
    kc, vc = O.compact(k[0], v[0], idx)
    assert np.array_equal(kc, k[0][[0, 3, 4, 18]]) and np.array_equal(vc, v[0][[0, 3, 4, 18]])


# ---------------------------------------------------------------- decode attention

def sdpa_ref(q, K, V, scale):
    """torch's CPU attention with GQA expansion; q [Hq,d], K,V [Hkv,n,d]."""
    tq = torch.from_numpy(q)[None, :, None, :]
    out = torch.nn.functional.scaled_dot_product_attention(
        tq, torch.from_numpy(K)[None], torch.from_numpy(V)[None], scale=scale, enable_gqa=True)
    return out[0, :, 0].numpy()


def test_decode_is_textbook_attention():
    r = np.random.default_rng(13)
    for Hq, Hkv in [(4, 2), (7, 1), (3, 3)]:
        q = r.standard_normal((Hq, 16))
        K = r.standard_normal((Hkv, 37, 16))
        V = r.standard_normal((Hkv, 37, 16))
        got = O.decode_attn(q, list(K), list(V), 0.17)
        np.testing.assert_allclose(got, sdpa_ref(q, K, V, 0.17), rtol=1e-11, atol=1e-13)
    got1 = brute.attend(q[0].tolist(), K[0].tolist(), V[0].tolist(), 0.17)
    np.testing.assert_allclose(got[0], got1, rtol=1e-12)


def test_full_budget_decode_equals_uncompressed_and_is_permutation_invariant():
    q, k, v = rand_case(17, Hq=4, Hkv=2, tau=4, m=21, d=8)
    psi_kv, _, _, _ = O.score(q, k, 0.35)
    cache = O.CompressedCache(1, 1, 2)
    cache.fill_layer(0, 0, psi_kv, 21, k, v)            # k_l = m keeps everything
    r = np.random.default_rng(1)
    dq, dk, dv = r.standard_normal((1, 4, 8)), r.standard_normal((1, 2, 8)), r.standard_normal((1, 2, 8))
    out = cache.decode_layer(0, dq, dk, dv, 0.35)
    Kf = np.concatenate([k, dk[0][:, None]], axis=1)
    Vf = np.concatenate([v, dv[0][:, None]], axis=1)
    np.testing.assert_allclose(out[0], sdpa_ref(dq[0], Kf, Vf, 0.35), rtol=1e-11, atol=1e-14)
    perm = r.permutation(22)
    out_p = O.decode_attn(dq[0], list(Kf[:, perm]), list(Vf[:, perm]), 0.35)
    np.testing.assert_allclose(out_p, out[0], rtol=1e-11, atol=1e-14)
    # without append the new token is not attended
    cache2 = O.CompressedCache(1, 1, 2)
    cache2.fill_layer(0, 0, psi_kv, 21, k, v)
    out2 = cache2.decode_layer(0, dq, None, None, 0.35)
    np.testing.assert_allclose(out2[0], sdpa_ref(dq[0], k, v, 0.35), rtol=1e-11, atol=1e-14)


def test_compressed_cache_keeps_topk_rows():
    q, k, v = rand_case(19, Hq=4, Hkv=2, tau=4, m=30, d=8)
    psi_kv, _, _, _ = O.score(q, k, 0.5)
    cache = O.CompressedCache(1, 1, 2)
    cache.fill_layer(0, 0, psi_kv, 7, k, v)
    for h in range(2):
        idx = cache.idx[0][0][h]
        assert len(idx) == 7 and np.all(np.diff(idx) > 0)
        assert psi_kv[h][idx].min() >= np.delete(psi_kv[h], idx).max()
        assert np.array_equal(cache.kc[0][0][h], k[h][idx])


# ---------------------------------------------------------------- numpy oracle vs pure loops

def test_oracle_equals_brute_force_on_tiny_inputs():
    for seed in range(4):
        q, k, _ = rand_case(30 + seed, Hq=4, Hkv=2, tau=3 + seed, m=11 + 3 * seed, d=5, spread=2.0)
        scale = 0.4 + 0.1 * seed
        A = np.array(brute.attention_rows(q.tolist(), k.tolist(), scale))
        A_o, _, _, _ = O.post_vision_attention(q, k, scale)
        np.testing.assert_allclose(A_o, A, rtol=1e-12, atol=1e-300)
        psi_b = np.array(brute.scores_kv(q.tolist(), k.tolist(), scale))
        np.testing.assert_allclose(O.score(q, k, scale)[0], psi_b, rtol=1e-12)


def test_compress_request_wires_the_stages_in_order():
    layers = []
    for l in range(3):
        q, k, _ = rand_case(40 + l, Hq=4, Hkv=2, tau=4, m=200, d=8, spread=1.0 + 2 * l)
        layers.append({"q_win": q, "k": k})
    scales = [0.35, 0.35, 0.35]
    psis, nnz, kk = O.compress_request(layers, scales, 200, 1, 10)
    assert nnz.shape == (3, 4) and len(psis) == 3
    assert list(kk) == list(O.allocate(nnz, 200, 1, 10)[0])
    assert nnz[0].sum() > nnz[2].sum() and kk[0] >= kk[2]      # sharper layers are sparser, get less


# ---------------------------------------------------------------- window attention with row statistics

def test_window_attention_equals_library_sdpa_with_the_causal_mask():
    q, k, v = rand_case(71, Hq=6, Hkv=2, tau=7, m=29, d=16)
    out, M, Z = O.window_attention(q, k, v, 0.21)
    mask = torch.from_numpy(O.causal_valid(29, 7))
    tq, tk, tv = (torch.from_numpy(x)[None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=0.21, enable_gqa=True)[0].numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    # the statistics are those of the scoring path: M + ln Z is the row's log-sum-exp
    s = torch.from_numpy(O.logits(q, k, 0.21)).masked_fill(~mask, -math.inf)
    np.testing.assert_allclose(M + np.log(Z), torch.logsumexp(s, dim=2).numpy(), rtol=1e-13)
    np.testing.assert_allclose(M, s.max(dim=2).values.numpy(), rtol=0, atol=0)


def test_window_attention_special_cases():
    q, k, v = rand_case(72, Hq=4, Hkv=2, tau=4, m=12, d=8)
    # constant values: every output row is that constant whatever the attention
    out, _, _ = O.window_attention(q, k, np.full_like(v, 2.5), 0.4)
    np.testing.assert_allclose(out, 2.5, rtol=1e-14)
    # window = whole prompt: row 0 sees only key 0 and returns v[0]; row i averages v[:i+1] for equal logits
    out, M, Z = O.window_attention(np.zeros((4, 12, 8)), k, v, 1.0)
    for h in range(4):
        for i in range(12):
            np.testing.assert_allclose(out[h, i], v[h // 2, : i + 1].mean(axis=0), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(Z, np.arange(1, 13)[None].repeat(4, 0), rtol=1e-14)
    assert np.all(M == 0.0)
    # a key that dominates row i drags the output to its value row; keys after the row's position are invisible
    kd = np.zeros((2, 12, 8)); kd[:, 3, 0] = 50.0; kd[:, 11, 0] = 80.0
    qd = np.zeros((4, 4, 8)); qd[:, :, 0] = 1.0
    out, _, _ = O.window_attention(qd, kd, v, 1.0)
    np.testing.assert_allclose(out[:, :3], np.broadcast_to(v[[0, 0, 1, 1]][:, None, 3], (4, 3, 8)), rtol=0, atol=1e-12)     # rows 8..10 do not see key 11
    np.testing.assert_allclose(out[:, 3], v[[0, 0, 1, 1], 11], rtol=0, atol=1e-10)              # row 11 does


def test_score_from_stats_equals_scores_and_follows_its_statistics():
    q, k, _ = rand_case(73, Hq=6, Hkv=3, tau=6, m=31, d=8)
    psi_kv, psi_h, M, Z = O.score(q, k, 0.3)
    kv2, h2 = O.score_from_stats(q, k, 0.3, M, Z)
    np.testing.assert_allclose(h2, psi_h, rtol=1e-13, atol=1e-300)
    np.testing.assert_allclose(kv2, psi_kv, rtol=1e-13, atol=1e-300)
    # the sweep takes the statistics as given: doubling Z halves the scores, raising M by ln 2 halves them too
    _, hz = O.score_from_stats(q, k, 0.3, M, 2.0 * Z)
    np.testing.assert_allclose(hz, 0.5 * psi_h, rtol=1e-13)
    _, hm = O.score_from_stats(q, k, 0.3, M + math.log(2.0), Z)
    np.testing.assert_allclose(hm, 0.5 * psi_h, rtol=1e-12)
    # and a library softmax under the mask, summed over the window rows
    s = torch.from_numpy(O.logits(q, k, 0.3)).masked_fill(~torch.from_numpy(O.causal_valid(31, 6)), -math.inf)
    np.testing.assert_allclose(h2, torch.softmax(s, dim=2).sum(dim=1).numpy(), rtol=1e-12)
