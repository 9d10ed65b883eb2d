"""Pins of the oracle's Quest representatives, page score and top-K selection
(Eq. 3; App. A.1) to invariants, brute force and the paper's budget arithmetic."""
import itertools
import os

import numpy as np
import pytest

import oracle
from helpers import exact_topk, topk_set_ok


def _cache(B, H, Tcap, D, seed):
    return np.random.default_rng(seed).standard_normal((B, H, Tcap, D)).astype(np.float32)


@pytest.mark.parametrize("P,T_valid", [(16, 128), (16, 117), (4, 30), (64, 128)])
def test_meta_brackets_every_key_and_is_attained(P, T_valid):
    kc = _cache(2, 2, 128, 8, seed=1)
    meta = oracle.quest_page_meta(kc, P, T_valid)
    Np = -(-T_valid // P)
    for p in range(Np):
        rows = kc[:, :, p * P:min((p + 1) * P, T_valid)]
        np.testing.assert_array_equal(meta[:, :, p, 0], rows.min(axis=2))
        np.testing.assert_array_equal(meta[:, :, p, 1], rows.max(axis=2))
    assert np.all(meta[:, :, Np:] == 0)  # pages past T_valid are not touched


def test_meta_page_size_one_is_the_key():
    kc = _cache(1, 2, 32, 8, seed=2)
    meta = oracle.quest_page_meta(kc, 1, 32)
    np.testing.assert_array_equal(meta[:, :, :, 0], kc)
    np.testing.assert_array_equal(meta[:, :, :, 1], kc)


def test_score_is_an_upper_bound_of_the_true_page_max():
    B, Hq, Hkv, D, P, T = 2, 4, 2, 16, 8, 160
    kc = _cache(B, Hkv, T, D, seed=3)
    q = np.random.default_rng(4).standard_normal((B, Hq, D)).astype(np.float32)
    meta = oracle.quest_page_meta(kc, P, T)
    s = oracle.quest_scores(q, meta, T // P)
    for b in range(B):
        for h in range(Hq):
            logits = kc[b, h // 2].astype(np.float64) @ q[b, h].astype(np.float64)
            true_max = logits.reshape(T // P, P).max(axis=1)
            assert np.all(s[b, h] >= true_max - 1e-12)
            assert np.any(s[b, h] > true_max + 1e-6)  # a box bound is loose in general


def test_score_equals_dot_product_when_page_is_one_key_or_constant():
    B, H, D, T = 1, 2, 8, 24
    kc = _cache(B, H, T, D, seed=5)
    q = np.random.default_rng(6).standard_normal((B, H, D)).astype(np.float32)
    s = oracle.quest_scores(q, oracle.quest_page_meta(kc, 1, T), T)
    want = np.einsum("bhtd,bhd->bht", kc.astype(np.float64), q.astype(np.float64))
    np.testing.assert_allclose(s, want, rtol=1e-13, atol=1e-13)
    kc2 = np.repeat(kc[:, :, ::4], 4, axis=2)  # every page of 4 holds one repeated key
    s2 = oracle.quest_scores(q, oracle.quest_page_meta(kc2, 4, T), T // 4)
    np.testing.assert_allclose(s2, want[:, :, ::4], rtol=1e-13, atol=1e-13)


def test_score_sign_cases():
    # one channel: q>0 picks the max, q<0 picks the min, q=0 contributes nothing
    meta = np.zeros((1, 1, 1, 2, 3), dtype=np.float32)
    meta[0, 0, 0, 0] = [-2, -5, 1]
    meta[0, 0, 0, 1] = [3, -1, 4]
    q = np.array([[[2.0, -3.0, 0.0]]], dtype=np.float32)
    assert oracle.quest_scores(q, meta, 1)[0, 0, 0] == 2 * 3 + (-3) * (-5) + 0


def test_score_is_the_dot_product_with_the_row_picked_by_the_sign_of_q():
    # with min <= max per channel, max(q lo, q hi) = q * (hi where q > 0, lo elsewhere): the form the
    # GPU kernels evaluate (a select per channel, then a plain dot product).  Pins the oracle's
    # two-product form against that identity, term by term exact in float64, for signed and zero q.
    rng = np.random.default_rng(41)
    B, Hq, Hkv, D, Np = 2, 4, 2, 64, 37
    lo = rng.standard_normal((B, Hkv, Np, D)).astype(np.float32)
    hi = lo + np.abs(rng.standard_normal((B, Hkv, Np, D))).astype(np.float32) * (rng.random((B, Hkv, Np, D)) > 0.2)
    meta = np.stack([lo, hi], axis=3)
    q = rng.standard_normal((B, Hq, D)).astype(np.float32)
    q[:, :, ::7] = 0.0
    q[:, :, 3::11] = -0.0
    got = oracle.quest_scores(q, meta, Np)
    for b in range(B):
        for h in range(Hq):
            qq = q[b, h].astype(np.float64)
            pick = np.where(qq > 0, hi[b, h // 2].astype(np.float64), lo[b, h // 2].astype(np.float64))
            want = (pick * qq).sum(axis=1)
            np.testing.assert_allclose(got[b, h], want, rtol=1e-14, atol=1e-14)


def test_topk_brute_force_all_subsets():
    r = np.random.default_rng(7)
    for trial in range(40):
        M = int(r.integers(1, 11))
        K = int(r.integers(0, M + 1))
        s = r.integers(0, 4, M).astype(np.float64)  # many exact ties
        got = oracle.topk_row(s, K)
        best = max((sum(s[list(c)]), tuple(-i for i in c)) for c in itertools.combinations(range(M), K))
        # the maximiser with the lexicographically smallest index tuple
        want = [-i for i in best[1]]
        assert list(got) == want
        np.testing.assert_array_equal(got, exact_topk(s, np.zeros(M, bool), K))


def test_topk_ties_take_lowest_index_and_forced_rank_first():
    s = np.array([1.0, 5, 5, 5, 0, 9])
    np.testing.assert_array_equal(oracle.topk_row(s, 3), [1, 2, 5])
    np.testing.assert_array_equal(oracle.topk_row(s, 3, forced=[0, 0, 0, 0, 1, 0]), [1, 4, 5])
    np.testing.assert_array_equal(oracle.topk_row(s, 6), np.arange(6))


def test_quest_select_forced_pages_inside_K():
    r = np.random.default_rng(8)
    s = r.standard_normal((2, 3, 40))
    idx = oracle.quest_select(s, 6, n_first=1, n_local=2)
    assert idx.shape == (2, 3, 6)
    for row_s, row in zip(s.reshape(-1, 40), idx.reshape(-1, 6)):
        assert row[0] == 0 and list(row[-2:]) == [38, 39]
        forced = np.zeros(40, bool)
        forced[[0, 38, 39]] = True
        np.testing.assert_array_equal(row, exact_topk(row_s, forced, 6))
        ok, why = topk_set_ok(row_s, forced, 6, row)
        assert ok, why
    # K = Np keeps everything
    np.testing.assert_array_equal(oracle.quest_select(s, 40, 1, 1)[0, 0], np.arange(40))


def test_page_size_one_selects_the_top_tokens():
    B, H, D, T, K = 1, 2, 8, 64, 5
    kc = _cache(B, H, T, D, seed=9)
    q = np.random.default_rng(10).standard_normal((B, H, D)).astype(np.float32)
    s = oracle.quest_scores(q, oracle.quest_page_meta(kc, 1, T), T)
    idx = oracle.quest_select(s, K, 0, 0)
    logits = np.einsum("bhtd,bhd->bht", kc.astype(np.float64), q.astype(np.float64))
    for h in range(H):
        assert set(idx[0, h]) == set(np.argsort(-logits[0, h])[:K])


def test_budget_arithmetic_of_the_paper():
    path = os.path.join(os.path.dirname(__file__), "golden", "budget_table.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 12
    for method, unit, K, num, den in rows:
        assert int(K) * int(unit) * int(den) == 4096 * int(num), (method, unit, K)
    # Quest at B=64, K=4, T=4096: 64 pages, first and last page kept inside K
    s = np.random.default_rng(11).standard_normal((1, 1, 64))
    idx = oracle.quest_select(s, 4, 1, 1)[0, 0]
    assert len(idx) == 4 and idx[0] == 0 and idx[-1] == 63


def test_group_score_bounds_the_groups_summed_logit_and_reduces_to_per_head():
    """Group-shared selection (an option, not in the paper): the group's page score is the sum
    of its heads' bounds, so it bounds the largest summed logit of any token of the page; with
    one query head per KV head it is the per-head score; with a page of one key it is the
    summed logit itself."""
    B, Hq, Hkv, D, P, T = 2, 8, 2, 16, 8, 160
    G = Hq // Hkv
    kc = _cache(B, Hkv, T, D, seed=13)
    q = np.random.default_rng(14).standard_normal((B, Hq, D)).astype(np.float32)
    meta = oracle.quest_page_meta(kc, P, T)
    sg = oracle.quest_scores_group(q, meta, T // P)
    assert sg.shape == (B, Hkv, T // P)
    for b in range(B):
        for kvh in range(Hkv):
            qsum = q[b, kvh * G:(kvh + 1) * G].astype(np.float64).sum(axis=0)
            logits = kc[b, kvh].astype(np.float64) @ qsum  # sum over the group of q_h . k
            assert np.all(sg[b, kvh] >= logits.reshape(T // P, P).max(axis=1) - 1e-12)
    q1 = q[:, :Hkv]
    np.testing.assert_array_equal(oracle.quest_scores_group(q1, meta, T // P), oracle.quest_scores(q1, meta, T // P))
    meta1 = oracle.quest_page_meta(kc, 1, T)
    s1 = oracle.quest_scores_group(q, meta1, T)
    for b in range(B):
        for kvh in range(Hkv):
            qsum = q[b, kvh * G:(kvh + 1) * G].astype(np.float64).sum(axis=0)
            np.testing.assert_allclose(s1[b, kvh], kc[b, kvh].astype(np.float64) @ qsum, rtol=1e-12, atol=1e-12)


def test_head_hit_rate_definition():
    """Sec. 2.3 (H1): a head scores 1 only if its selection holds the golden position at EVERY step.
    Hand-made lists with known answers: a head that always holds it, one that misses once, one
    without a golden position at some step, pages (unit 16) and tokens (unit 1)."""
    # 1 sequence, 3 heads, 3 steps, pages of 16 tokens, 4 selected pages per head
    idx = [np.array([[[0, 2, 5, 9], [0, 2, 5, 9], [1, 3, 4, 8]]]),
           np.array([[[0, 2, 6, 9], [0, 3, 6, 9], [1, 3, 4, 8]]]),
           np.array([[[0, 2, 6, 9], [0, 2, 6, 9], [1, 3, 4, 8]]])]
    gold = [np.array([[5 * 16 + 3, 5 * 16 + 3, 4 * 16]]),        # page 5, 5, 4: all present
            np.array([[2 * 16 + 15, 2 * 16 + 15, -1]]),          # page 2: head 1 misses it; head 2 has none
            np.array([[9 * 16, 9 * 16, 8 * 16 + 1]])]            # page 9, 9, 8: all present
    hit = oracle.head_hit(idx, gold, unit=16)
    assert hit.tolist() == [[True, False, True]]
    # the same lists read as token lists (unit 1): only exact positions count
    hit1 = oracle.head_hit(idx, [np.array([[5, 5, 4]]), np.array([[2, 2, -1]]), np.array([[9, 9, 7]])], unit=1)
    assert hit1.tolist() == [[True, False, False]]
    # one step: the hit is plain membership; against a brute-force check on random lists
    r = np.random.default_rng(3)
    for _ in range(20):
        M, K, B, H = 40, 7, 2, 3
        lists = np.stack([[np.sort(r.choice(M, K, replace=False)) for _ in range(H)] for _ in range(B)])
        g = r.integers(0, M * 4, (B, H))
        want = np.array([[(g[b, h] // 4) in lists[b, h].tolist() for h in range(H)] for b in range(B)])
        assert np.array_equal(oracle.head_hit([lists], [g], unit=4), want)
    # a uniformly random selector holds a given candidate with probability K / M per step
    M, K, n = 64, 16, 4000
    lists = np.stack([np.sort(r.choice(M, K, replace=False)) for _ in range(n)])[None]
    rate = oracle.head_hit([lists], [np.full((1, n), 37)], unit=1).mean()
    assert abs(rate - K / M) < 0.03
