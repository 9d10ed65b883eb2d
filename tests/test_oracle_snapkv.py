"""Pins of the oracle's SnapKV compression (App. A.1, SnapKV paragraph): probability
mass conservation, a library softmax / max-pool, limits, needle retention."""
import numpy as np
import pytest

import oracle
from helpers import exact_topk

torch = pytest.importorskip("torch")


def _inputs(B, Hq, Hkv, D, T, W, seed, Tcap=None):
    r = np.random.default_rng(seed)
    Tcap = Tcap or T
    qw = r.standard_normal((B, Hq, W, D)).astype(np.float32)
    kc = r.standard_normal((B, Hkv, Tcap, D)).astype(np.float32)
    vc = r.standard_normal((B, Hkv, Tcap, D)).astype(np.float32)
    return qw, kc, vc


def test_votes_match_library_softmax_and_conserve_mass():
    B, Hq, Hkv, D, T, W, scale = 2, 4, 2, 8, 60, 6, 0.4
    qw, kc, _ = _inputs(B, Hq, Hkv, D, T, W, seed=1, Tcap=64)
    votes, wm = oracle.snapkv_votes(qw, kc, T, scale, want_window_mass=True)
    G = Hq // Hkv
    logits = scale * torch.einsum("bhwd,bhtd->bhwt", torch.from_numpy(qw).double(),
                                  torch.from_numpy(kc[:, :, :T]).double().repeat_interleave(G, 1))
    pos = torch.arange(T - W, T)[:, None]
    logits = logits.masked_fill(torch.arange(T)[None, :] > pos, float("-inf"))
    A = torch.softmax(logits, -1).numpy()
    want = A[..., :T - W].sum(axis=2).reshape(B, Hkv, G, T - W).sum(axis=2)
    np.testing.assert_allclose(votes, want, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(wm, A[..., T - W:].sum(-1), rtol=1e-12, atol=1e-15)
    # every softmax row sums to one: votes + window mass = G * W per KV head
    np.testing.assert_allclose(votes.sum(-1) + wm.reshape(B, Hkv, G * W).sum(-1), G * W, rtol=1e-12)


def test_maxpool_matches_library_and_bounds():
    x = np.random.default_rng(2).standard_normal((3, 50))
    np.testing.assert_array_equal(oracle.maxpool1d(x, 1), x)
    for kern in (3, 7):
        got = oracle.maxpool1d(x, kern)
        want = torch.nn.functional.max_pool1d(torch.from_numpy(x)[None], kern, 1, kern // 2)[0].numpy()
        np.testing.assert_array_equal(got, want)
        assert np.all(got >= x)


def test_select_gather_order_ties_and_full_keep():
    B, H, D, T, W = 1, 2, 4, 40, 4
    _, kc, vc = _inputs(B, H, H, D, T, W, seed=3, Tcap=48)
    pooled = np.random.default_rng(4).integers(0, 5, (B, H, T - W)).astype(np.float64)  # exact ties
    idx, kco, vco = oracle.snapkv_select_gather(pooled, kc, vc, T, W, 10, Tcap_out=20)
    for h in range(H):
        want = exact_topk(pooled[0, h], np.zeros(T - W, bool), 10)
        np.testing.assert_array_equal(idx[0, h], want)
        np.testing.assert_array_equal(kco[0, h, :10], kc[0, h, want])
        np.testing.assert_array_equal(vco[0, h, :10], vc[0, h, want])
        np.testing.assert_array_equal(kco[0, h, 10:14], kc[0, h, T - W:T])  # then the window rows
        np.testing.assert_array_equal(vco[0, h, 10:14], vc[0, h, T - W:T])
        assert np.all(kco[0, h, 14:] == 0)
    idx, kco, vco = oracle.snapkv_select_gather(pooled, kc, vc, T, W, T - W)
    np.testing.assert_array_equal(kco, kc[:, :, :T])  # keeping everything = the full cache
    np.testing.assert_array_equal(vco, vc[:, :, :T])


def test_full_keep_decode_equals_dense_and_needle_is_retained():
    B, Hq, Hkv, D, T, W = 1, 4, 2, 16, 256, 8
    qw, kc, vc = _inputs(B, Hq, Hkv, D, T, W, seed=5)
    needle = 77
    kc[0, :, needle] = 4 * qw[0, ::2, 0]  # strongly aligned with the window queries' first row
    qw[0, :, :] = qw[0, :, :1] + 0.1 * qw[0]
    res = oracle.snapkv_compress(qw, kc, vc, T, 16, 7, 0.25)
    for h in range(Hkv):
        assert needle in res["idx"][0, h]
        assert np.all(np.diff(res["idx"][0, h]) > 0)
    full = oracle.snapkv_compress(qw, kc, vc, T, T - W, 7, 0.25)
    q = qw[:, :, -1]
    a, _ = oracle.sparse_attn_decode(q, full["kc"], full["vc"], 16, T, 0.25)
    b, _ = oracle.sparse_attn_decode(q, kc, vc, 16, T, 0.25)
    np.testing.assert_array_equal(a, b)
