"""Pins of the oracle's sparse evaluation (Eq. 4) and dense path: a library
attention routine in float64, closed-form special cases, invariances."""
import numpy as np
import pytest

import oracle

torch = pytest.importorskip("torch")


def _inputs(B, Hq, Hkv, D, Tcap, seed):
    r = np.random.default_rng(seed)
    q = r.standard_normal((B, Hq, D)).astype(np.float32)
    kc = r.standard_normal((B, Hkv, Tcap, D)).astype(np.float32)
    vc = r.standard_normal((B, Hkv, Tcap, D)).astype(np.float32)
    return q, kc, vc


def _sdpa(q, k, v, scale, causal=False):
    G = q.shape[1] // k.shape[1]
    tq = torch.from_numpy(q).double()
    tk = torch.from_numpy(k).double().repeat_interleave(G, dim=1)
    tv = torch.from_numpy(v).double().repeat_interleave(G, dim=1)
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale,
                                                            is_causal=causal).numpy()


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (8, 2)])
def test_dense_decode_matches_library_attention(Hq, Hkv):
    B, D, Tcap, T_valid, scale = 2, 16, 96, 83, 0.25
    q, kc, vc = _inputs(B, Hq, Hkv, D, Tcap, seed=1)
    out, lse = oracle.sparse_attn_decode(q, kc, vc, 16, T_valid, scale)
    want = _sdpa(q[:, :, None, :], kc[:, :, :T_valid], vc[:, :, :T_valid], scale)[:, :, 0]
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)
    G = Hq // Hkv
    logits = scale * np.einsum("bhd,bhtd->bht", q.astype(np.float64),
                               np.repeat(kc[:, :, :T_valid].astype(np.float64), G, axis=1))
    np.testing.assert_allclose(lse, torch.logsumexp(torch.from_numpy(logits), -1).numpy(), rtol=1e-13)


def test_full_budget_equals_dense_and_order_is_irrelevant():
    B, Hq, Hkv, D, P, Tcap, T_valid = 1, 4, 2, 8, 8, 64, 61
    q, kc, vc = _inputs(B, Hq, Hkv, D, Tcap, seed=2)
    dense, dlse = oracle.sparse_attn_decode(q, kc, vc, P, T_valid, 0.3)
    Np = -(-T_valid // P)
    idx = np.tile(np.arange(Np, dtype=np.int32), (B, Hq, 1))
    full, flse = oracle.sparse_attn_decode(q, kc, vc, P, T_valid, 0.3, idx)
    np.testing.assert_allclose(full, dense, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(flse, dlse, rtol=1e-13)
    perm = np.random.default_rng(3).permutation(Np)
    shuf, _ = oracle.sparse_attn_decode(q, kc, vc, P, T_valid, 0.3, idx[..., perm])
    np.testing.assert_allclose(shuf, dense, rtol=1e-12, atol=1e-13)


def test_sparse_subset_matches_library_attention_on_gathered_tokens():
    B, Hq, Hkv, D, P, Tcap, T_valid = 1, 2, 1, 8, 4, 40, 38
    q, kc, vc = _inputs(B, Hq, Hkv, D, Tcap, seed=4)
    idx = np.array([[[0, 3, 9], [2, 5, -1]]], dtype=np.int32)  # page 9 is partial; -1 skipped
    out, _ = oracle.sparse_attn_decode(q, kc, vc, P, T_valid, 0.5, idx)
    for h in range(Hq):
        toks = [t for p in idx[0, h] if p >= 0 for t in range(p * P, (p + 1) * P) if t < T_valid]
        want = _sdpa(q[:, h:h + 1, None, :], kc[:, :, toks], vc[:, :, toks], 0.5)[0, 0, 0]
        np.testing.assert_allclose(out[0, h], want, rtol=1e-12, atol=1e-13)


def test_constant_values_and_single_token():
    B, Hq, Hkv, D, P, Tcap = 1, 2, 2, 8, 4, 32
    q, kc, vc = _inputs(B, Hq, Hkv, D, Tcap, seed=5)
    vc[:] = 0.75
    idx = np.array([[[1, 4], [0, 7]]], dtype=np.int32)
    out, _ = oracle.sparse_attn_decode(q, kc, vc, P, 32, 1.0, idx)
    np.testing.assert_allclose(out, 0.75, rtol=1e-14)
    q, kc, vc = _inputs(B, Hq, Hkv, D, Tcap, seed=6)
    out, lse = oracle.sparse_attn_decode(q, kc, vc, P, 1, 1.0)  # one valid token => y = v_0
    np.testing.assert_allclose(out, vc[:, :, 0].astype(np.float64), rtol=1e-14)
    np.testing.assert_allclose(lse, np.einsum("bhd,bhd->bh", q.astype(np.float64),
                                              kc[:, :, 0].astype(np.float64)), rtol=1e-13)


def test_large_logits_do_not_overflow():
    B, Hq, Hkv, D, P, Tcap = 1, 1, 1, 4, 4, 8
    q, kc, vc = _inputs(B, Hq, Hkv, D, Tcap, seed=7)
    out, lse = oracle.sparse_attn_decode(q * 300, kc * 300, vc, P, 8, 1.0)
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2)])
def test_dense_prefill_matches_library_causal_attention(Hq, Hkv):
    B, D, T = 1, 8, 48
    r = np.random.default_rng(8)
    q = r.standard_normal((B, Hq, T, D)).astype(np.float32)
    kc = r.standard_normal((B, Hkv, 64, D)).astype(np.float32)
    vc = r.standard_normal((B, Hkv, 64, D)).astype(np.float32)
    out, _ = oracle.sparse_attn_prefill(q, kc, vc, T, 16, 0.35)
    want = _sdpa(q, kc[:, :, :T], vc[:, :, :T], 0.35, causal=True)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-13)
    # a row range gives the same rows
    part, _ = oracle.sparse_attn_prefill(q, kc, vc, T, 16, 0.35, t_begin=17, t_end=30)
    np.testing.assert_array_equal(part, out[:, :, 17:30])
