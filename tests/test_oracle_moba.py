"""Pins of the oracle's MoBA routing and block-sparse prefill attention (App. A.1,
MoBA paragraph; Eq. 3-4): brute force per token, the dense-causal limit against a
library attention, and special cases."""
import numpy as np
import pytest

import oracle
from helpers import exact_topk

torch = pytest.importorskip("torch")


def _inputs(B, Hq, Hkv, D, T, Tcap, seed):
    r = np.random.default_rng(seed)
    q = r.standard_normal((B, Hq, T, D)).astype(np.float32)
    kc = r.standard_normal((B, Hkv, Tcap, D)).astype(np.float32)
    vc = r.standard_normal((B, Hkv, Tcap, D)).astype(np.float32)
    return q, kc, vc


def test_block_means_match_numpy_and_ragged_tail():
    B, H, D, T, Tcap, block = 2, 2, 8, 70, 96, 16
    _, kc, _ = _inputs(B, H, H, D, T, Tcap, seed=1)
    m = oracle.moba_block_means(kc, T, block)
    assert m.shape == (B, H, 5, D)
    np.testing.assert_allclose(m[:, :, :4], kc[:, :, :64].astype(np.float64)
                               .reshape(B, H, 4, 16, D).mean(axis=3), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(m[:, :, 4], kc[:, :, 64:70].astype(np.float64).mean(axis=2),
                               rtol=1e-13, atol=1e-15)
    kc[:, :, 16:32] = kc[:, :, 16:17]  # a block of identical keys: mean = that key
    np.testing.assert_allclose(oracle.moba_block_means(kc, T, block)[:, :, 1],
                               kc[:, :, 16].astype(np.float64), rtol=1e-14)


@pytest.mark.parametrize("Hq,Hkv,n_first", [(2, 2, 0), (4, 2, 1)])
def test_routing_brute_force_per_token(Hq, Hkv, n_first):
    B, D, T, block, K = 1, 8, 200, 16, 3
    q, kc, _ = _inputs(B, Hq, Hkv, D, T, 208, seed=2)
    means = oracle.moba_block_means(kc, T, block)
    idx, sc = oracle.moba_select(q, means, T, block, K, n_first, want_scores=True)
    G = Hq // Hkv
    for h in range(Hq):
        for t in range(T):
            own = t // block
            s = np.array([q[0, h, t].astype(np.float64) @ means[0, h // G, j] for j in range(own + 1)])
            forced = np.zeros(own + 1, bool)
            forced[own] = True
            forced[:n_first] = True
            want = exact_topk(s, forced, min(K, own + 1))
            got = idx[0, h, t]
            np.testing.assert_array_equal(got[:len(want)], want)
            assert np.all(got[len(want):] == -1)
            assert own in got and np.all(got <= own)  # own block kept, nothing from the future
            np.testing.assert_allclose(sc[0, h, t, :own], s[:own], rtol=1e-13, atol=1e-14)
            assert np.all(np.isnan(sc[0, h, t, own:]))


def test_enough_blocks_is_dense_causal_attention():
    B, Hq, Hkv, D, T, block = 1, 4, 2, 8, 96, 16
    q, kc, vc = _inputs(B, Hq, Hkv, D, T, 96, seed=3)
    means = oracle.moba_block_means(kc, T, block)
    idx = oracle.moba_select(q, means, T, block, K=6)
    out, lse = oracle.sparse_attn_prefill(q, kc, vc, T, block, 0.4, idx)
    tq = torch.from_numpy(q).double()
    tk = torch.from_numpy(kc).double().repeat_interleave(2, dim=1)
    tv = torch.from_numpy(vc).double().repeat_interleave(2, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=0.4, is_causal=True)
    np.testing.assert_allclose(out, want.numpy(), rtol=1e-12, atol=1e-13)
    dense, dlse = oracle.sparse_attn_prefill(q, kc, vc, T, block, 0.4)
    np.testing.assert_allclose(out, dense, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse, dlse, rtol=1e-13)


def test_sparse_prefill_brute_force_rows():
    B, Hq, Hkv, D, T, block, K = 1, 2, 1, 8, 80, 16, 2
    q, kc, vc = _inputs(B, Hq, Hkv, D, T, 80, seed=4)
    idx = oracle.moba_select(q, oracle.moba_block_means(kc, T, block), T, block, K)
    out, _ = oracle.sparse_attn_prefill(q, kc, vc, T, block, 0.5, idx)
    np.testing.assert_allclose(out[0, :, 0], np.tile(vc[0, 0, 0].astype(np.float64), (Hq, 1)), rtol=1e-14)  # y_0 = v_0
    for h in range(Hq):
        for t in (5, 16, 37, 79):
            toks = [i for j in idx[0, h, t] if j >= 0 for i in range(j * block, (j + 1) * block) if i <= t]
            lg = 0.5 * kc[0, 0, toks].astype(np.float64) @ q[0, h, t].astype(np.float64)
            p = torch.softmax(torch.from_numpy(lg), 0).numpy()
            np.testing.assert_allclose(out[0, h, t], p @ vc[0, 0, toks].astype(np.float64),
                                       rtol=1e-12, atol=1e-13)
