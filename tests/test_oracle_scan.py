"""Pins of the oracle's gated decay recurrence (Sec. 2.1, Eq. 1) to facts that do
not depend on the oracle: the unrolled closed form, textbook special cases, a
library IIR filter, and structural invariants."""
import numpy as np
import pytest
from scipy.signal import lfilter

import oracle


def _rand(B, H, T, D, seed, gate_mean=4.2):
    r = np.random.default_rng(seed)
    k = r.standard_normal((B, H, T, D)).astype(np.float32)
    v = r.standard_normal((B, H, T, D)).astype(np.float32)
    g = (1 / (1 + np.exp(-(gate_mean + 0.5 * r.standard_normal((B, H, T, D)))))).astype(np.float32)
    return k, v, g


def _closed_form(x, g):
    """x~_t = sum_{s<=t} (prod_{r=s+1..t} g_r) (1-g_s) x_s, written out term by term."""
    x = x.astype(np.float64)
    g = g.astype(np.float64)
    T = x.shape[0]
    out = np.zeros_like(x)
    for t in range(T):
        for s in range(t + 1):
            out[t] += np.prod(g[s + 1:t + 1], axis=0) * (1 - g[s]) * x[s]
    return out


def test_closed_form_brute_force():
    k, v, g = _rand(1, 2, 96, 5, seed=1, gate_mean=1.0)
    ko, vo, sk, sv = oracle.rat_scan(k, v, g)
    for h in range(2):
        np.testing.assert_allclose(ko[0, h], _closed_form(k[0, h], g[0, h]), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(vo[0, h], _closed_form(v[0, h], g[0, h]), rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(sk, ko[:, :, -1])
    np.testing.assert_array_equal(sv, vo[:, :, -1])


def test_gate_zero_is_identity_bit_exact():
    k, v, g = _rand(2, 2, 64, 8, seed=2)
    ko, vo, _, _ = oracle.rat_scan(k, v, np.zeros_like(g))
    np.testing.assert_array_equal(ko, k.astype(np.float64))
    np.testing.assert_array_equal(vo, v.astype(np.float64))


def test_gate_one_holds_initial_state():
    k, v, g = _rand(1, 2, 40, 8, seed=3)
    s0k = np.random.default_rng(30).standard_normal((1, 2, 8))
    s0v = np.random.default_rng(31).standard_normal((1, 2, 8))
    ko, vo, sk, sv = oracle.rat_scan(k, v, np.ones_like(g), s0k, s0v)
    np.testing.assert_array_equal(ko, np.broadcast_to(s0k[:, :, None, :], ko.shape))
    np.testing.assert_array_equal(vo, np.broadcast_to(s0v[:, :, None, :], vo.shape))
    np.testing.assert_array_equal(sk, s0k)


@pytest.mark.parametrize("c", [0.5, 0.9, float(1 / (1 + np.exp(-4.2)))])
def test_constant_gate_is_geometric_ema(c):
    T, D = 300, 3
    cf = np.float32(c)
    c = float(cf)
    ones = np.ones((1, 1, T, D), dtype=np.float32)
    g = np.full((1, 1, T, D), cf, dtype=np.float32)
    ko, vo, _, _ = oracle.rat_scan(ones, 2 * ones, g)
    t = np.arange(1, T + 1, dtype=np.float64)
    np.testing.assert_allclose(ko[0, 0, :, 0], 1 - c ** t, rtol=1e-12)
    np.testing.assert_allclose(vo[0, 0, :, 1], 2 * (1 - c ** t), rtol=1e-12)
    # one-pole IIR filter y_t = c y_{t-1} + (1-c) x_t from a signal-processing library
    x = np.random.default_rng(4).standard_normal(T).astype(np.float32)
    kx = np.repeat(x[None, None, :, None], D, axis=3)
    ko, _, _, _ = oracle.rat_scan(kx, kx, g)
    np.testing.assert_allclose(ko[0, 0, :, 2], lfilter([1 - c], [1, -c], x.astype(np.float64)),
                               rtol=1e-10, atol=1e-13)


def test_impulse_response_and_effective_memory():
    # impulse at t=0 => k~_t = (1-g) g^t: weights sum to 1, mean lag g/(1-g); the gate
    # centre sigmoid(4.2) gives the "effective recurrence length of 64" regime of Sec. 2.1
    T = 4000
    c = np.float32(1 / (1 + np.exp(-4.2)))
    x = np.zeros((1, 1, T, 1), dtype=np.float32)
    x[0, 0, 0, 0] = 1
    ko, _, _, _ = oracle.rat_scan(x, x, np.full_like(x, c))
    w = ko[0, 0, :, 0]
    assert abs(w.sum() - 1) < 1e-12
    lag = float((np.arange(T) * w).sum())
    assert abs(lag - float(c) / (1 - float(c))) < 1e-6
    assert 60 <= lag + 1 <= 70


def test_convex_combination_bounds():
    k, v, g = _rand(1, 1, 200, 16, seed=5)
    ko, _, _, _ = oracle.rat_scan(k, v, g)
    lo = np.minimum(0, np.minimum.accumulate(k[0, 0].astype(np.float64), axis=0))
    hi = np.maximum(0, np.maximum.accumulate(k[0, 0].astype(np.float64), axis=0))
    assert np.all(ko[0, 0] >= lo - 1e-15) and np.all(ko[0, 0] <= hi + 1e-15)


@pytest.mark.parametrize("cut", [1, 17, 128, 255])
def test_split_invariance_with_carry(cut):
    k, v, g = _rand(2, 3, 256, 8, seed=6)
    ko, vo, sk, sv = oracle.rat_scan(k, v, g)
    k1, v1, s1k, s1v = oracle.rat_scan(k[:, :, :cut], v[:, :, :cut], g[:, :, :cut])
    k2, v2, s2k, s2v = oracle.rat_scan(k[:, :, cut:], v[:, :, cut:], g[:, :, cut:], s1k, s1v)
    np.testing.assert_array_equal(np.concatenate([k1, k2], axis=2), ko)
    np.testing.assert_array_equal(np.concatenate([v1, v2], axis=2), vo)
    np.testing.assert_array_equal(s2k, sk)
    np.testing.assert_array_equal(s2v, sv)


def test_units_and_channels_are_independent():
    k, v, g = _rand(2, 2, 50, 6, seed=7)
    ko, vo, _, _ = oracle.rat_scan(k, v, g)
    k2 = k.copy()
    k2[1, 0, :, 3] += 1
    ko2, vo2, _, _ = oracle.rat_scan(k2, v, g)
    diff = np.abs(ko2 - ko) > 0
    assert diff[1, 0, :, 3].all()
    diff[1, 0, :, 3] = False
    assert not diff.any()
    np.testing.assert_array_equal(vo2, vo)


def test_round_to_bf16_matches_torch_and_is_direct():
    torch = pytest.importorskip("torch")
    r = np.random.default_rng(8)
    x32 = (r.standard_normal(20000) * np.exp(r.uniform(-30, 30, 20000))).astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(oracle.round_to_bf16(x32.astype(np.float64)), want)
    # exact halfway cases go to the even neighbour
    np.testing.assert_array_equal(oracle.round_to_bf16(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8])),
                                  np.array([1.0, 1 + 2.0 ** -6], dtype=np.float32))
    # a double just above a halfway point must round up even though its float32
    # rounding would land exactly on the tie (no double rounding)
    x = 1 + 2.0 ** -8 + 2.0 ** -40
    assert np.float32(x) == np.float32(1 + 2.0 ** -8)
    assert oracle.round_to_bf16(np.array([x]))[0] == np.float32(1 + 2.0 ** -7)
