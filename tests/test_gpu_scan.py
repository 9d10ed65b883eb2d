"""GPU parity of rat_scan (Sec. 2.1, Eq. 1) against the float64 oracle, through the C ABI."""
import zlib

import numpy as np
import pytest
import torch

import oracle
from gpu_util import say, tdtype, to_dev, to_np
from helpers import bf16_store_ok, scan_close
from paper_2605_28640_amd import synth

pytestmark = pytest.mark.gpu


def _gate(r, shape, mean=4.2):
    return (1 / (1 + np.exp(-(mean + 0.5 * r.standard_normal(shape))))).astype(np.float32)


def _run_scan(rs, k, v, g, dtype, Tcap, t0=0, sk0=None, sv0=None, pieces=None):
    B, H, T, D = k.shape
    s = rs.make_shape(B, H, H, D, Tcap, 16, tdtype(dtype))
    kc = torch.zeros(B, H, Tcap, D, dtype=tdtype(dtype), device="cuda")
    vc = torch.zeros_like(kc)
    sk = torch.zeros(B, H, D, device="cuda") if sk0 is None else to_dev(sk0.astype(np.float32))
    sv = torch.zeros(B, H, D, device="cuda") if sv0 is None else to_dev(sv0.astype(np.float32))
    ws = rs.Workspace(rs.rat_scan_workspace_bytes(s, T))
    pieces = pieces or [(0, T)]
    for a, b in pieces:
        rs.rat_scan(s, to_dev(k[:, :, a:b], dtype), to_dev(v[:, :, a:b], dtype), to_dev(g[:, :, a:b]),
                    sk, sv, kc, vc, t0 + a, b - a, ws)
    torch.cuda.synchronize()
    ws.async_status()
    return to_np(kc), to_np(vc), to_np(sk), to_np(sv)


def test_c1_tiny_fp32(rs):
    w = synth.C1
    say("scan C1", w)
    k, v, g = synth.prefill(w)
    kc, vc, sk, sv = _run_scan(rs, k, v, g, "f32", w.T + 16)
    ko, vo, osk, osv = oracle.rat_scan(k, v, g)
    for got, want in ((kc[:, :, :w.T], ko), (vc[:, :, :w.T], vo), (sk, osk), (sv, osv)):
        ok, worst = scan_close(got, want)
        assert ok, worst
    assert np.all(kc[:, :, w.T:] == 0) and np.all(vc[:, :, w.T:] == 0)  # nothing written past T


def _random_scan_cases(seed, n):
    rng = np.random.default_rng(seed)
    return [(str(rng.choice(["bf16", "f32"])), int(rng.choice([64, 128])), int(rng.integers(1, 6000)),
             int(rng.integers(1, 3)), int(rng.integers(1, 4))) for _ in range(n)]


@pytest.mark.parametrize("dtype,D,T,B,H", [("bf16", 128, 3 * 128 + 37, 2, 3), ("bf16", 64, 700, 1, 2),
                                           ("f32", 128, 333, 1, 2), ("bf16", 128, 9, 1, 1),
                                           ("bf16", 128, 128, 1, 2)] + _random_scan_cases(20260528, 8))
def test_ragged_lengths_carry_in_and_offset(rs, dtype, D, T, B, H):
    say("scan ragged", dtype, D, T, B, H)
    r = np.random.default_rng(T)
    k = r.standard_normal((B, H, T, D)).astype(np.float32)
    v = r.standard_normal((B, H, T, D)).astype(np.float32)
    if dtype == "bf16":
        k, v = synth.to_bf16_grid(k), synth.to_bf16_grid(v)
    g = _gate(r, (B, H, T, D))
    sk0 = r.standard_normal((B, H, D)).astype(np.float32)
    sv0 = r.standard_normal((B, H, D)).astype(np.float32)
    t0, Tcap = 32, T + 64
    kc, vc, sk, sv = _run_scan(rs, k, v, g, dtype, Tcap, t0=t0, sk0=sk0, sv0=sv0)
    ko, vo, osk, osv = oracle.rat_scan(k, v, g, sk0, sv0)
    assert scan_close(sk, osk)[0] and scan_close(sv, osv)[0]
    if dtype == "f32":
        assert scan_close(kc[:, :, t0:t0 + T], ko)[0] and scan_close(vc[:, :, t0:t0 + T], vo)[0]
    else:
        assert bf16_store_ok(kc[:, :, t0:t0 + T], ko) and bf16_store_ok(vc[:, :, t0:t0 + T], vo)
        exact = np.mean(kc[:, :, t0:t0 + T] == oracle.round_to_bf16(ko))
        assert exact > 0.999, exact  # stored bits equal the oracle's rounding almost everywhere
    assert np.all(kc[:, :, :t0] == 0) and np.all(kc[:, :, t0 + T:] == 0)


@pytest.mark.parametrize("dtype,D,T,B,H", [("bf16", 128, 3 * 512 + 37, 1, 2), ("f32", 64, 1300, 2, 1),
                                           ("bf16", 64, 2048, 1, 3), ("bf16", 128, 20000, 1, 2)])
def test_channel_slab_mode(rs, knobs, dtype, D, T, B, H):
    """The few-heads form of the scan (a unit is a 32-channel slab of a (batch, head), chunks span
    more tokens) gives the same states; the last case also takes it by the library's own choice."""
    say("scan slab", dtype, D, T, B, H)
    if T < 16384:
        knobs.setenv("RATSPARSE_SCAN_SLAB", "1")
    r = np.random.default_rng(T + 1)
    k = r.standard_normal((B, H, T, D)).astype(np.float32)
    v = r.standard_normal((B, H, T, D)).astype(np.float32)
    if dtype == "bf16":
        k, v = synth.to_bf16_grid(k), synth.to_bf16_grid(v)
    g = _gate(r, (B, H, T, D))
    sk0 = r.standard_normal((B, H, D)).astype(np.float32)
    sv0 = r.standard_normal((B, H, D)).astype(np.float32)
    t0, Tcap = 16, T + 32
    kc, vc, sk, sv = _run_scan(rs, k, v, g, dtype, Tcap, t0=t0, sk0=sk0, sv0=sv0)
    ko, vo, osk, osv = oracle.rat_scan(k, v, g, sk0, sv0)
    assert scan_close(sk, osk)[0] and scan_close(sv, osv)[0]
    if dtype == "f32":
        assert scan_close(kc[:, :, t0:t0 + T], ko)[0] and scan_close(vc[:, :, t0:t0 + T], vo)[0]
    else:
        assert bf16_store_ok(kc[:, :, t0:t0 + T], ko) and bf16_store_ok(vc[:, :, t0:t0 + T], vo)
    assert np.all(kc[:, :, :t0] == 0) and np.all(kc[:, :, t0 + T:] == 0)


def test_decode_appends_and_split_invariance(rs):
    B, H, T, D = 1, 2, 600, 128
    r = np.random.default_rng(5)
    k = synth.to_bf16_grid(r.standard_normal((B, H, T, D)).astype(np.float32))
    v = synth.to_bf16_grid(r.standard_normal((B, H, T, D)).astype(np.float32))
    g = _gate(r, (B, H, T, D))
    ko, vo, osk, osv = oracle.rat_scan(k, v, g)
    pieces = [(0, 300), (300, 301), (301, 302), (302, 310), (310, 599), (599, 600)]
    say("scan pieces", pieces)
    kc, vc, sk, sv = _run_scan(rs, k, v, g, "bf16", T, pieces=pieces)
    assert scan_close(sk, osk)[0] and scan_close(sv, osv)[0]
    assert bf16_store_ok(kc, ko) and bf16_store_ok(vc, vo)


def test_special_gates(rs):
    B, H, T, D = 1, 2, 300, 128
    r = np.random.default_rng(6)
    k = synth.to_bf16_grid(r.standard_normal((B, H, T, D)).astype(np.float32))
    v = synth.to_bf16_grid(r.standard_normal((B, H, T, D)).astype(np.float32))
    kc, vc, sk, sv = _run_scan(rs, k, v, np.zeros_like(k), "bf16", T)
    np.testing.assert_array_equal(kc, k)  # g = 0: the cache is the input, bit for bit
    np.testing.assert_array_equal(vc, v)
    s0 = synth.to_bf16_grid(r.standard_normal((B, H, D)).astype(np.float32))
    kc, vc, sk, sv = _run_scan(rs, k, v, np.ones_like(k), "bf16", T, sk0=s0, sv0=-s0)
    np.testing.assert_array_equal(kc, np.broadcast_to(s0[:, :, None], kc.shape))  # g = 1: state held
    np.testing.assert_array_equal(sv, -s0)


def test_expired_wait_is_reported_and_workspace_recovers(rs):
    """A spin bound of zero makes chunks give up instead of waiting: every kernel still
    exits, the failure is reported, and the next call on the same workspace is correct."""
    B, H, T, D = 1, 2, 4096, 128
    r = np.random.default_rng(7)
    k = synth.to_bf16_grid(r.standard_normal((B, H, T, D)).astype(np.float32))
    g = _gate(r, (B, H, T, D))
    s = rs.make_shape(B, H, H, D, T, 16, torch.bfloat16)
    kc = torch.zeros(B, H, T, D, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    sk = torch.zeros(B, H, D, device="cuda")
    sv = torch.zeros_like(sk)
    ws = rs.Workspace(rs.rat_scan_workspace_bytes(s, T))
    tk, tg = to_dev(k, "bf16"), to_dev(g)
    rs.load().ratsparse_debug_set_spin_limit(0)
    try:
        rs.rat_scan(s, tk, tk, tg, sk, sv, kc, vc, 0, T, ws)
        try:
            ws.async_status()
            timed_out = False
        except rs.RatsparseError as e:
            timed_out = "wait expired" in str(e)
            assert timed_out
    finally:
        rs.load().ratsparse_debug_set_spin_limit(1 << 22)
    say("expired wait reported:", timed_out)
    sk.zero_()
    sv.zero_()
    rs.rat_scan(s, tk, tk, tg, sk, sv, kc, vc, 0, T, ws)
    ws.async_status()
    ko, _, osk, _ = oracle.rat_scan(k, k, g)
    assert scan_close(to_np(sk), osk)[0] and bf16_store_ok(to_np(kc), ko)


def _gates(kind, r, shape):
    """Gate regimes over the whole of [0, 1] (the library takes any activated gate, Eq. 1)."""
    if kind == "uniform":
        return r.uniform(0.0, 1.0, shape).astype(np.float32)
    if kind == "near0":
        return (10.0 ** r.uniform(-6.0, -3.0, shape)).astype(np.float32)
    if kind == "near1":
        return (1.0 - 2.0 ** -r.uniform(12.0, 20.0, shape)).astype(np.float32)
    # mixed: every channel of every head keeps one regime for the whole run, a few tokens reset (g = 0) or hold (g = 1)
    B, H, T, D = shape
    pick = r.integers(0, 4, (B, H, 1, D))
    g = np.where(pick == 0, _gates("uniform", r, shape),
                 np.where(pick == 1, _gates("near0", r, shape),
                          np.where(pick == 2, _gates("near1", r, shape), _gate(r, shape))))
    u = r.uniform(0, 1, (B, H, T, 1))
    g = np.where(u < 0.01, 0.0, np.where(u > 0.99, 1.0, g))
    return g.astype(np.float32)


@pytest.mark.parametrize("slab", ["0", "1"])
@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)])
@pytest.mark.parametrize("kind", ["uniform", "near0", "near1", "mixed"])
def test_gate_regimes(rs, knobs, kind, dtype, D, slab):
    """Eq. 1 with gates away from the workloads' sigmoid(N(4.2, 0.5)): uniform on [0, 1], close to 0
    (1e-6 .. 1e-3), close to 1 (1 - 2^-12 .. 1 - 2^-20) and a different regime per channel, in the
    full-row and the 32-channel-slab form, both storage types, several chunks and a ragged tail, with
    a carry-in and an offset, against the float64 oracle at 1e-5."""
    knobs.setenv("RATSPARSE_SCAN_SLAB", slab)
    B, H, T = 1, 2, 2500 + 37
    say("scan gates", kind, dtype, D, "slab", slab)
    r = np.random.default_rng(zlib.crc32(repr((kind, dtype, D, slab)).encode()))
    k = r.standard_normal((B, H, T, D)).astype(np.float32)
    v = r.standard_normal((B, H, T, D)).astype(np.float32)
    if dtype == "bf16":
        k, v = synth.to_bf16_grid(k), synth.to_bf16_grid(v)
    g = _gates(kind, r, (B, H, T, D))
    assert g.min() >= 0.0 and g.max() <= 1.0
    sk0 = r.standard_normal((B, H, D)).astype(np.float32)
    sv0 = r.standard_normal((B, H, D)).astype(np.float32)
    t0, Tcap = 48, T + 64
    kc, vc, sk, sv = _run_scan(rs, k, v, g, dtype, Tcap, t0=t0, sk0=sk0, sv0=sv0)
    ko, vo, osk, osv = oracle.rat_scan(k, v, g, sk0, sv0)
    assert scan_close(sk, osk)[0] and scan_close(sv, osv)[0]
    if dtype == "f32":
        for got, want in ((kc[:, :, t0:t0 + T], ko), (vc[:, :, t0:t0 + T], vo)):
            ok, worst = scan_close(got, want)
            assert ok, worst
    else:
        assert bf16_store_ok(kc[:, :, t0:t0 + T], ko) and bf16_store_ok(vc[:, :, t0:t0 + T], vo)
        exact = np.mean(kc[:, :, t0:t0 + T] == oracle.round_to_bf16(ko))
        assert exact > 0.999, exact
    assert np.all(kc[:, :, :t0] == 0) and np.all(kc[:, :, t0 + T:] == 0)


@pytest.mark.parametrize("dtype,T", [("bf16", 1000), ("f32", 520), ("bf16", 5)])
def test_scan_in_place(rs, dtype, T):
    """The one aliasing the interface allows: k_cache == k and v_cache == v when the layouts coincide
    (t0 = 0, T_new = Tcap)."""
    B, H, D = 2, 2, 128
    say("scan in place", dtype, T)
    r = np.random.default_rng(T)
    k = r.standard_normal((B, H, T, D)).astype(np.float32)
    v = r.standard_normal((B, H, T, D)).astype(np.float32)
    if dtype == "bf16":
        k, v = synth.to_bf16_grid(k), synth.to_bf16_grid(v)
    g = _gate(r, (B, H, T, D))
    s = rs.make_shape(B, H, H, D, T, 16, tdtype(dtype))
    tk, tv = to_dev(k, dtype), to_dev(v, dtype)
    sk = torch.zeros(B, H, D, device="cuda")
    sv = torch.zeros_like(sk)
    ws = rs.Workspace(rs.rat_scan_workspace_bytes(s, T))
    rs.rat_scan(s, tk, tv, to_dev(g), sk, sv, tk, tv, 0, T, ws)
    torch.cuda.synchronize()
    ws.async_status()
    ko, vo, osk, osv = oracle.rat_scan(k, v, g)
    assert scan_close(to_np(sk), osk)[0] and scan_close(to_np(sv), osv)[0]
    if dtype == "f32":
        assert scan_close(to_np(tk), ko)[0] and scan_close(to_np(tv), vo)[0]
    else:
        assert bf16_store_ok(to_np(tk), ko) and bf16_store_ok(to_np(tv), vo)
