"""Degenerate and boundary sizes through the C ABI against the oracle: a one-token cache, K = 1,
a cache filled to its capacity, 128-token pages, a one-token / one-block prefill, top-1 routing
(own block only), SnapKV that keeps nothing or a single position, and a one-row window."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import say, tdtype, to_dev, to_np
from helpers import attn_close, topk_set_ok
from paper_2605_28640_amd import synth

pytestmark = pytest.mark.gpu


def _cache(w, T, Tcap):
    w = w.scaled(T=T, n_needles=w.n_needles if T >= 64 else 0)  # no room for planted keys in a tiny cache
    k, v, g = synth.prefill(w)
    ko, vo, _, _ = oracle.rat_scan(k, v, g)
    kc = np.zeros((w.B, w.Hkv, Tcap, w.D), dtype=np.float32)
    vc = np.zeros_like(kc)
    bf = w.dtype == "bf16"
    kc[:, :, :T] = oracle.round_to_bf16(ko) if bf else ko.astype(np.float32)
    vc[:, :, :T] = oracle.round_to_bf16(vo) if bf else vo.astype(np.float32)
    return w, kc, vc


DECODE = [
    # workload, T_valid, Tcap, P, K, n_first, n_local
    (synth.C1, 1, 16, 16, 1, 0, 1),                                   # one token, one page
    (synth.C1.scaled(dtype="bf16"), 1, 16, 16, 1, 1, 0),              # the same page kept as "first"
    (synth.C2.scaled(Hq=4, Hkv=2), 17, 32, 16, 1, 0, 1),              # K = 1: only the newest page
    (synth.C2.scaled(Hq=4, Hkv=2), 1024, 1024, 16, 7, 1, 1),          # cache filled to its capacity
    (synth.C2.scaled(Hq=4, Hkv=4), 1000, 1024, 128, 3, 1, 1),         # 128-token pages, ragged last page
    (synth.C1, 300, 320, 32, 10, 3, 4),                               # several first / local pages, K = all 10 pages
    # the largest page count the selection takes (15360 keys in LDS), ragged last page
    (synth.C1.scaled(Hq=1, Hkv=1, dtype="bf16"), 15360 * 16 - 3, 15360 * 16, 16, 64, 1, 1),
]


@pytest.mark.parametrize("case", range(len(DECODE)))
def test_decode_edges(rs, knobs, case):
    w, T, Tcap, P, K, n_first, n_local = DECODE[case]
    say("decode edge", case, w.name, T, Tcap, P, K, n_first, n_local)
    w, kc, vc = _cache(w, T, Tcap)
    _, _, _, q = synth.decode_step(w, 0)
    Np = -(-T // P)
    scale = 1.0 / np.sqrt(w.D)
    dt = tdtype(w.dtype)
    tol = 2e-2 if w.dtype == "bf16" else 1e-4
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, P, dt)
    tkc, tvc, tq = to_dev(kc, w.dtype), to_dev(vc, w.dtype), to_dev(q, w.dtype)
    meta = torch.zeros(w.B, w.Hkv, Tcap // P, 2, w.D, dtype=dt, device="cuda")
    ws = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, T, Np))
    rs.quest_page_meta(s, tkc, meta, 0, T)
    ometa = oracle.quest_page_meta(kc, P, T)
    np.testing.assert_array_equal(to_np(meta)[:, :, :Np], ometa[:, :, :Np])
    idx = torch.full((w.B, w.Hq, K), -7, dtype=torch.int32, device="cuda")
    out = torch.zeros(w.B, w.Hq, w.D, dtype=dt, device="cuda")
    lse = torch.zeros(w.B, w.Hq, device="cuda")
    rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, None, K, meta, n_first, n_local, out, lse, idx, ws)
    gidx = to_np(idx)
    for two_launch in ("0", "1"):  # the one persistent launch and the two-launch form agree
        knobs.setenv("RATSPARSE_FUSED_TWO_LAUNCH", two_launch)
        out_m, idx_m = torch.zeros_like(out), torch.full_like(idx, -7)
        rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, None, K, meta, n_first, n_local, out_m, None, idx_m, ws)
        np.testing.assert_array_equal(to_np(idx_m), gidx)
        assert attn_close(to_np(out_m), to_np(out).astype(np.float64), tol)[0]
    knobs.delenv("RATSPARSE_FUSED_TWO_LAUNCH")
    osc = oracle.quest_scores(q, ometa, Np)
    forced = np.zeros(Np, bool)
    forced[:n_first] = True
    forced[Np - n_local:] = True
    oidx = oracle.quest_select(osc, K, n_first, n_local)
    identical = 0
    for b in range(w.B):
        for h in range(w.Hq):
            row = gidx[b, h]
            assert np.all(np.diff(row) > 0) and row[0] >= 0 and row[-1] < Np, row
            assert set(range(n_first)) <= set(row) and set(range(Np - n_local, Np)) <= set(row), row
            ok, why = topk_set_ok(osc[b, h], forced, K, row)  # the selection against the oracle's scores (Eq. 3)
            assert ok, (b, h, why)
            identical += np.array_equal(row, oidx[b, h])
    say("  selections identical to the oracle's: %d of %d" % (identical, w.B * w.Hq))
    want, wlse = oracle.sparse_attn_decode(q, kc, vc, P, T, scale, gidx)
    ok, worst = attn_close(to_np(out), want, tol)
    assert ok, worst
    np.testing.assert_allclose(to_np(lse), wlse, rtol=1e-3, atol=1e-3)
    if K == Np:  # every page: the dense result
        outd = torch.zeros_like(out)
        rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, None, 0, None, 0, 0, outd, None, None, ws)
        assert attn_close(to_np(outd), want, tol)[0]
    torch.cuda.synchronize()
    ws.async_status()


PREFILL = [
    # workload, T, Tcap, block, K
    (synth.C4.scaled(B=1, Hq=2, Hkv=2), 1, 16, 16, 1),      # one token
    (synth.C4.scaled(B=1, Hq=2, Hkv=1), 64, 64, 64, 2),     # one block: nothing to route
    (synth.C4.scaled(B=1, Hq=2, Hkv=2), 300, 304, 32, 1),   # top-1: every token attends its own block only
    (synth.C4.scaled(B=1, Hq=2, Hkv=2, D=64), 129, 144, 128, 2),  # a second block of one token
    (synth.C4.scaled(B=1, Hq=2, Hkv=1, D=64), 4096, 4096, 16, 32),  # the most blocks (256) and the largest K (32)
]


@pytest.mark.parametrize("case", range(len(PREFILL)))
def test_prefill_edges(rs, case):
    w, T, Tcap, block, K = PREFILL[case]
    say("prefill edge", case, T, Tcap, block, K)
    w, kc, vc = _cache(w, T, Tcap)
    q = synth.prefill_queries(w)
    Nb = -(-T // block)
    scale = 1.0 / np.sqrt(w.D)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, 16, torch.bfloat16)
    tq, tkc, tvc = to_dev(q, "bf16"), to_dev(kc, "bf16"), to_dev(vc, "bf16")
    means = torch.zeros(w.B, w.Hkv, Nb, w.D, device="cuda")
    idx = torch.full((w.B, w.Hq, T, K), -9, dtype=torch.int32, device="cuda")
    ws = rs.Workspace(max(rs.moba_select_prefill_workspace_bytes(s, T, block),
                          rs.sparse_attn_prefill_workspace_bytes(s, T, block, K)))
    rs.moba_select_prefill(s, tq, tkc, T, block, K, 0, means, idx, ws)
    gidx = to_np(idx)
    own = np.arange(T) // block
    for t in range(T):
        rows = gidx[:, :, t]
        assert np.all((rows == own[t]).sum(-1) == 1), (t, rows)          # own block always kept
        assert np.all((rows >= 0).sum(-1) == min(K, own[t] + 1)), (t, rows)  # all there is, -1 padded
    out = torch.zeros(w.B, w.Hq, T, w.D, dtype=torch.bfloat16, device="cuda")
    rs.sparse_attn_prefill(s, tq, tkc, tvc, T, block, scale, idx, K, out, None, ws)
    want, _ = oracle.sparse_attn_prefill(q, kc, vc, T, block, scale, gidx)
    ok, worst = attn_close(to_np(out), want)
    assert ok, worst
    rs.sparse_attn_prefill(s, tq, tkc, tvc, T, block, scale, None, 0, out, None, ws)
    wantd, _ = oracle.sparse_attn_prefill(q, kc, vc, T, block, scale)
    assert attn_close(to_np(out), wantd)[0]
    # token 0 attends only itself
    np.testing.assert_allclose(to_np(out)[:, :, 0], np.repeat(vc[:, :, 0], w.Hq // w.Hkv, axis=1), rtol=2 ** -7, atol=1e-6)
    torch.cuda.synchronize()
    ws.async_status()


SNAP = [
    # workload, T, Tcap, K_keep, pool
    (synth.C5.scaled(B=1, Hq=4, Hkv=2, W=32), 200, 208, 0, 7),    # keep nothing but the window
    (synth.C5.scaled(B=1, Hq=2, Hkv=2, W=32), 200, 208, 1, 7),    # a single position
    (synth.C5.scaled(B=1, Hq=2, Hkv=2, W=1), 100, 112, 10, 3),    # a one-row window
    (synth.C5.scaled(B=1, Hq=2, Hkv=2, W=32), 33, 48, 1, 7),      # a one-token prefix
    (synth.C5.scaled(B=1, Hq=2, Hkv=1, W=16), 9000, 9008, 3000, 5),  # three select slices, ragged
]


@pytest.mark.parametrize("case", range(len(SNAP)))
def test_snapkv_edges(rs, case):
    w, T, Tcap, K_keep, pool = SNAP[case]
    say("snapkv edge", case, T, Tcap, K_keep, pool, "W", w.W)
    w, kc, vc = _cache(w, T, Tcap)
    qw = synth.window_queries(w)
    W, L = w.W, T - w.W
    scale = 1.0 / np.sqrt(w.D)
    Tco = ((K_keep + W + 15) // 16) * 16
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, 16, torch.bfloat16)
    ws = rs.Workspace(rs.snapkv_compress_workspace_bytes(s, T, W))
    kco = torch.zeros(w.B, w.Hkv, Tco, w.D, dtype=torch.bfloat16, device="cuda")
    vco = torch.zeros_like(kco)
    idx = torch.full((w.B, w.Hkv, max(K_keep, 1)), -5, dtype=torch.int32, device="cuda")
    votes = torch.zeros(w.B, w.Hkv, L, device="cuda")
    rs.snapkv_compress(s, to_dev(qw, "bf16"), to_dev(kc, "bf16"), to_dev(vc, "bf16"), T, W, K_keep, pool, scale,
                       kco, vco, Tco, idx, votes, ws)
    opooled = oracle.maxpool1d(oracle.snapkv_votes(qw, kc, T, scale), pool)
    np.testing.assert_allclose(to_np(votes), opooled, rtol=2e-4, atol=1e-9)
    gidx = to_np(idx)[:, :, :K_keep]
    for b in range(w.B):
        for h in range(w.Hkv):
            row = gidx[b, h]
            assert np.all(np.diff(row) > 0) and np.all((row >= 0) & (row < L)), row
            if K_keep:
                thr = np.sort(opooled[b, h])[::-1][K_keep - 1]
                assert np.all(opooled[b, h, row] >= thr * (1 - 1e-4) - 1e-12), (row, thr)
            # kept rows, then the window rows
            src = np.concatenate([row, np.arange(L, T)])
            np.testing.assert_array_equal(to_np(kco)[b, h, :K_keep + W], kc[b, h, src])
            np.testing.assert_array_equal(to_np(vco)[b, h, :K_keep + W], vc[b, h, src])
    torch.cuda.synchronize()
    ws.async_status()


def test_out_of_range_knob_values_are_clamped(rs, knobs):
    """The tuning knobs are read at dispatch; values outside their range are clamped to it, so the
    work split changes at most: the scan (whose arithmetic does not depend on the grid) stays bit-equal,
    the persistent decode launch picks the same pages and agrees to the rounding of a different merge order."""
    B, H, D, T, P, K = 2, 4, 128, 2048, 16, 16
    dt = torch.bfloat16
    gen = torch.Generator(device="cuda").manual_seed(23)
    k = torch.randn(B, H, T, D, device="cuda", generator=gen).to(dt)
    v = torch.randn(B, H, T, D, device="cuda", generator=gen).to(dt)
    g = torch.sigmoid(4.2 + 0.5 * torch.randn(B, H, T, D, device="cuda", generator=gen))
    q = torch.randn(B, H, D, device="cuda", generator=gen).to(dt)
    s = rs.make_shape(B, H, H, D, T, P, dt)
    knobs.setenv("RATSPARSE_FUSED_TWO_LAUNCH", "0")  # the persistent launch, where the decode knobs apply
    knobs.setenv("RATSPARSE_FUSED_ONE_WG", "0")

    def run():
        kc = torch.zeros(B, H, T, D, dtype=dt, device="cuda")
        vc = torch.zeros_like(kc)
        sk = torch.zeros(B, H, D, device="cuda")
        sv = torch.zeros_like(sk)
        meta = torch.zeros(B, H, T // P, 2, D, dtype=dt, device="cuda")
        ws = rs.Workspace(max(rs.rat_scan_workspace_bytes(s, T), rs.sparse_attn_decode_workspace_bytes(s, T, K)))
        rs.rat_scan(s, k, v, g, sk, sv, kc, vc, 0, T, ws, meta)
        out = torch.zeros(B, H, D, dtype=dt, device="cuda")
        idx = torch.zeros(B, H, K, dtype=torch.int32, device="cuda")
        rs.sparse_attn_decode(s, q, kc, vc, T, 1.0 / np.sqrt(D), None, K, meta, 1, 1, out, None, idx, ws)
        torch.cuda.synchronize()
        ws.async_status()
        return kc, vc, sk, sv, meta, idx, out

    want = run()
    for values in ({"RATSPARSE_SCAN_GRID": "-1", "RATSPARSE_FUSED_GRID": "-3", "RATSPARSE_FUSED_FINE_PCT": "500"},
                  {"RATSPARSE_SCAN_GRID": "1000000000", "RATSPARSE_FUSED_GRID": "0", "RATSPARSE_FUSED_FINE_PCT": "-7",
                   "RATSPARSE_META_SPW": "1000000"}):
        say("knobs", values)
        for name, value in values.items():
            knobs.setenv(name, value)
        got = run()
        for a, b in zip(got[:6], want[:6]):
            assert torch.equal(a, b)
        assert torch.allclose(got[6].float(), want[6].float(), rtol=2e-2, atol=2e-2)
        for name in values:
            knobs.delenv(name)
