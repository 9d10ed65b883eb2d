"""Parity at the full sizes of the measured configurations, in the launch configuration
bench.py times.  The GPU path runs on the whole workload; the float64 oracle recomputes
sampled (batch, head) units, rows and steps one by one.  Each stage is compared on identical
stored bits: the scan against the oracle's scan of the same inputs, every later stage
against the oracle applied to the cache rows the GPU stored."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import say, to_dev, to_np
from helpers import attn_close, bf16_store_ok, scan_close, topk_set_ok
from paper_2605_28640_amd import synth

pytestmark = pytest.mark.gpu


def _prefill_on_gpu(rs, w, Tcap, P=16):
    k, v, g = synth.prefill(w)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, P, torch.bfloat16)
    kc = torch.zeros(w.B, w.Hkv, Tcap, w.D, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    sk = torch.zeros(w.B, w.Hkv, w.D, device="cuda")
    sv = torch.zeros_like(sk)
    ws = rs.Workspace(rs.rat_scan_workspace_bytes(s, w.T))
    rs.rat_scan(s, to_dev(k, "bf16"), to_dev(v, "bf16"), to_dev(g), sk, sv, kc, vc, 0, w.T, ws)
    torch.cuda.synchronize()
    ws.async_status()
    return s, (k, v, g), kc, vc, sk, sv


def _check_scan_units(units, inputs, kc, vc, sk, sv, T):
    k, v, g = inputs
    states = {}
    for (b, h) in units:
        ko, vo, osk, osv = oracle.rat_scan(k[b:b + 1, h:h + 1], v[b:b + 1, h:h + 1], g[b:b + 1, h:h + 1])
        assert bf16_store_ok(to_np(kc[b, h, :T]), ko[0, 0]) and bf16_store_ok(to_np(vc[b, h, :T]), vo[0, 0])
        assert scan_close(to_np(sk[b, h]), osk[0, 0])[0] and scan_close(to_np(sv[b, h]), osv[0, 0])[0]
        exact = np.mean(to_np(kc[b, h, :T]) == oracle.round_to_bf16(ko[0, 0]))
        assert exact > 0.999, exact
        states[(b, h)] = (osk, osv)
    return states


def _decode_run(rs, w, units, runs, dtype="bf16", dense_check=False):
    """Full-size Quest decode: prefill scan and bulk page metadata once, then for each
    (budget, steps, check_steps) of `runs` the decode steps of append + page-meta update + fused
    select/attend from the state after the prefill, checked on sampled units and steps against the
    oracle (every run rewrites the same appended rows, so it starts from the same cache)."""
    P = w.P
    bf = dtype == "bf16"
    tdt = torch.bfloat16 if bf else torch.float32
    max_steps = max(st for _, st, _ in runs)
    Tcap = w.T + ((max_steps + 16 + P - 1) // P) * P
    if bf:
        s, inputs, kc, vc, sk, sv = _prefill_on_gpu(rs, w, Tcap, P)
        states0 = _check_scan_units(sorted(set((b, kvh) for (b, kvh, _) in units)), inputs, kc, vc, sk, sv, w.T)
    else:
        k, v, g = synth.prefill(w)
        s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, P, tdt)
        kc = torch.zeros(w.B, w.Hkv, Tcap, w.D, device="cuda")
        vc = torch.zeros_like(kc)
        sk = torch.zeros(w.B, w.Hkv, w.D, device="cuda")
        sv = torch.zeros_like(sk)
        wsp = rs.Workspace(rs.rat_scan_workspace_bytes(s, w.T))
        rs.rat_scan(s, to_dev(k), to_dev(v), to_dev(g), sk, sv, kc, vc, 0, w.T, wsp)
        torch.cuda.synchronize()
        wsp.async_status()
        states0 = {}
        for (b, kvh) in sorted(set((b, kvh) for (b, kvh, _) in units)):
            ko, vo, osk, osv = oracle.rat_scan(k[b:b + 1, kvh:kvh + 1], v[b:b + 1, kvh:kvh + 1], g[b:b + 1, kvh:kvh + 1])
            assert scan_close(to_np(kc[b, kvh, :w.T]), ko[0, 0])[0] and scan_close(to_np(vc[b, kvh, :w.T]), vo[0, 0])[0]
            assert scan_close(to_np(sk[b, kvh]), osk[0, 0])[0] and scan_close(to_np(sv[b, kvh]), osv[0, 0])[0]
            states0[(b, kvh)] = (osk, osv)
        inputs = None
    del inputs
    stored_ok = bf16_store_ok if bf else (lambda x, y: scan_close(x, y)[0])
    tol = 2e-2 if bf else 1e-4
    meta = torch.zeros(w.B, w.Hkv, Tcap // P, 2, w.D, dtype=tdt, device="cuda")
    rs.quest_page_meta(s, kc, meta, 0, w.T)
    sk0, sv0 = sk.clone(), sv.clone()
    scale = 1.0 / np.sqrt(w.D)
    out = torch.zeros(w.B, w.Hq, w.D, dtype=tdt, device="cuda")
    for budget, steps, check_steps in runs:
        K = int(round(budget * (w.T // P)))
        say("  budget", budget, "K", K, "steps", steps)
        sk.copy_(sk0)
        sv.copy_(sv0)
        states = dict(states0)
        idx = torch.zeros(w.B, w.Hq, K, dtype=torch.int32, device="cuda")
        ws = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, Tcap, K))
        identical = checked = 0
        for i in range(steps):
            kd, vd, gd, qd = synth.decode_step(w, i)
            t = w.T + i
            rs.rat_scan(s, to_dev(kd, dtype), to_dev(vd, dtype), to_dev(gd), sk, sv, kc, vc, t, 1, None, meta)
            rs.sparse_attn_decode(s, to_dev(qd, dtype), kc, vc, t + 1, scale, None, K, meta, 1, 1, out, None, idx, ws)
            for (b, kvh) in states:  # the oracle follows every append of its units
                osk, osv = states[(b, kvh)]
                ko, vo, osk, osv = oracle.rat_scan(kd[b:b + 1, kvh:kvh + 1], vd[b:b + 1, kvh:kvh + 1],
                                                   gd[b:b + 1, kvh:kvh + 1], osk, osv)
                states[(b, kvh)] = (osk, osv)
                if i in check_steps:
                    assert stored_ok(to_np(kc[b, kvh, t]), ko[0, 0, 0]) and stored_ok(to_np(vc[b, kvh, t]), vo[0, 0, 0])
            if i not in check_steps:
                continue
            Tv = t + 1
            Np = -(-Tv // P)
            forced = np.zeros(Np, bool)
            forced[0] = forced[-1] = True
            for (b, kvh, h) in units:
                hk = to_np(kc[b:b + 1, kvh:kvh + 1])  # the rows the GPU stored
                hv = to_np(vc[b:b + 1, kvh:kvh + 1])
                ometa = oracle.quest_page_meta(hk, P, Tv)
                np.testing.assert_array_equal(to_np(meta[b, kvh, :Np]), ometa[0, 0, :Np])
                osc = oracle.quest_scores(qd[b:b + 1, h:h + 1], ometa, Np)
                got = to_np(idx[b, h])
                ok, why = topk_set_ok(osc[0, 0], forced, K, got)
                assert ok, (budget, i, b, h, why)
                identical += np.array_equal(got, oracle.quest_select(osc, K, 1, 1)[0, 0])
                checked += 1
                want, _ = oracle.sparse_attn_decode(qd[b:b + 1, h:h + 1], hk, hv, P, Tv, scale, got[None, None])
                ok, worst = attn_close(to_np(out[b, h]), want[0, 0], tol)
                assert ok, (budget, i, b, h, worst)
                if dense_check:  # full budget: every page selected equals the dense path, and both the oracle's dense result
                    outd = torch.zeros_like(out)
                    idxd = torch.zeros(w.B, w.Hq, Np, dtype=torch.int32, device="cuda")
                    wsd = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, Tcap, Np))
                    rs.sparse_attn_decode(s, to_dev(qd, dtype), kc, vc, Tv, scale, None, Np, meta, 1, 1, outd, None, idxd, wsd)
                    np.testing.assert_array_equal(to_np(idxd[b, h]), np.arange(Np))
                    wantd, _ = oracle.sparse_attn_decode(qd[b:b + 1, h:h + 1], hk, hv, P, Tv, scale)
                    assert attn_close(to_np(outd[b, h]), wantd[0, 0], tol)[0]
                    rs.sparse_attn_decode(s, to_dev(qd, dtype), kc, vc, Tv, scale, None, 0, None, 0, 0, outd, None, None, wsd)
                    assert attn_close(to_np(outd[b, h]), wantd[0, 0], tol)[0]
                    wsd.async_status()
        torch.cuda.synchronize()
        ws.async_status()
        say("  selections identical to the oracle's: %d of %d" % (identical, checked))


def test_c1_tiny_fp32_decode_chain(rs):
    """configs[0] as a chain: prefill scan, then all 16 decode steps (append + page bounds + select +
    attend) with 16-token pages at budget 1/8 (K = 16 of 128 pages), float32, every unit and every step
    against the oracle, and at every step the full-budget selection and the dense path against the
    oracle's dense attention (Eq. 1, 3, 4; App. A.1, Quest)."""
    w = synth.C1
    say("full size", w.name)
    units = [(b, h, h) for b in range(w.B) for h in range(w.Hq)]
    _decode_run(rs, w, units, [(1 / 8, w.steps, set(range(w.steps)))], dtype="f32", dense_check=True)


def test_c3_olmo_decode_64k(rs):
    """configs[2] at both of its budgets: 1/16 (K = 256, the headline launch) over all 512 steps and
    1/4 (K = 1024: other slice counts in the persistent launch) over 96 steps."""
    w = synth.C3
    say("full size", w.name)
    checks = {0, 1, 2, 255, 511} | set(range(31, 512, 32))
    _decode_run(rs, w, units=[(0, 0, 0), (3, 17, 17)],
                runs=[(1 / 16, w.steps, checks), (1 / 4, 96, {0, 1, 2, 15, 16, 47, 95})])


def test_c2_gqa_decode_32k(rs):
    """configs[1] at its three budgets (1/4, 1/8, 1/16), grouped-query heads."""
    w = synth.C2
    say("full size", w.name)
    checks = {0, 1, 2, 127, 255} | set(range(15, 256, 16))
    _decode_run(rs, w, units=[(0, 0, 1), (0, 5, 22)],
                runs=[(1 / 4, 64, checks), (1 / 8, 64, checks), (1 / 16, w.steps, checks)])


def test_c4_moba_prefill_32k(rs):
    w = synth.C4
    say("full size", w.name)
    T, block, K = w.T, w.block, w.topk_blocks
    s, inputs, kc, vc, sk, sv = _prefill_on_gpu(rs, w, T)
    _check_scan_units([(0, 3)], inputs, kc, vc, sk, sv, T)
    del inputs
    Nb = T // block
    heads = [3, 30]
    q_heads = {h: synth.prefill_queries_unit(w, 0, h) for h in heads}
    q = torch.zeros(w.B, w.Hq, T, w.D, dtype=torch.bfloat16, device="cuda")
    for h in range(w.Hq):
        q[0, h] = to_dev(q_heads[h] if h in q_heads else synth.prefill_queries_unit(w, 0, h), "bf16")
    means = torch.zeros(w.B, w.Hkv, Nb, w.D, device="cuda")
    idx = torch.zeros(w.B, w.Hq, T, K, dtype=torch.int32, device="cuda")
    out = torch.zeros(w.B, w.Hq, T, w.D, dtype=torch.bfloat16, device="cuda")
    ws = rs.Workspace(max(rs.moba_select_prefill_workspace_bytes(s, T, block),
                          rs.sparse_attn_prefill_workspace_bytes(s, T, block, K)))
    scale = 1.0 / np.sqrt(w.D)
    rs.moba_select_prefill(s, q, kc, T, block, K, 0, means, idx, ws)
    rs.sparse_attn_prefill(s, q, kc, vc, T, block, scale, idx, K, out, None, ws)
    torch.cuda.synchronize()
    rows = sorted(set([0, 1, 511, 512, 513, 1023, 16383, 16384, T - 1]) |
                  set(int(x) for x in np.random.default_rng(4).integers(0, T, 200)))
    for h in heads:
        hk, hv = to_np(kc[0:1, h:h + 1]), to_np(vc[0:1, h:h + 1])
        omeans = oracle.moba_block_means(hk, T, block)
        np.testing.assert_allclose(to_np(means[0, h]), omeans[0, 0], rtol=1e-5, atol=1e-6)
        qh = q_heads[h][None, None]
        gidx = to_np(idx[0, h])
        for t in rows:
            oi, osc = oracle.moba_select(qh, omeans, T, block, K, 0, t_begin=t, t_end=t + 1, want_scores=True)
            own = t // block
            take = min(K, own + 1)
            sc = np.where(np.isnan(osc[0, 0, 0, :own + 1]), 0.0, osc[0, 0, 0, :own + 1])
            forced = np.zeros(own + 1, bool)
            forced[own] = True
            ok, why = topk_set_ok(sc, forced, take, gidx[t, :take])
            assert ok and np.all(gidx[t, take:] == -1), (h, t, why, gidx[t])
            want, _ = oracle.sparse_attn_prefill(qh, hk, hv, T, block, scale, gidx[None, None, t:t + 1],
                                                 t_begin=t, t_end=t + 1)
            ok, worst = attn_close(to_np(out[0, h, t]), want[0, 0, 0])
            assert ok, (h, t, worst)
    ws.async_status()


def test_c5_snapkv_128k(rs):
    w = synth.C5
    say("full size", w.name)
    T, W = w.T, w.W
    K_keep = int(round(w.keep_frac * T))
    s, inputs, kc, vc, sk, sv = _prefill_on_gpu(rs, w, T)
    _check_scan_units([(0, 6)], inputs, kc, vc, sk, sv, T)
    del inputs
    qw = synth.window_queries(w)
    Tco = K_keep + W + 256
    kco = torch.zeros(w.B, w.Hkv, Tco, w.D, dtype=torch.bfloat16, device="cuda")
    vco = torch.zeros_like(kco)
    idx = torch.zeros(w.B, w.Hkv, K_keep, dtype=torch.int32, device="cuda")
    votes = torch.zeros(w.B, w.Hkv, T - W, device="cuda")
    ws = rs.Workspace(rs.snapkv_compress_workspace_bytes(s, T, W))
    scale = 1.0 / np.sqrt(w.D)
    rs.snapkv_compress(s, to_dev(qw, "bf16"), kc, vc, T, W, K_keep, w.pool, scale, kco, vco, Tco, idx, votes, ws)
    torch.cuda.synchronize()
    kvh = 6
    G = w.G
    hk, hv = to_np(kc[0:1, kvh:kvh + 1]), to_np(vc[0:1, kvh:kvh + 1])
    ov = oracle.snapkv_votes(qw[:, kvh * G:(kvh + 1) * G], hk, T, scale)
    op = oracle.maxpool1d(ov, w.pool)
    np.testing.assert_allclose(to_np(votes[0, kvh]), op[0, 0], rtol=3e-4, atol=1e-10)
    got = to_np(idx[0, kvh])
    ok, why = topk_set_ok(op[0, 0], np.zeros(T - W, bool), K_keep, got)
    assert ok, why
    for pos in synth.needle_positions(w, 0, kvh):  # the planted needles survive the compression
        assert pos in got
    rows = np.concatenate([got, np.arange(T - W, T)])
    np.testing.assert_array_equal(to_np(kco[0, kvh, :K_keep + W]), hk[0, 0, rows])
    np.testing.assert_array_equal(to_np(vco[0, kvh, :K_keep + W]), hv[0, 0, rows])
    # the one-sweep form: the window rows' log-sum-exp handed in (here from float32 torch ops on
    # the same cache; a prefill would supply it), against the same oracle votes
    qd_ = to_dev(qw, "bf16").float().view(w.B, w.Hkv, G * W, w.D)
    logits = torch.matmul(qd_, kc[:, :, :T].float().transpose(2, 3)).view(w.B, w.Hq, W, T) * scale
    future = torch.arange(T, device="cuda")[None, :] > (T - W + torch.arange(W, device="cuda"))[:, None]
    lse = torch.logsumexp(logits.masked_fill(future, float("-inf")), dim=-1).contiguous()
    del logits
    kco2, vco2, idx2, votes2 = torch.zeros_like(kco), torch.zeros_like(vco), torch.zeros_like(idx), torch.zeros_like(votes)
    rs.snapkv_compress_lse(s, to_dev(qw, "bf16"), kc, vc, T, W, K_keep, w.pool, scale, lse, kco2, vco2, Tco, idx2,
                           votes2, ws)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_np(votes2[0, kvh]), op[0, 0], rtol=3e-4, atol=1e-10)
    got2 = to_np(idx2[0, kvh])
    ok, why = topk_set_ok(op[0, 0], np.zeros(T - W, bool), K_keep, got2)
    assert ok, why
    rows2 = np.concatenate([got2, np.arange(T - W, T)])
    np.testing.assert_array_equal(to_np(kco2[0, kvh, :K_keep + W]), hk[0, 0, rows2])
    np.testing.assert_array_equal(to_np(vco2[0, kvh, :K_keep + W]), hv[0, 0, rows2])
    del kco2, vco2
    # dense decode over the compressed cache, a few steps
    sc = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tco, 16, torch.bfloat16)
    sk2 = sk.clone()
    sv2 = sv.clone()
    out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.bfloat16, device="cuda")
    ws2 = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(sc, Tco, 0))
    for i in range(8):
        kd, vd, gd, qd = synth.decode_step(w, i)
        n = K_keep + W + i
        rs.rat_scan(sc, to_dev(kd, "bf16"), to_dev(vd, "bf16"), to_dev(gd), sk2, sv2, kco, vco, n, 1, None)
        rs.sparse_attn_decode(sc, to_dev(qd, "bf16"), kco, vco, n + 1, scale, None, 0, None, 0, 0, out, None, None, ws2)
        ck, cv = to_np(kco[0:1, kvh:kvh + 1]), to_np(vco[0:1, kvh:kvh + 1])
        want, _ = oracle.sparse_attn_decode(qd[:, kvh * G:(kvh + 1) * G], ck, cv, 16, n + 1, scale)
        ok, worst = attn_close(to_np(out[0, kvh * G:(kvh + 1) * G]), want[0])
        assert ok, (i, worst)
    ws.async_status()
