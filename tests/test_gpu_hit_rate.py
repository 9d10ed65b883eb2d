"""The strict head-level hit rate of Sec. 2.3 (H1) as an instrument: the GPU kernel that folds each
decode step's page lists into per-head flags against the oracle's plain statement of the definition,
on a decode chain of the C2 shape (grouped-query heads, planted needles as golden positions)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import say, to_dev, to_np
from paper_2605_28640_amd import synth

pytestmark = pytest.mark.gpu


def gold_positions(w, step):
    """Golden token position of every (batch, query head) at a decode step: planted needle
    (step mod n) of the head's KV head (the decode queries look for the needles)."""
    g = np.full((w.B, w.Hq), -1, dtype=np.int32)
    for b in range(w.B):
        for h in range(w.Hq):
            pos = synth.needle_positions(w, b, h // w.G)
            if len(pos):
                g[b, h] = int(pos[step % len(pos)])
    return g


@pytest.mark.parametrize("K", [32, 2])
def test_hit_rate_of_a_decode_chain(rs, K):
    w = synth.C2.scaled(B=2, T=4096, steps=24)
    P, T = w.P, w.T
    say("hit rate", w.name, "T", T, "K", K)
    Tcap = T + 64
    k, v, g = synth.prefill(w)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, P, torch.bfloat16)
    kc = torch.zeros(w.B, w.Hkv, Tcap, w.D, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    sk = torch.zeros(w.B, w.Hkv, w.D, device="cuda")
    sv = torch.zeros_like(sk)
    meta = torch.zeros(w.B, w.Hkv, Tcap // P, 2, w.D, dtype=torch.bfloat16, device="cuda")
    ws = rs.Workspace(max(rs.rat_scan_workspace_bytes(s, T), rs.sparse_attn_decode_workspace_bytes(s, Tcap, K)))
    rs.rat_scan(s, to_dev(k, "bf16"), to_dev(v, "bf16"), to_dev(g), sk, sv, kc, vc, 0, T, ws, meta)
    out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros(w.B, w.Hq, K, dtype=torch.int32, device="cuda")
    hit = torch.ones(w.B, w.Hq, dtype=torch.uint8, device="cuda")
    scale = 1.0 / np.sqrt(w.D)
    gpu_lists, ref_lists, golds = [], [], []
    for i in range(w.steps):
        kd, vd, gd, qd = synth.decode_step(w, i)
        t = T + i
        rs.rat_scan(s, to_dev(kd, "bf16"), to_dev(vd, "bf16"), to_dev(gd), sk, sv, kc, vc, t, 1, None, meta)
        rs.sparse_attn_decode(s, to_dev(qd, "bf16"), kc, vc, t + 1, scale, None, K, meta, 1, 1, out, None, idx, ws)
        gold = gold_positions(w, i)
        if i % 5 == 4:
            gold[:, ::3] = -1  # some heads have no golden position at some steps
        rs.selection_hit_update(idx, to_dev(gold), P, hit)
        gpu_lists.append(to_np(idx).copy())
        golds.append(gold)
        Np = -(-(t + 1) // P)
        ometa = oracle.quest_page_meta(to_np(kc), P, t + 1)
        ref_lists.append(oracle.quest_select(oracle.quest_scores(qd, ometa, Np), K, 1, 1))
    ws.async_status()
    got = to_np(hit).astype(bool)
    want = oracle.head_hit(gpu_lists, golds, unit=P)   # the instrument itself: same lists, bit for bit
    np.testing.assert_array_equal(got, want)
    ref = oracle.head_hit(ref_lists, golds, unit=P)    # and the oracle's own selections
    same = sum(np.array_equal(a, b) for a, b in zip(gpu_lists, ref_lists))
    say("  hit rate gpu %.3f oracle %.3f; steps with identical lists %d of %d" % (got.mean(), ref.mean(), same, w.steps))
    if same == w.steps:  # identical selections: identical hits (a near-tie at the K-th score may otherwise decide one)
        np.testing.assert_array_equal(got, ref)
    else:
        assert np.mean(got != ref) <= 1.0 / 16
    if K == 32:
        assert got.mean() > 0.0   # some heads hold their needle's page at every step ...
    else:
        assert got.mean() == 0.0  # ... and K = 2 (the first and the last page only) never does
