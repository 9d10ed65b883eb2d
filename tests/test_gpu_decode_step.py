"""The replayable decode step (append one token of the gated cache, select pages, attend them,
with the sequence length held on the device) against the two calls it stands for (rat_scan
with one token, then sparse_attn_decode in its fused mode), bit for bit, eagerly and replayed
from a captured HIP graph; and its last step against the float64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import say, tdtype, to_dev, to_np
from helpers import attn_close, bf16_store_ok, scan_close, topk_set_ok
from paper_2605_28640_amd import synth

pytestmark = pytest.mark.gpu


class _Side:
    """One copy of the recurrent state, the caches and the page metadata after a prefill of T0 tokens."""

    def __init__(self, rs, w, s, T0, Tcap, P, k, v, g):
        dt = tdtype(w.dtype)
        self.sk = torch.zeros(w.B, w.Hkv, w.D, device="cuda")
        self.sv = torch.zeros_like(self.sk)
        self.kc = torch.zeros(w.B, w.Hkv, Tcap, w.D, dtype=dt, device="cuda")
        self.vc = torch.zeros_like(self.kc)
        self.meta = torch.zeros(w.B, w.Hkv, Tcap // P, 2, w.D, dtype=dt, device="cuda")
        ws = rs.Workspace(rs.rat_scan_workspace_bytes(s, T0))
        rs.rat_scan(s, k, v, g, self.sk, self.sv, self.kc, self.vc, 0, T0, ws, self.meta)
        torch.cuda.synchronize()

    def same_as(self, o):
        return all(torch.equal(a, b) for a, b in ((self.sk, o.sk), (self.sv, o.sv), (self.kc, o.kc),
                                                   (self.vc, o.vc), (self.meta, o.meta)))


CASES = [
    # workload, T0, steps, Tcap, P, K, n_first, n_local
    (synth.C2.scaled(B=2, Hq=8, Hkv=2), 300, 40, 1024, 16, 8, 1, 1),   # GQA bf16, crosses three page edges
    (synth.C1.scaled(B=1, Hq=4, Hkv=4), 2040, 20, 2304, 64, 5, 0, 1),   # f32 D=64, 64-token pages, one edge
    (synth.C3.scaled(B=1, Hq=8, Hkv=8), 9000, 12, 9216, 16, 36, 1, 2),  # several attention slices per unit
]


def _setup(rs, case):
    w, T0, steps, Tcap, P, K, n_first, n_local = CASES[case]
    w = w.scaled(T=T0)
    dt = tdtype(w.dtype)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, P, dt)
    k, v, g = synth.prefill(w)
    tk, tv, tg = to_dev(k, w.dtype), to_dev(v, w.dtype), to_dev(g)
    a = _Side(rs, w, s, T0, Tcap, P, tk, tv, tg)
    b = _Side(rs, w, s, T0, Tcap, P, tk, tv, tg)
    assert a.same_as(b)
    return w, s, (k, v, g), a, b


def _step_inputs(w, step):
    k, v, g, q = synth.decode_step(w, step)
    return to_dev(k, w.dtype), to_dev(v, w.dtype), to_dev(g), to_dev(q, w.dtype), (k, v, g, q)


def _force_form(knobs, form):
    """Both sides run the same form of select-then-attend: the persistent launch, one workgroup per
    (batch, head), or the two plain launches (the step takes one of the three by shape; the knobs force any)."""
    knobs.setenv("RATSPARSE_FUSED_TWO_LAUNCH", "0" if form == "persistent" else "1")
    knobs.setenv("RATSPARSE_FUSED_ONE_WG", "1" if form == "one_wg" else "0")


FORMS = ["persistent", "one_wg", "two_launch"]


@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("case", range(len(CASES)))
def test_step_equals_scan_then_fused_decode(rs, knobs, case, form):
    _force_form(knobs, form)
    _, T0, steps, Tcap, P, K, n_first, n_local = CASES[case]
    say("decode step case", case, T0, steps, Tcap, P, K)
    w, s, pre, a, b = _setup(rs, case)
    dt = tdtype(w.dtype)
    T_max = T0 + steps
    scale = 1.0 / np.sqrt(w.D)
    ws_a = rs.Workspace(rs.rat_decode_step_workspace_bytes(s, T_max, K))
    ws_b = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, T_max, K))
    rs.rat_decode_state_set(ws_a, T0)
    assert rs.rat_decode_state_get(ws_a) == T0
    out_a = torch.zeros(w.B, w.Hq, w.D, dtype=dt, device="cuda")
    out_b = torch.zeros_like(out_a)
    lse_a, lse_b = torch.zeros(w.B, w.Hq, device="cuda"), torch.zeros(w.B, w.Hq, device="cuda")
    idx_a = torch.zeros(w.B, w.Hq, K, dtype=torch.int32, device="cuda")
    idx_b = torch.zeros_like(idx_a)
    hist = list(pre)  # k, v, g of every token so far, for the oracle
    for t in range(steps):
        tk, tv, tg, tq, host = _step_inputs(w, t)
        rs.rat_decode_step(s, tk, tv, tg, a.sk, a.sv, a.kc, a.vc, a.meta, tq, scale, K, n_first, n_local, T_max,
                           out_a, lse_a, idx_a, ws_a)
        rs.rat_scan(s, tk, tv, tg, b.sk, b.sv, b.kc, b.vc, T0 + t, 1, None, b.meta)
        rs.sparse_attn_decode(s, tq, b.kc, b.vc, T0 + t + 1, scale, None, K, b.meta, n_first, n_local, out_b, lse_b,
                              idx_b, ws_b)
        torch.cuda.synchronize()
        assert torch.equal(idx_a, idx_b), t
        assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b), t
        hist = [np.concatenate([hist[i], host[i]], axis=2) for i in range(3)]
    assert a.same_as(b)
    assert rs.rat_decode_state_get(ws_a) == T_max
    ws_a.async_status()
    ws_b.async_status()

    # the last step against the oracle: scan of every token, selection on the stored keys, attention
    ko, vo, _, _ = oracle.rat_scan(*hist)
    kc = to_np(a.kc)[:, :, :T_max]
    if w.dtype == "bf16":
        assert bf16_store_ok(kc, ko)
    else:
        assert scan_close(kc, ko)[0]
    kfull, vfull = to_np(a.kc), to_np(a.vc)
    Np = -(-T_max // P)
    ometa = oracle.quest_page_meta(kfull, P, T_max)
    np.testing.assert_array_equal(to_np(a.meta)[:, :, :Np], ometa[:, :, :Np])
    osc = oracle.quest_scores(host[3], ometa, Np)
    forced = np.zeros(Np, dtype=bool)
    forced[:n_first] = True
    if n_local:
        forced[Np - n_local:] = True
    gidx = to_np(idx_a)
    for bb in range(w.B):
        for h in range(w.Hq):
            ok, why = topk_set_ok(osc[bb, h], forced, K, gidx[bb, h])
            assert ok, (bb, h, why)
    oout, _ = oracle.sparse_attn_decode(host[3], kfull, vfull, P, T_max, scale, gidx)
    ok, worst = attn_close(to_np(out_a), oout, 2e-2 if w.dtype == "bf16" else 1e-4)
    assert ok, worst


@pytest.mark.parametrize("form", FORMS)
def test_step_past_the_sized_length_changes_nothing_and_reports(rs, knobs, form):
    _force_form(knobs, form)
    w, T0, steps, Tcap, P, K, n_first, n_local = CASES[0]
    w, s, pre, a, b = _setup(rs, 0)
    dt = tdtype(w.dtype)
    scale = 1.0 / np.sqrt(w.D)
    T_max = T0 + 1
    ws = rs.Workspace(rs.rat_decode_step_workspace_bytes(s, T_max, K))
    rs.rat_decode_state_set(ws, T0)
    out = torch.zeros(w.B, w.Hq, w.D, dtype=dt, device="cuda")
    tk, tv, tg, tq, _ = _step_inputs(w, 0)

    def step():
        rs.rat_decode_step(s, tk, tv, tg, a.sk, a.sv, a.kc, a.vc, a.meta, tq, scale, K, n_first, n_local, T_max, out,
                           None, None, ws)

    step()
    ws.async_status()
    assert rs.rat_decode_state_get(ws) == T_max
    keep = (a.sk.clone(), a.kc.clone(), a.meta.clone(), out.clone())
    step()  # one more than the workspace was sized for
    with pytest.raises(rs.RatsparseError):
        ws.async_status()
    assert rs.rat_decode_state_get(ws) == T_max
    assert torch.equal(keep[0], a.sk) and torch.equal(keep[1], a.kc) and torch.equal(keep[2], a.meta)
    assert torch.equal(keep[3], out)


@pytest.mark.parametrize("form", FORMS)
def test_step_with_fewer_pages_than_K_changes_nothing_and_reports(rs, knobs, form):
    """A step taken while the sequence still has fewer pages than K must select (right after
    rat_decode_state_set with a short T) is refused by the attention kernel; the append of the same
    call must then leave the carries, the caches and the page bounds alone too, or a later replay
    would apply the gate to the carry a second time."""
    _force_form(knobs, form)
    w, T0, steps, Tcap, P, K, n_first, n_local = CASES[0]
    w, s, pre, a, b = _setup(rs, 0)
    dt = tdtype(w.dtype)
    scale = 1.0 / np.sqrt(w.D)
    T_max = Tcap
    T_short = 3 * P  # 3 pages, 4 after the append: fewer than K = 8
    assert (T_short + 1 + P - 1) // P < K
    ws = rs.Workspace(rs.rat_decode_step_workspace_bytes(s, T_max, K))
    rs.rat_decode_state_set(ws, T_short)
    out = torch.full((w.B, w.Hq, w.D), 7.0, dtype=dt, device="cuda")
    idx = torch.full((w.B, w.Hq, K), -3, dtype=torch.int32, device="cuda")
    tk, tv, tg, tq, _ = _step_inputs(w, 0)
    keep = [t.clone() for t in (a.sk, a.sv, a.kc, a.vc, a.meta, out, idx)]
    for _ in range(2):  # the second call sees exactly what the first saw
        rs.rat_decode_step(s, tk, tv, tg, a.sk, a.sv, a.kc, a.vc, a.meta, tq, scale, K, n_first, n_local, T_max, out,
                           None, idx, ws)
        with pytest.raises(rs.RatsparseError):
            ws.async_status()
        assert rs.rat_decode_state_get(ws) == T_short
        for was, now in zip(keep, (a.sk, a.sv, a.kc, a.vc, a.meta, out, idx)):
            assert torch.equal(was, now)
    # the first length at which K pages exist goes through, from the same workspace
    T_ok = (K - 1) * P
    rs.rat_decode_state_set(ws, T_ok)
    rs.rat_decode_step(s, tk, tv, tg, a.sk, a.sv, a.kc, a.vc, a.meta, tq, scale, K, n_first, n_local, T_max, out,
                       None, idx, ws)
    ws.async_status()
    assert rs.rat_decode_state_get(ws) == T_ok + 1
    np.testing.assert_array_equal(to_np(idx), np.broadcast_to(np.arange(K, dtype=np.int32), (w.B, w.Hq, K)))


@pytest.mark.parametrize("form", FORMS)
def test_step_replays_from_a_captured_graph(rs, knobs, form):
    _force_form(knobs, form)
    _, T0, steps, Tcap, P, K, n_first, n_local = CASES[0]
    w, s, pre, a, b = _setup(rs, 0)
    dt = tdtype(w.dtype)
    T_max = T0 + steps + 1
    scale = 1.0 / np.sqrt(w.D)
    ws_a = rs.Workspace(rs.rat_decode_step_workspace_bytes(s, T_max, K))
    ws_b = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, T_max, K))
    rs.rat_decode_state_set(ws_a, T0)
    out_a = torch.zeros(w.B, w.Hq, w.D, dtype=dt, device="cuda")
    out_b = torch.zeros_like(out_a)
    idx_a = torch.zeros(w.B, w.Hq, K, dtype=torch.int32, device="cuda")
    idx_b = torch.zeros_like(idx_a)
    tk, tv, tg, tq, _ = _step_inputs(w, 0)

    def step():
        rs.rat_decode_step(s, tk, tv, tg, a.sk, a.sv, a.kc, a.vc, a.meta, tq, scale, K, n_first, n_local, T_max,
                           out_a, None, idx_a, ws_a)

    def eager(t):
        rs.rat_scan(s, tk, tv, tg, b.sk, b.sv, b.kc, b.vc, T0 + t, 1, None, b.meta)
        rs.sparse_attn_decode(s, tq, b.kc, b.vc, T0 + t + 1, scale, None, K, b.meta, n_first, n_local, out_b, None,
                              idx_b, ws_b)

    step()  # step 0 eagerly, outside the capture: it advances the device's count like any other
    eager(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    assert rs.rat_decode_state_get(ws_a) == T0 + 1  # a capture runs nothing
    for t in range(1, steps + 1):
        nk, nv, ng, nq, _ = _step_inputs(w, t)
        tk.copy_(nk), tv.copy_(nv), tg.copy_(ng), tq.copy_(nq)
        torch.cuda.synchronize()
        graph.replay()
        eager(t)
        torch.cuda.synchronize()
        assert torch.equal(idx_a, idx_b), t
        assert torch.equal(out_a, out_b), t
    assert a.same_as(b)
    assert rs.rat_decode_state_get(ws_a) == T0 + steps + 1
    ws_a.async_status()


def test_step_at_the_measured_size_equals_the_two_calls(rs, knobs):
    """The measured configuration (batch 4, 32 heads, 64K context, 256 of 4096+ pages): several
    score and attention slices per unit, page count growing under the fixed work split."""
    _force_form(knobs, "persistent")
    B, H, D, P, K = 4, 32, 128, 16, 256
    T0, steps = 65536 - 6, 14  # crosses the edge of page 4096
    Tcap = 65536 + 64
    T_max = T0 + steps
    dt = torch.bfloat16
    s = rs.make_shape(B, H, H, D, Tcap, P, dt)
    gen = torch.Generator(device="cuda").manual_seed(11)
    sides = []
    kc0 = (torch.randn(B, H, Tcap, D, device="cuda", generator=gen) * 0.5).to(dt)
    vc0 = torch.randn(B, H, Tcap, D, device="cuda", generator=gen).to(dt)
    sk0 = torch.randn(B, H, D, device="cuda", generator=gen)
    sv0 = torch.randn(B, H, D, device="cuda", generator=gen)
    for _ in range(2):
        kc, vc = kc0.clone(), vc0.clone()
        meta = torch.zeros(B, H, Tcap // P, 2, D, dtype=dt, device="cuda")
        rs.quest_page_meta(s, kc, meta, 0, T0)
        sides.append((sk0.clone(), sv0.clone(), kc, vc, meta))
    del kc0, vc0
    a, b = sides
    scale = 1.0 / np.sqrt(D)
    ws_a = rs.Workspace(rs.rat_decode_step_workspace_bytes(s, T_max, K))
    ws_b = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, T_max, K))
    rs.rat_decode_state_set(ws_a, T0)
    out_a = torch.zeros(B, H, D, dtype=dt, device="cuda")
    out_b = torch.zeros_like(out_a)
    idx_a = torch.zeros(B, H, K, dtype=torch.int32, device="cuda")
    idx_b = torch.zeros_like(idx_a)
    for t in range(steps):
        say("full-size decode step", t)
        k = torch.randn(B, H, 1, D, device="cuda", generator=gen).to(dt)
        v = torch.randn(B, H, 1, D, device="cuda", generator=gen).to(dt)
        g = torch.rand(B, H, 1, D, device="cuda", generator=gen)
        q = torch.randn(B, H, D, device="cuda", generator=gen).to(dt)
        rs.rat_decode_step(s, k, v, g, a[0], a[1], a[2], a[3], a[4], q, scale, K, 1, 1, T_max, out_a, None, idx_a, ws_a)
        rs.rat_scan(s, k, v, g, b[0], b[1], b[2], b[3], T0 + t, 1, None, b[4])
        rs.sparse_attn_decode(s, q, b[2], b[3], T0 + t + 1, scale, None, K, b[4], 1, 1, out_b, None, idx_b, ws_b)
        torch.cuda.synchronize()
        assert torch.equal(idx_a, idx_b), t
        assert torch.equal(out_a, out_b), t
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    assert rs.rat_decode_state_get(ws_a) == T_max
    ws_a.async_status()
    ws_b.async_status()
