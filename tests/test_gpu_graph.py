"""The prefill entry points (MoBA routing, block-sparse attention, SnapKV compression, page
metadata) keep no per-call state on the host, so a HIP graph that captured them can be
replayed: every replay, with fresh inputs copied into the captured buffers and eager work in
between, must give the eager result bit for bit."""
import numpy as np
import pytest
import torch

from gpu_util import say
from paper_2605_28640_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("form", ["0", "1"])  # routed attention regrouped by block / by bit sets
def test_prefill_path_replays_from_a_captured_graph(rs, knobs, form):
    knobs.setenv("RATSPARSE_PREFILL_MASKED", form)
    B, H, D, T, block, K = 1, 8, 128, 1024, 128, 3
    dt = torch.bfloat16
    s = rs.make_shape(B, H, H, D, T, 16, dt)
    gen = torch.Generator(device="cuda").manual_seed(5)
    q = torch.randn(B, H, T, D, device="cuda", generator=gen).to(dt)
    kc = (torch.randn(B, H, T, D, device="cuda", generator=gen) * 0.5).to(dt)
    vc = torch.randn(B, H, T, D, device="cuda", generator=gen).to(dt)
    Nb = T // block
    means = torch.zeros(B, H, Nb, D, device="cuda")
    idx = torch.zeros(B, H, T, K, dtype=torch.int32, device="cuda")
    out = torch.zeros(B, H, T, D, dtype=dt, device="cuda")
    meta = torch.zeros(B, H, T // 16, 2, D, dtype=dt, device="cuda")
    ws = rs.Workspace(max(rs.moba_select_prefill_workspace_bytes(s, T, block),
                          rs.sparse_attn_prefill_workspace_bytes(s, T, block, K)))
    scale = 1.0 / np.sqrt(D)

    def run():
        rs.quest_page_meta(s, kc, meta, 0, T)
        rs.moba_select_prefill(s, q, kc, T, block, K, 0, means, idx, ws)
        rs.sparse_attn_prefill(s, q, kc, vc, T, block, scale, idx, K, out, None, ws)

    run()  # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()
    for rep in range(3):
        say("graph replay", rep)
        q.copy_(torch.randn(B, H, T, D, device="cuda", generator=gen).to(dt))
        kc.copy_((torch.randn(B, H, T, D, device="cuda", generator=gen) * 0.5).to(dt))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (idx.clone(), out.clone(), meta.clone())
        idx.zero_(), out.zero_(), meta.zero_()
        run()  # the same inputs, eagerly
        torch.cuda.synchronize()
        assert torch.equal(got[0], idx) and torch.equal(got[2], meta)
        assert torch.equal(got[1], out)
    ws.async_status()


@pytest.mark.parametrize("with_lse", [False, True])  # snapkv_compress / snapkv_compress_lse
def test_snapkv_compress_replays_from_a_captured_graph(rs, with_lse):
    B, Hq, Hkv, D, T, W, keep = 1, 8, 2, 128, 3000, 32, 400
    dt = torch.bfloat16
    Tcap = 3008
    s = rs.make_shape(B, Hq, Hkv, D, Tcap, 16, dt)
    gen = torch.Generator(device="cuda").manual_seed(9)
    qw = torch.randn(B, Hq, W, D, device="cuda", generator=gen).to(dt)
    kc = (torch.randn(B, Hkv, Tcap, D, device="cuda", generator=gen) * 0.5).to(dt)
    vc = torch.randn(B, Hkv, Tcap, D, device="cuda", generator=gen).to(dt)
    Tco = keep + W + 16
    kco = torch.zeros(B, Hkv, Tco, D, dtype=dt, device="cuda")
    vco = torch.zeros_like(kco)
    idx = torch.zeros(B, Hkv, keep, dtype=torch.int32, device="cuda")
    ws = rs.Workspace(rs.snapkv_compress_workspace_bytes(s, T, W))
    scale = 1.0 / np.sqrt(D)

    # For the replay check any finite normaliser will do: the votes only have to come out the same.
    lse = torch.randn(B, Hq, W, device="cuda", generator=gen) + 8.0

    def run():
        if with_lse:
            rs.snapkv_compress_lse(s, qw, kc, vc, T, W, keep, 7, scale, lse, kco, vco, Tco, idx, None, ws)
        else:
            rs.snapkv_compress(s, qw, kc, vc, T, W, keep, 7, scale, kco, vco, Tco, idx, None, ws)

    run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()
    for rep in range(3):
        say("snapkv graph replay", rep)
        qw.copy_(torch.randn(B, Hq, W, D, device="cuda", generator=gen).to(dt))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (idx.clone(), kco.clone(), vco.clone())
        idx.zero_(), kco.zero_(), vco.zero_()
        run()
        torch.cuda.synchronize()
        assert torch.equal(got[0], idx) and torch.equal(got[1], kco) and torch.equal(got[2], vco)
    ws.async_status()
