"""GPU parity of the Quest decode path (page metadata, page selection, attention over the
selected pages, fused select+attend, dense) against the float64 oracle, through the C ABI.
Later stages are fed the oracle's rounded cache so that both sides start from the same
stored bits."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import say, tdtype, to_dev, to_np
from helpers import attn_close, topk_set_ok
from paper_2605_28640_amd import synth

pytestmark = pytest.mark.gpu


def _cache_from_oracle(w, T, Tcap):
    """Oracle scan of the workload's prefill, rounded to the storage dtype."""
    w = w.scaled(T=T)
    k, v, g = synth.prefill(w)
    ko, vo, _, _ = oracle.rat_scan(k, v, g)
    kc = np.zeros((w.B, w.Hkv, Tcap, w.D), dtype=np.float32)
    vc = np.zeros_like(kc)
    if w.dtype == "bf16":
        kc[:, :, :T], vc[:, :, :T] = oracle.round_to_bf16(ko), oracle.round_to_bf16(vo)
    else:
        kc[:, :, :T], vc[:, :, :T] = ko.astype(np.float32), vo.astype(np.float32)
    return w, kc, vc


def _forced(Np, n_first, n_local):
    f = np.zeros(Np, dtype=bool)
    f[:n_first] = True
    if n_local:
        f[Np - n_local:] = True
    return f


CASES = [
    # workload, T_valid, Tcap, P, K, n_first, n_local
    (synth.C1, 2048, 2048 + 16, 16, 16, 1, 1),
    (synth.C1, 2041, 2048 + 16, 16, 16, 1, 1),                       # ragged last page
    (synth.C2.scaled(Hq=8, Hkv=2), 4096 + 5, 4096 + 64, 16, 32, 1, 1),  # GQA, bf16, D=128
    (synth.C3.scaled(B=2, Hq=2, Hkv=2), 8192, 8192, 64, 8, 1, 2),     # 64-token pages
    (synth.C1.scaled(dtype="bf16"), 1000, 1024, 32, 5, 0, 0),          # D=64 bf16, nothing forced
    # the paper's own Quest settings (App. A.1; Tables 3-4): T = 4096, 64-token pages with
    # top-16 / 8 / 4, 16-token pages with top-4
    (synth.C3.scaled(B=1, Hq=4, Hkv=4), 4096, 4096 + 64, 64, 16, 1, 1),
    (synth.C3.scaled(B=1, Hq=4, Hkv=4), 4096, 4096 + 64, 64, 8, 1, 1),
    (synth.C3.scaled(B=1, Hq=4, Hkv=4), 4096, 4096 + 64, 64, 4, 1, 1),
    (synth.C3.scaled(B=1, Hq=4, Hkv=4), 4096, 4096 + 64, 16, 4, 1, 1),
    # large pages
    (synth.C3.scaled(B=1, Hq=4, Hkv=2), 8192 + 77, 8192 + 512, 512, 5, 1, 1),
    (synth.C3.scaled(B=2, Hq=2, Hkv=2), 6000, 6144, 256, 6, 0, 1),
]


def _random_cases(seed, n):
    """Seeded random small shapes: head counts and grouping, both head dims and dtypes, every
    page size, ragged lengths, budgets from one page to all of them, 0-2 forced pages per end."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        Hkv = int(rng.integers(1, 4))
        G = int(rng.choice([1, 2, 4]))
        D = int(rng.choice([64, 128]))
        dtype = str(rng.choice(["bf16", "f32"]))
        P = int(rng.choice([16, 32, 64, 128, 256]))
        T = int(rng.integers(P + 1, 2500))
        Np = -(-T // P)
        Tcap = Np * P + P * int(rng.integers(0, 3))
        n_first, n_local = int(rng.integers(0, 3)), int(rng.integers(0, 3))
        forced = min(n_first + n_local, Np)
        K = int(rng.integers(max(1, forced), Np + 1))
        w = synth.C1.scaled(B=int(rng.integers(1, 4)), Hq=Hkv * G, Hkv=Hkv, D=D, dtype=dtype,
                            n_needles=0 if T < 64 else 4)
        out.append((w, T, Tcap, P, K, n_first, n_local))
    return out


CASES += _random_cases(20260528, 12)


@pytest.mark.parametrize("case", range(len(CASES)))
def test_meta_select_attend(rs, knobs, case):
    w, T, Tcap, P, K, n_first, n_local = CASES[case]
    say("quest case", case, w.name, T, Tcap, P, K, n_first, n_local)
    w, kc, vc = _cache_from_oracle(w, T, Tcap)
    _, _, _, q = synth.decode_step(w, 0)
    Np = -(-T // P)
    scale = 1.0 / np.sqrt(w.D)
    dt = tdtype(w.dtype)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, P, dt)
    tkc, tvc, tq = to_dev(kc, w.dtype), to_dev(vc, w.dtype), to_dev(q, w.dtype)
    meta = torch.zeros(w.B, w.Hkv, Tcap // P, 2, w.D, dtype=dt, device="cuda")
    ws = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, T, Np))

    # page metadata: bulk, bit-exact values
    rs.quest_page_meta(s, tkc, meta, 0, T)
    ometa = oracle.quest_page_meta(kc, P, T)
    np.testing.assert_array_equal(to_np(meta), ometa)

    # selection
    idx = torch.full((w.B, w.Hq, K), -7, dtype=torch.int32, device="cuda")
    scores = torch.zeros(w.B, w.Hq, Np, device="cuda")
    rs.quest_select_decode(s, tq, meta, T, K, n_first, n_local, idx, scores, ws)
    osc = oracle.quest_scores(q, ometa, Np)
    np.testing.assert_allclose(to_np(scores), osc, rtol=2e-6, atol=1e-5)
    oidx = oracle.quest_select(osc, K, n_first, n_local)
    gidx = to_np(idx)
    forced = _forced(Np, n_first, n_local)
    same = 0
    for b in range(w.B):
        for h in range(w.Hq):
            ok, why = topk_set_ok(osc[b, h], forced, K, gidx[b, h])
            assert ok, (b, h, why)
            same += np.array_equal(gidx[b, h], oidx[b, h])
    say("  identical index lists:", same, "of", w.B * w.Hq)

    # attention over the oracle's list
    out = torch.zeros(w.B, w.Hq, w.D, dtype=dt, device="cuda")
    lse = torch.zeros(w.B, w.Hq, device="cuda")
    rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, to_dev(oidx), K, None, 0, 0, out, lse, None, ws)
    oout, olse = oracle.sparse_attn_decode(q, kc, vc, P, T, scale, oidx)
    ok, worst = attn_close(to_np(out), oout, 2e-2 if w.dtype == "bf16" else 1e-4)
    assert ok, worst
    np.testing.assert_allclose(to_np(lse), olse, rtol=1e-4, atol=1e-4)

    # select-then-attend in one call, emitting its selection: as one persistent launch, as two
    # launches, and with the whole step of a (batch, head) inside one workgroup (the library
    # picks by shape; the knobs force each)
    oout2, _ = oracle.sparse_attn_decode(q, kc, vc, P, T, scale, gidx)
    for two_launch, one_wg in (("0", "0"), ("1", "0"), ("1", "1")):
        knobs.setenv("RATSPARSE_FUSED_TWO_LAUNCH", two_launch)
        knobs.setenv("RATSPARSE_FUSED_ONE_WG", one_wg)
        out2 = torch.zeros_like(out)
        idx2 = torch.full_like(idx, -7)
        rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, None, K, meta, n_first, n_local, out2, None, idx2, ws)
        np.testing.assert_array_equal(to_np(idx2), gidx)
        assert attn_close(to_np(out2), oout2, 2e-2 if w.dtype == "bf16" else 1e-4)[0]
        out3 = torch.zeros_like(out)
        lse3 = torch.zeros_like(lse)
        rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, None, K, meta, n_first, n_local, out3, lse3, None, ws)
        assert torch.equal(out3, out2)  # same result when the selection is not emitted
        _, olse2 = oracle.sparse_attn_decode(q, kc, vc, P, T, scale, gidx)
        np.testing.assert_allclose(to_np(lse3), olse2, rtol=1e-4, atol=1e-4)
    knobs.delenv("RATSPARSE_FUSED_TWO_LAUNCH")
    knobs.delenv("RATSPARSE_FUSED_ONE_WG")
    out4 = torch.zeros_like(out)
    rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, None, K, meta, n_first, n_local, out4, None, None, ws)  # own choice
    assert attn_close(to_np(out4), oout2, 2e-2 if w.dtype == "bf16" else 1e-4)[0]

    # dense path, and full budget = dense
    outd = torch.zeros_like(out)
    rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, None, 0, None, 0, 0, outd, lse, None, ws)
    od, odl = oracle.sparse_attn_decode(q, kc, vc, P, T, scale)
    assert attn_close(to_np(outd), od, 2e-2 if w.dtype == "bf16" else 1e-4)[0]
    np.testing.assert_allclose(to_np(lse), odl, rtol=1e-4, atol=1e-4)
    outf = torch.zeros_like(out)
    rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, None, Np, meta, n_first, n_local, outf, None, None, ws)
    assert attn_close(to_np(outf), od, 2e-2 if w.dtype == "bf16" else 1e-4)[0]
    torch.cuda.synchronize()
    ws.async_status()


@pytest.mark.parametrize("P,K,T", [(16, 1100, 19200 + 7), (64, 300, 64 * 330)])
def test_persistent_launch_with_one_long_item_per_unit(rs, knobs, P, K, T):
    """The persistent launch with its work split as coarsely as it goes: one score item and one attend item
    per (batch, head), so a wave walks 60-70 attention steps inside one item (its list entries come in more
    than once) and every score loop runs many rounds.  Same lists and outputs as the two-launch form, and
    the attention against the oracle."""
    w = synth.C2.scaled(B=1, Hq=2, Hkv=2)
    Tcap = -(-T // P) * P + P
    say("long items", P, K, T)
    w, kc, vc = _cache_from_oracle(w, T, Tcap)
    _, _, _, q = synth.decode_step(w, 0)
    Np = -(-T // P)
    scale = 1.0 / np.sqrt(w.D)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, P, torch.bfloat16)
    tkc, tvc, tq = to_dev(kc, "bf16"), to_dev(vc, "bf16"), to_dev(q, "bf16")
    meta = torch.zeros(w.B, w.Hkv, Tcap // P, 2, w.D, dtype=torch.bfloat16, device="cuda")
    rs.quest_page_meta(s, tkc, meta, 0, T)
    ws = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, T, K))
    res = {}
    for form, env in (("two launches", {"RATSPARSE_FUSED_TWO_LAUNCH": "1", "RATSPARSE_FUSED_ONE_WG": "0"}),
                      ("one launch, coarse", {"RATSPARSE_FUSED_TWO_LAUNCH": "0", "RATSPARSE_FUSED_ONE_WG": "0",
                                              "RATSPARSE_FUSED_SATT": "1", "RATSPARSE_FUSED_SSCORE": "1",
                                              "RATSPARSE_FUSED_FINE": "1"})):
        for k_, v_ in env.items():
            knobs.setenv(k_, v_)
        out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.bfloat16, device="cuda")
        lse = torch.zeros(w.B, w.Hq, device="cuda")
        idx = torch.full((w.B, w.Hq, K), -7, dtype=torch.int32, device="cuda")
        rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, None, K, meta, 1, 1, out, lse, idx, ws)
        torch.cuda.synchronize()
        ws.async_status()
        res[form] = (to_np(idx), to_np(out), to_np(lse))
        for k_ in env:
            knobs.delenv(k_)
    np.testing.assert_array_equal(res["one launch, coarse"][0], res["two launches"][0])
    gidx = res["two launches"][0]
    osc = oracle.quest_scores(q, oracle.quest_page_meta(kc, P, T), Np)
    for h in range(w.Hq):
        ok, why = topk_set_ok(osc[0, h], _forced(Np, 1, 1), K, gidx[0, h])
        assert ok, (h, why)
    oout, olse = oracle.sparse_attn_decode(q, kc, vc, P, T, scale, gidx)
    for form in res:
        assert attn_close(res[form][1], oout, 2e-2)[0], form
        np.testing.assert_allclose(res[form][2], olse, rtol=1e-4, atol=1e-4)


def test_incremental_meta_equals_bulk(rs):
    w, kc, vc = _cache_from_oracle(synth.C1.scaled(dtype="bf16"), 200, 256)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, 256, 16, torch.bfloat16)
    tkc = to_dev(kc, "bf16")
    inc = torch.zeros(w.B, w.Hkv, 16, 2, w.D, dtype=torch.bfloat16, device="cuda")
    rs.quest_page_meta(s, tkc, inc, 0, 150)
    for t in range(150, 200):
        rs.quest_page_meta(s, tkc, inc, t, t + 1)
    bulk = torch.zeros_like(inc)
    rs.quest_page_meta(s, tkc, bulk, 0, 200)
    assert torch.equal(inc, bulk)
    np.testing.assert_array_equal(to_np(bulk), oracle.quest_page_meta(kc, 16, 200))


def test_scan_with_meta_equals_separate_page_meta(rs):
    """rat_scan's optional page-metadata update (prefill path and one-token appends across page
    boundaries) leaves exactly what quest_page_meta computes from the stored cache."""
    for dtype, D, P in (("bf16", 128, 16), ("f32", 64, 32)):
        B, H, T0, steps = 1, 2, 300, 70
        Tcap = 384
        r = np.random.default_rng(11)
        mk = lambda n: r.standard_normal((B, H, n, D)).astype(np.float32)
        k, v = mk(T0 + steps), mk(T0 + steps)
        if dtype == "bf16":
            k, v = synth.to_bf16_grid(k), synth.to_bf16_grid(v)
        g = (1 / (1 + np.exp(-(4.2 + 0.5 * r.standard_normal((B, H, T0 + steps, D)))))).astype(np.float32)
        dt = tdtype(dtype)
        s = rs.make_shape(B, H, H, D, Tcap, P, dt)
        kc = torch.zeros(B, H, Tcap, D, dtype=dt, device="cuda")
        vc = torch.zeros_like(kc)
        sk = torch.zeros(B, H, D, device="cuda")
        sv = torch.zeros_like(sk)
        meta = torch.zeros(B, H, Tcap // P, 2, D, dtype=dt, device="cuda")
        ws = rs.Workspace(rs.rat_scan_workspace_bytes(s, T0))
        rs.rat_scan(s, to_dev(k[:, :, :T0], dtype), to_dev(v[:, :, :T0], dtype), to_dev(g[:, :, :T0]), sk, sv, kc, vc,
                    0, T0, ws, meta)
        for t in range(T0, T0 + steps):
            rs.rat_scan(s, to_dev(k[:, :, t:t + 1], dtype), to_dev(v[:, :, t:t + 1], dtype), to_dev(g[:, :, t:t + 1]),
                        sk, sv, kc, vc, t, 1, None, meta)
        want = torch.zeros_like(meta)
        rs.quest_page_meta(s, kc, want, 0, T0 + steps)
        assert torch.equal(meta, want)
        np.testing.assert_array_equal(to_np(meta), oracle.quest_page_meta(to_np(kc), P, T0 + steps))
        ws.async_status()


@pytest.mark.parametrize("slab", ["0", "1"])  # full rows, or 32-channel slabs (chunks four / two times as long)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("P", [16, 32, 64, 128, 256, 512])
@pytest.mark.parametrize("in_scan", ["1", "0"])
def test_scan_runs_leave_the_page_bounds(rs, knobs, in_scan, P, D, dtype, slab):
    """Long runs with the page metadata: where the scan kernel can (pages of 16 tokens up
    to the chunk length, a start on a chunk boundary) the bounds leave with the states, else the
    touched pages are recomputed afterwards; runs of both kinds back to back, with ragged ends,
    must leave what one bulk pass over the final cache computes.  The knob switches the first
    kind off, so both paths see every run."""
    knobs.setenv("RATSPARSE_SCAN_META", in_scan)
    knobs.setenv("RATSPARSE_SCAN_SLAB", slab)
    B, H = 2, 20  # 40 (batch, head) pairs: full-row chunks (128 tokens at 128 channels, 256 at 64)
    # (t0, T_new): aligned; aligned and a single chunk; unaligned; unaligned; unaligned and long
    runs = [(0, 256), (256, 100), (356, 156), (512, 521), (1033, 200), (1233, 3000)]  # 512: aligned for every form
    T = 4233
    Tcap = 4608  # a multiple of every page size
    r = np.random.default_rng(17)
    k = synth.to_bf16_grid(r.standard_normal((B, H, T, D)).astype(np.float32))
    v = synth.to_bf16_grid(r.standard_normal((B, H, T, D)).astype(np.float32))
    g = (1 / (1 + np.exp(-(4.2 + 0.5 * r.standard_normal((B, H, T, D)))))).astype(np.float32)
    dt = tdtype(dtype)
    s = rs.make_shape(B, H, H, D, Tcap, P, dt)
    kc = torch.zeros(B, H, Tcap, D, dtype=dt, device="cuda")
    vc = torch.zeros_like(kc)
    sk = torch.zeros(B, H, D, device="cuda")
    sv = torch.zeros_like(sk)
    meta = torch.zeros(B, H, Tcap // P, 2, D, dtype=dt, device="cuda")
    ws = rs.Workspace(rs.rat_scan_workspace_bytes(s, 3000))
    for t0, n in runs:
        rs.rat_scan(s, to_dev(k[:, :, t0:t0 + n], dtype), to_dev(v[:, :, t0:t0 + n], dtype), to_dev(g[:, :, t0:t0 + n]),
                    sk, sv, kc, vc, t0, n, ws, meta)
    want = torch.zeros_like(meta)
    rs.quest_page_meta(s, kc, want, 0, T)
    assert torch.equal(meta, want)
    np.testing.assert_array_equal(to_np(meta), oracle.quest_page_meta(to_np(kc), P, T))
    ws.async_status()


def test_exact_ties_take_the_lowest_index(rs):
    B, H, D, P, Np = 1, 2, 128, 16, 300
    r = np.random.default_rng(3)
    base = synth.to_bf16_grid(r.standard_normal((B, H, 7, P, D)).astype(np.float32))
    pick = r.integers(0, 7, Np)
    kc = base[:, :, pick].reshape(B, H, Np * P, D)  # only 7 distinct pages: scores tie exactly
    q = synth.to_bf16_grid(r.standard_normal((B, H, D)).astype(np.float32))
    s = rs.make_shape(B, H, H, D, Np * P, P, torch.bfloat16)
    meta = torch.zeros(B, H, Np, 2, D, dtype=torch.bfloat16, device="cuda")
    rs.quest_page_meta(s, to_dev(kc, "bf16"), meta, 0, Np * P)
    ws = rs.Workspace(rs.quest_select_decode_workspace_bytes(s, Np * P))
    osc = oracle.quest_scores(q, oracle.quest_page_meta(kc, P, Np * P), Np)
    for K in (1, 10, 64, 299, 300):
        idx = torch.zeros(B, H, K, dtype=torch.int32, device="cuda")
        rs.quest_select_decode(s, to_dev(q, "bf16"), meta, Np * P, K, 0, 0, idx, None, ws)
        np.testing.assert_array_equal(to_np(idx), oracle.quest_select(osc, K, 0, 0))


def test_listed_pages_with_skips_and_any_order(rs):
    w, kc, vc = _cache_from_oracle(synth.C1.scaled(dtype="bf16"), 512, 512)
    _, _, _, q = synth.decode_step(w, 1)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, 512, 16, torch.bfloat16)
    idx = np.array([[[31, 2, -1, 7, 19, 0], [5, -1, -1, 30, 1, 8]]], dtype=np.int32)
    ws = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, 505, 6))
    out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.bfloat16, device="cuda")
    rs.sparse_attn_decode(s, to_dev(q, "bf16"), to_dev(kc, "bf16"), to_dev(vc, "bf16"), 505, 0.125,
                          to_dev(idx), 6, None, 0, 0, out, None, None, ws)
    want, _ = oracle.sparse_attn_decode(q, kc, vc, 16, 505, 0.125, idx)
    assert attn_close(to_np(out), want)[0]


def test_argument_errors_are_reported(rs):
    s = rs.make_shape(1, 2, 2, 128, 256, 16, torch.bfloat16)
    t = torch.zeros(1 << 16, dtype=torch.bfloat16, device="cuda")
    i = torch.zeros(64, dtype=torch.int32, device="cuda")
    ws = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, 256, 16))
    with pytest.raises(rs.RatsparseError, match="invalid argument"):
        rs.quest_select_decode(s, t, t, 256, 17, 1, 1, i, None, ws)  # K > Np
    with pytest.raises(rs.RatsparseError, match="invalid argument"):
        rs.quest_select_decode(s, t, t, 256, 2, 2, 2, i, None, ws)  # more forced pages than K
    with pytest.raises(rs.RatsparseError, match="invalid argument"):
        rs.sparse_attn_decode(s, t, t, t, 257, 1.0, None, 0, None, 0, 0, t, None, None, ws)  # T > Tcap
    small = rs.Workspace(0)
    big = rs.make_shape(4, 32, 32, 128, 65536, 16, torch.bfloat16)
    with pytest.raises(rs.RatsparseError, match="workspace too small"):
        rs.sparse_attn_decode(big, t, t, t, 65536, 1.0, None, 0, None, 0, 0, t, None, None, small)


def test_random_selector_five_seeds(rs):
    """The random selector of the paper's H2 analysis (Sec. 2.3): uniform K-subsets of the pages
    drawn on the host, five seeds, evaluated through the listed-pages mode (Eq. 4 unchanged).
    Unsorted lists and a list that misses the newest page are legal inputs."""
    w, kc, vc = _cache_from_oracle(synth.C2.scaled(Hq=8, Hkv=2), 4096 + 5, 4096 + 64)
    T, Tcap, P, K = 4096 + 5, 4096 + 64, 16, 32
    Np = -(-T // P)
    _, _, _, q = synth.decode_step(w, 0)
    scale = 1.0 / np.sqrt(w.D)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, P, torch.bfloat16)
    tkc, tvc, tq = to_dev(kc, "bf16"), to_dev(vc, "bf16"), to_dev(q, "bf16")
    ws = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, T, K))
    for seed in range(5):
        r = np.random.default_rng(1000 + seed)
        ridx = np.stack([np.stack([r.choice(Np, size=K, replace=False) for _ in range(w.Hq)]) for _ in range(w.B)])
        ridx = ridx.astype(np.int32)
        out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.bfloat16, device="cuda")
        lse = torch.zeros(w.B, w.Hq, device="cuda")
        rs.sparse_attn_decode(s, tq, tkc, tvc, T, scale, to_dev(ridx), K, None, 0, 0, out, lse, None, ws)
        want, wlse = oracle.sparse_attn_decode(q, kc, vc, P, T, scale, ridx)
        ok, worst = attn_close(to_np(out), want)
        assert ok, (seed, worst)
        np.testing.assert_allclose(to_np(lse), wlse, rtol=1e-4, atol=1e-4)
    torch.cuda.synchronize()
    ws.async_status()


GROUP_CASES = [
    # workload, T_valid, Tcap, P, K, n_first, n_local
    (synth.C2.scaled(Hq=8, Hkv=2), 4096 + 5, 4096 + 64, 16, 32, 1, 1),   # G = 4, bf16
    (synth.C1.scaled(Hq=4, Hkv=2), 2041, 2048 + 16, 16, 16, 1, 1),       # G = 2, fp32, D = 64
    (synth.C2.scaled(B=2, Hq=8, Hkv=1), 3000, 3072, 64, 6, 0, 2),        # G = 8, 64-token pages
    (synth.C2.scaled(Hq=6, Hkv=2), 1000, 1024, 16, 8, 1, 1),             # G = 3: not offered
]


@pytest.mark.parametrize("case", range(len(GROUP_CASES)))
def test_group_shared_selection(rs, case):
    """The option for grouped-query attention: one page list per KV head from the summed
    scores of its query heads, attended by all of them."""
    w, T, Tcap, P, K, n_first, n_local = GROUP_CASES[case]
    say("group case", case, w.name, w.Hq, w.Hkv, T, P, K)
    w, kc, vc = _cache_from_oracle(w, T, Tcap)
    _, _, _, q = synth.decode_step(w, 0)
    Np = -(-T // P)
    G = w.Hq // w.Hkv
    scale = 1.0 / np.sqrt(w.D)
    dt = tdtype(w.dtype)
    tol = 2e-2 if w.dtype == "bf16" else 1e-4
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, P, dt)
    tkc, tvc, tq = to_dev(kc, w.dtype), to_dev(vc, w.dtype), to_dev(q, w.dtype)
    meta = torch.zeros(w.B, w.Hkv, Tcap // P, 2, w.D, dtype=dt, device="cuda")
    ws = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, T, Np))
    rs.quest_page_meta(s, tkc, meta, 0, T)
    ometa = oracle.quest_page_meta(kc, P, T)
    idx = torch.full((w.B, w.Hkv, K), -7, dtype=torch.int32, device="cuda")
    scores = torch.zeros(w.B, w.Hkv, Np, device="cuda")
    if G not in (2, 4, 8):
        with pytest.raises(rs.RatsparseError, match="status 2"):
            rs.quest_select_decode_group(s, tq, meta, T, K, n_first, n_local, idx, scores, ws)
        return
    rs.quest_select_decode_group(s, tq, meta, T, K, n_first, n_local, idx, scores, ws)
    osc = oracle.quest_scores_group(q, ometa, Np)
    np.testing.assert_allclose(to_np(scores), osc, rtol=4e-6, atol=2e-5)
    gidx = to_np(idx)
    forced = _forced(Np, n_first, n_local)
    for b in range(w.B):
        for kvh in range(w.Hkv):
            ok, why = topk_set_ok(osc[b, kvh], forced, K, gidx[b, kvh])
            assert ok, (b, kvh, why)
    # every query head of the group attends the group's list
    per_head = np.repeat(gidx, G, axis=1)
    want, wlse = oracle.sparse_attn_decode(q, kc, vc, P, T, scale, per_head)
    out = torch.zeros(w.B, w.Hq, w.D, dtype=dt, device="cuda")
    lse = torch.zeros(w.B, w.Hq, device="cuda")
    rs.sparse_attn_decode_group(s, tq, tkc, tvc, T, scale, idx, K, None, 0, 0, out, lse, None, ws)
    ok, worst = attn_close(to_np(out), want, tol)
    assert ok, worst
    np.testing.assert_allclose(to_np(lse), wlse, rtol=1e-4, atol=1e-4)
    # select, then attend, in one call; same list, same result
    out2 = torch.zeros_like(out)
    idx2 = torch.full_like(idx, -7)
    rs.sparse_attn_decode_group(s, tq, tkc, tvc, T, scale, None, K, meta, n_first, n_local, out2, None, idx2, ws)
    np.testing.assert_array_equal(to_np(idx2), gidx)
    assert torch.equal(out2, out)
    with pytest.raises(rs.RatsparseError, match="status 1"):  # no dense mode
        rs.sparse_attn_decode_group(s, tq, tkc, tvc, T, scale, None, 0, None, 0, 0, out2, None, None, ws)
    torch.cuda.synchronize()
    ws.async_status()
