"""GPU parity of MoBA routing (block means, gate scores, top-K blocks) and of the block-sparse
/ dense causal prefill attention against the float64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import say, to_dev, to_np
from helpers import attn_close, topk_set_ok
from paper_2605_28640_amd import synth

pytestmark = pytest.mark.gpu


def _setup(w, T, Tcap):
    w = w.scaled(T=T)
    k, v, g = synth.prefill(w)
    ko, vo, _, _ = oracle.rat_scan(k, v, g)
    kc = np.zeros((w.B, w.Hkv, Tcap, w.D), dtype=np.float32)
    vc = np.zeros_like(kc)
    kc[:, :, :T], vc[:, :, :T] = oracle.round_to_bf16(ko), oracle.round_to_bf16(vo)
    q = synth.prefill_queries(w)
    return w, q, kc, vc


CASES = [
    # workload, T, Tcap, block, K, n_first
    (synth.C4.scaled(B=1, Hq=2, Hkv=2), 2048, 2048, 512, 3, 0),
    (synth.C4.scaled(B=1, Hq=4, Hkv=2), 1000, 1024, 64, 4, 1),      # GQA, ragged tail block, first block kept
    (synth.C4.scaled(B=2, Hq=2, Hkv=2, D=64), 777, 800, 128, 2, 0),  # D=64, T not a multiple of anything
    (synth.C4.scaled(B=1, Hq=2, Hkv=1), 512, 512, 16, 8, 0),         # small blocks inside one row tile
    (synth.C4.scaled(B=2, Hq=4, Hkv=2), 1024, 1024, 128, 3, 0),      # 8 (batch, head) units: the XCD-aware tile order
    # the paper's own MoBA settings (App. A.1; Tables 3-4): T = 4096, 64-token blocks with
    # top-16 / 8 / 4, 128-token blocks with top-8 / 4
    (synth.C4.scaled(B=1, Hq=2, Hkv=2), 4096, 4096, 64, 16, 0),
    (synth.C4.scaled(B=1, Hq=2, Hkv=2), 4096, 4096, 64, 8, 1),
    (synth.C4.scaled(B=1, Hq=2, Hkv=2), 4096, 4096, 64, 4, 0),
    (synth.C4.scaled(B=1, Hq=2, Hkv=2), 4096, 4096, 128, 8, 0),
    (synth.C4.scaled(B=1, Hq=2, Hkv=2), 4096, 4096, 128, 4, 1),
]


def _random_cases(seed, n):
    """Seeded random small shapes: head counts and grouping, both head dims, block sizes from 16
    to 256, ragged lengths, 1-8 picked blocks, 0-1 always-kept leading blocks."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        Hkv = int(rng.integers(1, 3))
        G = int(rng.choice([1, 2]))
        D = int(rng.choice([64, 128]))
        block = int(rng.choice([16, 32, 64, 128, 256]))
        T = int(rng.integers(block + 1, 1400))
        Tcap = -(-T // 16) * 16 + 16 * int(rng.integers(0, 3))
        n_first = int(rng.integers(0, 2))
        K = int(rng.integers(1 + n_first, 9))
        w = synth.C4.scaled(B=int(rng.integers(1, 3)), Hq=Hkv * G, Hkv=Hkv, D=D)
        out.append((w, T, Tcap, block, K, n_first))
    return out


CASES += _random_cases(20260528, 8)


@pytest.mark.parametrize("case", range(len(CASES)))
def test_moba_select_and_sparse_prefill(rs, knobs, case):
    w, T, Tcap, block, K, n_first = CASES[case]
    say("moba case", case, T, Tcap, block, K, n_first)
    w, q, kc, vc = _setup(w, T, Tcap)
    Nb = -(-T // block)
    scale = 1.0 / np.sqrt(w.D)
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, Tcap, 16, torch.bfloat16)
    tq, tkc, tvc = to_dev(q, "bf16"), to_dev(kc, "bf16"), to_dev(vc, "bf16")
    means = torch.zeros(w.B, w.Hkv, Nb, w.D, device="cuda")
    idx = torch.full((w.B, w.Hq, T, K), -9, dtype=torch.int32, device="cuda")
    ws = rs.Workspace(max(rs.moba_select_prefill_workspace_bytes(s, T, block),
                          rs.sparse_attn_prefill_workspace_bytes(s, T, block, max(K, Nb))))
    rs.moba_select_prefill(s, tq, tkc, T, block, K, n_first, means, idx, ws)
    omeans = oracle.moba_block_means(kc, T, block)
    np.testing.assert_allclose(to_np(means), omeans, rtol=1e-5, atol=1e-6)
    oidx, osc = oracle.moba_select(q, omeans, T, block, K, n_first, want_scores=True)
    gidx = to_np(idx)
    same = 0
    for b in range(w.B):
        for h in range(w.Hq):
            for t in range(T):
                own = t // block
                take = min(K, own + 1)
                sc = np.where(np.isnan(osc[b, h, t, :own + 1]), 0.0, osc[b, h, t, :own + 1])
                forced = np.zeros(own + 1, bool)
                forced[own] = True
                forced[:n_first] = True
                row = gidx[b, h, t]
                assert np.all(row[take:] == -1), (b, h, t, row)
                ok, why = topk_set_ok(sc, forced, take, row[:take])
                assert ok, (b, h, t, why, row)
                same += np.array_equal(row, oidx[b, h, t])
    say("  rows with identical block lists:", same, "of", w.B * w.Hq * T)
    # the gate's other form (block-mean operands shared through LDS by six-wave workgroups, or
    # fetched by each one-wave workgroup; the library picks by size): the same routing bit for bit
    for form in ("0", "1"):
        knobs.setenv("RATSPARSE_GATE_SHARED", form)
        idx2 = torch.full_like(idx, -9)
        rs.moba_select_prefill(s, tq, tkc, T, block, K, n_first, means, idx2, ws)
        assert torch.equal(idx2, idx), form
    knobs.delenv("RATSPARSE_GATE_SHARED")

    # block-sparse attention over the GPU's own routing
    out = torch.zeros(w.B, w.Hq, T, w.D, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(w.B, w.Hq, T, device="cuda")
    oout, olse = oracle.sparse_attn_prefill(q, kc, vc, T, block, scale, gidx)
    # both forms of the routed kernel (the library picks by shape; the knob forces either):
    # regrouped by block, and - for up to 64 blocks of a multiple of 64 tokens - causal tiles
    # with a bit set of listed blocks per row
    for form in ("0", "1"):
        knobs.setenv("RATSPARSE_PREFILL_MASKED", form)
        out.zero_(), lse.zero_()
        rs.sparse_attn_prefill(s, tq, tkc, tvc, T, block, scale, idx, K, out, lse, ws)
        ok, worst = attn_close(to_np(out), oout)
        assert ok, (form, worst)
        np.testing.assert_allclose(to_np(lse), olse, rtol=2e-3, atol=2e-3)
        say("  sparse prefill, form", form, "worst relative row error", worst)
    knobs.delenv("RATSPARSE_PREFILL_MASKED")
    rs.sparse_attn_prefill(s, tq, tkc, tvc, T, block, scale, idx, K, out, lse, ws)  # the library's own choice
    assert attn_close(to_np(out), oout)[0]

    # dense causal path, and enough blocks = dense
    outd = torch.zeros_like(out)
    rs.sparse_attn_prefill(s, tq, tkc, tvc, T, block, scale, None, 0, outd, lse, ws)
    od, odl = oracle.sparse_attn_prefill(q, kc, vc, T, block, scale)
    ok, worst = attn_close(to_np(outd), od)
    assert ok, worst
    np.testing.assert_allclose(to_np(lse), odl, rtol=2e-3, atol=2e-3)
    if Nb <= 32:
        idx_all = torch.full((w.B, w.Hq, T, Nb), -9, dtype=torch.int32, device="cuda")
        rs.moba_select_prefill(s, tq, tkc, T, block, Nb, n_first, means, idx_all, ws)
        outf = torch.zeros_like(out)
        rs.sparse_attn_prefill(s, tq, tkc, tvc, T, block, scale, idx_all, Nb, outf, None, ws)
        assert attn_close(to_np(outf), od)[0]
    torch.cuda.synchronize()
    ws.async_status()


# (K, n_first, block): register picks (at most 64 blocks; lists of 4, 8, 16), score columns in LDS
# with top lists (more than 64 blocks), and LDS sweeps (K above 16)
@pytest.mark.parametrize("K,n_first,block", [(3, 0, 64), (4, 1, 64), (8, 0, 64), (16, 2, 64), (3, 0, 16), (8, 1, 16),
                                             (13, 0, 16), (20, 0, 64), (24, 1, 16)])
def test_moba_exact_ties_pick_lowest_blocks(rs, K, n_first, block):
    """A cache that repeats with the block length has identical block means, so every gate
    score of a query ties exactly: the routing must keep the query's own block, the first
    n_first blocks, and fill up with the lowest block indices (the oracle's tie rule)."""
    say("moba ties", K, n_first)
    w = synth.C4.scaled(B=1, Hq=2, Hkv=2, T=1024)
    T = 1024 if block == 64 else 1600  # 16 blocks, or 100 blocks of 16 tokens
    w = w.scaled(T=T)
    Nb = T // block
    rng = np.random.default_rng(7)
    one = oracle.round_to_bf16(rng.standard_normal((w.B, w.Hkv, block, w.D)).astype(np.float32))
    kc = np.tile(one, (1, 1, Nb, 1))
    q = oracle.round_to_bf16(rng.standard_normal((w.B, w.Hq, T, w.D)).astype(np.float32))
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, T, 16, torch.bfloat16)
    means = torch.zeros(w.B, w.Hkv, Nb, w.D, device="cuda")
    idx = torch.full((w.B, w.Hq, T, K), -9, dtype=torch.int32, device="cuda")
    ws = rs.Workspace(rs.moba_select_prefill_workspace_bytes(s, T, block))
    rs.moba_select_prefill(s, to_dev(q, "bf16"), to_dev(kc, "bf16"), T, block, K, n_first, means, idx, ws)
    omeans = oracle.moba_block_means(kc, T, block)
    oidx = oracle.moba_select(q, omeans, T, block, K, n_first)
    gidx = to_np(idx)
    for t in (0, 63, 64, 200, 511, 1023, T - 1):
        own = t // block
        # always kept: own block and the first n_first; the rest ties: lowest indices first
        want = sorted(set(list(range(min(K - 1, own))) + [own]))
        want = want + [-1] * (K - len(want))
        assert list(oidx[0, 0, t]) == want, (t, oidx[0, 0, t], want)  # the oracle follows the stated rule
    np.testing.assert_array_equal(gidx, oidx)
    ws.async_status()


@pytest.mark.parametrize("form", ["0", "1"])
def test_lists_are_taken_as_given(rs, knobs, form):
    """The attention follows the lists it is handed, whatever wrote them: rows whose own block is
    not listed do not attend it, rows with an empty list give zeros and a log-sum-exp of -inf,
    entries may come in any order.  Both forms of the routed kernel."""
    knobs.setenv("RATSPARSE_PREFILL_MASKED", form)
    w = synth.C4.scaled(B=1, Hq=4, Hkv=2, T=1536)
    T, block, K = 1536, 128, 4
    w, q, kc, vc = _setup(w, T, T)
    Nb = T // block
    rng = np.random.default_rng(99)
    idx = np.full((w.B, w.Hq, T, K), -1, dtype=np.int32)
    for b in range(w.B):
        for h in range(w.Hq):
            for t in range(T):
                own = t // block
                n = int(rng.integers(0, min(K, own + 1) + 1))  # sometimes nothing at all
                pick = rng.choice(own + 1, size=n, replace=False)  # may or may not hold the own block
                idx[b, h, t, :n] = pick  # unsorted
    s = rs.make_shape(w.B, w.Hq, w.Hkv, w.D, T, 16, torch.bfloat16)
    ws = rs.Workspace(rs.sparse_attn_prefill_workspace_bytes(s, T, block, K))
    out = torch.zeros(w.B, w.Hq, T, w.D, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(w.B, w.Hq, T, device="cuda")
    scale = 1.0 / np.sqrt(w.D)
    rs.sparse_attn_prefill(s, to_dev(q, "bf16"), to_dev(kc, "bf16"), to_dev(vc, "bf16"), T, block, scale,
                           torch.from_numpy(idx).cuda(), K, out, lse, ws)
    oout, olse = oracle.sparse_attn_prefill(q, kc, vc, T, block, scale, idx)
    empty = np.all(idx < 0, axis=-1)
    assert empty.any() and (~empty).any()
    got, glse = to_np(out), to_np(lse)
    assert np.all(got[empty] == 0) and np.all(np.isneginf(glse[empty]))
    ok, worst = attn_close(got[~empty], oout[~empty])
    assert ok, worst
    np.testing.assert_allclose(glse[~empty], olse[~empty], rtol=2e-3, atol=2e-3)
    ws.async_status()
