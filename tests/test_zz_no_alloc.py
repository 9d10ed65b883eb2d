"""sparse_attn_decode_static (the entry point that allocates nothing: its scratch is a device array
inside the library) against sparse_attn_decode on the same inputs, through the C ABI: two calls in a
row, the second on a smaller input, in every mode (fused select-then-attend in its three forms,
listed pages, dense), and the size limit."""
import ctypes

import numpy as np
import pytest
import torch

from gpu_util import say, to_np
from helpers import attn_close

pytestmark = pytest.mark.gpu


def _inputs(B, Hq, Hkv, D, T, Tcap, P, seed):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    dt = torch.bfloat16
    kc = torch.zeros(B, Hkv, Tcap, D, dtype=dt, device="cuda")
    vc = torch.zeros_like(kc)
    kc[:, :, :T] = (torch.randn(B, Hkv, T, D, device="cuda", generator=gen) * 0.5).to(dt)
    vc[:, :, :T] = torch.randn(B, Hkv, T, D, device="cuda", generator=gen).to(dt)
    q = torch.randn(B, Hq, D, device="cuda", generator=gen).to(dt)
    return q, kc, vc


def _both(rs, shape, T, K, mode, seed):
    """Run the workspace entry point and the static one on the same inputs; return both results."""
    B, Hq, Hkv, D, Tcap, P = shape
    s = rs.make_shape(B, Hq, Hkv, D, Tcap, P, torch.bfloat16)
    q, kc, vc = _inputs(B, Hq, Hkv, D, T, Tcap, P, seed)
    meta = torch.zeros(B, Hkv, Tcap // P, 2, D, dtype=torch.bfloat16, device="cuda")
    rs.quest_page_meta(s, kc, meta, 0, T)
    scale = 1.0 / np.sqrt(D)
    Np = -(-T // P)
    res = []
    listed = None
    if mode == "listed":
        r = np.random.default_rng(seed)
        listed = torch.from_numpy(np.stack([[np.sort(r.choice(Np, K, replace=False)) for _ in range(Hq)]
                                            for _ in range(B)]).astype(np.int32)).cuda()
    for static in (False, True):
        out = torch.full((B, Hq, D), 3.0, dtype=torch.bfloat16, device="cuda")
        lse = torch.full((B, Hq), 3.0, device="cuda")
        idx = torch.full((B, Hq, max(K, 1)), -1, dtype=torch.int32, device="cuda")
        args = dict(fused=(None, K, meta, 1, 1), listed=(listed, K, None, 0, 0), dense=(None, 0, None, 0, 0))[mode]
        idx_out = idx if mode == "fused" else None
        if static:
            err = torch.zeros(1, dtype=torch.int32, device="cuda")
            rs.sparse_attn_decode_static(s, q, kc, vc, T, scale, args[0], args[1], args[2], args[3], args[4], out, lse,
                                         idx_out, err)
            torch.cuda.synchronize()
            assert int(err.item()) == 0
        else:
            ws = rs.Workspace(rs.sparse_attn_decode_workspace_bytes(s, T, K if mode != "dense" else 0))
            rs.sparse_attn_decode(s, q, kc, vc, T, scale, args[0], args[1], args[2], args[3], args[4], out, lse,
                                  idx_out, ws)
            torch.cuda.synchronize()
            ws.async_status()
        res.append((out, lse, idx))
    return res


def _same(a, b, what):
    (out_a, lse_a, idx_a), (out_b, lse_b, idx_b) = a, b
    assert torch.equal(idx_a, idx_b), what                     # page lists: bit-exact
    ok, worst = attn_close(to_np(out_b), to_np(out_a).astype(np.float64))
    assert ok, (what, worst)                                   # attention rows: the 2e-2 rule
    np.testing.assert_allclose(to_np(lse_b), to_np(lse_a), rtol=1e-3, atol=1e-3)
    return torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b)


BIG = (2, 8, 4, 128, 8192 + 64, 16)     # B, Hq, Hkv, D, Tcap, P
SMALL = (1, 4, 4, 128, 1024, 16)


@pytest.mark.parametrize("form", ["default", "persistent", "two_launch", "one_wg"])
def test_fused_two_calls_in_a_row(rs, knobs, form):
    if form != "default":
        knobs.setenv("RATSPARSE_FUSED_TWO_LAUNCH", "1" if form == "two_launch" else "0")
        knobs.setenv("RATSPARSE_FUSED_ONE_WG", "1" if form == "one_wg" else "0")
    say("no-alloc fused", form)
    bit = _same(*_both(rs, BIG, 8192 + 5, 64, "fused", 1), (form, "first"))
    bit &= _same(*_both(rs, SMALL, 700, 9, "fused", 2), (form, "second, smaller"))  # finds the first call's leftovers
    say("  bit-equal outputs:", bool(bit))


@pytest.mark.parametrize("mode", ["listed", "dense"])
def test_listed_and_dense_two_calls_in_a_row(rs, mode):
    say("no-alloc", mode)
    _same(*_both(rs, BIG, 8192 + 5, 64, mode, 3), (mode, "first"))
    _same(*_both(rs, SMALL, 700, 9, mode, 4), (mode, "second, smaller"))


def test_size_limit_is_refused_before_anything_runs(rs):
    """A shape whose scratch would not fit the static array is turned down with its own status and
    nothing is enqueued; the largest measured configuration fits."""
    lib = rs.load()
    A = 1 << 20  # made-up aligned addresses: validation comes before any launch
    # batch 4, 32 heads, 64K tokens + 512 steps, K = 1024: the largest configured decode shape
    s = rs.make_shape(4, 32, 32, 128, 66048, 16, torch.bfloat16)
    assert rs.sparse_attn_decode_workspace_bytes(s, 66048, 1024) <= rs.RS_STATIC_SCRATCH_BYTES
    big = rs.make_shape(16, 32, 32, 128, 66048, 16, torch.bfloat16)
    assert rs.sparse_attn_decode_workspace_bytes(big, 66048, 1024) > rs.RS_STATIC_SCRATCH_BYTES
    st = lib.sparse_attn_decode_static(ctypes.byref(big), A, A, A, 66048, 0.1, None, 1024, A, 1, 1, A, None, None, A, None)
    assert st == 6 and b"static" in lib.ratsparse_status_string(st)
    assert lib.sparse_attn_decode_static(ctypes.byref(s), A, A, A, 66048, 0.1, None, 1024, A, 1, 1, A, None, None, None,
                                         None) == 1  # the error word is required
