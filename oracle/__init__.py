"""CPU oracle of the recurrence-augmented sparse-attention path (TEST INFRASTRUCTURE).

numpy front end to the plain-C double-precision routines in this directory.  Only
tests, the smoke check and the bench's cpu_baseline leg may import this package;
the product path never does, and this package imports nothing of the product.

Inputs are float32 arrays holding the stored values exactly (bf16 values are floats
with a zero low half); outputs are float64.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None

_i64 = ctypes.c_int64
_dbl = ctypes.c_double
_vp = ctypes.c_void_p


def lib():
    """Load the oracle library, building it with gcc if it is missing or stale."""
    global _lib
    if _lib is None:
        # RATSPARSE_REF_LIB: an already built variant of this library (the sanitizer test's)
        path = os.environ.get("RATSPARSE_REF_LIB") or _build.build(force=False)
        _lib = ctypes.CDLL(path)
        _lib.ref_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().ref_num_threads())


def set_num_threads(n: int) -> None:
    """OpenMP threads used by the following calls (timing aid)."""
    lib().ref_set_num_threads(ctypes.c_int(int(n)))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return _vp(a.ctypes.data) if a is not None else _vp(0)


def round_to_bf16(x):
    """RNE of float64 values to bfloat16, returned as float32 (exact)."""
    x = _f64(x)
    y = np.empty(x.shape, dtype=np.float32)
    lib().ref_round_to_bf16(_i64(x.size), _p(x), _p(y))
    return y


def topk_row(score, K, forced=None):
    score = _f64(score)
    M = score.shape[0]
    out = np.empty(K, dtype=np.int32)
    f = None if forced is None else np.ascontiguousarray(forced, dtype=np.uint8)
    lib().ref_topk_row(_i64(M), _p(score), _p(f), _i64(K), _p(out))
    return out


def rat_scan(k, v, g, state_k=None, state_v=None):
    """Eq. 1.  k, v, g: [B, H, T, D].  Returns (k_tilde, v_tilde, state_k, state_v), float64."""
    k, v, g = _f32(k), _f32(v), _f32(g)
    B, H, T, D = k.shape
    sk = np.zeros((B, H, D)) if state_k is None else _f64(state_k).copy()
    sv = np.zeros((B, H, D)) if state_v is None else _f64(state_v).copy()
    ko = np.empty((B, H, T, D), dtype=np.float64)
    vo = np.empty((B, H, T, D), dtype=np.float64)
    lib().ref_rat_scan(_i64(B * H), _i64(T), _i64(D), _p(k), _p(v), _p(g), _p(sk), _p(sv),
                       _p(ko), _p(vo))
    return ko, vo, sk, sv


def quest_page_meta(k_cache, P, T_valid):
    """k_cache: [B, Hkv, Tcap, D] -> meta [B, Hkv, Tcap/P, 2, D] float32 (pages past T_valid zero)."""
    k_cache = _f32(k_cache)
    B, H, Tcap, D = k_cache.shape
    assert Tcap % P == 0
    meta = np.zeros((B, H, Tcap // P, 2, D), dtype=np.float32)
    lib().ref_quest_page_meta(_i64(B * H), _i64(Tcap), _i64(D), _i64(P), _p(k_cache),
                              _i64(T_valid), _p(meta))
    return meta


def quest_scores(q, meta, Np):
    """q: [B, Hq, D]; meta: [B, Hkv, Np_cap, 2, D] -> scores [B, Hq, Np] float64."""
    q, meta = _f32(q), _f32(meta)
    B, Hq, D = q.shape
    Hkv, Np_cap = meta.shape[1], meta.shape[2]
    s = np.empty((B, Hq, Np), dtype=np.float64)
    lib().ref_quest_scores(_i64(B), _i64(Hq), _i64(Hkv), _i64(D), _i64(Np_cap), _p(q), _p(meta),
                           _i64(Np), _p(s))
    return s


def quest_scores_group(q, meta, Np):
    """Group-shared selection (an option for grouped-query attention, not in the paper): the
    page score of a KV head is the sum of the page scores of its query heads.
    q: [B, Hq, D]; meta: [B, Hkv, Np_cap, 2, D] -> scores [B, Hkv, Np] float64."""
    per_head = quest_scores(q, meta, Np)
    B, Hq, _ = per_head.shape
    Hkv = np.asarray(meta).shape[1]
    return per_head.reshape(B, Hkv, Hq // Hkv, Np).sum(axis=2)


def quest_select(scores, K, n_first, n_local):
    """scores: [B, Hq, Np] -> idx [B, Hq, K] int32 ascending."""
    scores = _f64(scores)
    B, Hq, Np = scores.shape
    assert 0 <= K <= Np
    idx = np.empty((B, Hq, K), dtype=np.int32)
    lib().ref_quest_select(_i64(B * Hq), _i64(Np), _p(scores), _i64(K), _i64(n_first),
                           _i64(n_local), _p(idx))
    return idx


def sparse_attn_decode(q, k_cache, v_cache, P, T_valid, scale, idx=None):
    """Eq. 4 at decode.  Returns (out [B, Hq, D], lse [B, Hq]) float64."""
    q, k_cache, v_cache = _f32(q), _f32(k_cache), _f32(v_cache)
    B, Hq, D = q.shape
    Hkv, Tcap = k_cache.shape[1], k_cache.shape[2]
    K = 0
    if idx is not None:
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        K = idx.shape[-1]
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    lib().ref_sparse_attn_decode(_i64(B), _i64(Hq), _i64(Hkv), _i64(D), _i64(Tcap), _i64(P),
                                 _p(q), _p(k_cache), _p(v_cache), _i64(T_valid), _dbl(scale),
                                 _p(idx), _i64(K), _p(out), _p(lse))
    return out, lse


def moba_block_means(k_cache, T, block):
    k_cache = _f32(k_cache)
    B, H, Tcap, D = k_cache.shape
    Nb = (T + block - 1) // block
    means = np.empty((B, H, Nb, D), dtype=np.float64)
    lib().ref_moba_block_means(_i64(B * H), _i64(T), _i64(Tcap), _i64(D), _i64(block),
                               _p(k_cache), _p(means))
    return means


def moba_select(q, means, T, block, K, n_first=0, t_begin=0, t_end=None, want_scores=False):
    """q: [B, Hq, T, D]; means: [B, Hkv, Nb, D] float64 -> idx [B, Hq, rows, K] (and scores)."""
    q, means = _f32(q), _f64(means)
    B, Hq, Tq, D = q.shape
    assert Tq == T
    Hkv, Nb = means.shape[1], means.shape[2]
    t_end = T if t_end is None else t_end
    rows = t_end - t_begin
    assert K >= n_first + 1
    idx = np.empty((B, Hq, rows, K), dtype=np.int32)
    sc = np.empty((B, Hq, rows, Nb), dtype=np.float64) if want_scores else None
    lib().ref_moba_select(_i64(B), _i64(Hq), _i64(Hkv), _i64(D), _i64(T), _i64(block), _i64(K),
                          _i64(n_first), _p(q), _p(means), _i64(t_begin), _i64(t_end), _p(idx),
                          _p(sc))
    return (idx, sc) if want_scores else idx


def sparse_attn_prefill(q, k_cache, v_cache, T, block, scale, idx=None, t_begin=0, t_end=None):
    """Eq. 4 at prefill for rows [t_begin, t_end).  Returns (out [B,Hq,rows,D], lse [B,Hq,rows])."""
    q, k_cache, v_cache = _f32(q), _f32(k_cache), _f32(v_cache)
    B, Hq, Tq, D = q.shape
    assert Tq == T
    Hkv, Tcap = k_cache.shape[1], k_cache.shape[2]
    t_end = T if t_end is None else t_end
    rows = t_end - t_begin
    K = 0
    if idx is not None:
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        K = idx.shape[-1]
        assert idx.shape == (B, Hq, rows, K)
    out = np.empty((B, Hq, rows, D), dtype=np.float64)
    lse = np.empty((B, Hq, rows), dtype=np.float64)
    lib().ref_sparse_attn_prefill(_i64(B), _i64(Hq), _i64(Hkv), _i64(D), _i64(T), _i64(Tcap),
                                  _i64(block), _p(q), _p(k_cache), _p(v_cache), _dbl(scale),
                                  _p(idx), _i64(K), _i64(t_begin), _i64(t_end), _p(out), _p(lse))
    return out, lse


def snapkv_votes(q_win, k_cache, T, scale, want_window_mass=False):
    """q_win: [B, Hq, W, D] -> votes [B, Hkv, T-W] float64 (and window mass [B, Hq, W])."""
    q_win, k_cache = _f32(q_win), _f32(k_cache)
    B, Hq, W, D = q_win.shape
    Hkv, Tcap = k_cache.shape[1], k_cache.shape[2]
    votes = np.empty((B, Hkv, T - W), dtype=np.float64)
    wm = np.empty((B, Hq, W), dtype=np.float64) if want_window_mass else None
    lib().ref_snapkv_votes(_i64(B), _i64(Hq), _i64(Hkv), _i64(D), _i64(T), _i64(Tcap), _i64(W),
                           _p(q_win), _p(k_cache), _dbl(scale), _p(votes), _p(wm))
    return (votes, wm) if want_window_mass else votes


def maxpool1d(x, kernel):
    x = _f64(x)
    assert kernel % 2 == 1
    L = x.shape[-1]
    out = np.empty_like(x)
    lib().ref_maxpool1d(_i64(x.size // L), _i64(L), _i64(kernel), _p(x), _p(out))
    return out


def snapkv_select_gather(pooled, k_cache, v_cache, T, W, K_keep, Tcap_out=None):
    """Returns (idx [B,Hkv,K_keep], kc [B,Hkv,Tcap_out,D], vc) with rows 0..K_keep+W-1 filled."""
    pooled, k_cache, v_cache = _f64(pooled), _f32(k_cache), _f32(v_cache)
    B, H, Tcap, D = k_cache.shape
    assert pooled.shape == (B, H, T - W) and 0 <= K_keep <= T - W
    Tcap_out = K_keep + W if Tcap_out is None else Tcap_out
    idx = np.empty((B, H, K_keep), dtype=np.int32)
    kc = np.zeros((B, H, Tcap_out, D), dtype=np.float32)
    vc = np.zeros((B, H, Tcap_out, D), dtype=np.float32)
    lib().ref_snapkv_select_gather(_i64(B * H), _i64(T), _i64(Tcap), _i64(D), _i64(W),
                                   _i64(K_keep), _p(pooled), _p(k_cache), _p(v_cache),
                                   _i64(Tcap_out), _p(idx), _p(kc), _p(vc))
    return idx, kc, vc


def snapkv_compress(q_win, k_cache, v_cache, T, K_keep, pool_kernel, scale, Tcap_out=None):
    """Votes -> pool -> top-K_keep -> gather.  Returns dict(votes, pooled, idx, kc, vc)."""
    W = q_win.shape[2]
    votes = snapkv_votes(q_win, k_cache, T, scale)
    pooled = maxpool1d(votes, pool_kernel)
    idx, kc, vc = snapkv_select_gather(pooled, k_cache, v_cache, T, W, K_keep, Tcap_out)
    return dict(votes=votes, pooled=pooled, idx=idx, kc=kc, vc=vc)


def head_hit(idx_steps, gold_steps, unit=1):
    """Strict head-level hit (Sec. 2.3, H1): Hit_h = 1 only if at every step t the golden position
    g_t is among the candidates head h selected at that step.  idx_steps: per step an int array
    [B, H, K] of selected candidates (pages or tokens); gold_steps: per step an int array [B, H] of
    golden token positions (negative: none at that step for that head); unit: tokens per candidate
    (page size for page lists, 1 for token lists).  Returns a bool array [B, H]."""
    hit = None
    for idx, gold in zip(idx_steps, gold_steps):
        idx, gold = np.asarray(idx), np.asarray(gold)
        if hit is None:
            hit = np.ones(gold.shape, dtype=bool)
        for b in range(gold.shape[0]):
            for h in range(gold.shape[1]):
                if gold[b, h] >= 0 and (gold[b, h] // unit) not in set(int(x) for x in idx[b, h]):
                    hit[b, h] = False
    return hit
