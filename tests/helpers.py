"""Comparison rules shared by the parity tests (no method arithmetic here)."""
import numpy as np


def scan_close(x, y):
    """fp32 scan states against the float64 oracle: |x-y| <= 1e-5 |y| + 1e-6 rms(y)."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    rms = np.sqrt(np.mean(y * y)) if y.size else 0.0
    err = np.abs(x - y)
    tol = 1e-5 * np.abs(y) + 1e-6 * rms
    return bool(np.all(err <= tol)), float(np.max(err - tol)) if y.size else 0.0


def bf16_ulp(y):
    """Spacing of the bfloat16 grid at |y| (float64 in, float64 out)."""
    y = np.abs(np.asarray(y, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(y, 2.0 ** -126)))
    return 2.0 ** (e - 7)


def bf16_store_ok(stored, exact):
    """A bf16 value written from an fp32 state that is within 1e-5 of `exact` must be
    one of the grid neighbours of `exact`: |stored-exact| <= ulp/2 + 1e-5|exact|
    (plus the rms floor of the scan tolerance)."""
    stored = np.asarray(stored, dtype=np.float64)
    exact = np.asarray(exact, dtype=np.float64)
    rms = np.sqrt(np.mean(exact * exact)) if exact.size else 0.0
    tol = 0.5 * bf16_ulp(exact) * (1 + 2.0 ** -6) + 1e-5 * np.abs(exact) + 1e-6 * rms
    return bool(np.all(np.abs(stored - exact) <= tol))


def attn_close(x, y, rate=2e-2):
    """Attention outputs, per row: ||x-y||_inf <= rate * max(||y||_inf, rms(y))."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    D = y.shape[-1]
    xr, yr = x.reshape(-1, D), y.reshape(-1, D)
    err = np.max(np.abs(xr - yr), axis=1)
    ref = np.maximum(np.max(np.abs(yr), axis=1), np.sqrt(np.mean(yr * yr, axis=1)))
    worst = float(np.max(err / np.maximum(ref, 1e-30))) if len(err) else 0.0
    return bool(np.all(err <= rate * ref)), worst


def topk_set_ok(scores, forced, K, got, band=1e-4):
    """Selection rule for one row.  `scores`: the oracle's float64 scores of the M
    candidates; `forced`: boolean mask of always-kept candidates; `got`: the index
    list under test.  With s_K the oracle's K-th best score among the free slots and
    band = 1e-4 |s_K|: every candidate above s_K + band must be chosen, none below
    s_K - band may be, forced ones must all be chosen, the list must hold K distinct
    ascending indices.  If no other candidate lies in the band the set is unique,
    so this demands bit-exact equality there."""
    scores = np.asarray(scores, dtype=np.float64)
    forced = np.asarray(forced, dtype=bool)
    got = np.asarray(got)
    M = scores.shape[0]
    if got.shape != (K,):
        return False, "wrong length"
    if K == 0:
        return True, ""
    if np.any(got < 0) or np.any(got >= M) or np.any(np.diff(got) <= 0):
        return False, "not distinct ascending in range"
    chosen = np.zeros(M, dtype=bool)
    chosen[got] = True
    if not np.all(chosen[forced]):
        return False, "forced candidate missing"
    free = K - int(forced.sum())
    if free < 0:
        return False, "more forced than K"
    if free == 0:
        return (True, "") if np.all(chosen == forced) else (False, "extra candidates")
    s_free = np.where(forced, -np.inf, scores)
    order = np.sort(s_free)[::-1]
    sK = order[free - 1]
    tol = band * abs(sK)
    must = (~forced) & (s_free > sK + tol)
    never = (~forced) & (s_free < sK - tol)
    if not np.all(chosen[must]):
        return False, "a candidate above the band is missing"
    if np.any(chosen[never]):
        return False, "a candidate below the band was chosen"
    return True, ""


def exact_topk(scores, forced, K):
    """Plain statement of Eq. 3 with lowest-index tie-break (numpy, for small rows)."""
    scores = np.asarray(scores, dtype=np.float64)
    forced = np.asarray(forced, dtype=bool)
    key = sorted(range(len(scores)), key=lambda i: (not forced[i], -scores[i], i))
    return np.array(sorted(key[:K]), dtype=np.int32)
