"""Thin ctypes binding over libratsparse.so: same names as the C ABI, argument
marshalling only.  torch supplies device memory and the current HIP stream; every step
of the method runs in the library's kernels.  There is no fallback: if the library is
not built, or a call returns an error, this raises."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libratsparse.so")

RS_F32, RS_BF16 = 0, 1
RS_WS_CTRL_BYTES = 65536
RS_STATIC_SCRATCH_BYTES = 16 << 20

_lib = None


class RatsparseError(RuntimeError):
    pass


class rs_shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("Tcap", ctypes.c_int32), ("P", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


_vp, _i64, _i32, _f32, _sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float,
                              ctypes.c_size_t)
_shp = ctypes.POINTER(rs_shape)

# every symbol include/ratsparse.h declares: name -> (restype, argtypes)
SIGNATURES = {
    "ratsparse_status_string": (ctypes.c_char_p, [_i32]),
    "ratsparse_version": (ctypes.c_char_p, []),
    "ratsparse_workspace_init": (_i32, [_vp, _sz, _vp]),
    "ratsparse_async_status": (_i32, [_vp, _vp]),
    "ratsparse_probe_read": (_i32, [_vp, _sz, _vp, _i32, _vp]),
    "ratsparse_probe_rw": (_i32, [_vp, _vp, _vp, _sz, _i32, _vp]),
    "ratsparse_debug_set_spin_limit": (None, [_i32]),
    "ratsparse_debug_reload_knobs": (None, []),
    "rat_scan_workspace_bytes": (_sz, [_shp, _i64]),
    "rat_scan": (_i32, [_shp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _vp, _sz, _vp]),
    "quest_page_meta": (_i32, [_shp, _vp, _vp, _i64, _i64, _vp]),
    "quest_select_decode_workspace_bytes": (_sz, [_shp, _i64]),
    "quest_select_decode": (_i32, [_shp, _vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "quest_select_decode_group": (_i32, [_shp, _vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "sparse_attn_decode_group": (_i32, [_shp, _vp, _vp, _vp, _i64, _f32, _vp, _i32, _vp, _i32, _i32, _vp,
                                        _vp, _vp, _vp, _sz, _vp]),
    "sparse_attn_decode_workspace_bytes": (_sz, [_shp, _i64, _i32]),
    "sparse_attn_decode": (_i32, [_shp, _vp, _vp, _vp, _i64, _f32, _vp, _i32, _vp, _i32, _i32, _vp,
                                  _vp, _vp, _vp, _sz, _vp]),
    "sparse_attn_decode_static": (_i32, [_shp, _vp, _vp, _vp, _i64, _f32, _vp, _i32, _vp, _i32, _i32, _vp,
                                         _vp, _vp, _vp, _vp]),
    "rat_decode_step_workspace_bytes": (_sz, [_shp, _i64, _i32]),
    "rat_decode_state_set": (_i32, [_vp, _sz, _i64, _vp]),
    "rat_decode_state_get": (_i32, [_vp, ctypes.POINTER(ctypes.c_int64), _vp]),
    "rat_decode_step": (_i32, [_shp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _f32, _i32, _i32, _i32, _i64,
                               _vp, _vp, _vp, _vp, _sz, _vp]),
    "selection_hit_update": (_i32, [_vp, _i32, _i32, _i32, _vp, _i32, _vp, _vp]),
    "moba_select_prefill_workspace_bytes": (_sz, [_shp, _i64, _i32]),
    "moba_select_prefill": (_i32, [_shp, _vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
    "sparse_attn_prefill_workspace_bytes": (_sz, [_shp, _i64, _i32, _i32]),
    "sparse_attn_prefill": (_i32, [_shp, _vp, _vp, _vp, _i64, _i32, _f32, _vp, _i32, _vp, _vp, _vp,
                                   _sz, _vp]),
    "snapkv_compress_workspace_bytes": (_sz, [_shp, _i64, _i32]),
    "snapkv_compress": (_i32, [_shp, _vp, _vp, _vp, _i64, _i32, _i32, _i32, _f32, _vp, _vp, _i64,
                               _vp, _vp, _vp, _sz, _vp]),
    "snapkv_compress_lse": (_i32, [_shp, _vp, _vp, _vp, _i64, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _i64,
                                   _vp, _vp, _vp, _sz, _vp]),
}


def load():
    """Load libratsparse.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RatsparseError(
                "libratsparse.so is not built: run `python -m paper_2605_28640_amd.build` "
                "(needs hipcc); there is no CPU fallback")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(status):
    if status != 0:
        raise RatsparseError("ratsparse: %s (status %d)" %
                             (load().ratsparse_status_string(status).decode(), status))


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return RS_BF16
    if t.dtype == torch.float32:
        return RS_F32
    raise RatsparseError("storage dtype must be float32 or bfloat16")


def make_shape(B, Hq, Hkv, D, Tcap, P, dtype):
    code = dtype if isinstance(dtype, int) else (RS_BF16 if dtype == torch.bfloat16 else RS_F32)
    return rs_shape(B, Hq, Hkv, D, Tcap, P, code)


class Workspace:
    """A device scratch buffer with zeroed control words."""

    def __init__(self, nbytes, device="cuda"):
        nbytes = max(int(nbytes), RS_WS_CTRL_BYTES)
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _check(load().ratsparse_workspace_init(self.buf.data_ptr(), self.buf.numel(), _stream()))

    @property
    def ptr(self):
        return self.buf.data_ptr()

    @property
    def nbytes(self):
        return self.buf.numel()

    def async_status(self):
        _check(load().ratsparse_async_status(self.ptr, _stream()))


def ratsparse_probe_read(src, nbytes, sink, streaming=0):
    _check(load().ratsparse_probe_read(_ptr(src), nbytes, _ptr(sink), streaming, _stream()))


def ratsparse_probe_rw(a, b, dst, nbytes, streaming=0):
    _check(load().ratsparse_probe_rw(_ptr(a), _ptr(b), _ptr(dst), nbytes, streaming, _stream()))


def rat_scan_workspace_bytes(s, T_new):
    return load().rat_scan_workspace_bytes(ctypes.byref(s), T_new)


def rat_scan(s, k, v, g, state_k, state_v, k_cache, v_cache, t0, T_new, ws=None, meta=None):
    _check(load().rat_scan(ctypes.byref(s), _ptr(k), _ptr(v), _ptr(g), _ptr(state_k), _ptr(state_v),
                           _ptr(k_cache), _ptr(v_cache), _ptr(meta), t0, T_new, ws.ptr if ws else None,
                           ws.nbytes if ws else 0, _stream()))


def quest_page_meta(s, k_cache, meta, t_begin, t_end):
    _check(load().quest_page_meta(ctypes.byref(s), _ptr(k_cache), _ptr(meta), t_begin, t_end, _stream()))


def quest_select_decode_workspace_bytes(s, T_valid):
    return load().quest_select_decode_workspace_bytes(ctypes.byref(s), T_valid)


def quest_select_decode(s, q, meta, T_valid, K, n_first, n_local, idx_out, scores_out, ws):
    _check(load().quest_select_decode(ctypes.byref(s), _ptr(q), _ptr(meta), T_valid, K, n_first, n_local,
                                      _ptr(idx_out), _ptr(scores_out), ws.ptr, ws.nbytes, _stream()))


def quest_select_decode_group(s, q, meta, T_valid, K, n_first, n_local, idx_out, scores_out, ws):
    _check(load().quest_select_decode_group(ctypes.byref(s), _ptr(q), _ptr(meta), T_valid, K, n_first, n_local,
                                            _ptr(idx_out), _ptr(scores_out), ws.ptr, ws.nbytes, _stream()))


def sparse_attn_decode_group(s, q, k_cache, v_cache, T_valid, scale, idx, K, meta, n_first, n_local, out,
                             lse_out, idx_out, ws):
    _check(load().sparse_attn_decode_group(ctypes.byref(s), _ptr(q), _ptr(k_cache), _ptr(v_cache), T_valid,
                                           scale, _ptr(idx), K, _ptr(meta), n_first, n_local, _ptr(out),
                                           _ptr(lse_out), _ptr(idx_out), ws.ptr, ws.nbytes, _stream()))


def rat_decode_step_workspace_bytes(s, T_max, K):
    return load().rat_decode_step_workspace_bytes(ctypes.byref(s), T_max, K)


def rat_decode_state_set(ws, T):
    _check(load().rat_decode_state_set(ws.ptr, ws.nbytes, T, _stream()))


def rat_decode_state_get(ws):
    T = ctypes.c_int64(0)
    _check(load().rat_decode_state_get(ws.ptr, ctypes.byref(T), _stream()))
    return T.value


def rat_decode_step(s, k, v, g, state_k, state_v, k_cache, v_cache, meta, q, scale, K, n_first, n_local, T_max,
                    out, lse_out, idx_out, ws):
    _check(load().rat_decode_step(ctypes.byref(s), _ptr(k), _ptr(v), _ptr(g), _ptr(state_k), _ptr(state_v),
                                  _ptr(k_cache), _ptr(v_cache), _ptr(meta), _ptr(q), scale, K, n_first, n_local,
                                  T_max, _ptr(out), _ptr(lse_out), _ptr(idx_out), ws.ptr, ws.nbytes, _stream()))


def selection_hit_update(idx, gold, unit, hit):
    B, H, K = idx.shape
    assert gold.shape == (B, H) and hit.shape == (B, H) and hit.dtype == torch.uint8
    _check(load().selection_hit_update(_ptr(idx), B, H, K, _ptr(gold), unit, _ptr(hit), _stream()))


def sparse_attn_decode_workspace_bytes(s, T_valid, K):
    return load().sparse_attn_decode_workspace_bytes(ctypes.byref(s), T_valid, K)


def sparse_attn_decode(s, q, k_cache, v_cache, T_valid, scale, idx, K, meta, n_first, n_local, out,
                       lse_out, idx_out, ws):
    _check(load().sparse_attn_decode(ctypes.byref(s), _ptr(q), _ptr(k_cache), _ptr(v_cache), T_valid,
                                     scale, _ptr(idx), K, _ptr(meta), n_first, n_local, _ptr(out),
                                     _ptr(lse_out), _ptr(idx_out), ws.ptr, ws.nbytes, _stream()))


def sparse_attn_decode_static(s, q, k_cache, v_cache, T_valid, scale, idx, K, meta, n_first, n_local, out,
                              lse_out, idx_out, async_err):
    _check(load().sparse_attn_decode_static(ctypes.byref(s), _ptr(q), _ptr(k_cache), _ptr(v_cache), T_valid,
                                            scale, _ptr(idx), K, _ptr(meta), n_first, n_local, _ptr(out),
                                            _ptr(lse_out), _ptr(idx_out), _ptr(async_err), _stream()))


def moba_select_prefill_workspace_bytes(s, T, block):
    return load().moba_select_prefill_workspace_bytes(ctypes.byref(s), T, block)


def moba_select_prefill(s, q, k_cache, T, block, K, n_first, means_out, idx_out, ws):
    _check(load().moba_select_prefill(ctypes.byref(s), _ptr(q), _ptr(k_cache), T, block, K, n_first,
                                      _ptr(means_out), _ptr(idx_out), ws.ptr, ws.nbytes, _stream()))


def sparse_attn_prefill_workspace_bytes(s, T, block, K):
    return load().sparse_attn_prefill_workspace_bytes(ctypes.byref(s), T, block, K)


def sparse_attn_prefill(s, q, k_cache, v_cache, T, block, scale, idx, K, out, lse_out, ws):
    _check(load().sparse_attn_prefill(ctypes.byref(s), _ptr(q), _ptr(k_cache), _ptr(v_cache), T, block,
                                      scale, _ptr(idx), K, _ptr(out), _ptr(lse_out), ws.ptr, ws.nbytes,
                                      _stream()))


def snapkv_compress_workspace_bytes(s, T, W):
    return load().snapkv_compress_workspace_bytes(ctypes.byref(s), T, W)


def snapkv_compress(s, q_win, k_cache, v_cache, T, W, K_keep, pool_kernel, scale, kc_out, vc_out,
                    Tcap_out, idx_out, votes_out, ws):
    _check(load().snapkv_compress(ctypes.byref(s), _ptr(q_win), _ptr(k_cache), _ptr(v_cache), T, W,
                                  K_keep, pool_kernel, scale, _ptr(kc_out), _ptr(vc_out), Tcap_out,
                                  _ptr(idx_out), _ptr(votes_out), ws.ptr, ws.nbytes, _stream()))


def snapkv_compress_lse(s, q_win, k_cache, v_cache, T, W, K_keep, pool_kernel, scale, lse_win, kc_out, vc_out,
                        Tcap_out, idx_out, votes_out, ws):
    _check(load().snapkv_compress_lse(ctypes.byref(s), _ptr(q_win), _ptr(k_cache), _ptr(v_cache), T, W,
                                      K_keep, pool_kernel, scale, _ptr(lse_win), _ptr(kc_out), _ptr(vc_out),
                                      Tcap_out, _ptr(idx_out), _ptr(votes_out), ws.ptr, ws.nbytes, _stream()))
