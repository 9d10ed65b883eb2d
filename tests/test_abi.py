"""The C-ABI library loads on a machine without a GPU and exports every symbol that
include/ratsparse.h declares; the binding declares the same set."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ratsparse.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"})


def test_library_exports_every_declared_symbol():
    from paper_2605_28640_amd import binding
    names = _declared()
    assert {"rat_scan", "quest_page_meta", "quest_select_decode", "moba_select_prefill",
            "snapkv_compress", "sparse_attn_decode", "sparse_attn_prefill"} <= set(names)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.SIGNATURES), set(names) ^ set(binding.SIGNATURES)


def test_status_strings_and_host_side_validation():
    from paper_2605_28640_amd import binding
    lib = binding.load()
    assert lib.ratsparse_status_string(0) == b"ok"
    assert b"gfx950" in lib.ratsparse_version()
    bad = binding.make_shape(1, 3, 2, 128, 64, 16, binding.RS_BF16)  # Hq not a multiple of Hkv
    assert lib.rat_scan_workspace_bytes(ctypes.byref(bad), 64) == 0
    s = binding.make_shape(1, 2, 2, 96, 64, 16, binding.RS_BF16)  # unsupported head dim
    assert lib.quest_page_meta(ctypes.byref(s), 16, 16, 0, 16, None) == 2
    s = binding.make_shape(1, 2, 2, 128, 64, 16, binding.RS_BF16)
    assert lib.quest_page_meta(ctypes.byref(s), None, None, 0, 16, None) == 1  # null pointers
    assert lib.quest_page_meta(ctypes.byref(s), 16, 16, 0, 65, None) == 1  # past the capacity
    assert lib.rat_scan_workspace_bytes(ctypes.byref(s), 4096) > binding.RS_WS_CTRL_BYTES


def test_every_entry_point_rejects_bad_arguments_before_touching_the_gpu():
    """Argument validation is synchronous and comes before any launch: with made-up (non-null,
    16-byte aligned, never dereferenced) addresses each entry point must answer with
    1 = invalid argument, 2 = unsupported or 3 = workspace too small."""
    from paper_2605_28640_amd import binding
    lib = binding.load()
    A = 1 << 20  # an aligned made-up address
    s = binding.make_shape(1, 4, 2, 128, 256, 16, binding.RS_BF16)
    sp = ctypes.byref(s)
    big = 1 << 30

    # rat_scan(s, k, v, g, state_k, state_v, k_cache, v_cache, meta, t0, T_new, ws, ws_bytes, stream)
    assert lib.rat_scan(sp, None, A, A, A, A, A, A, None, 0, 16, A, big, None) == 1
    assert lib.rat_scan(sp, A, A, A, A, A, A, A, None, 250, 16, A, big, None) == 1      # runs past Tcap
    assert lib.rat_scan(sp, A, A, A, A, A, A, A, None, 0, 0, A, big, None) == 1         # no tokens
    assert lib.rat_scan(sp, A, A, A, A, A, A, A, A + 4, 0, 16, A, big, None) == 1       # misaligned meta
    assert lib.rat_scan(sp, A, A, A, A, A, A, A, None, 0, 256, A, 16, None) == 3        # workspace too small

    # quest_select_decode(s, q, meta, T_valid, K, n_first, n_local, idx_out, scores_out, ws, ws_bytes, stream)
    assert lib.quest_select_decode(sp, A, A, 256, 17, 1, 1, A, None, A, big, None) == 1  # K > pages
    assert lib.quest_select_decode(sp, A, A, 256, 2, 2, 2, A, None, A, big, None) == 1   # forced pages > K
    assert lib.quest_select_decode(sp, A, A, 257, 4, 1, 1, A, None, A, big, None) == 1   # T_valid > Tcap
    assert lib.quest_select_decode(sp, A, None, 256, 4, 1, 1, A, None, A, big, None) == 1
    assert lib.quest_select_decode(sp, A, A, 256, 4, 1, 1, A, None, A, 16, None) == 3
    assert lib.quest_select_decode(sp, A, A, 256, 4, 1, 1, A, None, None, big, None) == 3

    # sparse_attn_decode(s, q, k_cache, v_cache, T_valid, scale, idx, K, meta, n_first, n_local, out,
    #                    lse_out, idx_out, ws, ws_bytes, stream)
    assert lib.sparse_attn_decode(sp, A, A, A, 0, 0.1, None, 0, None, 0, 0, A, None, None, A, big, None) == 1
    assert lib.sparse_attn_decode(sp, A, A, A, 256, 0.1, A, 17, None, 0, 0, A, None, None, A, big, None) == 1
    assert lib.sparse_attn_decode(sp, A, A, A, 256, 0.1, None, 4, A + 8, 1, 1, A, None, None, A, big, None) == 1
    assert lib.sparse_attn_decode(sp, A, A, A, 256, 0.1, None, 4, A, 1, 1, None, None, None, A, big, None) == 1
    assert lib.sparse_attn_decode(sp, A, A, A, 256, 0.1, None, 4, A, 1, 1, A, None, None, A, 16, None) == 3

    # sparse_attn_decode_static(s, q, k_cache, v_cache, T_valid, scale, idx, K, meta, n_first, n_local, out,
    #                           lse_out, idx_out, async_err, stream): validation precedes any GPU call
    assert lib.sparse_attn_decode_static(sp, A, A, A, 256, 0.1, None, 4, A, 1, 1, A, None, None, None, None) == 1
    assert lib.sparse_attn_decode_static(sp, A, A, A, 257, 0.1, None, 4, A, 1, 1, A, None, None, A, None) == 1
    assert lib.sparse_attn_decode_static(sp, A, A, A, 256, 0.1, None, 0, A, 1, 1, A, None, None, A, None) == 1
    huge = binding.make_shape(16, 32, 32, 128, 66048, 16, binding.RS_BF16)
    assert lib.sparse_attn_decode_static(ctypes.byref(huge), A, A, A, 66048, 0.1, None, 1024, A, 1, 1, A, None, None,
                                         A, None) == 6  # more scratch than the static array holds

    # rat_decode_step(s, k, v, g, state_k, state_v, k_cache, v_cache, meta, q, scale, K, n_first, n_local,
    #                 T_max, out, lse_out, idx_out, ws, ws_bytes, stream)
    assert lib.rat_decode_step(sp, A, A, A, A, A, A, A, None, A, 0.1, 4, 1, 1, 256, A, None, None, A, big, None) == 1
    assert lib.rat_decode_step(sp, A, A, A, A, A, A, A, A, A, 0.1, 17, 1, 1, 256, A, None, None, A, big, None) == 1
    assert lib.rat_decode_step(sp, A, A, A, A, A, A, A, A, A, 0.1, 4, 3, 2, 256, A, None, None, A, big, None) == 1
    assert lib.rat_decode_step(sp, A, A, A, A, A, A, A, A, A, 0.1, 4, 1, 1, 257, A, None, None, A, big, None) == 1
    assert lib.rat_decode_step(sp, A, A, A, A, A, A, A, A, A + 4, 0.1, 4, 1, 1, 256, A, None, None, A, big, None) == 1
    assert lib.rat_decode_step(sp, A, A, A, A, A, A, A, A, A, 0.1, 4, 1, 1, 256, A, None, None, A, 16, None) == 3
    assert lib.rat_decode_state_set(None, big, 0, None) == 1
    assert lib.rat_decode_state_set(A, big, -1, None) == 1
    assert lib.rat_decode_state_set(A, 16, 0, None) == 3
    assert lib.rat_decode_state_get(None, None, None) == 1
    assert lib.rat_decode_step_workspace_bytes(sp, 257, 4) == 0

    # selection_hit_update(idx, B, H, K, gold, unit, hit, stream)
    assert lib.selection_hit_update(None, 1, 2, 4, A, 16, A, None) == 1
    assert lib.selection_hit_update(A, 1, 2, 4, A, 0, A, None) == 1      # unit must be positive
    assert lib.selection_hit_update(A, 0, 2, 4, A, 16, A, None) == 1
    assert lib.selection_hit_update(A + 2, 1, 2, 4, A, 16, A, None) == 1  # misaligned list

    # moba_select_prefill(s, q, k_cache, T, block, K, n_first, means_out, idx_out, ws, ws_bytes, stream)
    assert lib.moba_select_prefill(sp, A, A, 256, 24, 3, 0, A, A, A, big, None) == 1     # block not a multiple of 16
    assert lib.moba_select_prefill(sp, A, A, 256, 64, 33, 0, A, A, A, big, None) == 1    # K > 32
    assert lib.moba_select_prefill(sp, A, A, 256, 64, 1, 1, A, A, A, big, None) == 1     # no room for own block
    assert lib.moba_select_prefill(sp, A, A, 512, 64, 3, 0, A, A, A, big, None) == 1     # T > Tcap
    assert lib.moba_select_prefill(sp, A, A, 256, 64, 3, 0, A, A, A, 16, None) == 3

    # sparse_attn_prefill(s, q, k_cache, v_cache, T, block, scale, idx, K, out, lse_out, ws, ws_bytes, stream)
    assert lib.sparse_attn_prefill(sp, A, A, A, 256, 64, 0.1, A, 0, A, None, A, big, None) == 1
    assert lib.sparse_attn_prefill(sp, A, A, A, 256, 64, 0.1, A + 4, 3, A, None, A, big, None) == 1
    assert lib.sparse_attn_prefill(sp, A, A, None, 256, 64, 0.1, None, 0, A, None, A, big, None) == 1
    assert lib.sparse_attn_prefill(sp, A, A, A, 256, 64, 0.1, A, 3, A, None, A, 16, None) == 3
    f32 = binding.make_shape(1, 4, 2, 128, 256, 16, binding.RS_F32)  # the matrix-core paths store bf16
    assert lib.sparse_attn_prefill(ctypes.byref(f32), A, A, A, 256, 64, 0.1, None, 0, A, None, A, big, None) == 2

    # snapkv_compress(s, q_win, k_cache, v_cache, T, W, K_keep, pool_kernel, scale, kc_out, vc_out,
    #                 Tcap_out, idx_out, votes_out, ws, ws_bytes, stream)
    assert lib.snapkv_compress(sp, A, A, A, 256, 32, 64, 4, 0.1, A, A, 128, A, None, A, big, None) == 1   # even pool
    assert lib.snapkv_compress(sp, A, A, A, 256, 256, 0, 7, 0.1, A, A, 512, A, None, A, big, None) == 1   # W >= T
    assert lib.snapkv_compress(sp, A, A, A, 256, 32, 225, 7, 0.1, A, A, 512, A, None, A, big, None) == 1  # keep > T - W
    assert lib.snapkv_compress(sp, A, A, A, 256, 32, 64, 7, 0.1, A, A, 64, A, None, A, big, None) == 1    # output too short
    assert lib.snapkv_compress(sp, A, A, A, 256, 32, 64, 7, 0.1, A, A, 128, A, None, A, 16, None) == 3

    # snapkv_compress_lse(..., scale, lse_win, kc_out, ...): the log-sum-exp is required
    assert lib.snapkv_compress_lse(sp, A, A, A, 256, 32, 64, 7, 0.1, None, A, A, 128, A, None, A, big, None) == 1
    assert lib.snapkv_compress_lse(sp, A, A, A, 256, 32, 64, 7, 0.1, A + 4, A, A, 128, A, None, A, big, None) == 1
    assert lib.snapkv_compress_lse(sp, A, A, A, 256, 32, 64, 4, 0.1, A, A, A, 128, A, None, A, big, None) == 1
    assert lib.snapkv_compress_lse(sp, A, A, A, 256, 32, 64, 7, 0.1, A, A, A, 128, A, None, A, 16, None) == 3

    # more pages than the selection's LDS keys hold
    huge = binding.make_shape(1, 1, 1, 64, 15361 * 16, 16, binding.RS_BF16)
    hp = ctypes.byref(huge)
    n = lib.sparse_attn_decode_workspace_bytes(hp, 15361 * 16, 4)
    assert lib.quest_select_decode(hp, A, A, 15361 * 16, 4, 1, 1, A, None, A, n, None) == 2
    assert lib.sparse_attn_decode(hp, A, A, A, 15361 * 16, 0.1, None, 4, A, 1, 1, A, None, None, A, n, None) == 2
    assert lib.rat_decode_step(hp, A, A, A, A, A, A, A, A, A, 0.1, 4, 1, 1, 15361 * 16, A, None, None, A, n, None) == 2

    # shapes
    for bad in (binding.make_shape(0, 4, 2, 128, 256, 16, binding.RS_BF16),
                binding.make_shape(1, 4, 2, 128, 250, 16, binding.RS_BF16)):  # Tcap not a multiple of P
        assert lib.quest_page_meta(ctypes.byref(bad), A, A, 0, 16, None) == 1
    odd_page = binding.make_shape(1, 4, 2, 128, 240, 48, binding.RS_BF16)
    assert lib.quest_page_meta(ctypes.byref(odd_page), A, A, 0, 16, None) == 2
    for code in (1, 2, 3, 4, 5):
        assert len(lib.ratsparse_status_string(code)) > 0
