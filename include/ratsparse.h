/*
 * ratsparse.h -- C ABI of the MI355X (gfx950) library for attention over an
 * exponentially-decaying-memory KV cache under query-aware sparsity.
 *
 * The library covers the data-parallel hot path of the method: the gated decay
 * recurrence that produces the augmented states (Sec. 2.1, Eq. 1), query-aware
 * candidate selection (Sec. 2.2, Eq. 3) in its three evaluated forms (Quest pages,
 * MoBA blocks, SnapKV tokens; App. A.1), and softmax attention over the selected
 * states (Sec. 2.2, Eq. 4), with the dense path as the full-budget case.
 *
 * Conventions (all entry points)
 *   - Every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned.
 *     The library allocates nothing, frees nothing and keeps no pointer after a call
 *     returns.  `const rs_shape *` is a HOST pointer, read during the call only.
 *   - Tensors are C-contiguous, last dimension fastest.  `dtype` is the storage
 *     type of q, k, v, both caches, page metadata and attention outputs (RS_F32 or
 *     RS_BF16).  Gates, recurrence carries, block means, votes, scores and lse are
 *     always float32; index lists are int32.  All arithmetic accumulates in float32.
 *   - Query head h reads KV head h / (Hq / Hkv).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void *; NULL = the
 *     default stream) and the call returns without waiting for it.  Arguments are
 *     validated synchronously before anything is enqueued.
 *   - Scratch memory is a caller buffer `ws` of at least <entry>_workspace_bytes()
 *     bytes.  Its first RS_WS_CTRL_BYTES are control words that must be zero when a
 *     call starts: zero them once with ratsparse_workspace_init(); every entry
 *     point leaves them zero again when its kernels have finished.  One workspace
 *     must not be used by two calls that can run at the same time.
 *   - Return value: RS_OK or an error code below.  Nothing is printed or thrown.
 *     A kernel-side failure of a bounded wait is recorded in the workspace and
 *     reported by ratsparse_async_status().
 *   - Outputs must not alias inputs, with one exception: rat_scan may run in place
 *     (k_cache == k and v_cache == v) when the two layouts coincide, i.e. t0 == 0 and
 *     T_new == Tcap; every row is read before it is overwritten.
 *   - Tuning knobs: a handful of RATSPARSE_* environment variables (work splits, grid sizes,
 *     forced kernel forms) are read once per process, under std::call_once, on the first
 *     call that needs one; after that no entry point touches the environment, and calls
 *     from several host threads see one consistent table.  Unset = the measured defaults.
 *     Changing the environment later has no effect (ratsparse_debug_reload_knobs is the
 *     test hook that re-reads it; do not call it while other threads are inside the library).
 *   - Threads: entry points may be called from several host threads as long as each call
 *     has its own workspace and stream; the only process-wide host state is the call-tag
 *     counter and the spin limit (both atomics) and the knob table above.
 *   - Stream capture: quest_page_meta, moba_select_prefill, sparse_attn_prefill and
 *     snapkv_compress keep no per-call state on the host and may be captured into a
 *     HIP graph and replayed.  rat_scan, quest_select_decode and sparse_attn_decode (and
 *     their _group forms) hand a fresh call tag to their kernels on every call (it tells this call's
 *     words in the workspace from stale ones) and must be called, not replayed.
 *     rat_decode_step keeps its tag and the sequence length on the device and may be replayed.
 */
#ifndef RATSPARSE_H
#define RATSPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    RS_OK = 0,
    RS_INVALID_ARG = 1,         /* null / misaligned pointer, non-positive size, K out of range, T > Tcap */
    RS_UNSUPPORTED = 2,         /* D not in {64,128}, page / block size not supported, dtype unknown */
    RS_WORKSPACE_TOO_SMALL = 3, /* ws == NULL or ws_bytes below <entry>_workspace_bytes() */
    RS_LAUNCH_FAILED = 4,       /* hipGetLastError() after a launch */
    RS_ASYNC_TIMEOUT = 5,       /* reported by ratsparse_async_status(): a bounded in-kernel wait expired */
    RS_SCRATCH_LIMIT = 6        /* sparse_attn_decode_static: the shape needs more than RS_STATIC_SCRATCH_BYTES */
};

enum { RS_F32 = 0, RS_BF16 = 1 };

/* bytes at the start of every workspace reserved for control words */
#define RS_WS_CTRL_BYTES 65536

/* size of the library's own scratch array, used by sparse_attn_decode_static only (16 MiB of
 * device memory on every GPU the library runs on, held until the process ends) */
#define RS_STATIC_SCRATCH_BYTES (16u << 20)

typedef struct rs_shape {
    int32_t B;     /* batch */
    int32_t Hq;    /* query heads */
    int32_t Hkv;   /* KV heads, divides Hq */
    int32_t D;     /* head dimension: 64 or 128 */
    int32_t Tcap;  /* rows per (batch, KV head) of the caches (row stride); multiple of P */
    int32_t P;     /* Quest page size in tokens: 16, 32, 64, 128, 256 or 512 (used by the page entry points) */
    int32_t dtype; /* RS_F32 or RS_BF16 */
} rs_shape;

const char *ratsparse_status_string(int32_t status);
const char *ratsparse_version(void);

/* Zero the control words of a freshly allocated workspace (needed once). */
int32_t ratsparse_workspace_init(void *ws, size_t ws_bytes, void *stream);

/* Waits for `stream`, then returns RS_OK, or RS_ASYNC_TIMEOUT if a kernel that used
 * `ws` gave up a bounded wait (its outputs are then undefined); clears the record. */
int32_t ratsparse_async_status(void *ws, void *stream);

/* Measurement aid (no part of the method): enqueue a plain streaming read of `bytes` bytes at
 * src (16-byte aligned device memory); sink is 4 bytes of device memory that is practically
 * never written; streaming != 0: with non-temporal loads (what the decode kernels use for K and
 * V rows).  The achieved rate is the read ceiling to hold a read-bound kernel against. */
int32_t ratsparse_probe_read(const void *src, size_t bytes, void *sink, int32_t streaming, void *stream);

/* Measurement aid (no part of the method): a plain streaming kernel with the traffic mix of
 * rat_scan (two bytes read for every byte written): dst[i] = a[i] ^ b[i] over `bytes` bytes of
 * each of the three 16-byte aligned device buffers; streaming != 0: with non-temporal loads and
 * stores (what rat_scan uses for whole rows).  3 * bytes over its duration is the rate a kernel
 * with that mix can be held against on this machine. */
int32_t ratsparse_probe_rw(const void *a, const void *b, void *dst, size_t bytes, int32_t streaming,
                           void *stream);

/* Test hook: the bound, in polls, of every in-kernel wait of calls made from now on (the
 * default is 1 << 22).  With 0 a kernel that would have to wait gives up at once, exits
 * normally and records RS_ASYNC_TIMEOUT: the error path can be tested without a hang. */
void ratsparse_debug_set_spin_limit(int32_t polls);

/* Test hook: read the RATSPARSE_* tuning variables again (they are read once per process). */
void ratsparse_debug_reload_knobs(void);

/* ---- Exponentially decaying memory: Sec. 2.1, Eq. 1 --------------------------------
 * For every (batch, KV head, channel):  s_t = g_t * s_{t-1} + (1 - g_t) * x_t  for the
 * T_new tokens given, for x = k and x = v with the same gate, starting from the carry.
 *   k, v   [B, Hkv, T_new, D] dtype      new keys / values
 *   g      [B, Hkv, T_new, D] float32    gates in [0, 1]
 *   state_k, state_v [B, Hkv, D] float32 in: s_{t0-1} (zeros for a fresh sequence);
 *                                        out: the unrounded state after the last token
 *   k_cache, v_cache [B, Hkv, Tcap, D] dtype   rows t0 .. t0+T_new-1 are written with
 *                                        the states rounded to nearest-even
 *   meta   [B, Hkv, Tcap/P, 2, D] dtype or NULL: if given, the Quest page metadata (as
 *                                        written by quest_page_meta) of every page that
 *                                        holds a new row is brought up to date in the same
 *                                        call; it must be current for the rows before t0
 * T_new = 1 is the decode-time append.  Requires 0 <= t0, t0 + T_new <= Tcap.
 * Evaluated as a chunked scan; the result equals the sequential recurrence up to
 * float32 rounding order. */
size_t rat_scan_workspace_bytes(const rs_shape *s, int64_t T_new);
int32_t rat_scan(const rs_shape *s, const void *k, const void *v, const float *g,
                 float *state_k, float *state_v, void *k_cache, void *v_cache, void *meta,
                 int64_t t0, int64_t T_new, void *ws, size_t ws_bytes, void *stream);

/* ---- Quest block representatives: App. A.1, Quest paragraph --------------------------
 * Per page of P tokens and per channel, the minimum and maximum stored key.
 *   k_cache [B, Hkv, Tcap, D] dtype
 *   meta    [B, Hkv, Tcap/P, 2, D] dtype   row 0 = min, row 1 = max
 * Recomputes every page that intersects [t_begin, t_end), over its tokens t < t_end
 * (the tokens of a page that lie before t_begin are read too).  Use [0, T) after a
 * prefill and [t, t+1) after appending token t. */
int32_t quest_page_meta(const rs_shape *s, const void *k_cache, void *meta, int64_t t_begin,
                        int64_t t_end, void *stream);

/* ---- Quest page selection at decode: Sec. 2.2, Eq. 3; App. A.1 ------------------------
 * score_p = sum_c max(q_c * min_{p,c}, q_c * max_{p,c}) over the Np = ceil(T_valid/P)
 * pages; per (batch, query head) the K best pages, larger score first, lower index
 * first among equal scores.  Pages 0 .. n_first-1 and the last n_local pages are
 * always kept and count inside K.
 *   q          [B, Hq, D] dtype
 *   meta       [B, Hkv, Tcap/P, 2, D] dtype, as quest_page_meta or rat_scan leave it: row 0 <= row 1 in
 *              every channel (the score is evaluated as q_c times the row the sign of q_c picks, which is
 *              the larger of the two products only then)
 *   idx_out    [B, Hq, K] int32, ascending
 *   scores_out [B, Hq, Np] float32 or NULL
 * Requires 1 <= K <= Np <= 15360 and K >= number of always-kept pages. */
size_t quest_select_decode_workspace_bytes(const rs_shape *s, int64_t T_valid);
int32_t quest_select_decode(const rs_shape *s, const void *q, const void *meta,
                            int64_t T_valid, int32_t K, int32_t n_first, int32_t n_local,
                            int32_t *idx_out, float *scores_out, void *ws, size_t ws_bytes,
                            void *stream);

/* ---- Sparse evaluation at decode: Sec. 2.2, Eq. 4 (f = softmax) -----------------------
 * y = softmax(scale * q K~_I^T) V~_I over the tokens t < T_valid of the selected pages.
 * Three modes:
 *   idx != NULL                 attend the K listed pages ([B, Hq, K] int32; entries < 0
 *                               are skipped; each page at most once);
 *   idx == NULL, meta != NULL   fused select-then-attend: selection exactly as
 *                               quest_select_decode, unselected KV is never read;
 *                               idx_out ([B, Hq, K] or NULL) receives the selection;
 *   idx == NULL, meta == NULL   dense attention over all tokens t < T_valid (full budget).
 *   out     [B, Hq, D] dtype
 *   lse_out [B, Hq] float32 or NULL: log-sum-exp of the scaled logits */
size_t sparse_attn_decode_workspace_bytes(const rs_shape *s, int64_t T_valid, int32_t K);
int32_t sparse_attn_decode(const rs_shape *s, const void *q, const void *k_cache,
                           const void *v_cache, int64_t T_valid, float scale,
                           const int32_t *idx, int32_t K, const void *meta, int32_t n_first,
                           int32_t n_local, void *out, float *lse_out, int32_t *idx_out,
                           void *ws, size_t ws_bytes, void *stream);

/* ---- sparse_attn_decode without a workspace and without any allocation ------------------
 * For callers that cannot allocate or size device memory at the call: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same three modes, same
 * kernels and same results as sparse_attn_decode; the scratch (control words, tagged scores,
 * tagged page lists, split partials) is a device array of RS_STATIC_SCRATCH_BYTES inside the
 * library instead of the caller's workspace.  The call itself allocates and frees nothing
 * (no hipMalloc, no hipFree, no library routine that allocates); the first call on a
 * device looks up that device's copy of the array.
 *   async_err  device uint32, caller-owned, required: set to 1 by a kernel whose bounded wait
 *              expired (outputs then undefined); the caller zeroes it and reads it after
 *              synchronising.  It stands in for ratsparse_async_status(), which needs a workspace.
 * Limit: sparse_attn_decode_workspace_bytes(s, T_valid, K) (K = 0 in the dense mode) must not
 * exceed RS_STATIC_SCRATCH_BYTES, else RS_SCRATCH_LIMIT and nothing is enqueued.  B = 4 with
 * 32 heads at 64K tokens, 16-token pages, K = 1024 needs 14.2 MiB.
 * Every call on a GPU uses that GPU's one array: calls that can overlap on one GPU (two
 * streams, two host threads) race and must be serialised by the caller.  The array keeps
 * the previous call's contents; each call first clears the control words with a small
 * kernel (not a memset node), so a call that gave up a wait does not poison the next.
 * Like sparse_attn_decode it draws a fresh tag per call: call it, do not replay it. */
int32_t sparse_attn_decode_static(const rs_shape *s, const void *q, const void *k_cache,
                                  const void *v_cache, int64_t T_valid, float scale,
                                  const int32_t *idx, int32_t K, const void *meta, int32_t n_first,
                                  int32_t n_local, void *out, float *lse_out, int32_t *idx_out,
                                  uint32_t *async_err, void *stream);

/* ---- Group-shared Quest selection (an option for grouped-query attention) --------------
 * Not in the paper, which selects per query head (Sec. 2.2 and 2.3 define the selected set per head);
 * offered for Hq / Hkv in {2, 4, 8} so that the query heads of a KV head share one page set:
 * Eq. 3 with the score of a page summed over the group,
 *   score_p = sum_{h in group} sum_c max(q_{h,c} * min_{p,c}, q_{h,c} * max_{p,c}),
 * still an upper bound of the group's summed logit of any token of the page.  Same rules
 * for always-kept pages, ties and order as quest_select_decode.
 *   idx_out    [B, Hkv, K] int32, ascending
 *   scores_out [B, Hkv, Np] float32 or NULL
 * sparse_attn_decode_group attends such a list (idx [B, Hkv, K], used by every query head
 * of the KV head), or with idx == NULL and meta != NULL selects and then attends (two
 * launches; idx_out [B, Hkv, K] or NULL).  It has no dense mode (RS_INVALID_ARG).
 * Workspaces are sized by the functions of the per-head forms. */
int32_t quest_select_decode_group(const rs_shape *s, const void *q, const void *meta,
                                  int64_t T_valid, int32_t K, int32_t n_first, int32_t n_local,
                                  int32_t *idx_out, float *scores_out, void *ws,
                                  size_t ws_bytes, void *stream);
int32_t sparse_attn_decode_group(const rs_shape *s, const void *q, const void *k_cache,
                                 const void *v_cache, int64_t T_valid, float scale,
                                 const int32_t *idx, int32_t K, const void *meta,
                                 int32_t n_first, int32_t n_local, void *out, float *lse_out,
                                 int32_t *idx_out, void *ws, size_t ws_bytes, void *stream);

/* ---- One decode step whose length lives on the device (replayable) --------------------
 * The decode loop with Quest (Sec. 2.2; App. A.1): append token T of the gated cache
 * (Eq. 1 step, as rat_scan with T_new = 1 and meta), then select K pages (Eq. 3) and
 * attend them (Eq. 4) over the T + 1 stored tokens, as sparse_attn_decode's fused mode.
 * T is not an argument: it is a 64-bit word of the workspace's control block, read by the
 * kernels and advanced by one when the step has finished, together with the step's tag.
 * No argument changes from step to step, so a stream capture of one call can be replayed
 * for every following token (the caller refreshes the contents of k, v, g, q in place).
 *   rat_decode_state_set   enqueue: tokens already in the cache := T (after a prefill)
 *   rat_decode_state_get   waits for `stream`, then reads the token count into *T (host)
 *   k, v [B, Hkv, 1, D] dtype; g [B, Hkv, 1, D] float32; q [B, Hq, D]; the rest as in
 *   rat_scan and sparse_attn_decode.  T_max: the largest T + 1 the workspace is sized for
 *   (<= Tcap).  Per query head; select-then-attend in the form sparse_attn_decode would take for
 *   the shape at T_max (one workgroup per (batch, head), the two plain launches, or the one
 *   persistent launch), each reading the length and the tag from the workspace.
 * A step that would pass T_max, or that finds fewer than K pages, changes nothing (neither
 * carries, caches, page bounds nor count: the append kernel applies the same test as the
 * attention kernel) except that it sets the asynchronous error word
 * (ratsparse_async_status -> RS_ASYNC_TIMEOUT).  n_first + n_local <= K is required.
 * rat_decode_state_set must have run on the workspace before the first step (it also
 * draws the first tag; a workspace that was only zeroed starts at T = 0 with a fixed tag). */
size_t rat_decode_step_workspace_bytes(const rs_shape *s, int64_t T_max, int32_t K);
int32_t rat_decode_state_set(void *ws, size_t ws_bytes, int64_t T, void *stream);
int32_t rat_decode_state_get(void *ws, int64_t *T, void *stream);
int32_t rat_decode_step(const rs_shape *s, const void *k, const void *v, const float *g,
                        float *state_k, float *state_v, void *k_cache, void *v_cache,
                        void *meta, const void *q, float scale, int32_t K, int32_t n_first,
                        int32_t n_local, int64_t T_max, void *out, float *lse_out,
                        int32_t *idx_out, void *ws, size_t ws_bytes, void *stream);

/* ---- Strict head-level hit rate: Sec. 2.3 (H1) -----------------------------------------
 * Hit_h = 1 only if, at every decoding step, the candidates head h selected hold the golden
 * answer position of that step.  One call folds one step in:
 *   hit[b, h] := 0 if gold[b, h] >= 0 and gold[b, h] / unit is not in idx[b, h, :]
 *   idx  [B, H, K] int32: the lists written by quest_select_decode / sparse_attn_decode
 *        (H = Hq, unit = P: a page holds the position) or by snapkv_compress (H = Hkv, unit = 1)
 *   gold [B, H] int32: the golden token position of this step; negative = none for that head
 *   hit  [B, H] uint8, in/out; set it to 1 before the first step.  Pointers 4-byte aligned.
 * The mean of hit over heads after the last step is the hit rate. */
int32_t selection_hit_update(const int32_t *idx, int32_t B, int32_t H, int32_t K, const int32_t *gold,
                             int32_t unit, uint8_t *hit, void *stream);

/* ---- MoBA routing at prefill: Sec. 2.2, Eq. 3; App. A.1, MoBA paragraph ----------------
 * Block representative = mean of the stored keys of a block of `block` tokens (the
 * tail block over its valid tokens).  Each query token t, in block b(t) = t / block,
 * scores the blocks j < b(t) by q_t . mean_j; its own block and the first n_first
 * blocks are always kept and count inside K.
 *   q         [B, Hq, T, D] dtype
 *   means_out [B, Hkv, ceil(T/block), D] float32
 *   idx_out   [B, Hq, T, K] int32, ascending, padded with -1 when fewer than K exist
 * block is a multiple of 16; ceil(T/block) <= 256; 1 + n_first <= K <= 32. */
size_t moba_select_prefill_workspace_bytes(const rs_shape *s, int64_t T, int32_t block);
int32_t moba_select_prefill(const rs_shape *s, const void *q, const void *k_cache, int64_t T,
                            int32_t block, int32_t K, int32_t n_first, float *means_out,
                            int32_t *idx_out, void *ws, size_t ws_bytes, void *stream);

/* ---- Sparse evaluation at prefill: Sec. 2.2, Eq. 4 ------------------------------------
 * For every query token t: softmax attention over the tokens i <= t of its listed
 * blocks (idx [B, Hq, T, K] as written by moba_select_prefill), or causal dense
 * attention when idx == NULL.  A row's entries are distinct block numbers not above the
 * row's own block, in any order, negative entries are skipped; only listed blocks are
 * attended (the own block too only if listed); a row with nothing listed gets zeros and a
 * log-sum-exp of -inf.
 *   out     [B, Hq, T, D] dtype
 *   lse_out [B, Hq, T] float32 or NULL
 * Runs on the bf16 matrix cores: dtype must be RS_BF16 (RS_UNSUPPORTED otherwise);
 * ceil(T/block) <= 256 when idx != NULL; T < 2^27. */
size_t sparse_attn_prefill_workspace_bytes(const rs_shape *s, int64_t T, int32_t block,
                                           int32_t K);
int32_t sparse_attn_prefill(const rs_shape *s, const void *q, const void *k_cache,
                            const void *v_cache, int64_t T, int32_t block, float scale,
                            const int32_t *idx, int32_t K, void *out, float *lse_out,
                            void *ws, size_t ws_bytes, void *stream);

/* ---- SnapKV cache compression: App. A.1, SnapKV paragraph; Eq. 3 over single tokens ----
 * The W observation queries sit at positions T-W .. T-1 and attend causally; the vote
 * of a prefix position i < T-W is its attention probability summed over the W rows and
 * over the query heads of its KV head's group; votes are max-pooled (window
 * pool_kernel, odd, stride 1, clipped at the ends); per KV head the K_keep best
 * positions are kept (lower index first among equal votes), in ascending order,
 * followed by the W window rows.
 *   q_win    [B, Hq, W, D] dtype
 *   kc_out, vc_out [B, Hkv, Tcap_out, D] dtype: rows 0 .. K_keep+W-1 written
 *   idx_out  [B, Hkv, K_keep] int32
 *   votes_out [B, Hkv, T-W] float32 or NULL: the pooled votes
 * Decoding afterwards: rat_scan appends into kc_out / vc_out from row K_keep+W, then
 * dense sparse_attn_decode over them.  dtype must be RS_BF16; pool_kernel odd, <= 63. */
size_t snapkv_compress_workspace_bytes(const rs_shape *s, int64_t T, int32_t W);
int32_t snapkv_compress(const rs_shape *s, const void *q_win, const void *k_cache,
                        const void *v_cache, int64_t T, int32_t W, int32_t K_keep,
                        int32_t pool_kernel, float scale, void *kc_out, void *vc_out,
                        int64_t Tcap_out, int32_t *idx_out, float *votes_out, void *ws,
                        size_t ws_bytes, void *stream);

/* The same with the window rows' log-sum-exp handed in (an option, not in the paper): the
 * votes need each window row's softmax normaliser over all the keys it sees, which
 * snapkv_compress gets from a first sweep over the keys.  A caller that has just run the
 * prefill attention of those rows already holds it (lse_out of sparse_attn_prefill, rows
 * T-W .. T-1, same queries and scale); with it the keys are swept once instead of twice.
 *   lse_win [B, Hq, W] float32: log sum_{i <= T-W+w} exp(scale * q_w . k_i), natural log
 * The values are taken on trust (device memory cannot be checked at the call): it has to
 * be the dense causal normaliser over this very k_cache, so the lse_out of a routed prefill
 * (listed blocks only) does not qualify, and a wrong or non-finite entry gives wrong votes
 * for that row, no error.  Everything else as snapkv_compress, same workspace size. */
int32_t snapkv_compress_lse(const rs_shape *s, const void *q_win, const void *k_cache,
                            const void *v_cache, int64_t T, int32_t W, int32_t K_keep,
                            int32_t pool_kernel, float scale, const float *lse_win, void *kc_out,
                            void *vc_out, int64_t Tcap_out, int32_t *idx_out, float *votes_out,
                            void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif
