/*
 * ratsparse_ref.h -- CPU oracle for the recurrence-augmented sparse-attention path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, double-precision statement of
 * what the path computes, written from the paper's equations.  It shares no code,
 * header, table or helper with the HIP library, and the product never calls it:
 * only the tests, the smoke check and the bench's cpu_baseline leg may.
 *
 * Conventions
 *   - every pointer is a HOST pointer;
 *   - all tensors are C-contiguous, last dimension fastest;
 *   - floating inputs are `float` arrays that hold the stored values exactly
 *     (a bf16 value is a float whose low 16 mantissa bits are zero);
 *   - every sum, product, exponential and comparison is carried out in `double`;
 *   - outputs are `double` (never rounded to the cache dtype here; the caller
 *     rounds with ref_round_to_bf16 where the method stores a value);
 *   - query head h reads KV head h / (Hq / Hkv).
 *
 * Every function below has a pin in tests/ (closed forms, library special cases,
 * brute force, invariants): none is "parity unpinned".  The accuracy tables of the
 * paper need its trained checkpoints and are not reproduced: that part is unpinned
 * and out of scope.
 */
#ifndef RATSPARSE_REF_H
#define RATSPARSE_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* number of threads the parallel-over-(batch,head) loops will use */
int ref_num_threads(void);
void ref_set_num_threads(int n);

/* Round-to-nearest-even of a double straight to bfloat16 (8 significant bits,
 * float32 exponent range), returned as the float holding that value. */
void ref_round_to_bf16(int64_t n, const double *x, float *y);

/* Top-K of one row of M candidates (Eq. 3).  Candidates with forced[i] != 0 rank
 * above every score; otherwise larger score first, and among equal scores the
 * lower index first.  Writes the K chosen indices in ascending order.
 * forced may be NULL.  Requires 0 <= K <= M. */
void ref_topk_row(int64_t M, const double *score, const uint8_t *forced, int64_t K,
                  int32_t *idx_out);

/* Gated decay recurrence (Sec. 2.1, Eq. 1), for both k and v with the shared gate:
 *   s_t = g_t * s_{t-1} + (1 - g_t) * x_t,   per (batch, head, channel).
 * k, v, g: [BH, T, D].  state_k, state_v: [BH, D], read as s_{-1} and overwritten
 * with s_{T-1}.  k_out, v_out: [BH, T, D] unrounded states. */
void ref_rat_scan(int64_t BH, int64_t T, int64_t D, const float *k, const float *v,
                  const float *g, double *state_k, double *state_v, double *k_out,
                  double *v_out);

/* Quest block representatives (App. A.1, Quest paragraph): per page of P tokens and
 * per channel the minimum and maximum stored key over tokens t < T_valid.
 * k_cache: [BH, Tcap, D].  meta: [BH, Tcap/P, 2, D], row 0 = min, row 1 = max.
 * Only pages 0 .. ceil(T_valid/P)-1 are written. */
void ref_quest_page_meta(int64_t BH, int64_t Tcap, int64_t D, int64_t P,
                         const float *k_cache, int64_t T_valid, float *meta);

/* Quest page score, the channelwise upper bound of q.k over the page's box:
 *   score_p = sum_c max(q_c * min_{p,c}, q_c * max_{p,c}).
 * q: [B, Hq, D]; meta: [B, Hkv, Np_cap, 2, D]; scores: [B, Hq, Np]. */
void ref_quest_scores(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t Np_cap,
                      const float *q, const float *meta, int64_t Np, double *scores);

/* Eq. 3 for Quest: top-K pages per (batch, query head); pages 0..n_first-1 and the
 * last n_local pages are always kept and count inside K.  idx: [B*Hq, K] ascending. */
void ref_quest_select(int64_t BHq, int64_t Np, const double *scores, int64_t K,
                      int64_t n_first, int64_t n_local, int32_t *idx);

/* Eq. 4 at decode: softmax(scale * q K~_I^T) V~_I over the tokens t < T_valid of
 * the listed pages (idx: [B, Hq, K], entries < 0 are skipped), or over all tokens
 * t < T_valid when idx == NULL.  out: [B, Hq, D]; lse: [B, Hq] = log sum exp of the
 * scaled logits (may be NULL). */
void ref_sparse_attn_decode(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t Tcap,
                            int64_t P, const float *q, const float *k_cache,
                            const float *v_cache, int64_t T_valid, double scale,
                            const int32_t *idx, int64_t K, double *out, double *lse);

/* MoBA block representatives: mean of the stored keys of each block over the
 * tokens t < T.  means: [BH, ceil(T/block), D]. */
void ref_moba_block_means(int64_t BH, int64_t T, int64_t Tcap, int64_t D, int64_t block,
                          const float *k_cache, double *means);

/* MoBA routing for query rows t in [t_begin, t_end): candidates are the blocks
 * strictly before the row's own block, scored q_t . mean_j; the own block and the
 * first n_first blocks are always kept and count inside K.  idx: [B, Hq, rows, K]
 * ascending, padded with -1.  scores (may be NULL): [B, Hq, rows, Nb], NaN where
 * the block is not a candidate. */
void ref_moba_select(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t T,
                     int64_t block, int64_t K, int64_t n_first, const float *q,
                     const double *means, int64_t t_begin, int64_t t_end, int32_t *idx,
                     double *scores);

/* Eq. 4 at prefill for rows t in [t_begin, t_end): softmax attention of q_t over
 * the tokens i <= t of its listed blocks (idx: [B, Hq, rows, K], -1 skipped), or
 * over all i <= t when idx == NULL.  q: [B, Hq, T, D]; out: [B, Hq, rows, D];
 * lse: [B, Hq, rows] (may be NULL). */
void ref_sparse_attn_prefill(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t T,
                             int64_t Tcap, int64_t block, const float *q,
                             const float *k_cache, const float *v_cache, double scale,
                             const int32_t *idx, int64_t K, int64_t t_begin,
                             int64_t t_end, double *out, double *lse);

/* SnapKV votes (App. A.1, SnapKV paragraph): the W observation queries sit at
 * positions T-W .. T-1; each attends causally to positions 0 .. its own; the vote
 * of prefix position i < T-W is its attention probability summed over the W rows
 * and over the query heads of the KV head's group.  q_win: [B, Hq, W, D];
 * votes: [B, Hkv, T-W]; window_mass (may be NULL): [B, Hq, W] = probability each
 * row leaves on the window columns. */
void ref_snapkv_votes(int64_t B, int64_t Hq, int64_t Hkv, int64_t D, int64_t T,
                      int64_t Tcap, int64_t W, const float *q_win, const float *k_cache,
                      double scale, double *votes, double *window_mass);

/* 1-D max pooling, stride 1, window `kernel` (odd) centred on each position and
 * clipped at the ends.  in, out: [rows, L]. */
void ref_maxpool1d(int64_t rows, int64_t L, int64_t kernel, const double *in, double *out);

/* Keep the K_keep best prefix positions per KV head (ties: lower index) in
 * ascending order, then the W window rows.  kc_out, vc_out: [BH, Tcap_out, D], rows
 * 0 .. K_keep+W-1 written.  idx: [BH, K_keep]. */
void ref_snapkv_select_gather(int64_t BH, int64_t T, int64_t Tcap, int64_t D, int64_t W,
                              int64_t K_keep, const double *pooled, const float *k_cache,
                              const float *v_cache, int64_t Tcap_out, int32_t *idx,
                              float *kc_out, float *vc_out);

#ifdef __cplusplus
}
#endif
#endif
