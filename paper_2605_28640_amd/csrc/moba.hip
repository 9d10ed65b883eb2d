// MoBA routing at prefill (App. A.1, MoBA paragraph; Sec. 2.2, Eq. 3): mean-pooled block
// representatives, per-query gate scores against the blocks before the query's own, and
// the top-K blocks per query token (own block and the first n_first always kept).
#include "common.h"
#include "knobs.h"

namespace rs {

// ------------------------------------------------------------------------------------
// block means: one workgroup per (block, batch*KV head); float32 accumulation
// ------------------------------------------------------------------------------------
template <typename ST, int D>
__global__ __launch_bounds__(256) void moba_block_means_kernel(const ST *__restrict__ k_cache,
                                                               float *__restrict__ means, uint16_t *__restrict__ split,
                                                               long Tcap, long T, int block, int Nb)
{
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;
    using R = Row8<ST>;
    __shared__ float s_acc[4][D];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rg = lane / LPR, c0 = (lane % LPR) * 8;
    const int j = blockIdx.x;
    const long bh = blockIdx.y;
    // The split terms are laid out as the gate's matrix operands: for block group g = j / 32,
    // term and 16-channel chunk c, the 64 lanes' 16-byte fragments follow each other (lane =
    // 32 * (channel half) + j % 32), so that a wave loads an operand as 1 KB of contiguous memory.
    const long Ng = (Nb + 31) / 32;
    auto split_at = [&](int term, int d) {
        return split + ((((bh * Ng + j / 32) * 3 + term) * (D / 16) + d / 16) * 64 + 32 * ((d % 16) / 8) + j % 32) * 8 + d % 8;
    };
    if (j >= Nb) {  // padding rows of the last group: zeros
        if (split && tid < D) *split_at(0, tid) = *split_at(1, tid) = *split_at(2, tid) = 0;
        return;
    }
    const long t0 = (long)j * block;
    const long t1 = (t0 + block < T) ? t0 + block : T;

    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.f;
    for (long t = t0 + wave * RPW + rg; t < t1; t += 4 * RPW) {
        float x[8];
        R::load(k_cache + (bh * Tcap + t) * D + c0, x);
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] += x[c];
    }
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) {
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] += shfl_xor_f(acc[c], m);
    }
    if (rg == 0) {
#pragma unroll
        for (int c = 0; c < 8; ++c) s_acc[wave][c0 + c] = acc[c];
    }
    __syncthreads();
    if (tid < D) {
        const float s = (s_acc[0][tid] + s_acc[1][tid]) + (s_acc[2][tid] + s_acc[3][tid]);
        const float m = s / (float)(t1 - t0);
        means[(bh * Nb + j) * D + tid] = m;
        if (split) {
            // the mean as three bfloat16 terms, m = m1 + m2 + m3 up to 2^-24 |m| (both remainders
            // are exact in float32): the operands of the matrix-core gate
            const __bf16 m1 = (__bf16)m;
            const float r1 = m - (float)m1;
            const __bf16 m2 = (__bf16)r1;
            const float r2 = r1 - (float)m2;
            const __bf16 m3 = (__bf16)r2;
            *split_at(0, tid) = __builtin_bit_cast(uint16_t, m1);
            *split_at(1, tid) = __builtin_bit_cast(uint16_t, m2);
            *split_at(2, tid) = __builtin_bit_cast(uint16_t, m3);
        }
    }
}

// ------------------------------------------------------------------------------------
// gate scores + top-K: one thread per query token, its q row in registers; the block mean
// is the same for the whole wave, so it is read through scalar loads and each score costs
// D fused multiply-adds and no LDS traffic.  Scores go to a per-thread LDS column; the K
// picks are K sweeps over that column (strictly-greater keeps the lowest index on ties).
// ------------------------------------------------------------------------------------
constexpr uint32_t kPickedBits = 0xffc00001u;  // NaN marker: compares false, so never picked twice

template <typename ST, int D>
__global__ __launch_bounds__(64) void moba_gate_topk_kernel(const ST *__restrict__ q,
                                                            const float *__restrict__ means,
                                                            int32_t *__restrict__ idx_out, int Hq, int Hkv, long T,
                                                            int block, int Nb, int K, int n_first)
{
    extern __shared__ float s_score[];  // [Nb][64]
    using R = Row8<ST>;
    const int lane = threadIdx.x;
    const int unit = blockIdx.y;  // b * Hq + h
    const int b = unit / Hq, h = unit % Hq, kvh = h / (Hq / Hkv);
    const long t_tile = (long)blockIdx.x * 64;
    const long t = t_tile + lane;
    const long tq = (t < T) ? t : T - 1;  // clamped row for the tail lanes (their result is dropped)
    const int own = (int)(tq / block);
    const long t_last = (t_tile + 63 < T) ? t_tile + 63 : T - 1;
    const int own_max = (int)(t_last / block);  // uniform over the wave

    float qv[D];
#pragma unroll
    for (int c = 0; c < D; c += 8) {
        float x[8];
        R::load(q + ((long)unit * T + tq) * D + c, x);
#pragma unroll
        for (int i = 0; i < 8; ++i) qv[c + i] = x[i];
    }
    const float *mbase = means + (long)(b * Hkv + kvh) * Nb * D;
    for (int j = 0; j <= own_max; ++j) {
        const float *m = mbase + (long)j * D;  // uniform address: scalar loads
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) s = fmaf(qv[c], m[c], s);
        if (j == own || j < n_first) s = INFINITY;  // always kept
        s_score[j * 64 + lane] = s;
    }
    // candidates of this row: blocks 0 .. own (entries past own are never read)
    const int avail = own + 1;
    const int take = (K < avail) ? K : avail;
    for (int r = 0; r < take; ++r) {
        float best = -INFINITY;
        int arg = -1;
        for (int j = 0; j <= own; ++j) {
            const float v = s_score[j * 64 + lane];
            if (__float_as_uint(v) == kPickedBits) continue;
            if (arg < 0 || v > best) {
                best = v;
                arg = j;
            }
        }
        if (arg >= 0) s_score[arg * 64 + lane] = __uint_as_float(kPickedBits);
    }
    if (t < T) {
        int32_t *dst = idx_out + ((long)unit * T + t) * K;
        int n = 0;
        for (int j = 0; j <= own; ++j)
            if (__float_as_uint(s_score[j * 64 + lane]) == kPickedBits) dst[n++] = j;
        for (; n < K; ++n) dst[n] = -1;
    }
}

// ------------------------------------------------------------------------------------
// bfloat16 queries: the gate scores of 64 query tokens against 32 blocks at a time on the
// matrix cores, S^T = M Q^T with v_mfma_f32_32x32x16_bf16.  The float32 block means come
// split into three bfloat16 terms (m = m1 + m2 + m3 up to 2^-24 |m|, written by the means
// kernel) and the three products accumulate in float32, so the scores keep float32 accuracy
// (the top-K needs it: a block mean rounded to bfloat16 would move scores by 2^-9).  A lane
// of the accumulator holds 16 blocks of ONE query.
// Picks, K <= 16: each half-lane keeps a sorted list of the KL = 4, 8 or 16 largest of its
// values (a v_max and KL - 1 v_med3 per value), the two halves of a query merge their lists,
// the take-th largest is the threshold, and the picked set is the bit mask of scores >=
// threshold; if that mask does not hold exactly `take` blocks (an exact tie at the threshold)
// the blocks above the threshold are taken and the tied ones fill up in index order.  With at
// most 64 candidate blocks the scores themselves stay in registers and no LDS is used; with
// more they go to a per-thread LDS column and are read back once against the threshold.
// K > 16: the scores go to the LDS column as in the scalar kernel and the picks are K sweeps.
// ------------------------------------------------------------------------------------
typedef __bf16 gate_bf16x8 __attribute__((ext_vector_type(8)));
typedef float gate_f32x16 __attribute__((ext_vector_type(16)));

// KL > 0 (K <= KL, KL in {4, 8, 16}): the K-th largest score of a query comes from sorted top
// lists kept in registers while the scores are formed; with at most 64 blocks (WIDE = false)
// the scores stay in registers too, with more (WIDE) they go to LDS columns and are read back
// once against the threshold.  KL = 0: picks by K sweeps over the LDS columns (K up to 32).
// NWV > 1 (register picks only): the waves of a workgroup share the unit's block-mean operands
// through LDS (at most 64 blocks: 48 KB at D = 128), fetched once per workgroup instead of once per
// 64-token tile from L2 -- with operands two chunks ahead, a wave otherwise waits an L2 round
// trip every other chunk.
template <int D, int KL, bool WIDE, int NWV>
__global__ __launch_bounds__(64 * NWV) __attribute__((amdgpu_waves_per_eu(NWV == 1 ? 2 : 1, 2))) void moba_gate_mfma_kernel(const bf16 *__restrict__ q, const uint16_t *__restrict__ split,
                                                           int32_t *__restrict__ idx_out, int Hq, int Hkv, long T,
                                                           int block, int Nb, int K, int n_first)
{
    constexpr int NC = D / 16;
    constexpr int CR = D / 8;    // 16-byte chunks per query row
    constexpr int RW = 64 / CR;  // rows one wave-wide direct load covers
    constexpr int NP = 64 / RW;  // direct loads per 64-row tile
    // A workgroup is one wave; it walks over tiles of 64 query tokens of one (batch, head).  The
    // tile's query rows come through LDS: row-contiguous direct loads (a lane fetching its own
    // row in 16-byte pieces would touch 64 cache lines per instruction), issued one tile ahead --
    // once the current tile's operands sit in registers and its matrix work is done -- so that
    // they land under the picks of the current tile.
    static_assert(NWV == 1 || (KL > 0 && !WIDE), "shared operands: register picks only");
    __shared__ __attribute__((aligned(1024))) uint16_t sQ_all[NWV * 64 * D];
    __shared__ __attribute__((aligned(1024))) uint16_t sM[NWV == 1 ? 8 : 2 * 3 * 32 * D];  // [group][term][chunk][lane][8]
    extern __shared__ float s_score[];  // [Nb rounded up to 32][64], only for the LDS picks
    const int lane = threadIdx.x & 63, lq = lane & 31, h = lane >> 5;
    const int wave = (NWV == 1) ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint16_t *sQ = sQ_all + wave * 64 * D;
    const int unit = blockIdx.y;  // b * Hq + h
    const int b = unit / Hq, hq = unit % Hq, kvh = hq / (Hq / Hkv);
    const long n_tiles = (T + 63) / 64;
    const long tile0 = (long)blockIdx.x * NWV + wave, tile_step = (long)gridDim.x * NWV;
    if constexpr (NWV > 1) {
        // the unit's operands into LDS: 1 KB per direct load, the waves take turns
        const LdsSource msrc = lds_source(split + (long)(b * Hkv + kvh) * ((Nb + 31) / 32) * 3 * 32 * D);
        const int n_kb = ((Nb + 31) / 32) * 3 * 32 * D * 2 / 1024;
        for (int i = wave; i < n_kb; i += NWV) load16_to_lds(msrc, (uint32_t)(i * 1024 + lane * 16), sM + i * 512);
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        __syncthreads();
    }
    if (tile0 >= n_tiles) return;

    const int srow = lane / CR;
    auto stage_q = [&](long t_tile) __attribute__((always_inline)) {
        const LdsSource src = lds_source(q + ((long)unit * T + t_tile) * D);
        const int last = (int)((T - 1 - t_tile < 63) ? T - 1 - t_tile : 63);  // rows past the end repeat the last one
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int row = i * RW + srow;
            const int r = (row < last) ? row : last;
            load16_to_lds(src, (uint32_t)(r * D + (((lane % CR) ^ chunk_swizzle<D>(row)) * 8)) * 2u, sQ + i * RW * D);
        }
    };
    stage_q(tile0 * 64);

    const uint16_t *sbase = split + (long)(b * Hkv + kvh) * ((Nb + 31) / 32) * 3 * 32 * D;  // wave-uniform
    const LdsSource means_src = lds_source(sbase);  // operand loads: descriptor + scalar offset + 16 bytes per lane
    // scores of blocks j0 .. j0 + 31 against this wave's 64 queries
    auto scores = [&](int j0, const gate_bf16x8 (&qf)[2][NC], gate_f32x16 (&acc)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[qt][v] = 0.f;
        const int frag = (j0 / 32) * 3 * 32 * D * 2;  // byte offset of the group's [term][chunk][lane][8]: 1 KB per operand
        // operands are fetched two chunks ahead of the matrix instructions that use them
        gate_bf16x8 m[3][3];
        auto fetch = [&](int c) __attribute__((always_inline)) {
#pragma unroll
            for (int term = 0; term < 3; ++term) {
                if constexpr (NWV > 1)
                    m[c % 3][term] = *reinterpret_cast<const gate_bf16x8 *>(sM + (frag + (term * NC + c) * 1024) / 2 + lane * 8);
                else
                    m[c % 3][term] = __builtin_bit_cast(gate_bf16x8, __builtin_amdgcn_raw_buffer_load_b128(means_src, lane * 16, frag + (term * NC + c) * 1024, 0));
            }
        };
        fetch(0);
        fetch(1);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (c + 2 < NC) fetch(c + 2);
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                acc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(m[c % 3][2], qf[qt][c], acc[qt], 0, 0, 0);
                acc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(m[c % 3][1], qf[qt][c], acc[qt], 0, 0, 0);
                acc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(m[c % 3][0], qf[qt][c], acc[qt], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the fetch distance: no sinking of the loads to their uses
        }
    };
    for (long tile = tile0; tile < n_tiles; tile += tile_step) {
    const long t_tile = tile * 64;
    const long t_last = (t_tile + 63 < T) ? t_tile + 63 : T - 1;
    const int own_max = (int)(t_last / block);  // uniform over the wave
    const bool more = tile + tile_step < n_tiles;
    // B operands: this lane's two query rows (tokens t_tile + lq and t_tile + 32 + lq, clamped)
    gate_bf16x8 qf[2][NC];
    int own_q[2];
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the tile's rows are in LDS
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const long t = t_tile + 32 * qt + lq;
        const long tc = (t < T) ? t : T - 1;
        own_q[qt] = (int)(tc / block);
        const int row = 32 * qt + lq;
        const int sw = chunk_swizzle<D>(row);
#pragma unroll
        for (int c = 0; c < NC; ++c) qf[qt][c] = *reinterpret_cast<const gate_bf16x8 *>(&sQ[row * D + (((2 * c + h) ^ sw) * 8)]);
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the operands are in registers, the LDS tile is free again
    // accumulator value v of lane (lq, h): block j0 + 8 (v / 4) + 4 h + v % 4, query lq
    if constexpr (KL > 0 && !WIDE) {
        float sc[2][2][16];  // [block group][query tile][value]; -inf: not a candidate
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            if (32 * g <= own_max) {
                gate_f32x16 acc[2];
                scores(32 * g, qf, acc);
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int j = 32 * g + 8 * (v / 4) + 4 * h + (v % 4);
                        float x = acc[qt][v];
                        if (j == own_q[qt] || j < n_first) x = INFINITY;  // always kept
                        sc[g][qt][v] = (j <= own_q[qt]) ? x : -INFINITY;
                    }
            } else {
#pragma unroll
                for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sc[g][qt][v] = -INFINITY;
            }
        }
        if (more) stage_q((tile + tile_step) * 64);  // lands under the picks
        // half h writes the picks of query tile h (token t_tile + 32 h + lq) as a 64-bit mask of blocks
        uint64_t picks = 0;
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            // the KL largest of this half-lane's values, then of both halves: a descending list,
            // a new value x enters by top[i] <- median(top[i-1], top[i], x) (old values), top[0] <- max
            float top[KL];
#pragma unroll
            for (int i = 0; i < KL; ++i) top[i] = -INFINITY;
            auto put = [&](float x) __attribute__((always_inline)) {
                float prev = top[0];
                top[0] = fmaxf(prev, x);
#pragma unroll
                for (int i = 1; i < KL; ++i) {
                    const float cur = top[i];
                    top[i] = __builtin_amdgcn_fmed3f(prev, cur, x);
                    prev = cur;
                }
            };
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int v = 0; v < 16; ++v) put(sc[g][qt][v]);
            float other[KL];
#pragma unroll
            for (int i = 0; i < KL; ++i) other[i] = shfl_xor_f(top[i], 32);
#pragma unroll
            for (int i = 0; i < KL; ++i) put(other[i]);
            const int avail = own_q[qt] + 1;
            const int take = (K < avail) ? K : avail;
            float thr = top[0];
#pragma unroll
            for (int i = 1; i < KL; ++i) thr = (take > i) ? top[i] : thr;  // top[take - 1]
            // blocks of this query (both halves) whose score passes `test` against the threshold
            auto blocks_where = [&](auto test) __attribute__((always_inline)) {
                uint32_t w[2];
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    uint32_t m = 0u;
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (test(sc[g][qt][v], thr)) m |= 1u << (8 * (v / 4) + (v % 4));
                    m <<= 4 * h;
                    w[g] = m | (uint32_t)__shfl_xor((int)m, 32, 64);
                }
                return ((uint64_t)w[1] << 32) | w[0];
            };
            uint64_t sel = blocks_where([](float x, float t) { return x >= t; });
            if (__any(__popcll(sel) != take)) {
                // an exact tie at the threshold: everything above it, then the tied blocks in index order
                const uint64_t above = blocks_where([](float x, float t) { return x > t; });
                uint64_t tied = sel & ~above;
                sel = above;
                for (int r = take - __popcll(above); r > 0; --r) {
                    sel |= tied & (0 - tied);
                    tied &= tied - 1;
                }
            }
            if (qt == h) picks = sel;
        }
        const long t = t_tile + 32 * h + lq;
        if (t < T) {
            int32_t *dst = idx_out + ((long)unit * T + t) * K;
            for (int n = 0; n < K; ++n) {
                dst[n] = picks ? (int32_t)__builtin_ctzll(picks) : -1;
                picks &= picks - 1;
            }
        }
        continue;
    } else if constexpr (KL > 0) {
        // more than 64 blocks: sorted top lists per query tile while the scores go to LDS columns
        float top[2][KL];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int i = 0; i < KL; ++i) top[qt][i] = -INFINITY;
        auto put = [&](float (&tl)[KL], float x) __attribute__((always_inline)) {
            float prev = tl[0];
            tl[0] = fmaxf(prev, x);
#pragma unroll
            for (int i = 1; i < KL; ++i) {
                const float cur = tl[i];
                tl[i] = __builtin_amdgcn_fmed3f(prev, cur, x);
                prev = cur;
            }
        };
        for (int j0 = 0; j0 <= own_max; j0 += 32) {
            gate_f32x16 acc[2];
            scores(j0, qf, acc);
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int j = j0 + 8 * (v / 4) + 4 * h + (v % 4);
                    float x = acc[qt][v];
                    if (j == own_q[qt] || j < n_first) x = INFINITY;  // always kept
                    s_score[j * 64 + 32 * qt + lq] = x;
                    put(top[qt], (j <= own_q[qt]) ? x : -INFINITY);
                }
        }
        if (more) stage_q((tile + tile_step) * 64);  // lands under the picks
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            float other[KL];
#pragma unroll
            for (int i = 0; i < KL; ++i) other[i] = shfl_xor_f(top[qt][i], 32);
#pragma unroll
            for (int i = 0; i < KL; ++i) put(top[qt], other[i]);
        }
        // from here thread = query token t_tile + lane = query tile h, row lq
        const long t = t_tile + lane;
        const int own = h ? own_q[1] : own_q[0];
        const int avail = own + 1;
        const int take = (K < avail) ? K : avail;
        float thr = h ? top[1][0] : top[0][0];
#pragma unroll
        for (int i = 1; i < KL; ++i) thr = (take > i) ? (h ? top[1][i] : top[0][i]) : thr;  // top[take - 1]
        __syncthreads();  // the score columns are complete
        uint64_t ge[4] = {0ull, 0ull, 0ull, 0ull}, gt[4] = {0ull, 0ull, 0ull, 0ull};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (64 * w > own_max) break;  // uniform
            for (int jj = 0; jj < 64 && 64 * w + jj <= own_max; jj += 4) {
                float v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = s_score[(64 * w + jj + i) * 64 + lane];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool cand = 64 * w + jj + i <= own;
                    if (cand && v[i] >= thr) ge[w] |= 1ull << (jj + i);
                    if (cand && v[i] > thr) gt[w] |= 1ull << (jj + i);
                }
            }
        }
        int n_ge = 0, n_gt = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            n_ge += __popcll(ge[w]);
            n_gt += __popcll(gt[w]);
        }
        if (n_ge != take) {
            // an exact tie at the threshold: everything above it, then the tied blocks in index order
            int r = take - n_gt;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint64_t tied = ge[w] & ~gt[w];
                ge[w] = gt[w];
                while (r > 0 && tied) {
                    ge[w] |= tied & (0 - tied);
                    tied &= tied - 1;
                    --r;
                }
            }
        }
        if (t < T) {
            int32_t *dst = idx_out + ((long)unit * T + t) * K;
            int n = 0;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                uint64_t word = ge[w];
                while (word && n < K) {
                    dst[n++] = 64 * w + (int32_t)__builtin_ctzll(word);
                    word &= word - 1;
                }
            }
            for (; n < K; ++n) dst[n] = -1;
        }
        __syncthreads();  // the score columns are rewritten by the next tile
        continue;
    } else {
        for (int j0 = 0; j0 <= own_max; j0 += 32) {
            gate_f32x16 acc[2];
            scores(j0, qf, acc);
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int j = j0 + 8 * (v / 4) + 4 * h + (v % 4);
                    float x = acc[qt][v];
                    if (j == own_q[qt] || j < n_first) x = INFINITY;  // always kept
                    s_score[j * 64 + 32 * qt + lq] = x;
                }
        }
    }
    if (more) stage_q((tile + tile_step) * 64);  // lands under the picks
    __syncthreads();
    // the picks: thread = query token, candidates 0 .. own.  The sweeps run to the wave-uniform
    // bound own_max in steps of four (rows up to the next multiple of 32 exist in LDS), so that
    // four LDS reads are in flight at a time; entries past the thread's own block are skipped.
    const long t = t_tile + lane;
    const long tq = (t < T) ? t : T - 1;
    const int own = (int)(tq / block);
    const int avail = own + 1;
    const int take = (K < avail) ? K : avail;
    for (int r = 0; r < take; ++r) {
        float best = -INFINITY;
        int arg = -1;
        for (int j = 0; j <= own_max; j += 4) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = s_score[(j + i) * 64 + lane];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool cand = (j + i <= own) && (__float_as_uint(v[i]) != kPickedBits);
                if (cand && (arg < 0 || v[i] > best)) {
                    best = v[i];
                    arg = j + i;
                }
            }
        }
        if (arg >= 0) s_score[arg * 64 + lane] = __uint_as_float(kPickedBits);
    }
    if (t < T) {
        int32_t *dst = idx_out + ((long)unit * T + t) * K;
        int n = 0;
        for (int j = 0; j <= own_max; j += 4) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = s_score[(j + i) * 64 + lane];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (j + i <= own && __float_as_uint(v[i]) == kPickedBits) dst[n++] = j + i;
        }
        for (; n < K; ++n) dst[n] = -1;
    }
    __syncthreads();  // the score columns are rewritten by the next tile
    }  // tiles
}

// workspace: the block means as three bfloat16 terms in matrix-operand order,
// [batch * KV heads][groups of 32 blocks][3][D / 16][64 lanes][8]
size_t moba_select_ws_bytes(const rs_shape *s, long T, int block)
{
    const size_t Ng = (size_t)(((T + block - 1) / block + 31) / 32);
    return RS_WS_CTRL_BYTES + (((size_t)s->B * s->Hkv * Ng * 32 * 3 * s->D * 2 + 255) & ~(size_t)255);
}

int moba_select_dispatch(const rs_shape *s, const void *q, const void *k_cache, long T, int block, int K,
                         int n_first, float *means_out, int32_t *idx_out, char *ws, hipStream_t stream)
{
    uint16_t *split = (uint16_t *)(ws + RS_WS_CTRL_BYTES);
    const int Nb = (int)((T + block - 1) / block);
    if (Nb > 256) return RS_UNSUPPORTED;  // one LDS score column per thread: Nb * 256 bytes
    const dim3 g1((unsigned)Nb, (unsigned)(s->B * s->Hkv));
    const dim3 g1p((unsigned)((Nb + 31) / 32 * 32), (unsigned)(s->B * s->Hkv));  // with the split's padding rows
    const dim3 g2((unsigned)((T + 63) / 64), (unsigned)(s->B * s->Hq));
    const size_t lds = (size_t)Nb * 64 * 4;
    const size_t lds_wave = (size_t)((Nb + 31) / 32 * 32) * 64 * 4;
    // the gate kernel: one-wave workgroups, about eight per CU, each walking over the 64-token
    // tiles of one (batch, head)
    const bool in_registers = K <= 16 && Nb <= 64;  // its register picks need no score columns
    const int kl = K <= 4 ? 4 : K <= 8 ? 8 : K <= 16 ? 16 : 0;
    const size_t lds_mfma = in_registers ? 0 : lds_wave;
    const long n_tiles = (T + 63) / 64, units = (long)s->B * s->Hq;
    long per_unit = (2048 + units - 1) / units;
    if (knobs().gate_waves != kKnobUnset) per_unit = ((long)knobs().gate_waves + units - 1) / units;
    if (per_unit < 1) per_unit = 1;
    const dim3 g3((unsigned)(n_tiles < per_unit ? n_tiles : per_unit), (unsigned)units);
    // six-wave workgroups with the operands in LDS (48 KB + 6 x 16 KB of query rows): one per CU
    long wg_per_unit = (256 + units - 1) / units;
    if (knobs().gate_wgs != kKnobUnset) wg_per_unit = ((long)knobs().gate_wgs + units - 1) / units;
    if (wg_per_unit < 1) wg_per_unit = 1;
    constexpr int nwv = 6;
    if (wg_per_unit > (n_tiles + nwv - 1) / nwv) wg_per_unit = (n_tiles + nwv - 1) / nwv;
    const dim3 g4((unsigned)wg_per_unit, (unsigned)units);
    const int eso = knobs().gate_shared;
    // worth its set-up from about 8192 tiles on (C4 0.148 -> 0.138 ms; 8 x 32 heads x 4096 tokens, blocks of 64,
    // top-8: 0.184 -> 0.150 ms; 32 heads x 4096 tokens: 0.026 against 0.031 ms the other way)
    const bool shared_ops = in_registers && (eso != kKnobUnset ? eso != 0 : units * n_tiles >= 8192);
#define RS_LAUNCH(ST, DD)                                                                                          \
    do {                                                                                                           \
        moba_block_means_kernel<ST, DD><<<g1, 256, 0, stream>>>((const ST *)k_cache, means_out, nullptr, s->Tcap, T, block, Nb); \
        moba_gate_topk_kernel<ST, DD><<<g2, 64, lds, stream>>>((const ST *)q, means_out, idx_out, s->Hq, s->Hkv, T,  \
                                                                block, Nb, K, n_first);                            \
    } while (0)
    if (s->dtype == RS_BF16) {
        if (s->D == 128) {
            moba_block_means_kernel<bf16, 128><<<g1p, 256, 0, stream>>>((const bf16 *)k_cache, means_out, split, s->Tcap, T, block, Nb);
#define RS_GATE1(DD, KLL, WW, LDS) moba_gate_mfma_kernel<DD, KLL, WW, 1><<<g3, 64, LDS, stream>>>((const bf16 *)q, split, idx_out, s->Hq, s->Hkv, T, block, Nb, K, n_first)
#define RS_GATE4(DD, KLL) moba_gate_mfma_kernel<DD, KLL, false, 6><<<g4, 384, 0, stream>>>((const bf16 *)q, split, idx_out, s->Hq, s->Hkv, T, block, Nb, K, n_first)
#define RS_GATE(DD)                                            \
    do {                                                       \
        if (kl == 0) RS_GATE1(DD, 0, true, lds_mfma);          \
        else if (!in_registers) {                              \
            if (kl == 4) RS_GATE1(DD, 4, true, lds_mfma);      \
            else if (kl == 8) RS_GATE1(DD, 8, true, lds_mfma); \
            else RS_GATE1(DD, 16, true, lds_mfma);             \
        } else if (shared_ops) {                               \
            if (kl == 4) RS_GATE4(DD, 4);                      \
            else if (kl == 8) RS_GATE4(DD, 8);                 \
            else RS_GATE4(DD, 16);                             \
        } else if (kl == 4) RS_GATE1(DD, 4, false, 0);         \
        else if (kl == 8) RS_GATE1(DD, 8, false, 0);           \
        else RS_GATE1(DD, 16, false, 0);                       \
    } while (0)
            RS_GATE(128);
        } else {
            moba_block_means_kernel<bf16, 64><<<g1p, 256, 0, stream>>>((const bf16 *)k_cache, means_out, split, s->Tcap, T, block, Nb);
            RS_GATE(64);
        }
#undef RS_GATE
#undef RS_GATE1
#undef RS_GATE4
    } else {
        if (s->D == 128) RS_LAUNCH(float, 128);
        else RS_LAUNCH(float, 64);
    }
#undef RS_LAUNCH
    return hipGetLastError() == hipSuccess ? RS_OK : RS_LAUNCH_FAILED;
}

}  // namespace rs
