// Quest at decode (App. A.1, Quest paragraph; Sec. 2.2, Eq. 3-4): page min/max
// representatives, page scores + top-K selection, and softmax attention over the
// selected pages (or over everything: the dense path).
//
// Lane mapping used throughout: a row of D channels is covered by LPR = D/8 lanes with
// 8 channels (one 16-byte bf16 load) each, so a wave touches RPW = 64/LPR rows per load
// instruction and every global access is a run of full 128/256-byte rows.
#include <cstdlib>
#include "common.h"
#include "knobs.h"
#include "select.h"

namespace rs {

// ------------------------------------------------------------------------------------
// page metadata: one wave per page
// ------------------------------------------------------------------------------------
template <typename ST, int D>
__global__ __launch_bounds__(256) void quest_page_meta_kernel(const ST *__restrict__ k_cache,
                                                              ST *__restrict__ meta, long Tcap, int P,
                                                              int p_begin, int n_pages, long t_end,
                                                              int segs_per_wave)
{
    // A wave owns a run of whole pages and walks it in segments of 16 rows (every page size is
    // a multiple of 16), four segments' loads in flight at a time; a page's bounds are folded
    // across the row groups and written when its last segment has been taken in.
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;
    constexpr int U = 16 / RPW;  // row loads of a lane per segment
    constexpr int J = 4;         // segments in flight
    using R = Row8<ST>;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rg = lane / LPR;
    const int c0 = (lane % LPR) * 8;
    const long bh = blockIdx.y;
    const long Np_cap = Tcap / P;
    const int spp = P / 16;  // segments per page
    const long seg_end = (long)n_pages * spp;
    const long seg0 = ((long)blockIdx.x * 4 + wave) * segs_per_wave;
    if (seg0 >= seg_end) return;
    const long seg1 = (seg0 + segs_per_wave < seg_end) ? seg0 + segs_per_wave : seg_end;
    const long t_base = (long)p_begin * P;
    const ST *kb = k_cache + bh * Tcap * D + c0;

    float lo[8], hi[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        lo[c] = INFINITY;
        hi[c] = -INFINITY;
    }
    for (long sg = seg0; sg < seg1; sg += J) {
        typename R::raw_t x[J][U];
#pragma unroll
        for (int j = 0; j < J; ++j)
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long t = t_base + (sg + j) * 16 + u * RPW + rg;
                x[j][u] = (sg + j < seg1 && t < t_end) ? R::load_raw(kb + t * D) : R::zero_raw();
            }
#pragma unroll
        for (int j = 0; j < J; ++j) {
            if (sg + j >= seg1) break;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const long t = t_base + (sg + j) * 16 + u * RPW + rg;
                if (t < t_end) {
                    float v[8];
                    R::unpack(x[j][u], v);
#pragma unroll
                    for (int c = 0; c < 8; ++c) {
                        lo[c] = fminf(lo[c], v[c]);
                        hi[c] = fmaxf(hi[c], v[c]);
                    }
                }
            }
            if ((sg + j + 1) % spp == 0) {  // the page is complete
#pragma unroll
                for (int m = LPR; m < 64; m <<= 1) {
#pragma unroll
                    for (int c = 0; c < 8; ++c) {
                        lo[c] = fminf(lo[c], shfl_xor_f(lo[c], m));
                        hi[c] = fmaxf(hi[c], shfl_xor_f(hi[c], m));
                    }
                }
                const long p = p_begin + (sg + j) / spp;
                ST *mrow = meta + ((bh * Np_cap + p) * 2) * D + c0;
                if (rg == 0) R::store(mrow, lo);
                if (rg == 1) R::store(mrow + D, hi);
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    lo[c] = INFINITY;
                    hi[c] = -INFINITY;
                }
            }
        }
    }
}

void page_meta_dispatch(int dtype, int D, const void *k_cache, void *meta, int BH, long Tcap, int P,
                        int p_begin, int n_pages, long t_end, hipStream_t stream)
{
    // whole pages per wave, four segments (16 KiB of bf16 rows at D = 128, every load in flight at
    // once) when the page size allows: measured on 2.4 GB of keys with 16-token pages, 1 / 2 / 4 /
    // 8 / 16 segments per wave give 4.0 / 5.1 / 5.4 / 5.3 / 5.0 TB/s
    const int spp = P / 16;
    const long segs = (long)n_pages * spp;
    int spw = 4;
    if (knobs().meta_spw != kKnobUnset && knobs().meta_spw > 0) spw = knobs().meta_spw;
    while (spw > 1 && (segs * BH) / spw < 8192) spw >>= 1;
    if (spw < spp) spw = spp;
    spw = (spw / spp) * spp;
    const long waves = (segs + spw - 1) / spw;
    const dim3 grid((unsigned)((waves + 3) / 4), (unsigned)BH);
    if (dtype == RS_BF16) {
        if (D == 128) quest_page_meta_kernel<bf16, 128><<<grid, 256, 0, stream>>>((const bf16 *)k_cache, (bf16 *)meta, Tcap, P, p_begin, n_pages, t_end, spw);
        else quest_page_meta_kernel<bf16, 64><<<grid, 256, 0, stream>>>((const bf16 *)k_cache, (bf16 *)meta, Tcap, P, p_begin, n_pages, t_end, spw);
    } else {
        if (D == 128) quest_page_meta_kernel<float, 128><<<grid, 256, 0, stream>>>((const float *)k_cache, (float *)meta, Tcap, P, p_begin, n_pages, t_end, spw);
        else quest_page_meta_kernel<float, 64><<<grid, 256, 0, stream>>>((const float *)k_cache, (float *)meta, Tcap, P, p_begin, n_pages, t_end, spw);
    }
}

constexpr int kSelThreads = 512;

// ------------------------------------------------------------------------------------
// page scores; the last workgroup of a unit to arrive runs the selection.  GQ = 1: a unit
// is a (batch, query head).  GQ = Hq / Hkv > 1 (group-shared selection, an option for
// grouped-query attention that is not in the paper): a unit is a (batch, KV head), the
// page score is the sum of the bounds of its GQ query heads and the list is theirs in common.
// ------------------------------------------------------------------------------------
template <typename ST, int D, int GQ>
__global__ __launch_bounds__(kSelThreads) void quest_score_select_kernel(
    const ST *__restrict__ q, const ST *__restrict__ meta, uint64_t *scores, float *scores_out, int32_t *idx_out,
    int Hq, int Hkv, long Np_cap, int Np, int K, int n_first, int n_local, int splits, uint32_t *unit_ctr,
    uint32_t *err, uint32_t tag, int spin_limit, const uint32_t *state, long T_max, int P)
{
    // state (the replayable decode step): the sequence length and the tag are not arguments but words of
    // the workspace (tokens in the cache + 1: the step's append has run); score rows keep the stride of T_max
    long np_stride = Np;
    if (state) {
        const long T_valid = *reinterpret_cast<const long *>(state + kCtrlStateT) + 1;
        tag = state[kCtrlStateTag];
        if (tag == 0u) tag = 0x5bd1e995u;
        Np = (int)((T_valid + P - 1) / P);
        np_stride = (T_max + P - 1) / P;
        if (T_valid > T_max || K > Np) {  // outside what the buffers were sized for: report, do nothing
            if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) atomicExch(err, 1u);
            return;
        }
    }
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;
    constexpr int UNR = 4;  // pages per lane in flight
    using R = Row8<ST>;
    __shared__ SelectShared<kSelThreads> sh;
    __shared__ int s_last;
    extern __shared__ uint32_t s_keys[];  // Np keys

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int rg = lane / LPR;
    const int c0 = (lane % LPR) * 8;
    const int unit = blockIdx.y;  // b * Hq + h (GQ = 1) or b * Hkv + kvh
    const int u0 = unit * GQ;     // first (batch, query head) of the unit
    const int b = u0 / Hq, h = u0 % Hq;
    const int kvh = h / (Hq / Hkv);
    const ST *mbase = meta + ((long)(b * Hkv + kvh) * Np_cap) * 2 * D;
    uint64_t *srow = scores + (long)unit * np_stride;

    float qv[GQ][8];
#pragma unroll
    for (int g = 0; g < GQ; ++g) R::load(q + (long)(u0 + g) * D + c0, qv[g]);
    BoundDot<ST> bound[GQ];
#pragma unroll
    for (int g = 0; g < GQ; ++g) bound[g].set(qv[g]);

    // this workgroup's pages: a contiguous slice, walked UNR * RPW pages per wave step.
    // The LPR lanes of a row group share their page numbers, so the group-local
    // shuffles only ever read active lanes.
    const int per = (Np + splits - 1) / splits;
    const int pb = blockIdx.x * per;
    const int pe = (pb + per < Np) ? pb + per : Np;
    constexpr int PPI = UNR * RPW * (kSelThreads / 64);  // pages per workgroup iteration
    for (int base = pb + wave * (UNR * RPW) + rg; base < pe; base += PPI) {
        typename R::raw_t mn[UNR], mx[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int p = base + u * RPW;
            if (p < pe) {
                mn[u] = R::load_raw(mbase + ((long)p * 2) * D + c0);
                mx[u] = R::load_raw(mbase + ((long)p * 2 + 1) * D + c0);
            } else {
                mn[u] = R::zero_raw();
                mx[u] = R::zero_raw();
            }
        }
        // lane u of a row group keeps page u's sum; the wave's UNR * RPW scores (adjacent words) then
        // leave with one store instruction
        float mine = 0.f;
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            float s = 0.f;
#pragma unroll
            for (int g = 0; g < GQ; ++g) s = bound[g].add(s, mn[u], mx[u]);
            s = group_sum<LPR>(s);
            if ((lane % LPR) == u) mine = s;
        }
        {
            const int p = base + (lane % LPR) * RPW;
            if ((lane % LPR) < UNR && p < pe) publish_f32(&srow[p], mine, tag);
        }
    }

    if (tid == 0) {
        const uint32_t prev = atomicAdd(&unit_ctr[unit], 1u);
        s_last = (prev == (uint32_t)splits - 1u);
        if (s_last) atomicExch(&unit_ctr[unit], 0u);  // every split has arrived: reset for the next call
    }
    __syncthreads();
    if (!s_last) return;

    gather_page_keys<kSelThreads>(srow, Np, n_first, n_local, tag, spin_limit, err,
                                  scores_out ? scores_out + (long)unit * Np : nullptr, s_keys);
    int32_t *dst = idx_out + (long)unit * K;
    select_topk_lds<kSelThreads>(s_keys, Np, K, sh, [dst](int pos, int p) { dst[pos] = p; });
}

// GQ: query heads per unit: 1, or Hq / Hkv (2, 4 or 8) for group-shared selection
int score_select_dispatch(int dtype, int D, int GQ, const void *q, const void *meta, uint64_t *scores,
                          float *scores_out, int32_t *idx_out, int B, int Hq, int Hkv, long Np_cap, int Np, int K,
                          int n_first, int n_local, int splits, uint32_t *unit_ctr, uint32_t *err, uint32_t tag,
                          int spin_limit, const uint32_t *state, long T_max, int P, hipStream_t stream)
{
    const dim3 grid((unsigned)splits, (unsigned)(B * Hq / GQ));
    if (Np > 15360) return RS_UNSUPPORTED;  // keys must fit 60 KiB of LDS
    if (GQ != 1 && GQ != 2 && GQ != 4 && GQ != 8) return RS_UNSUPPORTED;
    const size_t lds = (size_t)Np * 4;
#define RS_LAUNCH(ST, DD, GG)                                                                                      \
    quest_score_select_kernel<ST, DD, GG><<<grid, kSelThreads, lds, stream>>>(                                    \
        (const ST *)q, (const ST *)meta, scores, scores_out, idx_out, Hq, Hkv, Np_cap, Np, K, n_first, n_local, \
        splits, unit_ctr, err, tag, spin_limit, state, T_max, P)
#define RS_LAUNCH_G(ST, DD)                     \
    do {                                        \
        if (GQ == 8) RS_LAUNCH(ST, DD, 8);      \
        else if (GQ == 4) RS_LAUNCH(ST, DD, 4); \
        else if (GQ == 2) RS_LAUNCH(ST, DD, 2); \
        else RS_LAUNCH(ST, DD, 1);              \
    } while (0)
    if (dtype == RS_BF16) {
        if (D == 128) RS_LAUNCH_G(bf16, 128);
        else RS_LAUNCH_G(bf16, 64);
    } else {
        if (D == 128) RS_LAUNCH_G(float, 128);
        else RS_LAUNCH_G(float, 64);
    }
#undef RS_LAUNCH_G
#undef RS_LAUNCH
    return RS_OK;
}

// ------------------------------------------------------------------------------------
// decode attention over a list of 16-row tiles (selected pages, or all rows), split over
// workgroups; partial (m, l, o) per split; the last split to arrive merges them.
// ------------------------------------------------------------------------------------
template <typename ST, int D, int kAttThreads>
__global__ __launch_bounds__(kAttThreads) void decode_attend_kernel(
    const ST *__restrict__ q, const ST *__restrict__ k_cache, const ST *__restrict__ v_cache, const int32_t *idx,
    ST *__restrict__ out, float *__restrict__ lse_out, uint64_t *partial, int Hq, int Hkv, long Tcap, int P,
    long T_valid, int K, float scale, int splits, uint32_t *unit_ctr, uint32_t *err, uint32_t tag, int spin_limit,
    int idx_per_kv, uint32_t *state, long T_max)
{
    // state (the replayable decode step, listed pages): length and tag come from the workspace's words; the
    // last workgroup out of the grid advances them (every workgroup has read them by then)
    if (state) {
        T_valid = *reinterpret_cast<const long *>(state + kCtrlStateT) + 1;
        tag = state[kCtrlStateTag];
        if (tag == 0u) tag = 0x5bd1e995u;
        if (T_valid > T_max || (long)K > (T_valid + P - 1) / P) return;  // refused: the selection kernel has reported it
    }
    auto workgroup_done = [&]() {
        if (state && threadIdx.x == 0) {
            uint32_t *done = state + kCtrlDone;
            if (atomicAdd(done, 1u) == gridDim.x * gridDim.y - 1u) {
                atomicExch(done, 0u);
                *reinterpret_cast<long *>(state + kCtrlStateT) = T_valid;
                const uint32_t nt = tag + 0x85EBCA6Bu;
                state[kCtrlStateTag] = nt ? nt : 0x5bd1e995u;
            }
        }
    };
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;  // rows per load instruction
    constexpr int TR = 16;         // rows per tile
    constexpr int RPL = TR / RPW;  // rows per lane per tile (4 for D=128, 2 for D=64)
    constexpr int TPI = 2;         // tiles in flight per wave
    constexpr int kAttWaves = kAttThreads / 64;
    using R = Row8<ST>;
    __shared__ float s_m[kAttWaves], s_l[kAttWaves];
    __shared__ float s_o[kAttWaves][D];
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int rg = lane / LPR;
    const int c0 = (lane % LPR) * 8;
    const int unit = blockIdx.y;
    const int b = unit / Hq, h = unit % Hq;
    const int kvh = h / (Hq / Hkv);
    const ST *kb = k_cache + (long)(b * Hkv + kvh) * Tcap * D;
    const ST *vb = v_cache + (long)(b * Hkv + kvh) * Tcap * D;
    // a page list belongs to the query head, or (group-shared selection) to its KV head
    const int32_t *idx_row = idx ? idx + (long)(idx_per_kv ? b * Hkv + kvh : unit) * K : nullptr;

    RowDot<ST> qd;
    {
        float qv[8];
        R::load(q + (long)unit * D + c0, qv);
        qd.set(qv);
    }

    const int tiles_per_page = P / TR;
    const long n_tiles = idx ? (long)K * tiles_per_page : (T_valid + TR - 1) / TR;
    const long per = (n_tiles + splits - 1) / splits;
    const long tb = (long)blockIdx.x * per;
    const long te = (tb + per < n_tiles) ? tb + per : n_tiles;

    float m = -INFINITY, l = 0.f;
    float o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = 0.f;

    for (long t = tb + wave * TPI; t < te; t += kAttWaves * TPI) {
        long row0[TPI];
        typename R::raw_t kr[TPI][RPL], vr[TPI][RPL];
#pragma unroll
        for (int u = 0; u < TPI; ++u) {
            const long tt = t + u;
            row0[u] = T_valid;  // nothing to do
            if (tt < te) {
                if (idx) {
                    const int page = idx_row[tt / tiles_per_page];
                    if (page >= 0) row0[u] = (long)page * P + (tt % tiles_per_page) * TR;
                } else {
                    row0[u] = tt * TR;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < TPI; ++u) {
#pragma unroll
            for (int i = 0; i < RPL; ++i) {
                const long row = row0[u] + i * RPW + rg;
                if (row < T_valid) {
                    if (Hq == Hkv) {  // no other query head reads these rows: streaming loads
                        kr[u][i] = R::load_raw_nt(kb + row * D + c0);
                        vr[u][i] = R::load_raw_nt(vb + row * D + c0);
                    } else {
                        kr[u][i] = R::load_raw(kb + row * D + c0);
                        vr[u][i] = R::load_raw(vb + row * D + c0);
                    }
                } else {  // masked rows contribute nothing (and stale memory is never read)
                    kr[u][i] = R::zero_raw();
                    vr[u][i] = R::zero_raw();
                }
            }
        }
#pragma unroll
        for (int u = 0; u < TPI; ++u) {
            float s[RPL];
            float mt = m;
#pragma unroll
            for (int i = 0; i < RPL; ++i) {
                const float d = group_sum<LPR>(qd.dot(kr[u][i])) * scale;
                const long row = row0[u] + i * RPW + rg;
                s[i] = (row < T_valid) ? d : -INFINITY;
                mt = fmaxf(mt, s[i]);
            }
            if (mt != -INFINITY) {  // uniform over the lanes of a row group
                const float corr = __expf(m - mt);
                l *= corr;
#pragma unroll
                for (int c = 0; c < 8; ++c) o[c] *= corr;
#pragma unroll
                for (int i = 0; i < RPL; ++i) {
                    const float p = __expf(s[i] - mt);
                    l += p;
                    float x[8];
                    R::unpack(vr[u][i], x);
#pragma unroll
                    for (int c = 0; c < 8; ++c) o[c] = fmaf(p, x[c], o[c]);
                }
                m = mt;
            }
        }
    }

    // merge the row groups of the wave
#pragma unroll
    for (int mask = LPR; mask < 64; mask <<= 1) {
        const float m2 = shfl_xor_f(m, mask);
        const float l2 = shfl_xor_f(l, mask);
        const float mn = fmaxf(m, m2);
        const float a1 = (m == -INFINITY) ? 0.f : __expf(m - mn);
        const float a2 = (m2 == -INFINITY) ? 0.f : __expf(m2 - mn);
        l = l * a1 + l2 * a2;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const float o2 = shfl_xor_f(o[c], mask);
            o[c] = o[c] * a1 + o2 * a2;
        }
        m = mn;
    }
    if (rg == 0) {
        if ((lane % LPR) == 0) {
            s_m[wave] = m;
            s_l[wave] = l;
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) s_o[wave][c0 + c] = o[c];
    }
    __syncthreads();

    // merge the waves; thread c owns channel c
    uint64_t *part = partial + ((long)unit * splits + blockIdx.x) * (D + 2);
    if (tid < D) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kAttWaves; ++w) M = fmaxf(M, s_m[w]);
        float L = 0.f, O = 0.f;
#pragma unroll
        for (int w = 0; w < kAttWaves; ++w) {
            const float a = (s_m[w] == -INFINITY) ? 0.f : __expf(s_m[w] - M);
            L += s_l[w] * a;
            O += s_o[w][tid] * a;
        }
        if (splits == 1) {
            const float inv = (L > 0.f) ? 1.f / L : 0.f;
            from_f32(out[(long)unit * D + tid], O * inv);
            if (tid == 0 && lse_out) lse_out[unit] = (L > 0.f) ? M + __logf(L) : -INFINITY;
        } else {
            publish_f32(&part[2 + tid], O, tag);
            if (tid == 0) {
                publish_f32(&part[0], M, tag);
                publish_f32(&part[1], L, tag);
            }
        }
    }
    if (splits == 1) {
        workgroup_done();
        return;
    }

    if (tid == 0) {
        const uint32_t prev = atomicAdd(&unit_ctr[unit], 1u);
        s_last = (prev == (uint32_t)splits - 1u);
        if (s_last) atomicExch(&unit_ctr[unit], 0u);
    }
    __syncthreads();
    if (!s_last) {
        workgroup_done();
        return;
    }
    if (tid < D) {
        float M = -INFINITY, L = 0.f, O = 0.f;
        merge_partials(partial + (long)unit * splits * (D + 2), splits, D + 2, tid, tag, spin_limit, err, M, L, O);
        const float inv = (L > 0.f) ? 1.f / L : 0.f;
        from_f32(out[(long)unit * D + tid], O * inv);
        if (tid == 0 && lse_out) lse_out[unit] = (L > 0.f) ? M + __logf(L) : -INFINITY;
    }
    workgroup_done();
}

// ------------------------------------------------------------------------------------
// Short contexts (the paper's 4096 tokens): select-then-attend of one (batch, query head)
// inside one 512-thread workgroup -- page scores into LDS keys, the top-K selection, then
// attention over the picked pages with the waves splitting the tiles -- so nothing is handed
// between workgroups and the step is one launch.  Same score arithmetic, forced pages and tie
// rule as quest_score_select_kernel; the attention loop is decode_attend_kernel's.
// Dynamic LDS: Np keys, then K picked pages.
// ------------------------------------------------------------------------------------
constexpr int kUnitThreads = 512;

// STATE (the replayable decode step): the sequence length is not an argument but the workspace's
// token count + 1 (the step's append has run); Np_lds = the page count the LDS was sized for;
// the last workgroup out advances the count and the tag word.
template <typename ST, int D, bool STATE>
__global__ __launch_bounds__(kUnitThreads) void quest_unit_decode_kernel(
    const ST *__restrict__ q, const ST *__restrict__ meta, const ST *__restrict__ k_cache,
    const ST *__restrict__ v_cache, ST *__restrict__ out, float *__restrict__ lse_out, int32_t *__restrict__ idx_out,
    int Hq, int Hkv, long Tcap, int P, long T_valid, int Np, int K, int n_first, int n_local, float scale,
    int Np_lds, uint32_t *state, long T_max)
{
    if constexpr (STATE) {
        T_valid = *reinterpret_cast<const long *>(state + kCtrlStateT) + 1;
        Np = (int)((T_valid + P - 1) / P);
        if (T_valid > T_max || K > Np) {  // outside what the buffers were sized for: report, do nothing
            if (blockIdx.x == 0 && threadIdx.x == 0) atomicExch(state + kCtrlAsyncErr, 1u);
            return;
        }
    }
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;
    constexpr int UNR = 4;
    constexpr int NW = kUnitThreads / 64;
    constexpr int TR = 16;
    constexpr int RPL = TR / RPW;
    constexpr int TPI = 2;
    using R = Row8<ST>;
    __shared__ SelectShared<kUnitThreads> sh;
    __shared__ float s_m[NW], s_l[NW];
    __shared__ float s_o[NW][D];
    extern __shared__ uint32_t s_dyn[];
    uint32_t *s_keys = s_dyn;
    int *s_sel = reinterpret_cast<int *>(s_dyn + Np_lds);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int rg = lane / LPR;
    const int c0 = (lane % LPR) * 8;
    const int unit = blockIdx.x;
    const int b = unit / Hq, h = unit % Hq;
    const int kvh = h / (Hq / Hkv);
    const long Np_cap = Tcap / P;
    const ST *mbase = meta + ((long)(b * Hkv + kvh) * Np_cap) * 2 * D;
    const ST *kb = k_cache + (long)(b * Hkv + kvh) * Tcap * D;
    const ST *vb = v_cache + (long)(b * Hkv + kvh) * Tcap * D;

    float qv[8];
    R::load(q + (long)unit * D + c0, qv);
    BoundDot<ST> bound;
    bound.set(qv);

    // page scores (Eq. 3 with the min/max bound) -> order-preserving keys
    constexpr int PPI = UNR * RPW * NW;
    for (int base = wave * (UNR * RPW) + rg; base < Np; base += PPI) {
        typename R::raw_t mn[UNR], mx[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int p = base + u * RPW;
            if (p < Np) {
                mn[u] = R::load_raw(mbase + ((long)p * 2) * D + c0);
                mx[u] = R::load_raw(mbase + ((long)p * 2 + 1) * D + c0);
            } else {
                mn[u] = R::zero_raw();
                mx[u] = R::zero_raw();
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int p = base + u * RPW;
            const float s = group_sum<LPR>(bound.add(0.f, mn[u], mx[u]));
            if (p < Np && (lane % LPR) == 0) s_keys[p] = (p < n_first || p >= Np - n_local) ? 0xffffffffu : float_to_key(s);
        }
    }
    __syncthreads();
    int32_t *dst = idx_out ? idx_out + (long)unit * K : nullptr;
    select_topk_lds<kUnitThreads>(s_keys, Np, K, sh, [s_sel, dst](int pos, int p) {
        s_sel[pos] = p;
        if (dst) dst[pos] = p;
    });
    __syncthreads();

    // attention over the picked pages (Eq. 4): 16-row tiles, the waves take them in turn
    RowDot<ST> qd;
    qd.set(qv);
    const int tiles_per_page = P / TR;
    const int n_tiles = K * tiles_per_page;
    float m = -INFINITY, l = 0.f;
    float o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = 0.f;
    for (int t = wave * TPI; t < n_tiles; t += NW * TPI) {
        long row0[TPI];
        typename R::raw_t kr[TPI][RPL], vr[TPI][RPL];
#pragma unroll
        for (int u = 0; u < TPI; ++u) {
            const int tt = t + u;
            row0[u] = T_valid;  // nothing to do
            if (tt < n_tiles) row0[u] = (long)s_sel[tt / tiles_per_page] * P + (tt % tiles_per_page) * TR;
        }
#pragma unroll
        for (int u = 0; u < TPI; ++u)
#pragma unroll
            for (int i = 0; i < RPL; ++i) {
                const long row = row0[u] + i * RPW + rg;
                if (row < T_valid) {
                    kr[u][i] = R::load_raw(kb + row * D + c0);
                    vr[u][i] = R::load_raw(vb + row * D + c0);
                } else {
                    kr[u][i] = R::zero_raw();
                    vr[u][i] = R::zero_raw();
                }
            }
#pragma unroll
        for (int u = 0; u < TPI; ++u) {
            float s[RPL];
            float mt = m;
#pragma unroll
            for (int i = 0; i < RPL; ++i) {
                const float d = group_sum<LPR>(qd.dot(kr[u][i])) * scale;
                const long row = row0[u] + i * RPW + rg;
                s[i] = (row < T_valid) ? d : -INFINITY;
                mt = fmaxf(mt, s[i]);
            }
            if (mt != -INFINITY) {
                const float corr = __expf(m - mt);
                l *= corr;
#pragma unroll
                for (int c = 0; c < 8; ++c) o[c] *= corr;
#pragma unroll
                for (int i = 0; i < RPL; ++i) {
                    const float pr = __expf(s[i] - mt);
                    l += pr;
                    float x[8];
                    R::unpack(vr[u][i], x);
#pragma unroll
                    for (int c = 0; c < 8; ++c) o[c] = fmaf(pr, x[c], o[c]);
                }
                m = mt;
            }
        }
    }
    // merge the row groups of the wave, then the waves
#pragma unroll
    for (int mask = LPR; mask < 64; mask <<= 1) {
        const float m2 = shfl_xor_f(m, mask);
        const float l2 = shfl_xor_f(l, mask);
        const float mn = fmaxf(m, m2);
        const float a1 = (m == -INFINITY) ? 0.f : __expf(m - mn);
        const float a2 = (m2 == -INFINITY) ? 0.f : __expf(m2 - mn);
        l = l * a1 + l2 * a2;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const float o2 = shfl_xor_f(o[c], mask);
            o[c] = o[c] * a1 + o2 * a2;
        }
        m = mn;
    }
    if (rg == 0) {
        if ((lane % LPR) == 0) {
            s_m[wave] = m;
            s_l[wave] = l;
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) s_o[wave][c0 + c] = o[c];
    }
    __syncthreads();
    if (tid < D) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, s_m[w]);
        float L = 0.f, O = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float a = (s_m[w] == -INFINITY) ? 0.f : __expf(s_m[w] - M);
            L += s_l[w] * a;
            O += s_o[w][tid] * a;
        }
        const float inv = (L > 0.f) ? 1.f / L : 0.f;
        from_f32(out[(long)unit * D + tid], O * inv);
        if (tid == 0 && lse_out) lse_out[unit] = (L > 0.f) ? M + __logf(L) : -INFINITY;
    }
    if constexpr (STATE) {
        if (tid == 0 && atomicAdd(state + kCtrlDone, 1u) == gridDim.x - 1u) {  // every workgroup has read the state
            atomicExch(state + kCtrlDone, 0u);
            *reinterpret_cast<long *>(state + kCtrlStateT) = T_valid;
            const uint32_t nt = state[kCtrlStateTag] + 0x85EBCA6Bu;
            state[kCtrlStateTag] = nt ? nt : 0x5bd1e995u;
        }
    }
}

// state != NULL: the replayable step (T_valid = the largest length, Np = its page count)
void unit_decode_dispatch(int dtype, int D, const void *q, const void *meta, const void *k_cache, const void *v_cache,
                          void *out, float *lse_out, int32_t *idx_out, int B, int Hq, int Hkv, long Tcap, int P,
                          long T_valid, int Np, int K, int n_first, int n_local, float scale, uint32_t *state,
                          hipStream_t stream)
{
    const size_t lds = (size_t)(Np + K) * 4;
#define RS_LAUNCH1(ST, DD, SS)                                                                                   \
    quest_unit_decode_kernel<ST, DD, SS><<<(unsigned)(B * Hq), kUnitThreads, lds, stream>>>(                     \
        (const ST *)q, (const ST *)meta, (const ST *)k_cache, (const ST *)v_cache, (ST *)out, lse_out, idx_out, \
        Hq, Hkv, Tcap, P, T_valid, Np, K, n_first, n_local, scale, Np, state, T_valid)
#define RS_LAUNCH(ST, DD)                  \
    do {                                   \
        if (state) RS_LAUNCH1(ST, DD, true); \
        else RS_LAUNCH1(ST, DD, false);    \
    } while (0)
    if (dtype == RS_BF16) {
        if (D == 128) RS_LAUNCH(bf16, 128);
        else RS_LAUNCH(bf16, 64);
    } else {
        if (D == 128) RS_LAUNCH(float, 128);
        else RS_LAUNCH(float, 64);
    }
#undef RS_LAUNCH
#undef RS_LAUNCH1
}

void decode_attend_dispatch(int dtype, int D, const void *q, const void *k_cache, const void *v_cache,
                            const int32_t *idx, void *out, float *lse_out, uint64_t *partial, int B, int Hq,
                            int Hkv, long Tcap, int P, long T_valid, int K, float scale, int splits,
                            uint32_t *unit_ctr, uint32_t *err, uint32_t tag, int spin_limit, int idx_per_kv,
                            uint32_t *state, long T_max, hipStream_t stream)
{
    const dim3 grid((unsigned)splits, (unsigned)(B * Hq));
    constexpr int kAttThreads = 512;  // about one such workgroup per CU (see the split rule of the caller)
#define RS_LAUNCH(ST, DD)                                                                                   \
    decode_attend_kernel<ST, DD, kAttThreads><<<grid, kAttThreads, 0, stream>>>(                            \
        (const ST *)q, (const ST *)k_cache, (const ST *)v_cache, idx, (ST *)out, lse_out, partial, Hq, Hkv, \
        Tcap, P, T_valid, K, scale, splits, unit_ctr, err, tag, spin_limit, idx_per_kv, state, T_max)
    if (dtype == RS_BF16) {
        if (D == 128) RS_LAUNCH(bf16, 128);
        else RS_LAUNCH(bf16, 64);
    } else {
        if (D == 128) RS_LAUNCH(float, 128);
        else RS_LAUNCH(float, 64);
    }
#undef RS_LAUNCH
}

}  // namespace rs
