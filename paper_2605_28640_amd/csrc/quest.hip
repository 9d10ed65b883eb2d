// Quest at decode (App. A.1, Quest paragraph; Sec. 2.2, Eq. 3-4): page min/max
// representatives, page scores + top-K selection, and softmax attention over the
// selected pages (or over everything: the dense path).
//
// Lane mapping used throughout: a row of D channels is covered by LPR = D/8 lanes with
// 8 channels (one 16-byte bf16 load) each, so a wave touches RPW = 64/LPR rows per load
// instruction and every global access is a run of full 128/256-byte rows.
#include "common.h"

namespace rs {

// ------------------------------------------------------------------------------------
// page metadata: one wave per page
// ------------------------------------------------------------------------------------
template <typename ST, int D>
__global__ __launch_bounds__(256) void quest_page_meta_kernel(const ST *__restrict__ k_cache,
                                                              ST *__restrict__ meta, long Tcap, int P,
                                                              int p_begin, int n_pages, long t_end)
{
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;
    using R = Row8<ST>;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rg = lane / LPR;
    const int c0 = (lane % LPR) * 8;
    const int pl = blockIdx.x * 4 + wave;
    if (pl >= n_pages) return;
    const int p = p_begin + pl;
    const long bh = blockIdx.y;
    const long Np_cap = Tcap / P;
    const long tp = (long)p * P;
    const int valid = (int)((t_end - tp < P) ? (t_end - tp) : P);  // >= 1 by construction

    float lo[8], hi[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        lo[c] = INFINITY;
        hi[c] = -INFINITY;
    }
    for (int r = rg; r < valid; r += RPW) {
        float x[8];
        R::load(k_cache + (bh * Tcap + tp + r) * D + c0, x);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            lo[c] = fminf(lo[c], x[c]);
            hi[c] = fmaxf(hi[c], x[c]);
        }
    }
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            lo[c] = fminf(lo[c], shfl_xor_f(lo[c], m));
            hi[c] = fmaxf(hi[c], shfl_xor_f(hi[c], m));
        }
    }
    ST *mrow = meta + ((bh * Np_cap + p) * 2) * D + c0;
    if (rg == 0) R::store(mrow, lo);
    if (rg == 1) R::store(mrow + D, hi);
}

void page_meta_dispatch(int dtype, int D, const void *k_cache, void *meta, int BH, long Tcap, int P,
                        int p_begin, int n_pages, long t_end, hipStream_t stream)
{
    const dim3 grid((unsigned)((n_pages + 3) / 4), (unsigned)BH);
    if (dtype == RS_BF16) {
        if (D == 128) quest_page_meta_kernel<bf16, 128><<<grid, 256, 0, stream>>>((const bf16 *)k_cache, (bf16 *)meta, Tcap, P, p_begin, n_pages, t_end);
        else quest_page_meta_kernel<bf16, 64><<<grid, 256, 0, stream>>>((const bf16 *)k_cache, (bf16 *)meta, Tcap, P, p_begin, n_pages, t_end);
    } else {
        if (D == 128) quest_page_meta_kernel<float, 128><<<grid, 256, 0, stream>>>((const float *)k_cache, (float *)meta, Tcap, P, p_begin, n_pages, t_end);
        else quest_page_meta_kernel<float, 64><<<grid, 256, 0, stream>>>((const float *)k_cache, (float *)meta, Tcap, P, p_begin, n_pages, t_end);
    }
}

// ------------------------------------------------------------------------------------
// top-K of Np keys held in LDS or global memory, by a 256-thread workgroup.
// Radix select (4 passes of 8 bits) finds the K-th largest key; everything above it is
// taken, and of the keys equal to it the lowest indices; the result is written in
// ascending index order.
// ------------------------------------------------------------------------------------
constexpr int kSelThreads = 256;

struct SelectShared {
    uint32_t hist[256];
    int wave_tot[2][kSelThreads / 64];
    uint32_t prefix;
    int remaining;
};

__device__ __forceinline__ uint32_t page_key(const float *scores, int p, int Np, int n_first, int n_local)
{
    if (p < n_first || p >= Np - n_local) return 0xffffffffu;  // always kept: above every score
    return float_to_key(scores[p]);
}

// exclusive prefix over the workgroup of (x, y); returns totals through tot_x/tot_y
__device__ __forceinline__ void block_exclusive_scan2(int x, int y, int &ex, int &ey, int &tot_x, int &tot_y,
                                                      SelectShared &sh)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int ix = x, iy = y;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int px = __shfl_up(ix, d, 64), py = __shfl_up(iy, d, 64);
        if (lane >= d) {
            ix += px;
            iy += py;
        }
    }
    __syncthreads();
    if (lane == 63) {
        sh.wave_tot[0][wave] = ix;
        sh.wave_tot[1][wave] = iy;
    }
    __syncthreads();
    int bx = 0, by = 0;
    tot_x = 0;
    tot_y = 0;
#pragma unroll
    for (int w = 0; w < kSelThreads / 64; ++w) {
        if (w < wave) {
            bx += sh.wave_tot[0][w];
            by += sh.wave_tot[1][w];
        }
        tot_x += sh.wave_tot[0][w];
        tot_y += sh.wave_tot[1][w];
    }
    ex = bx + ix - x;
    ey = by + iy - y;
}

__device__ void select_topk_pages(const float *scores, int Np, int K, int n_first, int n_local,
                                  int32_t *idx_out, SelectShared &sh)
{
    const int tid = threadIdx.x;
    if (tid == 0) {
        sh.prefix = 0u;
        sh.remaining = K;
    }
    for (int pass = 3; pass >= 0; --pass) {
        sh.hist[tid] = 0u;
        __syncthreads();
        const uint32_t prefix = sh.prefix;
        const int shift = pass * 8;
        const uint32_t himask = (pass == 3) ? 0u : (0xffffffffu << (shift + 8));
        for (int p = tid; p < Np; p += kSelThreads) {
            const uint32_t key = page_key(scores, p, Np, n_first, n_local);
            if ((key & himask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns bins 4l .. 4l+3; suffix sums from the top bin downwards
            const uint32_t h0 = sh.hist[tid * 4], h1 = sh.hist[tid * 4 + 1], h2 = sh.hist[tid * 4 + 2],
                           h3 = sh.hist[tid * 4 + 3];
            const int own = (int)(h0 + h1 + h2 + h3);
            int suf = own;  // inclusive suffix over lanes >= tid
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int o = __shfl_down(suf, d, 64);
                if (tid + d < 64) suf += o;
            }
            const int above = suf - own;  // keys in bins of higher lanes
            const int rem = sh.remaining;
            if (above < rem && rem <= suf) {  // the K-th largest falls in this lane's bins
                int acc = above;
                int bin = tid * 4 + 3;
                const uint32_t hh[4] = {h0, h1, h2, h3};
                for (int b = 3; b >= 0; --b) {
                    if (acc + (int)hh[b] >= rem) {
                        bin = tid * 4 + b;
                        break;
                    }
                    acc += (int)hh[b];
                }
                sh.prefix = prefix | ((uint32_t)bin << shift);
                sh.remaining = rem - acc;
            }
        }
        __syncthreads();
    }
    const uint32_t kth = sh.prefix;   // the K-th largest key
    const int take_eq = sh.remaining;  // how many keys equal to it are taken (lowest indices)

    // contiguous index ranges per thread keep the output ascending
    const int per = (Np + kSelThreads - 1) / kSelThreads;
    const int p0 = tid * per;
    const int p1 = (p0 + per < Np) ? p0 + per : Np;
    int n_gt = 0, n_eq = 0;
    for (int p = p0; p < p1; ++p) {
        const uint32_t key = page_key(scores, p, Np, n_first, n_local);
        n_gt += key > kth;
        n_eq += key == kth;
    }
    int e_gt, e_eq, t_gt, t_eq;
    block_exclusive_scan2(n_gt, n_eq, e_gt, e_eq, t_gt, t_eq, sh);
    // selected before this thread = all greater ones + the equal ones that fit the quota
    int pos = e_gt + (e_eq < take_eq ? e_eq : take_eq);
    int eq_rank = e_eq;
    for (int p = p0; p < p1; ++p) {
        const uint32_t key = page_key(scores, p, Np, n_first, n_local);
        bool sel = key > kth;
        if (key == kth) {
            sel = eq_rank < take_eq;
            ++eq_rank;
        }
        if (sel) idx_out[pos++] = p;
    }
}

// ------------------------------------------------------------------------------------
// page scores; the last workgroup of a (batch, query head) to finish runs the selection
// ------------------------------------------------------------------------------------
template <typename ST, int D>
__global__ __launch_bounds__(kSelThreads) void quest_score_select_kernel(
    const ST *__restrict__ q, const ST *__restrict__ meta, float *scores, int32_t *idx_out, int Hq,
    int Hkv, long Np_cap, int Np, int K, int n_first, int n_local, int splits, uint32_t *unit_ctr)
{
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;
    using R = Row8<ST>;
    __shared__ SelectShared sh;
    __shared__ int s_last;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int rg = lane / LPR;
    const int c0 = (lane % LPR) * 8;
    const int unit = blockIdx.y;  // b * Hq + h
    const int b = unit / Hq, h = unit % Hq;
    const int kvh = h / (Hq / Hkv);
    const ST *mbase = meta + ((long)(b * Hkv + kvh) * Np_cap) * 2 * D;
    float *srow = scores + (long)unit * Np;

    float qv[8];
    R::load(q + (long)unit * D + c0, qv);

    // this workgroup's pages: a contiguous slice
    const int per = (Np + splits - 1) / splits;
    const int pb = blockIdx.x * per;
    const int pe = (pb + per < Np) ? pb + per : Np;
    constexpr int PPI = RPW * (kSelThreads / 64);  // pages per workgroup iteration
    // the LPR lanes of a row group share p, so they leave the loop together and the
    // group-local shuffles below only ever read active lanes
    for (int p = pb + wave * RPW + rg; p < pe; p += PPI) {
        float mn[8], mx[8];
        R::load(mbase + ((long)p * 2) * D + c0, mn);
        R::load(mbase + ((long)p * 2 + 1) * D + c0, mx);
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) s += fmaxf(qv[c] * mn[c], qv[c] * mx[c]);
        s = group_sum<LPR>(s);
        if ((lane % LPR) == 0) srow[p] = s;
    }

    // arrival counter: the last workgroup of this unit sees every score
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t prev = atomicAdd(&unit_ctr[unit], 1u);
        s_last = (prev == (uint32_t)splits - 1u);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    if (idx_out) select_topk_pages(srow, Np, K, n_first, n_local, idx_out + (long)unit * K, sh);
    if (tid == 0) atomicExch(&unit_ctr[unit], 0u);
}

void score_select_dispatch(int dtype, int D, const void *q, const void *meta, float *scores,
                           int32_t *idx_out, int B, int Hq, int Hkv, long Np_cap, int Np, int K,
                           int n_first, int n_local, int splits, uint32_t *unit_ctr, hipStream_t stream)
{
    const dim3 grid((unsigned)splits, (unsigned)(B * Hq));
#define RS_LAUNCH(ST, DD)                                                                                 \
    quest_score_select_kernel<ST, DD><<<grid, kSelThreads, 0, stream>>>((const ST *)q, (const ST *)meta, scores, \
                                                                        idx_out, Hq, Hkv, Np_cap, Np, K, n_first, \
                                                                        n_local, splits, unit_ctr)
    if (dtype == RS_BF16) {
        if (D == 128) RS_LAUNCH(bf16, 128);
        else RS_LAUNCH(bf16, 64);
    } else {
        if (D == 128) RS_LAUNCH(float, 128);
        else RS_LAUNCH(float, 64);
    }
#undef RS_LAUNCH
}

// ------------------------------------------------------------------------------------
// decode attention over a list of 16-row tiles (selected pages, or all rows), split over
// workgroups; partial (m, l, o) per split; the last split to finish merges them.
// ------------------------------------------------------------------------------------
constexpr int kAttThreads = 256;
constexpr int kAttWaves = kAttThreads / 64;

template <typename ST, int D>
__global__ __launch_bounds__(kAttThreads) void decode_attend_kernel(
    const ST *__restrict__ q, const ST *__restrict__ k_cache, const ST *__restrict__ v_cache,
    const int32_t *idx, ST *__restrict__ out, float *__restrict__ lse_out, float *partial, int Hq, int Hkv,
    long Tcap, int P, long T_valid, int K, float scale, int splits, uint32_t *unit_ctr)
{
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;        // rows per load instruction
    constexpr int TR = 16;               // rows per tile
    constexpr int RPL = TR / RPW;        // rows per lane per tile (4 for D=128, 2 for D=64)
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

    float qv[8];
    R::load(q + (long)unit * D + c0, qv);
#pragma unroll
    for (int c = 0; c < 8; ++c) qv[c] *= scale;

    const int tiles_per_page = P / TR;
    const long n_tiles = idx ? (long)K * tiles_per_page : (T_valid + TR - 1) / TR;
    const long per = (n_tiles + splits - 1) / splits;
    const long tb = (long)blockIdx.x * per;
    const long te = (tb + per < n_tiles) ? tb + per : n_tiles;

    float m = -INFINITY, l = 0.f;
    float o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = 0.f;

    for (long t = tb + wave; t < te; t += kAttWaves) {
        long row0;
        if (idx) {
            const int page = idx[(long)unit * K + t / tiles_per_page];
            if (page < 0) continue;
            row0 = (long)page * P + (t % tiles_per_page) * TR;
        } else {
            row0 = t * TR;
        }
        if (row0 >= T_valid) continue;
        typename R::raw_t kr[RPL], vr[RPL];
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            const long row = row0 + i * RPW + rg;
            if (row < T_valid) {
                kr[i] = R::load_raw(kb + row * D + c0);
                vr[i] = R::load_raw(vb + row * D + c0);
            } else {
                kr[i] = R::zero_raw();
                vr[i] = R::zero_raw();
            }
        }
        float s[RPL];
        float mt = m;
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            float x[8];
            R::unpack(kr[i], x);
            float d = 0.f;
#pragma unroll
            for (int c = 0; c < 8; ++c) d = fmaf(qv[c], x[c], d);
            d = group_sum<LPR>(d);
            const long row = row0 + i * RPW + rg;
            s[i] = (row < T_valid) ? d : -INFINITY;
            mt = fmaxf(mt, s[i]);
        }
        if (mt == -INFINITY) continue;  // this lane's row group saw no valid row yet
        const float corr = __expf(m - mt);
        l *= corr;
#pragma unroll
        for (int c = 0; c < 8; ++c) o[c] *= corr;
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            const float p = __expf(s[i] - mt);
            l += p;
            float x[8];
            R::unpack(vr[i], x);
#pragma unroll
            for (int c = 0; c < 8; ++c) o[c] = fmaf(p, x[c], o[c]);
        }
        m = mt;
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
    float *part = partial + ((long)unit * splits + blockIdx.x) * (D + 2);
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
            part[2 + tid] = O;
            if (tid == 0) {
                part[0] = M;
                part[1] = L;
            }
        }
    }
    if (splits == 1) return;

    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t prev = atomicAdd(&unit_ctr[unit], 1u);
        s_last = (prev == (uint32_t)splits - 1u);
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    if (tid < D) {
        const float *pu = partial + (long)unit * splits * (D + 2);
        float M = -INFINITY;
        for (int sidx = 0; sidx < splits; ++sidx) M = fmaxf(M, pu[(long)sidx * (D + 2)]);
        float L = 0.f, O = 0.f;
        for (int sidx = 0; sidx < splits; ++sidx) {
            const float ms = pu[(long)sidx * (D + 2)];
            const float a = (ms == -INFINITY) ? 0.f : __expf(ms - M);
            L += pu[(long)sidx * (D + 2) + 1] * a;
            O += pu[(long)sidx * (D + 2) + 2 + tid] * a;
        }
        const float inv = (L > 0.f) ? 1.f / L : 0.f;
        from_f32(out[(long)unit * D + tid], O * inv);
        if (tid == 0 && lse_out) lse_out[unit] = (L > 0.f) ? M + __logf(L) : -INFINITY;
    }
    if (tid == 0) atomicExch(&unit_ctr[unit], 0u);
}

void decode_attend_dispatch(int dtype, int D, const void *q, const void *k_cache, const void *v_cache,
                            const int32_t *idx, void *out, float *lse_out, float *partial, int B, int Hq,
                            int Hkv, long Tcap, int P, long T_valid, int K, float scale, int splits,
                            uint32_t *unit_ctr, hipStream_t stream)
{
    const dim3 grid((unsigned)splits, (unsigned)(B * Hq));
#define RS_LAUNCH(ST, DD)                                                                                   \
    decode_attend_kernel<ST, DD><<<grid, kAttThreads, 0, stream>>>(                                         \
        (const ST *)q, (const ST *)k_cache, (const ST *)v_cache, idx, (ST *)out, lse_out, partial, Hq, Hkv, \
        Tcap, P, T_valid, K, scale, splits, unit_ctr)
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
