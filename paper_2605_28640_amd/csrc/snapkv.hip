// SnapKV cache compression (App. A.1, SnapKV paragraph; Sec. 2.2, Eq. 3 over single tokens):
// the W observation queries at the end of the prompt attend causally; each prefix position
// collects its attention probability summed over the window and over the query heads of its
// KV head's group; the votes are max-pooled; per KV head the K_keep best positions are kept
// (ascending), followed by the window rows.
//
// The [G*W x T] score matrix of a KV head is a dense contraction, done on the matrix cores
// (v_mfma_f32_32x32x16_bf16) in two sweeps over the keys: sweep 1 forms S^T = K Q^T so that
// a lane owns one query row and gets its softmax max / sum cheaply; sweep 2 forms S = Q K^T
// so that a lane owns one key column and its vote is an in-lane sum over the query rows.
#include "common.h"
#include "knobs.h"
#include "select.h"

#include <type_traits>

namespace rs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kSnapKeysPerWg = 2048;  // keys per workgroup, at most (fewer when that leaves the chip idle)
constexpr int kSnapKT = 128;          // keys per step: four 32-key sub-tiles

// K tiles of 128 keys are double-buffered in LDS and filled by direct global -> LDS loads
// (unpadded rows, 16-byte chunks permuted by chunk_swizzle); the next tile's loads are issued
// between the current tile's matrix instructions.  Pass i of a tile: a lane fetches 16 bytes
// of row RPI i + srow; rows past the end of the keys repeat the last valid row (finite data,
// masked or never stored).
template <int D>
struct SnapStage {
    static constexpr int CR = D / 8;          // 16-byte chunks per row
    static constexpr int RW = 64 / CR;        // rows one wave-wide load covers
    static constexpr int RPI = 4 * RW;        // rows one pass of the four waves covers
    static constexpr int NP = kSnapKT / RPI;  // passes per tile
    int srow, gchunk, wave;
    __device__ __forceinline__ SnapStage()
    {
        const int lane = threadIdx.x & 63;
        wave = threadIdx.x >> 6;
        srow = wave * RW + lane / CR;
        gchunk = (lane % CR) ^ chunk_swizzle<D>(srow);
    }
    // kt: first row of the tile in global memory; rem: valid rows of the tile (>= 1)
    __device__ __forceinline__ void pass(const bf16 *kt, uint16_t *tile, int i, int rem) const
    {
        const int r = (i * RPI + srow < rem) ? i * RPI + srow : rem - 1;
        load16_to_lds(lds_source(kt), (uint32_t)(r * D + gchunk * 8) * 2u, tile + (i * RPI + wave * RW) * D);
    }
};

// sweep 1: partial softmax statistics (max, sum) per (query row, key chunk).  S^T = K Q^T: a
// lane owns one query row (a column of S^T), so its max and sum are in-lane reductions plus
// one cross-half shuffle.  Wave w holds rows 32 w .. 32 w + 31 of the 128-row tile.
template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void snapkv_stats_kernel(
    const bf16 *__restrict__ q_win, const bf16 *__restrict__ k_cache, float *__restrict__ stats, int Hq, int Hkv, long T,
    long Tcap, int W, int n_chunks, float scale, int keys_per_wg)
{
    constexpr int NC = D / 16;
    using Stage = SnapStage<D>;
    __shared__ __attribute__((aligned(1024))) uint16_t sK0[kSnapKT * D];
    __shared__ __attribute__((aligned(1024))) uint16_t sK1[kSnapKT * D];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, h = lane >> 5;
    const int chunk = blockIdx.x;
    const int bk = blockIdx.y;  // b * Hkv + kvh
    const int b = bk / Hkv, kvh = bk % Hkv;
    const int G = Hq / Hkv;
    const int R = G * W;  // query rows of this KV head
    const long L = T - W;
    const bf16 *kb = k_cache + (long)bk * Tcap * D;
    const long kc0 = (long)chunk * keys_per_wg;
    const long kc1 = (kc0 + keys_per_wg < T) ? kc0 + keys_per_wg : T;
    const int n_steps = (int)((kc1 - kc0 + kSnapKT - 1) / kSnapKT);
    const int n_row_tiles = (R + 127) / 128;
    const Stage st;
    uint32_t koff[NC];  // K operand: row lq of a sub-tile, chunk 2 c + h (elements)
    {
        const int sw = chunk_swizzle<D>(lq);
#pragma unroll
        for (int c = 0; c < NC; ++c) koff[c] = (uint32_t)(lq * D + (((2 * c + h) ^ sw) * 8));
    }
    const float cs = scale * 1.4426950408889634f;  // base-2 domain

    for (int rt = 0; rt < n_row_tiles; ++rt) {
        const int r = rt * 128 + wave * 32 + lq;
        const bool r_ok = r < R;
        const int g = r_ok ? r / W : 0, w = r_ok ? r % W : 0;
        {
            const int rem = (int)((kc1 - kc0 < kSnapKT) ? kc1 - kc0 : kSnapKT);
#pragma unroll
            for (int i = 0; i < Stage::NP; ++i) st.pass(kb + kc0 * D, sK0, i, rem);
        }
        bf16x8 qf[NC];
        {
            const bf16 *qrow = q_win + ((long)(b * Hq + kvh * G + g) * W + w) * D;
#pragma unroll
            for (int c = 0; c < NC; ++c) qf[c] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * c + 8 * h);
        }
        const long pos = L + w;  // absolute position of the query: keys <= pos are visible
        float m = -INFINITY, l = 0.f;
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        __syncthreads();

        auto step = [&](auto next_tag, auto buf_tag, int it) {
            constexpr bool NEXT = decltype(next_tag)::value;
            constexpr int BUF = decltype(buf_tag)::value;
            const uint16_t *cK = BUF ? sK1 : sK0;
            uint16_t *nK = BUF ? sK0 : sK1;
            const long k0 = kc0 + (long)it * kSnapKT;
            const long kn = k0 + kSnapKT;
            const int rem_n = (int)((kc1 - kn < kSnapKT) ? kc1 - kn : kSnapKT);
            // keys of this tile a lane may see, as offsets from k0: 0 .. hi (all 128 in the bulk)
            const long hi_l = ((pos < kc1 - 1) ? pos : kc1 - 1) - k0;
            const bool edge = (k0 + kSnapKT > kc1) || (k0 + kSnapKT - 1 > L);  // uniform
#pragma unroll
            for (int sp = 0; sp < 2; ++sp) {  // pairs of 32-key sub-tiles
                f32x16 sacc[2];
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sacc[u][v] = 0.f;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    if constexpr (NEXT) {
                        constexpr int every = (2 * NC) / Stage::NP;  // matrix-instruction pairs per load
                        if ((sp * NC + c) % every == 0) st.pass(kb + kn * D, nK, (sp * NC + c) / every, rem_n);
                    }
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&cK[32 * (2 * sp + u) * D + koff[c]]);
                        sacc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], sacc[u], 0, 0, 0);  // [key][row]
                    }
                }
                if (edge) {
                    const int hi = (int)((hi_l > kSnapKT) ? kSnapKT : ((hi_l < -1) ? -1 : hi_l)) - 4 * h;
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int e = 32 * (2 * sp + u) + 8 * (v / 4) + (v % 4);  // + 4 h: folded into hi
                            if (e > hi) sacc[u][v] = -INFINITY;
                        }
                }
                float mx = -INFINITY;
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[u][v]);
                mx = half_pair_max(mx) * cs;
                const float m_new = fmaxf(m, mx);
                const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
                float psum = 0.f;
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int v = 0; v < 16; ++v) psum += __builtin_amdgcn_exp2f(fmaf(sacc[u][v], cs, -m_safe));
                psum = half_pair_sum(psum);
                l = l * ((m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - m_safe)) + psum;
                m = m_new;
            }
            if constexpr (NEXT) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's loads have landed
            __syncthreads();
        };
        {
            using B0 = std::integral_constant<int, 0>;
            using B1 = std::integral_constant<int, 1>;
            int it = 0;
            for (; it + 2 < n_steps; it += 2) {
                step(std::true_type{}, B0{}, it);
                step(std::true_type{}, B1{}, it + 1);
            }
            if (it + 2 == n_steps) {
                step(std::true_type{}, B0{}, it);
                step(std::false_type{}, B1{}, it + 1);
            } else {
                step(std::false_type{}, B0{}, it);
            }
        }
        if (r_ok && h == 0) {  // (max, sum) back in the natural-log domain
            float *sp = stats + (((long)bk * n_chunks + chunk) * R + r) * 2;
            sp[0] = m * 0.6931471805599453f;
            sp[1] = l;
        }
    }
}

// sweep 2: the votes.  S = Q K^T: a lane owns one key column, and wave w takes the keys of
// sub-tile w of every 128-key step against all (up to 128) query rows of the row tile, so a
// key's vote is an in-lane sum plus one cross-half shuffle and is written straight out.  Only
// prefix keys (< L) are stored, and every window query sees all of them: no mask is needed.
template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void snapkv_votes_kernel(
    const bf16 *__restrict__ q_win, const bf16 *__restrict__ k_cache, const float *__restrict__ lse,
    float *__restrict__ votes, int Hq, int Hkv, long T, long Tcap, int W, float scale, int keys_per_wg)
{
    constexpr int NC = D / 16;
    using Stage = SnapStage<D>;
    __shared__ __attribute__((aligned(1024))) uint16_t sK0[kSnapKT * D];
    __shared__ __attribute__((aligned(1024))) uint16_t sK1[kSnapKT * D];

    __shared__ __attribute__((aligned(16))) float s_lse2[128];  // row log-sum-exp, base-2 domain

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, h = lane >> 5;
    const int chunk = blockIdx.x;
    const int bk = blockIdx.y;  // b * Hkv + kvh
    const int b = bk / Hkv, kvh = bk % Hkv;
    const int G = Hq / Hkv;
    const int R = G * W;
    const long L = T - W;
    const bf16 *kb = k_cache + (long)bk * Tcap * D;
    const long kc0 = (long)chunk * keys_per_wg;
    const long kc1 = (kc0 + keys_per_wg < L) ? kc0 + keys_per_wg : L;  // prefix keys only
    const int n_steps = (int)((kc1 - kc0 + kSnapKT - 1) / kSnapKT);
    const int n_row_tiles = (R + 127) / 128;
    const Stage st;
    uint32_t koff[NC];
    {
        const int sw = chunk_swizzle<D>(lq);
#pragma unroll
        for (int c = 0; c < NC; ++c) koff[c] = (uint32_t)((32 * wave + lq) * D + (((2 * c + h) ^ sw) * 8));
    }
    const float cs = scale * 1.4426950408889634f;

    for (int rt = 0; rt < n_row_tiles; ++rt) {
        {
            const int rem = (int)((kc1 - kc0 < kSnapKT) ? kc1 - kc0 : kSnapKT);
#pragma unroll
            for (int i = 0; i < Stage::NP; ++i) st.pass(kb + kc0 * D, sK0, i, rem);
        }
        // A operands: query rows 32 rg + lq of the row tile, rg = 0..3; and, for the 16 rows of
        // all rows of the tile, their log-sum-exp in LDS (base-2 domain; +inf for padding rows:
        // their votes vanish)
        bf16x8 qf[4][NC];
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const int r = rt * 128 + rg * 32 + lq;
            const int rc = (r < R) ? r : 0;
            const bf16 *qrow = q_win + ((long)(b * Hq + kvh * G + rc / W) * W + rc % W) * D;
#pragma unroll
            for (int c = 0; c < NC; ++c) qf[rg][c] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * c + 8 * h);
        }
        if (rt > 0) __syncthreads();  // the previous row tile's readers are done with s_lse2
        if (tid < 128) {
            const int rr = rt * 128 + tid;
            s_lse2[tid] = (rr < R) ? lse[(long)bk * R + rr] * 1.4426950408889634f : INFINITY;
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        __syncthreads();

        auto step = [&](auto next_tag, auto buf_tag, int it) {
            constexpr bool NEXT = decltype(next_tag)::value;
            constexpr int BUF = decltype(buf_tag)::value;
            const uint16_t *cK = BUF ? sK1 : sK0;
            uint16_t *nK = BUF ? sK0 : sK1;
            const long k0 = kc0 + (long)it * kSnapKT;
            const long kn = k0 + kSnapKT;
            const int rem_n = (int)((kc1 - kn < kSnapKT) ? kc1 - kn : kSnapKT);
            float vsum = 0.f;
#pragma unroll
            for (int rp = 0; rp < 2; ++rp) {  // pairs of 32-row groups
                f32x16 sacc[2];
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sacc[u][v] = 0.f;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    if constexpr (NEXT) {
                        constexpr int every = (2 * NC) / Stage::NP;
                        if ((rp * NC + c) % every == 0) st.pass(kb + kn * D, nK, (rp * NC + c) / every, rem_n);
                    }
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&cK[koff[c]]);
#pragma unroll
                    for (int u = 0; u < 2; ++u)
                        sacc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[2 * rp + u][c], kf, sacc[u], 0, 0, 0);  // [row][key]
                }
                // accumulator value v: row 8 (v / 4) + 4 h + v % 4 of the group
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        const float4 ls = *reinterpret_cast<const float4 *>(&s_lse2[(2 * rp + u) * 32 + 8 * qd + 4 * h]);
                        vsum += __builtin_amdgcn_exp2f(fmaf(sacc[u][4 * qd], cs, -ls.x));
                        vsum += __builtin_amdgcn_exp2f(fmaf(sacc[u][4 * qd + 1], cs, -ls.y));
                        vsum += __builtin_amdgcn_exp2f(fmaf(sacc[u][4 * qd + 2], cs, -ls.z));
                        vsum += __builtin_amdgcn_exp2f(fmaf(sacc[u][4 * qd + 3], cs, -ls.w));
                    }
            }
            vsum = half_pair_sum(vsum);
            const long key = k0 + 32 * wave + lq;
            if (h == 0 && key < kc1) {
                float *dst = votes + (long)bk * L + key;
                *dst = (rt == 0) ? vsum : *dst + vsum;
            }
            if constexpr (NEXT) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
            __syncthreads();
        };
        {
            using B0 = std::integral_constant<int, 0>;
            using B1 = std::integral_constant<int, 1>;
            int it = 0;
            for (; it + 2 < n_steps; it += 2) {
                step(std::true_type{}, B0{}, it);
                step(std::true_type{}, B1{}, it + 1);
            }
            if (it + 2 == n_steps) {
                step(std::true_type{}, B0{}, it);
                step(std::false_type{}, B1{}, it + 1);
            } else {
                step(std::false_type{}, B0{}, it);
            }
        }
    }
}

// log-sum-exp of each row over its key chunks: one wave per row, lanes over chunks
__global__ __launch_bounds__(256) void snapkv_lse_kernel(const float *__restrict__ stats, float *__restrict__ lse, int R,
                                                         int n_chunks, long rows_total)
{
    const long i = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (i >= rows_total) return;
    const long bk = i / R;
    const int r = (int)(i % R);
    float M = -INFINITY;
    for (int c = lane; c < n_chunks; c += 64) M = fmaxf(M, stats[((bk * n_chunks + c) * R + r) * 2]);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) M = fmaxf(M, shfl_xor_f(M, m));
    float Ls = 0.f;
    for (int c = lane; c < n_chunks; c += 64) {
        const float mc = stats[((bk * n_chunks + c) * R + r) * 2];
        if (mc != -INFINITY) Ls += stats[((bk * n_chunks + c) * R + r) * 2 + 1] * __expf(mc - M);
    }
    // fixed butterfly order: the same bits on every run
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) Ls += shfl_xor_f(Ls, m);
    if (lane == 0) lse[i] = M + __logf(Ls);
}

__global__ void snapkv_pool_kernel(const float *__restrict__ votes, float *__restrict__ pooled, long L, int kernel,
                                   long total, uint32_t *__restrict__ sel_hist, long n_hist)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    for (long z = i; z < n_hist; z += (long)gridDim.x * blockDim.x) sel_hist[z] = 0u;  // the select's bins start at zero
    if (i >= total) return;
    const long row = i / L, p = i % L;
    const int half = kernel / 2;
    const long lo = (p - half < 0) ? 0 : p - half;
    const long hi = (p + half > L - 1) ? L - 1 : p + half;
    float m = votes[row * L + lo];
    for (long j = lo + 1; j <= hi; ++j) m = fmaxf(m, votes[row * L + j]);
    pooled[i] = m;
}

// ------------------------------------------------------------------------------------
// top-K_keep of L pooled votes per (batch, KV head): radix select over the order-preserving
// keys, 8 bits per pass, spread over workgroups of 4096 positions each (one workgroup per
// head would leave most of the chip idle at 128K positions).  Pass p histograms the keys that
// match the bits fixed so far into 256 global bins; the next launch starts by locating the
// bin that holds the K-th largest key (every workgroup repeats that small search instead of
// passing it on).  After four passes the K-th key is known exactly; a count launch leaves,
// per workgroup, how many keys are above it and equal to it, and the emit launch writes the
// kept positions in ascending order (equal keys: lowest positions first).
// ------------------------------------------------------------------------------------
constexpr int kSelThreads = 256;
constexpr int kSelPerThread = 16;
constexpr int kSelSlice = kSelThreads * kSelPerThread;

// K-th largest key so far: the bits fixed by the first npass passes and the rank still wanted
// inside that prefix.  Called by the 64 lanes of one wave; every lane returns the result.
__device__ __forceinline__ void sel_resolve(const uint32_t *__restrict__ hist_bk, int npass, int K_keep,
                                            uint32_t &prefix, int &remaining)
{
    const int lane = threadIdx.x & 63;
    prefix = 0u;
    remaining = K_keep;
    for (int pp = 0; pp < npass; ++pp) {
        const uint32_t *hp = hist_bk + pp * 256;
        const uint4 hv = *reinterpret_cast<const uint4 *>(hp + lane * 4);
        const uint32_t hh[4] = {hv.x, hv.y, hv.z, hv.w};
        const int own = (int)(hh[0] + hh[1] + hh[2] + hh[3]);
        int suf = own;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_down(suf, d, 64);
            if (lane + d < 64) suf += o;
        }
        const int above = suf - own;
        const bool mine = above < remaining && remaining <= suf;
        int acc = above, bin = lane * 4;
        for (int bb = 3; bb >= 0; --bb) {
            if (acc + (int)hh[bb] >= remaining) {
                bin = lane * 4 + bb;
                break;
            }
            acc += (int)hh[bb];
        }
        const uint64_t who = __ballot(mine);  // exactly one lane while remaining <= candidates
        const int src = who ? (int)__builtin_ctzll(who) : 0;
        bin = __shfl(bin, src, 64);
        acc = __shfl(acc, src, 64);
        prefix |= (uint32_t)bin << (24 - 8 * pp);
        remaining -= acc;
    }
}

// this thread's 16 keys of the slice: position slice_base + 1024 wave + 64 j + lane (a wave
// walks its 1024 positions in order); positions past L are flagged invalid
__device__ __forceinline__ void sel_load_keys(const float *__restrict__ src, long L, long slice_base, uint32_t *key,
                                              uint32_t &valid)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float x[kSelPerThread];
    valid = 0u;
#pragma unroll
    for (int j = 0; j < kSelPerThread; ++j) {
        const long p = slice_base + wave * (64 * kSelPerThread) + j * 64 + lane;
        x[j] = (p < L) ? src[p] : 0.f;
        if (p < L) valid |= 1u << j;
    }
#pragma unroll
    for (int j = 0; j < kSelPerThread; ++j) key[j] = float_to_key(x[j]);
}

__global__ __launch_bounds__(kSelThreads) void snapkv_sel_hist_kernel(const float *__restrict__ pooled,
                                                                      uint32_t *__restrict__ hist, long L, int K_keep,
                                                                      int pass)
{
    __shared__ uint32_t lh[256];
    __shared__ uint32_t s_prefix;
    const int tid = threadIdx.x;
    const long bk = blockIdx.y;
    uint32_t key[kSelPerThread], valid;
    sel_load_keys(pooled + bk * L, L, (long)blockIdx.x * kSelSlice, key, valid);
    lh[tid] = 0u;
    if (tid < 64) {
        uint32_t prefix;
        int remaining;
        sel_resolve(hist + bk * 1024, pass, K_keep, prefix, remaining);
        if (tid == 0) s_prefix = prefix;
    }
    __syncthreads();
    const uint32_t prefix = s_prefix;
    const int shift = 24 - 8 * pass;
    const uint32_t himask = (pass == 0) ? 0u : (0xffffffffu << (shift + 8));
#pragma unroll
    for (int j = 0; j < kSelPerThread; ++j)
        if (((valid >> j) & 1u) && (key[j] & himask) == prefix) atomicAdd(&lh[(key[j] >> shift) & 255u], 1u);
    __syncthreads();
    if (lh[tid]) atomicAdd(&hist[(bk * 4 + pass) * 256 + tid], lh[tid]);
}

__global__ __launch_bounds__(kSelThreads) void snapkv_sel_count_kernel(const float *__restrict__ pooled,
                                                                       const uint32_t *__restrict__ hist,
                                                                       uint32_t *__restrict__ cnt, long L, int K_keep)
{
    __shared__ int s_gt[kSelThreads / 64], s_eq[kSelThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long bk = blockIdx.y;
    uint32_t key[kSelPerThread], valid;
    sel_load_keys(pooled + bk * L, L, (long)blockIdx.x * kSelSlice, key, valid);
    uint32_t kth;
    int take_eq;
    sel_resolve(hist + bk * 1024, 4, K_keep, kth, take_eq);  // every wave on its own
    int n_gt = 0, n_eq = 0;
#pragma unroll
    for (int j = 0; j < kSelPerThread; ++j) {
        const bool ok = (valid >> j) & 1u;
        n_gt += (ok && key[j] > kth) ? 1 : 0;
        n_eq += (ok && key[j] == kth) ? 1 : 0;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        n_gt += __shfl_xor(n_gt, d, 64);
        n_eq += __shfl_xor(n_eq, d, 64);
    }
    if (lane == 0) {
        s_gt[wave] = n_gt;
        s_eq[wave] = n_eq;
    }
    __syncthreads();
    if (tid == 0) {
        int g = 0, e = 0;
        for (int w2 = 0; w2 < kSelThreads / 64; ++w2) {
            g += s_gt[w2];
            e += s_eq[w2];
        }
        cnt[(bk * gridDim.x + blockIdx.x) * 2] = (uint32_t)g;
        cnt[(bk * gridDim.x + blockIdx.x) * 2 + 1] = (uint32_t)e;
    }
}

__global__ __launch_bounds__(kSelThreads) void snapkv_sel_emit_kernel(const float *__restrict__ pooled,
                                                                      const uint32_t *__restrict__ hist,
                                                                      const uint32_t *__restrict__ cnt,
                                                                      int32_t *__restrict__ idx_out, long L, int K_keep)
{
    __shared__ int s_gt[kSelThreads / 64], s_eq[kSelThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long bk = blockIdx.y;
    const long slice_base = (long)blockIdx.x * kSelSlice;
    int32_t *dst = idx_out + bk * K_keep;
    uint32_t key[kSelPerThread], valid;
    sel_load_keys(pooled + bk * L, L, slice_base, key, valid);
    uint32_t kth;
    int take_eq;
    sel_resolve(hist + bk * 1024, 4, K_keep, kth, take_eq);
    // keys above / equal in the slices before this one
    int gt_before = 0, eq_before = 0;
    for (int sl = lane; sl < (int)blockIdx.x; sl += 64) {
        gt_before += (int)cnt[(bk * gridDim.x + sl) * 2];
        eq_before += (int)cnt[(bk * gridDim.x + sl) * 2 + 1];
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        gt_before += __shfl_xor(gt_before, d, 64);
        eq_before += __shfl_xor(eq_before, d, 64);
    }
    // and in the waves before this one
    int n_gt = 0, n_eq = 0;
#pragma unroll
    for (int j = 0; j < kSelPerThread; ++j) {
        const bool ok = (valid >> j) & 1u;
        n_gt += __popcll(__ballot(ok && key[j] > kth));
        n_eq += __popcll(__ballot(ok && key[j] == kth));
    }
    if (lane == 0) {
        s_gt[wave] = n_gt;
        s_eq[wave] = n_eq;
    }
    __syncthreads();
    for (int w2 = 0; w2 < wave; ++w2) {
        gt_before += s_gt[w2];
        eq_before += s_eq[w2];
    }
#pragma unroll
    for (int j = 0; j < kSelPerThread; ++j) {
        const long p = slice_base + wave * (64 * kSelPerThread) + j * 64 + lane;
        const bool ok = (valid >> j) & 1u;
        const bool is_gt = ok && key[j] > kth, is_eq = ok && key[j] == kth;
        const uint64_t bg = __ballot(is_gt), be = __ballot(is_eq);
        const int gt_lane = __builtin_amdgcn_mbcnt_hi((uint32_t)(bg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bg, 0u));
        const int eq_lane = __builtin_amdgcn_mbcnt_hi((uint32_t)(be >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)be, 0u));
        const int eq_rank = eq_before + eq_lane;  // rank among all positions equal to the K-th vote
        if (is_gt || (is_eq && eq_rank < take_eq)) {
            const int eq_taken = (eq_rank < take_eq) ? eq_rank : take_eq;  // equal positions before this one that are kept
            dst[gt_before + gt_lane + (is_eq ? eq_rank : eq_taken)] = (int32_t)p;
        }
        gt_before += __popcll(bg);
        eq_before += __popcll(be);
    }
}

// copy the kept rows, then the window rows: one 16-byte chunk per thread
template <typename ST>
__global__ void snapkv_gather_kernel(const ST *__restrict__ k_cache, const ST *__restrict__ v_cache,
                                     const int32_t *__restrict__ idx, ST *__restrict__ kc_out, ST *__restrict__ vc_out,
                                     long T, long Tcap, long Tcap_out, int W, int K_keep, int D, long total)
{
    const int cpr = D * (int)sizeof(ST) / 16;  // chunks per row
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const long rows = K_keep + W;
    const long bk = i / (rows * cpr);
    const long rem = i % (rows * cpr);
    const long r = rem / cpr;
    const int c = (int)(rem % cpr);
    const long srow = (r < K_keep) ? idx[bk * K_keep + r] : (T - W) + (r - K_keep);
    const uint4 *ks = reinterpret_cast<const uint4 *>(k_cache + (bk * Tcap + srow) * D) + c;
    const uint4 *vs = reinterpret_cast<const uint4 *>(v_cache + (bk * Tcap + srow) * D) + c;
    reinterpret_cast<uint4 *>(kc_out + (bk * Tcap_out + r) * D)[c] = *ks;
    reinterpret_cast<uint4 *>(vc_out + (bk * Tcap_out + r) * D)[c] = *vs;
}

// Short prefixes (at most kSnapOneWgKeys positions per head): pooling, the top-K_keep selection
// and the ascending output in one launch, one 1024-thread workgroup per (batch, KV head) with
// the order-preserving keys of the pooled votes in LDS (the selection the decode kernels use:
// keys above the K-th, then equal ones by lowest position).  At these sizes the seven launches
// of the spread-out selection below cost more than the work in them.
constexpr int kSnapOneWgKeys = 15360;  // 60 KiB of keys
constexpr int kSnapOneWgThreads = 1024;

__global__ __launch_bounds__(kSnapOneWgThreads) void snapkv_pool_select_kernel(const float *__restrict__ votes,
                                                                               float *__restrict__ pooled_out,
                                                                               int32_t *__restrict__ idx_out, int L,
                                                                               int kernel, int K_keep)
{
    __shared__ SelectShared<kSnapOneWgThreads> sh;
    extern __shared__ uint32_t s_keys[];  // L keys
    const long bk = blockIdx.x;
    const float *row = votes + bk * L;
    const int half = kernel / 2;
    for (int p = threadIdx.x; p < L; p += kSnapOneWgThreads) {
        const int lo = (p - half < 0) ? 0 : p - half;
        const int hi = (p + half > L - 1) ? L - 1 : p + half;
        float m = row[lo];
        for (int j = lo + 1; j <= hi; ++j) m = fmaxf(m, row[j]);
        if (pooled_out) pooled_out[bk * L + p] = m;
        s_keys[p] = float_to_key(m);
    }
    __syncthreads();
    if (K_keep <= 0) return;
    int32_t *dst = idx_out + bk * K_keep;
    select_topk_lds<kSnapOneWgThreads>(s_keys, L, K_keep, sh, [dst](int pos, int p) { dst[pos] = p; });
}

static size_t al256s(size_t x) { return (x + 255) & ~(size_t)255; }

struct SnapLayout {
    int n_chunks, R, keys_per_wg;
    size_t off_stats, off_lse, off_votes, off_pooled, off_hist, off_cnt, total;
    int n_slices;
};

static SnapLayout snap_layout(const rs_shape *s, long T, int W)
{
    SnapLayout L;
    const long BK = (long)s->B * s->Hkv;
    L.R = (s->Hq / s->Hkv) * W;
    // keys per workgroup of the two sweeps: 2048, or fewer (a multiple of the 128-key step, at
    // least 256) when that many would leave fewer than about 512 workgroups
    long kpw = (T * BK / 512 + kSnapKT - 1) / kSnapKT * kSnapKT;
    kpw = kpw < 256 ? 256 : kpw > kSnapKeysPerWg ? kSnapKeysPerWg : kpw;
    L.keys_per_wg = (int)kpw;
    L.n_chunks = (int)((T + kpw - 1) / kpw);
    size_t o = RS_WS_CTRL_BYTES;
    L.off_stats = o;
    o += al256s((size_t)BK * L.n_chunks * L.R * 2 * 4);
    L.off_lse = o;
    o += al256s((size_t)BK * L.R * 4);
    L.off_votes = o;
    o += al256s((size_t)BK * (T - W) * 4);
    L.off_pooled = o;
    o += al256s((size_t)BK * (T - W) * 4);
    L.n_slices = (int)((T - W + kSelSlice - 1) / kSelSlice);
    L.off_hist = o;
    o += al256s((size_t)BK * 4 * 256 * 4);
    L.off_cnt = o;
    o += al256s((size_t)BK * L.n_slices * 2 * 4);
    L.total = o;
    return L;
}

size_t snapkv_ws_bytes(const rs_shape *s, long T, int W) { return (T > W) ? snap_layout(s, T, W).total : RS_WS_CTRL_BYTES; }

int snapkv_dispatch(const rs_shape *s, const void *q_win, const void *k_cache, const void *v_cache, long T, int W,
                    int K_keep, int pool_kernel, float scale, void *kc_out, void *vc_out, long Tcap_out,
                    int32_t *idx_out, float *votes_out, const float *lse_in, char *ws, hipStream_t stream)
{
    if (s->dtype != RS_BF16) return RS_UNSUPPORTED;  // the matrix-core path takes bf16 operands
    const SnapLayout Ly = snap_layout(s, T, W);
    const long BK = (long)s->B * s->Hkv;
    const long L = T - W;
    float *stats = (float *)(ws + Ly.off_stats), *lse = (float *)(ws + Ly.off_lse);
    float *votes = (float *)(ws + Ly.off_votes);
    float *pooled = votes_out ? votes_out : (float *)(ws + Ly.off_pooled);
    const dim3 grid((unsigned)Ly.n_chunks, (unsigned)BK);
    const bf16 *qw = (const bf16 *)q_win, *kc = (const bf16 *)k_cache;
    // the rows' log-sum-exp over all visible keys: handed in by the caller (the prefill attention of
    // the window rows has it), or from a first sweep over the keys
    if (lse_in) {
        lse = const_cast<float *>(lse_in);  // [B, Hq, W] is [B * Hkv][G * W]: only read
    } else {
        if (s->D == 128)
            snapkv_stats_kernel<128><<<grid, 256, 0, stream>>>(qw, kc, stats, s->Hq, s->Hkv, T, s->Tcap, W, Ly.n_chunks, scale, Ly.keys_per_wg);
        else
            snapkv_stats_kernel<64><<<grid, 256, 0, stream>>>(qw, kc, stats, s->Hq, s->Hkv, T, s->Tcap, W, Ly.n_chunks, scale, Ly.keys_per_wg);
        const long rows_total = BK * Ly.R;
        snapkv_lse_kernel<<<(unsigned)((rows_total + 3) / 4), 256, 0, stream>>>(stats, lse, Ly.R, Ly.n_chunks, rows_total);
    }
    // votes exist for prefix keys only: chunks that start past the prefix are not needed
    const dim3 grid2((unsigned)((L + Ly.keys_per_wg - 1) / Ly.keys_per_wg), (unsigned)BK);
    if (s->D == 128)
        snapkv_votes_kernel<128><<<grid2, 256, 0, stream>>>(qw, kc, lse, votes, s->Hq, s->Hkv, T, s->Tcap, W, scale, Ly.keys_per_wg);
    else
        snapkv_votes_kernel<64><<<grid2, 256, 0, stream>>>(qw, kc, lse, votes, s->Hq, s->Hkv, T, s->Tcap, W, scale, Ly.keys_per_wg);
    const long tot = BK * L;
    // knob 0: the spread-out selection at any length
    if (L <= kSnapOneWgKeys && knobs().snap_one_wg != 0) {
        snapkv_pool_select_kernel<<<(unsigned)BK, kSnapOneWgThreads, (size_t)L * 4, stream>>>(
            votes, votes_out, idx_out, (int)L, pool_kernel, K_keep);
    } else {
        uint32_t *sel_hist = (uint32_t *)(ws + Ly.off_hist), *sel_cnt = (uint32_t *)(ws + Ly.off_cnt);
        snapkv_pool_kernel<<<(unsigned)((tot + 255) / 256), 256, 0, stream>>>(votes, pooled, L, pool_kernel, tot, sel_hist, BK * 1024);
        if (K_keep > 0) {
            const dim3 gs((unsigned)Ly.n_slices, (unsigned)BK);
            for (int pass = 0; pass < 4; ++pass)
                snapkv_sel_hist_kernel<<<gs, kSelThreads, 0, stream>>>(pooled, sel_hist, L, K_keep, pass);
            snapkv_sel_count_kernel<<<gs, kSelThreads, 0, stream>>>(pooled, sel_hist, sel_cnt, L, K_keep);
            snapkv_sel_emit_kernel<<<gs, kSelThreads, 0, stream>>>(pooled, sel_hist, sel_cnt, idx_out, L, K_keep);
        }
    }
    const int cpr = s->D * 2 / 16;
    const long total = BK * (long)(K_keep + W) * cpr;
    snapkv_gather_kernel<bf16><<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(
        (const bf16 *)k_cache, (const bf16 *)v_cache, idx_out, (bf16 *)kc_out, (bf16 *)vc_out, T, s->Tcap, Tcap_out, W,
        K_keep, s->D, total);
    return hipGetLastError() == hipSuccess ? RS_OK : RS_LAUNCH_FAILED;
}

}  // namespace rs
