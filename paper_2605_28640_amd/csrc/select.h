// Fence-free cross-workgroup hand-off (tagged words) and the register-resident top-K
// selection shared by the decode kernels.
#pragma once

#include "common.h"

namespace rs {

// ------------------------------------------------------------------------------------
// Cross-workgroup hand-off without cache flushes.  Values that another workgroup must
// read within the same launch (page scores, split partials) are published as 64-bit
// words {tag : value} with agent-scope write-through stores; the reader polls each word
// with agent-scope loads until it carries the call's tag.  A word is its own validity
// flag, so no fence (and no L2 write-back / invalidate) is needed.  An arrival counter
// only elects the reader.  Waits are bounded; expiry is recorded in the workspace.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ void publish_f32(uint64_t *p, float v, uint32_t tag)
{
    store_u64_agent(p, ((uint64_t)tag << 32) | __float_as_uint(v));
}

__device__ __forceinline__ float acquire_f32(const uint64_t *p, uint32_t tag, int spin_limit, uint32_t *err)
{
    uint64_t w = load_u64_agent(p);
    int spins = 0;
    while ((uint32_t)(w >> 32) != tag) {
        if (++spins > spin_limit) {
            atomicExch(err, 1u);
            break;
        }
        __builtin_amdgcn_s_sleep(1);
        w = load_u64_agent(p);
    }
    return __uint_as_float((uint32_t)w);
}

// ------------------------------------------------------------------------------------
// top-K of up to 64*NT keys held in LDS by an NT-thread workgroup; thread t handles
// candidates t, t+NT, t+2NT, ...  Radix select (4 passes of 8 bits) finds the K-th
// largest key; every key above it is taken, and of the keys equal to it the lowest
// indices; the result is written in ascending index order.
// ------------------------------------------------------------------------------------
template <int NT>
struct SelectShared {
    uint32_t hist[256];
    int wave_tot[2][NT / 64];
    int ex_gt[NT], ex_eq[NT];  // exclusive counts before (row, wave)
    uint32_t prefix;
    int remaining;
};

// exclusive prefix over the workgroup of (x, y)
template <int NT>
__device__ __forceinline__ void block_exclusive_scan2(int x, int y, int &ex, int &ey, SelectShared<NT> &sh)
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
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        if (w < wave) {
            bx += sh.wave_tot[0][w];
            by += sh.wave_tot[1][w];
        }
    }
    ex = bx + ix - x;
    ey = by + iy - y;
}

__device__ __forceinline__ int lanes_below(uint64_t ballot)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

// emit(pos, p): called once per chosen candidate p with its rank pos in ascending order.
// keys: Np keys in LDS.  Requires Np <= 64 * NT.
template <int NT, typename Emit>
__device__ void select_topk_lds(const uint32_t *keys, int Np, int K, SelectShared<NT> &sh, Emit emit)
{
    constexpr int kSelWaves = NT / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int rows = (Np + NT - 1) / NT;
    if (tid == 0) {
        sh.prefix = 0u;
        sh.remaining = K;
    }
#pragma nounroll
    for (int pass = 3; pass >= 0; --pass) {
        if (tid < 256) sh.hist[tid] = 0u;
        __syncthreads();
        const uint32_t prefix = sh.prefix;
        const int shift = pass * 8;
        const uint32_t himask = (pass == 3) ? 0u : (0xffffffffu << (shift + 8));
        // run-length combine equal bins of successive keys: the top bytes of scores are
        // nearly all alike, which would serialise one LDS atomic per key
        int run_bin = -1, run_cnt = 0;
#pragma unroll 4
        for (int p = tid; p < Np; p += NT) {
            const uint32_t key = keys[p];
            const int bin = ((key & himask) == prefix) ? (int)((key >> shift) & 255u) : -1;
            if (bin != run_bin) {
                if (run_bin >= 0) atomicAdd(&sh.hist[run_bin], (uint32_t)run_cnt);
                run_bin = bin;
                run_cnt = 0;
            }
            ++run_cnt;
        }
        if (run_bin >= 0) atomicAdd(&sh.hist[run_bin], (uint32_t)run_cnt);
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
                int bin = tid * 4;
                const uint32_t hh[4] = {h0, h1, h2, h3};
                for (int bb = 3; bb >= 0; --bb) {
                    if (acc + (int)hh[bb] >= rem) {
                        bin = tid * 4 + bb;
                        break;
                    }
                    acc += (int)hh[bb];
                }
                sh.prefix = prefix | ((uint32_t)bin << shift);
                sh.remaining = rem - acc;
            }
        }
        __syncthreads();
    }
    const uint32_t kth = sh.prefix;    // the K-th largest key
    const int take_eq = sh.remaining;  // how many keys equal to it are taken (lowest indices)

    // Ascending output.  Candidate index = row * NT + wave * 64 + lane, so the order is
    // (row, wave, lane): count per (row, wave) with ballots, scan the table of counts
    // over the workgroup, and rank inside the wave with the ballot bits below the lane.
    for (int i = 0; i < rows; ++i) {
        const int p = i * NT + tid;
        const uint32_t key = (p < Np) ? keys[p] : 0u;
        const uint64_t bg = __ballot(p < Np && key > kth);
        const uint64_t be = __ballot(p < Np && key == kth);
        if (lane == 0) {  // entry (i, w) of the table belongs to thread i * kSelWaves + w
            sh.ex_gt[i * kSelWaves + wave] = __popcll(bg);
            sh.ex_eq[i * kSelWaves + wave] = __popcll(be);
        }
    }
    __syncthreads();
    int my_gt = 0, my_eq = 0;
    if (tid < rows * kSelWaves) {
        my_gt = sh.ex_gt[tid];
        my_eq = sh.ex_eq[tid];
    }
    int e_gt, e_eq;
    block_exclusive_scan2<NT>(my_gt, my_eq, e_gt, e_eq, sh);
    if (tid < rows * kSelWaves) {
        sh.ex_gt[tid] = e_gt;
        sh.ex_eq[tid] = e_eq;
    }
    __syncthreads();
    for (int i = 0; i < rows; ++i) {
        const int p = i * NT + tid;
        const uint32_t key = (p < Np) ? keys[p] : 0u;
        const bool is_gt = p < Np && key > kth, is_eq = p < Np && key == kth;
        const int gt_lane = lanes_below(__ballot(is_gt)), eq_lane = lanes_below(__ballot(is_eq));
        const int gt_before = sh.ex_gt[i * kSelWaves + wave];
        const int eq_before = sh.ex_eq[i * kSelWaves + wave];
        const int quota = take_eq - eq_before;  // equal keys this wave-row may still take
        if (is_gt || (is_eq && eq_lane < quota)) {
            const int eq_taken_before = (eq_before < take_eq ? eq_before : take_eq) +
                                        (quota > 0 ? (eq_lane < quota ? eq_lane : quota) : 0);
            emit(gt_before + gt_lane + eq_taken_before, p);
        }
    }
}

// Read the Np tagged scores of a unit into keys in LDS, a few loads in flight at a time;
// always-kept pages get the top key.  Ends with a workgroup barrier.
template <int NT>
__device__ __forceinline__ void gather_page_keys(const uint64_t *srow, int Np, int n_first, int n_local,
                                                 uint32_t tag, int spin_limit, uint32_t *err, float *scores_out,
                                                 uint32_t *keys)
{
    constexpr int BATCH = 8;
    const int tid = threadIdx.x;
    for (int p0 = tid; p0 < Np; p0 += BATCH * NT) {
        uint64_t wd[BATCH];
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            const int p = p0 + j * NT;
            wd[j] = (p < Np) ? load_u64_agent(&srow[p]) : 0ull;
        }
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            const int p = p0 + j * NT;
            if (p < Np) {
                float sc = __uint_as_float((uint32_t)wd[j]);
                if ((uint32_t)(wd[j] >> 32) != tag) sc = acquire_f32(&srow[p], tag, spin_limit, err);
                if (scores_out) scores_out[p] = sc;
                keys[p] = (p < n_first || p >= Np - n_local) ? 0xffffffffu : float_to_key(sc);
            }
        }
    }
    __syncthreads();
}

// Fold S published partials (m, l, o[channel]) of one unit into (M, L, O) for channel `ch`
// (start from M = -inf, L = O = 0, or from the caller's own partial): words are fetched
// four splits at a time, stragglers polled.  partial layout per split: word 0 = m,
// word 1 = l, word 2 + c = o[c].
__device__ __forceinline__ void merge_partials(const uint64_t *pu, int S, int stride, int ch, uint32_t tag,
                                               int spin_limit, uint32_t *err, float &M, float &L, float &O)
{
    for (int s0 = 0; s0 < S; s0 += 4) {
        uint64_t wm[4], wl[4], wo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint64_t *p = pu + (long)(s0 + j) * stride;
            const bool in = s0 + j < S;
            wm[j] = in ? load_u64_agent(p) : 0ull;
            wl[j] = in ? load_u64_agent(p + 1) : 0ull;
            wo[j] = in ? load_u64_agent(p + 2 + ch) : 0ull;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (s0 + j < S) {
                const uint64_t *p = pu + (long)(s0 + j) * stride;
                float ms = __uint_as_float((uint32_t)wm[j]), ls = __uint_as_float((uint32_t)wl[j]),
                      os = __uint_as_float((uint32_t)wo[j]);
                if ((uint32_t)(wm[j] >> 32) != tag) ms = acquire_f32(p, tag, spin_limit, err);
                if ((uint32_t)(wl[j] >> 32) != tag) ls = acquire_f32(p + 1, tag, spin_limit, err);
                if ((uint32_t)(wo[j] >> 32) != tag) os = acquire_f32(p + 2 + ch, tag, spin_limit, err);
                const float mn = fmaxf(M, ms);
                const float a1 = (M == -INFINITY) ? 0.f : __expf(M - mn);
                const float a2 = (ms == -INFINITY) ? 0.f : __expf(ms - mn);
                L = L * a1 + ls * a2;
                O = O * a1 + os * a2;
                M = mn;
            }
        }
    }
}

}  // namespace rs
