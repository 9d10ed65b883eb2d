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
    uint32_t hist[4][256];  // one histogram per radix pass, zeroed once
    int wave_tot[NT / 64];
    int ex_cnt[NT];  // (row, wave) table: greater-than count | equal count << 16
};

// wave64 inclusive prefix sum over ascending lanes, with DPP row shifts and row broadcasts
__device__ __forceinline__ int wave_incl_scan_dpp(int x)
{
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, false);  // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, false);  // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, false);  // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, false);  // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1, 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2, 3
    return x;
}

__device__ __forceinline__ int lanes_below(uint64_t ballot)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

struct NoMark {
    __device__ __forceinline__ void operator()(int) const {}
};

// emit(pos, p): called once per chosen candidate p with its rank pos in ascending order.
// keys: Np keys in LDS.  Requires Np <= 64 * NT.
template <int NT, typename Emit, typename Mark = NoMark>
__device__ void select_topk_lds(const uint32_t *keys, int Np, int K, SelectShared<NT> &sh, Emit emit,
                                Mark mark = Mark())
{
    constexpr int kSelWaves = NT / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int rows = (Np + NT - 1) / NT;
    for (int i = tid; i < 4 * 256; i += NT) (&sh.hist[0][0])[i] = 0u;
    __syncthreads();
    // every wave tracks the digits found so far and the rank still wanted (same in all waves)
    uint32_t prefix = 0u;
    int remaining = K;
#pragma nounroll
    for (int pass = 3; pass >= 0; --pass) {
        uint32_t *hist = sh.hist[pass];
        const int shift = pass * 8;
        const uint32_t himask = (pass == 3) ? 0u : (0xffffffffu << (shift + 8));
        for (int r0 = 0; r0 < rows; r0 += 4) {
            // fetch a batch of keys before touching the histogram (LDS atomics in between would
            // keep each key load waiting for the previous one)
            uint32_t kq[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p = (r0 + j) * NT + tid;
                kq[j] = (p < Np) ? keys[p] : 0u;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p = (r0 + j) * NT + tid;
                const bool in = p < Np && (kq[j] & himask) == prefix;
                const uint32_t bin = (kq[j] >> shift) & 255u;
                if (pass == 3) {
                    // the top bytes of scores are nearly all alike: one atomic per distinct
                    // value in the wave instead of one per key on the same address
                    uint64_t todo = __ballot(in);
                    while (todo) {
                        const int leader = (int)__builtin_ctzll(todo);
                        const uint32_t lb = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
                        const uint64_t same = __ballot(in && bin == lb);
                        if (lane == leader) atomicAdd(&hist[lb], (uint32_t)__popcll(same));
                        todo &= ~same;
                    }
                } else if (in) {
                    atomicAdd(&hist[bin], 1u);
                }
            }
        }
        __syncthreads();
        // lane l owns bins 4(63-l) .. 4(63-l)+3, so a prefix sum over ascending lanes counts
        // the keys in this lane's bins and every higher bin
        const int b0 = 4 * (63 - lane);
        const uint32_t h0 = hist[b0], h1 = hist[b0 + 1], h2 = hist[b0 + 2], h3 = hist[b0 + 3];
        const int own = (int)(h0 + h1 + h2 + h3);
        const int incl = wave_incl_scan_dpp(own);
        const int above = incl - own;
        int bin = 0, rem_new = 0;
        const bool found = above < remaining && remaining <= incl;  // the wanted rank falls in this lane's bins
        if (found) {
            int acc = above;
            bin = b0;
            const uint32_t hh[4] = {h0, h1, h2, h3};
            for (int bb = 3; bb >= 0; --bb) {
                if (acc + (int)hh[bb] >= remaining) {
                    bin = b0 + bb;
                    break;
                }
                acc += (int)hh[bb];
            }
            rem_new = remaining - acc;
        }
        const uint64_t who = __ballot(found);  // exactly one lane
        const int src = (int)__builtin_ctzll(who ? who : 1ull);
        bin = __builtin_amdgcn_readlane(bin, src);
        remaining = __builtin_amdgcn_readlane(rem_new, src);
        prefix |= (uint32_t)bin << shift;
        mark(8 + (3 - pass));
    }
    const uint32_t kth = prefix;   // the K-th largest key
    const int take_eq = remaining;  // how many keys equal to it are taken (lowest indices)

    // Ascending output.  Candidate index = row * NT + wave * 64 + lane, so the order is
    // (row, wave, lane): count per (row, wave) with ballots, scan the table of counts
    // over the workgroup, and rank inside the wave with the ballot bits below the lane.
    for (int r0 = 0; r0 < rows; r0 += 4) {
        uint32_t kq[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int p = (r0 + j) * NT + tid;
            kq[j] = (p < Np) ? keys[p] : 0u;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int p = (r0 + j) * NT + tid;
            const uint64_t bg = __ballot(p < Np && kq[j] > kth);
            const uint64_t be = __ballot(p < Np && kq[j] == kth);
            if (lane == 0 && r0 + j < rows) sh.ex_cnt[(r0 + j) * kSelWaves + wave] = __popcll(bg) | (__popcll(be) << 16);
        }
    }
    __syncthreads();
    {
        const int mine = (tid < rows * kSelWaves) ? sh.ex_cnt[tid] : 0;  // entry (i, w) belongs to thread i * waves + w
        const int incl = wave_incl_scan_dpp(mine);
        if (lane == 63) sh.wave_tot[wave] = incl;
        __syncthreads();
        int before = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w)
            if (w < wave) before += sh.wave_tot[w];
        if (tid < rows * kSelWaves) sh.ex_cnt[tid] = before + incl - mine;
        __syncthreads();
    }
    mark(12);
    for (int r0 = 0; r0 < rows; r0 += 4) {
        uint32_t kq[4];
        int pk[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int p = (r0 + j) * NT + tid;
            kq[j] = (p < Np) ? keys[p] : 0u;
            pk[j] = (r0 + j < rows) ? sh.ex_cnt[(r0 + j) * kSelWaves + wave] : 0;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int p = (r0 + j) * NT + tid;
            const bool is_gt = p < Np && kq[j] > kth, is_eq = p < Np && kq[j] == kth;
            const int gt_lane = lanes_below(__ballot(is_gt)), eq_lane = lanes_below(__ballot(is_eq));
            const int gt_before = pk[j] & 0xffff, eq_before = pk[j] >> 16;
            const int quota = take_eq - eq_before;  // equal keys this wave-row may still take
            if (is_gt || (is_eq && eq_lane < quota)) {
                const int eq_taken_before = (eq_before < take_eq ? eq_before : take_eq) +
                                            (quota > 0 ? (eq_lane < quota ? eq_lane : quota) : 0);
                emit(gt_before + gt_lane + eq_taken_before, p);
            }
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
    // ten loads in flight per thread: 4096 + a few pages of 16 tokens (a 64K context that has grown
    // by some steps) still come in with one round trip
    constexpr int BATCH = 10;
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

// Fold published partials (m, l, o[channel]) of one unit into (M, L, O) for channel `ch`
// (start from M = -inf, L = O = 0, or from the caller's own partial): of the S partials
// those numbered first, first + step, ... (so that several thread groups can share the
// work); words are fetched four splits at a time, stragglers polled.  partial layout per
// split: word 0 = m, word 1 = l, word 2 + c = o[c].
__device__ __forceinline__ void merge_partials(const uint64_t *pu, int S, int stride, int ch, uint32_t tag,
                                               int spin_limit, uint32_t *err, float &M, float &L, float &O,
                                               int first = 0, int step = 1)
{
    for (int s0 = first; s0 < S; s0 += 4 * step) {
        uint64_t wm[4], wl[4], wo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint64_t *p = pu + (long)(s0 + j * step) * stride;
            const bool in = s0 + j * step < S;
            wm[j] = in ? load_u64_agent(p) : 0ull;
            wl[j] = in ? load_u64_agent(p + 1) : 0ull;
            wo[j] = in ? load_u64_agent(p + 2 + ch) : 0ull;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (s0 + j * step < S) {
                const uint64_t *p = pu + (long)(s0 + j * step) * stride;
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
