// Sparse evaluation at prefill (Sec. 2.2, Eq. 4; App. A.1, MoBA paragraph): every query token
// attends, with a float32 softmax, the tokens i <= t of the blocks its routing picked; the
// dense causal path is the same kernel with every block picked.
//
// Queries of one tile pick different KV blocks, but the matrix cores want dense tiles, so the
// work is regrouped by KV block: for each (batch, head, KV block j) the query rows that
// picked j (and do not live in j) are bucketed into a list; tiles of 128 listed rows attend
// block j as a dense [128 x block] problem and leave a partial (lse, o) per (row, slot); the
// rows' own blocks are dense causal tiles of the same kernel, launched afterwards: their
// epilogue folds in the row's partials and writes the output.  Executed flops stay at the algorithmic count (plus tile padding).
//
// Tile kernel, per wave: 32 query rows against 64-key steps with v_mfma_f32_32x32x16_bf16.
// Scores are formed transposed, S^T = K Q^T, so that a lane holds the keys of ONE query and
// the softmax row reductions are in-lane plus one cross-half shuffle; O^T = V^T P^T then
// takes P^T straight from the accumulator registers, and V^T through LDS transpose reads of
// the row-major V tile.  K/V tiles are double-buffered in LDS and filled by direct
// global -> LDS loads (no staging registers): the next tile's loads are issued one at a time
// between the current tile's matrix instructions, one barrier per step.  Tiles are unpadded;
// an XOR permutation of the 16-byte chunks of each row keeps both operand reads conflict-free.
// The softmax runs in the base-2 domain (one FMA + one v_exp_f32 per score), moves its
// reference point (and rescales the accumulators) only when a row maximum has grown by more
// than 2^8, and masks only on steps a boundary crosses.  Partials are kept as bfloat16 o
// (float32 log-sum-exp).  Output rows and partial records pass through LDS on their way out
// and in, so that global memory sees whole 2 D-byte rows.
#include <cstdlib>

#include "common.h"
#include "knobs.h"

#include <type_traits>

namespace rs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kMT = 128;        // query rows per workgroup tile (4 waves x 32)
constexpr int kKT = 64;         // keys per step (two 32-key MFMA sub-tiles)
constexpr uint32_t kSlotShift = 27;
constexpr float kLazy = 8.f;    // slack (base-2 exponent) before the softmax reference point moves

// ------------------------------------------------------------------------------------
// bucketing of (row, slot) pairs by picked block
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prefill_count_kernel(const int32_t *__restrict__ idx, uint32_t *cnt, long T,
                                                            int block, int Nb, int K)
{
    __shared__ uint32_t hist[256];
    const int tid = threadIdx.x;
    const long bh = blockIdx.y;
    hist[tid] = 0u;
    __syncthreads();
    const long t = (long)blockIdx.x * 256 + tid;
    if (t < T) {
        const int own = (int)(t / block);
        const int32_t *row = idx + (bh * T + t) * K;
        for (int k = 0; k < K; ++k) {
            const int j = row[k];
            if (j >= 0 && j < Nb && j != own) atomicAdd(&hist[j], 1u);
        }
    }
    __syncthreads();
    if (tid < Nb && hist[tid]) atomicAdd(&cnt[bh * Nb + tid], hist[tid]);
}

// per (batch, head): list offsets and tile offsets by block; resets the fill cursors
// tile descriptor of the listed-row launch: block, first list entry, rows
struct TileDesc {
    uint32_t j, lbase, lcount, pad;
};

__global__ __launch_bounds__(256) void prefill_scan_kernel(const uint32_t *cnt, uint32_t *off, uint32_t *tile_off,
                                                           uint32_t *cursor, TileDesc *desc, long desc_stride, int Nb)
{
    __shared__ uint32_t s_c[256], s_t[256];
    const int tid = threadIdx.x;
    const long bh = blockIdx.x;
    const uint32_t c = (tid < Nb) ? cnt[bh * Nb + tid] : 0u;
    s_c[tid] = c;
    s_t[tid] = (c + kMT - 1) / kMT;
    __syncthreads();
    if (tid == 0) {
        uint32_t a = 0, b = 0;
        for (int j = 0; j < Nb; ++j) {
            const uint32_t cj = s_c[j], tj = s_t[j];
            s_c[j] = a;
            s_t[j] = b;
            a += cj;
            b += tj;
        }
        off[bh * (Nb + 1) + Nb] = a;
        tile_off[bh * (Nb + 1) + Nb] = b;
    }
    __syncthreads();
    if (tid < Nb) {
        off[bh * (Nb + 1) + tid] = s_c[tid];
        tile_off[bh * (Nb + 1) + tid] = s_t[tid];
        cursor[bh * Nb + tid] = 0u;
        // one descriptor per tile of this block, so a tile workgroup needs a single dependent load
        const uint32_t nt = (c + kMT - 1) / kMT;
        for (uint32_t i = 0; i < nt; ++i) {
            TileDesc d;
            d.j = (uint32_t)tid;
            d.lbase = s_c[tid] + i * kMT;
            d.lcount = (c - i * kMT < (uint32_t)kMT) ? c - i * kMT : (uint32_t)kMT;
            d.pad = 0u;
            desc[bh * desc_stride + s_t[tid] + i] = d;
        }
    }
}

__global__ __launch_bounds__(256) void prefill_fill_kernel(const int32_t *__restrict__ idx, const uint32_t *off,
                                                           uint32_t *cursor, uint32_t *list, long T, int block, int Nb,
                                                           int K, long list_stride)
{
    __shared__ uint32_t hist[256], base[256];
    const int tid = threadIdx.x;
    const long bh = blockIdx.y;
    hist[tid] = 0u;
    __syncthreads();
    const long t = (long)blockIdx.x * 256 + tid;
    const int own = (int)(t / block);
    const int32_t *row = idx + (bh * T + (t < T ? t : 0)) * K;
    if (t < T) {
        for (int k = 0; k < K; ++k) {
            const int j = row[k];
            if (j >= 0 && j < Nb && j != own) atomicAdd(&hist[j], 1u);
        }
    }
    __syncthreads();
    if (tid < Nb) {
        base[tid] = hist[tid] ? atomicAdd(&cursor[bh * Nb + tid], hist[tid]) : 0u;
        hist[tid] = 0u;
    }
    __syncthreads();
    if (t < T) {
        for (int k = 0; k < K; ++k) {
            const int j = row[k];
            if (j >= 0 && j < Nb && j != own) {
                const uint32_t r = atomicAdd(&hist[j], 1u);
                list[bh * list_stride + off[bh * (Nb + 1) + j] + base[j] + r] = (uint32_t)t | ((uint32_t)k << kSlotShift);
            }
        }
    }
}

// ------------------------------------------------------------------------------------
// tile attention
// ------------------------------------------------------------------------------------
struct PrefillParams {
    const bf16 *q, *k_cache, *v_cache;
    const int32_t *idx;        // NULL: dense causal
    const uint32_t *off, *tile_off, *cnt, *list;
    const TileDesc *desc;
    long desc_stride;
    uint16_t *part_o;          // [units][T][K][D] bf16
    float *part_lse;           // [units][T][K]
    bf16 *out;
    float *lse_out;
    int Hq, Hkv, Nb, K, block, n_diag;
    int phase;                 // 0: tiles of listed rows (partials); 1: own-block tiles, fold the partials, write y
    long T, Tcap, list_stride;
    float scale;
};

typedef short s16x4 __attribute__((ext_vector_type(4)));

// LDS transpose read (ds_read_b64_tr_b16): within a group of 16 lanes, lane L supplies the
// address of 4 consecutive 16-bit elements (row L of a 16 x 4 block); lane i receives column
// i % 4 of rows i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12.  With row L pointing at key (L / 4)
// of a key quad and at d offset 4 (L % 4), lane i ends up with V[key 0..3][d0 + i]: a 4-key x
// 16-channel block of row-major V, transposed into the MFMA operand layout.
__device__ __forceinline__ s16x4 lds_read_tr16(const uint16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
}

// MASKED: the routed form for dense routings (small blocks, many picks per row): contiguous
// causal tiles as in the dense case, each lane carrying the bit set of its row's listed blocks
// (nothing is attended that is not listed, the row's own block included);
// a 64-key step lies inside one block (block % 64 == 0), a lane whose row did not list it adds
// nothing there, and a wave none of whose rows listed it skips the step's arithmetic.
template <int D, bool MASKED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_attn_kernel(const PrefillParams a)
{
    constexpr int NC = D / 16;     // 16-wide d chunks of the QK^T contraction
    constexpr int NDT = D / 32;    // 32-wide d tiles of O^T
    constexpr int CR = D / 8;      // 16-byte chunks per row
    constexpr int RW = 64 / CR;    // rows one wave-wide load covers
    constexpr int RPI = 4 * RW;    // rows one pass of the four waves covers
    constexpr int CPT = kKT / RPI; // passes per tile (loads per thread per tile, for K and for V)
    // two K and two V buffers as separate objects, addressed with a compile-time buffer index:
    // the compiler then knows that a step's operand reads and its direct loads into the other
    // buffer cannot overlap, and puts no wait between them
    __shared__ __attribute__((aligned(1024))) uint16_t sK0[kKT * D];
    __shared__ __attribute__((aligned(1024))) uint16_t sK1[kKT * D];
    __shared__ __attribute__((aligned(1024))) uint16_t sV0[kKT * D];
    __shared__ __attribute__((aligned(1024))) uint16_t sV1[kKT * D];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, h = lane >> 5;
    // Workgroups are handed to the eight XCDs round-robin in launch order, and each XCD has an L2
    // of its own.  Launch slot L therefore runs on XCD L % 8; give that XCD whole (batch, head)
    // units (unit % 8 == XCD) and consecutive tiles of one unit, so that the workgroups resident
    // on an XCD stream the same K and V rows at about the same time and share them in its L2.
    int unit = blockIdx.y, xtile = blockIdx.x;
    {
        const unsigned nu = gridDim.y, nt = gridDim.x;
        if (nu % 8 == 0) {
            const unsigned L = blockIdx.y * nt + blockIdx.x;
            const unsigned xcd = L & 7, s = L >> 3;
            unit = (int)(xcd + 8 * (s / nt));
            xtile = (int)(s % nt);
        }
    }
    const int b = unit / a.Hq, hq = unit % a.Hq, kvh = hq / (a.Hq / a.Hkv);
    const bf16 *kb = a.k_cache + (long)(b * a.Hkv + kvh) * a.Tcap * D;
    const bf16 *vb = a.v_cache + (long)(b * a.Hkv + kvh) * a.Tcap * D;

    // ---- which tile is this ----
    bool gathered = false;
    long r0 = 0;            // first row of a contiguous tile
    long kv_begin, kv_end;  // keys visited
    uint32_t lbase = 0, lcount = 0;
    {
        const int x = xtile;
        if (MASKED || a.idx == nullptr) {  // dense causal (or routed by bit sets): heavy tiles first
            const int tile = a.n_diag - 1 - x;
            r0 = (long)tile * kMT;
            kv_begin = 0;
            kv_end = (r0 + kMT < a.T) ? r0 + kMT : a.T;
        } else if (a.phase == 1) {  // rows against their own blocks (causal inside)
            r0 = (long)x * kMT;
            kv_begin = (r0 / a.block) * a.block;
            kv_end = (r0 + kMT < a.T) ? r0 + kMT : a.T;
        } else {
            if ((uint32_t)x >= a.tile_off[(long)unit * (a.Nb + 1) + a.Nb]) return;
            const uint4 dd = *reinterpret_cast<const uint4 *>(a.desc + (long)unit * a.desc_stride + x);
            const int j = (int)dd.x;
            gathered = true;
            lbase = dd.y;
            lcount = dd.z;
            kv_begin = (long)j * a.block;
            kv_end = (kv_begin + a.block < a.T) ? kv_begin + a.block : a.T;
        }
    }

    // ---- staging: global -> LDS, 2 CPT wave-wide loads per tile and wave ----
    // Pass i of a tile: this lane fetches 16 bytes of row RPI i + srow; the wave's four (eight)
    // rows land contiguously.  Rows past kv_end are replaced by the tile's last valid row
    // (finite data; their scores are masked).
    const int srow = wave * RW + lane / CR;
    const int gchunk = (lane % CR) ^ chunk_swizzle<D>(srow);
    auto stage = [&](const bf16 *base, uint16_t *tile, int i, long k0) {
        const int rem = (int)((kv_end - k0 < kKT) ? kv_end - k0 : kKT);  // valid rows, >= 1
        const int r = (i * RPI + srow < rem) ? i * RPI + srow : rem - 1;
        load16_to_lds(lds_source(base + k0 * D), (uint32_t)(r * D + gchunk * 8) * 2u, tile + (i * RPI + wave * RW) * D);
    };
#pragma unroll
    for (int i = 0; i < CPT; ++i) {  // the first tile only needs the block: issue it before the row list is chased
        stage(kb, sK0, i, kv_begin);
        stage(vb, sV0, i, kv_begin);
    }

    // ---- this lane's query (a column of S^T) ----
    const int rq = wave * 32 + lq;
    long tq = -1;
    int slot = 0;
    if (gathered) {
        if ((uint32_t)rq < lcount) {
            const uint32_t e = a.list[(long)unit * a.list_stride + lbase + rq];
            tq = (long)(e & ((1u << kSlotShift) - 1u));
            slot = (int)(e >> kSlotShift);
        }
    } else if (r0 + rq < a.T) {
        tq = r0 + rq;
    }
    const bool causal = !gathered;
    const long own_begin = (!MASKED && a.idx != nullptr && !gathered && tq >= 0) ? (tq / a.block) * a.block : 0;
    // last key any lane of this wave may see (contiguous tiles): later steps are skipped by the wave
    // (a wave none of whose 32 rows exists skips every step; it still stages its share of the tiles)
    const bool wave_live = gathered ? ((uint32_t)(wave * 32) < lcount) : (r0 + wave * 32 < a.T);
    const long wave_last = !wave_live ? -1 : causal ? ((r0 + wave * 32 + 31 < a.T) ? r0 + wave * 32 + 31 : a.T - 1) : kv_end - 1;

    // keys visible to this lane's query, as 32-bit offsets from kv_begin (everything for a padding
    // lane: it never triggers the masking path, its results are dropped)
    int vis_lo = 0, vis_hi = (int)(kv_end - kv_begin) - 1;
    if (causal) {
        vis_lo = (int)(own_begin - kv_begin);
        vis_hi = (tq - kv_begin < vis_hi) ? (int)(tq - kv_begin) : vis_hi;
    }
    if (tq < 0) {
        vis_lo = INT32_MIN / 2;
        vis_hi = INT32_MAX / 2;
    }
    bf16x8 qf[NC];
    {
        const bf16 *qrow = a.q + ((long)unit * a.T + (tq >= 0 ? tq : 0)) * D;
#pragma unroll
        for (int c = 0; c < NC; ++c) qf[c] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * c + 8 * h);
    }

    // ---- routed by bit sets: the blocks this lane's row listed (its own block only if listed) ----
    uint64_t selmask = ~0ull;
    if constexpr (MASKED) {
        selmask = 0ull;
        if (tq >= 0) {
            const int32_t *row = a.idx + ((long)unit * a.T + tq) * a.K;
            for (int kk = 0; kk < a.K; ++kk) {
                const int j = row[kk];
                if (j >= 0 && j < 64) selmask |= 1ull << j;
            }
        }
    }
    // the blocks any row of this wave listed, as a scalar: steps outside it are skipped by the wave
    uint64_t wave_mask = ~0ull;
    if constexpr (MASKED) {
        uint32_t lo = (uint32_t)selmask, hi = (uint32_t)(selmask >> 32);
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            lo |= (uint32_t)__shfl_xor((int)lo, m);
            hi |= (uint32_t)__shfl_xor((int)hi, m);
        }
        wave_mask = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)hi) << 32) |
                    (uint32_t)__builtin_amdgcn_readfirstlane((int)lo);
    }

    // ---- operand addresses inside a tile (elements), fixed per lane ----
    // K operand: row 32 sub + lq, chunk 2 c + h.  V operand through the transpose read: lane =
    // 32 h + 16 dg + L supplies 8 bytes of row 32 sub + 16 c + 4 h + (L >> 2) (+ 8 for the
    // second read) at d = 32 dt + 16 dg + 4 (L & 3).  The swizzle only depends on the row
    // modulo 16, so sub and c enter as plain row offsets.
    const int L = lane & 15, dg = (lane >> 4) & 1;
    uint32_t koff[NC], voff[NDT][2];
    {
        const int sw = chunk_swizzle<D>(lq);
#pragma unroll
        for (int c = 0; c < NC; ++c) koff[c] = (uint32_t)(lq * D + (((2 * c + h) ^ sw) * 8));
        const int rowa = 4 * h + (L >> 2);
#pragma unroll
        for (int ab = 0; ab < 2; ++ab) {
            const int sv = chunk_swizzle<D>(rowa + 8 * ab);
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) {
                const int cg = 4 * dt + 2 * dg + ((L & 3) >> 1);
                voff[dt][ab] = (uint32_t)((rowa + 8 * ab) * D + ((cg ^ sv) * 8) + 4 * (L & 1));
            }
        }
    }

    f32x16 oacc[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
    // running max and sum in the base-2 domain: p = 2^(s * scale * log2(e) - m)
    const float cs = a.scale * 1.4426950408889634f;
    float m = -INFINITY, l = 0.f;

    const int n_steps = (int)((kv_end - kv_begin + kKT - 1) / kKT);
    const int steps_per_block = a.block / kKT;
    int cur_blk = 0, cur_rem = steps_per_block;  // MASKED: kv_begin = 0
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's part of tile 0 is in LDS
    __syncthreads();

    // One step: keys k0 .. k0 + 63 from buffer buf; with NEXT, the tile after it is staged
    // into the other buffer, one load at a time between the matrix instructions (a wave that
    // issues its loads in one burst stalls until the CU's vector memory path has taken them).
    auto step = [&](auto next_tag, auto buf_tag, int it) {
        constexpr bool NEXT = decltype(next_tag)::value;
        constexpr int BUF = decltype(buf_tag)::value;
        const long k0 = kv_begin + (long)it * kKT;
        const uint16_t *cK = BUF ? sK1 : sK0, *cV = BUF ? sV1 : sV0;
        uint16_t *nK = BUF ? sK0 : sK1, *nV = BUF ? sV0 : sV1;
        const long kn = k0 + kKT;

        bool sel = true;
        if constexpr (MASKED) sel = (selmask >> cur_blk) & 1ull;
        if (k0 > wave_last || (MASKED && !((wave_mask >> cur_blk) & 1ull))) {
            if constexpr (NEXT) {
#pragma unroll
                for (int i = 0; i < CPT; ++i) {
                    stage(kb, nK, i, kn);
                    stage(vb, nV, i, kn);
                }
            }
        } else {
            // S^T[key][query] = sum_d K[key][d] Q[query][d], two 32-key sub-tiles; consecutive
            // matrix instructions go to different accumulators (a dependent one issued back to
            // back waits for the previous result)
            // matrix phases run at raised priority: of the two waves that share a SIMD, the one
            // feeding the matrix pipe is issued first and the other's softmax fills the gaps
            __builtin_amdgcn_s_setprio(1);
            f32x16 sacc[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[sub][v] = 0.f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                if constexpr (NEXT) {
                    if (c % (NC / CPT) == 0) stage(kb, nK, c / (NC / CPT), kn);
                }
#pragma unroll
                for (int sub = 0; sub < 2; ++sub) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&cK[32 * sub * D + koff[c]]);
                    sacc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], sacc[sub], 0, 0, 0);
                }
            }
            // issue order for the block above: operand reads run two matrix-instruction pairs
            // ahead of their use, the direct loads go out one at a time in between
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int g = 0; g < NC - 2; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                if (NEXT && g < CPT) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
            // masks only where a boundary crosses this step (uniform over the wave)
            // (all in 32-bit offsets from kv_begin: the lane sees keys vis_lo .. vis_hi)
            __builtin_amdgcn_s_setprio(0);
            const int kr = it * kKT;
            if (__any(kr < vis_lo || kr + kKT - 1 > vis_hi)) {
                const int hi = ((vis_hi - kr > kKT) ? kKT : ((vis_hi - kr < -1) ? -1 : vis_hi - kr)) - 4 * h;
                const int lo = ((vis_lo - kr > kKT) ? kKT : ((vis_lo - kr < -1) ? -1 : vis_lo - kr)) - 4 * h;
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int e = 32 * sub + 8 * (v / 4) + (v % 4);  // + 4 h: folded into lo, hi
                        if (e > hi || e < lo) sacc[sub][v] = -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[sub][v]);
            mx = half_pair_max(mx) * cs;  // cs > 0: scaling commutes with max
            if (MASKED && !sel) mx = -INFINITY;
            // the reference point of the exponentials follows the running maximum lazily: it moves
            // only when the maximum has grown by more than kLazy (p then stays below 2^kLazy,
            // harmless in float32 and bfloat16), so the accumulators are rarely rescaled
            const float m_cand = fmaxf(m, mx);
            const float m_new = (m_cand - m > kLazy) ? m_cand : m;  // -inf -> finite counts as a move
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            if (__any(m_new != m)) {
                const float alpha = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - m_safe);
                l *= alpha;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
                m = m_new;
            }
            float psum = 0.f;
            // a row that did not list this step's block: every exponent is -inf, p = 0
            const float ebias = (MASKED && !sel) ? -INFINITY : -m_safe;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    sacc[sub][v] = __builtin_amdgcn_exp2f(fmaf(sacc[sub][v], cs, ebias));
                    psum += sacc[sub][v];
                }
            l += half_pair_sum(psum);
            __builtin_amdgcn_s_setprio(1);
            // P^T as the B operand: accumulator values 8c .. 8c+7 are this lane's keys
            // 16c + 4h + {0..3} and 16c + 8 + 4h + {0..3}; V^T is read in the same key order
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                bf16x8 pf[2];
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int s8 = 0; s8 < 8; ++s8) pf[c][s8] = (__bf16)sacc[sub][8 * c + s8];
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    if constexpr (NEXT) {
                        if (2 * sub + c < CPT) stage(vb, nV, 2 * sub + c, kn);
                    }
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) {
                        const uint16_t *vq = &cV[(32 * sub + 16 * c) * D];
                        union {
                            s16x4 s[2];
                            bf16x8 f;
                        } vf;
                        vf.s[0] = lds_read_tr16(vq + voff[dt][0]);
                        vf.s[1] = lds_read_tr16(vq + voff[dt][1]);
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.f, pf[c], oacc[dt], 0, 0, 0);
                    }
                }
            }
            // issue order for the P V block: the transposed operand reads (two per matrix
            // instruction) run ahead of their use, the direct loads go out in between
            __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
            for (int g = 0; g < 2 * NDT - 2; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
                if (NEXT && g < CPT) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
            __builtin_amdgcn_s_setprio(0);
        }
        if constexpr (MASKED) {  // block of the next step (wave-uniform counters, no division)
            if (--cur_rem == 0) {
                cur_rem = steps_per_block;
                ++cur_blk;
            }
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

    // ---- epilogue ----
    // Rows leave (and partial records enter) through LDS, so that global memory sees whole rows:
    // a lane that wrote its own row's channels straight from the accumulator layout would touch
    // 64 cache lines per store instruction.  After the last step's barrier the four tile buffers
    // are free; wave w takes buffer w as 64 private rows of D bf16 (two slots of 32 rows), chunks
    // permuted as in the K/V tiles.  Rows are in channel order: the lane of query row lq, half h
    // holds channels 32 dt + 8 g + 4 h + {0..3} in oacc[dt][4 g ..].
    if (!wave_live) return;  // no barrier below
    uint16_t *stg = (wave == 0) ? sK0 : (wave == 1) ? sK1 : (wave == 2) ? sV0 : sV1;
    const int sw_lq = chunk_swizzle<D>(lq);
    const int frow = lane / CR, fchunk = lane % CR;  // flush: RW rows of CR chunks per instruction
    auto put_rows = [&](float sc) __attribute__((always_inline)) {
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 w2;
                w2.x = pack_bf16x2(oacc[dt][4 * g] * sc, oacc[dt][4 * g + 1] * sc);
                w2.y = pack_bf16x2(oacc[dt][4 * g + 2] * sc, oacc[dt][4 * g + 3] * sc);
                *reinterpret_cast<uint2 *>(stg + lq * D + (((4 * dt + g) ^ sw_lq) * 8) + 4 * h) = w2;
            }
    };
    auto flush_rows = [&](auto dest_of_row) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 32 / RW; ++i) {
            const int row = i * RW + frow;
            bf16 *dst = dest_of_row(i, row);
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * D + ((fchunk ^ chunk_swizzle<D>(row)) * 8));
            if (dst) *reinterpret_cast<uint4 *>(dst + fchunk * 8) = v;
        }
    };
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
    const float lse = (l > 0.f) ? (m + __log2f(l)) * 0.6931471805599453f : -INFINITY;
    if (!MASKED && a.idx != nullptr && gathered) {
        // a partial record: the row's normalised output over one listed block as bf16 (channel
        // order), its log-sum-exp as float32 in an array of its own
        uint32_t ent[32 / RW];  // list entries of the rows this lane helps to flush
#pragma unroll
        for (int i = 0; i < 32 / RW; ++i) {
            const uint32_t rr = (uint32_t)(wave * 32 + i * RW + frow);
            ent[i] = (rr < lcount) ? a.list[(long)unit * a.list_stride + lbase + rr] : 0xffffffffu;
        }
        if (tq >= 0 && h == 0) a.part_lse[((long)unit * a.T + tq) * a.K + slot] = lse;
        put_rows(inv);
        flush_rows([&](int i, int) -> bf16 * {
            if (ent[i] == 0xffffffffu) return nullptr;
            const long t_r = (long)(ent[i] & ((1u << kSlotShift) - 1u));
            const int slot_r = (int)(ent[i] >> kSlotShift);
            return reinterpret_cast<bf16 *>(a.part_o) + (((long)unit * a.T + t_r) * a.K + slot_r) * D;
        });
        return;
    }
    const long wrow0 = r0 + wave * 32;  // contiguous tiles: the wave's first row
    float out_scale = inv;
    float out_lse = lse;
    if (!MASKED && a.idx != nullptr) {
        // own-block tile: fold in the partials the listed-row tiles left for this row's other
        // blocks (they ran in the previous launch).  Two slots at a time: their records of the
        // wave's 32 rows come in by row-contiguous direct loads, the lanes then pick their channels.
        const long tqc = (tq >= 0) ? tq : wrow0;  // padding lanes read a valid row and drop the result
        const int own = (int)(tqc / a.block);
        const long rbase = ((long)unit * a.T + tqc) * a.K;
        const int32_t *row = a.idx + rbase;
        bool own_listed = false;
        for (int k = 0; k < a.K; ++k) own_listed = own_listed || (row[k] == own);
        float M = own_listed ? lse : -INFINITY;  // an own block that is not listed does not count
        float wsum = (M == -INFINITY) ? 0.f : 1.f;
        {
            const float w_own = wsum * inv;  // o_own = oacc * inv
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[dt][v] *= w_own;
        }
        const int rows_here = (int)((a.T - wrow0 < 32) ? a.T - wrow0 : 32);  // >= 1
        for (int kc = 0; kc < a.K; kc += 2) {
            float ls[2];
            bool any_valid = false;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int k = kc + i;
                const int jk = (k < a.K) ? row[k] : -1;
                const bool valid = jk >= 0 && jk != own && tq >= 0;
                ls[i] = valid ? a.part_lse[rbase + k] : -INFINITY;
                any_valid = any_valid || valid;
            }
            if (!__any(any_valid)) continue;  // wave-uniform
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int k = (kc + i < a.K) ? kc + i : a.K - 1;
                const LdsSource src = lds_source(reinterpret_cast<const bf16 *>(a.part_o) + (((long)unit * a.T + wrow0) * a.K + k) * D);
#pragma unroll
                for (int j = 0; j < 32 / RW; ++j) {
                    const int rr = j * RW + frow;
                    const int rc = (rr < rows_here) ? rr : rows_here - 1;
                    load16_to_lds(src, (uint32_t)(rc * a.K * D + ((fchunk ^ chunk_swizzle<D>(rr)) * 8)) * 2u,
                                  stg + (i * 32 + j * RW) * D);
                }
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the records are in LDS
            uint2 rc2[2][4 * NDT];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int u = 0; u < 4 * NDT; ++u)
                    rc2[i][u] = *reinterpret_cast<const uint2 *>(stg + (i * 32 + lq) * D + ((u ^ sw_lq) * 8) + 4 * h);
            float Mn = M;
#pragma unroll
            for (int i = 0; i < 2; ++i) Mn = fmaxf(Mn, ls[i]);
            if (Mn != -INFINITY) {
                const float al = (M == -INFINITY) ? 0.f : __expf(M - Mn);
                M = Mn;
                wsum *= al;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[dt][v] *= al;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const float w = (ls[i] == -INFINITY) ? 0.f : __expf(ls[i] - M);
                    wsum += w;
                    if (ls[i] != -INFINITY) {  // a record that was never written may hold anything
#pragma unroll
                        for (int u = 0; u < 4 * NDT; ++u) {
                            const int dt = u >> 2, g = u & 3;
                            oacc[dt][4 * g] = fmaf(w, __uint_as_float(rc2[i][u].x << 16), oacc[dt][4 * g]);
                            oacc[dt][4 * g + 1] = fmaf(w, __uint_as_float(rc2[i][u].x & 0xffff0000u), oacc[dt][4 * g + 1]);
                            oacc[dt][4 * g + 2] = fmaf(w, __uint_as_float(rc2[i][u].y << 16), oacc[dt][4 * g + 2]);
                            oacc[dt][4 * g + 3] = fmaf(w, __uint_as_float(rc2[i][u].y & 0xffff0000u), oacc[dt][4 * g + 3]);
                        }
                    }
                }
            }
        }
        out_scale = (wsum > 0.f) ? 1.f / wsum : 0.f;
        out_lse = (wsum > 0.f) ? M + __logf(wsum) : -INFINITY;
    }
    if (tq >= 0 && h == 0 && a.lse_out) a.lse_out[(long)unit * a.T + tq] = out_lse;
    put_rows(out_scale);
    flush_rows([&](int, int row) -> bf16 * {
        return (wrow0 + row < a.T) ? a.out + ((long)unit * a.T + wrow0 + row) * D : nullptr;
    });
}

__global__ void prefill_zero_kernel(uint32_t *p, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

static size_t al256(size_t x) { return (x + 255) & ~(size_t)255; }

struct PrefillLayout {
    size_t off_cnt, off_off, off_tile, off_cursor, off_list, off_desc, off_part_lse, off_part_o, total;
    long list_stride, desc_stride;
};

static PrefillLayout prefill_layout(const rs_shape *s, long T, int block, int K)
{
    PrefillLayout L;
    const long units = (long)s->B * s->Hq;
    const long Nb = (T + block - 1) / block;
    size_t o = RS_WS_CTRL_BYTES;
    L.off_cnt = o;
    o += al256((size_t)units * Nb * 4);
    L.off_off = o;
    o += al256((size_t)units * (Nb + 1) * 4);
    L.off_tile = o;
    o += al256((size_t)units * (Nb + 1) * 4);
    L.off_cursor = o;
    o += al256((size_t)units * Nb * 4);
    L.list_stride = T * (K > 0 ? K : 0);
    L.off_list = o;
    o += al256((size_t)units * L.list_stride * 4);
    L.desc_stride = (T * (K > 1 ? K - 1 : 0) + kMT - 1) / kMT + Nb;  // upper bound of listed-row tiles per (batch, head)
    L.off_desc = o;
    o += al256((size_t)units * L.desc_stride * sizeof(TileDesc));
    L.off_part_lse = o;
    o += al256((size_t)units * T * (K > 0 ? K : 0) * 4);
    L.off_part_o = o;
    o += al256((size_t)units * T * (K > 0 ? K : 0) * s->D * 2);
    L.total = o;
    return L;
}

size_t prefill_ws_bytes(const rs_shape *s, long T, int block, int K) { return prefill_layout(s, T, block, K).total; }

int prefill_dispatch(const rs_shape *s, const void *q, const void *k_cache, const void *v_cache, long T, int block,
                     float scale, const int32_t *idx, int K, void *out, float *lse_out, char *ws, hipStream_t stream)
{
    if (s->dtype != RS_BF16) return RS_UNSUPPORTED;  // the matrix-core path takes bf16 operands
    const long units = (long)s->B * s->Hq;
    const int Nb = (int)((T + block - 1) / block);
    if (T >= (1L << kSlotShift)) return RS_UNSUPPORTED;
    PrefillParams p;
    p.q = (const bf16 *)q;
    p.k_cache = (const bf16 *)k_cache;
    p.v_cache = (const bf16 *)v_cache;
    p.idx = idx;
    p.out = (bf16 *)out;
    p.lse_out = lse_out;
    p.Hq = s->Hq;
    p.Hkv = s->Hkv;
    p.Nb = Nb;
    p.K = K;
    p.block = block;
    p.n_diag = (int)((T + kMT - 1) / kMT);
    p.T = T;
    p.Tcap = s->Tcap;
    p.scale = scale;
    p.off = p.tile_off = p.cnt = p.list = nullptr;
    p.desc = nullptr;
    p.desc_stride = 0;
    p.part_o = nullptr;
    p.part_lse = nullptr;
    p.list_stride = 0;
    p.phase = 2;
    if (idx && Nb > 256) return RS_UNSUPPORTED;
    // Routings that are dense for their length (small blocks, many picks: the paper's 64- and
    // 128-token blocks with top-8 / top-16 at 4K) run as causal tiles with a bit set per row
    // instead of being regrouped by block.  Regrouped, a row costs (K - 1) listed tiles' worth of
    // steps plus a fixed cost per tile (row list, scattered queries, partial records: about 4.3
    // steps) and the fold (about 9); by bit sets it costs the causal steps of its tile, some
    // skipped.  Measured at 8 x 32 heads x 4096 tokens (regrouped / bit sets / plain causal, ms):
    // blocks of 64: top-16 3.14 / 1.20 / 1.30, top-8 1.75 / 1.16, top-4 0.98 / 1.08;
    // blocks of 128: top-8 1.72 / 1.19, top-4 0.98 / 1.15; 8192 tokens, 128, top-8: 0.92 / 1.03.
    const bool can_mask = idx && Nb <= 64 && block % kKT == 0;
    const double by_sets = 0.85 * (p.n_diag + 4.0), regrouped = (K - 1) * (4.3 + block / 64.0) + 9.0;
    const int masked = can_mask ? knob_or(knobs().prefill_masked, by_sets < regrouped ? 1 : 0) : 0;
    if (masked) {
        const dim3 grid((unsigned)p.n_diag, (unsigned)units);
        if (s->D == 128) prefill_attn_kernel<128, true><<<grid, 256, 0, stream>>>(p);
        else prefill_attn_kernel<64, true><<<grid, 256, 0, stream>>>(p);
        return hipGetLastError() == hipSuccess ? RS_OK : RS_LAUNCH_FAILED;
    }
    if (idx) {
        const PrefillLayout L = prefill_layout(s, T, block, K);
        uint32_t *cnt = (uint32_t *)(ws + L.off_cnt), *off = (uint32_t *)(ws + L.off_off);
        uint32_t *tile_off = (uint32_t *)(ws + L.off_tile), *cursor = (uint32_t *)(ws + L.off_cursor);
        uint32_t *list = (uint32_t *)(ws + L.off_list);
        const long ncnt = units * Nb;
        prefill_zero_kernel<<<(unsigned)((ncnt + 255) / 256), 256, 0, stream>>>(cnt, ncnt);
        const dim3 gr((unsigned)((T + 255) / 256), (unsigned)units);
        prefill_count_kernel<<<gr, 256, 0, stream>>>(idx, cnt, T, block, Nb, K);
        TileDesc *desc = (TileDesc *)(ws + L.off_desc);
        prefill_scan_kernel<<<(unsigned)units, 256, 0, stream>>>(cnt, off, tile_off, cursor, desc, L.desc_stride, Nb);
        prefill_fill_kernel<<<gr, 256, 0, stream>>>(idx, off, cursor, list, T, block, Nb, K, L.list_stride);
        p.off = off;
        p.tile_off = tile_off;
        p.cnt = cnt;
        p.list = list;
        p.desc = desc;
        p.desc_stride = L.desc_stride;
        p.part_o = (uint16_t *)(ws + L.off_part_o);
        p.part_lse = (float *)(ws + L.off_part_lse);
        p.list_stride = L.list_stride;
    }
    if (idx) {
        // launch 1: tiles of listed rows leave partials; launch 2: own-block tiles fold them in
        const long gathered_tiles = p.desc_stride;  // upper bound per (batch, head)
        p.phase = 0;
        const dim3 g0((unsigned)gathered_tiles, (unsigned)units);
        if (K > 1) {
            if (s->D == 128) prefill_attn_kernel<128, false><<<g0, 256, 0, stream>>>(p);
            else prefill_attn_kernel<64, false><<<g0, 256, 0, stream>>>(p);
        }
        p.phase = 1;
    }
    const dim3 grid((unsigned)p.n_diag, (unsigned)units);
    if (s->D == 128) prefill_attn_kernel<128, false><<<grid, 256, 0, stream>>>(p);
    else prefill_attn_kernel<64, false><<<grid, 256, 0, stream>>>(p);
    return hipGetLastError() == hipSuccess ? RS_OK : RS_LAUNCH_FAILED;
}

}  // namespace rs
