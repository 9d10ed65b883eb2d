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
// the row-major V tile.  K/V tiles are double-buffered in LDS: the next tile's global loads
// are issued before the current tile's math and stored after it, one barrier per step.
// The softmax runs in the base-2 domain (one FMA + one v_exp_f32 per score), rescales the
// accumulators only when a row maximum moved, and masks only on steps a boundary crosses.
#include "common.h"

namespace rs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kMT = 128;        // query rows per workgroup tile (4 waves x 32)
constexpr int kKT = 64;         // keys per step (two 32-key MFMA sub-tiles)
constexpr int kPartStride = 4;  // floats before o in a partial record: [lse, -, -, -, o[D]]
constexpr uint32_t kSlotShift = 27;

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
__global__ __launch_bounds__(256) void prefill_scan_kernel(const uint32_t *cnt, uint32_t *off, uint32_t *tile_off,
                                                           uint32_t *cursor, int Nb)
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
    float *partial;            // [units][T][K][kPartStride + D]
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

template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_attn_kernel(const PrefillParams a)
{
    constexpr int NC = D / 16;   // 16-wide d chunks of the QK^T contraction
    constexpr int NDT = D / 32;  // 32-wide d tiles of O^T
    constexpr int LS = D + 16;   // LDS row stride (bf16): rows 8 banks apart, conflict-free transpose reads
    constexpr int CPT = kKT * D / 8 / 256;  // 16-byte chunks per thread per tile
    __shared__ __attribute__((aligned(16))) uint16_t sK[2][kKT * LS];
    __shared__ __attribute__((aligned(16))) uint16_t sV[2][kKT * LS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, h = lane >> 5;
    const int unit = blockIdx.y;
    const int b = unit / a.Hq, hq = unit % a.Hq, kvh = hq / (a.Hq / a.Hkv);
    const bf16 *kb = a.k_cache + (long)(b * a.Hkv + kvh) * a.Tcap * D;
    const bf16 *vb = a.v_cache + (long)(b * a.Hkv + kvh) * a.Tcap * D;

    // ---- which tile is this ----
    bool gathered = false;
    long r0 = 0;            // first row of a contiguous tile
    long kv_begin, kv_end;  // keys visited
    uint32_t lbase = 0, lcount = 0;
    {
        int x = blockIdx.x;
        if (a.idx == nullptr) {  // dense causal: heavy tiles first
            const int tile = a.n_diag - 1 - x;
            r0 = (long)tile * kMT;
            kv_begin = 0;
            kv_end = (r0 + kMT < a.T) ? r0 + kMT : a.T;
        } else if (a.phase == 1) {  // rows against their own blocks (causal inside)
            r0 = (long)x * kMT;
            kv_begin = (r0 / a.block) * a.block;
            kv_end = (r0 + kMT < a.T) ? r0 + kMT : a.T;
        } else {
            const uint32_t *to = a.tile_off + (long)unit * (a.Nb + 1);
            if ((uint32_t)x >= to[a.Nb]) return;
            int lo = 0, hi = a.Nb;  // largest j with to[j] <= x
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (to[mid] <= (uint32_t)x) lo = mid;
                else hi = mid;
            }
            const int j = lo;
            gathered = true;
            const uint32_t first = ((uint32_t)x - to[j]) * kMT;
            lbase = a.off[(long)unit * (a.Nb + 1) + j] + first;
            const uint32_t cj = a.cnt[(long)unit * a.Nb + j];
            lcount = (cj - first < (uint32_t)kMT) ? cj - first : (uint32_t)kMT;
            kv_begin = (long)j * a.block;
            kv_end = (kv_begin + a.block < a.T) ? kv_begin + a.block : a.T;
        }
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
    const long own_begin = (a.idx != nullptr && !gathered && tq >= 0) ? (tq / a.block) * a.block : 0;
    // last key any lane of this wave may see (contiguous tiles): later steps are skipped by the wave
    const long wave_last = causal ? ((r0 + wave * 32 + 31 < a.T) ? r0 + wave * 32 + 31 : a.T - 1) : kv_end - 1;

    bf16x8 qf[NC];
    {
        const bf16 *qrow = a.q + ((long)unit * a.T + (tq >= 0 ? tq : 0)) * D;
#pragma unroll
        for (int c = 0; c < NC; ++c) qf[c] = *reinterpret_cast<const bf16x8 *>(qrow + 16 * c + 8 * h);
    }

    f32x16 oacc[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
    // running max and sum in the base-2 domain: p = 2^(s * scale * log2(e) - m)
    const float cs = a.scale * 1.4426950408889634f;
    float m = -INFINITY, l = 0.f;

    // global -> registers -> LDS staging of one K/V tile (rows past kv_end are zero)
    uint4 kst[CPT], vst[CPT];
    auto fetch = [&](long k0) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int ch = i * 256 + tid;
            const int key = ch / (D / 8), d0 = (ch % (D / 8)) * 8;
            kst[i] = make_uint4(0u, 0u, 0u, 0u);
            vst[i] = kst[i];
            if (k0 + key < kv_end) {
                kst[i] = *reinterpret_cast<const uint4 *>(kb + (k0 + key) * D + d0);
                vst[i] = *reinterpret_cast<const uint4 *>(vb + (k0 + key) * D + d0);
            }
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int ch = i * 256 + tid;
            const int key = ch / (D / 8), d0 = (ch % (D / 8)) * 8;
            *reinterpret_cast<uint4 *>(&sK[buf][key * LS + d0]) = kst[i];
            *reinterpret_cast<uint4 *>(&sV[buf][key * LS + d0]) = vst[i];
        }
    };

    const int n_steps = (int)((kv_end - kv_begin + kKT - 1) / kKT);
    fetch(kv_begin);
    stash(0);
    __syncthreads();
    // lane decomposition for the transpose reads: lane = 32 h + 16 dg + L
    const int L = lane & 15, dg = (lane >> 4) & 1;

    for (int it = 0; it < n_steps; ++it) {
        const long k0 = kv_begin + (long)it * kKT;
        const int buf = it & 1;
        if (it + 1 < n_steps) fetch(k0 + kKT);  // next tile's loads fly during this tile's math

        if (k0 <= wave_last) {
            // S^T[key][query] = sum_d K[key][d] Q[query][d], two 32-key sub-tiles
            f32x16 sacc[2];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[sub][v] = 0.f;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&sK[buf][(32 * sub + lq) * LS + 16 * c + 8 * h]);
                    sacc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], sacc[sub], 0, 0, 0);
                }
            }
            // masks only where a boundary crosses this step (uniform over the wave)
            const bool lane_edge = (k0 + kKT > kv_end) || (causal && (k0 + kKT - 1 > tq || k0 < own_begin));
            if (__any(lane_edge && tq >= 0)) {
#pragma unroll
                for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const long key = k0 + 32 * sub + 8 * (v / 4) + 4 * h + (v % 4);
                        bool ok = key < kv_end;
                        if (causal) ok = ok && (key <= tq) && (key >= own_begin);
                        if (!ok) sacc[sub][v] = -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[sub][v]);
            mx = fmaxf(mx, shfl_xor_f(mx, 32)) * cs;  // cs > 0: scaling commutes with max
            const float m_new = fmaxf(m, mx);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            if (__any(m_new != m)) {  // rescale only when some row's maximum moved
                const float alpha = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - m_safe);
                l *= alpha;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
                m = m_new;
            }
            float psum = 0.f;
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    sacc[sub][v] = __builtin_amdgcn_exp2f(fmaf(sacc[sub][v], cs, -m_safe));
                    psum += sacc[sub][v];
                }
            psum += shfl_xor_f(psum, 32);
            l += psum;
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
                for (int dt = 0; dt < NDT; ++dt) {
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const uint16_t *vq = &sV[buf][(32 * sub + 16 * c + 4 * h + (L >> 2)) * LS + 32 * dt + 16 * dg + 4 * (L & 3)];
                        union {
                            s16x4 s[2];
                            bf16x8 f;
                        } vf;
                        vf.s[0] = lds_read_tr16(vq);
                        vf.s[1] = lds_read_tr16(vq + 8 * LS);
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.f, pf[c], oacc[dt], 0, 0, 0);
                    }
                }
            }
        }
        if (it + 1 < n_steps) stash(buf ^ 1);
        __syncthreads();
    }

    if (tq < 0) return;
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
    const float lse = (l > 0.f) ? (m + __log2f(l)) * 0.6931471805599453f : -INFINITY;
    if (a.idx != nullptr && gathered) {
        float *rec = a.partial + (((long)unit * a.T + tq) * a.K + slot) * (kPartStride + D);
        if (h == 0) rec[0] = lse;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * dt + 8 * g + 4 * h;
                *reinterpret_cast<float4 *>(rec + kPartStride + d) =
                    make_float4(oacc[dt][4 * g] * inv, oacc[dt][4 * g + 1] * inv, oacc[dt][4 * g + 2] * inv,
                                oacc[dt][4 * g + 3] * inv);
            }
    } else if (a.idx != nullptr) {
        // own-block tile: fold in the partials the listed-row tiles left for this row's other
        // blocks (they ran in the previous launch) and write the final output
        const int own = (int)(tq / a.block);
        const int32_t *row = a.idx + ((long)unit * a.T + tq) * a.K;
        const float *rec0 = a.partial + ((long)unit * a.T + tq) * a.K * (kPartStride + D);
        bool own_listed = false;
        for (int k = 0; k < a.K; ++k) own_listed = own_listed || (row[k] == own);
        const float lse_own = own_listed ? lse : -INFINITY;  // an own block that is not listed does not count
        float M = lse_own;
        for (int k = 0; k < a.K; ++k)
            if (row[k] >= 0 && row[k] != own) M = fmaxf(M, rec0[(long)k * (kPartStride + D)]);
        float wsum = (lse_own == -INFINITY) ? 0.f : __expf(lse_own - M);
        const float w_own = wsum * inv;  // o_own = oacc * inv
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[dt][v] *= w_own;
        for (int k = 0; k < a.K; ++k) {
            if (row[k] < 0 || row[k] == own) continue;
            const float *rk = rec0 + (long)k * (kPartStride + D);
            const float w = (rk[0] == -INFINITY) ? 0.f : __expf(rk[0] - M);
            wsum += w;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 o4 = *reinterpret_cast<const float4 *>(rk + kPartStride + 32 * dt + 8 * g + 4 * h);
                    oacc[dt][4 * g] = fmaf(w, o4.x, oacc[dt][4 * g]);
                    oacc[dt][4 * g + 1] = fmaf(w, o4.y, oacc[dt][4 * g + 1]);
                    oacc[dt][4 * g + 2] = fmaf(w, o4.z, oacc[dt][4 * g + 2]);
                    oacc[dt][4 * g + 3] = fmaf(w, o4.w, oacc[dt][4 * g + 3]);
                }
        }
        const float winv = (wsum > 0.f) ? 1.f / wsum : 0.f;
        bf16 *orow = a.out + ((long)unit * a.T + tq) * D;
        if (h == 0 && a.lse_out) a.lse_out[(long)unit * a.T + tq] = (wsum > 0.f) ? M + __logf(wsum) : -INFINITY;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * dt + 8 * g + 4 * h;
                uint2 w2;
                w2.x = f32_to_bf16_bits(oacc[dt][4 * g] * winv) | (f32_to_bf16_bits(oacc[dt][4 * g + 1] * winv) << 16);
                w2.y = f32_to_bf16_bits(oacc[dt][4 * g + 2] * winv) | (f32_to_bf16_bits(oacc[dt][4 * g + 3] * winv) << 16);
                *reinterpret_cast<uint2 *>(orow + d) = w2;
            }
    } else {
        bf16 *orow = a.out + ((long)unit * a.T + tq) * D;
        if (h == 0 && a.lse_out) a.lse_out[(long)unit * a.T + tq] = lse;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int d = 32 * dt + 8 * g + 4 * h;
                uint2 w;
                w.x = f32_to_bf16_bits(oacc[dt][4 * g] * inv) | (f32_to_bf16_bits(oacc[dt][4 * g + 1] * inv) << 16);
                w.y = f32_to_bf16_bits(oacc[dt][4 * g + 2] * inv) | (f32_to_bf16_bits(oacc[dt][4 * g + 3] * inv) << 16);
                *reinterpret_cast<uint2 *>(orow + d) = w;
            }
    }
}

__global__ void prefill_zero_kernel(uint32_t *p, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

static size_t al256(size_t x) { return (x + 255) & ~(size_t)255; }

struct PrefillLayout {
    size_t off_cnt, off_off, off_tile, off_cursor, off_list, off_partial, total;
    long list_stride;
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
    L.off_partial = o;
    o += al256((size_t)units * T * (K > 0 ? K : 0) * (kPartStride + s->D) * 4);
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
    p.partial = nullptr;
    p.list_stride = 0;
    p.phase = 2;
    if (idx) {
        if (Nb > 256) return RS_UNSUPPORTED;
        const PrefillLayout L = prefill_layout(s, T, block, K);
        uint32_t *cnt = (uint32_t *)(ws + L.off_cnt), *off = (uint32_t *)(ws + L.off_off);
        uint32_t *tile_off = (uint32_t *)(ws + L.off_tile), *cursor = (uint32_t *)(ws + L.off_cursor);
        uint32_t *list = (uint32_t *)(ws + L.off_list);
        const long ncnt = units * Nb;
        prefill_zero_kernel<<<(unsigned)((ncnt + 255) / 256), 256, 0, stream>>>(cnt, ncnt);
        const dim3 gr((unsigned)((T + 255) / 256), (unsigned)units);
        prefill_count_kernel<<<gr, 256, 0, stream>>>(idx, cnt, T, block, Nb, K);
        prefill_scan_kernel<<<(unsigned)units, 256, 0, stream>>>(cnt, off, tile_off, cursor, Nb);
        prefill_fill_kernel<<<gr, 256, 0, stream>>>(idx, off, cursor, list, T, block, Nb, K, L.list_stride);
        p.off = off;
        p.tile_off = tile_off;
        p.cnt = cnt;
        p.list = list;
        p.partial = (float *)(ws + L.off_partial);
        p.list_stride = L.list_stride;
    }
    if (idx) {
        // launch 1: tiles of listed rows leave partials; launch 2: own-block tiles fold them in
        const long gathered_tiles = (T * (K > 1 ? K - 1 : 0) + kMT - 1) / kMT + Nb;  // upper bound per (batch, head)
        p.phase = 0;
        const dim3 g0((unsigned)gathered_tiles, (unsigned)units);
        if (K > 1) {
            if (s->D == 128) prefill_attn_kernel<128><<<g0, 256, 0, stream>>>(p);
            else prefill_attn_kernel<64><<<g0, 256, 0, stream>>>(p);
        }
        p.phase = 1;
    }
    const dim3 grid((unsigned)p.n_diag, (unsigned)units);
    if (s->D == 128) prefill_attn_kernel<128><<<grid, 256, 0, stream>>>(p);
    else prefill_attn_kernel<64><<<grid, 256, 0, stream>>>(p);
    return hipGetLastError() == hipSuccess ? RS_OK : RS_LAUNCH_FAILED;
}

}  // namespace rs
