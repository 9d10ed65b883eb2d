// Sparse evaluation at prefill (Sec. 2.2, Eq. 4; App. A.1, MoBA paragraph): every query token
// attends, with a float32 softmax, the tokens i <= t of the blocks its routing picked; the
// dense causal path is the same kernel with every block picked.
//
// Queries of one tile pick different KV blocks, but the matrix cores want dense tiles, so the
// work is regrouped by KV block: for each (batch, head, KV block j) the query rows that
// picked j (and do not live in j) are bucketed into a list; tiles of 128 listed rows attend
// block j as a dense [128 x block] problem and leave a partial (lse, o) per (row, slot); the
// rows' own blocks are dense causal tiles of the same kernel; a last pass merges each row's
// partials.  Executed flops stay at the algorithmic count (plus tile padding).
//
// Tile kernel, per wave: 32 query rows against 32-key tiles with v_mfma_f32_32x32x16_bf16.
// Scores are formed transposed, S^T = K Q^T, so that a lane holds 16 keys of ONE query and
// the softmax row reductions are in-lane plus one cross-half shuffle; O^T = V^T P^T then
// takes P^T straight from the accumulator registers, and V^T from an LDS tile stored
// transposed.
#include "common.h"

namespace rs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kMT = 128;        // query rows per workgroup tile (4 waves x 32)
constexpr int kKT = 32;         // keys per step
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
    long T, Tcap, list_stride;
    float scale;
};

template <int D>
__global__ __launch_bounds__(256) void prefill_attn_kernel(const PrefillParams a)
{
    constexpr int NC = D / 16;   // 16-wide d chunks of the QK^T contraction
    constexpr int NDT = D / 32;  // 32-wide d tiles of O^T
    constexpr int KS = D + 8;    // LDS row stride of the K tile (bf16)
    constexpr int VS = kKT + 8;  // LDS row stride of the transposed V tile (bf16)
    __shared__ __attribute__((aligned(16))) uint16_t sK[kKT * KS];
    __shared__ __attribute__((aligned(16))) uint16_t sVt[D * VS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lq = lane & 31, h = lane >> 5;
    const int unit = blockIdx.y;
    const int b = unit / a.Hq, hq = unit % a.Hq, kvh = hq / (a.Hq / a.Hkv);
    const bf16 *kb = a.k_cache + (long)(b * a.Hkv + kvh) * a.Tcap * D;
    const bf16 *vb = a.v_cache + (long)(b * a.Hkv + kvh) * a.Tcap * D;

    // ---- which tile is this ----
    bool gathered = false;
    long r0 = 0;           // first row of a contiguous tile
    long kv_begin, kv_end;  // keys visited
    uint32_t lbase = 0, lcount = 0;
    {
        int x = blockIdx.x;
        if (a.idx == nullptr) {  // dense causal: heavy tiles first
            const int tile = a.n_diag - 1 - x;
            r0 = (long)tile * kMT;
            kv_begin = 0;
            kv_end = (r0 + kMT < a.T) ? r0 + kMT : a.T;
        } else if (x < a.n_diag) {  // rows against their own blocks (causal inside)
            r0 = (long)x * kMT;
            kv_begin = (r0 / a.block) * a.block;
            kv_end = (r0 + kMT < a.T) ? r0 + kMT : a.T;
        } else {
            x -= a.n_diag;
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
    float m = -INFINITY, l = 0.f;

    // keys this wave needs: contiguous tiles stop at their last row
    for (long k0 = kv_begin; k0 < kv_end; k0 += kKT) {
        __syncthreads();  // previous step's LDS reads are done
        // cooperative load: K tile as is, V tile transposed; rows past kv_end are zero
        constexpr int CHUNKS = kKT * D / 8;  // 16-byte chunks per tile
#pragma unroll
        for (int i = 0; i < CHUNKS / 256; ++i) {
            const int ch = i * 256 + tid;
            const int key = ch / (D / 8), d0 = (ch % (D / 8)) * 8;
            uint4 kk = make_uint4(0u, 0u, 0u, 0u), vv = kk;
            if (k0 + key < kv_end) {
                kk = *reinterpret_cast<const uint4 *>(kb + (k0 + key) * D + d0);
                vv = *reinterpret_cast<const uint4 *>(vb + (k0 + key) * D + d0);
            }
            *reinterpret_cast<uint4 *>(&sK[key * KS + d0]) = kk;
            const uint32_t w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sVt[(d0 + 2 * e) * VS + key] = (uint16_t)(w[e] & 0xffffu);
                sVt[(d0 + 2 * e + 1) * VS + key] = (uint16_t)(w[e] >> 16);
            }
        }
        __syncthreads();

        // S^T[key][query] = sum_d K[key][d] Q[query][d]
        f32x16 sacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(&sK[lq * KS + 16 * c + 8 * h]);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], sacc, 0, 0, 0);
        }
        // scale, mask, online softmax over this lane's 16 keys (+ the other half-wave's 16)
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const long key = k0 + 8 * (v / 4) + 4 * h + (v % 4);
            bool ok = (tq >= 0) && (key < kv_end);
            if (causal) ok = ok && (key <= tq) && (key >= own_begin);
            sacc[v] = ok ? sacc[v] * a.scale : -INFINITY;
            mx = fmaxf(mx, sacc[v]);
        }
        mx = fmaxf(mx, shfl_xor_f(mx, 32));
        const float m_new = fmaxf(m, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = (m == -INFINITY) ? 0.f : __expf(m - m_safe);
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            sacc[v] = __expf(sacc[v] - m_safe);
            psum += sacc[v];
        }
        psum += shfl_xor_f(psum, 32);
        l = l * alpha + psum;
        m = m_new;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
        // P^T as the B operand: values 8c .. 8c+7 of the accumulator are this lane's keys
        // 16c + 4h + {0..3} and 16c + 8 + 4h + {0..3}; V^T is read with the same key order
        bf16x8 pf[2];
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int s8 = 0; s8 < 8; ++s8) pf[c][s8] = (__bf16)sacc[8 * c + s8];
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint16_t *vrow = &sVt[(32 * dt + lq) * VS + 16 * c + 4 * h];
                const uint2 lo = *reinterpret_cast<const uint2 *>(vrow);
                const uint2 hi = *reinterpret_cast<const uint2 *>(vrow + 8);
                union {
                    uint4 u;
                    bf16x8 f;
                } vf;
                vf.u = make_uint4(lo.x, lo.y, hi.x, hi.y);
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.f, pf[c], oacc[dt], 0, 0, 0);
            }
        }
    }

    if (tq < 0) return;
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
    const float lse = (l > 0.f) ? m + __logf(l) : -INFINITY;
    if (a.idx != nullptr) {
        if (!gathered) {  // slot of the own block in this row's list
            const int own = (int)(tq / a.block);
            const int32_t *row = a.idx + ((long)unit * a.T + tq) * a.K;
            slot = -1;
            for (int k = 0; k < a.K; ++k)
                if (row[k] == own) slot = k;
            if (slot < 0) return;  // the own block was not listed for this row
        }
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

// merge the partials of each row: 32 lanes per row, 4 (or 2) channels per lane
template <int D>
__global__ __launch_bounds__(256) void prefill_merge_kernel(const int32_t *__restrict__ idx,
                                                            const float *__restrict__ partial, bf16 *__restrict__ out,
                                                            float *__restrict__ lse_out, long rows, int K)
{
    constexpr int CPL = D / 32;  // channels per lane
    const long r = (long)blockIdx.x * 8 + (threadIdx.x >> 5);
    const int ln = threadIdx.x & 31;
    if (r >= rows) return;
    const int32_t *row = idx + r * K;
    const float *rec = partial + r * K * (kPartStride + D);
    float M = -INFINITY;
    for (int k = 0; k < K; ++k)
        if (row[k] >= 0) M = fmaxf(M, rec[(long)k * (kPartStride + D)]);
    float L = 0.f, o[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) o[c] = 0.f;
    for (int k = 0; k < K; ++k) {
        if (row[k] < 0) continue;
        const float *rk = rec + (long)k * (kPartStride + D);
        const float w = (rk[0] == -INFINITY) ? 0.f : __expf(rk[0] - M);
        L += w;
#pragma unroll
        for (int c = 0; c < CPL; ++c) o[c] = fmaf(w, rk[kPartStride + ln * CPL + c], o[c]);
    }
    const float inv = (L > 0.f) ? 1.f / L : 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c) from_f32(out[r * D + ln * CPL + c], o[c] * inv);
    if (ln == 0 && lse_out) lse_out[r] = (L > 0.f) ? M + __logf(L) : -INFINITY;
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
    long grid_x = p.n_diag;
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
        // upper bound of gathered tiles per (batch, head): every row picks at most K-1 other blocks
        grid_x += (T * (K > 1 ? K - 1 : 0) + kMT - 1) / kMT + Nb;
    }
    const dim3 grid((unsigned)grid_x, (unsigned)units);
    if (s->D == 128) prefill_attn_kernel<128><<<grid, 256, 0, stream>>>(p);
    else prefill_attn_kernel<64><<<grid, 256, 0, stream>>>(p);
    if (idx) {
        const long rows = units * T;
        if (s->D == 128)
            prefill_merge_kernel<128><<<(unsigned)((rows + 7) / 8), 256, 0, stream>>>(idx, p.partial, p.out, lse_out, rows, K);
        else
            prefill_merge_kernel<64><<<(unsigned)((rows + 7) / 8), 256, 0, stream>>>(idx, p.partial, p.out, lse_out, rows, K);
    }
    return hipGetLastError() == hipSuccess ? RS_OK : RS_LAUNCH_FAILED;
}

}  // namespace rs
