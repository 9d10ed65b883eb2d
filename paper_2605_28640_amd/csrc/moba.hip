// MoBA routing at prefill (App. A.1, MoBA paragraph; Sec. 2.2, Eq. 3): mean-pooled block
// representatives, per-query gate scores against the blocks before the query's own, and
// the top-K blocks per query token (own block and the first n_first always kept).
#include "common.h"

namespace rs {

// ------------------------------------------------------------------------------------
// block means: one workgroup per (block, batch*KV head); float32 accumulation
// ------------------------------------------------------------------------------------
template <typename ST, int D>
__global__ __launch_bounds__(256) void moba_block_means_kernel(const ST *__restrict__ k_cache,
                                                               float *__restrict__ means, long Tcap, long T,
                                                               int block, int Nb)
{
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;
    using R = Row8<ST>;
    __shared__ float s_acc[4][D];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rg = lane / LPR, c0 = (lane % LPR) * 8;
    const int j = blockIdx.x;
    const long bh = blockIdx.y;
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
        means[(bh * Nb + j) * D + tid] = s / (float)(t1 - t0);
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

size_t moba_select_ws_bytes(const rs_shape *, long, int) { return RS_WS_CTRL_BYTES; }

int moba_select_dispatch(const rs_shape *s, const void *q, const void *k_cache, long T, int block, int K,
                         int n_first, float *means_out, int32_t *idx_out, char *, hipStream_t stream)
{
    const int Nb = (int)((T + block - 1) / block);
    if (Nb > 256) return RS_UNSUPPORTED;  // one LDS score column per thread: Nb * 256 bytes
    const dim3 g1((unsigned)Nb, (unsigned)(s->B * s->Hkv));
    const dim3 g2((unsigned)((T + 63) / 64), (unsigned)(s->B * s->Hq));
    const size_t lds = (size_t)Nb * 64 * 4;
#define RS_LAUNCH(ST, DD)                                                                                          \
    do {                                                                                                           \
        moba_block_means_kernel<ST, DD><<<g1, 256, 0, stream>>>((const ST *)k_cache, means_out, s->Tcap, T, block, Nb); \
        moba_gate_topk_kernel<ST, DD><<<g2, 64, lds, stream>>>((const ST *)q, means_out, idx_out, s->Hq, s->Hkv, T,  \
                                                                block, Nb, K, n_first);                            \
    } while (0)
    if (s->dtype == RS_BF16) {
        if (s->D == 128) RS_LAUNCH(bf16, 128);
        else RS_LAUNCH(bf16, 64);
    } else {
        if (s->D == 128) RS_LAUNCH(float, 128);
        else RS_LAUNCH(float, 64);
    }
#undef RS_LAUNCH
    return hipGetLastError() == hipSuccess ? RS_OK : RS_LAUNCH_FAILED;
}

}  // namespace rs
