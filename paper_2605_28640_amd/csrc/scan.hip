// Gated decay recurrence (Sec. 2.1, Eq. 1) as a single-pass chunked scan.
//
// s_t = g_t s_{t-1} + (1-g_t) x_t is a first-order linear recurrence: a run of tokens
// acts on the incoming state as s -> A s + B, and two runs compose as
// (A2, B2) o (A1, B1) = (A1 A2, A2 B1 + B2).  One workgroup owns one chunk of tokens of
// one (batch, KV head) for all D channels:
//   1. every lane loads NT consecutive tokens x 8 channels (16-byte loads) and keeps
//      them in registers; it folds them into its (A, Bk, Bv);
//   2. the row groups of a wave are scanned with wave shuffles, the waves of the
//      workgroup through LDS;
//   3. the chunk's incoming state comes from the previous chunk of the same head
//      through a value+tag record in global memory (chunks are numbered by a ticket
//      taken at start, so the predecessor is always already running); the chunk
//      publishes its outgoing state before doing anything else;
//   4. every lane replays its tokens from its incoming state out of registers and
//      stores the rounded states into the cache.
// Inputs are read once and outputs written once: 12 bytes per channel-token for a
// bf16 cache.
//
// The chunks of one unit form a serial chain (one hop is about 0.7 us), which bounds the
// time when there are few (batch, head) pairs.  The channels of Eq. 1 are independent, so
// the kernel can also take a unit to be a slab of DS < D channels of a (batch, head): more,
// shorter chains (a chunk then spans D / DS times as many tokens for the same bytes).
#include <cstdlib>

#include "common.h"
#include "knobs.h"

namespace rs {

// PAGE > 0 (a run that starts on a chunk boundary, PAGE a power of two from 16 tokens
// to the chunk length): a wave's tokens (16 or 32 in bfloat16, 8 or 16 in float32, at 128 or 64
// channels) are whole pages or an aligned part of one, so the page's channelwise min / max of the stored keys (App. A.1,
// Quest) leave with the states -- in-lane over the lane's four tokens, shuffles over the row
// groups of a page, and for pages longer than a wave's tokens a fold of the waves' bounds
// through LDS -- and the keys need no second pass.
template <typename ST, int D, int DS, int NT, int NW, int PAGE>
__global__ __launch_bounds__(NW * 64) void rat_scan_chunk_kernel(
    const ST *__restrict__ k, const ST *__restrict__ v, const float *__restrict__ g,
    float *__restrict__ state_k, float *__restrict__ state_v, ST *__restrict__ k_cache,
    ST *__restrict__ v_cache, int BH, long T_new, long t0, long Tcap, int n_chunks,
    uint32_t *ctrl, uint64_t *rec, uint32_t tag, int spin_limit, ST *__restrict__ meta, int deep)
{
    constexpr bool META = PAGE > 0;
    constexpr int TW = (64 / (DS / 8)) * NT;  // tokens of a wave
    static_assert(!META || (PAGE >= 16 && (NW * TW) % (PAGE > 0 ? PAGE : 1) == 0), "pages tile the chunk");
    constexpr bool PG_LDS = META && PAGE > TW;  // a page spans several waves
    __shared__ float s_pg[PG_LDS ? NW : 1][2][PG_LDS ? DS : 1];
    constexpr int LPR = DS / 8;      // lanes per row (of the slab)
    constexpr int RPW = 64 / LPR;    // row groups per wave
    constexpr int CHUNK = NW * RPW * NT;
    constexpr int NS = D / DS;       // slabs per (batch, head)
    using R = Row8<ST>;

    __shared__ int s_ticket;
    __shared__ float s_agg[NW][3][DS];
    __shared__ float s_carry[NW][2][DS];

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int rg = lane / LPR;
    const int c0 = (lane % LPR) * 8;

    // deep (many units, so every chain has slack): the waves that do not handle the chain send the next
    // chunk's loads out before the current chunk is touched, and the ticket after next is drawn a chunk
    // ahead; otherwise all loads of the next chunk go out behind the chain step.
    // Persistent workgroups: each keeps taking the next chunk (by ticket) until none is left.  The raw
    // inputs of a chunk live in registers from its loads to its replay; there are two such register sets,
    // and the loads of the NEXT ticket are issued before the current chunk is folded, chained and stored,
    // so that a workgroup always has a chunk's worth of reads in flight (one workgroup fills a CU: without
    // this its memory pipe idles through every fold, chain wait and replay).  The prefetched ticket is
    // larger than the one in work and tickets are handed out in increasing order, so the smallest
    // unfinished ticket is always some workgroup's chunk in work: the chain cannot deadlock.
    const int units = BH * NS;
    const int total = units * n_chunks;
    // (kept as 32-bit words: the sets are carried around the chunk loop, and this compiler's back end
    // fails on loop-carried 128-bit vector values)
    constexpr int KW = (int)(sizeof(typename R::raw_t) / 4);
    struct ChunkRegs {
        uint32_t kw[NT][KW], vw[NT][KW];
        float gw[NT][8];
    };
    auto next_ticket = [&]() __attribute__((always_inline)) -> int {
        __syncthreads();  // the previous use of s_ticket (and of the chunk's LDS) is over
        if (tid == 0) s_ticket = (int)atomicAdd(&ctrl[kCtrlTicket], 1u);
        __syncthreads();
        return s_ticket;
    };
    auto load_chunk = [&](int ticket, ChunkRegs &r) __attribute__((always_inline)) {
        const int j = ticket / units;
        const int unit = ticket % units;
        const int bh = unit / NS;
        const int ch0 = (unit % NS) * DS;
        const long tbase = (long)j * CHUNK + (long)(wave * RPW + rg) * NT;
        const long in_row0 = (long)bh * T_new;
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const long t = tbase + i;
            typename R::raw_t kq = R::zero_raw(), vq = R::zero_raw();
            float4 ga = make_float4(1.f, 1.f, 1.f, 1.f), gb = ga;  // past the end: the identity element (g = 1 keeps the state)
            if (t < T_new) {
                const long off = (in_row0 + t) * D + ch0 + c0;
                if constexpr (DS == D) {
                    // whole rows, read once: streaming loads (a slab shares its cache lines with the
                    // other slabs of the row, which come by other workgroups: those stay cached loads)
                    kq = R::load_raw_nt(k + off);
                    vq = R::load_raw_nt(v + off);
                    typedef float f32x4 __attribute__((ext_vector_type(4)));
                    const f32x4 xa = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(g + off));
                    const f32x4 xb = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(g + off + 4));
                    ga = make_float4(xa.x, xa.y, xa.z, xa.w);
                    gb = make_float4(xb.x, xb.y, xb.z, xb.w);
                } else {
                    kq = R::load_raw(k + off);
                    vq = R::load_raw(v + off);
                    ga = *reinterpret_cast<const float4 *>(g + off);
                    gb = *reinterpret_cast<const float4 *>(g + off + 4);
                }
            }
            __builtin_memcpy(r.kw[i], &kq, sizeof(kq));
            __builtin_memcpy(r.vw[i], &vq, sizeof(vq));
            r.gw[i][0] = ga.x; r.gw[i][1] = ga.y; r.gw[i][2] = ga.z; r.gw[i][3] = ga.w;
            r.gw[i][4] = gb.x; r.gw[i][5] = gb.y; r.gw[i][6] = gb.z; r.gw[i][7] = gb.w;
        }
    };
    // nt / nr: the next ticket and its register set (nt >= total: none).  The waves that handle the chain
    // (threads below DS) issue their share of the next chunk's loads only after the chain step: a wave's
    // loads return in order, so its polls of the predecessor's record would otherwise wait behind them.
    constexpr int kChainWaves = (DS + 63) / 64;
    auto process_chunk = [&](int ticket, ChunkRegs &r, int nt, ChunkRegs &nr) __attribute__((always_inline)) {
    const int j = ticket / units;   // chunk index along T
    const int unit = ticket % units;  // consecutive tickets walk the units first
    const int bh = unit / NS;
    const int ch0 = (unit % NS) * DS;  // first channel of the slab
    const long tbase = (long)j * CHUNK + (long)(wave * RPW + rg) * NT;
    typename R::raw_t kr[NT], vr[NT];
    float4 g0[NT], g1[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        __builtin_memcpy(&kr[i], r.kw[i], sizeof(kr[i]));
        __builtin_memcpy(&vr[i], r.vw[i], sizeof(vr[i]));
        g0[i] = make_float4(r.gw[i][0], r.gw[i][1], r.gw[i][2], r.gw[i][3]);
        g1[i] = make_float4(r.gw[i][4], r.gw[i][5], r.gw[i][6], r.gw[i][7]);
    }

    // the ticket after next is drawn now and parked in LDS at the first barrier: its round trip runs
    // under the fold (full-row form; the slab form draws its tickets one at a time)
    int ticket_ahead = 0;
    if constexpr (DS == D) {
        if (deep && tid == 0) ticket_ahead = (int)atomicAdd(&ctrl[kCtrlTicket], 1u);
    }

    // first look at the previous chunk's outgoing state, issued behind the data loads so that
    // its round trip overlaps the fold; the wait below re-polls only if it was not there yet
    uint64_t early0 = 0, early1 = 0;
    if (tid < DS && j > 0) {
        const uint64_t *p = rec + (((long)unit * n_chunks + (j - 1)) * 2) * DS + tid;
        early0 = load_u64_agent(p);
        early1 = load_u64_agent(p + DS);
    }

    // fold own tokens: state -> a * state + b
    float a[8], bk[8], bv[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        a[c] = 1.f;
        bk[c] = 0.f;
        bv[c] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        float kx[8], vx[8];
        R::unpack(kr[i], kx);
        R::unpack(vr[i], vx);
        const float gg[8] = {g0[i].x, g0[i].y, g0[i].z, g0[i].w, g1[i].x, g1[i].y, g1[i].z, g1[i].w};
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const float om = 1.f - gg[c];
            a[c] *= gg[c];
            bk[c] = fmaf(gg[c], bk[c], om * kx[c]);
            bv[c] = fmaf(gg[c], bv[c], om * vx[c]);
        }
    }

    if constexpr (RPW == 4) {
        // Four row groups = the four 16-lane rows of the wave.  Two register swaps (v_permlane16_swap,
        // v_permlane32_swap: no trip through the LDS crossbar) put both members of a pair of rows, then
        // both pairs, side by side in every lane; the wave's total and what precedes each row group
        // follow by composition (first X then Y: A = Ax Ay, B = Ay Bx + By).
        const bool odd = rg & 1, upper = rg >= 2;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const auto sa = __builtin_amdgcn_permlane16_swap(__float_as_uint(a[c]), __float_as_uint(a[c]), false, false);
            const auto sk = __builtin_amdgcn_permlane16_swap(__float_as_uint(bk[c]), __float_as_uint(bk[c]), false, false);
            const auto sv = __builtin_amdgcn_permlane16_swap(__float_as_uint(bv[c]), __float_as_uint(bv[c]), false, false);
            const float ae = __uint_as_float(sa[0]), ao = __uint_as_float(sa[1]);  // even / odd row of the pair
            const float ke = __uint_as_float(sk[0]), ko = __uint_as_float(sk[1]);
            const float ve = __uint_as_float(sv[0]), vo = __uint_as_float(sv[1]);
            const float PA = ae * ao, PK = fmaf(ao, ke, ko), PV = fmaf(ao, ve, vo);  // the pair
            const auto ta = __builtin_amdgcn_permlane32_swap(__float_as_uint(PA), __float_as_uint(PA), false, false);
            const auto tk = __builtin_amdgcn_permlane32_swap(__float_as_uint(PK), __float_as_uint(PK), false, false);
            const auto tv = __builtin_amdgcn_permlane32_swap(__float_as_uint(PV), __float_as_uint(PV), false, false);
            const float A0 = __uint_as_float(ta[0]), A1 = __uint_as_float(ta[1]);  // lower / upper pair
            const float K0 = __uint_as_float(tk[0]), K1 = __uint_as_float(tk[1]);
            const float V0 = __uint_as_float(tv[0]), V1 = __uint_as_float(tv[1]);
            if (rg == RPW - 1) {  // the wave's total
                s_agg[wave][0][c0 + c] = A0 * A1;
                s_agg[wave][1][c0 + c] = fmaf(A1, K0, K1);
                s_agg[wave][2][c0 + c] = fmaf(A1, V0, V1);
            }
            // what precedes this row group inside its wave: inside its pair, then the lower pair before it
            float xa = odd ? ae : 1.f, xk = odd ? ke : 0.f, xv = odd ? ve : 0.f;
            if (upper) {
                xk = fmaf(xa, K0, xk);
                xv = fmaf(xa, V0, xv);
                xa *= A0;
            }
            a[c] = xa;
            bk[c] = xk;
            bv[c] = xv;
        }
    } else {
    // inclusive scan over the row groups of the wave
#pragma unroll
    for (int d = 1; d < RPW; d <<= 1) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const float pa = shfl_up_f(a[c], d * LPR);
            const float pk = shfl_up_f(bk[c], d * LPR);
            const float pv = shfl_up_f(bv[c], d * LPR);
            if (rg >= d) {
                bk[c] = fmaf(a[c], pk, bk[c]);
                bv[c] = fmaf(a[c], pv, bv[c]);
                a[c] *= pa;
            }
        }
    }
    if (rg == RPW - 1) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            s_agg[wave][0][c0 + c] = a[c];
            s_agg[wave][1][c0 + c] = bk[c];
            s_agg[wave][2][c0 + c] = bv[c];
        }
    }
    // exclusive within the wave: what precedes this lane's tokens inside its wave
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float pa = shfl_up_f(a[c], LPR);
        const float pk = shfl_up_f(bk[c], LPR);
        const float pv = shfl_up_f(bv[c], LPR);
        a[c] = (rg == 0) ? 1.f : pa;
        bk[c] = (rg == 0) ? 0.f : pk;
        bv[c] = (rg == 0) ? 0.f : pv;
    }
    }
    if constexpr (DS == D) {
        if (deep && tid == 0) s_ticket = ticket_ahead;
    }
    __syncthreads();

    if (tid < DS) {
        const int c = tid;
        float A = 1.f, Bk = 0.f, Bv = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float aw = s_agg[w][0][c];
            Bk = fmaf(aw, Bk, s_agg[w][1][c]);
            Bv = fmaf(aw, Bv, s_agg[w][2][c]);
            A *= aw;
        }
        float Sk, Sv;
        if (j == 0) {
            Sk = state_k[bh * D + ch0 + c];
            Sv = state_v[bh * D + ch0 + c];
        } else {
            const uint64_t *p = rec + (((long)unit * n_chunks + (j - 1)) * 2) * DS + c;
            uint64_t w0 = early0, w1 = early1;
            int spins = 0;
            bool ok = ((uint32_t)(w0 >> 32) == tag) && ((uint32_t)(w1 >> 32) == tag);
            while (!ok) {
                if (++spins > spin_limit) break;
                __builtin_amdgcn_s_sleep(2);
                w0 = load_u64_agent(p);
                w1 = load_u64_agent(p + DS);
                ok = ((uint32_t)(w0 >> 32) == tag) && ((uint32_t)(w1 >> 32) == tag);
            }
            if (!ok) atomicExch(&ctrl[kCtrlAsyncErr], 1u);  // give up; outputs undefined
            Sk = __uint_as_float((uint32_t)w0);
            Sv = __uint_as_float((uint32_t)w1);
        }
        const float Ok = fmaf(A, Sk, Bk);
        const float Ov = fmaf(A, Sv, Bv);
        if (j == n_chunks - 1) {
            state_k[bh * D + ch0 + c] = Ok;
            state_v[bh * D + ch0 + c] = Ov;
        } else {
            uint64_t *p = rec + (((long)unit * n_chunks + j) * 2) * DS + c;
            store_u64_agent(p, ((uint64_t)tag << 32) | __float_as_uint(Ok));
            store_u64_agent(p + DS, ((uint64_t)tag << 32) | __float_as_uint(Ov));
        }
        float ck = Sk, cv = Sv;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            s_carry[w][0][c] = ck;
            s_carry[w][1][c] = cv;
            const float aw = s_agg[w][0][c];
            ck = fmaf(aw, ck, s_agg[w][1][c]);
            cv = fmaf(aw, cv, s_agg[w][2][c]);
        }
    }
    // the next chunk's loads go out here, behind the chain step: a wave's loads return in order, so
    // issued any earlier they would hold up the chain waves' polls of the predecessor's record
    if constexpr (DS == D) {  // (the slab form works on one chunk at a time)
        if ((wave < kChainWaves || !deep) && nt < total) load_chunk(nt, nr);
    }
    __syncthreads();

    // replay from the incoming state
    float sk[8], sv[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        sk[c] = fmaf(a[c], s_carry[wave][0][c0 + c], bk[c]);
        sv[c] = fmaf(a[c], s_carry[wave][1][c0 + c], bv[c]);
    }
    const long out_row0 = (long)bh * Tcap + t0;
    float plo[8], phi[8];  // META: bounds of the stored (rounded) keys of this lane's tokens
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        plo[c] = INFINITY;
        phi[c] = -INFINITY;
    }
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const long t = tbase + i;
        if (t < T_new) {
            float kx[8], vx[8];
            R::unpack(kr[i], kx);
            R::unpack(vr[i], vx);
            const float gg[8] = {g0[i].x, g0[i].y, g0[i].z, g0[i].w, g1[i].x, g1[i].y, g1[i].z, g1[i].w};
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const float om = 1.f - gg[c];
                sk[c] = fmaf(gg[c], sk[c], om * kx[c]);
                sv[c] = fmaf(gg[c], sv[c], om * vx[c]);
            }
            const long off = (out_row0 + t) * D + ch0 + c0;
            R::store_nt(k_cache + off, sk);
            R::store_nt(v_cache + off, sv);
            if constexpr (META) {
                float xs[8];  // the values just stored
                if constexpr (sizeof(ST) == 2) {
                    const uint32_t w[4] = {pack_bf16x2(sk[0], sk[1]), pack_bf16x2(sk[2], sk[3]), pack_bf16x2(sk[4], sk[5]),
                                           pack_bf16x2(sk[6], sk[7])};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        xs[2 * c] = __uint_as_float(w[c] << 16);
                        xs[2 * c + 1] = __uint_as_float(w[c] & 0xffff0000u);
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < 8; ++c) xs[c] = sk[c];
                }
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    plo[c] = fminf(plo[c], xs[c]);
                    phi[c] = fmaxf(phi[c], xs[c]);
                }
            }
        }
    }
    if constexpr (META) {
        if constexpr (!PG_LDS) {
            // PAGE / NT row groups make a page: fold them, then the first two lanes groups of a page write it
            constexpr int RGP = PAGE / NT;
#pragma unroll
            for (int msk = LPR; msk < LPR * RGP; msk <<= 1)
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    plo[c] = fminf(plo[c], shfl_xor_f(plo[c], msk));
                    phi[c] = fmaxf(phi[c], shfl_xor_f(phi[c], msk));
                }
            const long tp = (long)j * CHUNK + (long)wave * TW + (long)(rg / RGP) * PAGE;  // the page's first token
            if (tp < T_new && rg % RGP < 2) {
                const long page = (t0 + tp) / PAGE;
                ST *mrow = meta + (((long)bh * (Tcap / PAGE) + page) * 2) * D + ch0 + c0;
                if (rg % RGP == 0) R::store(mrow, plo);
                else R::store(mrow + D, phi);
            }
        } else {
            // a page spans WPP waves: each folds all its row groups, their bounds meet in LDS, and
            // wave w < NW / WPP writes page w of the chunk
            constexpr int WPP = PAGE / TW;
#pragma unroll
            for (int msk = LPR; msk < 64; msk <<= 1)
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    plo[c] = fminf(plo[c], shfl_xor_f(plo[c], msk));
                    phi[c] = fmaxf(phi[c], shfl_xor_f(phi[c], msk));
                }
            if (rg == 0) {
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    s_pg[wave][0][c0 + c] = plo[c];
                    s_pg[wave][1][c0 + c] = phi[c];
                }
            }
            __syncthreads();
            const long tp = (long)j * CHUNK + (long)wave * PAGE;  // first token of page `wave` of this chunk
            if (wave < NW / WPP && rg < 2 && tp < T_new) {
                float x[8];
#pragma unroll
                for (int c = 0; c < 8; ++c) x[c] = s_pg[wave * WPP][rg][c0 + c];
#pragma unroll
                for (int w2 = 1; w2 < WPP; ++w2)
#pragma unroll
                    for (int c = 0; c < 8; ++c) {
                        const float y = s_pg[wave * WPP + w2][rg][c0 + c];
                        x[c] = rg == 0 ? fminf(x[c], y) : fmaxf(x[c], y);
                    }
                const long page = (t0 + tp) / PAGE;
                R::store(meta + (((long)bh * (Tcap / PAGE) + page) * 2 + rg) * D + ch0 + c0, x);
            }
        }
    }

    };  // process_chunk

    // (one call site of process_chunk: the register sets change places by moves, which cost nothing next
    // to a chunk's work and wait for the prefetched loads no earlier than the fold would)
    ChunkRegs A, B;
    int tA = (int)blockIdx.x;  // one chunk per unit: the grid is the units, no tickets
    if (n_chunks > 1) tA = next_ticket();
    if (tA < total) {
        load_chunk(tA, A);
        int tB = total;
        if constexpr (DS == D) {
            if (n_chunks > 1) tB = next_ticket();
        }
        for (;;) {
            if constexpr (DS == D) {
                // the waves that do not handle the chain send the next chunk's loads ahead of everything
                if (deep && wave >= kChainWaves && tB < total) load_chunk(tB, B);
            }
            process_chunk(tA, A, tB, B);
            if constexpr (DS == D) {
                if (tB >= total) break;
                A = B;
                tA = tB;
                if (deep) {
                    __syncthreads();  // s_ticket was parked before the first barrier of process_chunk and is read by all here
                    tB = s_ticket;
                    __syncthreads();  // ... before the next chunk's thread 0 parks the following one
                } else {
                    tB = next_ticket();
                }
            } else {
                if (n_chunks == 1) break;
                tA = next_ticket();
                if (tA >= total) break;
                load_chunk(tA, A);
            }
        }
    }

    if (n_chunks > 1 && tid == 0) {
        if (atomicAdd(&ctrl[kCtrlDone], 1u) == gridDim.x - 1u) {  // last workgroup out resets the counters
            atomicExch(&ctrl[kCtrlTicket], 0u);
            atomicExch(&ctrl[kCtrlDone], 0u);
        }
    }
}

// few tokens (the decode-time append): one thread per (batch, head, channel)
template <typename ST>
__global__ __launch_bounds__(256) void rat_step_kernel(
    const ST *__restrict__ k, const ST *__restrict__ v, const float *__restrict__ g,
    float *__restrict__ state_k, float *__restrict__ state_v, ST *__restrict__ k_cache,
    ST *__restrict__ v_cache, ST *__restrict__ meta, int P, int BH, int D, long T_new, long t0, long Tcap,
    const uint32_t *__restrict__ pos_state, long T_max, int K_min_pages)
{
    const long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (long)BH * D) return;
    if (pos_state) {  // replayable step: the write position is the workspace's token count
        t0 = *reinterpret_cast<const long *>(pos_state + kCtrlStateT);
        // a step the attention kernel of the same call will refuse (past T_max, or fewer pages than
        // it must select) appends nothing either: the refused step leaves carries, caches and page
        // bounds as they were, and the attention kernel reports it
        if (t0 + T_new > T_max || (t0 + T_new + P - 1) / P < (long)K_min_pages) return;
    }
    const long bh = e / D;
    const int c = (int)(e % D);
    float sk = state_k[e], sv = state_v[e];
    for (long t = 0; t < T_new; ++t) {
        const long off = (bh * T_new + t) * D + c;
        const float gg = g[off];
        const float om = 1.f - gg;
        sk = fmaf(gg, sk, om * to_f32(k[off]));
        sv = fmaf(gg, sv, om * to_f32(v[off]));
        const long o = (bh * Tcap + t0 + t) * D + c;
        from_f32(k_cache[o], sk);
        from_f32(v_cache[o], sv);
        if (meta) {
            // Quest page min/max of the stored key: a page's first row starts it, later rows fold in
            const long row = t0 + t;
            ST *mn = meta + ((bh * (Tcap / P) + row / P) * 2) * D + c;
            const float x = to_f32(k_cache[o]);
            float lo = x, hi = x;
            if (row % P != 0) {
                lo = fminf(to_f32(mn[0]), x);
                hi = fmaxf(to_f32(mn[D]), x);
            }
            from_f32(mn[0], lo);
            from_f32(mn[D], hi);
        }
    }
    state_k[e] = sk;
    state_v[e] = sv;
}

template <typename ST, int D, int DS, int PAGE_ARG>
static int launch_scan(const void *k, const void *v, const float *g, float *state_k,
                       float *state_v, void *k_cache, void *v_cache, int BH, long T_new, long t0,
                       long Tcap, uint32_t *ctrl, uint64_t *rec, uint32_t tag, int spin_limit,
                       void *meta, hipStream_t stream)
{
    constexpr int NT = sizeof(ST) == 2 ? 4 : 2;
    constexpr int NW = 8;
    constexpr int CHUNK = NW * (64 / (DS / 8)) * NT;
    constexpr int PAGE = (PAGE_ARG <= CHUNK) ? PAGE_ARG : 0;  // larger pages never get here with the bounds asked for
    const int n_chunks = (int)((T_new + CHUNK - 1) / CHUNK);
    long grid = (long)BH * (D / DS) * n_chunks;
    if (n_chunks > 1) {
        static int per_cu = 0, cus = 0;  // resident workgroups of this kernel
        if (per_cu == 0) {
            int dev = 0, n = 0;
            (void)hipGetDevice(&dev);
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, rat_scan_chunk_kernel<ST, D, DS, NT, NW, PAGE>, NW * 64, 0) != hipSuccess || n < 1) n = 1;
            per_cu = n;
            if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        }
        long want = knob_or(knobs().scan_grid, per_cu * cus);
        if (want < 1) want = 1;
        if (want > (long)per_cu * cus) want = (long)per_cu * cus;  // the knob only narrows: every workgroup stays resident
        if (grid > want) grid = want;
    }
    rat_scan_chunk_kernel<ST, D, DS, NT, NW, PAGE><<<dim3((unsigned)grid), dim3(NW * 64), 0, stream>>>(
        (const ST *)k, (const ST *)v, g, state_k, state_v, (ST *)k_cache, (ST *)v_cache, BH, T_new,
        t0, Tcap, n_chunks, ctrl, rec, tag, spin_limit, (ST *)meta, (n_chunks > 1 && (long)BH * (D / DS) >= 128) ? 1 : 0);
    return 0;
}

int scan_chunk_tokens(int dtype, int D)
{
    const int NT = dtype == RS_BF16 ? 4 : 2;
    return 8 * (64 / (D / 8)) * NT;
}

// host entry used by the C ABI (arguments already validated)
bool scan_uses_step_kernel(long T_new) { return T_new <= 8; }

static bool scan_uses_slabs(int BH, long T_new)
{
    // few (batch, head) pairs and a long run: 32-channel slabs, so that the chunk chains are
    // shorter and there are more of them
    const int forced = knobs().scan_slab;
    return forced != kKnobUnset ? forced != 0 : (BH <= 16 && T_new >= 2048);
}

// whether the chunk kernel leaves the Quest page bounds of the rows it stores (else the caller
// recomputes the touched pages afterwards)
bool scan_writes_meta(int dtype, int D, int P, int BH, long T_new, long t0)
{
    if (scan_uses_step_kernel(T_new)) return true;  // the step kernel keeps the touched page current
    if (knobs().scan_meta == 0) return false;
    // chunk of the form in use: bfloat16 128 tokens at D = 128, 256 at D = 64 (float32: half); 32-channel slabs: D / 32 times that
    const long chunk = (long)scan_chunk_tokens(dtype, D) * (scan_uses_slabs(BH, T_new) ? D / 32 : 1);
    return P >= 16 && P <= chunk && (P & (P - 1)) == 0 && t0 % chunk == 0;
}

void scan_dispatch(int dtype, int D, const void *k, const void *v, const float *g, float *state_k,
                   float *state_v, void *k_cache, void *v_cache, void *meta, int P, int BH, long T_new, long t0,
                   long Tcap, uint32_t *ctrl, uint64_t *rec, uint32_t tag, int spin_limit,
                   hipStream_t stream)
{
    if (scan_uses_step_kernel(T_new)) {
        const long n = (long)BH * D;
        const unsigned blocks = (unsigned)((n + 255) / 256);
        if (dtype == RS_BF16)
            rat_step_kernel<bf16><<<blocks, 256, 0, stream>>>((const bf16 *)k, (const bf16 *)v, g, state_k, state_v,
                                                             (bf16 *)k_cache, (bf16 *)v_cache, (bf16 *)meta, P, BH, D, T_new, t0, Tcap, nullptr, 0, 0);
        else
            rat_step_kernel<float><<<blocks, 256, 0, stream>>>((const float *)k, (const float *)v, g, state_k, state_v,
                                                              (float *)k_cache, (float *)v_cache, (float *)meta, P, BH, D, T_new, t0, Tcap, nullptr, 0, 0);
        return;
    }
    const bool slab = scan_uses_slabs(BH, T_new);
#define RS_SCAN(ST, DD, DSS, MM) launch_scan<ST, DD, DSS, MM>(k, v, g, state_k, state_v, k_cache, v_cache, BH, T_new, t0, Tcap, ctrl, rec, tag, spin_limit, meta, stream)
    const bool in_scan = meta && scan_writes_meta(dtype, D, P, BH, T_new, t0);
    // page sizes up to 512 tokens have their own instantiation where they tile the form's chunk
#define RS_SCAN_P(ST, DD, DSS)                           \
    do {                                                 \
        if (!in_scan) RS_SCAN(ST, DD, DSS, 0);           \
        else if (P == 16) RS_SCAN(ST, DD, DSS, 16);      \
        else if (P == 32) RS_SCAN(ST, DD, DSS, 32);      \
        else if (P == 64) RS_SCAN(ST, DD, DSS, 64);      \
        else if (P == 128) RS_SCAN(ST, DD, DSS, 128);    \
        else if (P == 256) RS_SCAN(ST, DD, DSS, 256);    \
        else RS_SCAN(ST, DD, DSS, 512);                  \
    } while (0)
    if (dtype == RS_BF16) {
        if (D == 128) {
            if (slab) RS_SCAN_P(bf16, 128, 32);
            else RS_SCAN_P(bf16, 128, 128);
        } else {
            if (slab) RS_SCAN_P(bf16, 64, 32);
            else RS_SCAN_P(bf16, 64, 64);
        }
    } else {
        if (D == 128) {
            if (slab) RS_SCAN_P(float, 128, 32);
            else RS_SCAN_P(float, 128, 128);
        } else {
            if (slab) RS_SCAN_P(float, 64, 32);
            else RS_SCAN_P(float, 64, 64);
        }
    }
#undef RS_SCAN_P
#undef RS_SCAN
}

// the decode-time append of one token at the position the workspace's state words hold
void step_at_state_dispatch(int dtype, int D, const void *k, const void *v, const float *g, float *state_k,
                            float *state_v, void *k_cache, void *v_cache, void *meta, int P, int BH, long Tcap,
                            const uint32_t *pos_state, long T_max, int K, hipStream_t stream)
{
    const long n = (long)BH * D;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (dtype == RS_BF16)
        rat_step_kernel<bf16><<<blocks, 256, 0, stream>>>((const bf16 *)k, (const bf16 *)v, g, state_k, state_v,
                                                         (bf16 *)k_cache, (bf16 *)v_cache, (bf16 *)meta, P, BH, D, 1, 0, Tcap, pos_state, T_max, K);
    else
        rat_step_kernel<float><<<blocks, 256, 0, stream>>>((const float *)k, (const float *)v, g, state_k, state_v,
                                                          (float *)k_cache, (float *)v_cache, (float *)meta, P, BH, D, 1, 0, Tcap, pos_state, T_max, K);
}

}  // namespace rs
