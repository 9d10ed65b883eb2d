// Fused Quest decode (Sec. 2.2, Eq. 3-4; App. A.1): page scores, top-K page selection and
// attention over the selected pages in ONE persistent launch, so unselected KV is never
// read and no kernel boundary or cache flush sits between selection and attention.
//
// The grid is a fixed number of workgroups that pull work items by ticket:
//   tickets [0, n_score)         score item  = (unit, slice of its pages): stream the page
//                                min/max rows, publish one score per page; the unit's last
//                                slice then gathers the unit's scores, runs the radix top-K
//                                and publishes the ascending page list;
//   tickets [n_score, n_total)   attend item = (unit, slice of its K pages): wait for the
//                                unit's page list, stream the listed K/V pages with an
//                                online softmax, publish a partial (m, l, o); the unit's
//                                last slice folds in the other partials and writes y.
// unit = (batch, query head).  Everything another workgroup must read in the same launch
// travels as {tag : value} words (see select.h), so waiting is a bounded poll on data that
// an already-running workgroup is producing: whoever waits holds a larger ticket than the
// item it waits for, tickets are handed out in increasing order to running workgroups,
// and the item with the smallest outstanding ticket never waits.
#include "common.h"
#include "select.h"
#include "decode_fused.h"

namespace rs {

template <typename ST, int D, int kFusedThreads, bool STATE>
__global__ __launch_bounds__(kFusedThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void decode_fused_kernel(const FusedParams P_)
{
    constexpr int kFusedWaves = kFusedThreads / 64;
    constexpr int LPR = D / 8;
    constexpr int RPW = 64 / LPR;
    using R = Row8<ST>;
    const FusedParams &a = P_;
    // sequence length, page count and tag: kernel arguments, or (replayable step) the workspace's state words
    long T_valid_ = a.T_valid;
    int Np_ = a.Np;
    uint32_t tag_ = a.tag;
    long score_stride = a.Np;
    int reverse_ = a.reverse;
    if constexpr (STATE) {
        T_valid_ = *reinterpret_cast<const long *>(a.state + kCtrlStateT) + 1;
        tag_ = a.state[kCtrlStateTag];
        // a workspace that has only been zeroed holds tag 0, which zero-filled score, list and
        // partial words would already "carry": never hand off under tag 0
        if (tag_ == 0u) tag_ = 0x5bd1e995u;
        Np_ = (int)((T_valid_ + a.P - 1) / a.P);
        score_stride = (a.T_max + a.P - 1) / a.P;
        reverse_ = a.reverse ? (int)(T_valid_ & 1) : 0;
        if (T_valid_ > a.T_max || a.K > Np_) {  // outside what the buffers were sized for: report, do nothing
            if (blockIdx.x == 0 && threadIdx.x == 0) atomicExch(a.err, 1u);
            return;
        }
    }

    __shared__ SelectShared<kFusedThreads> sh;
    __shared__ float s_m[kFusedWaves], s_l[kFusedWaves];
    __shared__ float s_o[kFusedWaves][D];
    __shared__ int s_next;
    extern __shared__ uint32_t s_keys[];  // Np keys for the selection

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int rg = lane / LPR;
    const int cl = lane % LPR;
    const int c0 = cl * 8;
    // the units scored last are split finer: their attention is what the launch ends on
    const int n_score = a.units * a.S_score;
    const int u_coarse = a.units - a.units_fine;
    const int n_att_coarse = u_coarse * a.S_att;
    const int n_total = n_score + n_att_coarse + a.units_fine * a.S_att_fine;
    const int G = a.Hq / a.Hkv;

    // per-workgroup timeline for tuning: compiled in only with -DRS_FUSED_TRACE (never in the shipped library)
#ifdef RS_FUSED_TRACE
    int n_ev = 0;
    auto mark = [&](int item_, int phase) {
        if (a.trace && tid == 0 && n_ev < 64)
            a.trace[(long)blockIdx.x * 64 + n_ev++] = (wall_clock64() << 24) | ((uint64_t)(item_ & 0xfffff) << 4) | (uint64_t)phase;
    };
#else
    auto mark = [](int, int) {};
#endif
    if (tid == 0) s_next = (int)atomicAdd(a.ticket, 1u);
    __syncthreads();
    int item = s_next;
    while (item < n_total) {
        __syncthreads();  // s_next has been read by everyone; LDS of the previous item is free
        // The next ticket is taken late: during the last streaming step of an item that waits
        // for nobody, after the waiting for one that does.  A ticket held but not yet started
        // would make its waiters wait for the holder's whole current item.
        bool fetched = false;
        auto fetch_next = [&]() {
            if (tid == 0 && !fetched) {
                s_next = (int)atomicAdd(a.ticket, 1u);
                fetched = true;
            }
        };
        mark(item, 0);

        if (item < n_score) {
            // ------------------------------ score item ------------------------------
            int unit = item / a.S_score;
            const int slice = item % a.S_score;
            if (reverse_) unit = a.units - 1 - unit;
            const int b = unit / a.Hq, h = unit % a.Hq, kvh = h / G;
            const ST *mbase = (const ST *)a.meta + ((long)(b * a.Hkv + kvh) * a.Np_cap) * 2 * D;
            uint64_t *srow = a.scores + (long)unit * score_stride;
            float qv[8];
            R::load((const ST *)a.q + (long)unit * D + c0, qv);
            BoundDot<ST> bound;
            bound.set(qv);

            constexpr int UNR = 4;
            constexpr int PPI = UNR * RPW * kFusedWaves;  // pages per workgroup step
            const int per = (Np_ + a.S_score - 1) / a.S_score;
            const int pb = slice * per;
            const int pe = (pb + per < Np_) ? pb + per : Np_;
            const bool sel_here = (slice == a.S_score - 1);
            for (int base = pb + wave * (UNR * RPW) + rg; base < pe; base += PPI) {
                if (!sel_here && base + PPI >= pe) fetch_next();
                typename R::raw_t mn[UNR], mx[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const int p = base + u * RPW;
                    if (p < pe) {
                        if (a.nt_kv & 2) {
                            mn[u] = R::load_raw_nt(mbase + ((long)p * 2) * D + c0);
                            mx[u] = R::load_raw_nt(mbase + ((long)p * 2 + 1) * D + c0);
                        } else {
                            mn[u] = R::load_raw(mbase + ((long)p * 2) * D + c0);
                            mx[u] = R::load_raw(mbase + ((long)p * 2 + 1) * D + c0);
                        }
                    } else {
                        mn[u] = R::zero_raw();
                        mx[u] = R::zero_raw();
                    }
                }
                // the wave's UNR * RPW pages are consecutive.  Every lane of a row group holds the group's
                // sums; lane u of the group keeps page u's, and the UNR first lanes of the RPW groups then
                // publish the wave's scores with ONE store instruction of adjacent 8-byte words (whole lines
                // on the write-through path; which lane writes which word of a line does not matter)
                float mine = 0.f;
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    const float s = group_sum<LPR>(bound.add(0.f, mn[u], mx[u]));
                    if (cl == u) mine = s;
                }
                {
                    const int p = base + cl * RPW;
                    if (cl < UNR && p < pe) publish_f32(&srow[p], mine, tag_);
                }
            }
            mark(item, 1);
            // the unit's last slice carries the largest ticket: every other slice is already
            // running or done, so it can wait for their scores and run the selection
            if (sel_here) {
                __builtin_amdgcn_s_setprio(3);  // the unit's attention waits on this: go first on the CU
                gather_page_keys<kFusedThreads>(srow, Np_, a.n_first, a.n_local, tag_, a.spin_limit, a.err, nullptr,
                                                s_keys);
                mark(item, 7);
                uint64_t *dst = a.idx_tagged + (long)unit * a.K;
                int32_t *plain = a.idx_out ? a.idx_out + (long)unit * a.K : nullptr;
                const uint32_t tag = tag_;
                select_topk_lds<kFusedThreads>(s_keys, Np_, a.K, sh, [dst, plain, tag](int pos, int p) {
                    store_u64_agent(&dst[pos], ((uint64_t)tag << 32) | (uint32_t)p);
                    if (plain) plain[pos] = p;
                }, [&](int ph) { mark(item, ph); });
                __builtin_amdgcn_s_setprio(0);
                mark(item, 3);
            }
        } else {
            // ------------------------------ attend item -----------------------------
            const int it = item - n_score;
            int unit, slice, S_att;
            if (it < n_att_coarse) {
                S_att = a.S_att;
                unit = it / S_att;
                slice = it % S_att;
            } else {
                S_att = a.S_att_fine;
                unit = u_coarse + (it - n_att_coarse) / S_att;
                slice = (it - n_att_coarse) % S_att;
            }
            if (reverse_) unit = a.units - 1 - unit;
            const int b = unit / a.Hq, h = unit % a.Hq, kvh = h / G;
            const ST *kb = (const ST *)a.k_cache + (long)(b * a.Hkv + kvh) * a.Tcap * D;
            const ST *vb = (const ST *)a.v_cache + (long)(b * a.Hkv + kvh) * a.Tcap * D;
            const uint64_t *sel = a.idx_tagged + (long)unit * a.K;

            constexpr int TR = 16;
            constexpr int RPL = TR / RPW;
            constexpr int TPI = 2;
            RowDot<ST> qd;
            {
                float qv[8];
                R::load((const ST *)a.q + (long)unit * D + c0, qv);
                qd.set(qv);
            }

            const int tiles_per_page = a.P / TR;
            const int n_tiles = a.K * tiles_per_page;
            const int per = (n_tiles + S_att - 1) / S_att;
            const int tb = slice * per;
            const int te = (tb + per < n_tiles) ? tb + per : n_tiles;

            float m = -INFINITY, l = 0.f;
            float o[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) o[c] = 0.f;

            const bool finish = (slice == S_att - 1);  // largest ticket of the unit: folds the others
            // The list entries of the tiles this wave will take come in at once, one per lane (lane j: step
            // j / TPI, tile j % TPI of the step), each lane waiting for its own word if the selection is
            // still being written; the steps then read them lane to scalar.  Otherwise every step would
            // begin with a trip to memory for its entries before it can ask for the rows.
            constexpr int SPC = 64 / TPI;  // steps one such fetch covers
            uint32_t my_page = 0xffffffffu;
            int step_i = 0;
            for (int t = tb + wave * TPI; t < te; t += kFusedWaves * TPI, ++step_i) {
                if (!finish && t + kFusedWaves * TPI >= te) fetch_next();
                if (step_i % SPC == 0) {
                    const int mt = t + (lane / TPI) * (kFusedWaves * TPI) + (lane % TPI);
                    my_page = 0xffffffffu;
                    if (mt < te) {
                        const uint64_t *wp = &sel[mt / tiles_per_page];
                        uint64_t w2 = load_u64_agent(wp);
                        int spins = 0;
                        while ((uint32_t)(w2 >> 32) != tag_) {  // the selection is still being written
                            if (++spins > a.spin_limit) {
                                atomicExch(a.err, 1u);
                                break;
                            }
                            __builtin_amdgcn_s_sleep(2);
                            w2 = load_u64_agent(wp);
                        }
                        if ((uint32_t)(w2 >> 32) == tag_) my_page = (uint32_t)w2;  // else gave up: skip
                    }
                }
                long row0[TPI];
                typename R::raw_t kr[TPI][RPL], vr[TPI][RPL];
#pragma unroll
                for (int u = 0; u < TPI; ++u) {
                    row0[u] = T_valid_;
                    const uint32_t page = (uint32_t)__builtin_amdgcn_readlane((int)my_page, (step_i % SPC) * TPI + u);
                    if (t + u < te && page < (uint32_t)Np_) row0[u] = (long)page * a.P + ((t + u) % tiles_per_page) * TR;
                }
#pragma unroll
                for (int u = 0; u < TPI; ++u) {
#pragma unroll
                    for (int i = 0; i < RPL; ++i) {
                        const long row = row0[u] + i * RPW + rg;
                        if (row < T_valid_) {
                            if (a.nt_kv & 1) {
                                kr[u][i] = R::load_raw_nt(kb + row * D + c0);
                                vr[u][i] = R::load_raw_nt(vb + row * D + c0);
                            } else {
                                kr[u][i] = R::load_raw(kb + row * D + c0);
                                vr[u][i] = R::load_raw(vb + row * D + c0);
                            }
                        } else {
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
                        const float d = group_sum<LPR>(qd.dot(kr[u][i])) * a.scale;
                        const long row = row0[u] + i * RPW + rg;
                        s[i] = (row < T_valid_) ? d : -INFINITY;
                        mt = fmaxf(mt, s[i]);
                    }
                    if (mt != -INFINITY) {
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

            mark(item, 5);
            // merge the row groups of the wave, then the waves through LDS
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
                if (cl == 0) {
                    s_m[wave] = m;
                    s_l[wave] = l;
                }
#pragma unroll
                for (int c = 0; c < 8; ++c) s_o[wave][c0 + c] = o[c];
            }
            __syncthreads();
            float M = -INFINITY, L = 0.f, O = 0.f;
            if (tid < D) {
#pragma unroll
                for (int w = 0; w < kFusedWaves; ++w) M = fmaxf(M, s_m[w]);
#pragma unroll
                for (int w = 0; w < kFusedWaves; ++w) {
                    const float aw = (s_m[w] == -INFINITY) ? 0.f : __expf(s_m[w] - M);
                    L += s_l[w] * aw;
                    O += s_o[w][tid] * aw;
                }
            }
            if (!finish) {
                uint64_t *part = a.partial + ((long)unit * a.S_max + slice) * (D + 2);
                if (tid < D) {
                    publish_f32(&part[2 + tid], O, tag_);
                    if (tid == 0) {
                        publish_f32(&part[0], M, tag_);
                        publish_f32(&part[1], L, tag_);
                    }
                }
            } else if (S_att > 1) {
                // the other slices' partials: the kFusedThreads / D thread groups take every NG-th one each
                // (one round trip for up to 4 NG partials instead of one per four), then fold through LDS
                // (the selection's scratch is free during an attend item)
                constexpr int NG = kFusedThreads / D;
                static_assert(sizeof(SelectShared<kFusedThreads>) >= sizeof(float) * 3 * NG * D, "fold buffer");
                float *fold = reinterpret_cast<float *>(&sh);
                const int g = tid / D, ch = tid % D;
                float Mg = -INFINITY, Lg = 0.f, Og = 0.f;
                if (g == 0) {
                    Mg = M;
                    Lg = L;
                    Og = O;
                }
                merge_partials(a.partial + (long)unit * a.S_max * (D + 2), S_att - 1, D + 2, ch, tag_, a.spin_limit,
                               a.err, Mg, Lg, Og, g, NG);
                if (g > 0) {
                    fold[(g * 3 + 0) * D + ch] = Mg;
                    fold[(g * 3 + 1) * D + ch] = Lg;
                    fold[(g * 3 + 2) * D + ch] = Og;
                }
                __syncthreads();
                if (g == 0) {
#pragma unroll
                    for (int gg = 1; gg < NG; ++gg) {
                        const float m2 = fold[(gg * 3 + 0) * D + ch], l2 = fold[(gg * 3 + 1) * D + ch],
                                    o2 = fold[(gg * 3 + 2) * D + ch];
                        const float mn = fmaxf(Mg, m2);
                        const float a1 = (Mg == -INFINITY) ? 0.f : __expf(Mg - mn);
                        const float a2 = (m2 == -INFINITY) ? 0.f : __expf(m2 - mn);
                        Lg = Lg * a1 + l2 * a2;
                        Og = Og * a1 + o2 * a2;
                        Mg = mn;
                    }
                    M = Mg;
                    L = Lg;
                    O = Og;
                }
            }
            mark(item, 6);
            if (finish && tid < D) {
                const float inv = (L > 0.f) ? 1.f / L : 0.f;
                from_f32(((ST *)a.out)[(long)unit * D + tid], O * inv);
                if (tid == 0 && a.lse_out) a.lse_out[unit] = (L > 0.f) ? M + __logf(L) : -INFINITY;
            }
        }
        fetch_next();
        __syncthreads();
        item = s_next;
    }

    if (tid == 0) {
        if (atomicAdd(a.done, 1u) == gridDim.x - 1u) {  // last workgroup out resets the counters
            atomicExch(a.ticket, 0u);
            atomicExch(a.done, 0u);
            if constexpr (STATE) {  // every workgroup has read the state: the next step's length and tag
                *reinterpret_cast<long *>(a.state + kCtrlStateT) = T_valid_;
                const uint32_t nt = tag_ + 0x85EBCA6Bu;
                a.state[kCtrlStateTag] = nt ? nt : 0x5bd1e995u;
            }
        }
    }
}

template <typename ST, int D, int NT>
static int launch_fused(const FusedParams &prm, int np_lds, int grid, hipStream_t stream)
{
    if (np_lds > 15360) return RS_UNSUPPORTED;  // keys must fit 60 KiB of LDS
    if (prm.state) decode_fused_kernel<ST, D, NT, true><<<grid, NT, (size_t)np_lds * 4, stream>>>(prm);
    else decode_fused_kernel<ST, D, NT, false><<<grid, NT, (size_t)np_lds * 4, stream>>>(prm);
    return RS_OK;
}

int decode_fused_dispatch(int dtype, int D, const FusedParams &prm, int np_lds, int grid, hipStream_t stream)
{
    // two 512-thread workgroups per CU: one streams while the other selects or merges
    if (dtype == RS_BF16) return D == 128 ? launch_fused<bf16, 128, 512>(prm, np_lds, grid, stream) : launch_fused<bf16, 64, 512>(prm, np_lds, grid, stream);
    return D == 128 ? launch_fused<float, 128, 512>(prm, np_lds, grid, stream) : launch_fused<float, 64, 512>(prm, np_lds, grid, stream);
}

}  // namespace rs
