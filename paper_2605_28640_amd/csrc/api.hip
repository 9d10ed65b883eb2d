// C ABI of the library: argument validation, workspace layout, kernel dispatch.
#include <atomic>
#include <chrono>
#include <cstdlib>

#include <mutex>

#include "common.h"
#include "decode_fused.h"
#include "knobs.h"

namespace rs {
// scan.hip
int scan_chunk_tokens(int dtype, int D);
bool scan_writes_meta(int dtype, int D, int P, int BH, long T_new, long t0);
bool scan_uses_step_kernel(long T_new);
void scan_dispatch(int dtype, int D, const void *k, const void *v, const float *g, float *state_k,
                   float *state_v, void *k_cache, void *v_cache, void *meta, int P, int BH, long T_new, long t0,
                   long Tcap, uint32_t *ctrl, uint64_t *rec, uint32_t tag, int spin_limit, hipStream_t stream);
// quest.hip
void page_meta_dispatch(int dtype, int D, const void *k_cache, void *meta, int BH, long Tcap, int P,
                        int p_begin, int n_pages, long t_end, hipStream_t stream);
void step_at_state_dispatch(int dtype, int D, const void *k, const void *v, const float *g, float *state_k,
                            float *state_v, void *k_cache, void *v_cache, void *meta, int P, int BH, long Tcap,
                            const uint32_t *pos_state, long T_max, int K, hipStream_t stream);
void unit_decode_dispatch(int dtype, int D, const void *q, const void *meta, const void *k_cache, const void *v_cache,
                          void *out, float *lse_out, int32_t *idx_out, int B, int Hq, int Hkv, long Tcap, int P,
                          long T_valid, int Np, int K, int n_first, int n_local, float scale, uint32_t *state,
                          hipStream_t stream);
int score_select_dispatch(int dtype, int D, int GQ, const void *q, const void *meta, uint64_t *scores,
                          float *scores_out, int32_t *idx_out, int B, int Hq, int Hkv, long Np_cap, int Np, int K,
                          int n_first, int n_local, int splits, uint32_t *unit_ctr, uint32_t *err, uint32_t tag,
                          int spin_limit, const uint32_t *state, long T_max, int P, hipStream_t stream);
void decode_attend_dispatch(int dtype, int D, const void *q, const void *k_cache, const void *v_cache,
                            const int32_t *idx, void *out, float *lse_out, uint64_t *partial, int B, int Hq,
                            int Hkv, long Tcap, int P, long T_valid, int K, float scale, int splits,
                            uint32_t *unit_ctr, uint32_t *err, uint32_t tag, int spin_limit, int idx_per_kv,
                            uint32_t *state, long T_max, hipStream_t stream);
// moba.hip / prefill.hip / snapkv.hip
size_t moba_select_ws_bytes(const rs_shape *s, long T, int block);
int moba_select_dispatch(const rs_shape *s, const void *q, const void *k_cache, long T, int block, int K,
                         int n_first, float *means_out, int32_t *idx_out, char *ws, hipStream_t stream);
size_t prefill_ws_bytes(const rs_shape *s, long T, int block, int K);
int prefill_dispatch(const rs_shape *s, const void *q, const void *k_cache, const void *v_cache, long T,
                     int block, float scale, const int32_t *idx, int K, void *out, float *lse_out, char *ws,
                     hipStream_t stream);
size_t snapkv_ws_bytes(const rs_shape *s, long T, int W);
int snapkv_dispatch(const rs_shape *s, const void *q_win, const void *k_cache, const void *v_cache, long T,
                    int W, int K_keep, int pool_kernel, float scale, void *kc_out, void *vc_out, long Tcap_out,
                    int32_t *idx_out, float *votes_out, const float *lse_in, char *ws, hipStream_t stream);

__global__ void fill_zero_kernel(uint32_t *p, long n)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__global__ void decode_state_set_kernel(uint32_t *ctrl, long T, uint32_t tag)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *reinterpret_cast<long *>(ctrl + kCtrlStateT) = T;
        ctrl[kCtrlStateTag] = tag;
    }
}

static std::atomic<int> g_spin_limit{1 << 22};
static std::atomic<uint32_t> g_epoch{0};

static uint32_t next_tag()
{
    // a fresh 32-bit tag per call: records left in a workspace by earlier calls, or
    // whatever else the memory held, do not match it
    uint32_t e = g_epoch.load();
    if (e == 0) {
        const uint64_t now = (uint64_t)std::chrono::steady_clock::now().time_since_epoch().count();
        uint32_t seed = (uint32_t)(now ^ (now >> 32)) | 1u;
        g_epoch.compare_exchange_strong(e, seed);
    }
    uint32_t t = g_epoch.fetch_add(0x9E3779B1u) + 0x9E3779B1u;
    return t ? t : 0x5bd1e995u;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static size_t esize(int dtype) { return dtype == RS_BF16 ? 2 : 4; }

static int check_shape(const rs_shape *s, bool need_page)
{
    if (!s) return RS_INVALID_ARG;
    if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->Tcap <= 0) return RS_INVALID_ARG;
    if (s->Hq % s->Hkv != 0) return RS_INVALID_ARG;
    if (s->dtype != RS_F32 && s->dtype != RS_BF16) return RS_UNSUPPORTED;
    if (s->D != 64 && s->D != 128) return RS_UNSUPPORTED;
    if (need_page) {
        if (s->P != 16 && s->P != 32 && s->P != 64 && s->P != 128 && s->P != 256 && s->P != 512) return RS_UNSUPPORTED;
        if (s->Tcap % s->P != 0) return RS_INVALID_ARG;
    }
    if ((long)s->B * s->Hq > kMaxUnits) return RS_UNSUPPORTED;
    return RS_OK;
}

static int launch_status() { return hipGetLastError() == hipSuccess ? RS_OK : RS_LAUNCH_FAILED; }

// work split of the two-launch kernels: `target_wgs` workgroups in all (about one 512-thread
// workgroup per CU), never less than `min_items_per_split` items in a split
static int pick_splits(long units, long items, long min_items_per_split, long target_wgs)
{
    long s = (target_wgs + units - 1) / units;
    const long cap = items / min_items_per_split;
    if (s > cap) s = cap;
    if (s < 1) s = 1;
    if (s > 1024) s = 1024;
    return (int)s;
}

static int num_cus()
{
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}

static int env_or_unset(const char *name)
{
    const char *e = std::getenv(name);
    return e ? std::atoi(e) : kKnobUnset;
}

static Knobs g_knobs;
static std::once_flag g_knobs_once;

static void knobs_read()
{
    Knobs &k = g_knobs;
    k.score_wgs = env_or_unset("RATSPARSE_SCORE_WGS");
    k.attend_wgs = env_or_unset("RATSPARSE_ATTEND_WGS");
    k.fused_grid = env_or_unset("RATSPARSE_FUSED_GRID");
    k.fused_sscore = env_or_unset("RATSPARSE_FUSED_SSCORE");
    k.fused_satt = env_or_unset("RATSPARSE_FUSED_SATT");
    k.fused_fine = env_or_unset("RATSPARSE_FUSED_FINE");
    k.fused_fine_pct = env_or_unset("RATSPARSE_FUSED_FINE_PCT");
    k.fused_nt = env_or_unset("RATSPARSE_FUSED_NT");
    k.fused_pingpong = env_or_unset("RATSPARSE_FUSED_PINGPONG");
    k.fused_two_launch = env_or_unset("RATSPARSE_FUSED_TWO_LAUNCH");
    k.fused_one_wg = env_or_unset("RATSPARSE_FUSED_ONE_WG");
    k.scan_grid = env_or_unset("RATSPARSE_SCAN_GRID");
    k.scan_slab = env_or_unset("RATSPARSE_SCAN_SLAB");
    k.scan_meta = env_or_unset("RATSPARSE_SCAN_META");
    k.meta_spw = env_or_unset("RATSPARSE_META_SPW");
    k.gate_waves = env_or_unset("RATSPARSE_GATE_WAVES");
    k.gate_wgs = env_or_unset("RATSPARSE_GATE_WGS");
    k.gate_shared = env_or_unset("RATSPARSE_GATE_SHARED");
    k.prefill_masked = env_or_unset("RATSPARSE_PREFILL_MASKED");
    k.prefill_grid = env_or_unset("RATSPARSE_PREFILL_GRID");
    k.snap_one_wg = env_or_unset("RATSPARSE_SNAP_ONE_WG");
}

const Knobs &knobs()
{
    std::call_once(g_knobs_once, knobs_read);
    return g_knobs;
}

void knobs_reload()
{
    (void)knobs();
    knobs_read();
}

constexpr int kMaxAttSplits = 64;

struct DecodeLayout {
    int Np, splits_score, splits_att_max;
    size_t off_scores, off_idx, off_idx_tagged, off_partial, off_trace, total;
};

static DecodeLayout decode_layout(const rs_shape *s, long T_valid, int K)
{
    DecodeLayout L;
    const long units = (long)s->B * s->Hq;
    L.Np = (int)((T_valid + s->P - 1) / s->P);
    // 512-thread workgroups, about one per CU (128 pages per workgroup step)
    L.splits_score = pick_splits(units, L.Np, 128, knob_or(knobs().score_wgs, 256));
    const long dense_tiles = (T_valid + 15) / 16;
    L.splits_att_max = pick_splits(units, dense_tiles, 8, knob_or(knobs().attend_wgs, 512));
    if (L.splits_att_max < kMaxAttSplits) L.splits_att_max = kMaxAttSplits;
    size_t off = RS_WS_CTRL_BYTES;
    L.off_scores = off;
    off += align256((size_t)units * L.Np * 8);
    L.off_idx = off;
    off += align256((size_t)units * (K > 0 ? K : 1) * 4);
    L.off_idx_tagged = off;
    off += align256((size_t)units * (K > 0 ? K : 1) * 8);
    L.off_partial = off;
    off += align256((size_t)units * L.splits_att_max * (s->D + 2) * 8);
    L.off_trace = off;
#ifdef RS_FUSED_TRACE
    off += (size_t)4096 * 64 * 8;
#endif
    L.total = off;
    return L;
}

// work split and buffers of the one-launch decode (score -> select -> attend) for a sequence of
// T_valid tokens laid out by L; returns the grid
static long fused_setup(FusedParams &prm, const rs_shape *s, const DecodeLayout &L, char *w, const void *q,
                        const void *meta, const void *k_cache, const void *v_cache, void *out, float *lse_out,
                        int32_t *idx_out, long T_valid, int K, int n_first, int n_local, float scale,
                        uint32_t *err = nullptr)
{
    const long units = (long)s->B * s->Hq;
    uint32_t *ctr_score = (uint32_t *)w + kCtrlUnit0;
    uint32_t *ctr_att = ctr_score + kMaxUnits;
    prm.q = q; prm.meta = meta; prm.k_cache = k_cache; prm.v_cache = v_cache;
    prm.out = out; prm.lse_out = lse_out; prm.idx_out = idx_out;
    prm.scores = (uint64_t *)(w + L.off_scores);
    prm.idx_tagged = (uint64_t *)(w + L.off_idx_tagged);
    prm.partial = (uint64_t *)(w + L.off_partial);
    prm.ctr_score = ctr_score; prm.ctr_att = ctr_att;
    prm.ticket = (uint32_t *)w + kCtrlTicket; prm.done = (uint32_t *)w + kCtrlDone;
    prm.err = err ? err : (uint32_t *)w + kCtrlAsyncErr;
    prm.Hq = s->Hq; prm.Hkv = s->Hkv; prm.units = (int)units;
    prm.Tcap = s->Tcap; prm.Np_cap = s->Tcap / s->P; prm.T_valid = T_valid;
    prm.P = s->P; prm.Np = L.Np; prm.K = K; prm.n_first = n_first; prm.n_local = n_local;
    const Knobs &kn = knobs();
    int ss = knob_or(kn.fused_sscore, 0), sa = knob_or(kn.fused_satt, 0);
    if (ss <= 0) ss = (L.Np + 351) / 352;                      // ~350 pages (176 KiB of bf16 metadata) per item
    if (sa <= 0) sa = (int)(((long)K * (s->P / 16) + 31) / 32);  // ~32 tiles (256 KiB of bf16 K+V) per item
    if (ss > L.Np) ss = L.Np;
    if (sa > kMaxAttSplits) sa = kMaxAttSplits;
    if (sa > K) sa = K;
    prm.S_score = ss < 1 ? 1 : ss; prm.S_att = sa < 1 ? 1 : sa;
    int fine = knob_or(kn.fused_fine, 2) * prm.S_att;
    if (fine > kMaxAttSplits) fine = kMaxAttSplits;
    if (fine > K) fine = K;
    prm.S_att_fine = fine < prm.S_att ? prm.S_att : fine;
    int fine_pct = knob_or(kn.fused_fine_pct, 6);
    fine_pct = fine_pct < 0 ? 0 : fine_pct > 100 ? 100 : fine_pct;
    prm.units_fine = (int)(units * fine_pct / 100);
    prm.S_max = kMaxAttSplits;
    prm.reverse = knob_or(kn.fused_pingpong, 1) ? (int)(T_valid & 1) : 0;
    prm.nt_kv = knob_or(kn.fused_nt, 1);  // bit 0: K/V pages, bit 1: page metadata
    prm.scale = scale; prm.tag = 0; prm.spin_limit = g_spin_limit.load();
#ifdef RS_FUSED_TRACE
    prm.trace = (uint64_t *)(w + L.off_trace);
#else
    prm.trace = nullptr;
#endif
    prm.state = nullptr; prm.T_max = 0;
    const long items = units * (prm.S_score + prm.S_att) + (long)prm.units_fine * (prm.S_att_fine - prm.S_att);
    long grid = knob_or(kn.fused_grid, 2 * num_cus());
    if (grid > items) grid = items;
    if (grid < 1) grid = 1;
    return grid;
}

}  // namespace rs

using namespace rs;

namespace rs {
template <bool NT>
__global__ __launch_bounds__(512) void probe_read_kernel(const uint4 *__restrict__ src, size_t n16, size_t per_wg,
                                                         uint32_t *sink)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    // each workgroup streams one contiguous slice, eight 16-byte loads in flight per thread
    const size_t b = (size_t)blockIdx.x * per_wg;
    const size_t e = (b + per_wg < n16) ? b + per_wg : n16;
    uint32_t acc = 0u;
    for (size_t i = b + threadIdx.x; i < e; i += (size_t)512 * 8) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t j = i + (size_t)u * 512;
            v[u] = make_uint4(0u, 0u, 0u, 0u);
            if (j < e) {
                if constexpr (NT) {  // streaming loads, as the decode kernels use for K and V pages
                    const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src) + j);
                    v[u] = make_uint4(w.x, w.y, w.z, w.w);
                } else {
                    v[u] = src[j];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;  // keeps the loads alive; practically never taken
}
// two read streams, one write stream (the byte mix of the scan: 8 bytes read, 4 written per
// channel-token): dst = a ^ b in 16-byte pieces, a contiguous slice per workgroup; NT: with
// streaming (non-temporal) loads and stores, as the scan itself uses
template <bool NT>
__global__ __launch_bounds__(512) void probe_rw_kernel(const uint4 *__restrict__ a, const uint4 *__restrict__ b,
                                                       uint4 *__restrict__ dst, size_t n16, size_t per_wg)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const size_t lo = (size_t)blockIdx.x * per_wg;
    const size_t hi = (lo + per_wg < n16) ? lo + per_wg : n16;
    for (size_t i = lo + threadIdx.x; i < hi; i += (size_t)512 * 4) {
        u32x4 x[4], y[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const size_t j = i + (size_t)u * 512;
            x[u] = u32x4{0u, 0u, 0u, 0u};
            y[u] = x[u];
            if (j < hi) {
                if constexpr (NT) {
                    x[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a) + j);
                    y[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(b) + j);
                } else {
                    x[u] = reinterpret_cast<const u32x4 *>(a)[j];
                    y[u] = reinterpret_cast<const u32x4 *>(b)[j];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const size_t j = i + (size_t)u * 512;
            if (j < hi) {
                const u32x4 r = x[u] ^ y[u];
                if constexpr (NT) __builtin_nontemporal_store(r, reinterpret_cast<u32x4 *>(dst) + j);
                else reinterpret_cast<u32x4 *>(dst)[j] = r;
            }
        }
    }
}
}  // namespace rs

extern "C" {

const char *ratsparse_status_string(int32_t status)
{
    switch (status) {
        case RS_OK: return "ok";
        case RS_INVALID_ARG: return "invalid argument";
        case RS_UNSUPPORTED: return "unsupported shape or dtype";
        case RS_WORKSPACE_TOO_SMALL: return "workspace too small";
        case RS_LAUNCH_FAILED: return "kernel launch failed";
        case RS_ASYNC_TIMEOUT: return "a bounded in-kernel wait expired";
        case RS_SCRATCH_LIMIT: return "the shape needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

const char *ratsparse_version(void) { return "ratsparse 0.1 (gfx950)"; }

// measurement aid: a plain streaming read of `bytes` bytes (16-byte loads, a contiguous slice
// per workgroup), the ceiling a read-bound kernel can be held against on this machine
int32_t ratsparse_probe_read(const void *src, size_t bytes, void *sink, int32_t streaming, void *stream)
{
    if (!src || !sink || !aligned16(src) || bytes < 16) return RS_INVALID_ARG;
    const size_t n16 = bytes / 16;
    size_t blocks = (size_t)num_cus() * 4;
    if (blocks * 512 > n16) blocks = (n16 + 511) / 512;
    const size_t per_wg = (n16 + blocks - 1) / blocks;
    if (streaming)
        probe_read_kernel<true><<<(unsigned)blocks, 512, 0, (hipStream_t)stream>>>((const uint4 *)src, n16, per_wg, (uint32_t *)sink);
    else
        probe_read_kernel<false><<<(unsigned)blocks, 512, 0, (hipStream_t)stream>>>((const uint4 *)src, n16, per_wg, (uint32_t *)sink);
    return launch_status();
}

// measurement aid: a plain streaming kernel with the scan's traffic mix (reads 2 x bytes, writes bytes)
int32_t ratsparse_probe_rw(const void *a, const void *b, void *dst, size_t bytes, int32_t streaming, void *stream)
{
    if (!a || !b || !dst || !aligned16(a) || !aligned16(b) || !aligned16(dst) || bytes < 16) return RS_INVALID_ARG;
    const size_t n16 = bytes / 16;
    size_t blocks = (size_t)num_cus() * 8;
    if (blocks * 512 > n16) blocks = (n16 + 511) / 512;
    const size_t per_wg = (n16 + blocks - 1) / blocks;
    if (streaming)
        probe_rw_kernel<true><<<(unsigned)blocks, 512, 0, (hipStream_t)stream>>>((const uint4 *)a, (const uint4 *)b, (uint4 *)dst, n16, per_wg);
    else
        probe_rw_kernel<false><<<(unsigned)blocks, 512, 0, (hipStream_t)stream>>>((const uint4 *)a, (const uint4 *)b, (uint4 *)dst, n16, per_wg);
    return launch_status();
}

// test hook: bound of the scan's in-kernel wait, in polls
void ratsparse_debug_set_spin_limit(int32_t polls) { g_spin_limit.store(polls < 0 ? 0 : polls); }

// test hook: read the RATSPARSE_* tuning variables again (they are otherwise read once per process)
void ratsparse_debug_reload_knobs(void) { knobs_reload(); }

int32_t ratsparse_workspace_init(void *ws, size_t ws_bytes, void *stream)
{
    if (!ws || !aligned16(ws)) return RS_INVALID_ARG;
    if (ws_bytes < RS_WS_CTRL_BYTES) return RS_WORKSPACE_TOO_SMALL;
    const long n = RS_WS_CTRL_BYTES / 4;
    fill_zero_kernel<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>((uint32_t *)ws, n);
    return launch_status();
}

int32_t ratsparse_async_status(void *ws, void *stream)
{
    if (!ws) return RS_INVALID_ARG;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return RS_LAUNCH_FAILED;
    uint32_t flag = 0;
    if (hipMemcpy(&flag, ws, 4, hipMemcpyDeviceToHost) != hipSuccess) return RS_LAUNCH_FAILED;
    if (flag) {
        fill_zero_kernel<<<1, 64, 0, (hipStream_t)stream>>>((uint32_t *)ws, 3);  // error word and scan counters
        (void)hipStreamSynchronize((hipStream_t)stream);
        return RS_ASYNC_TIMEOUT;
    }
    return RS_OK;
}

size_t rat_scan_workspace_bytes(const rs_shape *s, int64_t T_new)
{
    if (check_shape(s, false) != RS_OK || T_new <= 0) return 0;
    const long chunk = scan_chunk_tokens(s->dtype, s->D);
    const long n_chunks = (T_new + chunk - 1) / chunk;
    return RS_WS_CTRL_BYTES + align256((size_t)s->B * s->Hkv * n_chunks * 2 * s->D * 8);
}

int32_t rat_scan(const rs_shape *s, const void *k, const void *v, const float *g, float *state_k,
                 float *state_v, void *k_cache, void *v_cache, void *meta, int64_t t0, int64_t T_new, void *ws,
                 size_t ws_bytes, void *stream)
{
    int st = check_shape(s, meta != nullptr);
    if (st != RS_OK) return st;
    if (meta && !aligned16(meta)) return RS_INVALID_ARG;
    if (!k || !v || !g || !state_k || !state_v || !k_cache || !v_cache) return RS_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(state_k) || !aligned16(state_v) ||
        !aligned16(k_cache) || !aligned16(v_cache))
        return RS_INVALID_ARG;
    if (T_new <= 0 || t0 < 0 || t0 + T_new > s->Tcap) return RS_INVALID_ARG;
    const long BH = (long)s->B * s->Hkv;
    const long chunk = scan_chunk_tokens(s->dtype, s->D);
    const long n_chunks = (T_new + chunk - 1) / chunk;
    if (BH * n_chunks > 0x7fffffffL) return RS_UNSUPPORTED;
    uint32_t *ctrl = nullptr;
    uint64_t *rec = nullptr;
    if (!scan_uses_step_kernel(T_new) && n_chunks > 1) {
        if (!ws || !aligned16(ws) || ws_bytes < rat_scan_workspace_bytes(s, T_new)) return RS_WORKSPACE_TOO_SMALL;
        ctrl = (uint32_t *)ws;
        rec = (uint64_t *)((char *)ws + RS_WS_CTRL_BYTES);
    }
    // the page bounds leave with the states where the kernel can do that (one token: always; long
    // runs: full-row form, a page size that tiles the chunk, chunk-aligned start); else a pass over the touched pages
    const bool in_scan = meta && scan_writes_meta(s->dtype, s->D, s->P, (int)BH, T_new, t0);
    scan_dispatch(s->dtype, s->D, k, v, g, state_k, state_v, k_cache, v_cache, in_scan ? meta : nullptr, s->P, (int)BH,
                  T_new, t0, s->Tcap, ctrl, rec, next_tag(), g_spin_limit.load(), (hipStream_t)stream);
    if (meta && !in_scan) {  // the pages the new rows touch are recomputed after the scan
        const int p_begin = (int)(t0 / s->P);
        const int p_end = (int)((t0 + T_new + s->P - 1) / s->P);
        page_meta_dispatch(s->dtype, s->D, k_cache, meta, (int)BH, s->Tcap, s->P, p_begin, p_end - p_begin, t0 + T_new,
                           (hipStream_t)stream);
    }
    return launch_status();
}

int32_t quest_page_meta(const rs_shape *s, const void *k_cache, void *meta, int64_t t_begin, int64_t t_end,
                        void *stream)
{
    int st = check_shape(s, true);
    if (st != RS_OK) return st;
    if (!k_cache || !meta || !aligned16(k_cache) || !aligned16(meta)) return RS_INVALID_ARG;
    if (t_begin < 0 || t_end <= t_begin || t_end > s->Tcap) return RS_INVALID_ARG;
    const int p_begin = (int)(t_begin / s->P);
    const int p_end = (int)((t_end + s->P - 1) / s->P);
    page_meta_dispatch(s->dtype, s->D, k_cache, meta, s->B * s->Hkv, s->Tcap, s->P, p_begin, p_end - p_begin, t_end,
                       (hipStream_t)stream);
    return launch_status();
}

static int check_select(const rs_shape *s, int64_t T_valid, int K, int n_first, int n_local)
{
    if (T_valid <= 0 || T_valid > s->Tcap) return RS_INVALID_ARG;
    const long Np = (T_valid + s->P - 1) / s->P;
    if (K < 1 || K > Np || n_first < 0 || n_local < 0) return RS_INVALID_ARG;
    long forced = (long)n_first + n_local;
    if (forced > Np) forced = Np;
    if (forced > K) return RS_INVALID_ARG;
    return RS_OK;
}

size_t quest_select_decode_workspace_bytes(const rs_shape *s, int64_t T_valid)
{
    if (check_shape(s, true) != RS_OK || T_valid <= 0) return 0;
    return decode_layout(s, T_valid, 1).total;
}

// group: one page list per (batch, KV head) from the summed scores of its query heads
static int32_t select_decode_impl(bool group, const rs_shape *s, const void *q, const void *meta, int64_t T_valid,
                                  int32_t K, int32_t n_first, int32_t n_local, int32_t *idx_out, float *scores_out,
                                  void *ws, size_t ws_bytes, void *stream)
{
    int st = check_shape(s, true);
    if (st != RS_OK) return st;
    const int GQ = group ? s->Hq / s->Hkv : 1;
    if (GQ != 1 && GQ != 2 && GQ != 4 && GQ != 8) return RS_UNSUPPORTED;
    if (!q || !meta || !idx_out || !aligned16(q) || !aligned16(meta) || !aligned16(idx_out)) return RS_INVALID_ARG;
    if (scores_out && !aligned16(scores_out)) return RS_INVALID_ARG;
    st = check_select(s, T_valid, K, n_first, n_local);
    if (st != RS_OK) return st;
    const DecodeLayout L = decode_layout(s, T_valid, 1);
    if (!ws || !aligned16(ws) || ws_bytes < L.total) return RS_WORKSPACE_TOO_SMALL;
    char *w = (char *)ws;
    st = score_select_dispatch(s->dtype, s->D, GQ, q, meta, (uint64_t *)(w + L.off_scores), scores_out, idx_out,
                               s->B, s->Hq, s->Hkv, s->Tcap / s->P, L.Np, K, n_first, n_local, L.splits_score,
                               (uint32_t *)w + kCtrlUnit0, (uint32_t *)w + kCtrlAsyncErr, next_tag(),
                               g_spin_limit.load(), nullptr, 0, s->P, (hipStream_t)stream);
    if (st != RS_OK) return st;
    return launch_status();
}

int32_t quest_select_decode(const rs_shape *s, const void *q, const void *meta, int64_t T_valid, int32_t K,
                            int32_t n_first, int32_t n_local, int32_t *idx_out, float *scores_out, void *ws,
                            size_t ws_bytes, void *stream)
{
    return select_decode_impl(false, s, q, meta, T_valid, K, n_first, n_local, idx_out, scores_out, ws, ws_bytes,
                              stream);
}

int32_t quest_select_decode_group(const rs_shape *s, const void *q, const void *meta, int64_t T_valid, int32_t K,
                                  int32_t n_first, int32_t n_local, int32_t *idx_out, float *scores_out, void *ws,
                                  size_t ws_bytes, void *stream)
{
    return select_decode_impl(true, s, q, meta, T_valid, K, n_first, n_local, idx_out, scores_out, ws, ws_bytes,
                              stream);
}

size_t sparse_attn_decode_workspace_bytes(const rs_shape *s, int64_t T_valid, int32_t K)
{
    if (check_shape(s, true) != RS_OK || T_valid <= 0) return 0;
    return decode_layout(s, T_valid, K).total;
}

static int32_t attn_decode_impl(bool group, const rs_shape *s, const void *q, const void *k_cache, const void *v_cache,
                                int64_t T_valid, float scale, const int32_t *idx, int32_t K, const void *meta,
                                int32_t n_first, int32_t n_local, void *out, float *lse_out, int32_t *idx_out,
                                void *ws, size_t ws_bytes, void *stream, uint32_t *err_word = nullptr)
{
    int st = check_shape(s, true);
    if (st != RS_OK) return st;
    const int GQ = group ? s->Hq / s->Hkv : 1;
    if (GQ != 1 && GQ != 2 && GQ != 4 && GQ != 8) return RS_UNSUPPORTED;
    if (!q || !k_cache || !v_cache || !out) return RS_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return RS_INVALID_ARG;
    if (T_valid <= 0 || T_valid > s->Tcap) return RS_INVALID_ARG;
    const bool listed = idx != nullptr, fused = !listed && meta != nullptr;
    const long Np = (T_valid + s->P - 1) / s->P;
    if (listed && (K < 1 || K > Np || !aligned16(idx))) return RS_INVALID_ARG;
    if (fused) {
        st = check_select(s, T_valid, K, n_first, n_local);
        if (st != RS_OK) return st;
        if (!aligned16(meta) || (idx_out && !aligned16(idx_out))) return RS_INVALID_ARG;
    }
    const int Kws = (listed || fused) ? K : 0;
    const DecodeLayout L = decode_layout(s, T_valid, Kws);
    if (!ws || !aligned16(ws) || ws_bytes < L.total) return RS_WORKSPACE_TOO_SMALL;
    char *w = (char *)ws;
    uint32_t *ctr_score = (uint32_t *)w + kCtrlUnit0;
    uint32_t *ctr_att = ctr_score + kMaxUnits;
    uint32_t *err = err_word ? err_word : (uint32_t *)w + kCtrlAsyncErr;  // where an expired in-kernel wait is recorded
    const long units = (long)s->B * s->Hq;
    const int32_t *use_idx = idx;
    const uint32_t tag = next_tag();
    if (group && !listed && !fused) return RS_INVALID_ARG;  // the dense path has no selection to share
    // One persistent launch when the step is long enough to be bound by bandwidth: at least about
    // 450 MB of page metadata and selected pages (some 90 us) over at least 512 pages per sequence.
    // Shorter steps are bound by latency, and there the two plain launches below measured faster:
    // 32 heads at 4096 tokens, batch 8, 8 of 64 pages 23 against 38 us; batch 64 117 against 130 us;
    // 32 query over 8 KV heads at 32K, batch 1, 29 against 33 us.  Long ones the other way: batch 4
    // at 64K (538 MB) 95 against 143 us, batch 32 at 8K 98 against 112 us.
    const double step_bytes = ((double)s->B * s->Hkv * Np * 2 + (double)units * K * s->P * 2) * s->D * esize(s->dtype);
    const int two_launch = knob_or(knobs().fused_two_launch, (step_bytes >= 450e6 && Np >= 512) ? 0 : 1);
    // Short contexts (the paper's 4096 tokens): the whole step of a (batch, query head) inside one
    // workgroup, one launch, nothing handed between workgroups.  Taken when a unit's metadata and
    // picked pages are small (at most 1.5 MB, and at most 512 KB unless there are 128 units or
    // more) and the step is not one of the long ones above.  32 heads at 4096 tokens, 64-token
    // pages, top-8 (one workgroup per unit / two launches / persistent launch, us): batch 1
    // 13 / 16 / 21, batch 8 20 / 24 / 39, batch 64 112 / 123 / 130; 8K and 16K at batch 8:
    // 28 / 32 / 44 and 47 / 52 / 59; the other way at 32K, batch 2: 51 / 34 / 47.
    const double unit_bytes = ((double)Np * 2 + (double)K * s->P * 2) * s->D * esize(s->dtype);
    const bool unit_rule = two_launch && unit_bytes <= 1.5e6 && (units >= 128 || unit_bytes <= 512e3);
    const int one_wg = knob_or(knobs().fused_one_wg, unit_rule ? 1 : 0);
    if (fused && !group && one_wg && Np <= 4096 && K <= 1024) {
        unit_decode_dispatch(s->dtype, s->D, q, meta, k_cache, v_cache, out, lse_out, idx_out, s->B, s->Hq, s->Hkv,
                             s->Tcap, s->P, T_valid, (int)Np, K, n_first, n_local, scale, nullptr, (hipStream_t)stream);
        return launch_status();
    }
    if (fused && !group && !two_launch) {
        // one persistent launch: score -> select -> attend, handed over through tagged words
        FusedParams prm;
        const long grid = fused_setup(prm, s, L, w, q, meta, k_cache, v_cache, out, lse_out, idx_out, T_valid, K, n_first,
                                      n_local, scale, err);
        prm.tag = tag;
        st = decode_fused_dispatch(s->dtype, s->D, prm, L.Np, (int)grid, (hipStream_t)stream);
        if (st != RS_OK) return st;
        return launch_status();
    }
    if (fused) {
        int32_t *sel = idx_out ? idx_out : (int32_t *)(w + L.off_idx);
        st = score_select_dispatch(s->dtype, s->D, GQ, q, meta, (uint64_t *)(w + L.off_scores), nullptr, sel, s->B,
                                   s->Hq, s->Hkv, s->Tcap / s->P, L.Np, K, n_first, n_local, L.splits_score,
                                   ctr_score, err, tag, g_spin_limit.load(), nullptr, 0, s->P, (hipStream_t)stream);
        if (st != RS_OK) return st;
        if (launch_status() != RS_OK) return RS_LAUNCH_FAILED;
        use_idx = sel;
    }
    const long tiles = use_idx ? (long)K * (s->P / 16) : (T_valid + 15) / 16;
    // 512-thread workgroups, about one per CU: fewer, fuller workgroups start sooner and leave fewer
    // partials to merge than many small ones (32 query / 8 KV heads, batch 1: dense over 16.5K rows
    // 29 -> 25 us, over 32K rows 45 -> 41 us, 128 listed pages 13.7 -> 10.1 us against 256 threads
    // and 512 workgroups).  A wave takes two tiles per step: past 16 steps per wave, twice the splits.
    int target = knob_or(knobs().attend_wgs, 0);
    if (target <= 0) {
        target = 256;
        if (tiles > (long)pick_splits(units, tiles, 8, 256) * 8 * 2 * 16) target = 512;
    }
    int splits = pick_splits(units, tiles, 8, target);
    if (splits > L.splits_att_max) splits = L.splits_att_max;
    decode_attend_dispatch(s->dtype, s->D, q, k_cache, v_cache, use_idx, out, lse_out,
                           (uint64_t *)(w + L.off_partial), s->B, s->Hq, s->Hkv, s->Tcap, s->P, T_valid, K, scale,
                           splits, ctr_att, err, tag, g_spin_limit.load(), group ? 1 : 0, nullptr, 0, (hipStream_t)stream);
    return launch_status();
}

int32_t sparse_attn_decode(const rs_shape *s, const void *q, const void *k_cache, const void *v_cache,
                           int64_t T_valid, float scale, const int32_t *idx, int32_t K, const void *meta,
                           int32_t n_first, int32_t n_local, void *out, float *lse_out, int32_t *idx_out, void *ws,
                           size_t ws_bytes, void *stream)
{
    return attn_decode_impl(false, s, q, k_cache, v_cache, T_valid, scale, idx, K, meta, n_first, n_local, out,
                            lse_out, idx_out, ws, ws_bytes, stream);
}

int32_t sparse_attn_decode_group(const rs_shape *s, const void *q, const void *k_cache, const void *v_cache,
                                 int64_t T_valid, float scale, const int32_t *idx, int32_t K, const void *meta,
                                 int32_t n_first, int32_t n_local, void *out, float *lse_out, int32_t *idx_out,
                                 void *ws, size_t ws_bytes, void *stream)
{
    return attn_decode_impl(true, s, q, k_cache, v_cache, T_valid, scale, idx, K, meta, n_first, n_local, out,
                            lse_out, idx_out, ws, ws_bytes, stream);
}

// ---- the entry point that allocates nothing -------------------------------------------------
// sparse_attn_decode for callers that can neither allocate nor bring a workspace: its scratch
// (control words, tagged scores, tagged page lists, split partials) is the file-scope device
// array below.  In host code the array's name is only a stand-in: the device address is taken
// once per device with hipGetSymbolAddress and kept; kernels, clears and copies use that address.
}  // extern "C"

static __device__ __align__(256) unsigned char scratch[RS_STATIC_SCRATCH_BYTES];

namespace rs {
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];  // per device: the address of that device's copy of `scratch`
static std::mutex g_scratch_mutex;

// device address of the current device's scratch array (resolved on the first call per device)
static int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RS_LAUNCH_FAILED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return RS_LAUNCH_FAILED;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return RS_OK;
}
}  // namespace rs

extern "C" {

int32_t sparse_attn_decode_static(const rs_shape *s, const void *q, const void *k_cache, const void *v_cache,
                                  int64_t T_valid, float scale, const int32_t *idx, int32_t K, const void *meta,
                                  int32_t n_first, int32_t n_local, void *out, float *lse_out, int32_t *idx_out,
                                  uint32_t *async_err, void *stream)
{
    int st = check_shape(s, true);
    if (st != RS_OK) return st;
    if (T_valid <= 0 || T_valid > s->Tcap) return RS_INVALID_ARG;
    if (!async_err || (reinterpret_cast<uintptr_t>(async_err) & 3u)) return RS_INVALID_ARG;
    const bool uses_list = idx != nullptr || meta != nullptr;
    if (uses_list && K < 1) return RS_INVALID_ARG;
    // the layout sparse_attn_decode would ask a workspace for must fit the static array
    if (decode_layout(s, T_valid, uses_list ? K : 0).total > (size_t)RS_STATIC_SCRATCH_BYTES) return RS_SCRATCH_LIMIT;
    void *ptr = nullptr;
    st = static_scratch(&ptr);
    if (st != RS_OK) return st;
    // the array keeps what the last call (or a call that gave up a wait) left: the control words
    // must start at zero.  A fill kernel, not a memset, so that the call can sit in a captured graph.
    const long n = RS_WS_CTRL_BYTES / 4;
    fill_zero_kernel<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>((uint32_t *)ptr, n);
    if (launch_status() != RS_OK) return RS_LAUNCH_FAILED;
    return attn_decode_impl(false, s, q, k_cache, v_cache, T_valid, scale, idx, K, meta, n_first, n_local, out,
                            lse_out, idx_out, ptr, (size_t)RS_STATIC_SCRATCH_BYTES, stream, async_err);
}

size_t rat_decode_step_workspace_bytes(const rs_shape *s, int64_t T_max, int32_t K)
{
    if (check_shape(s, true) != RS_OK || T_max <= 0 || T_max > s->Tcap) return 0;
    return decode_layout(s, T_max, K).total;
}

int32_t rat_decode_state_set(void *ws, size_t ws_bytes, int64_t T, void *stream)
{
    if (!ws || !aligned16(ws) || T < 0) return RS_INVALID_ARG;
    if (ws_bytes < RS_WS_CTRL_BYTES) return RS_WORKSPACE_TOO_SMALL;
    decode_state_set_kernel<<<1, 64, 0, (hipStream_t)stream>>>((uint32_t *)ws, (long)T, next_tag());
    return launch_status();
}

int32_t rat_decode_state_get(void *ws, int64_t *T, void *stream)
{
    if (!ws || !T) return RS_INVALID_ARG;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return RS_LAUNCH_FAILED;
    long t = 0;
    if (hipMemcpy(&t, (const uint32_t *)ws + kCtrlStateT, 8, hipMemcpyDeviceToHost) != hipSuccess) return RS_LAUNCH_FAILED;
    *T = t;
    return RS_OK;
}

int32_t rat_decode_step(const rs_shape *s, const void *k, const void *v, const float *g, float *state_k,
                        float *state_v, void *k_cache, void *v_cache, void *meta, const void *q, float scale,
                        int32_t K, int32_t n_first, int32_t n_local, int64_t T_max, void *out, float *lse_out,
                        int32_t *idx_out, void *ws, size_t ws_bytes, void *stream)
{
    int st = check_shape(s, true);
    if (st != RS_OK) return st;
    if (!k || !v || !g || !state_k || !state_v || !k_cache || !v_cache || !meta || !q || !out) return RS_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v) || !aligned16(g) || !aligned16(state_k) || !aligned16(state_v) ||
        !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(meta) || !aligned16(q) || !aligned16(out) ||
        (idx_out && !aligned16(idx_out)))
        return RS_INVALID_ARG;
    if (T_max <= 0 || T_max > s->Tcap || K < 1 || n_first < 0 || n_local < 0) return RS_INVALID_ARG;
    if ((long)n_first + n_local > K) return RS_INVALID_ARG;  // holds at every length, whatever the page count
    const DecodeLayout L = decode_layout(s, T_max, K);
    if (K > L.Np) return RS_INVALID_ARG;
    if (L.Np > 15360) return RS_UNSUPPORTED;  // the selection's keys must fit the LDS: before any launch
    if (!ws || !aligned16(ws) || ws_bytes < L.total) return RS_WORKSPACE_TOO_SMALL;
    char *w = (char *)ws;
    step_at_state_dispatch(s->dtype, s->D, k, v, g, state_k, state_v, k_cache, v_cache, meta, s->P, s->B * s->Hkv,
                           s->Tcap, (const uint32_t *)w, T_max, K, (hipStream_t)stream);
    if (launch_status() != RS_OK) return RS_LAUNCH_FAILED;
    // the form of select-then-attend, by the shape at T_max and the rule of sparse_attn_decode: one workgroup per
    // (batch, query head) for short contexts, the persistent launch for long bandwidth-bound steps, the two plain
    // launches in between; all three read the length and the tag from the workspace's state words
    const long units = (long)s->B * s->Hq;
    const double step_bytes = ((double)s->B * s->Hkv * L.Np * 2 + (double)units * K * s->P * 2) * s->D * esize(s->dtype);
    const int two_launch = knob_or(knobs().fused_two_launch, (step_bytes >= 450e6 && L.Np >= 512) ? 0 : 1);
    const double unit_bytes = ((double)L.Np * 2 + (double)K * s->P * 2) * s->D * esize(s->dtype);
    const bool unit_rule = two_launch && unit_bytes <= 1.5e6 && (units >= 128 || unit_bytes <= 512e3);
    if (knob_or(knobs().fused_one_wg, unit_rule ? 1 : 0) && L.Np <= 4096 && K <= 1024) {
        unit_decode_dispatch(s->dtype, s->D, q, meta, k_cache, v_cache, out, lse_out, idx_out, s->B, s->Hq, s->Hkv,
                             s->Tcap, s->P, T_max, L.Np, K, n_first, n_local, scale, (uint32_t *)w, (hipStream_t)stream);
        return launch_status();
    }
    if (two_launch) {
        uint32_t *ctr_score = (uint32_t *)w + kCtrlUnit0;
        uint32_t *ctr_att = ctr_score + kMaxUnits;
        uint32_t *err = (uint32_t *)w + kCtrlAsyncErr;
        int32_t *sel = idx_out ? idx_out : (int32_t *)(w + L.off_idx);
        st = score_select_dispatch(s->dtype, s->D, 1, q, meta, (uint64_t *)(w + L.off_scores), nullptr, sel, s->B, s->Hq,
                                   s->Hkv, s->Tcap / s->P, L.Np, K, n_first, n_local, L.splits_score, ctr_score, err, 0u,
                                   g_spin_limit.load(), (const uint32_t *)w, T_max, s->P, (hipStream_t)stream);
        if (st != RS_OK) return st;
        if (launch_status() != RS_OK) return RS_LAUNCH_FAILED;
        const long tiles = (long)K * (s->P / 16);
        int target = knob_or(knobs().attend_wgs, 0);
        if (target <= 0) {
            target = 256;
            if (tiles > (long)pick_splits(units, tiles, 8, 256) * 8 * 2 * 16) target = 512;
        }
        int splits = pick_splits(units, tiles, 8, target);
        if (splits > L.splits_att_max) splits = L.splits_att_max;
        decode_attend_dispatch(s->dtype, s->D, q, k_cache, v_cache, sel, out, lse_out, (uint64_t *)(w + L.off_partial),
                               s->B, s->Hq, s->Hkv, s->Tcap, s->P, T_max, K, scale, splits, ctr_att, err, 0u,
                               g_spin_limit.load(), 0, (uint32_t *)w, T_max, (hipStream_t)stream);
        return launch_status();
    }
    FusedParams prm;
    const long grid = fused_setup(prm, s, L, w, q, meta, k_cache, v_cache, out, lse_out, idx_out, T_max, K, n_first,
                                  n_local, scale);
    prm.reverse = knob_or(knobs().fused_pingpong, 1);  // the kernel takes the parity of the length it reads
    prm.state = (uint32_t *)w;
    prm.T_max = T_max;
    st = decode_fused_dispatch(s->dtype, s->D, prm, L.Np, (int)grid, (hipStream_t)stream);
    if (st != RS_OK) return st;
    return launch_status();
}

size_t moba_select_prefill_workspace_bytes(const rs_shape *s, int64_t T, int32_t block)
{
    if (check_shape(s, false) != RS_OK || T <= 0 || block <= 0) return 0;
    return moba_select_ws_bytes(s, T, block);
}

int32_t moba_select_prefill(const rs_shape *s, const void *q, const void *k_cache, int64_t T, int32_t block,
                            int32_t K, int32_t n_first, float *means_out, int32_t *idx_out, void *ws,
                            size_t ws_bytes, void *stream)
{
    int st = check_shape(s, false);
    if (st != RS_OK) return st;
    if (!q || !k_cache || !means_out || !idx_out) return RS_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(means_out) || !aligned16(idx_out)) return RS_INVALID_ARG;
    if (T <= 0 || T > s->Tcap || block <= 0 || block % 16 != 0) return RS_INVALID_ARG;
    const long Nb = (T + block - 1) / block;
    if (Nb > 256) return RS_UNSUPPORTED;  // one LDS score column per thread in the gate kernel
    if (n_first < 0 || K < 1 + n_first || K > 32) return RS_INVALID_ARG;
    if (!ws || !aligned16(ws) || ws_bytes < moba_select_ws_bytes(s, T, block)) return RS_WORKSPACE_TOO_SMALL;
    return moba_select_dispatch(s, q, k_cache, T, block, K, n_first, means_out, idx_out, (char *)ws,
                                (hipStream_t)stream);
}

size_t sparse_attn_prefill_workspace_bytes(const rs_shape *s, int64_t T, int32_t block, int32_t K)
{
    if (check_shape(s, false) != RS_OK || T <= 0 || block <= 0) return 0;
    return prefill_ws_bytes(s, T, block, K);
}

int32_t sparse_attn_prefill(const rs_shape *s, const void *q, const void *k_cache, const void *v_cache, int64_t T,
                            int32_t block, float scale, const int32_t *idx, int32_t K, void *out, float *lse_out,
                            void *ws, size_t ws_bytes, void *stream)
{
    int st = check_shape(s, false);
    if (st != RS_OK) return st;
    if (!q || !k_cache || !v_cache || !out) return RS_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return RS_INVALID_ARG;
    if (T <= 0 || T > s->Tcap || block <= 0 || block % 16 != 0) return RS_INVALID_ARG;
    if (idx && (K < 1 || K > 32 || !aligned16(idx))) return RS_INVALID_ARG;
    if (!ws || !aligned16(ws) || ws_bytes < prefill_ws_bytes(s, T, block, K)) return RS_WORKSPACE_TOO_SMALL;
    return prefill_dispatch(s, q, k_cache, v_cache, T, block, scale, idx, K, out, lse_out, (char *)ws,
                            (hipStream_t)stream);
}

size_t snapkv_compress_workspace_bytes(const rs_shape *s, int64_t T, int32_t W)
{
    if (check_shape(s, false) != RS_OK || T <= 0 || W <= 0) return 0;
    return snapkv_ws_bytes(s, T, W);
}

static int32_t snapkv_impl(const rs_shape *s, const void *q_win, const void *k_cache, const void *v_cache, int64_t T,
                           int32_t W, int32_t K_keep, int32_t pool_kernel, float scale, const float *lse_win,
                           bool need_lse, void *kc_out, void *vc_out, int64_t Tcap_out, int32_t *idx_out,
                           float *votes_out, void *ws, size_t ws_bytes, void *stream)
{
    int st = check_shape(s, false);
    if (st != RS_OK) return st;
    if (!q_win || !k_cache || !v_cache || !kc_out || !vc_out || !idx_out) return RS_INVALID_ARG;
    if (need_lse && (!lse_win || !aligned16(lse_win))) return RS_INVALID_ARG;
    if (!aligned16(q_win) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(kc_out) ||
        !aligned16(vc_out) || !aligned16(idx_out) || (votes_out && !aligned16(votes_out)))
        return RS_INVALID_ARG;
    if (T <= 0 || T > s->Tcap || W <= 0 || W >= T) return RS_INVALID_ARG;
    if (K_keep < 0 || K_keep > T - W || K_keep + W > Tcap_out) return RS_INVALID_ARG;
    if (pool_kernel < 1 || pool_kernel % 2 == 0 || pool_kernel > 63) return RS_INVALID_ARG;
    if (!ws || !aligned16(ws) || ws_bytes < snapkv_ws_bytes(s, T, W)) return RS_WORKSPACE_TOO_SMALL;
    return snapkv_dispatch(s, q_win, k_cache, v_cache, T, W, K_keep, pool_kernel, scale, kc_out, vc_out, Tcap_out,
                           idx_out, votes_out, lse_win, (char *)ws, (hipStream_t)stream);
}

int32_t snapkv_compress(const rs_shape *s, const void *q_win, const void *k_cache, const void *v_cache, int64_t T,
                        int32_t W, int32_t K_keep, int32_t pool_kernel, float scale, void *kc_out, void *vc_out,
                        int64_t Tcap_out, int32_t *idx_out, float *votes_out, void *ws, size_t ws_bytes,
                        void *stream)
{
    return snapkv_impl(s, q_win, k_cache, v_cache, T, W, K_keep, pool_kernel, scale, nullptr, false, kc_out, vc_out,
                       Tcap_out, idx_out, votes_out, ws, ws_bytes, stream);
}

int32_t snapkv_compress_lse(const rs_shape *s, const void *q_win, const void *k_cache, const void *v_cache, int64_t T,
                            int32_t W, int32_t K_keep, int32_t pool_kernel, float scale, const float *lse_win,
                            void *kc_out, void *vc_out, int64_t Tcap_out, int32_t *idx_out, float *votes_out,
                            void *ws, size_t ws_bytes, void *stream)
{
    return snapkv_impl(s, q_win, k_cache, v_cache, T, W, K_keep, pool_kernel, scale, lse_win, true, kc_out, vc_out,
                       Tcap_out, idx_out, votes_out, ws, ws_bytes, stream);
}

}  // extern "C"
