// Device-side helpers shared by the gfx950 kernels: storage-type access (bf16 / f32),
// wave64 shuffles and reductions, workspace control-word layout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ratsparse.h"

namespace rs {

constexpr int kWave = 64;

// ---- workspace control words (uint32 index into the first RS_WS_CTRL_BYTES) ----
constexpr int kCtrlAsyncErr = 0;  // set to 1 by a kernel whose bounded wait expired
constexpr int kCtrlTicket = 1;    // dynamic chunk ticket of the scan
constexpr int kCtrlDone = 2;      // finished-workgroup counter of the scan
constexpr int kCtrlStateT = 4;     // replayable decode step: tokens in the cache (64 bits: words 4 and 5)
constexpr int kCtrlStateTag = 6;   // replayable decode step: the tag of the next step
constexpr int kCtrlUnit0 = 64;    // per-(batch, head) arrival counters start here
constexpr int kCtrlWords = RS_WS_CTRL_BYTES / 4;
constexpr int kMaxUnits = (kCtrlWords - kCtrlUnit0) / 2;

struct bf16 {
    uint16_t bits;
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even float32 -> bfloat16 bits (NaN kept quiet)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// two float32 -> packed bfloat16 pair (a in the low half), round-to-nearest-even through the
// hardware conversion
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    bf16x2_t v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}

// 8 consecutive channels of one row: raw registers as loaded, and their float32 view
template <typename ST>
struct Row8;

template <>
struct Row8<bf16> {
    struct raw_t {
        uint4 r;
    };
    __device__ __forceinline__ static raw_t load_raw(const bf16 *p)
    {
        raw_t w;
        w.r = *reinterpret_cast<const uint4 *>(p);
        return w;
    }
    // streaming load: the line is not meant to stay in the caches
    __device__ __forceinline__ static raw_t load_raw_nt(const bf16 *p)
    {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
        raw_t w;
        w.r = make_uint4(v.x, v.y, v.z, v.w);
        return w;
    }
    __device__ __forceinline__ static raw_t zero_raw()
    {
        raw_t w;
        w.r = make_uint4(0u, 0u, 0u, 0u);
        return w;
    }
    __device__ __forceinline__ static void unpack(const raw_t &w, float (&x)[8])
    {
        x[0] = __uint_as_float(w.r.x << 16);
        x[1] = __uint_as_float(w.r.x & 0xffff0000u);
        x[2] = __uint_as_float(w.r.y << 16);
        x[3] = __uint_as_float(w.r.y & 0xffff0000u);
        x[4] = __uint_as_float(w.r.z << 16);
        x[5] = __uint_as_float(w.r.z & 0xffff0000u);
        x[6] = __uint_as_float(w.r.w << 16);
        x[7] = __uint_as_float(w.r.w & 0xffff0000u);
    }
    __device__ __forceinline__ static void load(const bf16 *p, float (&x)[8]) { unpack(load_raw(p), x); }
    __device__ __forceinline__ static void store(bf16 *p, const float (&x)[8])
    {
        uint4 r;
        r.x = pack_bf16x2(x[0], x[1]);
        r.y = pack_bf16x2(x[2], x[3]);
        r.z = pack_bf16x2(x[4], x[5]);
        r.w = pack_bf16x2(x[6], x[7]);
        *reinterpret_cast<uint4 *>(p) = r;
    }
    // streaming store: the row is not read again soon
    __device__ __forceinline__ static void store_nt(bf16 *p, const float (&x)[8])
    {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        u32x4 r;
        r.x = pack_bf16x2(x[0], x[1]);
        r.y = pack_bf16x2(x[2], x[3]);
        r.z = pack_bf16x2(x[4], x[5]);
        r.w = pack_bf16x2(x[6], x[7]);
        __builtin_nontemporal_store(r, reinterpret_cast<u32x4 *>(p));
    }
};

template <>
struct Row8<float> {
    struct raw_t {
        float4 a, b;
    };
    __device__ __forceinline__ static raw_t load_raw(const float *p)
    {
        raw_t w;
        w.a = *reinterpret_cast<const float4 *>(p);
        w.b = *reinterpret_cast<const float4 *>(p + 4);
        return w;
    }
    __device__ __forceinline__ static raw_t load_raw_nt(const float *p)
    {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
        const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p + 4));
        raw_t w;
        w.a = make_float4(a.x, a.y, a.z, a.w);
        w.b = make_float4(b.x, b.y, b.z, b.w);
        return w;
    }
    __device__ __forceinline__ static raw_t zero_raw()
    {
        raw_t w;
        w.a = make_float4(0.f, 0.f, 0.f, 0.f);
        w.b = w.a;
        return w;
    }
    __device__ __forceinline__ static void unpack(const raw_t &w, float (&x)[8])
    {
        x[0] = w.a.x; x[1] = w.a.y; x[2] = w.a.z; x[3] = w.a.w;
        x[4] = w.b.x; x[5] = w.b.y; x[6] = w.b.z; x[7] = w.b.w;
    }
    __device__ __forceinline__ static void load(const float *p, float (&x)[8]) { unpack(load_raw(p), x); }
    __device__ __forceinline__ static void store(float *p, const float (&x)[8])
    {
        *reinterpret_cast<float4 *>(p) = make_float4(x[0], x[1], x[2], x[3]);
        *reinterpret_cast<float4 *>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
    }
    __device__ __forceinline__ static void store_nt(float *p, const float (&x)[8])
    {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        f32x4 a, b;
        a.x = x[0]; a.y = x[1]; a.z = x[2]; a.w = x[3];
        b.x = x[4]; b.y = x[5]; b.z = x[6]; b.w = x[7];
        __builtin_nontemporal_store(a, reinterpret_cast<f32x4 *>(p));
        __builtin_nontemporal_store(b, reinterpret_cast<f32x4 *>(p + 4));
    }
};

// A bfloat16 pair times a bfloat16 pair added to a float (v_dot2c_f32_bf16): the products are exact
// in float32, the result is within one float32 rounding of the exact sum (checked against float64
// on 2^20 random operands, denormals included: 1.5e-7 of the sum of magnitudes at worst).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
// two float32 values that hold bfloat16 numbers (their low 16 bits are zero) as a packed pair
__device__ __forceinline__ uint32_t repack_bf16x2(float lo, float hi)
{
    return (__float_as_uint(lo) >> 16) | (__float_as_uint(hi) & 0xffff0000u);
}

// q . k over this lane's 8 channels of a row, to be summed over the row's lanes by the caller.
// bfloat16 storage: the query is kept as four packed pairs and a pair of channels costs one
// dot-product instruction; float32 storage: one fused multiply-add per channel.
template <typename ST>
struct RowDot;

template <>
struct RowDot<bf16> {
    uint32_t qp[4];
    // q: this lane's 8 channels of a bfloat16 query, unpacked
    __device__ __forceinline__ void set(const float (&q)[8])
    {
#pragma unroll
        for (int w = 0; w < 4; ++w) qp[w] = repack_bf16x2(q[2 * w], q[2 * w + 1]);
    }
    __device__ __forceinline__ float dot(const Row8<bf16>::raw_t &k) const
    {
        float d = dot2_bf16(qp[0], k.r.x, 0.f);
        d = dot2_bf16(qp[1], k.r.y, d);
        d = dot2_bf16(qp[2], k.r.z, d);
        return dot2_bf16(qp[3], k.r.w, d);
    }
};

template <>
struct RowDot<float> {
    float qf[8];
    __device__ __forceinline__ void set(const float (&q)[8])
    {
#pragma unroll
        for (int c = 0; c < 8; ++c) qf[c] = q[c];
    }
    __device__ __forceinline__ float dot(const Row8<float>::raw_t &k) const
    {
        const float x[8] = {k.a.x, k.a.y, k.a.z, k.a.w, k.b.x, k.b.y, k.b.z, k.b.w};
        float d = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) d = fmaf(qf[c], x[c], d);
        return d;
    }
};

// Channelwise upper bound of q . k over the keys of a page (App. A.1, Quest; the score of Eq. 3):
// sum_c max(q_c lo_c, q_c hi_c) with lo, hi the page's channelwise min / max rows.  With
// lo_c <= hi_c the larger product is q_c hi_c where q_c > 0 and q_c lo_c elsewhere, so the bound
// row is picked per channel first -- on the packed bfloat16 words one bit-select serves a channel
// pair -- and what remains is the plain q . (picked row) of RowDot (the products are the same
// floats the two-product form would have taken the maximum of).
template <typename ST>
struct BoundDot;

template <>
struct BoundDot<bf16> {
    RowDot<bf16> q;
    uint32_t m[4];  // per packed word: ones over the half whose channel has q > 0
    __device__ __forceinline__ void set(const float (&qv)[8])
    {
        q.set(qv);
#pragma unroll
        for (int w = 0; w < 4; ++w)
            m[w] = (qv[2 * w] > 0.f ? 0x0000ffffu : 0u) | (qv[2 * w + 1] > 0.f ? 0xffff0000u : 0u);
    }
    // s + this lane's part of the page's bound
    __device__ __forceinline__ float add(float s, const Row8<bf16>::raw_t &lo, const Row8<bf16>::raw_t &hi) const
    {
        const uint32_t l[4] = {lo.r.x, lo.r.y, lo.r.z, lo.r.w};
        const uint32_t h[4] = {hi.r.x, hi.r.y, hi.r.z, hi.r.w};
#pragma unroll
        for (int w = 0; w < 4; ++w) s = dot2_bf16(q.qp[w], (h[w] & m[w]) | (l[w] & ~m[w]), s);
        return s;
    }
};

template <>
struct BoundDot<float> {
    float qf[8];
    __device__ __forceinline__ void set(const float (&qv)[8])
    {
#pragma unroll
        for (int c = 0; c < 8; ++c) qf[c] = qv[c];
    }
    __device__ __forceinline__ float add(float s, const Row8<float>::raw_t &lo, const Row8<float>::raw_t &hi) const
    {
        const float l[8] = {lo.a.x, lo.a.y, lo.a.z, lo.a.w, lo.b.x, lo.b.y, lo.b.z, lo.b.w};
        const float h[8] = {hi.a.x, hi.a.y, hi.a.z, hi.a.w, hi.b.x, hi.b.y, hi.b.z, hi.b.w};
#pragma unroll
        for (int c = 0; c < 8; ++c) s = fmaf(qf[c], (qf[c] > 0.f) ? h[c] : l[c], s);
        return s;
    }
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return bf16_bits_to_f32(x.bits); }
__device__ __forceinline__ void from_f32(float &d, float x) { d = x; }
__device__ __forceinline__ void from_f32(bf16 &d, float x) { d.bits = __builtin_bit_cast(uint16_t, (__bf16)x); }

// One wave-wide direct load moves 64 x 16 bytes from global memory into 1 KB of LDS, lane l
// landing at byte 16 l of the destination; nothing passes through registers.  The source is
// named by a buffer descriptor (a wave-uniform base) plus a per-lane byte offset: the buffer
// form of the instruction only counts as a vector memory operation, so the compiler keeps
// exact counts for the LDS reads issued around it (with the global-address form it treats the
// LDS counter as out of order and turns every wait for an operand read into a wait for all of
// them, the ones issued just before included).
typedef __amdgpu_buffer_rsrc_t LdsSource;
__device__ __forceinline__ LdsSource lds_source(const void *base)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ void load16_to_lds(LdsSource src, uint32_t byte_offset, void *l)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(src, (__attribute__((address_space(3))) void *)l, 16, (int)byte_offset, 0, 0, 0);
}


// Tiles of K/V rows sit in LDS unpadded (a wave-wide load fills whole rows back to back), so the bank
// spread comes from permuting the 16-byte chunks inside each row: chunk c of row r is kept at
// position c ^ chunk_swizzle(r).  The permutation is chosen so that (a) 16 lanes reading the
// same chunk of 16 consecutive rows (the K operand) and (b) 32 lanes reading 64 bytes of each
// of 4 consecutive rows (the transposed V operand) both touch every bank once.
template <int D>
__device__ __forceinline__ int chunk_swizzle(int row)
{
    if constexpr (D == 128) {
        const int x = row & 15;
        return ((x & 3) << 2) | (x >> 2);
    } else {
        const int x = (row >> 1) & 7;
        return ((x & 1) << 2) | (x >> 1);
    }
}

// max / sum of a value with the one 32 lanes away, the same in both lanes, through
// v_permlane32_swap (no LDS round trip): swap(x, x) leaves [low half | low half] and
// [high half | high half]
__device__ __forceinline__ float half_pair_max(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_pair_sum(float x)
{
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ float shfl_xor_f(float v, int mask) { return __shfl_xor(v, mask, kWave); }
__device__ __forceinline__ float shfl_up_f(float v, int d) { return __shfl_up(v, d, kWave); }
__device__ __forceinline__ float shfl_f(float v, int src) { return __shfl(v, src, kWave); }

// a lane's value as seen through a data-parallel-primitive lane pattern (the move folds into the
// arithmetic instruction that uses it: no trip through the LDS crossbar, no wait)
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// sum over aligned groups of `width` lanes (power of two); every lane gets the sum.
// 16 lanes are a DPP row: four rotations within the row (by 8, 4, 2, 1) give every lane the same
// bits as the exchange-with-partner butterfly (a rotation by 8 is the exchange with lane ^ 8, and
// from then on both partners of an exchange hold equal values).  8 lanes are half a row: mirror
// within the half (lane i <-> 7 - i), then the two exchanges inside a quad.
template <int width>
__device__ __forceinline__ float group_sum(float v)
{
    if constexpr (width == 16) {
        v += dpp_f<0x128>(v);  // row_ror:8
        v += dpp_f<0x124>(v);  // row_ror:4
        v += dpp_f<0x122>(v);  // row_ror:2
        v += dpp_f<0x121>(v);  // row_ror:1
    } else if constexpr (width == 8) {
        v += dpp_f<0x141>(v);  // row_half_mirror
        v += dpp_f<0xB1>(v);   // quad_perm:[1,0,3,2]
        v += dpp_f<0x4E>(v);   // quad_perm:[2,3,0,1]
    } else {
#pragma unroll
        for (int m = width / 2; m >= 1; m >>= 1) v += shfl_xor_f(v, m);
    }
    return v;
}

__device__ __forceinline__ int wave_sum_i(int v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// agent-scope relaxed 64-bit accesses that go past the per-XCD L2 (value+tag records)
__device__ __forceinline__ void store_u64_agent(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t load_u64_agent(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// order-preserving map float32 -> uint32 (larger float <=> larger key); -0.0 and +0.0 are
// equal numbers and get the same key, so that a tie between them goes to the lower index
__device__ __forceinline__ uint32_t float_to_key(float f)
{
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace rs
