// Device helpers shared by all kernels: magnitude keys, nontemporal 16-byte accesses, guarded
// accesses at segment boundaries, ballots and wave reductions.  Part of scalecom.hip's single
// translation unit.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "geometry.h"

namespace {

__device__ __forceinline__ uint32_t magnitude_key(float x) { return __float_as_uint(x) & 0x7fffffffu; }

__device__ __forceinline__ float widen(float g) { return g; }
__device__ __forceinline__ float widen(uint16_t g) { return __uint_as_float(static_cast<uint32_t>(g) << 16); }

// Streaming accesses carry the nontemporal hint: every byte of mem and grad is touched once per
// pass, so keeping it in cache only evicts what is reused (measured: +3 to +10 % bandwidth).
typedef float vf4_t __attribute__((ext_vector_type(4)));
typedef uint32_t vu2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float4 load4(const float* p)
{
    const vf4_t v = __builtin_nontemporal_load(reinterpret_cast<const vf4_t*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float4 load4(const uint16_t* p)
{
    const vu2_t v = __builtin_nontemporal_load(reinterpret_cast<const vu2_t*>(p));
    float4 r;
    r.x = __uint_as_float(v.x << 16);
    r.y = __uint_as_float(v.x & 0xffff0000u);
    r.z = __uint_as_float(v.y << 16);
    r.w = __uint_as_float(v.y & 0xffff0000u);
    return r;
}
__device__ __forceinline__ void store4(float* p, const float4& v)
{
    vf4_t w;
    w.x = v.x;
    w.y = v.y;
    w.z = v.z;
    w.w = v.w;
    __builtin_nontemporal_store(w, reinterpret_cast<vf4_t*>(p));
}

// Stand-in gradient type for selecting on a plain vector: every element reads as +0, so that
// x = fma(lr, 0, v) has v's magnitude bits for any finite lr (non-finite v included).  Never
// dereferenced.
struct NoGrad {};
__device__ __forceinline__ float4 load4(const NoGrad*) { return make_float4(0.0f, 0.0f, 0.0f, 0.0f); }

// number of set bits of a wave-wide ballot that belong to lanes below the calling lane
__device__ __forceinline__ uint32_t lanes_below(uint64_t ballot)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(ballot >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(ballot), 0u));
}

// Reductions over the 64 lanes of a wave, result in a scalar register: data-parallel-primitive
// moves inside the vector ALU (shift right by 1, 2, 4, 8 lanes inside each row of 16, then the
// last lane of row 0 and of rows 0-1 broadcast to the rows that follow) instead of cross-lane reads
// through the LDS crossbar; lanes without a source take the identity 0.  All 64 lanes must be
// active at the call.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_move(uint32_t x)   // x of the lane CTRL names, 0 where there is none
{
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, ROW_MASK, 0xf, false));
}

template <typename Op>
__device__ __forceinline__ uint32_t wave_reduce_u32(uint32_t v, Op op)
{
    constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
    constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;
    v = op(v, dpp_move<kRowShr1, 0xf>(v));
    v = op(v, dpp_move<kRowShr2, 0xf>(v));
    v = op(v, dpp_move<kRowShr4, 0xf>(v));
    v = op(v, dpp_move<kRowShr8, 0xf>(v));                  // lane 15 of every row holds the row's result
    v = op(v, dpp_move<kRowBcast15, 0xa>(v));               // into rows 1 and 3
    v = op(v, dpp_move<kRowBcast31, 0xc>(v));               // into rows 2 and 3
    return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), kLanes - 1));
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
    return wave_reduce_u32(v, [](uint32_t a, uint32_t b) { return a + b; });
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    return wave_reduce_u32(v, [](uint32_t a, uint32_t b) { return a > b ? a : b; });
}

// 4 consecutive values starting at position p0 (a multiple of 4) of one learner's array;
// positions outside [begin, end) read as 0 and are never touched in memory.
template <typename T>
__device__ __forceinline__ float4 load_guarded(const T* base, int64_t p0, int64_t begin, int64_t end, bool full)
{
    if (full) return load4(base + p0);
    float v[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int64_t p = p0 + c;
        v[c] = (p >= begin && p < end) ? widen(base[p]) : 0.0f;
    }
    return make_float4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ float4 load_guarded(const NoGrad*, int64_t, int64_t, int64_t, bool)
{
    return make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}

__device__ __forceinline__ void store_guarded(float* base, int64_t p0, int64_t begin, int64_t end, bool full,
                                              const float4& v)
{
    if (full) {
        store4(base + p0, v);
        return;
    }
    const float a[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int64_t p = p0 + c;
        if (p >= begin && p < end) base[p] = a[c];
    }
}

// x = fma(lr, grad, mem): the error-feedback gradient of Alg. 1 line 6, one rounding.
__device__ __forceinline__ float4 accumulate4(const float4& m, const float4& g, float lr)
{
    return make_float4(fmaf(lr, g.x, m.x), fmaf(lr, g.y, m.y), fmaf(lr, g.z, m.z), fmaf(lr, g.w, m.w));
}

// The leader's (mem, grad) at the 4 positions of this lane (zeros where outside the segment).
template <typename G>
__device__ __forceinline__ void leader_load(const float* mem, const G* grad, int64_t p0, int64_t begin, int64_t end,
                                            float4& m, float4& g)
{
    m = make_float4(0, 0, 0, 0);
    g = m;
    if (p0 >= end || p0 + 3 < begin) return;
    const bool full = p0 >= begin && p0 + 3 < end;
    m = load_guarded(mem, p0, begin, end, full);
    g = load_guarded(grad, p0, begin, end, full);
}

// Magnitude keys of x = fma(lr, grad, mem) (Alg. 1 line 6) for those 4 positions; ok[c] tells
// whether the position belongs to the segment.
__device__ __forceinline__ void keys_from(const float4& m, const float4& g, float lr, int64_t p0, int64_t begin,
                                          int64_t end, uint32_t key[4], bool ok[4])
{
    const float4 x = accumulate4(m, g, lr);
    key[0] = magnitude_key(x.x);
    key[1] = magnitude_key(x.y);
    key[2] = magnitude_key(x.z);
    key[3] = magnitude_key(x.w);
#pragma unroll
    for (int c = 0; c < 4; ++c) ok[c] = (p0 + c >= begin) && (p0 + c < end);
}

template <typename G>
__device__ __forceinline__ void leader_keys(const float* mem, const G* grad, float lr, int64_t p0, int64_t begin,
                                            int64_t end, uint32_t key[4], bool ok[4])
{
    float4 m, g;
    leader_load(mem, grad, p0, begin, end, m, g);
    keys_from(m, g, lr, p0, begin, end, key, ok);
}

// Where a step expects its threshold (top 24 bits of the key).  Learners whose gradients differ in
// scale have thresholds that differ as much, so each leader's own last threshold is kept
// (lead_mine[seg], 0 before its first turn) and moved on by the growth the last leader saw over
// its cycle; without it, the last step's threshold.  Only a prediction: it decides how much work
// a step does, never what it selects.
__device__ __forceinline__ uint32_t predicted_t24(const uint32_t* pred, const uint32_t* lead_mine, int seg)
{
    uint32_t t24 = pred[1];
    if (lead_mine) {
        const uint32_t mine = lead_mine[seg];
        if (mine != 0u) {
            const float growth = pred[4] != 0u ? __uint_as_float(pred[4]) : 1.0f;
            const float f = __uint_as_float(mine << kBits2) * growth;
            t24 = (__float_as_uint(f) & 0x7fffffffu) >> kBits2;
        }
    }
    return t24;
}

// Records the threshold a step found (by one thread, for the next steps' predictions).
__device__ __forceinline__ void record_t24(uint32_t* pred, uint32_t* lead_mine, int seg, uint32_t t24)
{
    pred[1] = t24;
    if (lead_mine) {
        const uint32_t old = lead_mine[seg];
        float growth = 1.0f;
        if (old != 0u && t24 != 0u) {
            growth = __uint_as_float(t24 << kBits2) / __uint_as_float(old << kBits2);
            if (!(growth > 0.5f)) growth = 0.5f;
            if (!(growth < 2.0f)) growth = 2.0f;
        }
        pred[4] = __float_as_uint(growth);
        lead_mine[seg] = t24;
    }
}

// The exact value, once known, in place of the estimate that record_t24 was given.
__device__ __forceinline__ void refine_t24(uint32_t* pred, uint32_t* lead_mine, int seg, uint32_t t24)
{
    pred[1] = t24;
    if (lead_mine) lead_mine[seg] = t24;
}

// Membership bitmask layout: per wave tile four 64-bit words; bit l of word c belongs to
// position tile0 + 4*l + c, i.e. word c is the wave ballot of "element c of my lane is a member".
__device__ __forceinline__ void store_tile_masks(uint64_t* mask, size_t tile, const uint64_t b[4])
{
    ulonglong2* dst = reinterpret_cast<ulonglong2*>(mask + tile * 4);
    dst[0] = make_ulonglong2(b[0], b[1]);
    dst[1] = make_ulonglong2(b[2], b[3]);
}

}  // namespace
