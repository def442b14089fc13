// HIP kernels (gfx950 / CDNA4, 64-lane wavefronts) and C-ABI of ScaleCom's per-step
// compression path: CLT-k with low-pass-filtered error feedback (arXiv 2104.11125, Alg. 1
// lines 6, 7, 10; Eq. 2, 3, 5).  See include/scalecom.h for the contract of each entry point.
//
// Structure of one step (all on the context's stream, no host synchronisation).  The 31-bit
// magnitude key |x_L| of the leader's x_L = fma(lr, grad_L, mem_L) (recomputed on the fly, never
// stored) is resolved 12 + 12 + 7 bits at a time (radix select):
//
//   predicted   leader, ONE pass, for segments that carry the threshold bucket of the previous
//               step as a prediction: keys whose top 12 bits lie above a 5-bucket window around
//               it are members for sure (counted per 256-element wave tile, marked in the
//               membership bitmask); keys inside the window are copied, with their positions,
//               to a small candidate list and counted per bucket
//   hist0       leader, histogram of the top 12 key bits -- only for segments without a
//               prediction or whose window missed the k-th largest key (exact check on counts)
//   find<0>     per segment: the bucket holding the k-th largest key  (Eq. 2)
//   collect     leader, second pass -- only for segments that went through hist0: same job as
//               `predicted` with the now known bucket as the window
//   hist<1,2>   the remaining 12 + 7 key bits, histogrammed over the candidate list
//   find<1,2>   after level 2 the exact threshold key T and the number q of keys equal to T
//               that still belong to the set are known
//   tilecount   candidates above / equal to T are added to the per-tile counts and bitmasks
//               (a segment whose bucket does not fit the candidate list -- many equal keys --
//               takes levels 1, 2 and this step as full leader passes instead of the list)
//   scan, slots prefix sums of the counts over tiles: first output slot of every wave tile;
//               keys equal to T become members in position order until q are taken
//   update      every learner, one (learner, 1024 positions) pair per block: one read of
//               (mem, grad), one write of mem (Eq. 5); members also store x_i into a small
//               [learner][slot] staging array and learner 0 writes the index (Eq. 3)
//   reduce      reduced[t] = x_0[t] + x_1[t] + ... in learner order  (Alg. 1 line 10)
//
// In the steady state (predictions hold) hist0 and collect find nothing to do, and the leader's
// vector is read exactly once before the all-learner pass.  The prediction only decides how
// much work is done, never what is selected.  The output is ascending by position and
// deterministic.  Nothing here is a dense contraction, so there is no MFMA; the kernels are
// bound by HBM traffic (update, predicted) and by launch latency (the small ones).

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "scalecom.h"

namespace {

// ------------------------------------------------------------------------------------------
// geometry
// ------------------------------------------------------------------------------------------
constexpr int kLanes = 64;                       // wavefront width on CDNA
constexpr int kVec = 4;                          // elements per lane per access (16 B of fp32)
constexpr int kWaveTile = kLanes * kVec;         // 256 consecutive positions handled by one wave
constexpr int kTilesPerSuper = 32;               // wave tiles per supertile
constexpr int kSuper = kWaveTile * kTilesPerSuper;   // 8192 positions
constexpr int kBlock = 256;                      // threads per block in the streaming kernels
constexpr int kWaves = kBlock / kLanes;          // 4
constexpr int kUpdateBlocksPerSuper = kTilesPerSuper / kWaves;   // update: one wave tile per wave
constexpr int kChunk = 1024;                     // supertiles per chunk of the prefix scan

constexpr int kBits0 = 12, kBits1 = 12, kBits2 = 7;          // 31-bit key = 12 + 12 + 7
constexpr int kBins0 = 1 << kBits0, kBins1 = 1 << kBits1, kBins2 = 1 << kBits2;
constexpr int kHistGridMax = 2048;
constexpr int kFoldLastSearchMaxSt = 32768;      // up to this many supertiles k_tilecount searches the last level itself
constexpr int kCandSlice = 512;                  // candidate slots per supertile (1/16 of its positions)
constexpr uint32_t kModeFull = 0, kModeCand = 1;

struct SegDesc {          // one per tensor (segment of the flat vector)
    int32_t begin, end;   // positions [begin, end)
    int32_t k;            // size of this segment's index set
    int32_t out_base;     // first output slot of this segment
    int32_t st_first;     // first supertile
    int32_t st_count;     // number of supertiles
    int32_t chunk_first;  // first scan chunk
    int32_t chunk_count;
    int32_t sel_chunk;    // chunk-wise selector: elements per chunk of this segment (0 in exact mode)
    int32_t pad;
};

struct StDesc {           // one per supertile; carries what the streaming kernels need of its segment
    int32_t seg;
    int32_t a0;           // first position, a multiple of 4 (may lie up to 3 before begin)
    int32_t begin, end;   // the segment's positions [begin, end)
    int32_t slot_end;     // one past the segment's last output slot
    int32_t pad[3];
};

struct ChunkDesc {        // one per scan chunk: up to kChunk consecutive supertiles of one segment
    int32_t seg;
    int32_t st_begin;
    int32_t st_count;
    int32_t pad;
};

struct SegState {         // selection state of one segment; every field is rewritten by k_find<0> each step
    uint32_t prefix;      // key bits fixed so far (level 0: 12 bits, level 1: 24 bits)
    uint32_t k_rem;       // members still to be found inside the current bucket
    uint32_t T;           // threshold key (after level 2)
    uint32_t q;           // number of keys == T that are members (the lowest positions)
    uint32_t done;        // 1: empty index set, nothing to refine
    uint32_t mode;        // kModeCand: levels 1, 2 and the tile counts work on the candidate list
    uint32_t collected;   // 1: the candidate list was filled by the predicted single pass
    uint32_t pad;
};

constexpr uint32_t kWindow = 5;                  // predicted window: previous bucket +- 2 digits
// Counts of the predicted pass, per segment: [0] keys above the window, [1 + d] keys with the
// d-th digit of the window.  Blocks add into one of kPartSlots copies (same-address atomics from
// thousands of blocks would serialise); readers sum the copies.
constexpr int kPartSlots = 64;
constexpr int kPartWords = 8;

struct LearnerPtrs {
    float* mem[SCALECOM_MAX_LEARNERS];
    const void* grad[SCALECOM_MAX_LEARNERS];
};

// ------------------------------------------------------------------------------------------
// device helpers
// ------------------------------------------------------------------------------------------
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

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kLanes);
    return v;
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

// first and last top digit of the window collected around a predicted bucket (p = bucket + 1)
__device__ __forceinline__ uint32_t window_lo(uint32_t p) { return p >= 3 ? p - 3 : 0u; }
__device__ __forceinline__ uint32_t window_hi(uint32_t p) { return p + 1 < static_cast<uint32_t>(kBins0) ? p + 1 : kBins0 - 1u; }

// Did the predicted single pass see the k-th largest key inside its window?  If so: the key's
// top digit and how many members remain to be found inside that digit's bucket.  Exact: uses
// only counts gathered over the whole segment.
__device__ __forceinline__ bool spec_resolve(const uint32_t tot[1 + kWindow], bool overflow, uint32_t p, uint32_t k,
                                             uint32_t& digit, uint32_t& k_rem)
{
    if (p == 0 || overflow || k <= tot[0]) return false;
    const uint32_t lo = window_lo(p), hi = window_hi(p);
    uint32_t c = tot[0];
    for (uint32_t d = hi + 1; d-- > lo;) {
        const uint32_t n = tot[1 + d - lo];
        if (c + n >= k) {
            digit = d;
            k_rem = k - c;
            return true;
        }
        c += n;
    }
    return false;
}

// ------------------------------------------------------------------------------------------
// kernels
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kBlock) k_init(uint32_t* zero_from, size_t n_words)
{
    for (size_t i = blockIdx.x * static_cast<size_t>(kBlock) + threadIdx.x; i < n_words;
         i += static_cast<size_t>(gridDim.x) * kBlock)
        zero_from[i] = 0u;
}

// Membership bitmask layout: per wave tile four 64-bit words; bit l of word c belongs to
// position tile0 + 4*l + c, i.e. word c is the wave ballot of "element c of my lane is a member".
__device__ __forceinline__ void store_tile_masks(uint64_t* mask, size_t tile, const uint64_t b[4])
{
    ulonglong2* dst = reinterpret_cast<ulonglong2*>(mask + tile * 4);
    dst[0] = make_ulonglong2(b[0], b[1]);
    dst[1] = make_ulonglong2(b[2], b[3]);
}

struct CollectStage {       // LDS staging of one supertile's masks and tile counts in the collecting passes
    uint64_t mask[kTilesPerSuper][4];
    uint32_t cnt[kTilesPerSuper];
};

// The per-tile work of the "collect" pass, given the tile's keys: keys whose top digit lies above
// `hi` are members for sure (their count and ballots are staged for the tile); keys with a top
// digit in [lo, hi] are appended, with their positions, to the supertile's candidate slice `cand_dst`
// (in LDS or in memory; slots handed out through the block's LDS counter `fill`) and, if `wc` is given, counted per
// digit there, and, if `lh1` is given (then lo == hi), per second digit there.  Called by all lanes
// of a wave; n_above is the same in every lane.
template <bool ALL_OK>
__device__ __forceinline__ void collect_tile(const uint32_t key[4], const bool ok[4], uint32_t p0, uint32_t lo,
                                             uint32_t hi, int wt, int lane, uint32_t* fill, uint32_t* wc,
                                             uint32_t* lh1, uint32_t& n_above, CollectStage& stg, uint2* cand_dst)
{
    // top digit > hi  <=>  key >= (hi + 1) << 19;  lo <= top digit <= hi  <=>  key - (lo << 19) < span
    const uint32_t lo_key = lo << (kBits1 + kBits2);
    const uint32_t above_key = (hi + 1u) << (kBits1 + kBits2);   // 2^31 for the last digit: no key reaches it
    const uint32_t span = above_key - lo_key;
    n_above = 0;
    uint32_t n_in = 0;
    bool in[4];
    uint64_t above[4], inside[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        above[c] = __builtin_amdgcn_ballot_w64((ALL_OK || ok[c]) && key[c] >= above_key);
        n_above += __popcll(above[c]);
        in[c] = (ALL_OK || ok[c]) && key[c] - lo_key < span;
        inside[c] = __builtin_amdgcn_ballot_w64(in[c]);
        n_in += __popcll(inside[c]);
    }
    if (lane == 0) {
        stg.cnt[wt] = n_above;
#pragma unroll
        for (int c = 0; c < 4; ++c) stg.mask[wt][c] = above[c];
    }
    if (n_in == 0) return;                                 // wave-uniform
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(fill, n_in);
    base = __builtin_amdgcn_readfirstlane(base);
    uint32_t rank = base;
#pragma unroll
    for (int c = 0; c < 4; ++c) rank += lanes_below(inside[c]);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (in[c]) {
            if (rank < kCandSlice) cand_dst[rank] = make_uint2(key[c], p0 + c);
            if (wc) atomicAdd(&wc[(key[c] >> (kBits1 + kBits2)) - lo], 1u);
            if (lh1) atomicAdd(&lh1[(key[c] >> kBits2) & (kBins1 - 1)], 1u);   // counted whether or not it is listed
            ++rank;
        }
    }
}

// After the block's barrier: the staged masks and counts of the supertile, and its candidates if
// they were staged too, go out with full-width stores (lane-0 stores of 32 bytes per tile cost the collecting passes 8 % of their time).
__device__ __forceinline__ void collect_flush(const CollectStage& stg, const uint2* cand_stage, size_t tile0,
                                              uint32_t n_cand, uint32_t* __restrict__ wt_cnt,
                                              uint64_t* __restrict__ sel_mask, uint64_t* __restrict__ eq_mask,
                                              uint2* __restrict__ slice)
{
    static_assert(kTilesPerSuper * 4 * sizeof(uint64_t) == kLanes * sizeof(ulonglong2), "one 16-byte store per lane");
    static_assert(kBlock >= 2 * kLanes + kTilesPerSuper, "threads for the three flushes");
    const int t = threadIdx.x;
    if (t < kLanes) {
        const ulonglong2* src = reinterpret_cast<const ulonglong2*>(&stg.mask[0][0]);
        reinterpret_cast<ulonglong2*>(sel_mask + tile0 * 4)[t] = src[t];
    } else if (t < 2 * kLanes) {
        reinterpret_cast<ulonglong2*>(eq_mask + tile0 * 4)[t - kLanes] = make_ulonglong2(0ull, 0ull);
    } else if (t < 2 * kLanes + kTilesPerSuper) {
        wt_cnt[tile0 + (t - 2 * kLanes)] = stg.cnt[t - 2 * kLanes];
    }
    if (!cand_stage) return;                                // the candidates went to the slice directly
    const uint32_t n = n_cand < kCandSlice ? n_cand : kCandSlice;
    for (uint32_t e = threadIdx.x; e < n; e += kBlock) slice[e] = cand_stage[e];
}

// First look at the leader's vector (Eq. 2: finding the k-th largest magnitude), for segments
// that carry a prediction of their threshold bucket (the bucket found in the previous step).
// ONE pass, no histogram: keys whose top digit lies above a 5-digit window around the
// prediction are members for sure (counted per tile, marked in the mask), keys inside the
// window go to the candidate list and are counted per digit.  If the counts show afterwards
// that the k-th largest key fell inside the window, the threshold bucket is known exactly and
// no other full pass over the leader is needed.  The prediction only decides how much work is
// done, never what is selected.  One block per supertile.
// The 8 tiles a wave owns in a supertile of the predicted pass.  INSIDE: the whole supertile
// lies in the segment, so loads are unguarded and every position counts; otherwise both are
// checked per element.  Positions stay below 2^31 + 8192 and are kept in 32 bits.
template <typename G, bool INSIDE>
__device__ __forceinline__ uint32_t predicted_tiles(const float* __restrict__ mem, const G* __restrict__ grad, float lr,
                                                    const StDesc& d, uint32_t lo, uint32_t hi, int wave, int lane,
                                                    uint32_t* fill, uint32_t* wc, CollectStage& stg, uint2* cand_stage)
{
    constexpr int kIters = kTilesPerSuper / kWaves;
    constexpr uint32_t kStride = kWaves * kWaveTile;
    const int64_t begin = d.begin, end = d.end;
    // the next tile's loads are issued before this tile is processed (measured: neither a deeper
    // prefetch nor full unrolling changes the kernel's time)
    float4 m_cur, g_cur, m_nxt, g_nxt;
    uint32_t p_cur = static_cast<uint32_t>(d.a0) + wave * kWaveTile + lane * kVec;
    auto fetch = [&](uint32_t p0, float4& m, float4& g) {
        if (INSIDE) {
            m = load4(mem + p0);
            g = load4(grad + p0);
        } else {
            leader_load(mem, grad, p0, begin, end, m, g);
        }
    };
    fetch(p_cur, m_cur, g_cur);
    uint32_t above_acc = 0;
#pragma unroll 1
    for (int it = 0; it < kIters; ++it) {
        const int wt = it * kWaves + wave;
        if (it + 1 < kIters) fetch(p_cur + kStride, m_nxt, g_nxt);
        const float4 x = accumulate4(m_cur, g_cur, lr);
        const uint32_t key[4] = {magnitude_key(x.x), magnitude_key(x.y), magnitude_key(x.z), magnitude_key(x.w)};
        bool ok[4] = {true, true, true, true};
        if (!INSIDE) {
#pragma unroll
            for (int c = 0; c < 4; ++c) ok[c] = static_cast<int64_t>(p_cur) + c >= begin && static_cast<int64_t>(p_cur) + c < end;
        }
        uint32_t n_above;
        collect_tile<INSIDE>(key, ok, p_cur, lo, hi, wt, lane, fill, wc, nullptr, n_above, stg, cand_stage);
        above_acc += n_above;
        m_cur = m_nxt;
        g_cur = g_nxt;
        p_cur += kStride;
    }
    return above_acc;
}

template <typename G>
__global__ void __launch_bounds__(kBlock)
k_predicted(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const SegDesc* __restrict__ segs,
            const StDesc* __restrict__ sts, uint2* __restrict__ cand,
            uint32_t* __restrict__ st_cand_cnt, const uint32_t* __restrict__ preds, uint32_t* __restrict__ wt_cnt,
            uint64_t* __restrict__ sel_mask, uint64_t* __restrict__ eq_mask, uint32_t* __restrict__ part,
            uint32_t* __restrict__ overflow, uint32_t* __restrict__ next_scratch, size_t next_words)
{
    // The counters and histograms of a step live in one of two copies of a scratch zone; this
    // kernel, the first of a step, clears the copy the NEXT step will use (nothing else touches it
    // during this step), so no step needs a separate clearing pass.
    for (size_t i = blockIdx.x * static_cast<size_t>(kBlock) + threadIdx.x; i < next_words;
         i += static_cast<size_t>(gridDim.x) * kBlock)
        next_scratch[i] = 0u;

    const int st = blockIdx.x;
    const StDesc d = sts[st];
    const uint32_t p = preds[d.seg];                        // 0: none, else predicted bucket + 1
    if (p == 0 || segs[d.seg].k == 0) return;
    const uint32_t lo = window_lo(p), hi = window_hi(p);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes), lane = threadIdx.x % kLanes;
    __shared__ uint32_t fill;
    __shared__ uint32_t acc[kPartWords];                    // [0] above the window, [1 + d] per window digit
    __shared__ CollectStage stg;
    __shared__ uint2 cand_stage[kCandSlice];
    if (threadIdx.x == 0) fill = 0u;
    if (threadIdx.x < kPartWords) acc[threadIdx.x] = 0u;
    __syncthreads();

    uint2* slice = cand + static_cast<size_t>(st) * kCandSlice;
    uint32_t above_acc;
    if (d.a0 >= d.begin && static_cast<int64_t>(d.a0) + kSuper <= d.end)   // block-uniform
        above_acc = predicted_tiles<G, true>(mem, grad, lr, d, lo, hi, wave, lane, &fill, acc + 1, stg, cand_stage);
    else
        above_acc = predicted_tiles<G, false>(mem, grad, lr, d, lo, hi, wave, lane, &fill, acc + 1, stg, cand_stage);
    if (lane == 0 && above_acc) atomicAdd(&acc[0], above_acc);
    __syncthreads();
    collect_flush(stg, cand_stage, static_cast<size_t>(st) * kTilesPerSuper, fill, wt_cnt, sel_mask, eq_mask, slice);
    if (threadIdx.x == 0) {
        const uint32_t n = fill;
        st_cand_cnt[st] = n < kCandSlice ? n : kCandSlice;
        if (n > kCandSlice) overflow[d.seg] = 1u;           // every overflowing block stores the same value
    }
    if (threadIdx.x <= kWindow) {
        const uint32_t v = acc[threadIdx.x];
        if (v)
            atomicAdd(&part[(static_cast<size_t>(d.seg) * kPartSlots + st % kPartSlots) * kPartWords + threadIdx.x], v);
    }
}

// Histogram of the top 12 key bits of the leader's vector, for the segments that need it: those
// without a prediction, and those whose prediction failed (the k-th largest key was not inside
// the window k_predicted collected).
template <typename G>
__global__ void __launch_bounds__(kBlock)
k_hist0(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const SegDesc* __restrict__ segs,
        const StDesc* __restrict__ sts, int n_st, uint32_t* __restrict__ hist, const uint32_t* __restrict__ preds,
        const uint32_t* __restrict__ part, const uint32_t* __restrict__ overflow)
{
    __shared__ uint32_t lh[kBins0];
    __shared__ uint32_t tot_s[kPartWords];
    __shared__ int needed;

    const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
    const int st_lo = static_cast<int>(static_cast<int64_t>(blockIdx.x) * n_st / gridDim.x);
    const int st_hi = static_cast<int>(static_cast<int64_t>(blockIdx.x + 1) * n_st / gridDim.x);

    bool lh_ready = false;
    // walk the block's supertiles segment by segment: a segment that needs no histogram (the
    // steady state) costs one look at its counters, not one per supertile
    int st = st_lo;
    while (st < st_hi) {
        const int cur = sts[st].seg;
        const SegDesc sd = segs[cur];
        const int seg_hi = sd.st_first + sd.st_count < st_hi ? sd.st_first + sd.st_count : st_hi;
        const uint32_t p = preds[cur];
        const uint32_t k = static_cast<uint32_t>(sd.k);
        if (k != 0 && p != 0) {                             // did the prediction hold?  (block-uniform branch)
            if (threadIdx.x < kPartWords) tot_s[threadIdx.x] = 0u;
            __syncthreads();
            for (int i = threadIdx.x; i < kPartSlots * kPartWords; i += kBlock) {
                const uint32_t v = part[static_cast<size_t>(cur) * kPartSlots * kPartWords + i];
                if (v) atomicAdd(&tot_s[i % kPartWords], v);
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                uint32_t tot[1 + kWindow], digit, k_rem;
                for (uint32_t j = 0; j <= kWindow; ++j) tot[j] = tot_s[j];
                needed = !spec_resolve(tot, overflow[cur] != 0, p, k, digit, k_rem);
            }
        } else if (threadIdx.x == 0) {
            needed = k != 0;
        }
        __syncthreads();
        const bool histogram = needed != 0;
        __syncthreads();
        if (histogram) {
            if (!lh_ready) {                                // the histogram is only cleared when it is used
                for (int b = threadIdx.x; b < kBins0; b += kBlock) lh[b] = 0u;
                __syncthreads();
                lh_ready = true;
            }
            const int64_t begin = sd.begin, end = sd.end;
            for (int s2 = st; s2 < seg_hi; ++s2) {
                const int64_t a0 = sts[s2].a0;
#pragma unroll 2
                for (int it = 0; it < kTilesPerSuper / kWaves; ++it) {
                    const int64_t p0 = a0 + (it * kWaves + wave) * kWaveTile + lane * kVec;
                    if (p0 >= end) continue;
                    uint32_t key[4];
                    bool ok[4];
                    leader_keys(mem, grad, lr, p0, begin, end, key, ok);
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (ok[c]) atomicAdd(&lh[key[c] >> (kBits1 + kBits2)], 1u);
                }
            }
            __syncthreads();                                // flush the segment's counts
            for (int b = threadIdx.x; b < kBins0; b += kBlock) {
                const uint32_t v = lh[b];
                if (v) {
                    atomicAdd(&hist[static_cast<size_t>(cur) * kBins0 + b], v);
                    lh[b] = 0u;
                }
            }
            __syncthreads();
        }
        st = seg_hi;
    }
}

// What the level-1 pass writes when it also has to collect (see k_hist).
struct CollectOut {
    SegState* state;
    uint32_t* wt_cnt;
    uint64_t* sel_mask;
    uint64_t* eq_mask;
    uint2* cand;
    uint32_t* st_cand_cnt;
};

// Histogram of the next digit of the leader's magnitude keys, per segment.  LEVEL 1: bits 18..7
// of keys whose top 12 bits equal the chosen bucket; LEVEL 2: last 7 bits of keys matching 24
// bits.  Candidate mode reads the keys from the candidate list, full mode recomputes them from
// the leader's vector.
// LEVEL 1 is also the second full pass over the leader's vector for segments in candidate mode
// whose list the predicted pass did not fill (no prediction, or one that missed): per wave tile,
// keys above the level-0 bucket are members for sure, keys inside the bucket go to the
// supertile's slice of the candidate list and are counted here directly.  A slice that overflows
// (bucket keys clustered in one place) sends the whole segment back to full-pass mode for the
// kernels that follow; this kernel's counts are complete either way.
template <typename G, int LEVEL>
__global__ void __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(8)))   // 2048 blocks = 8 waves on every SIMD
k_hist(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const StDesc* __restrict__ sts, int n_st,
       const SegState* __restrict__ state, uint32_t* __restrict__ hist, const uint2* __restrict__ cand,
       const uint32_t* __restrict__ st_cand_cnt, CollectOut out)
{
    static_assert(LEVEL == 1 || LEVEL == 2, "level 0 is k_hist0");
    constexpr int NB = LEVEL == 1 ? kBins1 : kBins2;
    __shared__ uint32_t lh[NB];
    for (int b = threadIdx.x; b < NB; b += kBlock) lh[b] = 0u;
    __syncthreads();

    const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
    const int st_lo = static_cast<int>(static_cast<int64_t>(blockIdx.x) * n_st / gridDim.x);
    const int st_hi = static_cast<int>(static_cast<int64_t>(blockIdx.x + 1) * n_st / gridDim.x);

    auto count = [&](uint32_t key, uint32_t prefix) {
        if (LEVEL == 1) {
            if ((key >> (kBits1 + kBits2)) == prefix) atomicAdd(&lh[(key >> kBits2) & (kBins1 - 1)], 1u);
        } else {
            if ((key >> kBits2) == prefix) atomicAdd(&lh[key & (kBins2 - 1)], 1u);
        }
    };

    int cur = -1;
    uint32_t prefix = 0;
    bool skip = false, from_list = false, collect = false;
    for (int st = st_lo; st < st_hi; ++st) {
        const StDesc d = sts[st];
        if (d.seg != cur) {
            if (cur >= 0) {   // flush the finished segment's counts
                __syncthreads();
                for (int b = threadIdx.x; b < NB; b += kBlock) {
                    const uint32_t v = lh[b];
                    if (v) {
                        atomicAdd(&hist[static_cast<size_t>(cur) * NB + b], v);
                        lh[b] = 0u;
                    }
                }
                __syncthreads();
            }
            cur = d.seg;
            const SegState ss = state[cur];
            prefix = ss.prefix;
            skip = ss.done != 0;
            from_list = ss.mode == kModeCand;
            collect = LEVEL == 1 && from_list && ss.collected == 0;
        }
        if (skip) continue;
        if constexpr (LEVEL == 1) {
            if (collect) {   // block-uniform: no list yet, this pass makes it
                __shared__ uint32_t fill;
                __shared__ CollectStage stg;
                if (threadIdx.x == 0) fill = 0u;
                __syncthreads();
                const int64_t begin = d.begin, end = d.end;
                uint2* slice = out.cand + static_cast<size_t>(st) * kCandSlice;   // written directly: LDS is the histogram's
                for (int it = 0; it < kTilesPerSuper / kWaves; ++it) {
                    const int wt = it * kWaves + wave;
                    const int64_t p0 = static_cast<int64_t>(d.a0) + wt * kWaveTile + lane * kVec;
                    uint32_t key[4] = {0, 0, 0, 0};
                    bool ok[4] = {false, false, false, false};
                    if (p0 < end) leader_keys(mem, grad, lr, p0, begin, end, key, ok);
                    uint32_t n_above;
                    collect_tile<false>(key, ok, static_cast<uint32_t>(p0), prefix, prefix, wt, lane, &fill, nullptr, lh, n_above,
                                        stg, slice);
                }
                __syncthreads();
                collect_flush(stg, nullptr, static_cast<size_t>(st) * kTilesPerSuper, fill, out.wt_cnt, out.sel_mask, out.eq_mask,
                              slice);
                if (threadIdx.x == 0) {
                    const uint32_t n = fill;
                    out.st_cand_cnt[st] = n < kCandSlice ? n : kCandSlice;
                    if (n > kCandSlice) out.state[cur].mode = kModeFull;   // every overflowing block stores the same value
                }
                __syncthreads();   // the staging area is reused for the block's next supertile
                continue;
            }
        }
        if (from_list) {   // keys of this supertile that were copied to the candidate list
            const uint32_t cnt = st_cand_cnt[st];
            const uint2* slice = cand + static_cast<size_t>(st) * kCandSlice;
            for (uint32_t e = threadIdx.x; e < cnt; e += kBlock) count(slice[e].x, prefix);
            continue;
        }
        const int64_t begin = d.begin, end = d.end;
#pragma unroll 2
        for (int it = 0; it < kTilesPerSuper / kWaves; ++it) {
            const int64_t p0 = static_cast<int64_t>(d.a0) + (it * kWaves + wave) * kWaveTile + lane * kVec;
            if (p0 >= end) continue;
            uint32_t key[4];
            bool ok[4];
            leader_keys(mem, grad, lr, p0, begin, end, key, ok);
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (ok[c]) count(key[c], prefix);
        }
    }
    if (cur >= 0) {
        __syncthreads();
        for (int b = threadIdx.x; b < NB; b += kBlock) {
            const uint32_t v = lh[b];
            if (v) atomicAdd(&hist[static_cast<size_t>(cur) * NB + b], v);
        }
    }
}

// One block per segment: locate, from the top of the histogram, the bucket that holds the
// k_rem-th largest key of the current bucket, and narrow the state to it.
template <int LEVEL>
__global__ void __launch_bounds__(kBlock)
k_find(const SegDesc* __restrict__ segs, SegState* __restrict__ state, const uint32_t* __restrict__ hist,
       uint32_t* __restrict__ preds, const uint32_t* __restrict__ part, const uint32_t* __restrict__ overflow)
{
    constexpr int NB = LEVEL == 0 ? kBins0 : (LEVEL == 1 ? kBins1 : kBins2);
    constexpr int BITS = LEVEL == 0 ? kBits0 : (LEVEL == 1 ? kBits1 : kBits2);
    constexpr int CH = NB >= kBlock ? NB / kBlock : 1;     // bins per thread
    constexpr int ACTIVE = NB >= kBlock ? kBlock : NB;     // threads that own bins
    const int seg = blockIdx.x;
    const uint32_t* h = hist + static_cast<size_t>(seg) * NB;
    __shared__ uint32_t above[kWaves];   // per-wave totals

    SegState s = state[seg];
    if (LEVEL == 0) {
        s.prefix = 0;
        s.k_rem = static_cast<uint32_t>(segs[seg].k);
        s.done = s.k_rem == 0 ? 1u : 0u;
        s.T = 0xffffffffu;     // above every key: nothing is a member
        s.q = 0;
        s.mode = kModeFull;
        s.collected = 0;
        if (s.done) {
            if (threadIdx.x == 0) state[seg] = s;
            return;
        }
        // a prediction that held: the single pass already produced everything level 0 gives
        __shared__ int resolved;
        __shared__ uint32_t tot_s[kPartWords];
        const uint32_t p = preds[seg];
        if (p != 0) {                                       // block-uniform: sum the slotted copies of the counters
            if (threadIdx.x < kPartWords) tot_s[threadIdx.x] = 0u;
            __syncthreads();
            for (int i = threadIdx.x; i < kPartSlots * kPartWords; i += kBlock) {
                const uint32_t v = part[static_cast<size_t>(seg) * kPartSlots * kPartWords + i];
                if (v) atomicAdd(&tot_s[i % kPartWords], v);
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            uint32_t tot[1 + kWindow], digit, k_rem;
            resolved = 0;
            if (p != 0) {
                for (uint32_t j = 0; j <= kWindow; ++j) tot[j] = tot_s[j];
                if (spec_resolve(tot, overflow[seg] != 0, p, s.k_rem, digit, k_rem)) {
                    resolved = 1;
                    s.prefix = digit;
                    s.k_rem = k_rem;
                    s.mode = kModeCand;
                    s.collected = 1;
                    state[seg] = s;
                    preds[seg] = digit + 1;
                }
            }
        }
        __syncthreads();
        if (resolved) return;
    } else if (s.done) {
        return;
    }

    const int t = threadIdx.x;
    uint32_t mine = 0;
    if (t < ACTIVE)
        for (int b = 0; b < CH; ++b) mine += h[t * CH + b];
    // inclusive suffix sums over threads: within a wave by shuffles, across the 4 waves through LDS
    const int lane = t % kLanes, wave = t / kLanes;
    uint32_t suf = mine;
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) {
        const uint32_t v = __shfl_down(suf, off, kLanes);
        if (lane + off < kLanes) suf += v;
    }
    if (lane == 0) above[wave] = suf;                       // the wave's total
    __syncthreads();
    for (int w = wave + 1; w < kWaves; ++w) suf += above[w];
    const uint32_t incl = suf;               // keys in my chunk and all higher chunks
    const uint32_t excl = incl - mine;       // keys strictly above my chunk
    if (t < ACTIVE && excl < s.k_rem && s.k_rem <= incl) {
        uint32_t c = excl;
        for (int b = CH - 1; b >= 0; --b) {
            const uint32_t n = h[t * CH + b];
            if (c + n >= s.k_rem) {
                const uint32_t digit = static_cast<uint32_t>(t * CH + b);
                s.prefix = (s.prefix << BITS) | digit;
                s.k_rem -= c;
                if (LEVEL == 0) {
                    // the bucket's keys go to the candidate list if its slots can hold them
                    const uint64_t slots = static_cast<uint64_t>(segs[seg].st_count) * kCandSlice;
                    s.mode = n <= slots ? kModeCand : kModeFull;
                    preds[seg] = digit + 1;                 // prediction for the next step
                }
                if (LEVEL == 2) {
                    s.T = s.prefix;
                    s.q = s.k_rem;
                }
                state[seg] = s;
                break;
            }
            c += n;
        }
    }
}

// The last search of the threshold (7 key bits, 128 counters), done by every block that needs the
// result instead of by a kernel of its own (k_find<2>, which is launched instead when there are so
// many blocks that their added barriers cost more than the launch): from the top of the histogram, the bin that holds the
// k_rem-th largest key of the current 24-bit bucket.  All threads of the block call it; `bcast`
// is three words of LDS.  Returns the threshold key T and sets q, the number of keys equal to T that
// are members.  The histogram is 512 bytes, so re-reading it in every block is cheap (the 16 KB
// histograms of the earlier levels are not: those searches stay kernels).
__device__ __forceinline__ uint32_t find_threshold(const uint32_t* __restrict__ h, uint32_t prefix24, uint32_t k_rem,
                                                   uint32_t* bcast, uint32_t& q)
{
    static_assert(kBins2 == 2 * kLanes, "two waves hold the last level's counters");
    const int t = threadIdx.x, lane = t % kLanes;
    const uint32_t mine = t < kBins2 ? h[t] : 0u;
    uint32_t suf = mine;                                    // inclusive suffix sum inside the wave
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) {
        const uint32_t v = __shfl_down(suf, off, kLanes);
        if (lane + off < kLanes) suf += v;
    }
    if (t == kLanes) bcast[0] = suf;                        // total of bins 64..127
    if (t == kBins2) {                                      // if the counts were corrupted: nothing is a member
        bcast[1] = 0xffffffffu;
        bcast[2] = 0u;
    }
    __syncthreads();
    if (t < kLanes) suf += bcast[0];
    const uint32_t excl = suf - mine;                       // keys in higher bins
    if (t < kBins2 && excl < k_rem && k_rem <= suf) {       // exactly one bin qualifies
        bcast[1] = (prefix24 << kBits2) | static_cast<uint32_t>(t);
        bcast[2] = k_rem - excl;
    }
    __syncthreads();
    q = bcast[2];
    return bcast[1];
}

// Per wave tile of the leader's vector: number of keys above the threshold (low half of the
// packed counter) and equal to it (high half), and the two bitmasks that go with them.
// Full-pass mode recomputes every key; candidate mode adds the listed keys to what k_collect
// started.  Also leaves the supertile's totals for the prefix scan.
template <typename G>
__global__ void __launch_bounds__(kBlock)
k_tilecount(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const SegDesc* __restrict__ segs,
            const StDesc* __restrict__ sts, SegState* __restrict__ state, const uint32_t* __restrict__ hist2,
            uint32_t* __restrict__ wt_cnt, const uint2* __restrict__ cand, const uint32_t* __restrict__ st_cand_cnt,
            uint64_t* __restrict__ sel_mask, uint64_t* __restrict__ eq_mask, uint2* __restrict__ st_sum)
{
    const int st = blockIdx.x;
    const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
    const StDesc d = sts[st];
    const SegState ss = state[d.seg];
    const size_t tile0 = static_cast<size_t>(st) * kTilesPerSuper;
    __shared__ uint32_t cnt[kTilesPerSuper];
    __shared__ uint32_t bcast[3];
    uint32_t T = ss.T, q = ss.q;                            // an empty index set keeps T above every key
    if (!ss.done && hist2) {                                // block-uniform; without hist2 a kernel has searched already
        T = find_threshold(hist2 + static_cast<size_t>(d.seg) * kBins2, ss.prefix, ss.k_rem, bcast, q);
        if (st == segs[d.seg].st_first && threadIdx.x == 0) {   // for the tie quota of the slot pass
            state[d.seg].T = T;
            state[d.seg].q = q;
        }
    }

    if (!ss.done && ss.mode == kModeCand) {
        if (threadIdx.x < kTilesPerSuper) cnt[threadIdx.x] = wt_cnt[tile0 + threadIdx.x];
        __syncthreads();
        const uint32_t n = st_cand_cnt[st];
        const uint2* slice = cand + static_cast<size_t>(st) * kCandSlice;
        uint32_t* sel32 = reinterpret_cast<uint32_t*>(sel_mask);
        uint32_t* eq32 = reinterpret_cast<uint32_t*>(eq_mask);
        for (uint32_t e = threadIdx.x; e < n; e += kBlock) {
            const uint2 ce = slice[e];
            if (ce.x >= T) {
                const uint32_t rel = ce.y - static_cast<uint32_t>(d.a0);
                const uint32_t wt = rel / kWaveTile, l = (rel % kWaveTile) / kVec, c = rel % kVec;
                const size_t word = ((tile0 + wt) * 4 + c) * 2 + (l >> 5);
                if (ce.x > T) {
                    atomicAdd(&cnt[wt], 1u);
                    atomicOr(&sel32[word], 1u << (l & 31));
                } else {
                    atomicAdd(&cnt[wt], 0x10000u);
                    atomicOr(&eq32[word], 1u << (l & 31));
                }
            }
        }
        __syncthreads();
    } else {
        const int64_t begin = d.begin, end = d.end;
        for (int it = 0; it < kTilesPerSuper / kWaves; ++it) {
            const int wt = it * kWaves + wave;
            const int64_t p0 = static_cast<int64_t>(d.a0) + wt * kWaveTile + lane * kVec;
            uint32_t key[4] = {0, 0, 0, 0};
            bool ok[4] = {false, false, false, false};
            if (p0 < end) leader_keys(mem, grad, lr, p0, begin, end, key, ok);
            uint64_t gt[4], eq[4];
            uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                gt[c] = __ballot(ok[c] && key[c] > T);
                eq[c] = __ballot(ok[c] && key[c] == T);
                n_gt += __popcll(gt[c]);
                n_eq += __popcll(eq[c]);
            }
            if (lane == 0) {
                cnt[wt] = n_gt | (n_eq << 16);             // at most 256 each
                store_tile_masks(sel_mask, tile0 + wt, gt);
                store_tile_masks(eq_mask, tile0 + wt, eq);
            }
        }
        __syncthreads();
    }
    if (threadIdx.x < kLanes) {
        const uint32_t v = threadIdx.x < kTilesPerSuper ? cnt[threadIdx.x] : 0u;
        if (threadIdx.x < kTilesPerSuper) wt_cnt[tile0 + threadIdx.x] = v;
        const uint32_t s2 = wave_sum(v);                   // at most 8192 each: no carry between halves
        if (threadIdx.x == 0) st_sum[st] = make_uint2(s2 & 0xffffu, s2 >> 16);
    }
}

// Prefix scan, level 1: one block per chunk of up to 1024 supertiles of one segment; exclusive
// prefix of (above, equal) inside the chunk and the chunk's totals.
__global__ void __launch_bounds__(kChunk)
k_scan(const ChunkDesc* __restrict__ chunks, const uint2* __restrict__ st_sum, uint2* __restrict__ st_prefix,
       uint2* __restrict__ chunk_tot)
{
    const ChunkDesc cd = chunks[blockIdx.x];
    const int wave = threadIdx.x / kLanes, lane = threadIdx.x % kLanes;
    __shared__ uint2 wtot[kChunk / kLanes];
    const int i = threadIdx.x;
    const uint2 v = i < cd.st_count ? st_sum[cd.st_begin + i] : make_uint2(0, 0);
    uint2 inc = v;
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) {
        const uint32_t ax = __shfl_up(inc.x, off, kLanes), ay = __shfl_up(inc.y, off, kLanes);
        if (lane >= off) {
            inc.x += ax;
            inc.y += ay;
        }
    }
    if (lane == kLanes - 1) wtot[wave] = inc;
    __syncthreads();
    uint2 before = make_uint2(0, 0), total = make_uint2(0, 0);
    for (int w = 0; w < kChunk / kLanes; ++w) {
        const uint2 t = wtot[w];
        if (w < wave) {
            before.x += t.x;
            before.y += t.y;
        }
        total.x += t.x;
        total.y += t.y;
    }
    if (i < cd.st_count) st_prefix[cd.st_begin + i] = make_uint2(before.x + inc.x - v.x, before.y + inc.y - v.y);
    if (i == 0) chunk_tot[blockIdx.x] = total;
}

// Prefix scan, level 2, one wave per supertile: first output slot of each of its 32 wave tiles
// = members in earlier chunks + earlier supertiles of the chunk + earlier tiles of the
// supertile.  Keys equal to the threshold become members here, in position order, until the
// segment's quota q is used up (Eq. 2 with ties resolved towards the lowest positions).
__global__ void __launch_bounds__(kBlock)
k_slots(const SegDesc* __restrict__ segs, const StDesc* __restrict__ sts, int n_st, const SegState* __restrict__ state,
        const uint32_t* __restrict__ wt_cnt, const uint2* __restrict__ st_prefix, const uint2* __restrict__ chunk_tot,
        uint64_t* __restrict__ sel_mask, const uint64_t* __restrict__ eq_mask, uint32_t* __restrict__ tile_slot)
{
    const int st = blockIdx.x * kWaves + threadIdx.x / kLanes;
    const int lane = threadIdx.x % kLanes;
    if (st >= n_st) return;                                 // whole wave
    const StDesc d = sts[st];
    const SegDesc sd = segs[d.seg];
    const uint32_t q = state[d.seg].q;

    // totals of the segment's earlier chunks
    const int my_chunk = (st - sd.st_first) / kChunk;
    uint32_t cx = 0, cy = 0;
    for (int c = lane; c < my_chunk; c += kLanes) {
        const uint2 t = chunk_tot[sd.chunk_first + c];
        cx += t.x;
        cy += t.y;
    }
    cx = wave_sum(cx);
    cy = wave_sum(cy);
    const uint2 sp = st_prefix[st];

    const size_t tile = static_cast<size_t>(st) * kTilesPerSuper + lane;   // lanes 0..31 own one tile each
    const uint32_t packed = lane < kTilesPerSuper ? wt_cnt[tile] : 0u;
    uint32_t inc = packed;
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) {
        const uint32_t a = __shfl_up(inc, off, kLanes);
        if (lane >= off) inc += a;
    }
    const uint32_t excl = inc - packed;                     // halves stay below 8192: no carry
    const uint32_t gt_before = cx + sp.x + (excl & 0xffffu);
    const uint32_t eq_before = cy + sp.y + (excl >> 16);
    if (lane >= kTilesPerSuper) return;
    tile_slot[tile] = static_cast<uint32_t>(sd.out_base) + gt_before + (eq_before < q ? eq_before : q);

    const uint32_t own_eq = packed >> 16;
    uint32_t take = q > eq_before ? q - eq_before : 0u;     // ties of this tile that are members
    if (take > own_eq) take = own_eq;
    if (take == 0) return;
    uint64_t s4[4], e4[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        s4[c] = sel_mask[tile * 4 + c];
        e4[c] = eq_mask[tile * 4 + c];
    }
    if (take == own_eq) {
#pragma unroll
        for (int c = 0; c < 4; ++c) s4[c] |= e4[c];
    } else {                                                // the one tile where the quota runs out
        for (int l = 0; l < kLanes && take > 0; ++l) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (take > 0 && ((e4[c] >> l) & 1ull)) {
                    s4[c] |= 1ull << l;
                    --take;
                }
            }
        }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) sel_mask[tile * 4 + c] = s4[c];
}

// The all-learner pass, one (learner, 4 wave tiles) pair per block and consecutive blocks on
// consecutive learners: accumulate (Alg. 1 line 6), low-pass memory update with the residual
// zeroed on the index set (Eq. 5), and for members the learner's own value x_i (Eq. 3) into
// vals[learner][slot].  Membership and slots come from the leader's bitmask and prefix
// counts, so no learner's block reads another learner's data.
// INSIDE: all 1024 positions of the block belong to the segment, so the two streaming loads and
// the store need no guards and are issued back to back; otherwise every access is guarded.
template <typename G, bool INSIDE>
__device__ __forceinline__ void update_block(float* __restrict__ mem, const G* __restrict__ grad, float lr, float beta,
                                             float one_minus_beta, const StDesc& d, int wave, int lane, uint32_t rel0,
                                             const uint64_t S[4], uint32_t before, uint32_t total, uint32_t slot0,
                                             float* __restrict__ my_vals, int32_t* __restrict__ idx_out,
                                             float* stage_val, int32_t* stage_pos)
{
    // position of this lane's 4 elements; below 2^31 + 8192, so 32 bits hold it
    const uint32_t p0 = static_cast<uint32_t>(d.a0) + rel0;
    const int64_t begin = d.begin, end = d.end;
    const bool full = INSIDE || (static_cast<int64_t>(p0) >= begin && static_cast<int64_t>(p0) + 3 < end);
    const bool any_ok = INSIDE || (static_cast<int64_t>(p0) + 3 >= begin && static_cast<int64_t>(p0) < end);
    float4 m = make_float4(0, 0, 0, 0), x = m;
    if (INSIDE) {
        m = load4(mem + p0);
        const float4 g = load4(grad + p0);
        x = accumulate4(m, g, lr);
    } else if (any_ok) {
        m = load_guarded(mem, p0, begin, end, full);
        const float4 g = load_guarded(grad, p0, begin, end, full);
        x = accumulate4(m, g, lr);
    }
    bool sel[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) sel[c] = (S[c] >> lane) & 1ull;

    if (any_ok) {
        // Eq. 5: residual is x off the index set, 0 on it
        float4 out;
        out.x = fmaf(beta, sel[0] ? 0.0f : x.x, one_minus_beta * m.x);
        out.y = fmaf(beta, sel[1] ? 0.0f : x.y, one_minus_beta * m.y);
        out.z = fmaf(beta, sel[2] ? 0.0f : x.z, one_minus_beta * m.z);
        out.w = fmaf(beta, sel[3] ? 0.0f : x.w, one_minus_beta * m.w);
        if (INSIDE)
            store4(mem + p0, out);
        else
            store_guarded(mem, p0, begin, end, full, out);
    }

    if (total == 0) return;                                 // no member in the block's tiles (block-uniform)
    // The block's members occupy consecutive output slots (tiles are consecutive): compact them
    // through LDS and write them with one contiguous store.
    uint32_t rank = before;
#pragma unroll
    for (int c = 0; c < 4; ++c) rank += lanes_below(S[c]);
    const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (sel[c]) {
            stage_val[rank] = xs[c];
            if (idx_out) stage_pos[rank] = static_cast<int32_t>(p0 + c);
            ++rank;
        }
    }
    __syncthreads();
    const uint32_t slot_end = static_cast<uint32_t>(d.slot_end);
    for (uint32_t j = threadIdx.x; j < total; j += kBlock) {
        if (slot0 + j < slot_end) {                         // the bound only matters if the counts were corrupted
            my_vals[slot0 + j] = stage_val[j];
            if (idx_out) idx_out[slot0 + j] = stage_pos[j];
        }
    }
}

template <typename G>
__global__ void __launch_bounds__(kBlock)
k_update(LearnerPtrs lp, float lr, float beta, float one_minus_beta, const StDesc* __restrict__ sts, int n_st,
         const uint64_t* __restrict__ sel_mask, const uint32_t* __restrict__ tile_slot, float* __restrict__ vals,
         int64_t k_total, int32_t* __restrict__ idx_out)
{
    // grid = (learners, groups of 4 wave tiles split over y and z): x runs fastest, so blocks that
    // are scheduled together work on the same positions of different learners
    const int learner = blockIdx.x;
    const int group = blockIdx.y + blockIdx.z * gridDim.y;
    const int st = group / kUpdateBlocksPerSuper;
    if (st >= n_st) return;                                 // padding of the 3-d grid (whole block)
    // the wave's index is the same in all of its lanes: say so, and everything derived from it
    // (mask words, counts) stays in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
    const int lane = threadIdx.x % kLanes;
    const int wt0 = (group % kUpdateBlocksPerSuper) * kWaves;   // the block's first wave tile
    const StDesc d = sts[st];

    // membership of the block's 4 tiles (128 bytes) and the block's first output slot: small,
    // cache-resident, issued together with the streaming loads so that nothing waits on a
    // second round trip.  Tiles past the end of the segment have empty masks.
    const size_t tile0 = static_cast<size_t>(st) * kTilesPerSuper + wt0;
    const ulonglong2* mw = reinterpret_cast<const ulonglong2*>(sel_mask + tile0 * 4);
    ulonglong2 w[2 * kWaves];
#pragma unroll
    for (int j = 0; j < 2 * kWaves; ++j) w[j] = mw[j];
    const uint32_t slot0 = tile_slot[tile0];

    // my tile's ballots, and how many members the block's earlier tiles and the whole block hold
    uint64_t S[4] = {0, 0, 0, 0};
    uint32_t before = 0, total = 0;
#pragma unroll
    for (int t = 0; t < kWaves; ++t) {
        const uint32_t n = __popcll(w[2 * t].x) + __popcll(w[2 * t].y) + __popcll(w[2 * t + 1].x) + __popcll(w[2 * t + 1].y);
        if (t < wave) before += n;
        total += n;
        if (t == wave) {
            S[0] = w[2 * t].x;
            S[1] = w[2 * t].y;
            S[2] = w[2 * t + 1].x;
            S[3] = w[2 * t + 1].y;
        }
    }

    float* mem = lp.mem[learner];
    const G* grad = static_cast<const G*>(lp.grad[learner]);
    float* my_vals = vals + static_cast<size_t>(learner) * static_cast<size_t>(k_total);
    int32_t* my_idx = learner == 0 ? idx_out : nullptr;    // one learner's blocks write the positions
    const uint32_t rel0 = static_cast<uint32_t>((wt0 + wave) * kWaveTile + lane * kVec);
    const int64_t blk0 = static_cast<int64_t>(d.a0) + wt0 * kWaveTile;
    __shared__ float stage_val[kWaves * kWaveTile];
    __shared__ int32_t stage_pos[kWaves * kWaveTile];
    if (blk0 >= d.begin && blk0 + kWaves * kWaveTile <= d.end)
        update_block<G, true>(mem, grad, lr, beta, one_minus_beta, d, wave, lane, rel0, S, before, total, slot0, my_vals, my_idx,
                              stage_val, stage_pos);
    else
        update_block<G, false>(mem, grad, lr, beta, one_minus_beta, d, wave, lane, rel0, S, before, total, slot0, my_vals,
                               my_idx, stage_val, stage_pos);
}

// Sum of the learners' values at the index set, learner 0 first (Alg. 1 line 10 without 1/n).
__global__ void __launch_bounds__(kBlock)
k_reduce(const float* __restrict__ vals, int n_learners, int64_t k_total, float* __restrict__ red_out)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (t >= k_total) return;
    float s = vals[t];
    for (int i = 1; i < n_learners; ++i) s = s + vals[static_cast<size_t>(i) * static_cast<size_t>(k_total) + t];
    red_out[t] = s;
}

// ------------------------------------------------------------------------------------------
// chunk-wise selection (the selector of the paper's own implementation: Sec. 4, App. E)
// ------------------------------------------------------------------------------------------
// Largest value of v over the 64 lanes, in a scalar register.  Data-parallel-primitive moves inside
// the vector ALU (shift right by 1, 2, 4, 8 lanes inside each row of 16, then row 0's and rows
// 0-1's last lane broadcast to the following rows) instead of cross-lane reads through the LDS
// crossbar; lanes without a source take the identity 0.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
    constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;
    auto mx = [](uint32_t a, uint32_t b) { return a > b ? a : b; };
    v = mx(v, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), kRowShr1, 0xf, 0xf, false)));
    v = mx(v, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), kRowShr2, 0xf, 0xf, false)));
    v = mx(v, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), kRowShr4, 0xf, 0xf, false)));
    v = mx(v, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), kRowShr8, 0xf, 0xf, false)));
    v = mx(v, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), kRowBcast15, 0xa, 0xf, false)));
    v = mx(v, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), kRowBcast31, 0xc, 0xf, false)));
    return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), kLanes - 1));
}

// Leader pass of the chunk-wise selector, one wave per wave tile: every element becomes the word
// (magnitude key << 32 | ~position), so that the largest word of a chunk is its largest
// magnitude at the lowest position; for each chunk of the tile's segment that overlaps the tile
// the wave reduces its part and merges it into best[out_base + chunk] with one 64-bit atomic max
// (a chunk touches at most chunk/256 + 2 tiles).  Chunks are counted from the segment's first
// element.  Also clears the tile's membership mask.
template <typename G>
__global__ void __launch_bounds__(kBlock)
k_chunk_select(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const SegDesc* __restrict__ segs,
               const StDesc* __restrict__ sts, int n_st, unsigned long long* __restrict__ best,
               uint64_t* __restrict__ sel_mask)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes), lane = threadIdx.x % kLanes;
    const int64_t group = static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x;   // 4 wave tiles
    const int st = static_cast<int>(group / kUpdateBlocksPerSuper);
    if (st >= n_st) return;                                 // whole block
    const int wt = static_cast<int>(group % kUpdateBlocksPerSuper) * kWaves + wave;
    const StDesc d = sts[st];
    const SegDesc sd = segs[d.seg];
    const size_t tile = static_cast<size_t>(st) * kTilesPerSuper + wt;
    if (lane == 0) {
        const uint64_t zero[4] = {0, 0, 0, 0};
        store_tile_masks(sel_mask, tile, zero);
    }
    // positions and chunk sizes are below 2^31 + 8192: 32-bit arithmetic throughout
    const uint32_t begin = static_cast<uint32_t>(sd.begin), end = static_cast<uint32_t>(sd.end);
    const uint32_t ch = static_cast<uint32_t>(sd.sel_chunk);
    const uint32_t tile_first = static_cast<uint32_t>(d.a0) + static_cast<uint32_t>(wt) * kWaveTile;
    const uint32_t v_lo = tile_first > begin ? tile_first : begin;             // the tile's part of the segment
    const uint32_t v_hi = tile_first + kWaveTile < end ? tile_first + kWaveTile : end;
    if (v_lo >= v_hi) return;                               // whole wave: the tile lies outside the segment
    const uint32_t p0 = tile_first + lane * kVec;
    float4 m, g;
    if (tile_first >= begin && tile_first + kWaveTile <= end) {   // wave-uniform: the whole tile belongs to the segment
        m = load4(mem + p0);
        g = load4(grad + p0);
    } else {
        leader_load(mem, grad, p0, static_cast<int64_t>(begin), static_cast<int64_t>(end), m, g);
    }
    const float4 x = accumulate4(m, g, lr);
    const uint32_t key[4] = {magnitude_key(x.x), magnitude_key(x.y), magnitude_key(x.z), magnitude_key(x.w)};
    const uint32_t j_first = (v_lo - begin) / ch, j_last = (v_hi - 1 - begin) / ch;
    uint32_t lo = begin + j_first * ch;                     // at most v_lo: no overflow
    for (uint32_t j = j_first; j <= j_last; ++j, lo += ch) { // wave-uniform trip count
        // positions of chunk j: lo <= p < lo + chunk, i.e. p - lo < chunk (unsigned; lo + chunk may pass 2^32),
        // and p < end.  The largest word (key << 32 | ~position) in two 32-bit steps: the largest key,
        // then the largest ~position among the elements that have it.  ~position is never 0, so a
        // result of 0 means that no element of the chunk lies in this tile.
        bool in[4];
        uint32_t k_here = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            in[c] = p0 + c - lo < ch && p0 + c < end;
            if (in[c] && key[c] > k_here) k_here = key[c];
        }
        const uint32_t k_max = wave_max_u32(k_here);
        uint32_t inv_here = 0;                              // element c = 0 has the largest ~position of the lane
#pragma unroll
        for (int c = 3; c >= 0; --c)
            if (in[c] && key[c] == k_max) inv_here = 0xffffffffu - (p0 + c);
        const uint32_t inv_max = wave_max_u32(inv_here);
        if (lane == 0)
            atomicMax(&best[static_cast<uint32_t>(sd.out_base) + j], (static_cast<unsigned long long>(k_max) << 32) | inv_max);
    }
}

// After the leader pass: position of each chunk's winner to idx_out and to the membership mask;
// first output slot of every wave tile (chunk j of a segment owns slot out_base + j); and the
// other copy of best[] is cleared for the next step.
__global__ void __launch_bounds__(kBlock)
k_chunk_marks(const SegDesc* __restrict__ segs, int n_tensors, const StDesc* __restrict__ sts,
              const unsigned long long* __restrict__ best, unsigned long long* __restrict__ best_next, int64_t k_total,
              int64_t n_tiles, uint64_t* __restrict__ sel_mask, uint32_t* __restrict__ tile_slot,
              int32_t* __restrict__ idx_out)
{
    const int64_t t = (static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x) * kBlock + threadIdx.x;
    if (t < k_total) {
        // the segment that owns output slot t: the last one whose first slot is <= t (a segment without
        // slots shares its first slot with its successor, so it is never the last such one while t < k_total)
        int lo = 0, hi = n_tensors - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) / 2;
            if (segs[mid].out_base <= t) lo = mid; else hi = mid - 1;
        }
        const SegDesc sd = segs[lo];
        const uint32_t pos = 0xffffffffu - static_cast<uint32_t>(best[t]);
        idx_out[t] = static_cast<int32_t>(pos);
        const uint32_t rel = pos - (static_cast<uint32_t>(sd.begin) & ~static_cast<uint32_t>(kVec - 1));
        const size_t tile = static_cast<size_t>(sd.st_first) * kTilesPerSuper + rel / kWaveTile;
        const uint32_t l = (rel % kWaveTile) / kVec, c = rel % kVec;
        atomicOr(reinterpret_cast<uint32_t*>(sel_mask) + (tile * 4 + c) * 2 + (l >> 5), 1u << (l & 31));
        best_next[t] = 0ull;
    }
    if (t < n_tiles) {
        // winners of the segment before this tile: one per chunk that ends before it, plus the
        // straddling chunk's winner if it lies before the tile
        const StDesc d = sts[t / kTilesPerSuper];
        const SegDesc sd = segs[d.seg];
        const uint32_t begin = static_cast<uint32_t>(sd.begin), end = static_cast<uint32_t>(sd.end);
        const uint32_t ch = static_cast<uint32_t>(sd.sel_chunk);
        const uint32_t first = static_cast<uint32_t>(d.a0) + static_cast<uint32_t>(t % kTilesPerSuper) * kWaveTile;
        uint32_t slot = static_cast<uint32_t>(sd.out_base);
        if (first >= end) {
            slot += static_cast<uint32_t>(sd.k);            // past the segment: its mask is empty
        } else if (first > begin) {
            const uint32_t j = (first - begin) / ch;
            slot += j;
            if (begin + j * ch < first) {
                const uint32_t pos = 0xffffffffu - static_cast<uint32_t>(best[static_cast<uint32_t>(sd.out_base) + j]);
                if (pos < first) ++slot;
            }
        }
        tile_slot[t] = slot;
    }
}

// Weight update on the index set (Alg. 1 lines 10 and 12): theta[idx[t]] -= scale * vals[t].
__global__ void __launch_bounds__(kBlock)
k_apply_update(float* __restrict__ theta, const int32_t* __restrict__ idx, const float* __restrict__ vals, int64_t k,
               float neg_scale)
{
    const int64_t t = (static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x) * kBlock + threadIdx.x;
    if (t >= k) return;
    const int32_t j = idx[t];
    theta[j] = fmaf(neg_scale, vals[t], theta[j]);
}

// Similarity diagnostics (Sec. 3) --------------------------------------------------------------
// y[p] = sum over learners 0..n-1, left to right, of x_i[p] = fma(lr, grad_i[p], mem_i[p]): the
// all-reduced error-feedback gradient whose top-k is the "true top-k" (times n, which does not
// change the order of magnitudes).
template <typename G>
__global__ void __launch_bounds__(kBlock)
k_sum_x(const LearnerPtrs lp, int n_learners, float lr, int64_t begin, int64_t end, float* __restrict__ y)
{
    const int64_t p = begin + (static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x) * kBlock + threadIdx.x;
    if (p >= end) return;
    float acc = fmaf(lr, widen(static_cast<const G*>(lp.grad[0])[p]), lp.mem[0][p]);
    for (int i = 1; i < n_learners; ++i) acc += fmaf(lr, widen(static_cast<const G*>(lp.grad[i])[p]), lp.mem[i][p]);
    y[p] = acc;
}

__global__ void __launch_bounds__(kBlock) k_set_ks(const SegDesc* __restrict__ segs, int n_tensors, int32_t* __restrict__ d)
{
    const int s = blockIdx.x * kBlock + threadIdx.x;
    if (s < n_tensors) d[s] = segs[s].k;
}

// d[seg] -= |A and B| over the membership masks of two selections: with d preset to k, what is
// left is the number of positions of one index set that the other one lacks (Eq. 6: the binarised
// vectors differ in 2d places).  One wave per supertile.
__global__ void __launch_bounds__(kBlock)
k_mask_overlap(const StDesc* __restrict__ sts, int n_st, const uint64_t* __restrict__ mask_a,
               const uint64_t* __restrict__ mask_b, int32_t* __restrict__ d)
{
    const int st = blockIdx.x * kWaves + threadIdx.x / kLanes;
    if (st >= n_st) return;
    const int lane = threadIdx.x % kLanes;
    const size_t w0 = static_cast<size_t>(st) * kTilesPerSuper * 4;   // 4 words per wave tile
    uint32_t both = 0;
    for (int w = lane; w < kTilesPerSuper * 4; w += kLanes) both += __popcll(mask_a[w0 + w] & mask_b[w0 + w]);
    both = wave_sum(both);
    if (lane == 0 && both) atomicSub(&d[sts[st].seg], static_cast<int32_t>(both));
}

// Partial sums of a.b, a.a and b.b in binary64, added into acc[1..3].
__global__ void __launch_bounds__(kBlock)
k_dots(const float* __restrict__ a, const float* __restrict__ b, int64_t numel, double* __restrict__ acc)
{
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int64_t j = blockIdx.x * static_cast<int64_t>(kBlock) + threadIdx.x; j < numel;
         j += static_cast<int64_t>(gridDim.x) * kBlock) {
        const double x = a[j], y = b[j];
        ab += x * y;
        aa += x * x;
        bb += y * y;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        ab += __shfl_xor(ab, off, kLanes);
        aa += __shfl_xor(aa, off, kLanes);
        bb += __shfl_xor(bb, off, kLanes);
    }
    __shared__ double part[3][kWaves];
    if (threadIdx.x % kLanes == 0) {
        part[0][threadIdx.x / kLanes] = ab;
        part[1][threadIdx.x / kLanes] = aa;
        part[2][threadIdx.x / kLanes] = bb;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        double t = 0.0;
        for (int w = 0; w < kWaves; ++w) t += part[threadIdx.x][w];
        atomicAdd(&acc[1 + threadIdx.x], t);
    }
}

// acc[0] = 1 - a.b / (|a| |b|)
__global__ void k_cosine_final(double* __restrict__ acc)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) acc[0] = 1.0 - acc[1] / (sqrt(acc[2]) * sqrt(acc[3]));
}

// Plain streaming copy, one 16-byte nontemporal load and store per thread: the yardstick the
// other kernels' bandwidth and the profiler's byte counters are compared with.
__global__ void __launch_bounds__(kBlock) k_copy(const vf4_t* __restrict__ src, vf4_t* __restrict__ dst, size_t n16)
{
    const size_t i = (static_cast<size_t>(blockIdx.y) * gridDim.x + blockIdx.x) * kBlock + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline int64_t max_supertiles(int64_t numel_max, int n_tensors_max)
{
    return numel_max / kSuper + 2 * static_cast<int64_t>(n_tensors_max) + 2;
}

inline int64_t max_chunks(int64_t numel_max, int n_tensors_max)
{
    return max_supertiles(numel_max, n_tensors_max) / kChunk + static_cast<int64_t>(n_tensors_max) + 1;
}

struct WsLayout {
    size_t segs, sts, chunks, preds, state, wt_cnt, st_sum, st_prefix, chunk_tot, st_cand_cnt, cand, sel_mask, eq_mask,
        tile_slot, vals, best, total;
    // per-step counters and histograms: two copies of one zone, used alternately (offsets inside a copy)
    size_t zone[2], zone_bytes, z_overflow, z_part, z_hist0, z_hist1, z_hist2;
};

WsLayout layout_for(int64_t numel_max, int n_tensors_max, int n_learners_max, int64_t k_max)
{
    const size_t nt = static_cast<size_t>(n_tensors_max);
    const size_t nst = static_cast<size_t>(max_supertiles(numel_max, n_tensors_max));
    const size_t nch = static_cast<size_t>(max_chunks(numel_max, n_tensors_max));
    const size_t ntile = nst * kTilesPerSuper;
    WsLayout l{};
    size_t o = 0;
    auto take = [&](size_t bytes) {
        const size_t at = o;
        o = align_up(o + bytes, 256);
        return at;
    };
    l.segs = take(nt * sizeof(SegDesc));
    l.sts = take(nst * sizeof(StDesc));
    l.chunks = take(nch * sizeof(ChunkDesc));
    l.preds = take(nt * sizeof(uint32_t));
    l.state = take(nt * sizeof(SegState));
    {
        size_t z = 0;
        auto ztake = [&](size_t bytes) {
            const size_t at = z;
            z = align_up(z + bytes, 256);
            return at;
        };
        l.z_overflow = ztake(nt * sizeof(uint32_t));
        l.z_part = ztake(nt * kPartSlots * kPartWords * sizeof(uint32_t));
        l.z_hist0 = ztake(nt * kBins0 * sizeof(uint32_t));
        l.z_hist1 = ztake(nt * kBins1 * sizeof(uint32_t));
        l.z_hist2 = ztake(nt * kBins2 * sizeof(uint32_t));
        l.zone_bytes = z;
    }
    l.zone[0] = take(l.zone_bytes);
    l.zone[1] = take(l.zone_bytes);
    l.wt_cnt = take(ntile * sizeof(uint32_t));
    l.st_sum = take(nst * sizeof(uint2));
    l.st_prefix = take(nst * sizeof(uint2));
    l.chunk_tot = take(nch * sizeof(uint2));
    l.st_cand_cnt = take(nst * sizeof(uint32_t));
    l.cand = take(nst * kCandSlice * sizeof(uint2));
    l.sel_mask = take(ntile * 4 * sizeof(uint64_t));
    l.eq_mask = take(ntile * 4 * sizeof(uint64_t));
    l.tile_slot = take(ntile * sizeof(uint32_t));
    l.vals = take(static_cast<size_t>(n_learners_max) * static_cast<size_t>(k_max) * sizeof(float));
    l.best = take(2 * static_cast<size_t>(k_max) * sizeof(unsigned long long));   // chunk-wise selector, two copies
    l.total = o;
    return l;
}

bool sizes_ok(int64_t numel_max, int n_tensors_max, int n_learners_max, int64_t k_max)
{
    return numel_max >= 0 && numel_max <= INT32_MAX && n_tensors_max >= 1 && n_learners_max >= 1 &&
           n_learners_max <= SCALECOM_MAX_LEARNERS && k_max >= 0 && k_max <= numel_max;
}

}  // namespace

struct scalecom_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    char* ws = nullptr;
    int n_learners_max = 0;
    int64_t numel_max = 0;
    int64_t k_max = 0;
    int n_tensors_max = 0;
    scalecom_grad_dtype gdt = SCALECOM_GRAD_F32;
    WsLayout lay{};
    // tables of the layout used last, kept on the device until the layout changes
    std::vector<int64_t> cached_offsets, cached_ks, cached_chunks;
    int n_st = 0, n_chunks = 0;
    int parity = 0;                  // which copy of the scratch zone the next step uses
    bool scratch_clean = false;      // false: both copies must be cleared before the next step
    int best_parity = 0;             // same scheme for the chunk-wise selector's per-chunk maxima
    bool best_clean = false;
    char* pinned = nullptr;          // staging for the table upload
    size_t pinned_bytes = 0;
    hipEvent_t upload_done = nullptr;
    bool upload_pending = false;
    // optional per-phase timing: events recorded on the context's stream between kernel groups
    std::vector<hipEvent_t> prof_events;     // (SCALECOM_N_PHASES + 1) per recorded step
    int prof_cap = 0, prof_steps = 0;
    int prof_every = 1, prof_seen = 0;   // of the calls since timing began, every prof_every-th is recorded
    bool prof_all = false;           // false: only the boundaries of the all-learner pass are recorded
    std::string last_error;
};

namespace {

scalecom_status fail(scalecom_ctx* ctx, scalecom_status st, const std::string& msg)
{
    if (ctx) ctx->last_error = msg;
    return st;
}

#define SC_HIP(ctx, call)                                                                              \
    do {                                                                                               \
        hipError_t e_ = (call);                                                                        \
        if (e_ != hipSuccess)                                                                          \
            return fail((ctx), SCALECOM_EHIP, std::string(#call) + ": " + hipGetErrorString(e_));      \
    } while (0)

struct DeviceGuard {   // make the context's device current for the duration of a call
    int prev = -1;
    bool changed = false;
    hipError_t enter(int device)
    {
        hipError_t e = hipGetDevice(&prev);
        if (e != hipSuccess) return e;
        if (prev != device) {
            e = hipSetDevice(device);
            changed = e == hipSuccess;
        }
        return e;
    }
    ~DeviceGuard()
    {
        if (changed) (void)hipSetDevice(prev);
    }
};

size_t pinned_bytes_for(int64_t numel_max, int n_tensors_max)
{
    return align_up(sizeof(SegDesc) * static_cast<size_t>(n_tensors_max), 256) +
           align_up(sizeof(StDesc) * static_cast<size_t>(max_supertiles(numel_max, n_tensors_max)), 256) +
           sizeof(ChunkDesc) * static_cast<size_t>(max_chunks(numel_max, n_tensors_max));
}

// Rebuild and upload the segment, supertile and chunk tables if the layout differs from the cached one.
scalecom_status ensure_tables(scalecom_ctx* ctx, int n_tensors, const int64_t* offsets, const int64_t* ks,
                              const int64_t* sel_chunks = nullptr)
{
    // chunk sizes of the chunk-wise selector (0: exact selection) are part of the layout: two
    // chunk sizes can give the same number of chunks
    std::vector<int64_t> ch(static_cast<size_t>(n_tensors), 0);
    if (sel_chunks) ch.assign(sel_chunks, sel_chunks + n_tensors);
    const bool same = ctx->cached_ks.size() == static_cast<size_t>(n_tensors) &&
                      std::memcmp(ctx->cached_offsets.data(), offsets, sizeof(int64_t) * (n_tensors + 1)) == 0 &&
                      std::memcmp(ctx->cached_ks.data(), ks, sizeof(int64_t) * n_tensors) == 0 && ctx->cached_chunks == ch;
    if (same) return SCALECOM_OK;

    if (ctx->upload_pending) {   // staging memory may still be read by an earlier copy
        SC_HIP(ctx, hipEventSynchronize(ctx->upload_done));
        ctx->upload_pending = false;
    }
    const int64_t st_cap = max_supertiles(ctx->numel_max, ctx->n_tensors_max);
    const int64_t ch_cap = max_chunks(ctx->numel_max, ctx->n_tensors_max);
    SegDesc* segs = reinterpret_cast<SegDesc*>(ctx->pinned);
    const size_t st_off = align_up(sizeof(SegDesc) * static_cast<size_t>(ctx->n_tensors_max), 256);
    StDesc* sts = reinterpret_cast<StDesc*>(ctx->pinned + st_off);
    const size_t ch_off = st_off + align_up(sizeof(StDesc) * static_cast<size_t>(st_cap), 256);
    ChunkDesc* chunks = reinterpret_cast<ChunkDesc*>(ctx->pinned + ch_off);
    int64_t n_st = 0, n_ch = 0, out = 0;
    for (int s = 0; s < n_tensors; ++s) {
        const int64_t b = offsets[s], e = offsets[s + 1];
        const int64_t a_first = b & ~static_cast<int64_t>(kVec - 1);
        const int64_t count = e > b ? (e - a_first + kSuper - 1) / kSuper : 0;
        const int64_t n_chunks = (count + kChunk - 1) / kChunk;
        if (n_st + count > st_cap || n_ch + n_chunks > ch_cap) return fail(ctx, SCALECOM_ENOMEM, "tile table overflow");
        segs[s] = SegDesc{static_cast<int32_t>(b),    static_cast<int32_t>(e),     static_cast<int32_t>(ks[s]),
                          static_cast<int32_t>(out),  static_cast<int32_t>(n_st),  static_cast<int32_t>(count),
                          static_cast<int32_t>(n_ch), static_cast<int32_t>(n_chunks), static_cast<int32_t>(ch[s]), 0};
        for (int64_t j = 0; j < count; ++j)
            sts[n_st + j] = StDesc{s, static_cast<int32_t>(a_first + j * kSuper), static_cast<int32_t>(b),
                                   static_cast<int32_t>(e), static_cast<int32_t>(out + ks[s]), {0, 0, 0}};
        for (int64_t c = 0; c < n_chunks; ++c)
            chunks[n_ch + c] = ChunkDesc{s, static_cast<int32_t>(n_st + c * kChunk),
                                         static_cast<int32_t>(std::min<int64_t>(kChunk, count - c * kChunk)), 0};
        n_st += count;
        n_ch += n_chunks;
        out += ks[s];
    }
    SC_HIP(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.segs, segs, sizeof(SegDesc) * n_tensors, hipMemcpyHostToDevice,
                               ctx->stream));
    if (n_st > 0) {
        SC_HIP(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.sts, sts, sizeof(StDesc) * n_st, hipMemcpyHostToDevice,
                                   ctx->stream));
        SC_HIP(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.chunks, chunks, sizeof(ChunkDesc) * n_ch, hipMemcpyHostToDevice,
                                   ctx->stream));
    }
    // predictions of the previous layout's buckets mean nothing for this one
    k_init<<<1, kBlock, 0, ctx->stream>>>(reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.preds),
                                          static_cast<size_t>(ctx->n_tensors_max));
    ctx->scratch_clean = false;
    SC_HIP(ctx, hipEventRecord(ctx->upload_done, ctx->stream));
    ctx->upload_pending = true;
    ctx->n_st = static_cast<int>(n_st);
    ctx->n_chunks = static_cast<int>(n_ch);
    ctx->cached_offsets.assign(offsets, offsets + n_tensors + 1);
    ctx->cached_ks.assign(ks, ks + n_tensors);
    ctx->cached_chunks = ch;
    return SCALECOM_OK;
}

// Is the step that is being enqueued one whose phase boundaries are recorded?  (Counts the call.)
bool timed_step(scalecom_ctx* ctx)
{
    if (ctx->prof_steps >= ctx->prof_cap) return false;
    return ctx->prof_seen++ % ctx->prof_every == 0;
}

// The all-learner pass and the sum over learners, shared by the exact and the chunk-wise selector:
// both leave the membership mask and the first output slot of every wave tile behind.
template <typename G, typename Mark>
void launch_update_reduce(scalecom_ctx* ctx, const LearnerPtrs& lp, int n_learners, int64_t k_total, float beta, float lr,
                          int32_t* idx_out, float* red_out, Mark&& mark)
{
    char* ws = ctx->ws;
    const WsLayout& l = ctx->lay;
    hipStream_t s = ctx->stream;
    const int n_st = ctx->n_st;
    const StDesc* sts = reinterpret_cast<const StDesc*>(ws + l.sts);
    const uint64_t* sel_mask = reinterpret_cast<const uint64_t*>(ws + l.sel_mask);
    const uint32_t* tile_slot = reinterpret_cast<const uint32_t*>(ws + l.tile_slot);
    float* vals = reinterpret_cast<float*>(ws + l.vals);
    // groups of 4 wave tiles over grid y and z (y is limited to 65535); surplus groups find no supertile
    const int64_t groups = static_cast<int64_t>(n_st) * kUpdateBlocksPerSuper;
    const unsigned gz = static_cast<unsigned>((groups + 65534) / 65535);
    const unsigned gy = static_cast<unsigned>((groups + gz - 1) / gz);
    k_update<G><<<dim3(n_learners, gy, gz), kBlock, 0, s>>>(lp, lr, beta, 1.0f - beta, sts, n_st, sel_mask, tile_slot, vals,
                                                           k_total, idx_out);
    mark(4);
    if (k_total > 0)
        k_reduce<<<static_cast<unsigned>((k_total + kBlock - 1) / kBlock), kBlock, 0, s>>>(vals, n_learners, k_total,
                                                                                           red_out);
}

// The exact selection on one vector x = fma(lr, grad, mem) (Eq. 2): every kernel from the first
// look at the vector to the output slot of every wave tile.  Leaves the membership mask, the
// tile slots and the threshold behind.  `preds` holds one bucket prediction per segment (read and
// rewritten).  Uses one copy of the scratch zone and leaves the other one cleared.
template <typename G, typename Mark>
void launch_select(scalecom_ctx* ctx, const float* memL, const G* gradL, float lr, int n_tensors, uint32_t* preds,
                   Mark&& mark)
{
    char* ws = ctx->ws;
    const WsLayout& l = ctx->lay;
    const SegDesc* segs = reinterpret_cast<const SegDesc*>(ws + l.segs);
    const StDesc* sts = reinterpret_cast<const StDesc*>(ws + l.sts);
    const ChunkDesc* chunks = reinterpret_cast<const ChunkDesc*>(ws + l.chunks);
    SegState* state = reinterpret_cast<SegState*>(ws + l.state);
    char* zone = ws + l.zone[ctx->parity];
    uint32_t* overflow = reinterpret_cast<uint32_t*>(zone + l.z_overflow);
    uint32_t* part = reinterpret_cast<uint32_t*>(zone + l.z_part);
    uint32_t* hist0 = reinterpret_cast<uint32_t*>(zone + l.z_hist0);
    uint32_t* hist1 = reinterpret_cast<uint32_t*>(zone + l.z_hist1);
    uint32_t* hist2 = reinterpret_cast<uint32_t*>(zone + l.z_hist2);
    uint32_t* next_zone = reinterpret_cast<uint32_t*>(ws + l.zone[ctx->parity ^ 1]);
    const size_t zone_words = l.zone_bytes / sizeof(uint32_t);
    uint32_t* wt_cnt = reinterpret_cast<uint32_t*>(ws + l.wt_cnt);
    uint2* st_sum = reinterpret_cast<uint2*>(ws + l.st_sum);
    uint2* st_prefix = reinterpret_cast<uint2*>(ws + l.st_prefix);
    uint2* chunk_tot = reinterpret_cast<uint2*>(ws + l.chunk_tot);
    uint32_t* st_cand_cnt = reinterpret_cast<uint32_t*>(ws + l.st_cand_cnt);
    uint2* cand = reinterpret_cast<uint2*>(ws + l.cand);
    uint64_t* sel_mask = reinterpret_cast<uint64_t*>(ws + l.sel_mask);
    uint64_t* eq_mask = reinterpret_cast<uint64_t*>(ws + l.eq_mask);
    uint32_t* tile_slot = reinterpret_cast<uint32_t*>(ws + l.tile_slot);
    hipStream_t s = ctx->stream;
    const int n_st = ctx->n_st;

    if (!ctx->scratch_clean) {   // first step, new layout, or a failed step: clear both scratch copies
        const size_t words = 2 * zone_words;   // the two copies are adjacent
        const int grid = static_cast<int>(std::min<size_t>((words + kBlock - 1) / kBlock, 4096));
        k_init<<<grid, kBlock, 0, s>>>(reinterpret_cast<uint32_t*>(ws + l.zone[0]), words);
    }
    const int hgrid = std::min(n_st, kHistGridMax);
    ctx->scratch_clean = false;             // until every kernel of this selection has been enqueued
    k_predicted<G><<<n_st, kBlock, 0, s>>>(memL, gradL, lr, segs, sts, cand, st_cand_cnt, preds, wt_cnt, sel_mask, eq_mask,
                                           part, overflow, next_zone, zone_words);
    k_hist0<G><<<hgrid, kBlock, 0, s>>>(memL, gradL, lr, segs, sts, n_st, hist0, preds, part, overflow);
    k_find<0><<<n_tensors, kBlock, 0, s>>>(segs, state, hist0, preds, part, overflow);
    mark(1);
    const CollectOut cout{state, wt_cnt, sel_mask, eq_mask, cand, st_cand_cnt};
    k_hist<G, 1><<<hgrid, kBlock, 0, s>>>(memL, gradL, lr, sts, n_st, state, hist1, cand, st_cand_cnt, cout);
    k_find<1><<<n_tensors, kBlock, 0, s>>>(segs, state, hist1, preds, part, overflow);
    k_hist<G, 2><<<hgrid, kBlock, 0, s>>>(memL, gradL, lr, sts, n_st, state, hist2, cand, st_cand_cnt, cout);
    // the last search: inside k_tilecount's blocks, or a kernel of its own when those are very many
    const bool fold_last = n_st <= kFoldLastSearchMaxSt;
    if (!fold_last) k_find<2><<<n_tensors, kBlock, 0, s>>>(segs, state, hist2, preds, part, overflow);
    mark(2);
    k_tilecount<G><<<n_st, kBlock, 0, s>>>(memL, gradL, lr, segs, sts, state, fold_last ? hist2 : nullptr, wt_cnt, cand, st_cand_cnt, sel_mask, eq_mask,
                                           st_sum);
    k_scan<<<ctx->n_chunks, kChunk, 0, s>>>(chunks, st_sum, st_prefix, chunk_tot);
    k_slots<<<(n_st + kWaves - 1) / kWaves, kBlock, 0, s>>>(segs, sts, n_st, state, wt_cnt, st_prefix, chunk_tot, sel_mask,
                                                            eq_mask, tile_slot);
    if (hipPeekAtLastError() == hipSuccess) {   // the copy for the next selection was cleared by this one
        ctx->parity ^= 1;
        ctx->scratch_clean = true;
    }
}

template <typename G>
scalecom_status launch_step(scalecom_ctx* ctx, const LearnerPtrs& lp, int n_learners, int n_tensors, int64_t k_total,
                            float beta, float lr, int leader, int32_t* idx_out, float* red_out)
{
    hipStream_t s = ctx->stream;
    // phase boundaries for scalecom_timing_*: one event before the first kernel, one after each phase
    const bool timed = timed_step(ctx);
    hipEvent_t* ev = timed ? &ctx->prof_events[static_cast<size_t>(ctx->prof_steps) * (SCALECOM_N_PHASES + 1)] : nullptr;
    auto mark = [&](int boundary) {   // boundaries 3 and 4 enclose the all-learner pass
        if (timed && (ctx->prof_all || boundary == 3 || boundary == 4)) (void)hipEventRecord(ev[boundary], s);
    };
    if (ctx->n_st > 0) {
        mark(0);
        launch_select<G>(ctx, lp.mem[leader], static_cast<const G*>(lp.grad[leader]), lr, n_tensors,
                         reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.preds), mark);
        mark(3);
        launch_update_reduce<G>(ctx, lp, n_learners, k_total, beta, lr, idx_out, red_out, mark);
        mark(5);
        if (timed) ++ctx->prof_steps;
    }
    SC_HIP(ctx, hipGetLastError());
    return SCALECOM_OK;
}

// One step with the chunk-wise selector: leader pass (per-chunk maxima), marks, then the same
// all-learner pass and reduction as the exact path.
template <typename G>
scalecom_status launch_chunked(scalecom_ctx* ctx, const LearnerPtrs& lp, int n_learners, int n_tensors, int64_t k_total,
                               float beta, float lr, int leader, int32_t* idx_out, float* red_out)
{
    char* ws = ctx->ws;
    const WsLayout& l = ctx->lay;
    hipStream_t s = ctx->stream;
    unsigned long long* best = reinterpret_cast<unsigned long long*>(ws + l.best) + static_cast<size_t>(ctx->best_parity) * ctx->k_max;
    unsigned long long* best_next =
        reinterpret_cast<unsigned long long*>(ws + l.best) + static_cast<size_t>(ctx->best_parity ^ 1) * ctx->k_max;
    uint64_t* sel_mask = reinterpret_cast<uint64_t*>(ws + l.sel_mask);
    uint32_t* tile_slot = reinterpret_cast<uint32_t*>(ws + l.tile_slot);
    const SegDesc* segs = reinterpret_cast<const SegDesc*>(ws + l.segs);
    const StDesc* sts = reinterpret_cast<const StDesc*>(ws + l.sts);
    const bool timed = timed_step(ctx);
    hipEvent_t* ev = timed ? &ctx->prof_events[static_cast<size_t>(ctx->prof_steps) * (SCALECOM_N_PHASES + 1)] : nullptr;
    auto mark = [&](int boundary) {   // boundaries 3 and 4 enclose the all-learner pass
        if (timed && (ctx->prof_all || boundary == 3 || boundary == 4)) (void)hipEventRecord(ev[boundary], s);
    };
    auto grid2 = [](int64_t blocks) {   // x up to 2^20 blocks, the rest over y
        const unsigned gx = static_cast<unsigned>(std::min<int64_t>(blocks, 1 << 20));
        return dim3(gx, static_cast<unsigned>((blocks + gx - 1) / gx));
    };
    mark(0);
    if (!ctx->best_clean) {             // first chunked step of this context, or one failed before: clear both copies
        const size_t words = 4 * static_cast<size_t>(ctx->k_max);   // 2 copies x 2 words per entry
        const int grid = static_cast<int>(std::min<size_t>((words + kBlock - 1) / kBlock, 4096));
        k_init<<<grid, kBlock, 0, s>>>(reinterpret_cast<uint32_t*>(ws + l.best), words);
    }
    ctx->best_clean = false;
    const int64_t n_tiles = static_cast<int64_t>(ctx->n_st) * kTilesPerSuper;
    k_chunk_select<G><<<grid2(n_tiles / kWaves), kBlock, 0, s>>>(lp.mem[leader], static_cast<const G*>(lp.grad[leader]), lr,
                                                                 segs, sts, ctx->n_st, best, sel_mask);
    mark(1);
    mark(2);
    k_chunk_marks<<<grid2((std::max(n_tiles, k_total) + kBlock - 1) / kBlock), kBlock, 0, s>>>(
        segs, n_tensors, sts, best, best_next, k_total, n_tiles, sel_mask, tile_slot, idx_out);
    mark(3);
    launch_update_reduce<G>(ctx, lp, n_learners, k_total, beta, lr, idx_out, red_out, mark);
    mark(5);
    if (timed) ++ctx->prof_steps;
    SC_HIP(ctx, hipGetLastError());
    ctx->best_parity ^= 1;
    ctx->best_clean = true;
    return SCALECOM_OK;
}

// Argument checks shared by the step and the diagnostics: the layout (segments and set sizes) ...
scalecom_status check_layout(scalecom_ctx* ctx, int n_tensors, const int64_t* offsets, const int64_t* ks, int64_t& k_total)
{
    if (!offsets || !ks) return fail(ctx, SCALECOM_EINVAL, "null argument");
    if (n_tensors < 1 || n_tensors > ctx->n_tensors_max) return fail(ctx, SCALECOM_EINVAL, "n_tensors out of range");
    if (offsets[0] < 0 || offsets[n_tensors] > ctx->numel_max) return fail(ctx, SCALECOM_EINVAL, "offsets out of range");
    k_total = 0;
    for (int s = 0; s < n_tensors; ++s) {
        const int64_t len = offsets[s + 1] - offsets[s];
        if (len < 0) return fail(ctx, SCALECOM_EINVAL, "offsets must be non-decreasing");
        if (ks[s] < 0 || ks[s] > len) return fail(ctx, SCALECOM_EINVAL, "k must satisfy 0 <= k <= segment length");
        k_total += ks[s];
    }
    if (k_total > ctx->k_max) return fail(ctx, SCALECOM_EINVAL, "k exceeds the context's k_max");
    return SCALECOM_OK;
}

// ... and the learners' buffers, gathered into the kernel argument.
scalecom_status check_learners(scalecom_ctx* ctx, float* const* mem, const void* const* grad, int n_learners,
                               LearnerPtrs& lp)
{
    if (!mem || !grad) return fail(ctx, SCALECOM_EINVAL, "null argument");
    if (n_learners < 1 || n_learners > ctx->n_learners_max) return fail(ctx, SCALECOM_EINVAL, "n_learners out of range");
    const uintptr_t galign = ctx->gdt == SCALECOM_GRAD_BF16 ? 8 : 16;
    for (int i = 0; i < n_learners; ++i) {
        if (!mem[i] || !grad[i]) return fail(ctx, SCALECOM_EINVAL, "null learner buffer");
        if (reinterpret_cast<uintptr_t>(mem[i]) % 16 || reinterpret_cast<uintptr_t>(grad[i]) % galign)
            return fail(ctx, SCALECOM_EINVAL, "learner buffer is not aligned");
        lp.mem[i] = mem[i];
        lp.grad[i] = grad[i];
    }
    for (int i = n_learners; i < SCALECOM_MAX_LEARNERS; ++i) {
        lp.mem[i] = nullptr;
        lp.grad[i] = nullptr;
    }
    return SCALECOM_OK;
}

scalecom_status step_common(scalecom_ctx* ctx, float* const* mem, const void* const* grad, int n_learners,
                            int n_tensors, const int64_t* offsets, const int64_t* ks, float beta, float lr,
                            int64_t step, int32_t* idx_out, float* red_out, const int64_t* chunks = nullptr)
{
    if (!ctx) return SCALECOM_EINVAL;
    ctx->last_error.clear();
    if (!mem || !grad || !offsets || !ks) return fail(ctx, SCALECOM_EINVAL, "null argument");
    if (n_learners < 1 || n_learners > ctx->n_learners_max) return fail(ctx, SCALECOM_EINVAL, "n_learners out of range");
    if (!(beta > 0.0f && beta <= 1.0f)) return fail(ctx, SCALECOM_EINVAL, "beta must satisfy 0 < beta <= 1");
    if (!std::isfinite(lr)) return fail(ctx, SCALECOM_EINVAL, "lr must be finite");
    if (step < 0) return fail(ctx, SCALECOM_EINVAL, "step must be >= 0");
    int64_t k_total = 0;
    scalecom_status st = check_layout(ctx, n_tensors, offsets, ks, k_total);
    if (st != SCALECOM_OK) return st;
    if (offsets[n_tensors] == offsets[0]) return SCALECOM_OK;   // nothing to do
    if (k_total > 0 && (!idx_out || !red_out)) return fail(ctx, SCALECOM_EINVAL, "null output");
    LearnerPtrs lp;
    st = check_learners(ctx, mem, grad, n_learners, lp);
    if (st != SCALECOM_OK) return st;

    DeviceGuard guard;
    SC_HIP(ctx, guard.enter(ctx->device));
    st = ensure_tables(ctx, n_tensors, offsets, ks, chunks);
    if (st != SCALECOM_OK) return st;
    const int leader = static_cast<int>(step % n_learners);    // Alg. 1 line 6: CLT-k of learner mod(t, n)
    if (chunks) {                                               // chunk-wise selector
        if (ctx->gdt == SCALECOM_GRAD_BF16)
            return launch_chunked<uint16_t>(ctx, lp, n_learners, n_tensors, k_total, beta, lr, leader, idx_out, red_out);
        return launch_chunked<float>(ctx, lp, n_learners, n_tensors, k_total, beta, lr, leader, idx_out, red_out);
    }
    if (ctx->gdt == SCALECOM_GRAD_BF16)
        return launch_step<uint16_t>(ctx, lp, n_learners, n_tensors, k_total, beta, lr, leader, idx_out, red_out);
    return launch_step<float>(ctx, lp, n_learners, n_tensors, k_total, beta, lr, leader, idx_out, red_out);
}

// Scratch of scalecom_hamming_distance: the summed vector, a copy of the leader's membership
// mask, and bucket predictions of its own (so the step's predictions stay untouched).
struct DiagLayout {
    size_t y, mask, preds, total;
};

DiagLayout diag_layout(int64_t numel_max, int n_tensors_max)
{
    DiagLayout d{};
    const size_t ntile = static_cast<size_t>(max_supertiles(numel_max, n_tensors_max)) * kTilesPerSuper;
    d.y = 0;
    d.mask = align_up(static_cast<size_t>(numel_max) * sizeof(float), 256);
    d.preds = d.mask + align_up(ntile * 4 * sizeof(uint64_t), 256);
    d.total = d.preds + align_up(static_cast<size_t>(n_tensors_max) * sizeof(uint32_t), 256);
    return d;
}

template <typename G>
scalecom_status launch_hamming(scalecom_ctx* ctx, const LearnerPtrs& lp, int n_learners, int n_tensors, int64_t begin,
                               int64_t end, float lr, int leader, char* scratch, int32_t* d_out)
{
    const WsLayout& l = ctx->lay;
    hipStream_t s = ctx->stream;
    const DiagLayout dl = diag_layout(ctx->numel_max, ctx->n_tensors_max);
    float* y = reinterpret_cast<float*>(scratch + dl.y);
    uint64_t* mask_a = reinterpret_cast<uint64_t*>(scratch + dl.mask);
    uint32_t* preds = reinterpret_cast<uint32_t*>(scratch + dl.preds);
    const SegDesc* segs = reinterpret_cast<const SegDesc*>(ctx->ws + l.segs);
    const StDesc* sts = reinterpret_cast<const StDesc*>(ctx->ws + l.sts);
    const uint64_t* sel_mask = reinterpret_cast<const uint64_t*>(ctx->ws + l.sel_mask);
    const size_t mask_bytes = static_cast<size_t>(ctx->n_st) * kTilesPerSuper * 4 * sizeof(uint64_t);
    auto no_mark = [](int) {};

    k_set_ks<<<(n_tensors + kBlock - 1) / kBlock, kBlock, 0, s>>>(segs, n_tensors, d_out);
    if (ctx->n_st > 0) {
        // the leader's index set (Eq. 3)
        k_init<<<1, kBlock, 0, s>>>(preds, static_cast<size_t>(n_tensors));
        launch_select<G>(ctx, lp.mem[leader], static_cast<const G*>(lp.grad[leader]), lr, n_tensors, preds, no_mark);
        SC_HIP(ctx, hipMemcpyAsync(mask_a, sel_mask, mask_bytes, hipMemcpyDeviceToDevice, s));
        // the top-k of the summed error-feedback gradients
        const int64_t blocks = (end - begin + kBlock - 1) / kBlock;
        const unsigned gx = static_cast<unsigned>(std::min<int64_t>(blocks, 1 << 20));
        k_sum_x<G><<<dim3(gx, static_cast<unsigned>((blocks + gx - 1) / gx)), kBlock, 0, s>>>(lp, n_learners, lr, begin, end, y);
        k_init<<<1, kBlock, 0, s>>>(preds, static_cast<size_t>(n_tensors));
        launch_select<NoGrad>(ctx, y, static_cast<const NoGrad*>(nullptr), 0.0f, n_tensors, preds, no_mark);
        k_mask_overlap<<<(ctx->n_st + kWaves - 1) / kWaves, kBlock, 0, s>>>(sts, ctx->n_st, mask_a, sel_mask, d_out);
    }
    SC_HIP(ctx, hipGetLastError());
    return SCALECOM_OK;
}

}  // namespace

extern "C" {

size_t scalecom_workspace_bytes(int64_t numel_max, int n_tensors_max, int n_learners_max, int64_t k_max)
{
    if (!sizes_ok(numel_max, n_tensors_max, n_learners_max, k_max)) return 0;
    return layout_for(numel_max, n_tensors_max, n_learners_max, k_max).total;
}

scalecom_status scalecom_init(scalecom_ctx** out, int device, void* hip_stream, void* workspace,
                              size_t workspace_bytes, int n_learners_max, int64_t numel_max, int64_t k_max,
                              int n_tensors_max, scalecom_grad_dtype grad_dtype)
{
    if (!out) return SCALECOM_EINVAL;
    *out = nullptr;
    if (device < 0 || !sizes_ok(numel_max, n_tensors_max, n_learners_max, k_max) ||
        (grad_dtype != SCALECOM_GRAD_F32 && grad_dtype != SCALECOM_GRAD_BF16))
        return SCALECOM_EINVAL;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256) return SCALECOM_EINVAL;
    const WsLayout lay = layout_for(numel_max, n_tensors_max, n_learners_max, k_max);
    if (workspace_bytes < lay.total) return SCALECOM_ENOMEM;

    scalecom_ctx* ctx = new (std::nothrow) scalecom_ctx;
    if (!ctx) return SCALECOM_ENOMEM;
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->ws = static_cast<char*>(workspace);
    ctx->n_learners_max = n_learners_max;
    ctx->numel_max = numel_max;
    ctx->k_max = k_max;
    ctx->n_tensors_max = n_tensors_max;
    ctx->gdt = grad_dtype;
    ctx->lay = lay;

    auto bail = [&](scalecom_status st) {
        scalecom_destroy(ctx);
        return st;
    };
    DeviceGuard guard;
    if (guard.enter(device) != hipSuccess) return bail(SCALECOM_EHIP);
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return bail(SCALECOM_EHIP);
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return bail(SCALECOM_EUNSUPPORTED);
    ctx->pinned_bytes = pinned_bytes_for(numel_max, n_tensors_max);
    if (hipHostMalloc(reinterpret_cast<void**>(&ctx->pinned), ctx->pinned_bytes, hipHostMallocDefault) != hipSuccess)
        return bail(SCALECOM_ENOMEM);
    if (hipEventCreateWithFlags(&ctx->upload_done, hipEventDisableTiming) != hipSuccess) return bail(SCALECOM_EHIP);
    *out = ctx;
    return SCALECOM_OK;
}

scalecom_status scalecom_step(scalecom_ctx* ctx, float* const* mem, const void* const* grad, int n_learners,
                              int64_t numel, int64_t k, float beta, float lr, int64_t step, int32_t* idx_out,
                              float* reduced_vals_out)
{
    if (!ctx) return SCALECOM_EINVAL;
    if (numel < 0 || numel > ctx->numel_max) return fail(ctx, SCALECOM_EINVAL, "numel out of range");
    const int64_t offsets[2] = {0, numel};
    return step_common(ctx, mem, grad, n_learners, 1, offsets, &k, beta, lr, step, idx_out, reduced_vals_out);
}

scalecom_status scalecom_step_chunked(scalecom_ctx* ctx, float* const* mem, const void* const* grad, int n_learners,
                                      int64_t numel, int64_t chunk, float beta, float lr, int64_t step,
                                      int32_t* idx_out, float* reduced_vals_out)
{
    if (!ctx) return SCALECOM_EINVAL;
    if (numel < 0 || numel > ctx->numel_max) return fail(ctx, SCALECOM_EINVAL, "numel out of range");
    if (chunk < 1) return fail(ctx, SCALECOM_EINVAL, "chunk must be >= 1");
    const int64_t offsets[2] = {0, numel};
    const int64_t k = (numel + chunk - 1) / chunk;               // one position per chunk
    return step_common(ctx, mem, grad, n_learners, 1, offsets, &k, beta, lr, step, idx_out, reduced_vals_out, &chunk);
}

scalecom_status scalecom_step_layers_chunked(scalecom_ctx* ctx, float* const* mem, const void* const* grad,
                                             int n_learners, int n_tensors, const int64_t* offsets,
                                             const int64_t* chunks, float beta, float lr, int64_t step,
                                             int32_t* idx_out, float* reduced_vals_out)
{
    if (!ctx) return SCALECOM_EINVAL;
    if (!offsets || !chunks) return fail(ctx, SCALECOM_EINVAL, "null argument");
    if (n_tensors < 1 || n_tensors > ctx->n_tensors_max) return fail(ctx, SCALECOM_EINVAL, "n_tensors out of range");
    std::vector<int64_t> ks(static_cast<size_t>(n_tensors));
    for (int s = 0; s < n_tensors; ++s) {
        if (chunks[s] < 1) return fail(ctx, SCALECOM_EINVAL, "chunk must be >= 1");
        const int64_t len = offsets[s + 1] - offsets[s];
        if (len < 0) return fail(ctx, SCALECOM_EINVAL, "offsets must be non-decreasing");
        ks[s] = (len + chunks[s] - 1) / chunks[s];               // one position per chunk
    }
    return step_common(ctx, mem, grad, n_learners, n_tensors, offsets, ks.data(), beta, lr, step, idx_out,
                       reduced_vals_out, chunks);
}

scalecom_status scalecom_step_layers(scalecom_ctx* ctx, float* const* mem, const void* const* grad, int n_learners,
                                     int n_tensors, const int64_t* offsets, const int64_t* ks, float beta, float lr,
                                     int64_t step, int32_t* idx_out, float* reduced_vals_out)
{
    return step_common(ctx, mem, grad, n_learners, n_tensors, offsets, ks, beta, lr, step, idx_out,
                       reduced_vals_out);
}

scalecom_status scalecom_apply_update(scalecom_ctx* ctx, float* theta, int64_t numel, const int32_t* idx,
                                      const float* vals, int64_t k, float scale)
{
    if (!ctx) return SCALECOM_EINVAL;
    ctx->last_error.clear();
    if (k < 0 || numel < 0 || !std::isfinite(scale)) return fail(ctx, SCALECOM_EINVAL, "bad size or scale");
    if (k == 0) return SCALECOM_OK;
    if (!theta || !idx || !vals) return fail(ctx, SCALECOM_EINVAL, "null argument");
    DeviceGuard guard;
    SC_HIP(ctx, guard.enter(ctx->device));
    const int64_t blocks = (k + kBlock - 1) / kBlock;
    const unsigned gx = static_cast<unsigned>(std::min<int64_t>(blocks, 1 << 20));
    const unsigned gy = static_cast<unsigned>((blocks + gx - 1) / gx);
    k_apply_update<<<dim3(gx, gy), kBlock, 0, ctx->stream>>>(theta, idx, vals, k, -scale);
    SC_HIP(ctx, hipGetLastError());
    return SCALECOM_OK;
}

size_t scalecom_hamming_scratch_bytes(int64_t numel_max, int n_tensors_max)
{
    if (numel_max < 0 || numel_max > INT32_MAX || n_tensors_max < 1) return 0;
    return diag_layout(numel_max, n_tensors_max).total;
}

scalecom_status scalecom_hamming_distance(scalecom_ctx* ctx, float* const* mem, const void* const* grad, int n_learners,
                                          int n_tensors, const int64_t* offsets, const int64_t* ks, float lr,
                                          int64_t step, void* scratch, size_t scratch_bytes, int32_t* d_out)
{
    if (!ctx) return SCALECOM_EINVAL;
    ctx->last_error.clear();
    if (!std::isfinite(lr)) return fail(ctx, SCALECOM_EINVAL, "lr must be finite");
    if (step < 0) return fail(ctx, SCALECOM_EINVAL, "step must be >= 0");
    int64_t k_total = 0;
    scalecom_status st = check_layout(ctx, n_tensors, offsets, ks, k_total);
    if (st != SCALECOM_OK) return st;
    LearnerPtrs lp;
    st = check_learners(ctx, mem, grad, n_learners, lp);
    if (st != SCALECOM_OK) return st;
    if (!d_out) return fail(ctx, SCALECOM_EINVAL, "null output");
    if (!scratch || reinterpret_cast<uintptr_t>(scratch) % 256) return fail(ctx, SCALECOM_EINVAL, "scratch must be 256-byte aligned");
    if (scratch_bytes < diag_layout(ctx->numel_max, ctx->n_tensors_max).total)
        return fail(ctx, SCALECOM_ENOMEM, "scratch smaller than scalecom_hamming_scratch_bytes");
    DeviceGuard guard;
    SC_HIP(ctx, guard.enter(ctx->device));
    st = ensure_tables(ctx, n_tensors, offsets, ks);
    if (st != SCALECOM_OK) return st;
    const int leader = static_cast<int>(step % n_learners);
    if (ctx->gdt == SCALECOM_GRAD_BF16)
        return launch_hamming<uint16_t>(ctx, lp, n_learners, n_tensors, offsets[0], offsets[n_tensors], lr, leader,
                                        static_cast<char*>(scratch), d_out);
    return launch_hamming<float>(ctx, lp, n_learners, n_tensors, offsets[0], offsets[n_tensors], lr, leader,
                                 static_cast<char*>(scratch), d_out);
}

scalecom_status scalecom_cosine_distance(scalecom_ctx* ctx, const float* a, const float* b, int64_t numel, double* out)
{
    if (!ctx) return SCALECOM_EINVAL;
    ctx->last_error.clear();
    if (!a || !b || !out) return fail(ctx, SCALECOM_EINVAL, "null argument");
    if (numel < 0) return fail(ctx, SCALECOM_EINVAL, "numel out of range");
    if (reinterpret_cast<uintptr_t>(out) % 8) return fail(ctx, SCALECOM_EINVAL, "out is not aligned");
    DeviceGuard guard;
    SC_HIP(ctx, guard.enter(ctx->device));
    k_init<<<1, kBlock, 0, ctx->stream>>>(reinterpret_cast<uint32_t*>(out), 8);
    if (numel > 0) {
        const int grid = static_cast<int>(std::min<int64_t>((numel + kBlock - 1) / kBlock, 2048));
        k_dots<<<grid, kBlock, 0, ctx->stream>>>(a, b, numel, out);
    }
    k_cosine_final<<<1, kLanes, 0, ctx->stream>>>(out);
    SC_HIP(ctx, hipGetLastError());
    return SCALECOM_OK;
}

scalecom_status scalecom_layer_ks(int n_tensors, const double* flops_per_gradient, const int64_t* sizes,
                                  const uint8_t* uncompressed, int64_t* ks_out, int64_t* rates_out)
{
    if (n_tensors < 0 || (n_tensors > 0 && (!flops_per_gradient || !sizes || !ks_out))) return SCALECOM_EINVAL;
    for (int s = 0; s < n_tensors; ++s)
        if (!(flops_per_gradient[s] > 0.0) || sizes[s] < 0) return SCALECOM_EINVAL;
    for (int s = 0; s < n_tensors; ++s) {
        // Sec. 4: 25X for a FLOPs/gradient ratio in [196, inf), 50X for [128, 196), 400X below 128;
        // a layer kept out of compression (App. E: the first convolution; every layer during the
        // warm-up epochs) sends all of its elements
        int64_t rate = flops_per_gradient[s] >= 196.0 ? 25 : (flops_per_gradient[s] >= 128.0 ? 50 : 400);
        if (uncompressed && uncompressed[s]) rate = 1;
        ks_out[s] = (sizes[s] + rate - 1) / rate;
        if (rates_out) rates_out[s] = rate;
    }
    return SCALECOM_OK;
}

scalecom_status scalecom_stream_copy(scalecom_ctx* ctx, void* dst, const void* src, size_t bytes)
{
    if (!ctx) return SCALECOM_EINVAL;
    if (!dst || !src || bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16)
        return fail(ctx, SCALECOM_EINVAL, "copy needs 16-byte aligned pointers and size");
    if (bytes == 0) return SCALECOM_OK;
    DeviceGuard guard;
    SC_HIP(ctx, guard.enter(ctx->device));
    const size_t n16 = bytes / 16;
    const size_t blocks = (n16 + kBlock - 1) / kBlock;
    const unsigned gx = static_cast<unsigned>(std::min<size_t>(blocks, 1u << 20));
    const unsigned gy = static_cast<unsigned>((blocks + gx - 1) / gx);
    if (gy > 65535) return fail(ctx, SCALECOM_EINVAL, "copy too large");
    k_copy<<<dim3(gx, gy), kBlock, 0, ctx->stream>>>(static_cast<const vf4_t*>(src), static_cast<vf4_t*>(dst), n16);
    SC_HIP(ctx, hipGetLastError());
    return SCALECOM_OK;
}

scalecom_status scalecom_timing_begin(scalecom_ctx* ctx, int max_steps, int all_phases, int every)
{
    if (!ctx) return SCALECOM_EINVAL;
    if (max_steps < 0 || max_steps > 4096) return fail(ctx, SCALECOM_EINVAL, "max_steps out of range");
    if (every < 1) return fail(ctx, SCALECOM_EINVAL, "every must be >= 1");
    DeviceGuard guard;
    SC_HIP(ctx, guard.enter(ctx->device));
    const size_t need = static_cast<size_t>(max_steps) * (SCALECOM_N_PHASES + 1);
    while (ctx->prof_events.size() < need) {
        hipEvent_t e;
        // timing only: no system-scope fence (cache write-back) when the event is reached
        SC_HIP(ctx, hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
        ctx->prof_events.push_back(e);
    }
    ctx->prof_cap = max_steps;
    ctx->prof_steps = 0;
    ctx->prof_every = every;
    ctx->prof_seen = 0;
    ctx->prof_all = all_phases != 0;
    return SCALECOM_OK;
}

scalecom_status scalecom_timing_read(scalecom_ctx* ctx, float* phase_ms, int capacity_steps, int* n_steps_out)
{
    if (!ctx) return SCALECOM_EINVAL;
    if (!n_steps_out || capacity_steps < 0 || (capacity_steps > 0 && !phase_ms))
        return fail(ctx, SCALECOM_EINVAL, "null argument");
    DeviceGuard guard;
    SC_HIP(ctx, guard.enter(ctx->device));
    SC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const int n = std::min(ctx->prof_steps, capacity_steps);
    for (int t = 0; t < n; ++t) {
        hipEvent_t* ev = &ctx->prof_events[static_cast<size_t>(t) * (SCALECOM_N_PHASES + 1)];
        for (int p = 0; p < SCALECOM_N_PHASES; ++p) {
            float* out = &phase_ms[t * SCALECOM_N_PHASES + p];
            *out = 0.0f;
            if (ctx->prof_all || p == 3) SC_HIP(ctx, hipEventElapsedTime(out, ev[p], ev[p + 1]));
        }
    }
    *n_steps_out = n;
    ctx->prof_cap = 0;   // recording stops until the next scalecom_timing_begin
    ctx->prof_steps = 0;
    return SCALECOM_OK;
}

const char* scalecom_strerror(scalecom_status status)
{
    switch (status) {
        case SCALECOM_OK: return "ok";
        case SCALECOM_EINVAL: return "invalid argument";
        case SCALECOM_ENOMEM: return "out of memory or workspace too small";
        case SCALECOM_EHIP: return "HIP runtime error";
        case SCALECOM_EUNSUPPORTED: return "unsupported device (gfx950 required)";
    }
    return "unknown status";
}

const char* scalecom_last_error(const scalecom_ctx* ctx) { return ctx ? ctx->last_error.c_str() : ""; }

void scalecom_destroy(scalecom_ctx* ctx)
{
    if (!ctx) return;
    if (ctx->pinned || ctx->upload_done || !ctx->prof_events.empty()) {
        DeviceGuard guard;
        if (guard.enter(ctx->device) == hipSuccess) {
            (void)hipStreamSynchronize(ctx->stream);
            if (ctx->upload_done) (void)hipEventDestroy(ctx->upload_done);
            for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
            if (ctx->pinned) (void)hipHostFree(ctx->pinned);
        }
    }
    delete ctx;
}

}  // extern "C"
