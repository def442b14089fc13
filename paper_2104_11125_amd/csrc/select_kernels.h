// Exact top-k selection on the leader's vector x_L = fma(lr, grad_L, mem_L) (Eq. 2, Alg. 1 line 6):
// radix select over the 31-bit magnitude key, 12 + 12 + 7 bits.  Kernels in the order a step runs
// them: k_predicted, k_level0, k_level<1>, k_level<2>, k_tilecount, (k_scan,) k_slots.
// Part of scalecom.hip's single translation unit.
#pragma once

#include <hip/hip_runtime.h>

#include "device_helpers.h"
#include "geometry.h"

namespace {

__global__ void __launch_bounds__(kBlock) k_init(uint32_t* zero_from, size_t n_words)
{
    for (size_t i = blockIdx.x * static_cast<size_t>(kBlock) + threadIdx.x; i < n_words;
         i += static_cast<size_t>(gridDim.x) * kBlock)
        zero_from[i] = 0u;
}

struct CollectStage {       // LDS staging of one supertile's masks and tile counts in the collecting passes
    uint64_t mask[kTilesPerSuper][4];
    uint32_t cnt[kTilesPerSuper];
};

// The magnitude keys of the 8 wave tiles a wave owns in one supertile (tile it * kWaves + wave,
// 4 keys per lane and tile; bit 4*it + c of okm says whether the element belongs to the segment).
// All loads are issued before the first value is used: lanes whose four elements lie inside the
// segment first (no branch between their loads), then the at most two lanes of the segment that
// straddle its ends, element by element.  For the passes where few blocks work (fallbacks, small
// segments) and nothing else hides a round trip to memory.
template <typename G>
__device__ __forceinline__ void supertile_keys(const float* __restrict__ mem, const G* __restrict__ grad, float lr,
                                               int64_t a0, int64_t begin, int64_t end, int wave, int lane,
                                               uint32_t (&key)[kTilesPerSuper / kWaves * kVec], uint32_t& okm)
{
    constexpr int kIters = kTilesPerSuper / kWaves;
    float4 m4[kIters], g4[kIters];
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int64_t p0 = a0 + (it * kWaves + wave) * kWaveTile + lane * kVec;
        m4[it] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        g4[it] = m4[it];
        if (p0 >= begin && p0 + 3 < end) {
            m4[it] = load4(mem + p0);
            g4[it] = load4(grad + p0);
        }
    }
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int64_t p0 = a0 + (it * kWaves + wave) * kWaveTile + lane * kVec;
        const bool straddles = !(p0 >= begin && p0 + 3 < end) && p0 + 3 >= begin && p0 < end;
        if (straddles) {
            m4[it] = load_guarded(mem, p0, begin, end, false);
            g4[it] = load_guarded(grad, p0, begin, end, false);
        }
    }
    okm = 0;
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int64_t p0 = a0 + (it * kWaves + wave) * kWaveTile + lane * kVec;
        uint32_t k4[4];
        bool ok[4];
        keys_from(m4[it], g4[it], lr, p0, begin, end, k4, ok);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            key[4 * it + c] = k4[c];
            okm |= (ok[c] ? 1u : 0u) << (4 * it + c);
        }
    }
}

// The per-tile work of the "collect" pass, given the tile's keys: keys from lo_key + span on are
// members for sure (their count and ballots are staged for the tile); the `span` keys from lo_key
// on are appended, with their positions, to the supertile's candidate slice `cand_dst` (in LDS or
// in memory; slots handed out through the block's LDS counter `fill`) and, if `lh1` is given (then
// the range is one twelve-bit bucket), counted per second digit there.  Called by all lanes of a
// wave; n_above and n_in are the same in every lane.
template <bool ALL_OK>
__device__ __forceinline__ void collect_tile(const uint32_t key[4], const bool ok[4], uint32_t p0, uint32_t lo_key,
                                             uint32_t span, int wt, int lane, uint32_t* fill, uint32_t* lh1,
                                             uint32_t& n_above, uint32_t& n_in, CollectStage& stg, uint2* cand_dst)
{
    const uint32_t above_key = lo_key + span;               // at most 2^31, which no key reaches
    n_above = 0;
    n_in = 0;
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
            if (lh1) atomicAdd(&lh1[(key[c] >> kBits2) & (kBins1 - 1)], 1u);   // counted whether or not it is listed
            ++rank;
        }
    }
}

// After the block's barrier: the staged masks and counts of the supertile, and its candidates if
// they were staged too, go out with full-width stores (lane-0 stores of 32 bytes per tile cost the
// collecting passes 8 % of their time).
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

// The 8 tiles a wave owns in a supertile of the predicted pass.  INSIDE: the whole supertile
// lies in the segment, so loads are unguarded and every position counts; otherwise both are
// checked per element.  Positions stay below 2^31 + 8192 and are kept in 32 bits.
template <typename G, bool INSIDE>
__device__ __forceinline__ uint32_t predicted_tiles(const float* __restrict__ mem, const G* __restrict__ grad, float lr,
                                                    const StDesc& d, uint32_t lo_key, uint32_t span, int wave, int lane,
                                                    uint32_t* fill, uint32_t& in_acc, CollectStage& stg, uint2* cand_stage)
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
    in_acc = 0;
#pragma unroll 1
    for (int it = 0; it < kIters; ++it) {
        const int wt = it * kWaves + wave;
        if (it + 1 < kIters) fetch(p_cur + kStride, m_nxt, g_nxt);
        const float4 x = accumulate4(m_cur, g_cur, lr);
        const uint32_t key[4] = {magnitude_key(x.x), magnitude_key(x.y), magnitude_key(x.z), magnitude_key(x.w)};
        bool ok[4] = {true, true, true, true};
        if (!INSIDE) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int64_t pos = static_cast<int64_t>(p_cur) + c;
                ok[c] = pos >= begin && pos < end;
            }
        }
        uint32_t n_above, n_in;
        collect_tile<INSIDE>(key, ok, p_cur, lo_key, span, wt, lane, fill, nullptr, n_above, n_in, stg, cand_stage);
        above_acc += n_above;
        in_acc += n_in;
        m_cur = m_nxt;
        g_cur = g_nxt;
        p_cur += kStride;
    }
    return above_acc;
}

// First look at the leader's vector (Eq. 2: finding the k-th largest magnitude), for segments
// that carry a prediction: the top 24 bits of the threshold expected (predicted_t24) and a width w.
// ONE pass, no histogram in LDS: keys above the 2^w keys centred on the expected threshold are
// members for sure (counted per tile, marked in the mask); keys among those 2^w go to the
// candidate list and are counted per 128 keys (the resolution of the search's second level) with
// atomics in memory.  If the counts show afterwards that the k-th largest key fell inside the
// range, the top 24 bits of the threshold are known exactly and no other full pass over the
// leader is needed.  The prediction only decides how much work is done, never what is selected.
// One block per supertile.
template <typename G>
__global__ void __launch_bounds__(kBlock)
k_predicted(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const SegDesc* __restrict__ segs,
            const StDesc* __restrict__ sts, uint2* __restrict__ cand,
            uint32_t* __restrict__ st_cand_cnt, const uint32_t* __restrict__ preds, uint32_t* __restrict__ wt_cnt,
            uint64_t* __restrict__ sel_mask, uint64_t* __restrict__ eq_mask, uint32_t* __restrict__ part,
            uint32_t* __restrict__ overflow, uint32_t* __restrict__ p_used, uint32_t* __restrict__ hist1_spec,
            const uint32_t* __restrict__ lead_mine)
{
    const int st = blockIdx.x;
    const StDesc d = sts[st];
    const uint32_t* pred = preds + static_cast<size_t>(d.seg) * kPredWords;
    const uint32_t have = pred[0];
    const uint32_t w = clamp_width(pred[2]);                // (whatever the memory holds, the counts stay in their words)
    const uint32_t t24 = predicted_t24(pred, lead_mine, d.seg);
    const SegDesc sd = segs[d.seg];
    if (have == 0 || sd.k == 0 || sd.st_count == 1) return;   // (one supertile: k_level0 searches it directly)
    // the range: 2^w keys centred on the middle of the expected threshold's 128 keys, aligned to 128,
    // cut off at key 0 and at 2^31
    const uint32_t span = 1u << w;
    const uint32_t sh = spec_bin_shift(w);                  // bins of 2^sh keys; the range starts at a multiple of that
    const uint32_t mid = (t24 << kBits2) | (kBins2 / 2);
    uint32_t base = mid > span / 2 ? (mid - span / 2) & ~((1u << sh) - 1u) : 0u;
    if (base > (1u << 31) - span) base = (1u << 31) - span;
    // the prediction this step works with, for the kernel that checks it (preds is rewritten there)
    if (st == sd.st_first && threadIdx.x == 0) {
        uint32_t* used = p_used + static_cast<size_t>(d.seg) * kPredWords;
        used[0] = 1u;
        used[1] = base;
        used[2] = w;
        used[3] = pred[3];                                  // steps in a row with the threshold in the range's middle half
    }
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes), lane = threadIdx.x % kLanes;
    __shared__ uint32_t fill;
    __shared__ uint32_t acc[2];                             // keys above the range, keys inside it
    __shared__ CollectStage stg;
    __shared__ uint2 cand_stage[kCandSlice];
    __shared__ uint32_t wide_cnt[1 << kSpecWideBinsLog];    // the block's counts of a wide range's bins
    const bool wide = w > kSpecBitsMax;                     // block-uniform
    if (threadIdx.x == 0) fill = 0u;
    if (threadIdx.x < 2) acc[threadIdx.x] = 0u;
    if (wide && threadIdx.x < (1 << kSpecWideBinsLog)) wide_cnt[threadIdx.x] = 0u;
    __syncthreads();

    uint2* slice = cand + static_cast<size_t>(st) * kCandSlice;
    // the range's 2^(w-sh) counts exist in as many copies as 4096 words hold, one copy per residue of the
    // supertile number: with few bins all the atomics of a step would otherwise hit a few cache lines
    const uint32_t copy = static_cast<uint32_t>(st) & ((1u << (kBits1 - (w - sh))) - 1u);
    uint32_t* h1 = hist1_spec + static_cast<size_t>(d.seg) * kBins1 + (copy << (w - sh));
    uint32_t above_acc, in_acc;
    if (d.a0 >= d.begin && static_cast<int64_t>(d.a0) + kSuper <= d.end)   // block-uniform
        above_acc = predicted_tiles<G, true>(mem, grad, lr, d, base, span, wave, lane, &fill, in_acc, stg, cand_stage);
    else
        above_acc = predicted_tiles<G, false>(mem, grad, lr, d, base, span, wave, lane, &fill, in_acc, stg, cand_stage);
    if (lane == 0 && above_acc) atomicAdd(&acc[0], above_acc);
    if (lane == 0 && in_acc) atomicAdd(&acc[1], in_acc);
    __syncthreads();
    collect_flush(stg, nullptr, static_cast<size_t>(st) * kTilesPerSuper, fill, wt_cnt, sel_mask, eq_mask, slice);
    // The staged candidates go to the supertile's slice and are counted per bin on the way,
    // outside the streaming loop.  (If the slice overflowed the counts are incomplete, and nothing
    // reads them.)
    static_assert(kCandSlice == 2 * kBlock, "two staged candidates per thread");
    const uint32_t n = fill < kCandSlice ? fill : kCandSlice;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t e = j * kBlock + threadIdx.x;
        if (e < n) {
            const uint2 ce = cand_stage[e];
            slice[e] = ce;
            if (wide)
                atomicAdd(&wide_cnt[(ce.x - base) >> sh], 1u);
            else
                atomicAdd(&h1[(ce.x - base) >> sh], 1u);
        }
    }
    if (wide) {                                             // block-uniform
        __syncthreads();
        if (threadIdx.x < (1 << kSpecWideBinsLog)) {
            const uint32_t v = wide_cnt[threadIdx.x];
            if (v) atomicAdd(&h1[threadIdx.x], v);
        }
    }
    if (threadIdx.x == 0) {
        st_cand_cnt[st] = n;
        if (fill > kCandSlice) overflow[d.seg] = 1u;        // every overflowing block stores the same value
    }
    if (threadIdx.x < 2) {
        const uint32_t v = acc[threadIdx.x];
        if (v)
            atomicAdd(&part[(static_cast<size_t>(d.seg) * kPartSlots + st % kPartSlots) * kPartWords + threadIdx.x], v);
    }
}

// One digit of the radix search, by all threads of a block: the bin of h[0 .. NB) that holds the
// k_rem-th largest key counted there, from the top.  The one thread that owns that bin returns true
// with the bin, its count and the number of keys above it; `above` is kWaves words of LDS.
template <int NB>
__device__ __forceinline__ bool search_digit(const uint32_t* __restrict__ h, uint32_t k_rem, uint32_t* above,
                                             uint32_t& digit, uint32_t& n_digit, uint32_t& n_above)
{
    constexpr int CH = NB >= kBlock ? NB / kBlock : 1;     // bins per thread
    constexpr int ACTIVE = NB >= kBlock ? kBlock : NB;     // threads that own bins
    const int t = threadIdx.x, lane = t % kLanes, wave = t / kLanes;
    uint32_t mine = 0;
    if (t < ACTIVE) {
#pragma unroll
        for (int b = 0; b < CH; ++b) mine += h[t * CH + b];
    }
    // inclusive suffix sums over threads: within a wave by shuffles, across the 4 waves through LDS
    uint32_t suf = mine;
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) {
        const uint32_t v = __shfl_down(suf, off, kLanes);
        if (lane + off < kLanes) suf += v;
    }
    if (lane == 0) above[wave] = suf;                       // the wave's total
    __syncthreads();
    for (int w = wave + 1; w < kWaves; ++w) suf += above[w];
    const uint32_t incl = suf;               // keys in my bins and all higher ones
    const uint32_t excl = incl - mine;       // keys strictly above my bins
    bool found = false;
    if (t < ACTIVE && excl < k_rem && k_rem <= incl) {      // one thread: its bins are read again, not kept
        uint32_t c = excl;
        for (int b = CH - 1; b >= 0 && !found; --b) {
            const uint32_t n = h[t * CH + b];
            if (c + n >= k_rem) {
                digit = static_cast<uint32_t>(t * CH + b);
                n_digit = n;
                n_above = c;
                found = true;
            }
            c += n;
        }
    }
    return found;
}

// How many of the block's keys are >= cand: each thread brings NK keys (bit j of `valid` says
// whether v[j] counts); `partial` is kWaves words of LDS that nobody else touches until the next
// barrier.  All threads call it; the result is the same in every thread.
template <int NK>
__device__ __forceinline__ uint32_t block_count_at_least(const uint32_t (&v)[NK], uint32_t valid, uint32_t cand,
                                                         uint32_t* partial, int lane, int wave)
{
    uint32_t c = 0;
#pragma unroll
    for (int j = 0; j < NK; ++j) c += (((valid >> j) & 1u) && v[j] >= cand) ? 1u : 0u;
    c = wave_sum(c);
    if (lane == 0) partial[wave] = c;
    __syncthreads();
    uint32_t total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) total += partial[w];
    return total;
}

// The k-th largest of the block's keys (1 <= k <= number of valid keys), bit by bit from the top:
// T keeps a bit if at least k keys are >= T with that bit set.  One barrier per bit, the waves'
// partial counts in alternating halves of `partial` (2 * kWaves words of LDS).  q = how many keys
// equal to T belong to the k largest.  No histogram: its atomics would all hit the few top digits
// that gradient-like keys share.
template <int NK>
__device__ __forceinline__ uint32_t block_kth_largest(const uint32_t (&v)[NK], uint32_t valid, uint32_t k,
                                                      uint32_t* partial, int lane, int wave, uint32_t& q)
{
    uint32_t T = 0;
    for (int bit = 30; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        if (block_count_at_least<NK>(v, valid, cand, partial + (bit & 1) * kWaves, lane, wave) >= k) T = cand;
    }
    q = T == 0x7fffffffu ? k : k - block_count_at_least<NK>(v, valid, T + 1u, partial + kWaves, lane, wave);
    return T;
}

// The same search by ONE wave over keys that its lanes hold (a few hundred keys): no LDS and no
// barrier per bit, only a reduction over the lanes.  All 64 lanes of the wave call it.
template <int NK>
__device__ __forceinline__ uint32_t wave_kth_largest(const uint32_t (&v)[NK], uint32_t valid, uint32_t k, uint32_t& q)
{
    auto count_at_least = [&](uint32_t cand) {
        uint32_t c = 0;
#pragma unroll
        for (int j = 0; j < NK; ++j) c += (((valid >> j) & 1u) && v[j] >= cand) ? 1u : 0u;
        return wave_sum(c);
    };
    uint32_t T = 0;
    for (int bit = 30; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        if (count_at_least(cand) >= k) T = cand;
    }
    q = T == 0x7fffffffu ? k : k - count_at_least(T + 1u);
    return T;
}

// The width of the next step's range of finely counted keys, after a step whose range (2^w keys,
// holding in_range keys in all) held the threshold in its bin `bin`; `slots` is what the segment's
// candidate list can take, `calm` the number of steps in a row in which the threshold fell into the
// range's middle half (updated).  Wider at once if the threshold fell outside the middle half, or
// if the range held few keys -- unless twice as many keys would crowd the candidate list.
// Narrower only after kCalmSteps calm steps, if the range holds many more keys than needed (the
// index set's size, and enough for the spread of an order statistic of that rank), and at once if
// it holds more than three quarters of what the candidate list can take.
__device__ __forceinline__ uint32_t next_width(uint32_t w, uint32_t bin, uint32_t in_range, uint32_t k, uint64_t slots,
                                               uint32_t& calm)
{
    const uint32_t n_bins = 1u << (w - spec_bin_shift(w));
    uint64_t want = k > 64u ? k : 64u;
    if (static_cast<uint64_t>(k) < 256u * 256u) {           // 16 * sqrt(k) > k
        uint32_t r = 1;
        while (r * r < k) ++r;
        if (16u * r > want) want = 16u * r;
    }
    if (want > slots / 4) want = slots / 4;
    const bool middle = bin >= n_bins / 4 && bin < n_bins - n_bins / 4;
    const bool room = 8ull * in_range <= 3 * slots;         // twice as many still below 3/4 of the slots
    calm = middle ? calm + 1u : 0u;
    uint32_t w_next = w;
    if (4ull * in_range > 3 * slots && w > kSpecBitsMin) {
        w_next = w - 1;
        calm = 0u;
    } else if ((!middle || 5ull * in_range < 3 * want) && room && w < kSpecBitsWide) {
        w_next = w + 1;
        calm = 0u;
    } else if (calm >= kCalmSteps && 2ull * in_range > 3 * want && w > kSpecBitsMin) {
        w_next = w - 1;
        calm = 0u;
    }
    return w_next;
}

// The selection state of a segment exists in three copies, one per level of the search: each
// level's kernel reads the copy the previous one left and the segment's first block writes the
// next, so no block reads what another block of the same launch wrote.
struct StateCopies {
    SegState* level0;
    SegState* level1;
    SegState* level2;           // what the tile counts and the slot pass read
};

// A segment of one supertile (up to 8192 elements; with hundreds of tensors, half of them) is
// finished by its one block: the threshold is found on the keys the block holds in registers, and
// the tile counts and masks are written.  No range from the predicted pass: the k-th largest of so
// few values moves by several per cent from step to step, more than a range that the candidate list
// can hold covers; what is kept from the previous step is where to look first.  `s` arrives with
// k_rem = k and nothing found; lh (kBins0 words), tot_s (kPartWords), res (2), above (kWaves) are
// LDS of the calling kernel.  All threads of the block call it.
template <typename G>
__device__ __forceinline__ void select_one_supertile(const float* __restrict__ mem, const G* __restrict__ grad, float lr,
                                                     const HistBlock& hb, uint32_t k, SegState s,
                                                     const StateCopies& states, uint32_t* __restrict__ pred,
                                                     uint32_t* __restrict__ lead_mine,
                                                     uint32_t* __restrict__ wt_cnt, uint64_t* __restrict__ sel_mask,
                                                     uint64_t* __restrict__ eq_mask, uint2* __restrict__ st_sum,
                                                     uint32_t* lh, uint32_t* tot_s, uint32_t* res, uint32_t* above)
{
    const int t = threadIdx.x, wave = t / kLanes, lane = t % kLanes;
    const int cur = hb.seg;
    constexpr int kIters = kTilesPerSuper / kWaves;
    constexpr int kMine = kIters * kVec;                // 32 keys per thread
    constexpr uint32_t kListMax = 8 * kBlock;           // keys near the threshold, 8 per thread
    static_assert(kListMax <= kBins0, "the list lives in the histogram's words");
    uint32_t key[kMine];
    uint32_t okm;                                       // bit 4*it + c: the element belongs to the segment
    supertile_keys(mem, grad, lr, static_cast<int64_t>(hb.a0), static_cast<int64_t>(hb.begin),
                   static_cast<int64_t>(hb.end), wave, lane, key, okm);
    // The search runs over the few keys near the previous step's threshold if the k largest are
    // among them (one count tells), over all keys otherwise.
    uint32_t* partial = tot_s;                          // 2 x kWaves words
    static_assert(kPartWords >= 2 * kWaves, "room for the partial counts");
    const uint32_t t_prev = predicted_t24(pred, lead_mine, cur) << kBits2;   // 0 before the first step
    const uint32_t n_seg = static_cast<uint32_t>(hb.end - hb.begin);
    uint32_t lo = t_prev > (1u << (kBits1 + kBits2)) ? t_prev - (1u << (kBits1 + kBits2)) : 0u;
    uint32_t n_near = n_seg;
    if (lo != 0u) {                                     // block-uniform
        // (counted in the second half of `partial`: the search starts in the first)
        n_near = block_count_at_least<kMine>(key, okm, lo, partial + kWaves, lane, wave);
        if (n_near < k) {                               // the threshold fell by more than that: every key is a candidate
            lo = 0u;
            n_near = n_seg;
            __syncthreads();                            // (the partial counts have been read)
        }
    }
    uint32_t T, q;
    if (n_near <= kListMax) {                           // block-uniform (n_near >= k holds)
        // my keys >= lo go to consecutive words of the list: exclusive prefix of the threads' counts
        uint32_t near = 0;
#pragma unroll
        for (int j = 0; j < kMine; ++j) near |= (((okm >> j) & 1u) && key[j] >= lo ? 1u : 0u) << j;
        uint32_t incl = __popc(near);
#pragma unroll
        for (int off = 1; off < kLanes; off <<= 1) {
            const uint32_t a = __shfl_up(incl, off, kLanes);
            if (lane >= off) incl += a;
        }
        if (lane == kLanes - 1) above[wave] = incl;     // the wave's total
        __syncthreads();
        uint32_t slot = incl - __popc(near);
        for (int w2 = 0; w2 < wave; ++w2) slot += above[w2];
#pragma unroll
        for (int j = 0; j < kMine; ++j)
            if ((near >> j) & 1u) lh[slot++] = key[j];
        __syncthreads();
        // the first wave searches the list by itself (8 keys per lane if they are few, else 32)
        if (wave == 0) {
            if (n_near <= 8u * kLanes) {
                uint32_t mine[8];
                uint32_t have_mask = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t e = j * kLanes + lane;
                    mine[j] = e < n_near ? lh[e] : 0u;
                    have_mask |= (e < n_near ? 1u : 0u) << j;
                }
                T = wave_kth_largest<8>(mine, have_mask, k, q);
            } else {
                uint32_t mine[kListMax / kLanes];
                uint32_t have_mask = 0;
#pragma unroll
                for (int j = 0; j < static_cast<int>(kListMax / kLanes); ++j) {
                    const uint32_t e = j * kLanes + lane;
                    mine[j] = e < n_near ? lh[e] : 0u;
                    have_mask |= (e < n_near ? 1u : 0u) << j;
                }
                T = wave_kth_largest<kListMax / kLanes>(mine, have_mask, k, q);
            }
            if (lane == 0) {
                res[0] = T;
                res[1] = q;
            }
        }
        __syncthreads();
        T = res[0];
        q = res[1];
    } else {
        T = block_kth_largest<kMine>(key, okm, k, partial, lane, wave, q);
    }
    // the tile counts and masks of the supertile, from the keys at hand (what k_tilecount does otherwise)
    const size_t tile0 = static_cast<size_t>(hb.st_lo) * kTilesPerSuper;
    __syncthreads();                                    // (the last partial counts have been read)
    uint32_t* cnt = lh;                                 // the histogram's words: unused on this path
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int wt = it * kWaves + wave;
        uint64_t gt[4], eq[4];
        uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool ok = (okm >> (4 * it + c)) & 1u;
            gt[c] = __ballot(ok && key[4 * it + c] > T);
            eq[c] = __ballot(ok && key[4 * it + c] == T);
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
    if (t < kLanes) {
        const uint32_t v = t < kTilesPerSuper ? cnt[t] : 0u;
        if (t < kTilesPerSuper) wt_cnt[tile0 + t] = v;
        const uint32_t s2 = wave_sum(v);               // at most 8192 each: no carry between halves
        if (t == 0) st_sum[hb.st_lo] = make_uint2(s2 & 0xffffu, s2 >> 16);
    }
    if (t == 0) {
        s.prefix = T;
        s.k_rem = q;
        s.T = T;
        s.q = q;
        s.l1_done = 1;
        s.l2_done = 1;
        state_at(states.level0, cur) = s;               // final: every level's copy (the level kernels pass it by)
        state_at(states.level1, cur) = s;
        state_at(states.level2, cur) = s;
        pred[0] = 0u;                                   // no range for the predicted pass ...
        record_t24(pred, lead_mine, cur, T >> kBits2);  // ... but where to look first in the next steps
    }
}

// Level 0 of the search, for every segment: did the predicted pass see the k-th largest key inside
// its range?  Then the top 24 bits of the threshold follow from a search of that pass's counts, and
// the width of the next step's range is chosen from how many keys this one held and where the
// threshold fell in it.  Otherwise (no prediction, or a miss) the blocks that hold the segment's
// supertiles count the top 12 key bits of the leader's vector, and the search of that histogram is
// left to the blocks of the next kernel (state.pending).  One block per entry of the block table
// (supertiles of one segment); the segment's first block writes the state either way, and no
// block reads what another block of the same kernel wrote.
template <typename G>
__global__ void __launch_bounds__(kBlock)
k_level0(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const SegDesc* __restrict__ segs,
         const HistBlock* __restrict__ hblocks, StateCopies states, bool small_elsewhere, uint32_t* __restrict__ hist,
         uint32_t* __restrict__ preds, const uint32_t* __restrict__ p_used, const uint32_t* __restrict__ part,
         const uint32_t* __restrict__ overflow, const uint32_t* __restrict__ hist1_spec, uint32_t* __restrict__ lead_mine,
         uint32_t* __restrict__ wt_cnt, uint64_t* __restrict__ sel_mask, uint64_t* __restrict__ eq_mask,
         uint2* __restrict__ st_sum, unsigned long long* __restrict__ stats)
{
    __shared__ uint32_t lh[kBins0];
    __shared__ uint32_t tot_s[kPartWords];
    __shared__ uint32_t res[3];                             // outcome flag, digit(s), members left
    __shared__ uint32_t above[kWaves];
    __shared__ uint32_t flag;
    static_assert(kPartSlots * kPartWords == 2 * kBlock, "two counter words per thread");

    const int t = threadIdx.x, wave = t / kLanes, lane = t % kLanes;
    const HistBlock hb = hblocks[blockIdx.x];
    const int cur = hb.seg;
    const bool owner = hb.owner != 0;                       // this block writes the segment's state
    if (stats && blockIdx.x == 0 && t == 0) atomicAdd(&stats[kStatSteps], 1ull);
    // everything the segment number addresses is requested at once
    const uint32_t* my_part = part + static_cast<size_t>(cur) * kPartSlots * kPartWords;
    const SegDesc sd = segs[cur];
    const uint32_t* used = p_used + static_cast<size_t>(cur) * kPredWords;
    const uint32_t have = used[0], base = used[1], w = clamp_width(used[2]);
    const uint32_t ov = overflow[cur];
    const uint32_t w0 = my_part[t], w1 = my_part[kBlock + t];
    const uint32_t k = static_cast<uint32_t>(sd.k);
    uint32_t* pred = preds + static_cast<size_t>(cur) * kPredWords;
    SegState s{};                                           // every field is written each step
    s.k_rem = k;
    s.T = 0xffffffffu;                                      // above every key: nothing is a member
    s.mode = kModeFull;
    s.l1_bits = kBits1;
    SegState* state = states.level0;
    if (k == 0) {                                           // block-uniform: an empty index set
        if (owner && t == 0) {
            s.done = 1;
            state_at(state, cur) = s;
        }
        return;
    }
    if (sd.st_count == 1) {                                 // block-uniform
        // (a context for several tensors has k_small do this beside the leader pass)
        if (!small_elsewhere)
            select_one_supertile(mem, grad, lr, hb, k, s, states, pred, lead_mine, wt_cnt, sel_mask, eq_mask, st_sum, lh,
                                 tot_s, res, above);
        return;
    }
    if (t == 0) flag = 0u;
    bool hit = false;
    if (have != 0) {                                        // block-uniform: sum the slotted copies of the counters
        if (t < kPartWords) tot_s[t] = 0u;
        __syncthreads();
        if (w0) atomicAdd(&tot_s[t % kPartWords], w0);
        if (w1) atomicAdd(&tot_s[(kBlock + t) % kPartWords], w1);
        __syncthreads();
        // exact: the range holds the k-th largest key iff fewer than k keys lie above it and at least k
        // above or inside it (and every key inside it was listed)
        hit = ov == 0 && tot_s[0] < k && k - tot_s[0] <= tot_s[1];
    }
    if (hit) {                                              // block-uniform: the prediction held
        if (!owner) return;
        const uint32_t above_range = tot_s[0], in_range = tot_s[1];
        // add up the copies of the range's counts (word = copy * n_bins + bin) in LDS, then search there
        const uint32_t sh = spec_bin_shift(w);
        const uint32_t n_bins = 1u << (w - sh);
        const uint32_t* h1 = hist1_spec + static_cast<size_t>(cur) * kBins1;
        constexpr int kPer = kBins1 / kBlock;
        uint32_t mine[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) mine[j] = h1[j * kBlock + t];
        for (int b = t; b < kBins1; b += kBlock) lh[b] = 0u;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kPer; ++j)
            if (mine[j]) atomicAdd(&lh[(j * kBlock + t) & (n_bins - 1u)], mine[j]);
        __syncthreads();
        uint32_t bin, n_bin, n_above;
        if (search_digit<kBins1>(lh, k - above_range, above, bin, n_bin, n_above)) {
            res[1] = (base >> sh) + bin;                    // the key's top 31 - sh bits (24 up to w = 19)
            res[2] = k - above_range - n_above;
            res[0] = bin;
            flag = 1u;
        }
        __syncthreads();
        if (t == 0) {
            if (flag) {
                s.prefix = res[1];
                s.k_rem = res[2];
                s.mode = kModeCand;
                s.collected = 1;
                // a wide range's bins leave sh - 7 bits to level 1, which counts them on the listed keys
                s.l1_done = sh == kBits2 ? 1u : 0u;
                s.l1_bits = sh - kBits2;
                if (stats && sh != kBits2) atomicAdd(&stats[kStatWideRange], 1ull);
                uint32_t calm = used[3];
                const uint32_t w_next =
                    next_width(w, res[0], in_range, k, static_cast<uint64_t>(sd.st_count) * kCandSlice, calm);
                pred[3] = calm;
                pred[0] = 1u;
                // (of a wide range's bin its middle, until level 1 has resolved it)
                record_t24(pred, lead_mine, cur, sh == kBits2 ? res[1] : ((res[1] << sh) | (1u << (sh - 1))) >> kBits2);
                pred[2] = w_next;
            } else {                                        // only if the counts were corrupted: nothing is selected
                s.done = 1;
                pred[0] = 0u;
            }
            state_at(state, cur) = s;
        }
        return;
    }

    s.w_next = kSpecBitsMax;                                // (the search of this histogram chooses it)
    // no prediction, or one that failed: count the top digits of my part of the segment
    for (int b = t; b < kBins0; b += kBlock) lh[b] = 0u;
    __syncthreads();
    const int64_t begin = hb.begin, end = hb.end;
    for (int s2 = hb.st_lo; s2 < hb.st_hi; ++s2) {
        const int64_t a0 = static_cast<int64_t>(hb.a0) + static_cast<int64_t>(s2 - hb.st_lo) * kSuper;
        uint32_t key[kTilesPerSuper / kWaves * kVec];
        uint32_t okm;
        supertile_keys(mem, grad, lr, a0, begin, end, wave, lane, key, okm);
#pragma unroll
        for (int j = 0; j < kTilesPerSuper / kWaves * kVec; ++j)
            if ((okm >> j) & 1u) atomicAdd(&lh[key[j] >> (kBits1 + kBits2)], 1u);
    }
    __syncthreads();
    uint32_t* h = hist + static_cast<size_t>(cur) * kBins0;
    for (int b = t; b < kBins0; b += kBlock) {
        const uint32_t v = lh[b];
        if (v) atomicAdd(&h[b], v);
    }
    if (owner && t == 0) {
        s.pending = 1;                                      // the next kernel's blocks search the histogram
        state_at(state, cur) = s;
        pred[0] = 0u;                                       // until the levels that follow have found the threshold
        if (stats) atomicAdd(&stats[have != 0 ? kStatMissed : kStatNoPrediction], 1ull);
    }
}

// The segments of one supertile with a non-empty index set, one block each (host-built table):
// select_one_supertile as a kernel of its own, which the host runs beside the leader pass.
template <typename G>
__global__ void __launch_bounds__(kBlock)
k_small(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const SegDesc* __restrict__ segs,
        const HistBlock* __restrict__ small, StateCopies states, uint32_t* __restrict__ preds,
        uint32_t* __restrict__ lead_mine, uint32_t* __restrict__ wt_cnt, uint64_t* __restrict__ sel_mask,
        uint64_t* __restrict__ eq_mask, uint2* __restrict__ st_sum)
{
    __shared__ uint32_t lh[kBins0];
    __shared__ uint32_t tot_s[kPartWords];
    __shared__ uint32_t res[3];
    __shared__ uint32_t above[kWaves];
    const HistBlock hb = small[blockIdx.x];
    SegState s{};
    s.k_rem = static_cast<uint32_t>(segs[hb.seg].k);
    s.T = 0xffffffffu;
    s.mode = kModeFull;
    s.l1_bits = kBits1;
    select_one_supertile(mem, grad, lr, hb, s.k_rem, s, states, preds + static_cast<size_t>(hb.seg) * kPredWords, lead_mine,
                         wt_cnt, sel_mask, eq_mask, st_sum, lh, tot_s, res, above);
}

// What the level-1 pass writes when it also has to collect (see k_level).
struct CollectOut {
    uint32_t* wt_cnt;
    uint64_t* sel_mask;
    uint64_t* eq_mask;
    uint2* cand;
    uint32_t* st_cand_cnt;
    uint32_t* full_flag;     // per segment: a slice overflowed, the kernels that follow work in full mode
};

// Levels 1 and 2 of the search, one block per entry of the block table: first the search of the
// previous level's histogram if it is still pending (every block of the segment does it for
// itself: the histogram is complete since the previous kernel ended, and re-reading its 16 KB
// costs less than a launch), then the histogram of the next digit of the leader's magnitude keys.
// LEVEL 1: bits 18..7 of keys whose top 12 bits equal the chosen bucket -- or, after a hit of a
// range wider than 2^19 keys, the l1_bits bits that its 64 bins left open, counted on the listed
// keys; a segment whose top 24 bits k_level0 found already (the steady state) is skipped.
// LEVEL 2: last 7 bits of keys matching 24 bits; the search follows in k_tilecount.  Candidate mode reads the keys
// from the candidate list, full mode recomputes them from the leader's vector.  The state comes
// from state_in and goes, through the segment's first block, to state_out: no block reads what
// another block of the same kernel wrote.
// LEVEL 1 is also the second full pass over the leader's vector for segments in candidate mode
// whose list the predicted pass did not fill (no prediction, or one that missed): per wave tile,
// keys above the level-0 bucket are members for sure, keys inside the bucket go to the
// supertile's slice of the candidate list and are counted here directly.  A slice that overflows
// (bucket keys clustered in one place) sends the whole segment back to full-pass mode for the
// kernels that follow; this kernel's counts are complete either way.
template <typename G, int LEVEL>
__global__ void __launch_bounds__(kBlock)
k_level(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const SegDesc* __restrict__ segs,
        const HistBlock* __restrict__ hblocks, const SegState* __restrict__ state_in, SegState* __restrict__ state_out,
        const uint32_t* __restrict__ hist_prev, uint32_t* __restrict__ hist, uint32_t* __restrict__ preds,
        uint32_t* __restrict__ lead_mine, CollectOut out, unsigned long long* __restrict__ stats)
// in candidate mode out.cand and out.st_cand_cnt are read, when collecting they are written
{
    static_assert(LEVEL == 1 || LEVEL == 2, "level 0 is k_level0");
    constexpr int NB = LEVEL == 1 ? kBins1 : kBins2;
    constexpr int NB_PREV = LEVEL == 1 ? kBins0 : kBins1;
    constexpr int BITS_PREV = LEVEL == 1 ? kBits0 : kBits1;
    __shared__ uint32_t lh[NB];
    __shared__ uint32_t res[4];                             // found, digit, keys above it, its count
    __shared__ uint32_t above[kWaves];

    const int t = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(t / kLanes), lane = t % kLanes;
    const HistBlock hb = hblocks[blockIdx.x];
    const int cur = hb.seg;
    const bool owner = hb.owner != 0;                       // this block passes the segment's state on
    SegState ss = state_at(state_in, cur);
    const int st_count = segs[cur].st_count;
    const uint32_t went_full = LEVEL == 2 ? out.full_flag[cur] : 0u;
    if (went_full) ss.mode = kModeFull;

    // 12, or what a wide range's counts left open (never more than 12: the counters are kBins1 words)
    const uint32_t l1_bits = ss.l1_bits < static_cast<uint32_t>(kBits1) ? ss.l1_bits : static_cast<uint32_t>(kBits1);
    auto count = [&](uint32_t key, uint32_t prefix) {
        if (LEVEL == 1) {
            if ((key >> (l1_bits + kBits2)) == prefix) atomicAdd(&lh[(key >> kBits2) & ((1u << l1_bits) - 1u)], 1u);
        } else {
            if ((key >> kBits2) == prefix) atomicAdd(&lh[key & (kBins2 - 1)], 1u);
        }
    };

    if (ss.done == 0 && ss.pending != 0) {                  // block-uniform: the previous level's search
        if (t == 0) res[0] = 0u;
        uint32_t digit, n_digit, n_above;                   // (search_digit's barrier orders the store above)
        const uint32_t* hp = hist_prev + static_cast<size_t>(cur) * NB_PREV;
        if constexpr (LEVEL == 2) {
            // level 1's counts exist in 2^(12 - l1_bits) slotted copies (word = copy << l1_bits | bin): added up
            // in LDS, then searched there
            __shared__ uint32_t sum1[kBins1];
            for (int b = t; b < kBins1; b += kBlock) sum1[b] = 0u;
            uint32_t mine[kBins1 / kBlock];
#pragma unroll
            for (int j = 0; j < kBins1 / kBlock; ++j) mine[j] = hp[j * kBlock + t];
            __syncthreads();
#pragma unroll
            for (int j = 0; j < kBins1 / kBlock; ++j)
                if (mine[j]) atomicAdd(&sum1[(j * kBlock + t) & ((1u << l1_bits) - 1u)], mine[j]);
            __syncthreads();
            hp = sum1;
        }
        if (search_digit<NB_PREV>(hp, ss.k_rem, above, digit, n_digit, n_above)) {
            res[1] = digit;
            res[2] = n_above;
            res[3] = n_digit;
            res[0] = 1u;
        }
        __syncthreads();
        if (res[0]) {
            ss.prefix = (ss.prefix << (LEVEL == 1 ? static_cast<uint32_t>(BITS_PREV) : l1_bits)) | res[1];
            ss.k_rem -= res[2];
            if (LEVEL == 1) {
                // the bucket's keys go to the candidate list if its slots can hold them
                const uint64_t slots = static_cast<uint64_t>(st_count) * kCandSlice;
                ss.mode = res[3] <= slots ? kModeCand : kModeFull;
                // The width of the next step's range: the widest that would hold at most half of what the
                // candidate list can take, judged by how many keys the threshold's bucket of 2^19 keys holds
                // (the range will lie around the same threshold, and the density there changes slowly).
                uint64_t would = res[3];
                uint32_t fit = kSpecBitsMax;
                while (would > slots / 2 && fit > static_cast<uint32_t>(kSpecBitsMin)) {
                    would >>= 1;
                    --fit;
                }
                while (2 * would <= slots / 2 && fit < static_cast<uint32_t>(kSpecBitsWide)) {
                    would <<= 1;
                    ++fit;
                }
                ss.w_next = fit;
            } else if (owner && t == 0) {
                uint32_t* pred = preds + static_cast<size_t>(cur) * kPredWords;
                if (ss.collected == 0) {                    // no prediction held in this step: one for the next
                    pred[0] = 1u;
                    record_t24(pred, lead_mine, cur, ss.prefix);
                    pred[2] = ss.w_next;
                    pred[3] = 0u;
                } else {                                    // a wide range held: k_level0 recorded the middle of its bin
                    refine_t24(pred, lead_mine, cur, ss.prefix);
                }
            }
        } else {                                            // only if the counts were corrupted: nothing is selected
            ss.done = 1;
        }
        ss.pending = 0;
    }
    if (ss.done != 0 || (LEVEL == 1 ? ss.l1_done != 0 : ss.l2_done != 0)) {  // block-uniform: nothing to count
        if (owner && t == 0) state_at(state_out, cur) = ss;
        return;
    }
    for (int b = t; b < NB; b += kBlock) lh[b] = 0u;
    __syncthreads();
    const uint32_t prefix = ss.prefix;
    const bool from_list = ss.mode == kModeCand;
    if (LEVEL == 2 && stats && owner && t == 0 && !from_list) atomicAdd(&stats[kStatFullMode], 1ull);
    const bool collect = LEVEL == 1 && from_list && ss.collected == 0;
    const int64_t begin = hb.begin, end = hb.end;
    if (from_list && !collect) {
        // keys that were copied to the candidate list, one wave per supertile: the count and the first
        // 64 slots (most supertiles list fewer keys) of four supertiles are requested at once, so
        // that a block with many supertiles does not wait for one round trip after the other
        constexpr int kAhead = 4;
        for (int s0 = hb.st_lo + wave; s0 < hb.st_hi; s0 += kAhead * kWaves) {
            uint32_t cnt[kAhead], key0[kAhead];
#pragma unroll
            for (int j = 0; j < kAhead; ++j) {
                const int s2 = s0 + j * kWaves;
                const bool have = s2 < hb.st_hi;            // wave-uniform
                cnt[j] = have ? out.st_cand_cnt[s2] : 0u;   // at most kCandSlice (stored clamped)
                key0[j] = have ? out.cand[static_cast<size_t>(s2) * kCandSlice + lane].x : 0u;
            }
            // the second 64 slots where the count says so (a range that holds about as many keys as the
            // index set has members lists 70 to 150 per supertile), and the rest of all four slices at once
            // if one of them holds more than 128 (wide ranges): no trip to memory waits for another
            constexpr int kRounds = kCandSlice / kLanes - 2;
            uint32_t key1[kAhead], more[kAhead][kRounds];
            const bool long_slices =
                cnt[0] > 2 * kLanes || cnt[1] > 2 * kLanes || cnt[2] > 2 * kLanes || cnt[3] > 2 * kLanes;
            static_assert(kAhead == 4, "the test above names four counts");
#pragma unroll
            for (int j = 0; j < kAhead; ++j) {              // (a wave without a supertile has count 0 and reads nothing)
                const uint2* sl = out.cand + static_cast<size_t>(s0 + j * kWaves) * kCandSlice;
                key1[j] = static_cast<uint32_t>(kLanes + lane) < cnt[j] ? sl[kLanes + lane].x : 0u;
            }
            if (long_slices) {                              // wave-uniform
#pragma unroll
                for (int j = 0; j < kAhead; ++j) {
                    const uint2* sl = out.cand + static_cast<size_t>(s0 + j * kWaves) * kCandSlice;
#pragma unroll
                    for (int r = 0; r < kRounds; ++r) {
                        const uint32_t e = (r + 2) * kLanes + lane;
                        more[j][r] = e < cnt[j] ? sl[e].x : 0u;
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < kAhead; ++j) {
                if (static_cast<uint32_t>(lane) < cnt[j]) count(key0[j], prefix);
                if (static_cast<uint32_t>(kLanes + lane) < cnt[j]) count(key1[j], prefix);
                if (long_slices) {
#pragma unroll
                    for (int r = 0; r < kRounds; ++r)
                        if ((r + 2) * kLanes + lane < cnt[j]) count(more[j][r], prefix);
                }
            }
        }
    } else {
        for (int s2 = hb.st_lo; s2 < hb.st_hi; ++s2) {
            const int64_t a0 = static_cast<int64_t>(hb.a0) + static_cast<int64_t>(s2 - hb.st_lo) * kSuper;
            if constexpr (LEVEL == 1) {
                if (collect) {   // block-uniform: no list yet, this pass makes it
                    __shared__ uint32_t fill;
                    __shared__ CollectStage stg;
                    if (t == 0) fill = 0u;
                    __syncthreads();
                    uint2* slice = out.cand + static_cast<size_t>(s2) * kCandSlice;   // written directly: LDS is the histogram's
                    for (int it = 0; it < kTilesPerSuper / kWaves; ++it) {
                        const int wt = it * kWaves + wave;
                        const int64_t p0 = a0 + wt * kWaveTile + lane * kVec;
                        uint32_t key[4] = {0, 0, 0, 0};
                        bool ok[4] = {false, false, false, false};
                        if (p0 < end) leader_keys(mem, grad, lr, p0, begin, end, key, ok);
                        uint32_t n_above, n_in;
                        collect_tile<false>(key, ok, static_cast<uint32_t>(p0), prefix << (kBits1 + kBits2),
                                            1u << (kBits1 + kBits2), wt, lane, &fill, lh, n_above, n_in, stg, slice);
                    }
                    __syncthreads();
                    collect_flush(stg, nullptr, static_cast<size_t>(s2) * kTilesPerSuper, fill, out.wt_cnt, out.sel_mask,
                                  out.eq_mask, slice);
                    if (t == 0) {
                        const uint32_t n = fill;
                        out.st_cand_cnt[s2] = n < kCandSlice ? n : kCandSlice;
                        if (n > kCandSlice) out.full_flag[cur] = 1u;   // every overflowing block stores the same value
                    }
                    __syncthreads();   // the staging area is reused for the block's next supertile
                    continue;
                }
            }
#pragma unroll 2
            for (int it = 0; it < kTilesPerSuper / kWaves; ++it) {
                const int64_t p0 = a0 + (it * kWaves + wave) * kWaveTile + lane * kVec;
                if (p0 >= end) continue;
                uint32_t key[4];
                bool ok[4];
                leader_keys(mem, grad, lr, p0, begin, end, key, ok);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (ok[c]) count(key[c], prefix);
            }
        }
    }
    __syncthreads();                                        // flush my counts of the segment
    uint32_t* h = hist + static_cast<size_t>(cur) * NB;
    // Level 1 after a hit of a wide range counts few bits: its 2^l1_bits counters exist in as many
    // copies as 4096 words hold, one per residue of the block number (atomics on the same few lines are
    // carried out one after the other at the memory side).  Twelve bits: one copy.
    if (LEVEL == 1) h += (blockIdx.x & ((1u << (kBits1 - l1_bits)) - 1u)) << l1_bits;
    for (int b = t; b < NB; b += kBlock) {
        const uint32_t v = lh[b];
        if (v) atomicAdd(&h[b], v);
    }
    if (owner && t == 0) {
        if (LEVEL == 1) ss.pending = 1;                     // the next kernel's blocks search this histogram
        state_at(state_out, cur) = ss;
    }
}

// The last search of the threshold (7 key bits, 128 counters), done by every wave that needs the
// result instead of by a kernel of its own: from the top of the histogram, the bin that holds the
// k_rem-th largest key of the current 24-bit bucket.  Each lane brings the counts of bins `lane`
// and `64 + lane`; all 64 lanes call it.  Returns the threshold key T and sets q, the number of
// keys equal to T that are members.  The histogram is 512 bytes, so re-reading it in every wave is
// cheap (the 16 KB histograms of the earlier levels are searched once per block of the kernel
// that follows them).
__device__ __forceinline__ uint32_t find_threshold(uint32_t h_lo, uint32_t h_hi, uint32_t prefix24, uint32_t k_rem,
                                                   int lane, uint32_t& q)
{
    static_assert(kBins2 == 2 * kLanes, "two counters of the last level per lane");
    uint32_t suf_lo = h_lo, suf_hi = h_hi;                  // inclusive suffix sums over the lanes
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) {
        const uint32_t a = __shfl_down(suf_lo, off, kLanes), b = __shfl_down(suf_hi, off, kLanes);
        if (lane + off < kLanes) {
            suf_lo += a;
            suf_hi += b;
        }
    }
    suf_lo += __builtin_amdgcn_readfirstlane(suf_hi);       // bins 64..127 lie above every bin of the low half
    const uint32_t above_lo = suf_lo - h_lo, above_hi = suf_hi - h_hi;   // keys in higher bins
    // exactly one bin qualifies, unless the counts were corrupted: then nothing is a member
    const uint64_t hit_hi = __builtin_amdgcn_ballot_w64(above_hi < k_rem && k_rem <= suf_hi);
    const uint64_t hit_lo = __builtin_amdgcn_ballot_w64(above_lo < k_rem && k_rem <= suf_lo);
    uint32_t T = 0xffffffffu;
    q = 0u;
    if (hit_hi) {                                           // wave-uniform
        const int src = __ffsll(static_cast<unsigned long long>(hit_hi)) - 1;
        T = (prefix24 << kBits2) | static_cast<uint32_t>(kLanes + src);
        q = k_rem - __shfl(above_hi, src, kLanes);
    } else if (hit_lo) {
        const int src = __ffsll(static_cast<unsigned long long>(hit_lo)) - 1;
        T = (prefix24 << kBits2) | static_cast<uint32_t>(src);
        q = k_rem - __shfl(above_lo, src, kLanes);
    }
    return T;
}

// Orders one wave's LDS accesses: what its lanes wrote or added before is seen by its lanes after.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Per wave tile of the leader's vector: number of keys above the threshold (low half of the
// packed counter) and equal to it (high half), and the two bitmasks that go with them.
// Full-pass mode recomputes every key; candidate mode adds the listed keys to what the collecting
// pass started.  Also leaves the supertile's totals for the prefix scan.  One WAVE per supertile
// and no barrier between the waves of a block: a block per supertile spent its time waiting at
// barriers with most of its threads idle (a supertile lists a few dozen to a few hundred keys).
template <typename G>
__global__ void __launch_bounds__(kBlock)
k_tilecount(const float* __restrict__ mem, const G* __restrict__ grad, float lr, const SegDesc* __restrict__ segs,
            const StDesc* __restrict__ sts, int n_st, SegState* __restrict__ state, const uint32_t* __restrict__ hist2,
            uint32_t* __restrict__ wt_cnt, const uint2* __restrict__ cand, const uint32_t* __restrict__ st_cand_cnt,
            uint64_t* __restrict__ sel_mask, uint64_t* __restrict__ eq_mask, uint2* __restrict__ st_sum, bool one_seg,
            bool many)
{
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes), lane = threadIdx.x % kLanes;
    const int st = blockIdx.x * kWaves + wave;
    if (st >= n_st) return;                                 // whole wave
    __shared__ uint32_t cnt_s[kWaves][kTilesPerSuper];
    uint32_t* cnt = cnt_s[wave];
    const size_t tile0 = static_cast<size_t>(st) * kTilesPerSuper;
    // Everything the supertile's number alone addresses is requested before the first dependent load
    // returns: its descriptor, its candidate count, the first 64 slots of its slice (used up to the
    // count, in candidate mode only) and the tiles' running counts.  With very many supertiles
    // (`many`, the same for the whole grid) the kernel is bound by its traffic, not by round trips:
    // slices are a quarter to a tenth full, so the slots are then read up to the count only.
    const uint2* slice = cand + static_cast<size_t>(st) * kCandSlice;
    const StDesc d = sts[st];
    const uint32_t n_listed = st_cand_cnt[st];
    uint2 ce_early;
    if (many)
        ce_early = static_cast<uint32_t>(lane) < n_listed ? slice[lane] : make_uint2(0u, 0u);
    else
        ce_early = slice[lane];
    const uint32_t cnt_pre = lane < kTilesPerSuper ? wt_cnt[tile0 + lane] : 0u;
    // what the segment number addresses: a second round trip, unless the layout has one segment only
    // (one_seg, the same for the whole grid): then nothing below waits for the descriptor
    SegState ss;
    uint32_t h_lo, h_hi;
    int st_first;
    if (one_seg) {
        ss = state_at(state, 0);
        h_lo = hist2[lane];
        h_hi = hist2[kLanes + lane];
        st_first = 0;
    } else {
        ss = state_at(state, d.seg);
        const uint32_t* h2 = hist2 + static_cast<size_t>(d.seg) * kBins2;
        h_lo = h2[lane];
        h_hi = h2[kLanes + lane];
        st_first = segs[d.seg].st_first;
    }
    if (ss.l2_done) return;                                 // whole wave: counted by the block that searched it
    uint32_t T = ss.T, q = ss.q;                            // an empty index set keeps T above every key
    if (!ss.done) {                                         // wave-uniform
        T = find_threshold(h_lo, h_hi, ss.prefix, ss.k_rem, lane, q);
        if (st == st_first && lane == 0) {                  // for the tie quota of the slot pass
            state_at(state, d.seg).T = T;
            state_at(state, d.seg).q = q;
        }
    }

    uint32_t v = 0u;                                        // lanes 0..31: the packed counter of one tile each
    if (!ss.done && ss.mode == kModeCand) {
        if (lane < kTilesPerSuper) cnt[lane] = cnt_pre;
        wave_lds_fence();
        const uint32_t n = n_listed < kCandSlice ? n_listed : kCandSlice;   // never use what lies past the count
        uint32_t* sel32 = reinterpret_cast<uint32_t*>(sel_mask);
        uint32_t* eq32 = reinterpret_cast<uint32_t*>(eq_mask);
        // what a listed key means for the masks: 0 nothing; else bit 31, bit 30 = above T, position in the supertile
        auto classify = [&](const uint2 ce, uint32_t e) {
            const uint32_t rel = ce.y - static_cast<uint32_t>(d.a0);
            const bool ok = e < n && ce.x >= T && rel < kSuper;   // (a listed position lies in its supertile)
            return ok ? (0x80000000u | (ce.x > T ? 0x40000000u : 0u) | rel) : 0u;
        };
        auto mark = [&](uint32_t what) {
            const uint32_t rel = what & (kSuper - 1);
            const uint32_t wt = rel / kWaveTile, l = (rel % kWaveTile) / kVec, c = rel % kVec;
            const size_t word = ((tile0 + wt) * 4 + c) * 2 + (l >> 5);
            if (what & 0x40000000u) {
                atomicAdd(&cnt[wt], 1u);
                atomicOr(&sel32[word], 1u << (l & 31));
            } else {
                atomicAdd(&cnt[wt], 0x10000u);
                atomicOr(&eq32[word], 1u << (l & 31));
            }
        };
        // Of a long slice all keys are requested before the first one is used, and what each means is
        // worked out before the first atomic is issued: an atomic between a load and its use makes that
        // use wait for the atomic as well, one trip to memory after the other.
        if (n <= 2 * kLanes) {                              // wave-uniform: the usual slice, one or two rounds
            for (uint32_t e = lane; e < n; e += kLanes) {
                const uint32_t what = classify(e < kLanes ? ce_early : slice[e], e);
                if (what) mark(what);
            }
        } else {                                            // a slice of a wide range: up to 512 keys
            constexpr int kRounds = kCandSlice / kLanes;
            uint2 ent[kRounds];
            ent[0] = ce_early;
#pragma unroll
            for (int r = 1; r < kRounds; ++r) {
                const uint32_t e = r * kLanes + lane;
                ent[r] = e < n ? slice[e] : make_uint2(0u, 0u);
            }
            uint32_t what[kRounds];
#pragma unroll
            for (int r = 0; r < kRounds; ++r) what[r] = classify(ent[r], r * kLanes + lane);
#pragma unroll
            for (int r = 0; r < kRounds; ++r)
                if (what[r]) mark(what[r]);
        }
        wave_lds_fence();
        if (lane < kTilesPerSuper) v = cnt[lane];
    } else {
        const int64_t begin = d.begin, end = d.end;
#pragma unroll 2
        for (int wt = 0; wt < kTilesPerSuper; ++wt) {
            const int64_t p0 = static_cast<int64_t>(d.a0) + wt * kWaveTile + lane * kVec;
            uint32_t key[4] = {0, 0, 0, 0};
            bool ok[4] = {false, false, false, false};
            if (!ss.done && p0 < end) leader_keys(mem, grad, lr, p0, begin, end, key, ok);   // (no members: nothing is read)
            uint64_t gt[4], eq[4];
            uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                gt[c] = __ballot(ok[c] && key[c] > T);
                eq[c] = __ballot(ok[c] && key[c] == T);
                n_gt += __popcll(gt[c]);
                n_eq += __popcll(eq[c]);
            }
            if (lane == wt) v = n_gt | (n_eq << 16);        // at most 256 each
            if (lane == 0) {
                store_tile_masks(sel_mask, tile0 + wt, gt);
                store_tile_masks(eq_mask, tile0 + wt, eq);
            }
        }
    }
    if (lane < kTilesPerSuper) wt_cnt[tile0 + lane] = v;
    const uint32_t s2 = wave_sum(v);                        // at most 8192 each: no carry between halves
    if (lane == 0) st_sum[st] = make_uint2(s2 & 0xffffu, s2 >> 16);
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

// The end of the slot pass for one supertile, by all 64 lanes of a wave (lanes 0..31 own one wave
// tile each): `packed` is the tile's counter (members / keys equal to the threshold), px and py the
// members and ties in the segment's earlier supertiles, q the segment's quota of ties.
__device__ __forceinline__ void finish_slots(size_t tile, uint32_t packed, uint32_t px, uint32_t py, uint32_t q,
                                             uint32_t out_base, int lane, uint64_t* __restrict__ sel_mask,
                                             const uint64_t* __restrict__ eq_mask, uint32_t* __restrict__ tile_slot)
{
    uint32_t inc = packed;
#pragma unroll
    for (int off = 1; off < kLanes; off <<= 1) {
        const uint32_t a = __shfl_up(inc, off, kLanes);
        if (lane >= off) inc += a;
    }
    const uint32_t excl = inc - packed;                     // halves stay below 8192: no carry
    const uint32_t gt_before = px + (excl & 0xffffu);
    const uint32_t eq_before = py + (excl >> 16);
    if (lane >= kTilesPerSuper) return;
    tile_slot[tile] = out_base + gt_before + (eq_before < q ? eq_before : q);

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

// Prefix scan, level 2, one wave per supertile: first output slot of each of its 32 wave tiles
// = members in the segment's earlier supertiles + earlier tiles of the supertile.  Keys equal to
// the threshold become members here, in position order, until the segment's quota q is used up
// (Eq. 2 with ties resolved towards the lowest positions).
// OWN_SCAN (up to kOwnScanMaxSt supertiles): blocks of 16 waves add up the supertile totals before
// their first supertile themselves, which saves the k_scan launch; each block reads at most n_st
// totals, n_st^2 / 32 in all.  Otherwise the prefixes come from k_scan (per chunk of 1024
// supertiles) and the chunk totals.
template <bool OWN_SCAN>
__global__ void __launch_bounds__(OWN_SCAN ? kSlotsOwnScanBlock : kBlock)
k_slots(const SegDesc* __restrict__ segs, const StDesc* __restrict__ sts, int n_st, const SegState* __restrict__ state,
        const uint32_t* __restrict__ wt_cnt, const uint2* __restrict__ st_sum, const uint2* __restrict__ st_prefix,
        const uint2* __restrict__ chunk_tot, uint64_t* __restrict__ sel_mask, const uint64_t* __restrict__ eq_mask,
        uint32_t* __restrict__ tile_slot, bool one_seg)
{
    constexpr int kThreads = OWN_SCAN ? kSlotsOwnScanBlock : kBlock;
    constexpr int kWavesHere = kThreads / kLanes;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
    const int lane = threadIdx.x % kLanes;
    const int st0 = blockIdx.x * kWavesHere;                // the block's first supertile (exists: the grid is exact)
    const int st = st0 + wave;
    uint32_t px = 0, py = 0;                                // members / ties in the segment's earlier supertiles
    // Requests are grouped by what addresses them, so that each group costs one round trip: first what the
    // supertile numbers address, then what the segment numbers address, then the totals to add up.
    const bool live = st < n_st;                            // whole wave
    const int st_c = live ? st : st0;
    const StDesc d = sts[st_c];
    const size_t tile = static_cast<size_t>(st_c) * kTilesPerSuper + lane;  // lanes 0..31 own one tile each
    const uint32_t packed = lane < kTilesPerSuper ? wt_cnt[tile] : 0u;
    // (with one segment only -- one_seg, the same for the whole grid -- nothing here waits for the descriptor)
    const int seg0 = (OWN_SCAN && !one_seg) ? sts[st0].seg : 0;
    SegDesc sd;
    uint32_t q;
    if (one_seg) {
        sd = segs[0];
        q = state_at(state, 0).q;
    } else {
        sd = segs[d.seg];
        q = state_at(state, d.seg).q;
    }
    if (OWN_SCAN) {
        // all threads: totals of the supertiles between the start of the first supertile's segment and st0
        __shared__ uint32_t part_x[kWavesHere], part_y[kWavesHere];
        const int seg0_first = segs[seg0].st_first;
        // the block's own supertiles before mine that belong to my segment (at most 15)
        const int j_own = (sd.st_first > st0 ? sd.st_first : st0) + lane;
        const uint2 t_own = (live && j_own < st) ? st_sum[j_own] : make_uint2(0, 0);
        uint32_t bx = 0, by = 0;
        for (int j = seg0_first + static_cast<int>(threadIdx.x); j < st0; j += kThreads) {
            const uint2 t = st_sum[j];
            bx += t.x;
            by += t.y;
        }
        bx = wave_sum(bx);
        by = wave_sum(by);
        if (lane == 0) {
            part_x[wave] = bx;
            part_y[wave] = by;
        }
        __syncthreads();
        if (!live) return;                                  // whole wave
        if (one_seg || d.seg == seg0) {                     // wave-uniform
            for (int w = 0; w < kWavesHere; ++w) {
                px += part_x[w];
                py += part_y[w];
            }
        }
        px += wave_sum(t_own.x);
        py += wave_sum(t_own.y);
    } else {
        if (!live) return;                                  // whole wave
        // totals of the segment's earlier chunks, then the prefix inside my chunk
        const int my_chunk = (st - sd.st_first) / kChunk;
        uint32_t cx = 0, cy = 0;
        for (int c = lane; c < my_chunk; c += kLanes) {
            const uint2 t = chunk_tot[sd.chunk_first + c];
            cx += t.x;
            cy += t.y;
        }
        const uint2 sp = st_prefix[st];
        px = wave_sum(cx) + sp.x;
        py = wave_sum(cy) + sp.y;
    }

    finish_slots(tile, packed, px, py, q, static_cast<uint32_t>(sd.out_base), lane, sel_mask, eq_mask, tile_slot);
}


// The same pass for very many supertiles (always with k_scan's prefixes): a wave takes kSlotsBatch
// consecutive supertiles and requests what their numbers address all at once, instead of one wave per
// supertile in a dozen rounds that each wait for their own round trips.
__global__ void __launch_bounds__(kBlock)
k_slots_many(const SegDesc* __restrict__ segs, const StDesc* __restrict__ sts, int n_st, const SegState* __restrict__ state,
             const uint32_t* __restrict__ wt_cnt, const uint2* __restrict__ st_prefix, const uint2* __restrict__ chunk_tot,
             uint64_t* __restrict__ sel_mask, const uint64_t* __restrict__ eq_mask, uint32_t* __restrict__ tile_slot,
             bool one_seg)
{
    constexpr int B = kSlotsBatch;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kLanes);
    const int lane = threadIdx.x % kLanes;
    const int st_begin = (blockIdx.x * kWaves + wave) * B;
    if (st_begin >= n_st) return;                           // whole wave
    StDesc d[B];
    uint32_t packed[B];
    uint2 sp[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const int st_c = st_begin + j < n_st ? st_begin + j : n_st - 1;
        d[j] = sts[st_c];
        packed[j] = lane < kTilesPerSuper ? wt_cnt[static_cast<size_t>(st_c) * kTilesPerSuper + lane] : 0u;
        sp[j] = st_prefix[st_c];
    }
    SegDesc sd = segs[0];
    uint32_t q = state_at(state, 0).q;
    int cur_seg = 0, cur_chunk = -1;
    uint32_t cx = 0, cy = 0;                                // totals of the segment's chunks before cur_chunk
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const int st = st_begin + j;
        if (st >= n_st) break;                              // whole wave
        if (!one_seg && d[j].seg != cur_seg) {              // wave-uniform
            cur_seg = d[j].seg;
            sd = segs[cur_seg];
            q = state_at(state, cur_seg).q;
            cur_chunk = -1;
        }
        const int my_chunk = (st - sd.st_first) / kChunk;
        if (my_chunk != cur_chunk) {                        // wave-uniform: once per wave, as a rule
            uint32_t ax = 0, ay = 0;
            for (int c = lane; c < my_chunk; c += kLanes) {
                const uint2 t = chunk_tot[sd.chunk_first + c];
                ax += t.x;
                ay += t.y;
            }
            cx = wave_sum(ax);
            cy = wave_sum(ay);
            cur_chunk = my_chunk;
        }
        finish_slots(static_cast<size_t>(st) * kTilesPerSuper + lane, packed[j], cx + sp[j].x, cy + sp[j].y, q,
                     static_cast<uint32_t>(sd.out_base), lane, sel_mask, eq_mask, tile_slot);
    }
}

}  // namespace
