// Chunk-wise selection, the selector of the paper's own implementation (Sec. 4, App. E, Fig. A2).
// Part of scalecom.hip's single translation unit.
#pragma once

#include <hip/hip_runtime.h>

#include "device_helpers.h"
#include "geometry.h"

namespace {

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
            atomicMax(&best[static_cast<uint32_t>(sd.out_base) + j],
                      (static_cast<unsigned long long>(k_max) << 32) | inv_max);
    }
}

// After the leader pass: position of each chunk's winner to idx_out and to the membership mask;
// first output slot of every wave tile (chunk j of a segment owns slot out_base + j).  (best[] is
// zeroed again by the all-learner pass that follows.)
__global__ void __launch_bounds__(kBlock)
k_chunk_marks(const SegDesc* __restrict__ segs, int n_tensors, const StDesc* __restrict__ sts,
              const unsigned long long* __restrict__ best, int64_t k_total, int64_t n_tiles,
              uint64_t* __restrict__ sel_mask, uint32_t* __restrict__ tile_slot, int32_t* __restrict__ idx_out)
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
        if (pos >= static_cast<uint32_t>(sd.begin) && pos < static_cast<uint32_t>(sd.end)) {   // always, unless best[] was corrupted
            const uint32_t rel = pos - (static_cast<uint32_t>(sd.begin) & ~static_cast<uint32_t>(kVec - 1));
            const size_t tile = static_cast<size_t>(sd.st_first) * kTilesPerSuper + rel / kWaveTile;
            const uint32_t l = (rel % kWaveTile) / kVec, c = rel % kVec;
            atomicOr(reinterpret_cast<uint32_t*>(sel_mask) + (tile * 4 + c) * 2 + (l >> 5), 1u << (l & 31));
        }
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

}  // namespace
