// The all-learner pass (Alg. 1 lines 6, 7, 10; Eq. 3, 5) and the sum over learners.
// Part of scalecom.hip's single translation unit.
#pragma once

#include <hip/hip_runtime.h>

#include "device_helpers.h"
#include "geometry.h"

namespace {

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
         int64_t k_total, int32_t* __restrict__ idx_out, int learner0, uint32_t* __restrict__ clear_from,
         size_t clear_words)
{
    // grid = (learners, groups of 4 wave tiles split over y and z): x runs fastest, so blocks that
    // are scheduled together work on the same positions of different learners
    const int learner = learner0 + blockIdx.x;
    const int group = blockIdx.y + blockIdx.z * gridDim.y;
    // The selection's per-step counters and histograms have been read for the last time before this
    // kernel starts; the blocks of its first learner zero them on the way, so that the next step finds
    // them clean and no step pays for a clearing launch.
    if (clear_words != 0 && blockIdx.x == 0) {              // block-uniform
        const size_t stride = static_cast<size_t>(gridDim.y) * gridDim.z * kBlock;
        for (size_t i = static_cast<size_t>(group) * kBlock + threadIdx.x; i < clear_words; i += stride) clear_from[i] = 0u;
    }
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
        update_block<G, true>(mem, grad, lr, beta, one_minus_beta, d, wave, lane, rel0, S, before, total, slot0, my_vals,
                              my_idx, stage_val, stage_pos);
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

}  // namespace
