// Kernels beside the hot path: weight update on the index set (Alg. 1 lines 10, 12), similarity
// diagnostics (Sec. 2, Sec. 3), the copy yardstick.  Part of scalecom.hip's single translation unit.
#pragma once

#include <hip/hip_runtime.h>

#include "device_helpers.h"
#include "geometry.h"

namespace {

// Weight update on the index set (Alg. 1 lines 10 and 12): theta[idx[t]] -= scale * vals[t].
__global__ void __launch_bounds__(kBlock)
k_apply_update(float* __restrict__ theta, int64_t numel, const int32_t* __restrict__ idx, const float* __restrict__ vals,
               int64_t k, float neg_scale)
{
    const int64_t t = (static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x) * kBlock + threadIdx.x;
    if (t >= k) return;
    const int32_t j = idx[t];
    if (j < 0 || j >= numel) return;                        // a position outside theta is skipped, never touched
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

}  // namespace
