// C-ABI and host side of ScaleCom's per-step compression path on gfx950 (CDNA4, 64-lane
// wavefronts): CLT-k with low-pass-filtered error feedback (arXiv 2104.11125, Alg. 1 lines 6, 7,
// 10; Eq. 2, 3, 5).  See include/scalecom.h for the contract of each entry point.  The kernels
// live in the headers included below (one translation unit).
//
// Structure of one step (all on the context's stream, no host synchronisation).  The 31-bit
// magnitude key |x_L| of the leader's x_L = fma(lr, grad_L, mem_L) (recomputed on the fly, never
// stored) is resolved 12 + 12 + 7 bits at a time (radix select):
//
//   predicted   leader, ONE pass, for segments that carry a prediction: a range of keys around the
//               threshold the step expects (this leader's last one, moved on by the recent
//               growth), whose width follows how densely the keys lie there (with error feedback
//               they pile up below the threshold) and how far the threshold moves between steps.
//               Keys above the range are members for sure (counted per 256-element wave tile,
//               marked in the membership bitmask); keys inside it are copied, with their
//               positions, to a small candidate list and counted per 128 keys (in 64 bins if the
//               range is wider than 2^19 keys)
//   level0      per segment: did the k-th largest key fall inside the range (exact check on
//               counts)?  Then the top 24 bits of the threshold follow from the range's counts
//               (Eq. 2; of a wide range the bin, whose open bits level 1 then resolves on the
//               listed keys).  Otherwise (no prediction, or a miss): histogram of the top 12 key bits
//               of the leader's vector.  A segment of one supertile is finished here by its one
//               block, without prediction
//   level<1>    a histogram of level0 is searched by every block that needs the result; then the
//               next 12 key bits, histogrammed over the candidate list -- nothing to do if they
//               are known already; for segments that went through the level-0 histogram this is
//               the second leader pass that makes the list
//   level<2>    (search of level 1's histogram, then) the last 7 key bits
//   tilecount   the exact threshold key T and the number q of keys equal to T that still belong
//               to the set (every wave searches the last 128 counters for itself);
//               candidates above / equal to T are added to the per-tile counts and bitmasks
//               (a segment whose bucket does not fit the candidate list -- many equal keys --
//               takes levels 1, 2 and this step as full leader passes instead of the list)
//   scan, slots prefix sums of the counts over tiles: first output slot of every wave tile;
//               keys equal to T become members in position order until q are taken
//   update      every learner (eight per launch), one (learner, 1024 positions) pair per block: one read of
//               (mem, grad), one write of mem (Eq. 5); members also store x_i into a small
//               [learner][slot] staging array and learner 0 writes the index (Eq. 3)
//   reduce      reduced[t] = x_0[t] + x_1[t] + ... in learner order  (Alg. 1 line 10)
//
// In the steady state (predictions hold) the leader's vector is read exactly once before the
// all-learner pass, and 8 kernels make a step (up to 8 learners and 84 M elements).  No kernel reads what another block of the same
// launch wrote, so there are no fences or waits between blocks.  The prediction only decides how much work is
// done, never what is selected.  The output is ascending by position and deterministic.
// Nothing here is a dense contraction, so there is no MFMA; the kernels are bound by HBM traffic
// (update, predicted) and by launch latency (the small ones).
// The chunk-wise selector (scalecom_step_chunked, scalecom_step_layers_chunked) replaces everything
// before `update` by chunk_select + chunk_marks.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "scalecom.h"

#include "geometry.h"
#include "device_helpers.h"
#include "select_kernels.h"
#include "update_kernels.h"
#include "chunk_kernels.h"
#include "aux_kernels.h"

namespace {

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
constexpr size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int64_t max_supertiles(int64_t numel_max, int n_tensors_max)
{
    return numel_max / kSuper + 2 * static_cast<int64_t>(n_tensors_max) + 2;
}

constexpr int64_t max_chunks(int64_t numel_max, int n_tensors_max)
{
    return max_supertiles(numel_max, n_tensors_max) / kChunk + static_cast<int64_t>(n_tensors_max) + 1;
}

struct WsLayout {
    size_t segs, sts, chunks, hblocks, small, preds, stats, state, wt_cnt, st_sum, st_prefix, chunk_tot, st_cand_cnt, cand, sel_mask,
        eq_mask, tile_slot, vals, best, total;
    // per-step counters and histograms: one zone, all zero between steps (offsets inside the zone)
    size_t zone, zone_bytes, z_overflow, z_p_used, z_full_flag, z_part, z_hist0, z_hist1, z_hist1_spec, z_hist2;
};

constexpr WsLayout layout_for(int64_t numel_max, int n_tensors_max, int n_learners_max, int64_t k_max)
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
    l.hblocks = take((kHistGridMax + nt) * sizeof(HistBlock));
    l.small = take(nt * sizeof(HistBlock));              // the segments of one supertile, one block each
    // per segment: the prediction for the next step; then per learner and segment: that leader's last threshold
    l.preds = take((kPredWords + static_cast<size_t>(n_learners_max)) * nt * sizeof(uint32_t));
    l.stats = take(kStatWords * sizeof(unsigned long long));   // what the selections of this context ran into
    l.state = take(3 * nt * kStateStride);               // after level 0, after level 1, after level 2
    {
        size_t z = 0;
        auto ztake = [&](size_t bytes) {
            const size_t at = z;
            z = align_up(z + bytes, 256);
            return at;
        };
        l.z_overflow = ztake(nt * sizeof(uint32_t));
        l.z_p_used = ztake(kPredWords * nt * sizeof(uint32_t));
        l.z_full_flag = ztake(nt * sizeof(uint32_t));
        l.z_part = ztake(nt * kPartSlots * kPartWords * sizeof(uint32_t));
        l.z_hist0 = ztake(nt * kBins0 * sizeof(uint32_t));
        l.z_hist1 = ztake(nt * kBins1 * sizeof(uint32_t));
        l.z_hist1_spec = ztake(nt * kBins1 * sizeof(uint32_t));
        l.z_hist2 = ztake(nt * kBins2 * sizeof(uint32_t));
        l.zone_bytes = z;
    }
    l.zone = take(l.zone_bytes);
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
    l.best = take(static_cast<size_t>(k_max) * sizeof(unsigned long long));       // chunk-wise selector: a word per chunk
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
    int n_st = 0, n_chunks = 0, n_hblocks = 0, n_small = 0;
    // segments of one supertile are searched by a kernel of their own, on a second stream beside the
    // leader pass (contexts for more than one tensor only)
    hipStream_t side = nullptr;
    hipEvent_t fork_ev = nullptr, join_ev = nullptr;
    bool scratch_clean = false;      // true: the scratch zone is all zero (every step leaves it so)
    bool best_clean = false;         // same for the chunk-wise selector's per-chunk maxima
    bool stats_ready = false;        // the selection counters have been zeroed
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
           align_up(sizeof(ChunkDesc) * static_cast<size_t>(max_chunks(numel_max, n_tensors_max)), 256) +
           align_up(sizeof(HistBlock) * (kHistGridMax + static_cast<size_t>(n_tensors_max)), 256) +
           sizeof(HistBlock) * static_cast<size_t>(n_tensors_max);
}

// Rebuild and upload the segment, supertile, chunk and block tables if the layout differs from the cached one.
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
    const size_t hb_off = ch_off + align_up(sizeof(ChunkDesc) * static_cast<size_t>(ch_cap), 256);
    HistBlock* hblocks = reinterpret_cast<HistBlock*>(ctx->pinned + hb_off);
    const size_t sm_off =
        hb_off + align_up(sizeof(HistBlock) * (kHistGridMax + static_cast<size_t>(ctx->n_tensors_max)), 256);
    HistBlock* small = reinterpret_cast<HistBlock*>(ctx->pinned + sm_off);
    int64_t n_st = 0, n_ch = 0, out = 0;
    for (int s = 0; s < n_tensors; ++s) {
        const int64_t b = offsets[s], e = offsets[s + 1];
        const int64_t a_first = b & ~static_cast<int64_t>(kVec - 1);
        const int64_t count = e > b ? (e - a_first + kSuper - 1) / kSuper : 0;
        const int64_t n_chunks = (count + kChunk - 1) / kChunk;
        if (n_st + count > st_cap || n_ch + n_chunks > ch_cap) return fail(ctx, SCALECOM_ENOMEM, "tile table overflow");
        // a chunk longer than the segment selects like one of the segment's length, and that fits 32 bits
        const int64_t sel_chunk = std::min<int64_t>(ch[s], std::max<int64_t>(e - b, 1));
        segs[s] = SegDesc{static_cast<int32_t>(b),    static_cast<int32_t>(e),     static_cast<int32_t>(ks[s]),
                          static_cast<int32_t>(out),  static_cast<int32_t>(n_st),  static_cast<int32_t>(count),
                          static_cast<int32_t>(n_ch), static_cast<int32_t>(n_chunks), static_cast<int32_t>(sel_chunk), 0};
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
    // blocks of the search levels' kernels: every segment's supertiles in runs of equal length, so
    // that a block never holds supertiles of two segments
    const int64_t per_block = std::max<int64_t>(1, (n_st + kHistGridMax - 1) / kHistGridMax);
    int64_t n_hb = 0, n_small = 0;
    for (int s = 0; s < n_tensors; ++s) {
        const int64_t first = segs[s].st_first, count = segs[s].st_count;
        for (int64_t j = 0; j < count; j += per_block, ++n_hb)
            hblocks[n_hb] = HistBlock{s,
                                      static_cast<int32_t>(first + j),
                                      static_cast<int32_t>(first + std::min(count, j + per_block)),
                                      j == 0 ? 1 : 0,
                                      sts[first + j].a0,
                                      segs[s].begin,
                                      segs[s].end,
                                      0};
        // a segment of one supertile with a non-empty index set: searched by one block of k_small
        if (count == 1 && ks[s] > 0 && ctx->side) small[n_small++] = hblocks[n_hb - 1];
    }
    SC_HIP(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.segs, segs, sizeof(SegDesc) * n_tensors, hipMemcpyHostToDevice,
                               ctx->stream));
    if (n_st > 0) {
        SC_HIP(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.sts, sts, sizeof(StDesc) * n_st, hipMemcpyHostToDevice,
                                   ctx->stream));
        SC_HIP(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.chunks, chunks, sizeof(ChunkDesc) * n_ch, hipMemcpyHostToDevice,
                                   ctx->stream));
        SC_HIP(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.hblocks, hblocks, sizeof(HistBlock) * n_hb, hipMemcpyHostToDevice,
                                   ctx->stream));
        if (n_small > 0)
            SC_HIP(ctx, hipMemcpyAsync(ctx->ws + ctx->lay.small, small, sizeof(HistBlock) * n_small, hipMemcpyHostToDevice,
                                       ctx->stream));
    }
    // predictions of the previous layout's buckets mean nothing for this one
    k_init<<<1, kBlock, 0, ctx->stream>>>(reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.preds),
                                          (kPredWords + static_cast<size_t>(ctx->n_learners_max)) *
                                              static_cast<size_t>(ctx->n_tensors_max));
    if (!ctx->stats_ready) {
        k_init<<<1, kBlock, 0, ctx->stream>>>(reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.stats),
                                              kStatWords * sizeof(unsigned long long) / sizeof(uint32_t));
        ctx->stats_ready = true;
    }
    ctx->scratch_clean = false;
    SC_HIP(ctx, hipEventRecord(ctx->upload_done, ctx->stream));
    ctx->upload_pending = true;
    ctx->n_st = static_cast<int>(n_st);
    ctx->n_chunks = static_cast<int>(n_ch);
    ctx->n_hblocks = static_cast<int>(n_hb);
    ctx->n_small = static_cast<int>(n_small);
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
// The first launch of the pass also zeroes `clear_words` words from `clear_from`: the selection's
// per-step scratch, which nothing reads any more at that point, so that the next step finds it clean.
template <typename G, typename Mark>
void launch_update_reduce(scalecom_ctx* ctx, const LearnerPtrs& lp, int n_learners, int64_t k_total, float beta, float lr,
                          int32_t* idx_out, float* red_out, uint32_t* clear_from, size_t clear_words, Mark&& mark)
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
    for (int l0 = 0; l0 < n_learners; l0 += kUpdateLearnersPerLaunch) {
        const int nl = std::min(kUpdateLearnersPerLaunch, n_learners - l0);
        k_update<G><<<dim3(nl, gy, gz), kBlock, 0, s>>>(lp, lr, beta, 1.0f - beta, sts, n_st, sel_mask, tile_slot, vals,
                                                       k_total, idx_out, l0, clear_from, l0 == 0 ? clear_words : 0);
    }
    mark(4);
    if (k_total > 0)
        k_reduce<<<static_cast<unsigned>((k_total + kBlock - 1) / kBlock), kBlock, 0, s>>>(vals, n_learners, k_total,
                                                                                           red_out);
}

// The exact selection on one vector x = fma(lr, grad, mem) (Eq. 2): every kernel from the first
// look at the vector to the output slot of every wave tile.  Leaves the membership mask, the
// tile slots and the threshold behind.  `preds` holds one bucket prediction per segment (read and
// rewritten), `stats` the context's selection counters (null: nothing is counted).  Expects the scratch zone zeroed (clears it first if the context says it is not) and
// leaves it used: nothing reads the zone after this function's last kernel, and the caller has
// it cleared (the all-learner pass does that on the way, see launch_update_reduce), or, with
// `clear_after`, a clearing kernel is enqueued here.
template <typename G, typename Mark>
void launch_select(scalecom_ctx* ctx, const float* memL, const G* gradL, float lr, int n_tensors, uint32_t* preds,
                   uint32_t* lead_mine, unsigned long long* stats, bool clear_after, Mark&& mark)
{
    char* ws = ctx->ws;
    const WsLayout& l = ctx->lay;
    hipStream_t s = ctx->stream;
    const SegDesc* segs = reinterpret_cast<const SegDesc*>(ws + l.segs);
    const StDesc* sts = reinterpret_cast<const StDesc*>(ws + l.sts);
    const ChunkDesc* chunks = reinterpret_cast<const ChunkDesc*>(ws + l.chunks);
    const HistBlock* hblocks = reinterpret_cast<const HistBlock*>(ws + l.hblocks);
    // each level's kernel reads the state the previous one left and writes its own copy
    SegState* state0 = reinterpret_cast<SegState*>(ws + l.state);
    SegState* state1 = &state_at(state0, static_cast<size_t>(ctx->n_tensors_max));
    SegState* state = &state_at(state1, static_cast<size_t>(ctx->n_tensors_max));   // what the kernels after the search read
    char* zone = ws + l.zone;
    uint32_t* overflow = reinterpret_cast<uint32_t*>(zone + l.z_overflow);
    uint32_t* p_used = reinterpret_cast<uint32_t*>(zone + l.z_p_used);
    uint32_t* full_flag = reinterpret_cast<uint32_t*>(zone + l.z_full_flag);
    uint32_t* part = reinterpret_cast<uint32_t*>(zone + l.z_part);
    uint32_t* hist0 = reinterpret_cast<uint32_t*>(zone + l.z_hist0);
    uint32_t* hist1 = reinterpret_cast<uint32_t*>(zone + l.z_hist1);
    uint32_t* hist1_spec = reinterpret_cast<uint32_t*>(zone + l.z_hist1_spec);
    uint32_t* hist2 = reinterpret_cast<uint32_t*>(zone + l.z_hist2);
    const size_t zone_words = l.zone_bytes / sizeof(uint32_t);
    auto clear_zone = [&]() {
        const int grid = static_cast<int>(std::min<size_t>((zone_words + kBlock - 1) / kBlock, 4096));
        k_init<<<grid, kBlock, 0, s>>>(reinterpret_cast<uint32_t*>(zone), zone_words);
    };
    uint32_t* wt_cnt = reinterpret_cast<uint32_t*>(ws + l.wt_cnt);
    uint2* st_sum = reinterpret_cast<uint2*>(ws + l.st_sum);
    uint2* st_prefix = reinterpret_cast<uint2*>(ws + l.st_prefix);
    uint2* chunk_tot = reinterpret_cast<uint2*>(ws + l.chunk_tot);
    uint32_t* st_cand_cnt = reinterpret_cast<uint32_t*>(ws + l.st_cand_cnt);
    uint2* cand = reinterpret_cast<uint2*>(ws + l.cand);
    uint64_t* sel_mask = reinterpret_cast<uint64_t*>(ws + l.sel_mask);
    uint64_t* eq_mask = reinterpret_cast<uint64_t*>(ws + l.eq_mask);
    uint32_t* tile_slot = reinterpret_cast<uint32_t*>(ws + l.tile_slot);
    const int n_st = ctx->n_st;

    if (!ctx->scratch_clean) clear_zone();  // first step, new layout, or a step that failed half-way
    const int hgrid = ctx->n_hblocks;       // one block per entry of the block table
    ctx->scratch_clean = false;             // until the zone has been cleared again
    const StateCopies states{state0, state1, state};
    // Segments of one supertile: their blocks take 15-20 us from first load to last store whatever else
    // runs, so they run beside the leader pass on the context's second stream instead of holding up one
    // of the short kernels that follow it.  What they write nobody else touches before the join.
    const bool fork = ctx->n_small > 0 && ctx->side != nullptr;
    if (fork) {
        (void)hipEventRecord(ctx->fork_ev, s);
        (void)hipStreamWaitEvent(ctx->side, ctx->fork_ev, 0);
        k_small<G><<<ctx->n_small, kBlock, 0, ctx->side>>>(memL, gradL, lr, segs,
                                                          reinterpret_cast<const HistBlock*>(ws + l.small), states, preds,
                                                          lead_mine, wt_cnt, sel_mask, eq_mask, st_sum);
        (void)hipEventRecord(ctx->join_ev, ctx->side);
    }
    k_predicted<G><<<n_st, kBlock, 0, s>>>(memL, gradL, lr, segs, sts, cand, st_cand_cnt, preds, wt_cnt, sel_mask, eq_mask,
                                           part, overflow, p_used, hist1_spec, lead_mine);
    if (fork) (void)hipStreamWaitEvent(s, ctx->join_ev, 0);
    k_level0<G><<<hgrid, kBlock, 0, s>>>(memL, gradL, lr, segs, hblocks, states, fork, hist0, preds, p_used, part, overflow,
                                         hist1_spec, lead_mine, wt_cnt, sel_mask, eq_mask, st_sum, stats);
    mark(1);
    const CollectOut collect_out{wt_cnt, sel_mask, eq_mask, cand, st_cand_cnt, full_flag};
    k_level<G, 1><<<hgrid, kBlock, 0, s>>>(memL, gradL, lr, segs, hblocks, state0, state1, hist0, hist1, preds, lead_mine,
                                           collect_out, stats);
    k_level<G, 2><<<hgrid, kBlock, 0, s>>>(memL, gradL, lr, segs, hblocks, state1, state, hist1, hist2, preds, lead_mine,
                                           collect_out, stats);
    mark(2);
    k_tilecount<G><<<(n_st + kWaves - 1) / kWaves, kBlock, 0, s>>>(memL, gradL, lr, segs, sts, n_st, state, hist2, wt_cnt,
                                                                   cand, st_cand_cnt, sel_mask, eq_mask, st_sum,
                                                                   n_tensors == 1, n_st > kManySupertiles);
    if (n_st <= kOwnScanMaxSt) {   // few supertiles: the slot kernel adds up the totals before each block itself
        constexpr int per_block = kSlotsOwnScanBlock / kLanes;
        k_slots<true><<<(n_st + per_block - 1) / per_block, kSlotsOwnScanBlock, 0, s>>>(
            segs, sts, n_st, state, wt_cnt, st_sum, st_prefix, chunk_tot, sel_mask, eq_mask, tile_slot, n_tensors == 1);
    } else {
        k_scan<<<ctx->n_chunks, kChunk, 0, s>>>(chunks, st_sum, st_prefix, chunk_tot);
        if (n_st > kManySupertiles)
            k_slots_many<<<(n_st + kWaves * kSlotsBatch - 1) / (kWaves * kSlotsBatch), kBlock, 0, s>>>(
                segs, sts, n_st, state, wt_cnt, st_prefix, chunk_tot, sel_mask, eq_mask, tile_slot, n_tensors == 1);
        else
            k_slots<false><<<(n_st + kWaves - 1) / kWaves, kBlock, 0, s>>>(segs, sts, n_st, state, wt_cnt, st_sum, st_prefix,
                                                                           chunk_tot, sel_mask, eq_mask, tile_slot,
                                                                           n_tensors == 1);
    }
    if (clear_after) {
        clear_zone();
        if (hipPeekAtLastError() == hipSuccess) ctx->scratch_clean = true;
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
        uint32_t* preds = reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.preds);
        // this leader's own last thresholds, kept behind the per-segment predictions
        uint32_t* lead_mine = preds + (static_cast<size_t>(kPredWords) + static_cast<size_t>(leader)) *
                                          static_cast<size_t>(ctx->n_tensors_max);
        launch_select<G>(ctx, lp.mem[leader], static_cast<const G*>(lp.grad[leader]), lr, n_tensors, preds, lead_mine,
                         reinterpret_cast<unsigned long long*>(ctx->ws + ctx->lay.stats), false, mark);
        mark(3);
        launch_update_reduce<G>(ctx, lp, n_learners, k_total, beta, lr, idx_out, red_out,
                                reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.zone), ctx->lay.zone_bytes / sizeof(uint32_t),
                                mark);
        mark(5);
        if (timed) ++ctx->prof_steps;
    }
    SC_HIP(ctx, hipGetLastError());
    ctx->scratch_clean = true;               // the all-learner pass has left the scratch zone zeroed
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
    unsigned long long* best = reinterpret_cast<unsigned long long*>(ws + l.best);
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
    if (!ctx->best_clean) {             // first chunked step of this context, or one that failed half-way
        const size_t words = 2 * static_cast<size_t>(ctx->k_max);   // 2 words per entry
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
        segs, n_tensors, sts, best, k_total, n_tiles, sel_mask, tile_slot, idx_out);
    mark(3);
    // nothing reads the per-chunk maxima any more: the all-learner pass zeroes this call's entries on the way
    launch_update_reduce<G>(ctx, lp, n_learners, k_total, beta, lr, idx_out, red_out, reinterpret_cast<uint32_t*>(best),
                            2 * static_cast<size_t>(k_total), mark);
    mark(5);
    if (timed) ++ctx->prof_steps;
    SC_HIP(ctx, hipGetLastError());
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
    d.total = d.preds + align_up(kPredWords * static_cast<size_t>(n_tensors_max) * sizeof(uint32_t), 256);
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
        k_init<<<1, kBlock, 0, s>>>(preds, kPredWords * static_cast<size_t>(n_tensors));
        launch_select<G>(ctx, lp.mem[leader], static_cast<const G*>(lp.grad[leader]), lr, n_tensors, preds, nullptr, nullptr,
                         true, no_mark);
        SC_HIP(ctx, hipMemcpyAsync(mask_a, sel_mask, mask_bytes, hipMemcpyDeviceToDevice, s));
        // the top-k of the summed error-feedback gradients
        const int64_t blocks = (end - begin + kBlock - 1) / kBlock;
        const unsigned gx = static_cast<unsigned>(std::min<int64_t>(blocks, 1 << 20));
        const dim3 grid(gx, static_cast<unsigned>((blocks + gx - 1) / gx));
        k_sum_x<G><<<grid, kBlock, 0, s>>>(lp, n_learners, lr, begin, end, y);
        k_init<<<1, kBlock, 0, s>>>(preds, kPredWords * static_cast<size_t>(n_tensors));
        launch_select<NoGrad>(ctx, y, static_cast<const NoGrad*>(nullptr), 0.0f, n_tensors, preds, nullptr, nullptr, true,
                              no_mark);
        k_mask_overlap<<<(ctx->n_st + kWaves - 1) / kWaves, kBlock, 0, s>>>(sts, ctx->n_st, mask_a, sel_mask, d_out);
    }
    SC_HIP(ctx, hipGetLastError());
    return SCALECOM_OK;
}

// ------------------------------------------------------------------------------------------
// scalecom_step_static: the whole-vector step for callers that cannot allocate device memory.
// Its workspace is a static device array of the library, one copy per GPU, laid out like a
// caller's workspace for the largest sizes the entry point accepts.
// ------------------------------------------------------------------------------------------
constexpr int64_t kStaticNumelMax = SCALECOM_STATIC_NUMEL_MAX;
constexpr int kStaticLearnersMax = SCALECOM_STATIC_LEARNERS_MAX;
constexpr int64_t kStaticKMax = SCALECOM_STATIC_K_MAX;
constexpr WsLayout kStaticLayout = layout_for(kStaticNumelMax, 1, kStaticLearnersMax, kStaticKMax);
constexpr size_t kStaticBytes = kStaticLayout.total;
static_assert(kStaticBytes <= (size_t{16} << 20), "the static workspace stays modest");

// In host code this name is only a handle for hipGetSymbolAddress: it is not a device address.
static __device__ __align__(256) unsigned char static_scratch[kStaticBytes];

constexpr int kStaticDevicesMax = 64;
struct StaticSlot {                 // host side of one GPU's static workspace
    std::mutex lock;                // the host state below; the GPU work of two calls is ordered by the caller
    char* ptr = nullptr;            // device address of this GPU's copy of static_scratch
    scalecom_ctx ctx;               // a context without staging memory: its tables are built on the device
    int64_t numel = -1, k = -1;     // the layout whose tables and predictions the workspace holds
    int gdt = -1;
};
StaticSlot g_static[kStaticDevicesMax];
thread_local std::string g_static_error;   // detail of this thread's last failed scalecom_step_static

scalecom_status static_fail(scalecom_status st, const std::string& msg)
{
    g_static_error = msg;
    return st;
}

// The tables of a whole-vector layout (one segment [0, numel) with an index set of k positions),
// written by the GPU: what ensure_tables builds on the host and uploads for offsets = {0, numel}.
__global__ void __launch_bounds__(kBlock)
k_flat_tables(SegDesc* __restrict__ segs, StDesc* __restrict__ sts, ChunkDesc* __restrict__ chunks,
              HistBlock* __restrict__ hblocks, int32_t numel, int32_t k, int32_t n_st, int32_t n_ch, int32_t per_block,
              int32_t n_hb)
{
    const int32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i == 0) segs[0] = SegDesc{0, numel, k, 0, 0, n_st, 0, n_ch, 0, 0};
    if (i < n_st) sts[i] = StDesc{0, i * kSuper, 0, numel, k, {0, 0, 0}};
    if (i < n_ch) chunks[i] = ChunkDesc{0, i * kChunk, n_st - i * kChunk < kChunk ? n_st - i * kChunk : kChunk, 0};
    if (i < n_hb) {
        const int32_t lo = i * per_block, hi = lo + per_block < n_st ? lo + per_block : n_st;
        hblocks[i] = HistBlock{0, lo, hi, i == 0 ? 1 : 0, lo * kSuper, 0, numel, 0};
    }
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
    if (n_tensors_max > 1) {                // (a whole vector of one supertile is handled in the main chain)
        if (hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&ctx->fork_ev, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&ctx->join_ev, hipEventDisableTiming) != hipSuccess)
            return bail(SCALECOM_EHIP);
    }
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

scalecom_status scalecom_step_static(int device, void* hip_stream, float* const* mem, const void* const* grad,
                                     int n_learners, int64_t numel, int64_t k, float beta, float lr, int64_t step,
                                     scalecom_grad_dtype grad_dtype, int32_t* idx_out, float* reduced_vals_out)
{
    g_static_error.clear();
    if (device < 0 || device >= kStaticDevicesMax) return static_fail(SCALECOM_EINVAL, "device ordinal out of range");
    if (grad_dtype != SCALECOM_GRAD_F32 && grad_dtype != SCALECOM_GRAD_BF16)
        return static_fail(SCALECOM_EINVAL, "unknown grad_dtype");
    if (numel < 0 || numel > kStaticNumelMax)
        return static_fail(SCALECOM_EINVAL, "numel exceeds SCALECOM_STATIC_NUMEL_MAX (use scalecom_step with a workspace)");
    if (n_learners < 1 || n_learners > kStaticLearnersMax)
        return static_fail(SCALECOM_EINVAL, "n_learners exceeds SCALECOM_STATIC_LEARNERS_MAX (use scalecom_step with a workspace)");
    if (k < 0 || k > numel) return static_fail(SCALECOM_EINVAL, "k must satisfy 0 <= k <= numel");
    if (k > kStaticKMax)
        return static_fail(SCALECOM_EINVAL, "k exceeds SCALECOM_STATIC_K_MAX (use scalecom_step with a workspace)");
    if (!(beta > 0.0f && beta <= 1.0f)) return static_fail(SCALECOM_EINVAL, "beta must satisfy 0 < beta <= 1");
    if (!std::isfinite(lr)) return static_fail(SCALECOM_EINVAL, "lr must be finite");
    if (step < 0) return static_fail(SCALECOM_EINVAL, "step must be >= 0");
    if (!mem || !grad) return static_fail(SCALECOM_EINVAL, "null argument");
    if (numel == 0) return SCALECOM_OK;                         // nothing to do
    if (k > 0 && (!idx_out || !reduced_vals_out)) return static_fail(SCALECOM_EINVAL, "null output");

    StaticSlot& slot = g_static[device];
    std::lock_guard<std::mutex> hold(slot.lock);
    scalecom_ctx* ctx = &slot.ctx;
    auto hip_fail = [&](const char* what, hipError_t e) {
        return static_fail(SCALECOM_EHIP, std::string(what) + ": " + hipGetErrorString(e));
    };
    DeviceGuard guard;
    hipError_t e = guard.enter(device);
    if (e != hipSuccess) return hip_fail("hipSetDevice", e);
    if (!slot.ptr) {                                            // first call on this GPU: where its copy of the array lives
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, device);
        if (e != hipSuccess) return hip_fail("hipGetDeviceProperties", e);
        if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
            return static_fail(SCALECOM_EUNSUPPORTED, "the device is not a gfx950 GPU");
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch));
        if (e != hipSuccess || !p) return hip_fail("hipGetSymbolAddress(static_scratch)", e);
        slot.ptr = static_cast<char*>(p);
        ctx->device = device;
        ctx->ws = slot.ptr;
        ctx->n_learners_max = kStaticLearnersMax;
        ctx->numel_max = kStaticNumelMax;
        ctx->k_max = kStaticKMax;
        ctx->n_tensors_max = 1;
        ctx->lay = kStaticLayout;
    }
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->gdt = grad_dtype;
    LearnerPtrs lp;
    if (check_learners(ctx, mem, grad, n_learners, lp) != SCALECOM_OK) return static_fail(SCALECOM_EINVAL, ctx->last_error);

    if (slot.numel != numel || slot.k != k || slot.gdt != static_cast<int>(grad_dtype)) {
        // another layout than the last call's: new tables, no predictions, counters and histograms cleared
        const WsLayout& l = ctx->lay;
        const int32_t n_st = static_cast<int32_t>((numel + kSuper - 1) / kSuper);
        const int32_t n_ch = (n_st + kChunk - 1) / kChunk;
        const int32_t per_block = std::max<int32_t>(1, (n_st + kHistGridMax - 1) / kHistGridMax);
        const int32_t n_hb = (n_st + per_block - 1) / per_block;
        k_flat_tables<<<(n_st + kBlock - 1) / kBlock, kBlock, 0, ctx->stream>>>(
            reinterpret_cast<SegDesc*>(slot.ptr + l.segs), reinterpret_cast<StDesc*>(slot.ptr + l.sts),
            reinterpret_cast<ChunkDesc*>(slot.ptr + l.chunks), reinterpret_cast<HistBlock*>(slot.ptr + l.hblocks),
            static_cast<int32_t>(numel), static_cast<int32_t>(k), n_st, n_ch, per_block, n_hb);
        k_init<<<1, kBlock, 0, ctx->stream>>>(reinterpret_cast<uint32_t*>(slot.ptr + l.preds),
                                              (kPredWords + static_cast<size_t>(kStaticLearnersMax)));
        k_init<<<1, kBlock, 0, ctx->stream>>>(reinterpret_cast<uint32_t*>(slot.ptr + l.stats),
                                              kStatWords * sizeof(unsigned long long) / sizeof(uint32_t));
        ctx->stats_ready = true;
        ctx->scratch_clean = false;                             // the zone is cleared before the selection starts
        ctx->n_st = n_st;
        ctx->n_chunks = n_ch;
        ctx->n_hblocks = n_hb;
        slot.numel = slot.k = -1;                               // until the step below has been enqueued
        slot.gdt = -1;
    }
    const int leader = static_cast<int>(step % n_learners);    // Alg. 1 line 6: CLT-k of learner mod(t, n)
    const scalecom_status st =
        grad_dtype == SCALECOM_GRAD_BF16
            ? launch_step<uint16_t>(ctx, lp, n_learners, 1, k, beta, lr, leader, idx_out, reduced_vals_out)
            : launch_step<float>(ctx, lp, n_learners, 1, k, beta, lr, leader, idx_out, reduced_vals_out);
    if (st != SCALECOM_OK) return static_fail(st, ctx->last_error);
    slot.numel = numel;
    slot.k = k;
    slot.gdt = static_cast<int>(grad_dtype);
    return SCALECOM_OK;
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
    k_apply_update<<<dim3(gx, gy), kBlock, 0, ctx->stream>>>(theta, numel, idx, vals, k, -scale);
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
    if (!scratch || reinterpret_cast<uintptr_t>(scratch) % 256)
        return fail(ctx, SCALECOM_EINVAL, "scratch must be 256-byte aligned");
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

scalecom_status scalecom_selection_stats(scalecom_ctx* ctx, uint64_t* counts_out, int reset)
{
    static_assert(SCALECOM_N_STATS <= kStatWords && SCALECOM_STAT_MISSED == kStatMissed &&
                      SCALECOM_STAT_NO_PREDICTION == kStatNoPrediction && SCALECOM_STAT_FULL_MODE == kStatFullMode &&
                      SCALECOM_STAT_WIDE_RANGE == kStatWideRange && SCALECOM_STAT_STEPS == kStatSteps,
                  "the header's indices are the kernels'");
    if (!ctx) return SCALECOM_EINVAL;
    ctx->last_error.clear();
    if (!counts_out) return fail(ctx, SCALECOM_EINVAL, "null argument");
    for (int j = 0; j < SCALECOM_N_STATS; ++j) counts_out[j] = 0;
    if (!ctx->stats_ready) return SCALECOM_OK;              // no step yet: the counters were never started
    DeviceGuard guard;
    SC_HIP(ctx, guard.enter(ctx->device));
    SC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    unsigned long long host[kStatWords];
    SC_HIP(ctx, hipMemcpy(host, ctx->ws + ctx->lay.stats, sizeof host, hipMemcpyDeviceToHost));
    for (int j = 0; j < SCALECOM_N_STATS; ++j) counts_out[j] = host[j];
    if (reset) {
        k_init<<<1, kBlock, 0, ctx->stream>>>(reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.stats),
                                              kStatWords * sizeof(unsigned long long) / sizeof(uint32_t));
        SC_HIP(ctx, hipGetLastError());
    }
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

const char* scalecom_last_error(const scalecom_ctx* ctx) { return ctx ? ctx->last_error.c_str() : g_static_error.c_str(); }

void scalecom_destroy(scalecom_ctx* ctx)
{
    if (!ctx) return;
    if (ctx->pinned || ctx->upload_done || ctx->side || !ctx->prof_events.empty()) {
        DeviceGuard guard;
        if (guard.enter(ctx->device) == hipSuccess) {
            (void)hipStreamSynchronize(ctx->stream);
            if (ctx->side) {
                (void)hipStreamSynchronize(ctx->side);
                (void)hipStreamDestroy(ctx->side);
            }
            if (ctx->fork_ev) (void)hipEventDestroy(ctx->fork_ev);
            if (ctx->join_ev) (void)hipEventDestroy(ctx->join_ev);
            if (ctx->upload_done) (void)hipEventDestroy(ctx->upload_done);
            for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
            if (ctx->pinned) (void)hipHostFree(ctx->pinned);
        }
    }
    delete ctx;
}

}  // extern "C"
