/*
 * scalecom.h -- C-ABI of the MI355X (gfx950) implementation of ScaleCom's per-step gradient
 * compression path: the cyclic local top-k compressor (CLT-k) with low-pass-filtered error
 * feedback (ScaleCom, arXiv 2104.11125, Algorithm 1 lines 6, 7 and 10; Eq. 2, 3, 5).
 *
 * n learners are simulated as n separate buffers on ONE GPU.  One call to scalecom_step
 * performs, for iteration `step`:
 *
 *   x_i   = mem_i + lr * grad_i                  for every learner i        (Alg. 1 line 6)
 *   I     = positions of the k largest |x_L|,    L = step mod n_learners    (Eq. 2, leader rule)
 *           ties ordered by position, lowest first; reported ascending
 *   v_i   = x_i restricted to I                  (CLT-k, Eq. 3)
 *   out   = sum_i v_i, added in the order i = 0, 1, ..., n-1   (Alg. 1 line 10 without 1/n)
 *   mem_i = (1-beta) * mem_i + beta * (x_i - CLT-k(x_i))       (Eq. 5, Alg. 1 line 7)
 *
 * All arithmetic is IEEE binary32: x = fma(lr, grad, mem); the update is
 * fma(beta, r, (1-beta)*mem) with r = 0 on I and r = x elsewhere.  bfloat16 gradients are
 * widened exactly.  |x| is compared on the bit pattern with the sign bit cleared, so the
 * index set is a pure function of the input bits (NaN patterns rank above infinity).
 *
 * Conventions
 *  - Pointers marked [device] are GPU global memory of the device given to scalecom_init;
 *    pointers marked [host] are ordinary process memory, read before the call returns.
 *  - The caller owns every buffer, including the workspace; the library allocates no
 *    device memory.  Per context it keeps pinned host staging for its tile tables
 *    (about numel_max / 256 + 140 * n_tensors_max + 64 KB bytes).
 *  - The workspace is the caller's allocation but the library's to use: from scalecom_init until
 *    scalecom_destroy it holds the library's tables, counters and threshold predictions, and
 *    the caller must neither write to it nor hand it to anything else.  What it holds never
 *    changes a result, but kernels follow the tables in it.
 *  - The result of a call depends only on its arguments.  The context remembers, per tensor
 *    (and per learner, for its turns as leader), where the threshold fell in earlier steps and
 *    uses it to skip a pass over the leader when the guess holds (checked exactly); this changes
 *    the time a step takes, never its result.
 *  - All work is enqueued on the HIP stream given to scalecom_init; calls do not wait for
 *    the GPU.  Outputs are valid once that stream has reached the end of the call's work.
 *    A context created with n_tensors_max > 1 also owns a second stream: inside a step one
 *    kernel is forked onto it and joined again with two events, so it never runs ahead of or
 *    behind the context's stream.  A context must not be used from two threads at once.
 *  - HIP graphs: once a layout (numel or offsets, k or ks or chunk sizes) has been used in one
 *    call, further steps with it enqueue kernels only (no copies or memsets, and no events or
 *    waits besides that fork and join, which a stream capture follows; scalecom_timing_begin
 *    must not be in effect), so they can be captured on the context's
 *    stream.  One thing is decided on the host when a step is enqueued and is therefore frozen
 *    in a graph: the leader (step mod n_learners).  A graph of one step may be replayed for every
 *    step with that leader; a graph of n_learners consecutive steps for every such cycle.
 *  - Errors are return codes; nothing is thrown.  scalecom_last_error gives the detail.
 */
#ifndef SCALECOM_H
#define SCALECOM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct scalecom_ctx scalecom_ctx; /* opaque */

typedef enum {
    SCALECOM_OK = 0,
    SCALECOM_EINVAL = 1,      /* an argument is outside what the header allows          */
    SCALECOM_ENOMEM = 2,      /* host allocation failed, or the workspace is too small  */
    SCALECOM_EHIP = 3,        /* a HIP runtime call failed (text in scalecom_last_error) */
    SCALECOM_EUNSUPPORTED = 4 /* the device is not a gfx950 GPU                          */
} scalecom_status;

typedef enum {
    SCALECOM_GRAD_F32 = 0, /* gradients are binary32                          */
    SCALECOM_GRAD_BF16 = 1 /* gradients are bfloat16 (upper half of binary32) */
} scalecom_grad_dtype;

/* Largest n_learners accepted (the paper scales to 64 learners, abstract and Table 3). */
#define SCALECOM_MAX_LEARNERS 64

/*
 * Bytes of device workspace needed for up to n_learners_max learners with vectors of up to
 * numel_max elements each, split into at most n_tensors_max segments (1 for whole-vector
 * use), with index sets of at most k_max positions in total per step.  Pure host arithmetic
 * (about 0.8 * numel_max + (4 * n_learners_max + 16) * k_max + 105 KB * n_tensors_max bytes).
 * Returns 0 if an argument is out of range (numel_max < 0 or > 2^31 - 1, n_tensors_max < 1,
 * n_learners_max outside 1 .. SCALECOM_MAX_LEARNERS, k_max < 0 or > numel_max).
 */
size_t scalecom_workspace_bytes(int64_t numel_max, int n_tensors_max, int n_learners_max, int64_t k_max);

/*
 * Create a context bound to one device and one stream.
 *   out             [host]   receives the context
 *   device                   HIP device ordinal
 *   hip_stream               hipStream_t on that device, as void* (NULL = the default stream)
 *   workspace       [device] at least scalecom_workspace_bytes(numel_max, n_tensors_max,
 *                            n_learners_max, k_max) bytes, 256-byte aligned; must outlive the
 *                            context and is the library's to use until scalecom_destroy (see
 *                            Conventions); need not be initialised
 *   n_learners_max           1 .. SCALECOM_MAX_LEARNERS
 *   k_max                    0 .. numel_max: largest k (sum of ks for scalecom_step_layers) used later
 *   grad_dtype               element type of every grad buffer passed later
 * EINVAL for bad arguments, ENOMEM for a short workspace, EHIP / EUNSUPPORTED for device trouble.
 */
scalecom_status scalecom_init(scalecom_ctx** out, int device, void* hip_stream, void* workspace,
                              size_t workspace_bytes, int n_learners_max, int64_t numel_max, int64_t k_max,
                              int n_tensors_max, scalecom_grad_dtype grad_dtype);

/*
 * One iteration over whole vectors (the operation stated at the top of this file).
 *   mem              [host] array of n_learners [device] pointers, each float[numel], 16-byte
 *                    aligned; read and overwritten in place (Eq. 5)
 *   grad             [host] array of n_learners [device] pointers, each numel gradients of the
 *                    context's grad_dtype, 16-byte aligned (8 for bfloat16); never written
 *   n_learners       1 .. n_learners_max
 *   numel            0 .. numel_max      (0: nothing is done)
 *   k                0 .. min(numel, k_max)   (0: the index set is empty, memories still updated)
 *   beta             0 < beta <= 1       (Eq. 5; beta = 1 is plain error feedback)
 *   lr               finite; multiplies the gradient before it is added to the memory
 *   step             >= 0; the leader is learner step mod n_learners
 *   idx_out          [device] int32[k]: the index set, ascending
 *   reduced_vals_out [device] float[k]: reduced_vals_out[t] = sum over learners of x_i[idx_out[t]]
 * Buffers must not overlap each other.  EINVAL if any rule above is broken.
 */
scalecom_status scalecom_step(scalecom_ctx* ctx, float* const* mem, const void* const* grad, int n_learners,
                              int64_t numel, int64_t k, float beta, float lr, int64_t step,
                              int32_t* idx_out, float* reduced_vals_out);

/*
 * scalecom_step for callers that cannot allocate device memory or pass a workspace along: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  No context and
 * no workspace argument: the scratch memory is a static device array inside the library
 * (about 8.5 MB, held by every GPU the library is used on until the process ends), which bounds
 * the sizes: numel <= SCALECOM_STATIC_NUMEL_MAX, n_learners <= SCALECOM_STATIC_LEARNERS_MAX,
 * k <= SCALECOM_STATIC_K_MAX; anything larger is EINVAL (the detail names the limit) and belongs
 * to scalecom_step.  The call allocates nothing, on the device or through any library: it looks up
 * the array's address once per device (first call), then only enqueues kernels on hip_stream.
 * Same operation, arithmetic and results as scalecom_step, bit for bit.
 *   device           HIP device ordinal (0 .. 63) that owns every buffer
 *   hip_stream       hipStream_t on that device, as void* (NULL = the default stream)
 *   grad_dtype       element type of the grad buffers of this call
 *   all other arguments as for scalecom_step
 * All calls on one GPU share that GPU's array, which also carries the threshold predictions
 * from one call to the next (they are dropped when numel, k or grad_dtype change): calls on one
 * GPU must not overlap -- enqueue them on one stream, or order the streams yourself -- or they
 * race.  The detail of a failure is scalecom_last_error(NULL) on the calling thread.
 */
#define SCALECOM_STATIC_NUMEL_MAX 4194304
#define SCALECOM_STATIC_LEARNERS_MAX 8
#define SCALECOM_STATIC_K_MAX 131072
scalecom_status scalecom_step_static(int device, void* hip_stream, float* const* mem, const void* const* grad,
                                     int n_learners, int64_t numel, int64_t k, float beta, float lr, int64_t step,
                                     scalecom_grad_dtype grad_dtype, int32_t* idx_out, float* reduced_vals_out);

/*
 * One iteration with a separate index set per tensor (per-layer compression rates, Sec. 4):
 * each learner's vector is cut into n_tensors consecutive segments
 * [offsets[s], offsets[s+1]), and segment s gets the ks[s] largest-magnitude positions of
 * the leader's x inside that segment.  The leader is the same for all segments of a step.
 *   offsets          [host] int64[n_tensors + 1], non-decreasing, offsets[0] >= 0,
 *                    offsets[n_tensors] <= numel_max; elements outside the segments are untouched
 *   ks               [host] int64[n_tensors], 0 <= ks[s] <= length of segment s, sum <= k_max
 *   idx_out          [device] int32[sum ks]: positions in the whole vector, segment after
 *                    segment, ascending inside a segment
 *   reduced_vals_out [device] float[sum ks], paired with idx_out
 * Other arguments as for scalecom_step; 1 <= n_tensors <= n_tensors_max.
 */
scalecom_status scalecom_step_layers(scalecom_ctx* ctx, float* const* mem, const void* const* grad,
                                     int n_learners, int n_tensors, const int64_t* offsets,
                                     const int64_t* ks, float beta, float lr, int64_t step,
                                     int32_t* idx_out, float* reduced_vals_out);

/*
 * One iteration over whole vectors with the chunk-wise selector of the paper's own implementation
 * (Sec. 4: the buffer is divided into chunks that are searched independently; App. E, Fig. A2:
 * one position per chunk) in place of the exact top-k: the leader's x is cut into consecutive
 * chunks of `chunk` elements (the last may be shorter) and each chunk contributes the position
 * of its largest |x|, the lowest position among equals.  Everything else -- leader rule, gather,
 * sum over learners, Eq. 5 -- is as in scalecom_step.  The index set has ceil(numel / chunk)
 * positions, which must not exceed the context's k_max.
 *   chunk            >= 1 (the compression rate; the paper uses 25 .. 400)
 *   idx_out          [device] int32[ceil(numel / chunk)], ascending: entry j lies in chunk j
 *   reduced_vals_out [device] float[ceil(numel / chunk)]
 * Other arguments and errors as for scalecom_step.
 */
scalecom_status scalecom_step_chunked(scalecom_ctx* ctx, float* const* mem, const void* const* grad, int n_learners,
                                      int64_t numel, int64_t chunk, float beta, float lr, int64_t step,
                                      int32_t* idx_out, float* reduced_vals_out);

/*
 * The chunk-wise selector with a chunk size per tensor: the paper compresses layer by layer, each
 * at its own rate (Sec. 4), with the selector of scalecom_step_chunked.  Segment s is cut into
 * chunks of chunks[s] elements counted from offsets[s] (its last chunk may be shorter) and
 * contributes one position per chunk, ceil(length_s / chunks[s]) positions; an empty segment
 * contributes none.  Segments follow each other in the outputs as in scalecom_step_layers.
 *   chunks           [host] int64[n_tensors], each >= 1 (scalecom_layer_ks' rates_out can be passed)
 *   idx_out          [device] int32[sum of ceil(length_s / chunks[s])], ascending
 *   reduced_vals_out [device] float[same], paired with idx_out
 * The number of positions must not exceed the context's k_max.  Other arguments and errors as for
 * scalecom_step_layers.
 */
scalecom_status scalecom_step_layers_chunked(scalecom_ctx* ctx, float* const* mem, const void* const* grad,
                                             int n_learners, int n_tensors, const int64_t* offsets,
                                             const int64_t* chunks, float beta, float lr, int64_t step,
                                             int32_t* idx_out, float* reduced_vals_out);

/*
 * Weight update on the index set (Alg. 1 lines 10 and 12): theta[idx[t]] -= scale * vals[t] for
 * t < k, one rounding per entry (fma(-scale, vals[t], theta[idx[t]])).  With the outputs of a
 * step, scale = 1 / n_learners applies the averaged compressed gradient when lr was the step
 * size, and scale = alpha / n_learners when lr was 1.  Enqueued on the context's stream, so it
 * may directly follow the step that produced idx and vals.
 *   theta   [device] float[numel], updated in place at the k positions only
 *   idx     [device] int32[k], distinct positions in [0, numel); an entry outside that range is
 *           skipped (no memory is touched for it)
 *   vals    [device] float[k]
 *   scale   finite
 * EINVAL for null pointers (when k > 0), k < 0, numel < 0 or non-finite scale.
 */
scalecom_status scalecom_apply_update(scalecom_ctx* ctx, float* theta, int64_t numel, const int32_t* idx,
                                      const float* vals, int64_t k, float scale);

/*
 * Similarity diagnostic of Sec. 3 (Eq. 6, Fig. 3): per tensor, the Hamming distance d between the
 * index set CLT-k would use at `step` (the top-k of the leader's x = fma(lr, grad, mem), Eq. 3)
 * and the "true top-k", the top-k of the all-reduced error-feedback gradient sum_i x_i (summed
 * over learners 0..n-1 left to right in fp32; the 1/n of the mean does not change the set).  Both
 * sets have ks[s] members, the binarised vectors of Eq. 6 differ in 2 d places, and
 * d_out[s] = ks[s] - |intersection| (the paper plots d / k).  Same tie rule as scalecom_step.
 * Reads mem and grad, modifies neither.  The threshold predictions that scalecom_step_layers keeps
 * for a layout survive a call with the same offsets and ks; a call with other offsets or ks is
 * a change of layout like any other, after which the next step starts without predictions (its
 * result is the same, it takes two more passes over the leader).
 *   mem, grad, n_learners, n_tensors, offsets, ks, lr, step: as for scalecom_step_layers
 *   scratch       [device] at least scalecom_hamming_scratch_bytes(numel_max, n_tensors_max) bytes
 *                 (the context's maxima), 256-byte aligned, caller-owned, contents undefined afterwards
 *   d_out         [device] int32[n_tensors]
 * Asynchronous on the context's stream.  EINVAL / ENOMEM as for scalecom_step_layers, plus ENOMEM
 * for a scratch that is too small.
 */
size_t scalecom_hamming_scratch_bytes(int64_t numel_max, int n_tensors_max);
scalecom_status scalecom_hamming_distance(scalecom_ctx* ctx, float* const* mem, const void* const* grad, int n_learners,
                                          int n_tensors, const int64_t* offsets, const int64_t* ks, float lr,
                                          int64_t step, void* scratch, size_t scratch_bytes, int32_t* d_out);

/*
 * Cosine distance 1 - a.b / (|a| |b|) of two fp32 vectors (Sec. 2 measures the similarity of two
 * learners' memories with it), accumulated in binary64.
 *   a, b   [device] float[numel]
 *   out    [device] double[4], 8-byte aligned: out[0] the distance, out[1..3] = a.b, a.a, b.b
 * The order of the partial sums is not fixed: results agree to a few ulp of binary64 between
 * runs.  A zero vector gives NaN.  Asynchronous on the context's stream.
 */
scalecom_status scalecom_cosine_distance(scalecom_ctx* ctx, const float* a, const float* b, int64_t numel, double* out);

/*
 * Per-layer sizes of the index sets from the paper's rate guidance (Sec. 4): a layer whose
 * FLOPs-per-gradient ratio is >= 196 is compressed 25X, one in [128, 196) 50X, one below 128
 * 400X; ks_out[s] = ceil(sizes[s] / rate), ready for scalecom_step_layers.  A layer marked as
 * uncompressed (App. E keeps the first convolution out of compression, Sec. 4 every layer during
 * the warm-up epochs) gets rate 1, k = its size: scalecom_step_layers then sums all of its
 * elements over the learners and leaves (1 - beta) * mem behind.  Pure host arithmetic.
 *   flops_per_gradient [host] double[n_tensors], each > 0
 *   sizes              [host] int64[n_tensors], each >= 0
 *   uncompressed       [host] uint8[n_tensors] (non-zero: not compressed) or NULL: none
 *   ks_out             [host] int64[n_tensors]
 *   rates_out          [host] int64[n_tensors] or NULL: the rate chosen per layer
 * EINVAL for null pointers, n_tensors < 0, a ratio that is not > 0, or a negative size.
 */
scalecom_status scalecom_layer_ks(int n_tensors, const double* flops_per_gradient, const int64_t* sizes,
                                  const uint8_t* uncompressed, int64_t* ks_out, int64_t* rates_out);

/*
 * How often the exact selection could not finish on its single pass over the leader, counted on
 * the device since scalecom_init (or the last reset) over the (step, tensor) pairs with a
 * non-empty index set and a tensor of more than 8192 elements.  The single pass works on a range
 * of magnitudes around the threshold that the context expects from earlier steps; the counts tell
 * how often that held.  Results never depend on it, step times do.  Diagnostic: waits for the
 * context's stream, then copies the counters to the host; nothing in scalecom_step* waits.
 *   counts_out [host] uint64[SCALECOM_N_STATS]:
 *     [SCALECOM_STAT_MISSED]        the threshold fell outside the expected range: two more passes
 *                                   over the leader's vector in that step
 *     [SCALECOM_STAT_NO_PREDICTION] nothing was expected yet (first step of a layout): same cost
 *     [SCALECOM_STAT_FULL_MODE]     so many equal or clustered magnitudes at the threshold that the
 *                                   last two search levels were passes over the leader's vector too
 *     [SCALECOM_STAT_WIDE_RANGE]    the range was wider than 2^19 magnitudes and held the threshold:
 *                                   one more pass over the listed magnitudes, none over the vector
 *     [SCALECOM_STAT_STEPS]         calls of scalecom_step / scalecom_step_layers counted
 *   reset      non-zero: the counters start again from zero after this call
 */
#define SCALECOM_N_STATS 5
#define SCALECOM_STAT_MISSED 0
#define SCALECOM_STAT_NO_PREDICTION 1
#define SCALECOM_STAT_FULL_MODE 2
#define SCALECOM_STAT_WIDE_RANGE 3
#define SCALECOM_STAT_STEPS 4
scalecom_status scalecom_selection_stats(scalecom_ctx* ctx, uint64_t* counts_out, int reset);

/*
 * Optional per-phase GPU timing, for benchmarks.  Not part of the paper's method: it only
 * records HIP events on the context's stream between the kernel groups of a step.
 * Phases of one step, in order:
 *   0  first look at the leader (Eq. 2): single predicted pass, or histogram of the top 12 bits
 *      of the magnitude keys, + search of the threshold bucket
 *   1  remaining 19 key bits resolved (on the candidate list; a second pass over the leader makes
 *      that list when the prediction missed): exact threshold and tie quota
 *   2  per-tile member counts, prefix sums, output slot of every tile, ties resolved
 *   3  all-learner pass: accumulate, low-pass memory update, members' values staged (Eq. 3, 5)
 *   4  sum of the staged values over learners (Alg. 1 line 10)
 *
 * scalecom_timing_begin: of the following calls of scalecom_step* on this context, every
 * `every`-th (the first, the (every + 1)-th, ...; every >= 1) records phase boundaries, until
 * max_steps (0 .. 4096) calls have been recorded.  With all_phases = 0 only the two boundaries of
 * phase 3, the dominant kernel, are recorded; with all_phases != 0 all six.  An event costs the
 * stream a few microseconds, so a throughput measurement should record two boundaries on a
 * sample of its steps.  scalecom_timing_read: waits for the stream, writes
 * phase_ms[t * SCALECOM_N_PHASES + p] = milliseconds of phase p of recorded step t (0 for phases
 * that were not recorded) for at most capacity_steps steps, stores the number of steps written in
 * *n_steps_out, and stops recording.
 *   phase_ms     [host] float[capacity_steps * SCALECOM_N_PHASES]
 *   n_steps_out  [host]
 */
#define SCALECOM_N_PHASES 5
scalecom_status scalecom_timing_begin(scalecom_ctx* ctx, int max_steps, int all_phases, int every);
scalecom_status scalecom_timing_read(scalecom_ctx* ctx, float* phase_ms, int capacity_steps, int* n_steps_out);

/*
 * Measurement aid, not part of the paper's method: copy `bytes` bytes from src to dst
 * [device, 16-byte aligned, bytes a multiple of 16, not overlapping] with a plain streaming
 * kernel on the context's stream.  Its bandwidth is the practical ceiling the other kernels
 * are compared with, and its known traffic calibrates the profiler's byte counters.
 */
scalecom_status scalecom_stream_copy(scalecom_ctx* ctx, void* dst, const void* src, size_t bytes);

/* Static text for a status code. */
const char* scalecom_strerror(scalecom_status status);

/* Detail of the last failure on this context ("" if none); valid until the next call on it.
 * With NULL: of the calling thread's last scalecom_step_static. */
const char* scalecom_last_error(const scalecom_ctx* ctx);

/* Waits for the context's stream, frees the context's host memory.  NULL is allowed. */
void scalecom_destroy(scalecom_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* SCALECOM_H */
