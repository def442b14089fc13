// CPU oracle for ScaleCom's per-step compression path (CLT-k with low-pass-filtered error
// feedback).  TEST INFRASTRUCTURE ONLY: it exists so that the GPU library can be checked
// against a plain, slow, single-threaded statement of what the paper's method computes.
// Nothing in the product path may call it, and it shares no code with the HIP kernels.
//
// Every function below is a direct statement of one step of Algorithm 1 of the paper
// (ScaleCom, arXiv 2104.11125), with the floating-point evaluation order fixed so that an
// independent implementation can reproduce the selected index set bit for bit:
//
//   accumulate      x_i = m_i + lr * grad_i             Alg. 1 line 6 (argument of CLT-k), Sec. 2 footnote
//   top-k index set I^k(x_L), L = step mod n            Eq. 2, leader rule of Alg. 1 line 6
//   (or one position per chunk of the leader's vector   Sec. 4, App. E: chunk-wise selection)
//   CLT-k gather    (g_i)_j = (x_i)_j for j in I        Eq. 3
//   reduction       g = sum_i g_i (the 1/n is left out) Alg. 1 line 10, Eq. 1
//   memory update   m_i <- (1-b) m_i + b (x_i - g_i)    Eq. 5, Alg. 1 line 7
//
// Arithmetic is IEEE binary32 throughout because membership of the index set is decided by
// comparing binary32 magnitudes; both sides of a parity test must take that decision in the
// same precision.  The only fused operations are the two written as std::fmaf; the file is
// compiled with -ffp-contract=off so the compiler adds none.
//
// Parity pins: every function here is pinned by tests that do not call it to produce their
// expected value (hand-worked examples built from Eq. 2/3/5, brute-force sorting in Python,
// float64 closed forms, the beta = 1 special case, the telescoping identity of Appendix C).
// Nothing in this file is "parity unpinned".

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <iterator>
#include <vector>

namespace {

enum { GRAD_F32 = 0, GRAD_BF16 = 1 };

// bfloat16 is the upper half of a binary32 pattern, so widening is exact.
inline float widen_bf16(uint16_t h)
{
    uint32_t bits = static_cast<uint32_t>(h) << 16;
    float f;
    std::memcpy(&f, &bits, sizeof f);
    return f;
}

inline float grad_at(const void* grad, int grad_dtype, int64_t j)
{
    if (grad_dtype == GRAD_BF16) return widen_bf16(static_cast<const uint16_t*>(grad)[j]);
    return static_cast<const float*>(grad)[j];
}

// Magnitude of a binary32 value as an unsigned integer: dropping the sign bit of the
// pattern is monotone in |x| for every finite value and infinity, makes +0 and -0 equal,
// and gives NaN patterns a fixed (largest) rank.
inline uint32_t magnitude_key(float x)
{
    uint32_t bits;
    std::memcpy(&bits, &x, sizeof bits);
    return bits & 0x7fffffffu;
}

}  // namespace

extern "C" {

// x = m + lr * grad for one learner (Alg. 1 line 6; "error-feedback gradient" = memory plus
// the newly computed gradient).  One rounding: fmaf(lr, grad, m).
int oracle_accumulate(const float* mem, const void* grad, int grad_dtype, int64_t numel, float lr,
                      float* acc)
{
    if (numel < 0 || (numel > 0 && (!mem || !grad || !acc))) return 1;
    for (int64_t j = 0; j < numel; ++j) acc[j] = std::fmaf(lr, grad_at(grad, grad_dtype, j), mem[j]);
    return 0;
}

// I^k(x) by the plain definition (Eq. 2): order all positions by magnitude, largest first,
// equal magnitudes by position, smallest first; keep the first k; report them in ascending
// position.  Eq. 2 alone admits more than k members when magnitudes tie at the cut; the
// position rule picks exactly k of them.
int oracle_topk_sort(const float* x, int64_t numel, int64_t k, int32_t* idx_out)
{
    if (numel < 0 || k < 0 || k > numel || numel > INT32_MAX) return 1;
    std::vector<int32_t> order(static_cast<size_t>(numel));
    for (int64_t j = 0; j < numel; ++j) order[j] = static_cast<int32_t>(j);
    std::sort(order.begin(), order.end(), [x](int32_t a, int32_t b) {
        const uint32_t ka = magnitude_key(x[a]), kb = magnitude_key(x[b]);
        if (ka != kb) return ka > kb;
        return a < b;
    });
    std::sort(order.begin(), order.begin() + k);
    for (int64_t t = 0; t < k; ++t) idx_out[t] = order[t];
    return 0;
}

// The same set, without sorting everything: each position becomes one 64-bit word
// (magnitude in the high half, complemented position in the low half), so that "larger
// word" means "larger magnitude, or equal magnitude and smaller position"; a selection
// (std::nth_element) puts the k largest words in front.
int oracle_topk_select(const float* x, int64_t numel, int64_t k, int32_t* idx_out)
{
    if (numel < 0 || k < 0 || k > numel || numel > INT32_MAX) return 1;
    if (k == 0) return 0;
    std::vector<uint64_t> word(static_cast<size_t>(numel));
    for (int64_t j = 0; j < numel; ++j)
        word[j] = (static_cast<uint64_t>(magnitude_key(x[j])) << 32) |
                  static_cast<uint64_t>(0xffffffffu - static_cast<uint32_t>(j));
    if (k < numel) std::nth_element(word.begin(), word.begin() + k, word.end(), std::greater<uint64_t>());
    for (int64_t t = 0; t < k; ++t)
        idx_out[t] = static_cast<int32_t>(0xffffffffu - static_cast<uint32_t>(word[t] & 0xffffffffu));
    std::sort(idx_out, idx_out + k);
    return 0;
}

// Chunk-wise selection, the selector the paper's own implementation used in place of an exact
// top-k (Sec. 4 "divides the whole buffer into chunks", App. E "chunk-wise quasi-sorting", demo of
// Fig. A2: 8 values, two chunks, one position chosen in each): the vector is cut into consecutive
// chunks of `chunk` elements (the last may be shorter) and each chunk contributes the position
// of its largest magnitude, the lowest position among equals.  ceil(numel / chunk) positions,
// ascending.
int oracle_chunk_select(const float* x, int64_t numel, int64_t chunk, int32_t* idx_out)
{
    if (numel < 0 || chunk < 1 || numel > INT32_MAX) return 1;
    int64_t t = 0;
    for (int64_t start = 0; start < numel; start += chunk, ++t) {
        const int64_t stop = std::min(start + chunk, numel);
        int64_t best = start;
        for (int64_t j = start + 1; j < stop; ++j)
            if (magnitude_key(x[j]) > magnitude_key(x[best])) best = j;
        idx_out[t] = static_cast<int32_t>(best);
    }
    return 0;
}

// Non-zero entries of CLT^k_L(x_i): the learner's own values at the leader's positions (Eq. 3).
int oracle_gather(const float* acc, const int32_t* idx, int64_t k, float* vals)
{
    for (int64_t t = 0; t < k; ++t) vals[t] = acc[idx[t]];
    return 0;
}

// Reduction over learners of the sparsified vectors (Alg. 1 line 10 without the 1/n):
// learner 0 first, then 1, 2, ... added one at a time.
int oracle_reduce(const float* const* vals, int n_learners, int64_t k, float* reduced)
{
    if (n_learners < 1) return 1;
    for (int64_t t = 0; t < k; ++t) {
        float s = vals[0][t];
        for (int i = 1; i < n_learners; ++i) s = s + vals[i][t];
        reduced[t] = s;
    }
    return 0;
}

// Eq. 5: m <- (1-beta) m + beta (x - g), where g = CLT-k of x, i.e. x on the index set and 0
// elsewhere.  The residual x - g is x off the set and exactly 0 on it (taken as 0 also when
// x is not finite, so a selected entry is always fully removed).
int oracle_memory_update(float* mem, const float* acc, const int32_t* idx, int64_t k, int64_t numel,
                         float beta)
{
    std::vector<uint8_t> in_set(static_cast<size_t>(numel), 0);
    for (int64_t t = 0; t < k; ++t) {
        if (idx[t] < 0 || idx[t] >= numel) return 1;
        in_set[idx[t]] = 1;
    }
    const float one_minus_beta = 1.0f - beta;
    for (int64_t j = 0; j < numel; ++j) {
        const float residual = in_set[j] ? 0.0f : acc[j];
        const float kept = one_minus_beta * mem[j];
        mem[j] = std::fmaf(beta, residual, kept);
    }
    return 0;
}

// Weight update of Alg. 1 lines 10 and 12 on the index set: theta[idx[t]] -= scale * reduced[t],
// with scale = alpha / n when `reduced` is the plain sum of the learners' values (line 10 divides
// by n, line 12 multiplies by alpha), or 1 / n when the step size was already applied in the
// accumulate.  One rounding per entry: fmaf(-scale, reduced, theta).
int oracle_apply_update(float* theta, int64_t numel, const int32_t* idx, const float* reduced, int64_t k, float scale)
{
    for (int64_t t = 0; t < k; ++t) {
        if (idx[t] < 0 || idx[t] >= numel) return 1;
        theta[idx[t]] = std::fmaf(-scale, reduced[t], theta[idx[t]]);
    }
    return 0;
}

// Compression rate of a layer from its FLOPs-per-gradient ratio (Sec. 4, "conservative engineering
// guidance"): 25X for a ratio in [196, inf), 50X for [128, 196), 400X for (0, 128).
int64_t oracle_layer_rate(double flops_per_gradient)
{
    if (flops_per_gradient >= 196.0) return 25;
    if (flops_per_gradient >= 128.0) return 50;
    return 400;
}

// Similarity diagnostics of Sec. 3.  Hamming distance between the leader's index set and the
// "true top-k", the top-k of the all-reduced error-feedback gradient y = sum_i x_i (Lemma 1 takes
// the mean; the positive factor 1/n does not change the set): both sets have k members, the
// binarised vectors of Eq. 6 differ in 2d places, and d = k - |intersection| is returned
// (Fig. 3 plots d / k).  Nothing is modified.
int64_t oracle_hamming_distance(const float* const* mem, const void* const* grad, int grad_dtype, int n_learners,
                                int64_t numel, int64_t k, float lr, int64_t step)
{
    if (n_learners < 1 || numel < 0 || k < 0 || k > numel || step < 0) return -1;
    const int leader = static_cast<int>(step % n_learners);
    std::vector<float> acc(static_cast<size_t>(numel)), y(static_cast<size_t>(numel)), xl(static_cast<size_t>(numel));
    for (int i = 0; i < n_learners; ++i) {
        oracle_accumulate(mem[i], grad[i], grad_dtype, numel, lr, acc.data());
        if (i == leader) xl = acc;
        for (int64_t j = 0; j < numel; ++j) y[j] = i == 0 ? acc[j] : y[j] + acc[j];
    }
    std::vector<int32_t> a(static_cast<size_t>(k)), b(static_cast<size_t>(k));
    if (oracle_topk_select(xl.data(), numel, k, a.data()) || oracle_topk_select(y.data(), numel, k, b.data())) return -1;
    std::vector<int32_t> both;
    std::set_intersection(a.begin(), a.end(), b.begin(), b.end(), std::back_inserter(both));
    return k - static_cast<int64_t>(both.size());
}

// Cosine distance 1 - a.b / (|a| |b|) of two vectors (footnote of Sec. 2: similarity of two
// learners' memories), accumulated in binary64.
double oracle_cosine_distance(const float* a, const float* b, int64_t numel)
{
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int64_t j = 0; j < numel; ++j) {
        ab += static_cast<double>(a[j]) * static_cast<double>(b[j]);
        aa += static_cast<double>(a[j]) * static_cast<double>(a[j]);
        bb += static_cast<double>(b[j]) * static_cast<double>(b[j]);
    }
    return 1.0 - ab / (std::sqrt(aa) * std::sqrt(bb));
}

// One iteration of Alg. 1 lines 6, 7 and 10 for n learners whose vectors are split into
// n_tensors consecutive segments [offsets[s], offsets[s+1]); the index set of each segment
// is chosen inside that segment with its own k (per-layer compression, Sec. 4) by the same
// leader L = step mod n.  idx_out receives positions in the whole vector, segment after
// segment, ascending inside a segment; reduced_out pairs with it.  mem is updated in place.
int oracle_step_layers(float* const* mem, const void* const* grad, int grad_dtype, int n_learners,
                       int n_tensors, const int64_t* offsets, const int64_t* ks, float beta, float lr,
                       int64_t step, int32_t* idx_out, float* reduced_out)
{
    if (n_learners < 1 || n_tensors < 0 || step < 0) return 1;
    if (!(beta > 0.0f && beta <= 1.0f)) return 1;
    const int leader = static_cast<int>(step % n_learners);
    int64_t out = 0;
    for (int s = 0; s < n_tensors; ++s) {
        const int64_t begin = offsets[s], len = offsets[s + 1] - offsets[s], k = ks[s];
        if (len < 0 || k < 0 || k > len) return 1;
        std::vector<float> acc(static_cast<size_t>(len));
        std::vector<int32_t> local(static_cast<size_t>(k));
        const size_t gsz = grad_dtype == GRAD_BF16 ? 2 : 4;

        // leader: accumulate, then its own top-k positions
        oracle_accumulate(mem[leader] + begin, static_cast<const char*>(grad[leader]) + gsz * begin,
                          grad_dtype, len, lr, acc.data());
        if (oracle_topk_select(acc.data(), len, k, local.data())) return 1;

        // every learner: accumulate, keep its values on the leader's set, update its memory
        std::vector<std::vector<float>> vals(static_cast<size_t>(n_learners));
        std::vector<const float*> vptr(static_cast<size_t>(n_learners));
        for (int i = 0; i < n_learners; ++i) {
            oracle_accumulate(mem[i] + begin, static_cast<const char*>(grad[i]) + gsz * begin, grad_dtype,
                              len, lr, acc.data());
            vals[i].resize(static_cast<size_t>(k));
            oracle_gather(acc.data(), local.data(), k, vals[i].data());
            if (oracle_memory_update(mem[i] + begin, acc.data(), local.data(), k, len, beta)) return 1;
            vptr[i] = vals[i].data();
        }
        oracle_reduce(vptr.data(), n_learners, k, reduced_out + out);
        for (int64_t t = 0; t < k; ++t) idx_out[out + t] = static_cast<int32_t>(begin + local[t]);
        out += k;
    }
    return 0;
}

// One iteration with the chunk-wise selector on the leader instead of the exact top-k; everything
// else (leader rule, Eq. 3 gather, reduction, Eq. 5 memory update) as in oracle_step_layers.
int oracle_step_chunked(float* const* mem, const void* const* grad, int grad_dtype, int n_learners, int64_t numel,
                        int64_t chunk, float beta, float lr, int64_t step, int32_t* idx_out, float* reduced_out)
{
    if (n_learners < 1 || numel < 0 || chunk < 1 || step < 0) return 1;
    if (!(beta > 0.0f && beta <= 1.0f)) return 1;
    const int leader = static_cast<int>(step % n_learners);
    const int64_t k = (numel + chunk - 1) / chunk;
    std::vector<float> acc(static_cast<size_t>(numel));
    oracle_accumulate(mem[leader], grad[leader], grad_dtype, numel, lr, acc.data());
    if (oracle_chunk_select(acc.data(), numel, chunk, idx_out)) return 1;
    std::vector<std::vector<float>> vals(static_cast<size_t>(n_learners));
    std::vector<const float*> vptr(static_cast<size_t>(n_learners));
    for (int i = 0; i < n_learners; ++i) {
        oracle_accumulate(mem[i], grad[i], grad_dtype, numel, lr, acc.data());
        vals[i].resize(static_cast<size_t>(k));
        oracle_gather(acc.data(), idx_out, k, vals[i].data());
        if (oracle_memory_update(mem[i], acc.data(), idx_out, k, numel, beta)) return 1;
        vptr[i] = vals[i].data();
    }
    if (k > 0) oracle_reduce(vptr.data(), n_learners, k, reduced_out);
    return 0;
}

// The same with a separate chunk size per segment (the paper compresses layer by layer, each at
// its own rate, Sec. 4): segment s contributes one position per chunk of chunks[s] consecutive
// elements counted from the segment's start, ceil(len_s / chunks[s]) positions, in the order of the
// chunks; segments follow each other in idx_out as in oracle_step_layers.  A segment of length 0
// contributes nothing.
int oracle_step_layers_chunked(float* const* mem, const void* const* grad, int grad_dtype, int n_learners,
                               int n_tensors, const int64_t* offsets, const int64_t* chunks, float beta, float lr,
                               int64_t step, int32_t* idx_out, float* reduced_out)
{
    if (n_learners < 1 || n_tensors < 0 || step < 0) return 1;
    if (!(beta > 0.0f && beta <= 1.0f)) return 1;
    const size_t gsz = grad_dtype == GRAD_BF16 ? 2 : 4;
    std::vector<float*> m(static_cast<size_t>(n_learners));
    std::vector<const void*> g(static_cast<size_t>(n_learners));
    int64_t out = 0;
    for (int s = 0; s < n_tensors; ++s) {
        const int64_t begin = offsets[s], len = offsets[s + 1] - offsets[s];
        if (len < 0 || chunks[s] < 1) return 1;
        if (len == 0) continue;
        const int64_t k = (len + chunks[s] - 1) / chunks[s];
        for (int i = 0; i < n_learners; ++i) {
            m[i] = mem[i] + begin;
            g[i] = static_cast<const char*>(grad[i]) + gsz * begin;
        }
        // the segment on its own is the whole-vector case; its positions are then shifted by begin
        if (oracle_step_chunked(m.data(), g.data(), grad_dtype, n_learners, len, chunks[s], beta, lr, step,
                                idx_out + out, reduced_out + out))
            return 1;
        for (int64_t t = 0; t < k; ++t) idx_out[out + t] += static_cast<int32_t>(begin);
        out += k;
    }
    return 0;
}

// Whole-vector form: one segment covering everything.
int oracle_step(float* const* mem, const void* const* grad, int grad_dtype, int n_learners, int64_t numel,
                int64_t k, float beta, float lr, int64_t step, int32_t* idx_out, float* reduced_out)
{
    const int64_t offsets[2] = {0, numel};
    return oracle_step_layers(mem, grad, grad_dtype, n_learners, 1, offsets, &k, beta, lr, step, idx_out,
                              reduced_out);
}

}  // extern "C"
