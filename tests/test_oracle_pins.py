"""Pins for the CPU oracle: each test derives its expected value from the paper's equations,
from brute force, from float64 / exact rational arithmetic or from a library routine --
never from the oracle itself.  All of them run without a GPU."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from helpers import (bf16_bits_from_f32, bf16_bits_to_f32, brute_topk, load_golden, mag_key,
                     round_fraction_to_f32)


def f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


# ---------------------------------------------------------------- hand-worked examples (Eq. 2, 3, 5)
@pytest.mark.parametrize("name", ["e1_step0.txt", "e2_step1.txt", "e3_lr.txt"])
def test_hand_worked_examples(golden_dir, name):
    g = load_golden(os.path.join(golden_dir, name))
    mem = [f32(g["mem_0"]), f32(g["mem_1"])]
    grad = [f32(g["grad_0"]), f32(g["grad_1"])]
    idx, red = oracle.step(mem, grad, g["k"], g["beta"], g["lr"], g["step"])
    assert idx.tolist() == g["idx"].astype(int).tolist()
    assert red.tolist() == g["reduced"].tolist()
    assert mem[0].tolist() == g["mem_0_out"].tolist()
    assert mem[1].tolist() == g["mem_1_out"].tolist()


def test_hand_worked_example_beta_one(golden_dir):
    g = load_golden(os.path.join(golden_dir, "e1_step0.txt"))
    mem = [f32(g["mem_0"]), f32(g["mem_1"])]
    grad = [f32(g["grad_0"]), f32(g["grad_1"])]
    idx, red = oracle.step(mem, grad, g["k"], 1.0, g["lr"], g["step"])
    assert idx.tolist() == [1, 4] and red.tolist() == [-7.0, -5.0]
    assert mem[0].tolist() == g["mem_0_out_beta1"].tolist()
    assert mem[1].tolist() == g["mem_1_out_beta1"].tolist()


def test_two_examples_chain(golden_dir):
    """Running e1 then e2 on carried memory gives e2's result (memory is the only state)."""
    g1 = load_golden(os.path.join(golden_dir, "e1_step0.txt"))
    g2 = load_golden(os.path.join(golden_dir, "e2_step1.txt"))
    mem = [f32(g1["mem_0"]), f32(g1["mem_1"])]
    oracle.step(mem, [f32(g1["grad_0"]), f32(g1["grad_1"])], 2, 0.5, 1.0, 0)
    idx, red = oracle.step(mem, [f32(g2["grad_0"]), f32(g2["grad_1"])], 2, 0.5, 1.0, 1)
    assert idx.tolist() == [3, 4] and red.tolist() == [3.25, 3.0]
    assert mem[0].tolist() == g2["mem_0_out"].tolist() and mem[1].tolist() == g2["mem_1_out"].tolist()


# ---------------------------------------------------------------- top-k index set (Eq. 2)
def _adversarial_vectors(rng):
    yield f32([0.0])
    yield f32([-0.0, 0.0, -0.0, 0.0])
    yield f32([1.0] * 17)
    yield f32([1.0, -1.0] * 9)
    yield f32([2.0, 1.0] * 8 + [2.0])
    yield f32([0.0] * 10 + [1e-45, -1e-45] + [0.0] * 5)              # denormals beat zeros
    yield f32([np.inf, -np.inf, 3.0e38, 1.0, np.nan, -2.0])           # non-finite: order by bit pattern
    for n in (1, 2, 3, 7, 8, 31, 64):
        yield f32(rng.choice([-2.0, -1.0, -0.5, 0.0, 0.5, 1.0, 2.0], size=n))   # heavy ties
        yield f32(rng.standard_normal(n))
        yield f32(rng.standard_normal(n) * 10.0 ** rng.integers(-30, 30, size=n))  # wide exponent range


def test_topk_matches_brute_force_all_k():
    rng = np.random.default_rng(20201)
    for x in _adversarial_vectors(rng):
        for k in range(0, x.size + 1):
            want = brute_topk(x, k)
            assert oracle.topk_sort(x, k).tolist() == want.tolist(), (x, k)
            assert oracle.topk_select(x, k).tolist() == want.tolist(), (x, k)


def test_topk_select_matches_library_argsort():
    """Against NumPy's stable argsort of -|x| (a different routine from the oracle's)."""
    rng = np.random.default_rng(7)
    for n, k in ((1000, 10), (65_537, 655), (200_000, 1786), (200_000, 200_000), (200_000, 1)):
        x = f32(rng.standard_normal(n) * 1e-3)
        x[rng.integers(0, n, size=n // 50)] = x[0]          # plant equal magnitudes
        x[rng.integers(0, n, size=n // 50)] = -x[0]
        want = np.sort(np.argsort(-np.abs(x.astype(np.float64)), kind="stable")[:k])
        got = oracle.topk_select(x, k)
        assert np.array_equal(got, want.astype(np.int32))
        if n <= 70_000:
            assert np.array_equal(oracle.topk_sort(x, k), got)


def test_topk_tie_straddling_cut_takes_lowest_positions():
    x = f32([5, 3, 3, 3, 3, 1])
    assert oracle.topk_select(x, 3).tolist() == [0, 1, 2]
    x = f32([1, -3, 3, 5, -3, 3])
    assert oracle.topk_select(x, 3).tolist() == [1, 2, 3]


def test_topk_energy_is_maximal_over_all_subsets():
    """Top-k keeps the most energy of any k-subset (contraction property, Sec. 3 / Lemma 1)."""
    rng = np.random.default_rng(3)
    x = f32(rng.standard_normal(9))
    for k in (1, 3, 5):
        sel = oracle.topk_select(x, k)
        best = max(sum(float(x[j]) ** 2 for j in c) for c in itertools.combinations(range(9), k))
        assert sum(float(x[j]) ** 2 for j in sel) == pytest.approx(best, rel=1e-12)


def test_topk_contraction_no_worse_than_random_k():
    rng = np.random.default_rng(4)
    x = f32(rng.standard_normal(50_000))
    k = 500
    sel = oracle.topk_select(x, k)
    e_sel = float(np.sum(x[sel].astype(np.float64) ** 2))
    e_all = float(np.sum(x.astype(np.float64) ** 2))
    assert e_all - e_sel <= (1.0 - k / x.size) * e_all


# ---------------------------------------------------------------- accumulate (Alg. 1 line 6)
def test_accumulate_is_single_rounding_of_exact_value():
    rng = np.random.default_rng(11)
    m = f32(rng.standard_normal(300))
    g = f32(rng.standard_normal(300) * 3.0)
    lr = np.float32(0.1)
    acc = oracle.accumulate(m, g, float(lr))
    two_roundings_differ = 0
    for j in range(m.size):
        exact = Fraction(float(m[j])) + Fraction(float(lr)) * Fraction(float(g[j]))
        assert acc[j] == round_fraction_to_f32(exact), j
        two_roundings_differ += acc[j] != np.float32(np.float32(lr * g[j]) + m[j])
    assert two_roundings_differ > 0      # the sample does tell fused from unfused evaluation


def test_accumulate_lr_one_is_plain_sum_and_zero_memory_is_scaling():
    rng = np.random.default_rng(12)
    m, g = f32(rng.standard_normal(1000)), f32(rng.standard_normal(1000))
    assert np.array_equal(oracle.accumulate(m, g, 1.0), m + g)
    z = np.zeros(1000, np.float32)
    assert np.array_equal(oracle.accumulate(z, g, 0.25), g * np.float32(0.25))


def test_accumulate_bf16_gradients_widen_exactly():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(13)
    g32 = f32(rng.standard_normal(4096) * 1e-3)
    tb = torch.from_numpy(g32).to(torch.bfloat16)
    bits = tb.view(torch.int16).numpy().view(np.uint16).copy()
    assert np.array_equal(bits, bf16_bits_from_f32(g32))               # helper agrees with the library's rounding
    widened = tb.to(torch.float32).numpy()
    assert np.array_equal(widened, bf16_bits_to_f32(bits))
    m = f32(rng.standard_normal(4096) * 1e-3)
    assert np.array_equal(oracle.accumulate(m, bits, 0.5), oracle.accumulate(m, widened, 0.5))


# ---------------------------------------------------------------- whole step: closed forms and invariants
def _random_problem(rng, n, numel, scale=1e-3, mem_scale=1e-3):
    shared = rng.standard_normal(numel)
    grad = [f32(scale * (shared + 0.5 * rng.standard_normal(numel))) for _ in range(n)]
    mem = [f32(mem_scale * rng.standard_normal(numel)) for _ in range(n)]
    return mem, grad


def test_step_against_float64_closed_form():
    """Everything recomputed in float64 from Eq. 2, 3, 5 with NumPy; the oracle's binary32
    results must agree to rounding, and its index set must be a valid top-k of the float64
    leader vector up to a 1-ulp tie."""
    rng = np.random.default_rng(21)
    n, numel, k, beta, lr, step = 5, 20_000, 200, 0.3, 0.1, 7
    mem, grad = _random_problem(rng, n, numel)
    mem0 = [m.copy() for m in mem]
    idx, red = oracle.step(mem, grad, k, beta, lr, step)
    lr64, beta64 = float(np.float32(lr)), float(np.float32(beta))
    acc = [mem0[i].astype(np.float64) + lr64 * grad[i].astype(np.float64) for i in range(n)]
    leader = step % n
    assert leader == 2
    mag = np.abs(acc[leader])
    assert idx.size == k and np.all(np.diff(idx) > 0)
    rest = np.setdiff1d(np.arange(numel), idx)
    assert mag[idx].min() >= mag[rest].max() * (1 - 2.0 ** -22)
    want_red = sum(a[idx] for a in acc)
    assert np.allclose(red, want_red, rtol=1e-6, atol=1e-6 * np.abs(want_red).max())
    for i in range(n):
        m64 = mem0[i].astype(np.float64)
        resid = acc[i].copy()
        resid[idx] = 0.0
        want = (1 - beta64) * m64 + beta64 * resid                   # Eq. 5 as printed
        other = m64 + beta64 * (lr64 * grad[i].astype(np.float64) - (acc[i] - resid))   # m + beta (grad - g)
        assert np.allclose(want, other, rtol=0, atol=1e-15)
        assert np.allclose(mem[i], want, rtol=1e-6, atol=1e-6 * np.abs(want).max())
        # selected entries keep (1 - beta) of their old memory: not zero
        assert np.allclose(mem[i][idx], (1 - beta64) * m64[idx], rtol=1e-6, atol=1e-12)
        assert np.count_nonzero(mem[i][idx]) == k


def test_leader_follows_step_mod_n():
    """The index set at step t is the plain top-k of learner (t mod n)'s own vector (Remark 1),
    and of nobody else's."""
    rng = np.random.default_rng(22)
    n, numel, k = 4, 4096, 40
    for step in range(0, 9):
        mem, grad = _random_problem(rng, n, numel)
        grad = [f32(rng.standard_normal(numel)) for _ in range(n)]     # independent: sets differ
        accs = [oracle.accumulate(mem[i], grad[i], 0.5) for i in range(n)]
        idx, _ = oracle.step([m.copy() for m in mem], grad, k, 0.5, 0.5, step)
        for i in range(n):
            same = np.array_equal(idx, brute_topk(accs[i], k))
            assert same == (i == step % n)


def test_reduction_commutes_with_sparsification():
    """Eq. 1: sparsify-then-sum equals sum-then-sparsify; with the same order of additions the
    two are the same binary32 numbers."""
    rng = np.random.default_rng(23)
    n, numel, k = 6, 5000, 77
    mem, grad = _random_problem(rng, n, numel)
    accs = [oracle.accumulate(mem[i], grad[i], 0.1) for i in range(n)]
    dense = accs[0].copy()
    for i in range(1, n):
        dense = dense + accs[i]
    idx, red = oracle.step(mem, grad, k, 0.2, 0.1, 3)
    assert np.array_equal(red, dense[idx])


def test_memory_update_rounds_the_kept_part_then_fuses_the_residual():
    """Eq. 5 in binary32, rounding by rounding: 1 - beta is rounded once, kept = RN((1 - beta) * m),
    then m' = RN(kept + beta * r) with the product beta * r exact (one fused multiply-add); r is x off
    the index set and 0 on it.  Expected values come from exact rational arithmetic, and the sample
    is checked to tell this evaluation from an unfused multiply-then-add, from a fused kept part,
    and from the other algebraic form m + beta * (r - m)."""
    rng = np.random.default_rng(25)
    numel = 400
    m = f32(rng.standard_normal(numel) * 1e-3)
    x = f32(rng.standard_normal(numel) * 1e-3)
    idx = np.arange(0, numel, 7, dtype=np.int32)                       # members: residual 0 there
    in_set = np.zeros(numel, bool)
    in_set[idx] = True
    for beta in (0.1, 0.2, 0.3, 0.7):
        b = np.float32(beta)
        omb = round_fraction_to_f32(Fraction(1) - Fraction(float(b)))  # 1 - beta, one rounding
        assert omb == np.float32(1.0) - b
        got = m.copy()
        oracle.memory_update(got, x, idx, float(b))
        differs = {"unfused": 0, "kept_fused": 0, "other_form": 0}
        for j in range(numel):
            r = np.float32(0.0) if in_set[j] else x[j]
            kept = round_fraction_to_f32(Fraction(float(omb)) * Fraction(float(m[j])))
            want = round_fraction_to_f32(Fraction(float(kept)) + Fraction(float(b)) * Fraction(float(r)))
            assert got[j] == want, (beta, j)
            # neighbouring evaluations that the pin must tell apart
            unfused = np.float32(kept + np.float32(b * r))
            kept_fused = round_fraction_to_f32(Fraction(float(omb)) * Fraction(float(m[j])) +
                                               Fraction(float(b)) * Fraction(float(r)))
            other = np.float32(m[j] + np.float32(b * np.float32(r - m[j])))
            differs["unfused"] += got[j] != unfused
            differs["kept_fused"] += got[j] != kept_fused
            differs["other_form"] += got[j] != other
        assert all(v > 0 for v in differs.values()), (beta, differs)
        assert np.array_equal(got[idx], (omb * m[idx]).astype(np.float32))   # on the set: (1 - beta) * m, one rounding


def test_beta_one_is_plain_error_feedback():
    rng = np.random.default_rng(24)
    n, numel, k = 3, 3000, 30
    mem, grad = _random_problem(rng, n, numel)
    accs = [oracle.accumulate(mem[i], grad[i], 0.1) for i in range(n)]
    idx, red = oracle.step(mem, grad, k, 1.0, 0.1, 1)
    total = np.zeros(k, np.float32)
    for i in range(n):
        assert np.all(mem[i][idx] == 0.0)
        sent = np.zeros(numel, np.float32)
        sent[idx] = accs[i][idx]
        assert np.array_equal(mem[i] + sent, accs[i])                  # nothing lost: memory + sent = x
    assert np.array_equal(red, oracle.reduce([a[idx] for a in accs]))


def test_residual_energy_identity():
    """||x - CLT(x)||^2 = ||x||^2 - sum of squares of the kept values (used in Lemma 1)."""
    rng = np.random.default_rng(25)
    n, numel, k = 3, 3000, 50
    mem, grad = _random_problem(rng, n, numel)
    accs = [oracle.accumulate(mem[i], grad[i], 1.0).astype(np.float64) for i in range(n)]
    idx, _ = oracle.step(mem, grad, k, 1.0, 1.0, 0)
    for i in range(n):
        lhs = float(np.sum(mem[i].astype(np.float64) ** 2))           # beta = 1: memory is the residual
        rhs = float(np.sum(accs[i] ** 2) - np.sum(accs[i][idx] ** 2))
        assert lhs == pytest.approx(rhs, rel=1e-9)


def test_memory_telescopes_over_steps():
    """Summing Eq. 5 over iterations: mean_i m_i^T = beta * sum_t (mean_i lr grad_i^t - g^t / n),
    the identity behind theta^t - v^t = (alpha / beta) mean memory in Appendix C."""
    rng = np.random.default_rng(26)
    n, numel, k, beta, lr, T = 4, 2048, 20, 0.25, 0.5, 9
    mem = [np.zeros(numel, np.float32) for _ in range(n)]
    acc64 = np.zeros(numel)
    for t in range(T):
        _, grad = _random_problem(rng, n, numel)
        idx, red = oracle.step(mem, grad, k, beta, lr, t)
        sent = np.zeros(numel)
        sent[idx] = red.astype(np.float64)
        acc64 += float(np.float32(lr)) * np.mean([g.astype(np.float64) for g in grad], axis=0) - sent / n
    mean_mem = np.mean([m.astype(np.float64) for m in mem], axis=0)
    assert np.allclose(mean_mem, float(np.float32(beta)) * acc64, rtol=0, atol=5e-6 * np.abs(acc64).max())


def test_per_tensor_index_sets():
    """Per-layer mode: every segment gets its own top-k of the same leader, positions are
    reported in the whole vector; equals running the whole-vector step on each slice."""
    rng = np.random.default_rng(27)
    n = 3
    sizes = [1, 64, 5, 1000, 333, 2]
    ks = [1, 1, 5, 10, 4, 0]
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    numel = int(offsets[-1])
    mem, grad = _random_problem(rng, n, numel)
    mem_ref = [m.copy() for m in mem]
    idx, red = oracle.step_layers(mem, grad, offsets, ks, 0.5, 0.1, 4)
    pos = 0
    for s, (size, k) in enumerate(zip(sizes, ks)):
        a, b = int(offsets[s]), int(offsets[s + 1])
        sub_mem = [m[a:b].copy() for m in mem_ref]
        sub_idx, sub_red = oracle.step(sub_mem, [f32(g[a:b]) for g in grad], k, 0.5, 0.1, 4)
        leader_acc = oracle.accumulate(f32(mem_ref[1][a:b]), f32(grad[1][a:b]), 0.1)   # 4 mod 3 = 1
        assert np.array_equal(sub_idx, brute_topk(leader_acc, k))
        assert np.array_equal(idx[pos:pos + k], sub_idx + a)
        assert np.array_equal(red[pos:pos + k], sub_red)
        for i in range(n):
            assert np.array_equal(mem[i][a:b], sub_mem[i])
        pos += k
    assert pos == idx.size


def test_degenerate_sizes():
    z = [np.zeros(16, np.float32) for _ in range(2)]
    g = [np.zeros(16, np.float32) for _ in range(2)]
    idx, red = oracle.step(z, g, 4, 0.1, 0.1, 0)                       # all zero: lowest positions
    assert idx.tolist() == [0, 1, 2, 3] and red.tolist() == [0, 0, 0, 0]
    idx, red = oracle.step(z, g, 0, 0.1, 0.1, 0)                       # k = 0: nothing selected
    assert idx.size == 0 and red.size == 0
    m = [f32([1, 2, 3]), f32([4, 5, 6])]
    g = [f32([1, 1, 1]), f32([2, 2, 2])]
    idx, red = oracle.step(m, g, 3, 0.5, 1.0, 1)                       # k = numel: everything selected
    assert idx.tolist() == [0, 1, 2] and red.tolist() == [8, 10, 12]
    assert m[0].tolist() == [0.5, 1.0, 1.5] and m[1].tolist() == [2.0, 2.5, 3.0]
    with pytest.raises(ValueError):
        oracle.step(m, g, 4, 0.5, 1.0, 0)                              # k > numel
    with pytest.raises(ValueError):
        oracle.step(m, g, 1, 0.0, 1.0, 0)                              # beta outside (0, 1]


# ---------------------------------------------------------------- chunk-wise selection (Sec. 4, App. E)
def test_chunk_selection_hand_worked_example(golden_dir):
    g = load_golden(os.path.join(golden_dir, "e4_chunks.txt"))
    mem = [f32(g["mem_0"]), f32(g["mem_1"])]
    grad = [f32(g["grad_0"]), f32(g["grad_1"])]
    idx, red = oracle.step_chunked(mem, grad, g["chunk"], g["beta"], g["lr"], g["step"])
    assert idx.tolist() == g["idx"].astype(int).tolist()
    assert red.tolist() == g["reduced"].tolist()
    assert mem[0].tolist() == g["mem_0_out"].tolist()
    assert mem[1].tolist() == g["mem_1_out"].tolist()


def test_chunk_selection_against_brute_force():
    rng = np.random.default_rng(31)
    for n in (1, 2, 5, 16, 17, 100, 1000):
        for kind in ("normal", "ties"):
            x = f32(rng.standard_normal(n)) if kind == "normal" else f32(rng.choice([-1.0, 0.0, 1.0, -0.0], size=n))
            for chunk in (1, 2, 3, 4, 7, 16, n, n + 5):
                want = [max(range(a, min(a + chunk, n)), key=lambda j: (mag_key(x[j]), -j)) for a in range(0, n, chunk)]
                assert oracle.chunk_select(x, chunk).tolist() == want, (n, kind, chunk)


def test_chunk_selection_special_cases_are_top_k():
    """chunk >= numel is the top-1; chunk = 1 selects everything; and when the k largest entries
    happen to sit one per chunk, chunk-wise selection IS the top-k of Eq. 2."""
    rng = np.random.default_rng(32)
    x = f32(rng.standard_normal(4096) * 1e-3)
    assert oracle.chunk_select(x, 4096).tolist() == oracle.topk_select(x, 1).tolist()
    assert oracle.chunk_select(x, 10_000).tolist() == oracle.topk_select(x, 1).tolist()
    assert oracle.chunk_select(x, 1).tolist() == list(range(4096))
    y = f32(rng.standard_normal(64 * 50) * 1e-3)
    peaks = np.arange(64) * 50 + rng.integers(0, 50, size=64)
    y[peaks] = np.float32(1.0) + f32(rng.random(64))
    assert oracle.chunk_select(y, 50).tolist() == oracle.topk_select(y, 64).tolist() == sorted(peaks.tolist())


def test_chunk_selection_keeps_no_more_energy_than_top_k():
    rng = np.random.default_rng(33)
    x = f32(rng.standard_normal(30_000))
    for chunk in (10, 100, 112):
        sel = oracle.chunk_select(x, chunk)
        top = oracle.topk_select(x, sel.size)
        e = lambda idx: float(np.sum(x[idx].astype(np.float64) ** 2))
        assert e(sel) <= e(top) and e(sel) >= sel.size / x.size * float(np.sum(x.astype(np.float64) ** 2))
        assert np.all(sel // chunk == np.arange(sel.size))            # exactly one position in every chunk


def test_chunked_step_equals_primitives():
    """The chunked step is the same Eq. 3 / Alg. 1 line 10 / Eq. 5 pipeline with another index set."""
    rng = np.random.default_rng(34)
    n, numel, chunk = 4, 5003, 37
    mem, grad = _random_problem(rng, n, numel)
    accs = [oracle.accumulate(mem[i], grad[i], 0.3) for i in range(n)]
    want_idx = oracle.chunk_select(accs[2], chunk)                    # step 6 -> leader 2
    want_mem = [m.copy() for m in mem]
    for i in range(n):
        oracle.memory_update(want_mem[i], accs[i], want_idx, 0.2)
    idx, red = oracle.step_chunked(mem, grad, chunk, 0.2, 0.3, 6)
    assert np.array_equal(idx, want_idx)
    assert np.array_equal(red, oracle.reduce([a[want_idx] for a in accs]))
    for i in range(n):
        assert np.array_equal(mem[i], want_mem[i])


def test_chunked_layers_step_is_the_chunked_step_per_segment():
    """Per-layer chunk sizes: every segment on its own is the whole-vector case (positions shifted
    by the segment's start); elements outside all segments keep their bits; brute force on the
    leader's segment decides the positions."""
    rng = np.random.default_rng(35)
    n = 3
    sizes = [0, 5, 1, 40, 0, 1000, 333]
    chunks = [7, 2, 9, 40, 1, 112, 400]
    offsets = np.concatenate([[2], 2 + np.cumsum(sizes)])
    numel = int(offsets[-1]) + 4
    mem, grad = _random_problem(rng, n, numel)
    before = [m.copy() for m in mem]
    step, lr, beta = 4, 0.3, 0.2                                       # leader 1
    x_leader = oracle.accumulate(mem[1], grad[1], lr)
    want_idx = []
    for a, b, ch in zip(offsets[:-1], offsets[1:], chunks):
        for c0 in range(int(a), int(b), ch):
            want_idx.append(max(range(c0, min(c0 + ch, int(b))), key=lambda j: (mag_key(x_leader[j]), -j)))
    ref_mem = [m.copy() for m in mem]
    ref_idx, ref_red = [], []
    for a, b, ch in zip(offsets[:-1], offsets[1:], chunks):
        if b == a:
            continue
        sub_m = [np.ascontiguousarray(m[a:b]) for m in ref_mem]
        sub_g = [np.ascontiguousarray(g[a:b]) for g in grad]
        i2, r2 = oracle.step_chunked(sub_m, sub_g, ch, beta, lr, step)
        for m, sm in zip(ref_mem, sub_m):
            m[a:b] = sm
        ref_idx += (i2 + a).tolist(); ref_red += r2.tolist()
    idx, red = oracle.step_layers_chunked(mem, grad, offsets, chunks, beta, lr, step)
    assert idx.tolist() == want_idx == ref_idx
    assert red.tolist() == ref_red
    for i in range(n):
        assert np.array_equal(mem[i], ref_mem[i])
        assert np.array_equal(mem[i][:2], before[i][:2]) and np.array_equal(mem[i][-4:], before[i][-4:])
    with pytest.raises(ValueError):
        oracle.step_layers_chunked(mem, grad, offsets, [0] * len(chunks), beta, lr, step)


# ---------------------------------------------------------------- weight update and rate guidance
def test_apply_update_closed_form_and_full_iteration():
    """Alg. 1 lines 10 and 12 on the index set: with every learner sending the same gradient g,
    zero memory and k = numel, the compressed average is g and theta moves by -alpha * g exactly."""
    rng = np.random.default_rng(41)
    n, numel, alpha = 4, 257, 0.5
    g = f32(rng.integers(-8, 9, size=numel) / 8.0)                    # dyadic: every step below is exact
    theta = f32(rng.integers(-64, 65, size=numel) / 16.0)
    want = theta - np.float32(alpha) * g
    mem = [np.zeros(numel, np.float32) for _ in range(n)]
    idx, red = oracle.step(mem, [g.copy() for _ in range(n)], numel, 1.0, 1.0, 0)
    oracle.apply_update(theta, idx, red, alpha / n)
    assert np.array_equal(theta, want)
    # sparse case against float64, untouched entries stay bit-identical
    theta = f32(rng.standard_normal(1000)); before = theta.copy()
    idx = np.array([3, 10, 999], np.int32); red = f32([0.3, -1.7, 2.5])
    oracle.apply_update(theta, idx, red, 0.125)
    assert np.allclose(theta[idx], before[idx].astype(np.float64) - 0.125 * red.astype(np.float64), rtol=1e-7)
    rest = np.setdiff1d(np.arange(1000), idx)
    assert np.array_equal(theta[rest], before[rest])
    with pytest.raises(ValueError):
        oracle.apply_update(theta, np.array([1000], np.int32), f32([1.0]), 1.0)


def test_layer_rate_guidance_table():
    """Sec. 4: 25X for FLOPs/gradient in [196, inf), 50X for [128, 196), 400X for (0, 128)."""
    for ratio, rate in ((1e6, 25), (196.0, 25), (195.999, 50), (128.0, 50), (127.999, 400), (1.0, 400), (1e-3, 400)):
        assert oracle.layer_rate(ratio) == rate


# ---------------------------------------------------------------- similarity diagnostics (Sec. 2, Sec. 3)
def test_hamming_distance_extremes_and_brute_force():
    rng = np.random.default_rng(51)
    n, numel, k = 4, 3000, 60
    base = f32(rng.standard_normal(numel))
    zeros = [np.zeros(numel, np.float32) for _ in range(n)]
    # identical learners: the sum is n * x, same order of magnitudes, distance 0
    assert oracle.hamming_distance(zeros, [base.copy() for _ in range(n)], k, 1.0, 2) == 0
    # the leader alone is large on a support where the others vanish and the rest cancel it
    lead = np.zeros(numel, np.float32); lead[:k] = 5.0
    other = np.zeros(numel, np.float32); other[:k] = -5.0; other[k:2 * k] = 3.0
    assert oracle.hamming_distance(zeros[:2], [lead, other], k, 1.0, 0) == k
    # brute force on random data, with memory and lr
    mem, grad = _random_problem(rng, n, numel)
    for step in range(n):
        accs = [oracle.accumulate(mem[i], grad[i], 0.3) for i in range(n)]
        y = accs[0].copy()
        for i in range(1, n):
            y = y + accs[i]
        want = k - len(set(brute_topk(accs[step % n], k).tolist()) & set(brute_topk(y, k).tolist()))
        assert oracle.hamming_distance(mem, grad, k, 0.3, step) == want
        assert 0 <= want <= k


def test_cosine_distance_closed_forms():
    rng = np.random.default_rng(52)
    a = f32(rng.standard_normal(5000))
    assert oracle.cosine_distance(a, f32(3.0 * a)) == pytest.approx(0.0, abs=1e-7)
    assert oracle.cosine_distance(a, f32(-a)) == pytest.approx(2.0, abs=1e-7)
    e1 = np.zeros(8, np.float32); e1[0] = 2.0
    e2 = np.zeros(8, np.float32); e2[3] = -7.0
    assert oracle.cosine_distance(e1, e2) == 1.0
    b = f32(rng.standard_normal(5000))
    want = 1.0 - float(np.dot(a.astype(np.float64), b.astype(np.float64))) / (
        float(np.linalg.norm(a.astype(np.float64))) * float(np.linalg.norm(b.astype(np.float64))))
    assert oracle.cosine_distance(a, b) == pytest.approx(want, rel=1e-12)
