"""GPU parity: the HIP library, called through its C-ABI, against the CPU oracle, element by
element on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle

from paper_2104_11125_amd import binding, workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import gpu_util
    return gpu_util


# ------------------------------------------------------------------ workload recipes at oracle-friendly sizes
def test_tiny_config_full(gu):
    gu.run_workload(workloads.by_name("tiny"))


@pytest.mark.parametrize("numel", [1_000_003, 262_144 + 8192 * 3 + 5])
def test_resnet_recipe_ragged(gu, numel):
    # several supertiles (8192 positions each) and a tail that is not a multiple of 4
    gu.run_workload(workloads.scaled(workloads.by_name("resnet50_sized"), numel, steps=3))


def test_transformer_recipe_heavy_tails(gu):
    gu.run_workload(workloads.scaled(workloads.by_name("transformer_base_sized"), 700_001, steps=3))


def test_bf16_recipe(gu):
    gu.run_workload(workloads.scaled(workloads.by_name("large_bf16"), 600_002, steps=3))


def test_many_learners(gu):
    gu.run_workload(workloads.scaled(workloads.by_name("tiny"), 50_001, n_learners=64, steps=2))


@pytest.mark.parametrize("n", [8, 9, 17])
def test_learner_counts_around_the_launch_size(gu, n):
    """The all-learner pass goes over eight learners per launch: one launch exactly, one more for a
    single learner, and two full ones plus one; long enough for leaders out of every launch."""
    gu.run_workload(workloads.scaled(workloads.by_name("tiny"), 30_011, n_learners=n, steps=n + 2))


def test_single_learner(gu):
    gu.run_workload(workloads.scaled(workloads.by_name("tiny"), 70_000, n_learners=1, steps=2))


# ------------------------------------------------------------------ per-tensor index sets
def test_per_layer_small_odd_layout(gu):
    w = workloads.per_layer_workload(name="per_layer_small", n_learners=5, n_tensors=40, lo=1, hi=40_000, rate=100,
                                     steps=3, seed=77)
    gu.run_workload(w)


def test_per_layer_empty_and_full_segments(gu):
    n = 3
    sizes = [0, 1, 7, 0, 8192, 8193, 300, 2, 0]
    ks = [0, 1, 7, 0, 1, 8193, 0, 1, 0]
    offsets = np.concatenate([[3], 3 + np.cumsum(sizes)]).tolist()     # the first segment does not start at 0
    numel = offsets[-1] + 5                                            # and the last one stops before the end
    g = torch.Generator(device="cpu").manual_seed(5)
    mem = [torch.randn(numel, generator=g).to(gu.DEV) for _ in range(n)]
    grad = [torch.randn(numel, generator=g).to(gu.DEV) for _ in range(n)]
    ref = [m.cpu().numpy().copy() for m in mem]
    untouched = [m.cpu().numpy().copy() for m in mem]
    ctx = binding.scalecom_init(numel, n, torch.float32, len(ks), gu.DEV)
    for step in range(3):
        gu.compare_step(ctx, mem, grad, ref, step, 0.5, 0.25, offsets=offsets, ks=ks, what="segments")
    for i in range(n):   # outside the segments nothing is written
        assert np.array_equal(mem[i].cpu().numpy()[:3], untouched[i][:3])
        assert np.array_equal(mem[i].cpu().numpy()[offsets[-1]:], untouched[i][offsets[-1]:])
    ctx.close()


# ------------------------------------------------------------------ degenerate and adversarial inputs
def _adversarial(numel, kind, rng):
    if kind == "all_equal":
        return np.full(numel, 0.5, np.float32)
    if kind == "two_valued":
        return rng.choice(np.array([1.0, -1.0, 2.0, -2.0], np.float32), size=numel)
    if kind == "zeros":
        return np.zeros(numel, np.float32)
    if kind == "signed_zeros":
        return rng.choice(np.array([0.0, -0.0], np.float32), size=numel)
    if kind == "denormals":
        return (rng.integers(-40, 40, size=numel).astype(np.float32) * np.float32(1e-45)).astype(np.float32)
    if kind == "few_levels":   # many ties at every level of the key
        return rng.choice(np.array([1.0, 1.0000001, 1.0000002, 0.99999994, -1.0, 3.0], np.float32), size=numel)
    if kind == "nonfinite":
        x = rng.standard_normal(numel).astype(np.float32)
        x[rng.integers(0, numel, size=max(1, numel // 50))] = np.inf
        x[rng.integers(0, numel, size=max(1, numel // 50))] = -np.inf
        x[rng.integers(0, numel, size=max(1, numel // 70))] = np.nan
        return x
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["all_equal", "two_valued", "zeros", "signed_zeros", "denormals", "few_levels",
                                  "nonfinite"])
def test_adversarial_values(gu, kind):
    rng = np.random.default_rng(hash(kind) % 1000)
    n = 3
    for numel in (1, 3, 255, 256, 257, 8191, 8192, 8193, 40_003):
        ks = sorted({0, 1, numel // 3, numel - 1, numel} - {-1})
        ctx = binding.scalecom_init(numel, n, torch.float32, 1, gu.DEV)
        for k in ks:
            grads = [_adversarial(numel, kind, rng) for _ in range(n)]
            mems = [_adversarial(numel, kind, rng) if kind != "nonfinite" else np.zeros(numel, np.float32)
                    for _ in range(n)]
            mem = [torch.from_numpy(m.copy()).to(gu.DEV) for m in mems]
            grad = [torch.from_numpy(g).to(gu.DEV) for g in grads]
            ref = [m.copy() for m in mems]
            for step in range(2):
                gu.compare_step(ctx, mem, grad, ref, step, 0.25, 1.0, k=k, what=f"{kind} numel={numel} k={k}")
        ctx.close()


def test_threshold_ties_across_tiles(gu):
    """The threshold value repeated in every wave tile and supertile: members among the equal
    keys are the lowest positions, wherever the tile boundaries fall."""
    numel, n = 3 * 8192 + 777, 2
    x = np.full(numel, 1.0, np.float32)
    x[::5] = 2.0                                   # above the threshold
    x[3::7] = 0.5                                  # below
    above = int(np.count_nonzero(x == 2.0))
    ties = int(np.count_nonzero(x == 1.0))
    ctx = binding.scalecom_init(numel, n, torch.float32, 1, gu.DEV)
    for take in (0, 1, 255, 256, 257, 8192, ties - 1, ties):
        mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
        grad = [torch.from_numpy(x.copy()).to(gu.DEV), torch.from_numpy(-x).to(gu.DEV)]
        ref = [np.zeros(numel, np.float32) for _ in range(n)]
        gu.compare_step(ctx, mem, grad, ref, 0, 1.0, 1.0, k=above + take, what=f"ties take={take}")
    ctx.close()


def test_bucket_keys_clustered_in_one_place(gu):
    """Leader vector sorted by magnitude: the keys around the threshold sit next to each other,
    which overflows the per-supertile candidate slots and must fall back to full passes."""
    numel, n = 40 * 8192 + 123, 3
    rng = np.random.default_rng(99)
    base = np.sort(np.abs(rng.standard_normal(numel).astype(np.float32)))
    grads = [base * np.float32(1e-3), (base[::-1] * np.float32(1e-3)).copy(),
             rng.standard_normal(numel).astype(np.float32)]
    ctx = binding.scalecom_init(numel, n, torch.float32, 1, gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    grad = [torch.from_numpy(g).to(gu.DEV) for g in grads]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]
    for step in range(3):                       # leaders: ascending, descending, random
        gu.compare_step(ctx, mem, grad, ref, step, 0.5, 1.0, k=numel // 100, what="clustered")
    assert ctx.scalecom_selection_stats()["full_mode"] >= 1      # the sorted leaders did take the full passes
    ctx.close()


def test_threshold_jumps_between_steps(gu):
    """The library predicts each step's threshold bucket from the previous step (same context,
    same layout) to save a pass over the leader; the prediction must never change the result.
    Gradient scale and lr jump by orders of magnitude from step to step, so predictions miss,
    hit, and land just inside / outside their window."""
    w = workloads.scaled(workloads.by_name("resnet50_sized"), 300_007, n_learners=3, steps=1)
    ctx = binding.scalecom_init(w.numel, w.n_learners, torch.float32, 1, gu.DEV)
    mem = workloads.zero_memories(w, gu.DEV)
    ref = [m.cpu().numpy().copy() for m in mem]
    base = workloads.gradients(w, 0, gu.DEV)
    scales = [1.0, 1.0, 100.0, 1.04, 1.0, 1e-3, 1.09, 0.92, 1.2, 0.8, 1e4, 1.0]
    for step, sc in enumerate(scales):
        grad = [g * sc for g in base]
        lr = 0.1 if step % 5 else 1.0
        gu.compare_step(ctx, mem, grad, ref, step, 0.5, lr, k=w.k, what=f"scale {sc}")
    ctx.close()


def test_selection_stats_count_misses(gu):
    """The device counters behind scalecom_selection_stats: the first step of a layout has no
    prediction, a gradient scale that jumps by 100 is a sure miss (the widest range spans two
    binades), and a step repeated on the same inputs from the same state must hit the third time
    (the leader's own last threshold is the centre of its range).  Results are compared as ever."""
    w = workloads.scaled(workloads.by_name("resnet50_sized"), 300_007, n_learners=3, steps=1)
    ctx = binding.scalecom_init(w.numel, w.n_learners, torch.float32, 1, gu.DEV)
    assert ctx.scalecom_selection_stats() == {"missed": 0, "no_prediction": 0, "full_mode": 0, "wide_range": 0, "steps": 0}
    mem = workloads.zero_memories(w, gu.DEV)
    ref = [m.cpu().numpy().copy() for m in mem]
    base = workloads.gradients(w, 0, gu.DEV)
    seen = []
    for step, sc in enumerate([1.0, 1.0, 100.0]):
        gu.compare_step(ctx, mem, [g * sc for g in base], ref, step, 0.5, 0.1, k=w.k, what=f"scale {sc}")
        seen.append(ctx.scalecom_selection_stats())
    assert [s["steps"] for s in seen] == [1, 2, 3]
    assert [s["no_prediction"] for s in seen] == [1, 1, 1]
    assert seen[0]["missed"] == 0 and seen[2]["missed"] == seen[1]["missed"] + 1          # the jump
    # the same step three times from the same state
    mem0, ref0 = [m.clone() for m in mem], [r.copy() for r in ref]
    for rep in range(3):
        for m, m0, r, r0 in zip(mem, mem0, ref, ref0):
            m.copy_(m0)
            r[:] = r0
        gu.compare_step(ctx, mem, base, ref, 3, 0.5, 0.1, k=w.k, what=f"repeat {rep}")
        seen.append(ctx.scalecom_selection_stats())
    assert seen[-1]["steps"] == 6 and seen[-1]["missed"] == seen[-2]["missed"]            # third time: a hit
    assert seen[-1]["no_prediction"] == 1
    # a diagnostic selection is not a step and counts nothing; reset starts again from zero
    ctx.scalecom_hamming_distance(mem, base, [0, w.numel], [w.k], 0.1, 0)
    assert ctx.scalecom_selection_stats(reset=True)["steps"] == 6
    gu.compare_step(ctx, mem, base, ref, 4, 0.5, 0.1, k=w.k, what="after reset")
    after = ctx.scalecom_selection_stats()
    assert after["steps"] == 1 and after["no_prediction"] == 0      # same layout: the diagnostic left the predictions alone
    ctx.close()


def test_per_layer_predictions(gu):
    """Per-tensor mode keeps one prediction per tensor; tensors' thresholds move independently."""
    w = workloads.per_layer_workload(name="per_layer_pred", n_learners=3, n_tensors=25, lo=8, hi=60_000, rate=50,
                                     steps=1, seed=78)
    ctx = binding.scalecom_init(w.numel, w.n_learners, torch.float32, w.n_tensors, gu.DEV)
    mem = workloads.zero_memories(w, gu.DEV)
    ref = [m.cpu().numpy().copy() for m in mem]
    base = workloads.gradients(w, 0, gu.DEV)
    g = torch.Generator(device="cpu").manual_seed(3)
    for step in range(6):
        # every tensor gets its own scale factor each step
        factors = torch.exp(torch.randn(w.n_tensors, generator=g) * (0.05 if step % 2 else 2.0))
        scale = torch.ones(w.numel)
        for t in range(w.n_tensors):
            scale[w.offsets[t]:w.offsets[t + 1]] = factors[t]
        scale = scale.to(gu.DEV)
        grad = [b * scale for b in base]
        gu.compare_step(ctx, mem, grad, ref, step, 0.3, 0.5, offsets=w.offsets, ks=w.ks, what=f"step {step}")
    ctx.close()


# ------------------------------------------------------------------ chunk-wise selector
@pytest.mark.parametrize("numel,chunk", [(1, 1), (5, 1), (7, 3), (1000, 112), (100_003, 112), (100_003, 400),
                                         (65_536, 256), (65_536, 64), (40_000, 100), (9_000, 9_000), (9_000, 20_000),
                                         (8_193, 255), (300_001, 25)])
def test_chunked_selector(gu, numel, chunk):
    n = 3
    g = torch.Generator(device="cpu").manual_seed(numel * 31 + chunk)
    mem = [(torch.randn(numel, generator=g) * 1e-3).to(gu.DEV) for _ in range(n)]
    grad = [(torch.randn(numel, generator=g) * 1e-3).to(gu.DEV) for _ in range(n)]
    ref = [m.cpu().numpy().copy() for m in mem]
    ctx = binding.scalecom_init(numel, n, torch.float32, 1, gu.DEV)
    for step in range(3):
        gu.compare_step(ctx, mem, grad, ref, step, 0.3, 0.7, chunk=chunk, what=f"chunk={chunk} numel={numel}")
    ctx.close()


def test_chunked_selector_ties_bf16_and_mixed_calls(gu):
    """Equal magnitudes inside a chunk go to the lowest position; bf16 gradients; and exact and
    chunk-wise steps alternate on one context without disturbing each other."""
    numel, n, chunk = 50_007, 4, 112
    rng = np.random.default_rng(5)
    vals = rng.choice(np.array([1.0, -1.0, 0.5, 0.0], np.float32), size=(n, numel))
    ctx = binding.scalecom_init(numel, n, torch.bfloat16, 1, gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    grad = [torch.from_numpy(v).to(gu.DEV).to(torch.bfloat16) for v in vals]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]
    for step in range(6):
        if step % 2:
            gu.compare_step(ctx, mem, grad, ref, step, 0.5, 1.0, k=numel // 100, what="mixed exact")
        else:
            gu.compare_step(ctx, mem, grad, ref, step, 0.5, 1.0, chunk=chunk, what="mixed chunked")
    ctx.close()


def test_chunked_selector_per_layer(gu):
    """A chunk size per tensor: odd layouts (empty segments, chunk larger than the tensor, chunk 1,
    segments that start and end inside a wave tile), rates from the paper's guidance, and steps
    of the other kinds in between on the same context."""
    n = 3
    sizes = [0, 5, 1, 40, 0, 1000, 333, 8192, 8193, 70_001, 2, 20_000]
    chunks = [7, 2, 9, 40, 1, 112, 400, 25, 50, 400, 5, 1]
    offsets = np.concatenate([[3], 3 + np.cumsum(sizes)]).tolist()
    numel = offsets[-1] + 5
    g = torch.Generator(device="cpu").manual_seed(21)
    mem = [(torch.randn(numel, generator=g) * 1e-3).to(gu.DEV) for _ in range(n)]
    grad = [(torch.randn(numel, generator=g) * 1e-3).to(gu.DEV) for _ in range(n)]
    ref = [m.cpu().numpy().copy() for m in mem]
    ctx = binding.scalecom_init(numel, n, torch.float32, len(sizes), gu.DEV)
    ks = [-(-sz // 100) for sz in sizes]
    for step in range(6):
        if step == 3:      # an exact per-layer step in between
            gu.compare_step(ctx, mem, grad, ref, step, 0.3, 0.7, offsets=offsets, ks=ks, what="exact between chunked")
        else:
            gu.compare_step(ctx, mem, grad, ref, step, 0.3, 0.7, offsets=offsets, chunks=chunks, what="chunked layers")
    # same number of chunks, other chunk sizes: the cached layout must not be reused
    chunks2 = [c + 1 if sz and -(-sz // c) == -(-sz // (c + 1)) else c for sz, c in zip(sizes, chunks)]
    assert chunks2 != chunks
    gu.compare_step(ctx, mem, grad, ref, 6, 0.3, 0.7, offsets=offsets, chunks=chunks2, what="chunk sizes changed")
    # the paper's rate guidance feeds it directly
    _, rates = binding.scalecom_layer_ks([300.0, 150.0, 64.0] * 4, sizes)
    gu.compare_step(ctx, mem, grad, ref, 7, 0.3, 0.7, offsets=offsets, chunks=rates, what="rates of the guidance")
    # many positions, then few, then more again: the per-chunk maxima of a longer earlier call must not survive
    for step, ch in ((8, 1), (9, 400), (10, 7), (11, 3)):
        gu.compare_step(ctx, mem, grad, ref, step, 0.3, 0.7, offsets=offsets, chunks=[ch] * len(sizes),
                        what=f"all chunks {ch}")
    # chunk sizes far beyond the tensors, beyond 32 bits too: one position per non-empty tensor
    huge = [2 ** 32, 2 ** 40, 2 ** 62, 2 ** 31, 2 ** 32 + 1, 2 ** 33] * 2
    gu.compare_step(ctx, mem, grad, ref, 12, 0.3, 0.7, offsets=offsets, chunks=huge, what="huge chunks")
    with pytest.raises(binding.ScaleComError):
        ctx.scalecom_step_layers_chunked(mem, grad, offsets, [0] * len(sizes), 0.3, 0.7, 0)
    ctx.close()
    flat = binding.scalecom_init(numel, n, torch.float32, 1, gu.DEV)
    gu.compare_step(flat, mem, grad, ref, 13, 0.3, 0.7, chunk=2 ** 40, what="one huge chunk")
    flat.close()


def test_apply_update_after_a_step(gu):
    """Alg. 1 lines 10 and 12: the step's outputs applied to the weights on the same stream."""
    import oracle
    w = workloads.scaled(workloads.by_name("resnet50_sized"), 400_003, n_learners=4, steps=1)
    ctx = binding.scalecom_init(w.numel, w.n_learners, torch.float32, 1, gu.DEV)
    mem = workloads.zero_memories(w, gu.DEV)
    ref = [m.cpu().numpy().copy() for m in mem]
    g = torch.Generator(device="cpu").manual_seed(8)
    theta = torch.randn(w.numel, generator=g).to(gu.DEV)
    theta_ref = theta.cpu().numpy().copy()
    for step in range(3):
        grad = workloads.gradients(w, step, gu.DEV)
        idx, red = gu.compare_step(ctx, mem, grad, ref, step, w.beta, w.lr, k=w.k, what="apply")
        ctx.scalecom_apply_update(theta, idx, red, 1.0 / w.n_learners)
        oracle.apply_update(theta_ref, idx.cpu().numpy(), red.cpu().numpy(), 1.0 / w.n_learners)
        torch.cuda.synchronize()
        gu.assert_same("theta", theta.cpu().numpy(), theta_ref, 1e-6, f"step {step}")
    ctx.scalecom_apply_update(theta, idx[:0], red[:0], 1.0)          # k = 0: nothing happens
    bad = torch.tensor([-1, w.numel, 2 ** 31 - 1, 5], dtype=torch.int32, device=gu.DEV)   # outside theta: skipped
    before = theta.clone()
    ctx.scalecom_apply_update(theta, bad, torch.ones(4, device=gu.DEV), 1.0)
    torch.cuda.synchronize()
    before[5] -= 1.0
    assert torch.equal(theta, before)
    with pytest.raises(binding.ScaleComError):
        ctx.scalecom_apply_update(theta, idx, red, float("nan"))
    ctx.close()


# ------------------------------------------------------------------ similarity diagnostics (Sec. 3)
def _oracle_d(gu, mem, grad, offsets, ks, lr, step):
    import oracle
    mem_h = [m.cpu().numpy() for m in mem]
    grad_h = [gu.to_host(g) for g in grad]
    out = []
    for s, k in enumerate(ks):
        a, b = offsets[s], offsets[s + 1]
        if b == a:
            out.append(0)
            continue
        out.append(oracle.hamming_distance([np.ascontiguousarray(m[a:b]) for m in mem_h],
                                           [np.ascontiguousarray(g[a:b]) for g in grad_h], int(k), lr, step))
    return np.array(out, np.int32)


@pytest.mark.parametrize("recipe,numel", [("resnet50_sized", 300_001), ("large_bf16", 150_002)])
def test_hamming_distance_between_steps(gu, recipe, numel):
    """d between the leader's set and the true top-k, asked for between ordinary steps: exact,
    leaves the memories alone and does not disturb the steps that follow."""
    w = workloads.scaled(workloads.by_name(recipe), numel, n_learners=4, steps=4)
    gd = torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32
    ctx = binding.scalecom_init(w.numel, w.n_learners, gd, 1, gu.DEV)
    mem = workloads.zero_memories(w, gu.DEV)
    ref = [m.cpu().numpy().copy() for m in mem]
    for step in range(4):
        grad = workloads.gradients(w, step, gu.DEV)
        d = ctx.scalecom_hamming_distance(mem, grad, [0, w.numel], [w.k], w.lr, step)
        torch.cuda.synchronize()
        want = _oracle_d(gu, mem, grad, [0, w.numel], [w.k], w.lr, step)
        print(f"[hamming] {recipe} step {step}: d/k = {int(want[0])}/{w.k}", flush=True)
        assert np.array_equal(d.cpu().numpy(), want)
        for i in range(w.n_learners):
            gu.assert_same("mem", mem[i].cpu().numpy(), ref[i], None, f"untouched, learner {i}")
        gu.compare_step(ctx, mem, grad, ref, step, w.beta, w.lr, k=w.k, what="after hamming")
    ctx.close()


def test_hamming_distance_per_layer_and_extremes(gu):
    n = 3
    sizes = [0, 1, 7, 8192, 8193, 300, 2, 0, 40_000]
    ks = [0, 1, 3, 100, 8193, 0, 1, 0, 400]
    offsets = np.concatenate([[4], 4 + np.cumsum(sizes)]).tolist()
    numel = offsets[-1] + 3
    g = torch.Generator(device="cpu").manual_seed(15)
    mem = [torch.randn(numel, generator=g).to(gu.DEV) for _ in range(n)]
    shared = torch.randn(numel, generator=g)
    grad = [(shared + 0.5 * torch.randn(numel, generator=g)).to(gu.DEV) for _ in range(n)]
    ctx = binding.scalecom_init(numel, n, torch.float32, len(ks), gu.DEV)
    for step in range(n):
        d = ctx.scalecom_hamming_distance(mem, grad, offsets, ks, 0.7, step)
        torch.cuda.synchronize()
        assert np.array_equal(d.cpu().numpy(), _oracle_d(gu, mem, grad, offsets, ks, 0.7, step))
    # identical learners: distance 0; a leader whose large entries the others cancel: distance k
    k = 50
    same = [grad[0].clone() for _ in range(n)]
    zeros = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    d = ctx.scalecom_hamming_distance(zeros, same, [0, numel], [k], 1.0, 1)
    assert d.cpu().tolist() == [0]
    lead = torch.zeros(numel); lead[:k] = 5.0
    other = torch.zeros(numel); other[:k] = -5.0; other[k:2 * k] = 3.0
    d = ctx.scalecom_hamming_distance(zeros[:2], [lead.to(gu.DEV), other.to(gu.DEV)], [0, numel], [k], 1.0, 0)
    assert d.cpu().tolist() == [k]
    # non-finite sums rank above every finite value on both sides
    bad = [gr.clone() for gr in grad]
    bad[1][1000] = float("inf"); bad[2][1000] = float("-inf"); bad[0][2000] = float("inf"); bad[2][3000] = float("nan")
    d = ctx.scalecom_hamming_distance(mem, bad, [0, numel], [k], 0.7, 2)
    torch.cuda.synchronize()
    assert np.array_equal(d.cpu().numpy(), _oracle_d(gu, mem, bad, [0, numel], [k], 0.7, 2))
    with pytest.raises(binding.ScaleComError):
        ctx.scalecom_hamming_distance(mem, grad, [0, numel], [numel + 1], 0.7, 0)
    ctx.close()


def test_cosine_distance(gu):
    import oracle
    ctx = binding.scalecom_init(16, 1, torch.float32, 1, gu.DEV)
    g = torch.Generator(device="cpu").manual_seed(16)
    for numel in (1, 255, 1_000_003):
        a = torch.randn(numel, generator=g)
        b = (0.3 * a + torch.randn(numel, generator=g))
        out = ctx.scalecom_cosine_distance(a.to(gu.DEV), b.to(gu.DEV)).cpu().numpy()
        want = oracle.cosine_distance(a.numpy(), b.numpy())
        assert abs(out[0] - want) <= 1e-12 * max(1.0, abs(want)), (numel, out[0], want)
        a64, b64 = a.numpy().astype(np.float64), b.numpy().astype(np.float64)
        np.testing.assert_allclose(out[1:], [a64 @ b64, a64 @ a64, b64 @ b64], rtol=1e-12)
    a = torch.randn(4096, generator=g).to(gu.DEV)
    assert abs(float(ctx.scalecom_cosine_distance(a, a * 2)[0])) < 1e-12
    assert abs(float(ctx.scalecom_cosine_distance(a, -a)[0]) - 2.0) < 1e-12
    ctx.close()


# ------------------------------------------------------------------ randomized layouts and values
@pytest.mark.parametrize("seed", range(32))
def test_randomized_layouts_values_and_modes(gu, seed):
    """Seeded random problems: learner count, tensor layout (gaps, empty tensors, unaligned starts),
    set sizes from 0 to everything, value distributions with heavy ties, both gradient types, and
    exact, chunk-wise and diagnostic calls mixed on one context.  Every output is compared."""
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 10))
    n_tensors = int(rng.integers(1, 13))
    sizes = [int(v) for v in rng.choice([0, 1, 3, 255, 256, 257, 1000, 8191, 8192, 8193, 30_000, 70_000], size=n_tensors)]
    gaps = [int(v) for v in rng.integers(0, 7, size=n_tensors + 1)]
    offsets, pos = [], gaps[0]
    for sz, gap in zip(sizes, gaps[1:]):
        offsets.append(pos)
        pos += sz
    offsets.append(pos)                                        # tensors are back to back; a gap only in front
    numel = pos + gaps[-1]
    bf16 = bool(seed % 2)
    kind = ["normal", "rounded", "few_levels", "sparse"][seed % 4]
    def draw(scale):
        x = rng.standard_normal(numel).astype(np.float32) * np.float32(scale)
        if kind == "rounded":
            x = np.round(x * 8) / 8 * np.float32(scale)        # many exact ties
        elif kind == "few_levels":
            x = rng.choice(np.array([-2, -1, -0.0, 0.0, 1, 2], np.float32), size=numel) * np.float32(scale)
        elif kind == "sparse":
            x = np.where(rng.random(numel) < 0.9, np.float32(0), x)
        return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    mem = [draw(1e-3).to(gu.DEV) for _ in range(n)]
    grad = [draw(1e-2).to(gu.DEV) for _ in range(n)]
    if bf16:
        grad = [g.to(torch.bfloat16) for g in grad]
    ref = [m.cpu().numpy().copy() for m in mem]
    ctx = binding.scalecom_init(max(numel, 1), n, torch.bfloat16 if bf16 else torch.float32, n_tensors, gu.DEV)
    what = f"seed {seed}: n={n} sizes={sizes} kind={kind} bf16={bf16}"
    print("[random]", what, flush=True)
    for step in range(5):
        beta = float(rng.choice([1.0, 0.5, 0.1]))
        lr = float(rng.choice([1.0, 0.3, 0.0]))
        mode = int(rng.integers(0, 4))
        if mode == 0:                                          # per-tensor exact sets, sizes from 0 to everything
            ks = [int(rng.choice([0, 1, sz // 100, sz // 2, sz])) if sz else 0 for sz in sizes]
            gu.compare_step(ctx, mem, grad, ref, step, beta, lr, offsets=offsets, ks=ks, what=what + f" ks={ks}")
        elif mode == 1:                                        # per-tensor chunk sizes
            chunks = [int(rng.choice([1, 2, 7, 100, 112, 400, 100_000])) for _ in sizes]
            gu.compare_step(ctx, mem, grad, ref, step, beta, lr, offsets=offsets, chunks=chunks,
                            what=what + f" chunks={chunks}")
        elif mode == 2 and numel > 0:                          # the whole vector as one tensor
            k = int(rng.choice([0, 1, numel // 100, numel]))
            gu.compare_step(ctx, mem, grad, ref, step, beta, lr, k=k, what=what + f" flat k={k}")
        else:                                                  # diagnostic between steps: nothing changes
            ks = [sz // 50 for sz in sizes]
            d = ctx.scalecom_hamming_distance(mem, grad, offsets, ks, lr, step)
            torch.cuda.synchronize()
            assert np.array_equal(d.cpu().numpy(), _oracle_d(gu, mem, grad, offsets, ks, lr, step)), what
            for i in range(n):
                gu.assert_same("mem", mem[i].cpu().numpy(), ref[i], None, what + " untouched")
    ctx.close()


@pytest.mark.parametrize("seed", range(12))
def test_randomized_prediction_walk(gu, seed):
    """One layout kept for many steps while the gradients' scale drifts, jumps and collapses into
    ties: the predicted single pass hits, misses and overflows, and every step stays exact."""
    rng = np.random.default_rng(2000 + seed)
    n = int(rng.integers(2, 6))
    n_tensors = [1, 1, 3, 8][seed % 4]
    sizes = [int(v) for v in rng.choice([300, 9_000, 40_000, 120_000], size=n_tensors)]
    offsets = np.concatenate([[seed % 4], (seed % 4) + np.cumsum(sizes)]).tolist()
    numel = offsets[-1] + 2
    ks = [max(1, sz // int(rng.choice([25, 100, 400]))) for sz in sizes]
    bf16 = seed % 3 == 0
    ctx = binding.scalecom_init(numel, n, torch.bfloat16 if bf16 else torch.float32, n_tensors, gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]
    shared = rng.standard_normal(numel).astype(np.float32)
    scale = 1e-3
    for step in range(10):
        move = rng.choice(["drift", "drift", "drift", "jump_up", "jump_down", "ties", "same"])
        if move == "drift":
            scale *= float(rng.uniform(0.8, 1.25))
        elif move == "jump_up":
            scale *= 64.0
        elif move == "jump_down":
            scale /= 64.0
        grads = []
        for i in range(n):
            g = (shared + 0.5 * rng.standard_normal(numel).astype(np.float32)) * np.float32(scale)
            if move == "ties":
                g = np.sign(g) * np.float32(scale)             # two magnitudes only: the bucket overflows every list
            t = torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32)).to(gu.DEV)
            grads.append(t.to(torch.bfloat16) if bf16 else t)
        what = f"seed {seed} step {step} {move} sizes={sizes} ks={ks} bf16={bf16}"
        if n_tensors == 1 and offsets[0] == 0:
            gu.compare_step(ctx, mem, grads, ref, step, 0.3, 1.0, k=ks[0], what=what)
        else:
            gu.compare_step(ctx, mem, grads, ref, step, 0.3, 1.0, offsets=offsets, ks=ks, what=what)
    ctx.close()


@pytest.mark.parametrize("scale", [1e-44, 3e-39, 1e-30, 1.0, 1e30, 5e36])
def test_prediction_at_the_ends_of_the_key_range(gu, scale):
    """The same scale for several steps, so that the prediction and the finely counted keys around
    the previous threshold are in use, with thresholds among the subnormals (the counted range is
    cut off at key 0, and few distinct values exist), at the smallest normal numbers and close to
    the largest finite ones."""
    rng = np.random.default_rng(77)
    numel, n, k = 50_021, 3, 500
    ctx = binding.scalecom_init(numel, n, torch.float32, 1, gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]
    shared = rng.standard_normal(numel)
    for step in range(5):
        grads = []
        for i in range(n):
            g = ((shared + 0.5 * rng.standard_normal(numel)) * scale).astype(np.float32)
            grads.append(torch.from_numpy(g).to(gu.DEV))
        gu.compare_step(ctx, mem, grads, ref, step, 0.3, 1.0, k=k, what=f"scale {scale} step {step}")
    ctx.close()


def test_long_run_into_the_piled_up_state(gu):
    """Several hundred steps from zero memory: error feedback lets the magnitudes pile up just below
    the threshold (a twelve-bit bucket around it comes to hold several per cent of all elements), the
    range of finely counted keys narrows step by step, and its counts go to several slotted copies.
    Index set and reduced values are compared at every step, the memories every 25 steps."""
    rng = np.random.default_rng(9)
    n, beta, lr = 3, 0.1, 0.1
    sizes = [150_001, 37, 20_000, 3_000]
    offsets = np.concatenate([[2], 2 + np.cumsum(sizes)]).tolist()
    numel = offsets[-1] + 1
    ks = [1_500, 1, 200, 30]
    ctx = binding.scalecom_init(numel, n, torch.float32, len(sizes), gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]
    pool = [[((rng.standard_normal(numel) + 0.5 * rng.standard_normal(numel)) * 1e-3).astype(np.float32)
             for _ in range(n)] for _ in range(5)]
    pool_dev = [[torch.from_numpy(g).to(gu.DEV) for g in gs] for gs in pool]
    for step in range(400):
        host, dev = pool[step % 5], pool_dev[step % 5]
        idx, red = ctx.scalecom_step_layers(mem, dev, offsets, ks, beta, lr, step)
        want_idx, want_red = oracle.step_layers(ref, host, offsets, ks, beta, lr, step)
        gu.assert_same("idx", idx.cpu().numpy(), want_idx, None, f"long run step {step}")
        gu.assert_same("reduced", red.cpu().numpy(), want_red, 1e-5, f"long run step {step}")
        if step % 25 == 24:
            for i in range(n):
                gu.assert_same("mem", mem[i].cpu().numpy(), ref[i], 1e-6, f"long run step {step} learner {i}")
    # the state the test is about was reached: the leader's bucket around the threshold is crowded
    x = np.abs(ref[0][offsets[0]:offsets[1]] + np.float32(lr) * pool[0][0][offsets[0]:offsets[1]])
    t = np.sort(x)[-ks[0]]
    crowd = np.mean((x >= t * 0.97) & (x <= t * 1.03))
    assert crowd > 3 * ks[0] / sizes[0], f"no pile-up around the threshold ({crowd:.4f})"
    ctx.close()


def test_long_run_bf16_flat(gu):
    """The same for one flat vector with bf16 gradients (300 steps)."""
    rng = np.random.default_rng(10)
    n, numel, k, beta, lr = 4, 200_003, 2_000, 0.1, 0.1
    ctx = binding.scalecom_init(numel, n, torch.bfloat16, 1, gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]
    pool_dev = [[torch.from_numpy(((rng.standard_normal(numel) + 0.5 * rng.standard_normal(numel)) * 1e-3)
                                  .astype(np.float32)).to(gu.DEV).to(torch.bfloat16) for _ in range(n)]
                for _ in range(6)]
    pool = [[gu.to_host(g) for g in gs] for gs in pool_dev]
    for step in range(300):
        idx, red = ctx.scalecom_step(mem, pool_dev[step % 6], k, beta, lr, step)
        want_idx, want_red = oracle.step(ref, pool[step % 6], k, beta, lr, step)
        gu.assert_same("idx", idx.cpu().numpy(), want_idx, None, f"long bf16 run step {step}")
        gu.assert_same("reduced", red.cpu().numpy(), want_red, 1e-5, f"long bf16 run step {step}")
    for i in range(n):
        gu.assert_same("mem", mem[i].cpu().numpy(), ref[i], 1e-6, f"long bf16 run learner {i}")
    ctx.close()


@pytest.mark.parametrize("seed", range(6))
def test_randomized_long_runs(gu, seed):
    """120 steps on a random layout (tensors of one and of several supertiles, any learner count,
    rate, beta, lr, gradient type): the ranges of the predicted pass adapt while the magnitudes pile
    up, and every step's index set and reduced values are compared."""
    rng = np.random.default_rng(50_000 + seed)
    n = int(rng.integers(2, 6))
    nt = int(rng.integers(1, 7))
    sizes = [int(rng.choice([300, 5000, 8192, 9000, 40_000, 150_000])) for _ in range(nt)]
    off0 = int(rng.integers(0, 5))
    offsets = np.concatenate([[off0], off0 + np.cumsum(sizes)]).tolist()
    numel = offsets[-1] + int(rng.integers(0, 3))
    rate = int(rng.choice([25, 100, 400]))
    ks = [max(1, s // rate) for s in sizes]
    bf16 = bool(rng.integers(0, 2))
    beta = float(rng.choice([0.1, 0.3, 1.0]))
    lr = float(rng.choice([0.1, 1.0]))
    ctx = binding.scalecom_init(numel, n, torch.bfloat16 if bf16 else torch.float32, nt, gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]
    shared = rng.standard_normal(numel)
    pool_dev = []
    for _ in range(4):
        gs = []
        for _ in range(n):
            g = torch.from_numpy(((shared + 0.5 * rng.standard_normal(numel)) * 1e-3).astype(np.float32)).to(gu.DEV)
            gs.append(g.to(torch.bfloat16) if bf16 else g)
        pool_dev.append(gs)
    pool = [[gu.to_host(g) for g in gs] for gs in pool_dev]
    what = f"seed {seed} sizes={sizes} ks={ks} n={n} bf16={bf16} beta={beta} lr={lr}"
    for step in range(120):
        idx, red = ctx.scalecom_step_layers(mem, pool_dev[step % 4], offsets, ks, beta, lr, step)
        want_idx, want_red = oracle.step_layers(ref, pool[step % 4], offsets, ks, beta, lr, step)
        gu.assert_same("idx", idx.cpu().numpy(), want_idx, None, f"{what} step {step}")
        gu.assert_same("reduced", red.cpu().numpy(), want_red, 1e-5, f"{what} step {step}")
    for i in range(n):
        gu.assert_same("mem", mem[i].cpu().numpy(), ref[i], 1e-6, f"{what} learner {i}")
    ctx.close()


@pytest.mark.parametrize("spread", [0.1, 0.9, 30.0])
def test_learners_whose_gradients_differ_in_scale(gu, spread):
    """Learners on differently distributed data: learner i's gradients are scaled by a factor of its
    own (up to 1 + spread), so the leaders' thresholds differ from step to step by as much, and a
    prediction has to follow each leader's own history.  Tensors of one and of several supertiles;
    after 90 steps the learner count changes, and with it the cycle of leaders."""
    rng = np.random.default_rng(77)
    n, beta, lr = 4, 0.1, 0.1
    sizes = [120_001, 5_000, 30_000]
    offsets = np.concatenate([[1], 1 + np.cumsum(sizes)]).tolist()
    numel = offsets[-1]
    ks = [1_200, 50, 300]
    ctx = binding.scalecom_init(numel, n, torch.float32, len(sizes), gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]
    scale = [1.0 + spread * i / (n - 1) for i in range(n)]
    pool = [[((rng.standard_normal(numel) + 0.5 * rng.standard_normal(numel)) * 1e-3 * scale[i]).astype(np.float32)
             for i in range(n)] for _ in range(5)]
    pool_dev = [[torch.from_numpy(g).to(gu.DEV) for g in gs] for gs in pool]
    for step in range(150):
        m = n if step < 90 else n - 1
        host, dev = pool[step % 5][:m], pool_dev[step % 5][:m]
        idx, red = ctx.scalecom_step_layers(mem[:m], dev, offsets, ks, beta, lr, step)
        want_idx, want_red = oracle.step_layers(ref[:m], host, offsets, ks, beta, lr, step)
        gu.assert_same("idx", idx.cpu().numpy(), want_idx, None, f"spread {spread} step {step}")
        gu.assert_same("reduced", red.cpu().numpy(), want_red, 1e-5, f"spread {spread} step {step}")
    for i in range(n):
        gu.assert_same("mem", mem[i].cpu().numpy(), ref[i], 1e-6, f"spread {spread} learner {i}")
    ctx.close()


@pytest.mark.parametrize("sigma", [0.05, 0.3])
def test_gradient_norm_that_changes_from_step_to_step(gu, sigma):
    """Every step's gradients carry a random common factor (log-normal, applied through lr), as the
    gradient norm of a minibatch does: while the memories are small the threshold follows it, so
    the range of finely counted keys grows beyond one twelve-bit bucket (coarser counts, the open
    bits resolved on the listed keys) and shrinks again as the magnitudes pile up."""
    rng = np.random.default_rng(88)
    n, beta, lr = 3, 0.1, 0.1
    sizes = [200_003, 20_000, 6_000, 70_000]
    offsets = np.concatenate([[3], 3 + np.cumsum(sizes)]).tolist()
    numel = offsets[-1] + 2
    ks = [500, 200, 60, 2_800]
    ctx = binding.scalecom_init(numel, n, torch.float32, len(sizes), gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]
    pool = [[((rng.standard_normal(numel) + 0.5 * rng.standard_normal(numel)) * 1e-3).astype(np.float32)
             for _ in range(n)] for _ in range(5)]
    pool_dev = [[torch.from_numpy(g).to(gu.DEV) for g in gs] for gs in pool]
    for step in range(220):
        lr_t = float(np.float32(lr * np.exp(rng.normal(0.0, sigma))))
        idx, red = ctx.scalecom_step_layers(mem, pool_dev[step % 5], offsets, ks, beta, lr_t, step)
        want_idx, want_red = oracle.step_layers(ref, pool[step % 5], offsets, ks, beta, lr_t, step)
        gu.assert_same("idx", idx.cpu().numpy(), want_idx, None, f"sigma {sigma} step {step}")
        gu.assert_same("reduced", red.cpu().numpy(), want_red, 1e-5, f"sigma {sigma} step {step}")
    for i in range(n):
        gu.assert_same("mem", mem[i].cpu().numpy(), ref[i], 1e-6, f"sigma {sigma} learner {i}")
    ctx.close()


# ------------------------------------------------------------------ behaviour of the boundary
def test_deterministic_and_resumable(gu):
    """Same inputs give the same bytes; stopping after 2 steps, saving the memories and
    continuing in a fresh context equals 4 steps in a row (memory is the only state)."""
    w = workloads.scaled(workloads.by_name("resnet50_sized"), 123_457, n_learners=4, steps=4)

    def run(first, last, mem):
        ctx = binding.scalecom_init(w.numel, w.n_learners, torch.float32, 1, gu.DEV)
        outs = []
        for step in range(first, last):
            idx, red = ctx.scalecom_step(mem, workloads.gradients(w, step, gu.DEV), w.k, w.beta, w.lr, step)
            outs.append((idx.cpu().numpy().copy(), red.cpu().numpy().copy()))
        ctx.close()
        return outs

    mem_a = workloads.zero_memories(w, gu.DEV)
    outs_a = run(0, 4, mem_a)
    mem_b = workloads.zero_memories(w, gu.DEV)
    outs_b = run(0, 2, mem_b)
    saved = [m.cpu() for m in mem_b]
    mem_c = [s.to(gu.DEV) for s in saved]
    outs_b += run(2, 4, mem_c)
    for (ia, ra), (ib, rb) in zip(outs_a, outs_b):
        assert ia.tobytes() == ib.tobytes() and ra.tobytes() == rb.tobytes()
    for a, c in zip(mem_a, mem_c):
        assert torch.equal(a, c)


def test_side_stream_and_changing_k(gu):
    """A context bound to a non-default stream; k and numel change between calls on one context."""
    w = workloads.scaled(workloads.by_name("tiny"), 90_001, n_learners=3, steps=1)
    stream = torch.cuda.Stream(device=gu.DEV)
    grad = workloads.gradients(w, 0, gu.DEV)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        ctx = binding.scalecom_init(w.numel, w.n_learners, torch.float32, 1, gu.DEV, stream=stream)
        for step, (numel, k) in enumerate([(90_001, 900), (90_001, 17), (4097, 4097), (90_001, 900), (12, 0)]):
            mem = [torch.zeros(numel, device=gu.DEV) for _ in range(w.n_learners)]
            g = [x[:numel].clone() for x in grad]
            ref = [np.zeros(numel, np.float32) for _ in range(w.n_learners)]
            stream.synchronize()
            gu.compare_step(ctx, mem, g, ref, step, 0.5, 0.5, k=k, what=f"numel={numel} k={k}")
        ctx.close()


def test_timing_records_a_sample_of_the_steps(gu):
    """Phase timing: every second call recorded, two boundaries or all six; results unaffected."""
    w = workloads.scaled(workloads.by_name("resnet50_sized"), 300_001, n_learners=3, steps=1)
    ctx = binding.scalecom_init(w.numel, w.n_learners, torch.float32, 1, gu.DEV)
    mem = workloads.zero_memories(w, gu.DEV)
    ref = [m.cpu().numpy().copy() for m in mem]
    grad = workloads.gradients(w, 0, gu.DEV)
    ctx.scalecom_timing_begin(10, every=2)
    for step in range(5):
        gu.compare_step(ctx, mem, grad, ref, step, w.beta, w.lr, k=w.k, what="timed")
    rec = ctx.scalecom_timing_read(10)
    assert len(rec) == 3                                    # calls 0, 2 and 4
    assert all(r[3] > 0.0 and r[0] == 0.0 and r[4] == 0.0 for r in rec)
    ctx.scalecom_timing_begin(2, all_phases=True)
    for step in range(5, 9):
        gu.compare_step(ctx, mem, grad, ref, step, w.beta, w.lr, k=w.k, what="timed all")
    rec = ctx.scalecom_timing_read(10)
    assert len(rec) == 2 and all(all(v > 0.0 for v in r) for r in rec)
    assert ctx.scalecom_timing_read(10) == []               # recording has stopped
    with pytest.raises(binding.ScaleComError):
        ctx.scalecom_timing_begin(4, every=0)
    ctx.close()


def test_argument_errors(gu):
    numel, n = 1000, 2
    ctx = binding.scalecom_init(numel, n, torch.float32, 2, gu.DEV)
    mem = [torch.zeros(numel, device=gu.DEV) for _ in range(n)]
    grad = [torch.ones(numel, device=gu.DEV) for _ in range(n)]
    before = [m.clone() for m in mem]

    def status(fn):
        with pytest.raises(binding.ScaleComError) as e:
            fn()
        return e.value.status

    E = binding.SCALECOM_EINVAL
    assert status(lambda: ctx.scalecom_step(mem, grad, numel + 1, 0.5, 0.1, 0)) == E      # k > numel
    assert status(lambda: ctx.scalecom_step(mem, grad, -1, 0.5, 0.1, 0)) == E
    assert status(lambda: ctx.scalecom_step(mem, grad, 10, 0.0, 0.1, 0)) == E             # beta outside (0, 1]
    assert status(lambda: ctx.scalecom_step(mem, grad, 10, 1.5, 0.1, 0)) == E
    assert status(lambda: ctx.scalecom_step(mem, grad, 10, float("nan"), 0.1, 0)) == E
    assert status(lambda: ctx.scalecom_step(mem, grad, 10, 0.5, float("inf"), 0)) == E
    assert status(lambda: ctx.scalecom_step(mem, grad, 10, 0.5, 0.1, -1)) == E
    assert status(lambda: ctx.scalecom_step_chunked(mem, grad, 0, 0.5, 0.1, 0)) == E      # chunk < 1
    small = binding.scalecom_init(numel, n, torch.float32, 1, gu.DEV, k_max=5)
    assert status(lambda: small.scalecom_step(mem, grad, 6, 0.5, 0.1, 0)) == E           # k > k_max of the context
    assert status(lambda: small.scalecom_step_chunked(mem, grad, 100, 0.5, 0.1, 0)) == E  # 10 chunks > k_max
    small.close()
    assert status(lambda: ctx.scalecom_step(mem * 2, grad * 2, 10, 0.5, 0.1, 0)) == E     # more learners than the context allows
    big = [torch.zeros(numel + 1, device=gu.DEV) for _ in range(n)]
    assert status(lambda: ctx.scalecom_step(big, big, 10, 0.5, 0.1, 0)) == E              # numel > numel_max
    odd = [m[1:] for m in big]                                                            # 4-byte aligned only
    assert status(lambda: ctx.scalecom_step(odd, odd, 10, 0.5, 0.1, 0)) == E
    assert status(lambda: ctx.scalecom_step_layers(mem, grad, [0, 600, 500], [1, 0], 0.5, 0.1, 0)) == E
    assert status(lambda: ctx.scalecom_step_layers(mem, grad, [0, 10, 20, 30], [1, 1, 1], 0.5, 0.1, 0)) == E
    # the binding refuses learners whose buffers differ in length, and segments that end beyond them
    short = [mem[0], mem[1][:numel - 4]]
    with pytest.raises(ValueError):
        ctx.scalecom_step(short, grad, 10, 0.5, 0.1, 0)
    with pytest.raises(ValueError):
        ctx.scalecom_step(mem, [grad[0], grad[1][:numel - 4]], 10, 0.5, 0.1, 0)
    with pytest.raises(ValueError):
        ctx.scalecom_step_layers(mem, grad, [0, 500, numel + 1], [1, 1], 0.5, 0.1, 0)
    torch.cuda.synchronize()
    for m, b in zip(mem, before):
        assert torch.equal(m, b)                                                          # a rejected call changes nothing
    with pytest.raises(binding.ScaleComError):
        binding.scalecom_init(numel, 65, torch.float32, 1, gu.DEV)
    ctx.close()
