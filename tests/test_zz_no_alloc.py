"""scalecom_step_static, the entry point for callers that cannot allocate: its workspace is a
static device array of the library.  Checked through the C-ABI against scalecom_step (the entry
point it is a variant of) on the same inputs, bit for bit: index set, reduced values and every
learner's memory; two calls in a row with the second one smaller, then runs with the memory
carried (so the predictions kept in the static array are in use), bfloat16 gradients, and the
size limits.  Runs last: the array is shared by every call in the process.
"""
import numpy as np
import pytest
import torch

from paper_2104_11125_amd import binding, workloads

pytestmark = pytest.mark.gpu


def _both(gu, ctx, w, mem_s, mem_c, step, what):
    """One step through scalecom_step_static (on mem_s) and through scalecom_step (on mem_c)."""
    grad = workloads.gradients(w, step, gu.DEV)
    idx_s = torch.full((w.k,), -1, dtype=torch.int32, device=gu.DEV)
    red_s = torch.full((w.k,), float("nan"), dtype=torch.float32, device=gu.DEV)
    # (allocation events, not bytes in use: a garbage collection during the call may free earlier tests' tensors)
    before = torch.cuda.memory_stats(gu.DEV)["allocation.all.allocated"]
    print(f"[static] {what}: n={w.n_learners} numel={w.numel} k={w.k} step={step}", flush=True)
    binding.scalecom_step_static(mem_s, grad, w.k, w.beta, w.lr, step, idx_s, red_s)
    assert torch.cuda.memory_stats(gu.DEV)["allocation.all.allocated"] == before
    idx_c, red_c = ctx.scalecom_step(mem_c, grad, w.k, w.beta, w.lr, step)
    torch.cuda.synchronize()
    gu.assert_same("idx", idx_s.cpu().numpy(), idx_c.cpu().numpy(), None, f"{what} step {step}")
    gu.assert_same("reduced", red_s.cpu().numpy(), red_c.cpu().numpy(), 1e-5, f"{what} step {step}")
    for i, (a, b) in enumerate(zip(mem_s, mem_c)):
        gu.assert_same("mem", a.cpu().numpy(), b.cpu().numpy(), 1e-6, f"{what} step {step} learner {i}")


def _start(gu, w, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    mem_s = [(2e-4 * torch.randn(w.numel, generator=g)).to(gu.DEV) for _ in range(w.n_learners)]
    mem_c = [m.clone() for m in mem_s]
    gd = torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32
    return mem_s, mem_c, binding.scalecom_init(w.numel, w.n_learners, gd, 1, gu.DEV, k_max=w.k)


def test_static_workspace_step_matches_scalecom_step():
    import gpu_util as gu

    large = workloads.scaled(workloads.by_name("tiny"), 1_000_003, n_learners=4, steps=1)
    small = workloads.scaled(workloads.by_name("resnet50_sized"), 200_001, n_learners=3, steps=1)
    # two calls in a row, the second with a smaller input
    ms_l, mc_l, ctx_l = _start(gu, large, 1)
    ms_s, mc_s, ctx_s = _start(gu, small, 2)
    _both(gu, ctx_l, large, ms_l, mc_l, 0, "first call")
    _both(gu, ctx_s, small, ms_s, mc_s, 0, "second call, smaller")
    # memory carried over several steps at one size: the predictions kept in the static array are used
    for step in range(1, 7):
        _both(gu, ctx_s, small, ms_s, mc_s, step, "smaller, carried")
    # back to the larger size (its tables and predictions were dropped in between), then alternating
    for step in range(1, 4):
        _both(gu, ctx_l, large, ms_l, mc_l, step, "larger again")
    _both(gu, ctx_s, small, ms_s, mc_s, 7, "alternating")
    _both(gu, ctx_l, large, ms_l, mc_l, 4, "alternating")
    ctx_l.close()
    ctx_s.close()
    # bfloat16 gradients, the largest length the array takes, k = 0 and k at the limit
    L = binding.lib()
    assert (binding.SCALECOM_STATIC_NUMEL_MAX, binding.SCALECOM_STATIC_LEARNERS_MAX, binding.SCALECOM_STATIC_K_MAX) == \
        (4_194_304, 8, 131_072)
    full = workloads.Workload("static_full", 5, 8, binding.SCALECOM_STATIC_NUMEL_MAX, 32, 0.5, "normal", 0.1, 0.1, 1, "bf16")
    assert full.k == binding.SCALECOM_STATIC_K_MAX
    ms, mc, ctx = _start(gu, full, 3)
    for step in range(3):
        _both(gu, ctx, full, ms, mc, step, "largest, bf16")
    ctx.close()
    none = workloads.Workload("static_k0", 1, 2, 70_001, 10 ** 9, 0.5, "normal", 0.1, 0.1, 1)
    assert none.k == 0
    ms, mc, ctx = _start(gu, none, 4)
    _both(gu, ctx, none, ms, mc, 0, "k = 0")
    ctx.close()
    # sizes beyond the array are refused, with the limit named, and nothing is touched
    n = binding.SCALECOM_STATIC_NUMEL_MAX + 1
    big = [torch.zeros(n, device=gu.DEV)]
    out_i = torch.zeros(8, dtype=torch.int32, device=gu.DEV)
    out_r = torch.zeros(8, dtype=torch.float32, device=gu.DEV)
    with pytest.raises(binding.ScaleComError) as e:
        binding.scalecom_step_static(big, big, 8, 0.5, 0.1, 0, out_i, out_r)
    assert e.value.status == binding.SCALECOM_EINVAL and "SCALECOM_STATIC_NUMEL_MAX" in str(e.value)
    nine = [torch.zeros(1000, device=gu.DEV) for _ in range(9)]
    with pytest.raises(binding.ScaleComError) as e:
        binding.scalecom_step_static(nine, nine, 8, 0.5, 0.1, 0, out_i, out_r)
    assert "SCALECOM_STATIC_LEARNERS_MAX" in str(e.value)
    wide = [torch.zeros(binding.SCALECOM_STATIC_NUMEL_MAX, device=gu.DEV)]
    many = binding.SCALECOM_STATIC_K_MAX + 1
    with pytest.raises(binding.ScaleComError) as e:
        binding.scalecom_step_static(wide, wide, many, 0.5, 0.1, 0, torch.zeros(many, dtype=torch.int32, device=gu.DEV),
                                     torch.zeros(many, dtype=torch.float32, device=gu.DEV))
    assert "SCALECOM_STATIC_K_MAX" in str(e.value)
    assert L.scalecom_last_error(None) != b""
    torch.cuda.synchronize()
    assert not big[0].any() and not out_i.any()


def test_static_workspace_step_replayed_as_graphs():
    """One of the callers the entry point is for: code under HIP graph capture.  After one eager cycle
    (the first call on a device looks the array up, the first call with a layout writes its tables) a
    step per leader is captured and replayed with new gradients; every step is compared with
    scalecom_step on a copy of the memories."""
    import gpu_util as gu

    w = workloads.scaled(workloads.by_name("resnet50_sized"), 300_007, n_learners=3, steps=1)
    n = w.n_learners
    side = torch.cuda.Stream(device=gu.DEV)
    ms, mc, ctx = _start(gu, w, 5)
    grads = [torch.zeros(w.numel, device=gu.DEV) for _ in range(n)]
    idx_s = torch.full((w.k,), -1, dtype=torch.int32, device=gu.DEV)
    red_s = torch.full((w.k,), float("nan"), dtype=torch.float32, device=gu.DEV)

    def upload(step):
        for dst, src in zip(grads, workloads.gradients(w, step, gu.DEV)):
            dst.copy_(src)
        torch.cuda.synchronize()

    def check(step, what):
        side.synchronize()
        idx_c, red_c = ctx.scalecom_step(mc, grads, w.k, w.beta, w.lr, step)
        torch.cuda.synchronize()
        gu.assert_same("idx", idx_s.cpu().numpy(), idx_c.cpu().numpy(), None, f"{what} step {step}")
        gu.assert_same("reduced", red_s.cpu().numpy(), red_c.cpu().numpy(), 1e-5, f"{what} step {step}")
        for i, (a, b) in enumerate(zip(ms, mc)):
            gu.assert_same("mem", a.cpu().numpy(), b.cpu().numpy(), 1e-6, f"{what} step {step} learner {i}")

    for step in range(n):
        upload(step)
        print(f"[static] eager step {step} before the capture", flush=True)
        binding.scalecom_step_static(ms, grads, w.k, w.beta, w.lr, step, idx_s, red_s, stream=side)
        check(step, "eager")
    graphs = []
    for leader in range(n):                             # recorded, not run
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            binding.scalecom_step_static(ms, grads, w.k, w.beta, w.lr, n + leader, idx_s, red_s, stream=side)
        graphs.append(g)
    for step in range(n, 4 * n):
        upload(step)                                    # eager work and a synchronisation between replays
        print(f"[static] replay of leader {step % n}'s graph, step {step}", flush=True)
        graphs[step % n].replay()
        check(step, "replay")
    ctx.close()
