"""Single steps captured into HIP graphs and replayed.

A step enqueues kernels only (once its layout's tables are on the device), and everything it
needs from earlier steps lives in device memory, so one captured step can be replayed for any later
step with the same leader: the leader (step mod n) is the one thing the host decides at enqueue
time.  The test captures one graph per leader and drives a training-like loop with them: new
gradients are written into the captured buffers eagerly, with a synchronisation, between replays,
one step of every cycle is enqueued eagerly instead of replayed, and every step is compared with
the oracle stepping through the same inputs.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_11125_amd import binding

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("chunk,layered", [(None, False), (100, False), (None, True)])
def test_graph_replay_of_single_steps(chunk, layered):
    """layered: per-tensor index sets, with tensors of one supertile among them (their search runs
    on the context's second stream, which the capture has to follow)."""
    import gpu_util as gu

    dev = gu.DEV
    rng = np.random.default_rng(31)
    n, numel, k, beta, lr = 3, 300_007, 3_000, 0.3, 1.0
    sizes = [5_000, 300, 120_000, 8_192, 70_000, 64, 96_451]
    offsets = np.concatenate([[0], np.cumsum(sizes)]).tolist()
    ks = [-(-sz // 100) for sz in sizes]
    assert offsets[-1] == numel
    if layered:
        k = sum(ks)
    n_out = k if chunk is None else -(-numel // chunk)
    side = torch.cuda.Stream(device=dev)
    shared = rng.standard_normal(numel)

    def host_gradients():
        return [((shared + 0.5 * rng.standard_normal(numel)) * 1e-3).astype(np.float32) for _ in range(n)]

    with torch.cuda.stream(side):
        ctx = binding.scalecom_init(numel, n, torch.float32, len(sizes) if layered else 1, dev, stream=side, k_max=n_out)
        mem = [torch.zeros(numel, device=dev) for _ in range(n)]
        grads = [torch.zeros(numel, device=dev) for _ in range(n)]
        idx = torch.zeros(n_out, dtype=torch.int32, device=dev)
        red = torch.zeros(n_out, dtype=torch.float32, device=dev)
    ref = [np.zeros(numel, np.float32) for _ in range(n)]

    def enqueue(step):
        if layered:
            ctx.scalecom_step_layers(mem, grads, offsets, ks, beta, lr, step, idx, red)
        elif chunk is None:
            ctx.scalecom_step(mem, grads, k, beta, lr, step, idx, red)
        else:
            ctx.scalecom_step_chunked(mem, grads, chunk, beta, lr, step, idx, red)

    def check(host, step, what):
        side.synchronize()
        if layered:
            want_idx, want_red = oracle.step_layers(ref, host, offsets, ks, beta, lr, step)
        elif chunk is None:
            want_idx, want_red = oracle.step(ref, host, k, beta, lr, step)
        else:
            want_idx, want_red = oracle.step_chunked(ref, host, chunk, beta, lr, step)
        gu.assert_same("idx", idx.cpu().numpy(), want_idx, None, f"{what} step {step}")
        gu.assert_same("reduced", red.cpu().numpy(), want_red, 1e-5, f"{what} step {step}")
        for i in range(n):
            gu.assert_same("mem", mem[i].cpu().numpy(), ref[i], 1e-6, f"{what} step {step} learner {i}")

    def upload(host):
        with torch.cuda.stream(side):
            for i in range(n):
                grads[i].copy_(torch.from_numpy(host[i]))
        side.synchronize()

    # one eager cycle first: tables uploaded, scratch cleared, predictions in place
    for step in range(n):
        host = host_gradients()
        upload(host)
        with torch.cuda.stream(side):
            enqueue(step)
        check(host, step, "eager")

    graphs = []
    for leader in range(n):                             # recorded, not run: one step per leader
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            enqueue(n + leader)
        graphs.append(g)
    for step in range(n, 5 * n):
        host = host_gradients()
        upload(host)                                    # eager work and a synchronisation between replays
        if step % (n + 1) == 0:                         # now and then an eager step between the replays
            with torch.cuda.stream(side):
                enqueue(step)
            check(host, step, "eager between replays")
        else:
            graphs[step % n].replay()
            check(host, step, f"replay of leader {step % n}'s graph")
    ctx.close()
