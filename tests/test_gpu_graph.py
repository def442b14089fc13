"""A cycle of steps captured into a HIP graph and replayed.

The library keeps two things on the host that a captured graph freezes: which learner leads
(step mod n) and which of the two copies of its per-step scratch zone a step uses (they
alternate).  A graph of lcm(2, n) consecutive steps, starting at a multiple of that number, ends
in the state it started from, so it can be replayed any number of times.  Every replay is compared
with the oracle stepping through the same inputs; between replays the test overwrites the
gradient buffers eagerly and synchronises, as a training loop would.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2104_11125_amd import binding

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("chunk", [None, 100])
def test_graph_replay_of_a_step_cycle(chunk):
    import gpu_util as gu

    dev = gu.DEV
    rng = np.random.default_rng(31)
    n, numel, k, beta, lr = 3, 300_007, 3_000, 0.3, 1.0
    cycle = math.lcm(2, n)
    n_out = k if chunk is None else -(-numel // chunk)
    side = torch.cuda.Stream(device=dev)
    shared = rng.standard_normal(numel)

    def host_gradients():
        return [[((shared + 0.5 * rng.standard_normal(numel)) * 1e-3).astype(np.float32) for _ in range(n)]
                for _ in range(cycle)]

    with torch.cuda.stream(side):
        ctx = binding.scalecom_init(numel, n, torch.float32, 1, dev, stream=side, k_max=n_out)
        mem = [torch.zeros(numel, device=dev) for _ in range(n)]
        grads = [[torch.zeros(numel, device=dev) for _ in range(n)] for _ in range(cycle)]
        idx = [torch.zeros(n_out, dtype=torch.int32, device=dev) for _ in range(cycle)]
        red = [torch.zeros(n_out, dtype=torch.float32, device=dev) for _ in range(cycle)]
    ref = [np.zeros(numel, np.float32) for _ in range(n)]

    def enqueue_cycle(first_step):
        for j in range(cycle):
            if chunk is None:
                ctx.scalecom_step(mem, grads[j], k, beta, lr, first_step + j, idx[j], red[j])
            else:
                ctx.scalecom_step_chunked(mem, grads[j], chunk, beta, lr, first_step + j, idx[j], red[j])

    def check_cycle(host, first_step, what):
        side.synchronize()
        for j in range(cycle):
            if chunk is None:
                want_idx, want_red = oracle.step(ref, host[j], k, beta, lr, first_step + j)
            else:
                want_idx, want_red = oracle.step_chunked(ref, host[j], chunk, beta, lr, first_step + j)
            gu.assert_same("idx", idx[j].cpu().numpy(), want_idx, None, f"{what} step {first_step + j}")
            gu.assert_same("reduced", red[j].cpu().numpy(), want_red, 1e-5, f"{what} step {first_step + j}")
        for i in range(n):      # the memories after the whole cycle
            gu.assert_same("mem", mem[i].cpu().numpy(), ref[i], 1e-6, f"{what} learner {i}")

    def upload(host):
        with torch.cuda.stream(side):
            for j in range(cycle):
                for i in range(n):
                    grads[j][i].copy_(torch.from_numpy(host[j][i]))
        side.synchronize()

    # one eager cycle first: tables uploaded, scratch cleared, predictions in place
    host = host_gradients()
    upload(host)
    with torch.cuda.stream(side):
        enqueue_cycle(0)
    check_cycle(host, 0, "eager")

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue_cycle(cycle)                        # recorded, not run
    for r in range(1, 4):
        host = host_gradients()
        upload(host)                                # eager work and a synchronisation between replays
        graph.replay()
        check_cycle(host, r * cycle, f"replay {r}")
    ctx.close()
