"""A denoising step recorded into a HIP graph (the paper runs its iterations under CUDA Graphs, Section 3): the entry
points only enqueue kernels on the caller's stream (no allocation, no wait, no memset), so a step can be captured.
The graph is replayed several times with eager steps and synchronisations in between, and every replay must give
the eager step's bits."""
import numpy as np
import pytest

import dinfer_inputs as di
from harness import GpuRun, OracleRun, make_case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["c1", "batch_bf16"])
def test_captured_step_replays_bit_exact(name):
    import torch
    tiny = di.model_preset("tiny")
    wl = {"c1": di.Workload("c1", tiny, 1, 32, 64, 64, seed_index=1),
          "batch_bf16": di.Workload("batch_bf16", di.configs.scaled(tiny, dtype="bf16", logit_scale=1.0), 3, 64, 17, 140,
                                    precommit=True, seed_index=8)}[name]
    cfg, w, inp = make_case(wl)
    ns, S = inp.block_tokens.shape
    cap = int(inp.prefix_len.max()) + S + 16
    ora = OracleRun(cfg, w, inp, cap)
    g = GpuRun(cfg, w, inp, ns * S, cap)
    g.inject_prefix(ora.caches)
    tok0, mask0 = g.tokens.clone(), g.mask.clone()

    def one(threshold):
        g.tokens.copy_(tok0)
        g.mask.copy_(mask0)
        g.ctx.step(g.tokens, g.mask, g.prefix_len, g.page_table, threshold, 0, g.conf, g.argmax, g.n_committed)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (g.tokens, g.mask, g.conf, g.argmax, g.n_committed)]

    one(0.05)
    eager = snapshot()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one(0.05)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one(0.05)
    for rep in range(4):
        one(0.9)                                    # eager work with another threshold between the replays
        other = snapshot()
        graph.replay()
        got = snapshot()
        for a, b in zip(eager, got):
            assert torch.equal(a, b), rep
        assert not torch.equal(other[1], got[1]) or torch.equal(other[0], got[0])
    g.close()
