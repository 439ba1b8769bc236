"""The per-launch stage profile of the library (a benchmark aid, no part of the method): every launch of the chosen
stage inside the sampled forwards is bracketed by an event pair, the sampling takes every n-th forward, and a step
gives the same bits with and without the brackets."""
import pytest

import dinfer_inputs as di
from harness import GpuRun, OracleRun, make_case
from paper_2510_08666_amd import binding

pytestmark = pytest.mark.gpu


def test_profile_counts_and_sampling():
    import torch
    tiny = di.model_preset("tiny")
    wl = di.Workload("c1", tiny, 1, 32, 64, 64, seed_index=1)
    cfg, w, inp = make_case(wl)
    ns, S = inp.block_tokens.shape
    cap = int(inp.prefix_len.max()) + S + 16
    ora = OracleRun(cfg, w, inp, cap)
    g = GpuRun(cfg, w, inp, ns * S, cap)
    g.inject_prefix(ora.caches)
    tok0, mask0 = g.tokens.clone(), g.mask.clone()

    def steps(n):
        for _ in range(n):
            g.tokens.copy_(tok0)
            g.mask.copy_(mask0)
            g.ctx.step(g.tokens, g.mask, g.prefix_len, g.page_table, 0.9, 0, g.conf, g.argmax, g.n_committed)
        torch.cuda.synchronize()
        return [t.clone() for t in (g.tokens, g.mask, g.conf, g.argmax, g.n_committed)]

    plain = steps(1)
    g.ctx.profile_start(binding.STAGE_EXPERT_GATE_UP)           # default: every forward
    timed = steps(3)
    n, ms = g.ctx.profile_stop()
    assert n == 3 * cfg.n_layers and ms > 0.0
    for a, b in zip(plain, timed):
        assert torch.equal(a, b)

    g.ctx.profile_every(3)
    g.ctx.profile_start(binding.STAGE_EXPERT_GATE_UP)
    timed = steps(7)                                            # forwards 0, 3 and 6 are sampled
    n, ms = g.ctx.profile_stop()
    assert n == 3 * cfg.n_layers and ms > 0.0
    for a, b in zip(plain, timed):
        assert torch.equal(a, b)

    g.ctx.profile_start(binding.STAGE_LM_HEAD)                  # the setting stays; one LM-head launch per step
    steps(4)                                                    # forwards 0 and 3
    n, ms = g.ctx.profile_stop()
    assert n == 2

    g.ctx.profile_every(1)
    with pytest.raises(binding.DinferError):
        g.ctx.profile_every(0)
    with pytest.raises(binding.DinferError):
        g.ctx.profile_stop()                                    # no profile running
    g.close()
