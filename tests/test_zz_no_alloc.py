"""The allocation-free variant of the smoothing step (dinfer_step_smooth_static) against dinfer_step_smooth, through
the C-ABI: same kernels, so every output must be equal bit for bit.  Two calls in a row share the static scratch, the
second with a smaller input (fewer block tokens, then also a smaller vocabulary): what the first call left behind
must not leak into the second."""
import numpy as np
import pytest

import dinfer_inputs as di
from harness import GpuRun, OracleRun, make_case

pytestmark = pytest.mark.gpu


def _run_pair(wl, alpha, fixed_k=3, steps=2):
    """`steps` smoothing steps of a block through both entry points from the same start; returns the two traces."""
    cfg, w, inp = make_case(wl)
    ns, S = inp.block_tokens.shape
    cap = int(inp.prefix_len.max()) + 2 * S + 16
    g = GpuRun(cfg, w, inp, max(ns * S, int(sum(len(t) for t in inp.prefix_tokens))), cap)
    if inp.prefix_len.max() > 0:
        g.prefill()
    torch = g.torch
    rng = np.random.default_rng(11)
    delta0 = (cfg.init_std * rng.standard_normal((ns, S, cfg.hidden))).astype(np.float32)
    traces = []
    for static in (False, True):
        g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
        delta = torch.from_numpy(delta0.copy()).to(g.dev)
        scratch = None if static else g.ctx.smooth_scratch(ns * S)
        out = []
        for _ in range(steps):
            if static:
                g.ctx.step_smooth_static(g.tokens, g.mask, g.prefix_len, g.page_table, 0.5, fixed_k, alpha, delta, g.conf,
                                         g.argmax, g.n_committed)
            else:
                g.ctx.step_smooth(g.tokens, g.mask, g.prefix_len, g.page_table, 0.5, fixed_k, alpha, delta, scratch,
                                  g.conf, g.argmax, g.n_committed)
            torch.cuda.synchronize()
            st = g.state()
            st["delta"] = delta.cpu().numpy()
            out.append(st)
        traces.append(out)
    g.close()
    return traces


def _assert_equal(traces):
    plain, static = traces
    for a, b in zip(plain, static):
        for key in ("tokens", "mask", "conf", "argmax", "n_committed", "delta"):
            assert np.array_equal(a[key], b[key]), key
        assert a["n_committed"].sum() > 0


def test_static_scratch_two_calls_second_smaller():
    tiny = di.model_preset("tiny")
    big = di.Workload("na_big", tiny, 2, 32, 30, 50, threshold=0.9, seed_index=41)                 # 64 tokens, vocab 4096
    small = di.Workload("na_small", di.configs.scaled(tiny, vocab=1000, dtype="bf16"), 1, 20, 40, 40,
                        threshold=0.9, seed_index=42)                                              # 20 tokens, vocab 1000
    _assert_equal(_run_pair(big, 0.4))
    _assert_equal(_run_pair(small, 0.7))
    # and the large one again behind the small one
    _assert_equal(_run_pair(big, 0.4))


def test_static_scratch_rejects_what_does_not_fit():
    from paper_2510_08666_amd import binding
    from paper_2510_08666_amd.binding import DinferError
    cfg = di.configs.scaled(di.model_preset("tiny"), vocab=400000)      # 64 tokens x 400000 ids of float32 logits: 102 MB
    wl = di.Workload("na_huge", cfg, 2, 32, 0, 0, threshold=0.9, seed_index=43)
    inp = di.make_workload_inputs(wl)
    g_cfg = binding.make_config(cfg, 128)
    assert binding.lib.dinfer_smooth_scratch_bytes(g_cfg, 64) > (48 << 20)
    import torch
    ctx = binding.Context(cfg, inp.n_pages, 2, 64, 128)     # weights stay uninitialised: the call must be refused before any launch
    dev = ctx.device
    tokens = torch.from_numpy(inp.block_tokens.copy()).to(dev)
    mask = torch.from_numpy(inp.mask_bits.view(np.int64).copy()).to(dev)
    prefix = torch.zeros(2, dtype=torch.int32, device=dev)
    pt = torch.from_numpy(inp.page_table).to(dev)
    delta = torch.zeros((2, 32, cfg.hidden), dtype=torch.float32, device=dev)
    conf = torch.zeros((2, 32), dtype=torch.float32, device=dev)
    am = torch.zeros((2, 32), dtype=torch.int32, device=dev)
    nc = torch.zeros(2, dtype=torch.int32, device=dev)
    with pytest.raises(DinferError) as e:
        ctx.step_smooth_static(tokens, mask, prefix, pt, 0.5, 0, 0.3, delta, conf, am, nc)
    assert e.value.code == -3 and "static scratch" in str(e.value)
    ctx.close()
