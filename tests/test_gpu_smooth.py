"""GPU parity of the step with iteration smoothing over several steps of a block, through the C-ABI, against the
oracle.  Teacher-forced: after every step the oracle continues from the GPU's tokens, mask and retained expected
embeddings."""
import numpy as np
import pytest

import dinfer_inputs as di
import oracle
from harness import GpuRun, OracleRun, bars_for, check_routing, compare_logits, compare_step, make_case

pytestmark = pytest.mark.gpu


def _variant(name):
    tiny = di.model_preset("tiny")
    W = di.Workload
    sc = di.configs.scaled
    return {
        "c1": W("c1", tiny, 1, 32, 64, 64, threshold=0.9, seed_index=1),
        "c1_bf16": W("c1_bf16", sc(tiny, dtype="bf16"), 1, 32, 64, 64, threshold=0.9, seed_index=1),
        # two sequences, ragged block: 2 x 20 tokens, two token tiles
        "pair": W("pair", tiny, 2, 20, 30, 50, threshold=0.9, seed_index=6),
        # a vocabulary that is not a multiple of anything (padding of the contraction)
        "odd_vocab": W("odd_vocab", sc(tiny, vocab=1000), 1, 32, 40, 40, threshold=0.9, seed_index=9),
    }[name]


@pytest.fixture(scope="module", params=["c1", "c1_bf16", "pair", "odd_vocab"])
def case(request):
    wl = _variant(request.param)
    cfg, w, inp = make_case(wl)
    ns, S = inp.block_tokens.shape
    cap = int(inp.prefix_len.max()) + 2 * S + 16
    ora = OracleRun(cfg, w, inp, cap)
    gpu = GpuRun(cfg, w, inp, ns * S, cap)
    yield wl, cfg, inp, ora, gpu, bars_for(cfg)
    gpu.close()


def test_smoothing_steps_match_oracle(case):
    wl, cfg, inp, ora, g, bars = case
    ns, S = inp.block_tokens.shape
    H = cfg.hidden
    g.inject_prefix(ora.caches)
    sm = g.smooth_state()
    tokens, masks = inp.block_tokens.copy(), inp.mask_bits.copy()
    delta_tol = 2e-3 if cfg.dtype == "f32" else 8e-2       # relative to the row's largest |delta|
    fixed_k = 3
    moved = False
    for step in range(4):
        alpha = (0.0, 0.4, 0.7, 1.0)[step]      # large, so that the effect on the logits clears the bf16 tolerance
        delta_in = sm["delta"].cpu().numpy().astype(np.float64)
        g.set_state(tokens, masks, inp.prefix_len)
        got = g.step_smooth(sm, alpha, 0.5, fixed_k)
        delta_out = sm["delta"].cpu().numpy()
        logits = g.logits(ns * S).reshape(ns, S, -1)
        routing = g.routing().reshape(cfg.n_layers, ns, S, cfg.top_k)
        for s in range(ns):
            kc, vc = ora.caches[s]
            keep = kc.copy(), vc.copy()
            P = int(inp.prefix_len[s])
            d = np.ascontiguousarray(delta_in[s])
            tr = oracle.Trace(cfg, S, forced_idx=routing[:, s])
            ref = ora.o.step_smooth(tokens[s], int(masks[s]), P, kc, vc, 0.5, alpha, d, fixed_k, want_logits=True, trace=tr)
            check_routing(tr, routing[:, s], cfg.top_k, bars)
            compare_logits(ref["logits"], logits[s], bars)
            compare_step(ref, got["tokens"][s], got["mask"][s], got["conf"][s], got["argmax"][s], got["n_committed"][s],
                         tokens[s], masks[s], 0.5, fixed_k, bars, ref["logits"])
            for i in range(S):
                if (int(masks[s]) >> i) & 1:
                    scale = np.abs(d[i]).max()
                    assert np.abs(delta_out[s, i] - d[i]).max() <= delta_tol * scale, (step, s, i)
                else:
                    assert np.array_equal(delta_out[s, i], delta_in[s, i].astype(np.float32)), "a decided row moved"
            if step > 0:
                plain = ora.o.step(tokens[s], int(masks[s]), P, kc, vc, 2.0, want_logits=True)["logits"]
                kc[...], vc[...] = keep
                if np.abs(plain - ref["logits"]).max() > 3 * bars.logit_rel * np.abs(plain).max():
                    moved = True
            kc[...], vc[...] = keep
        tokens, masks = got["tokens"].copy(), got["mask"].copy()
    assert moved, "the retained embeddings never changed the logits: the test does not exercise the smoothing"


def test_alpha_zero_equals_the_plain_step(case):
    wl, cfg, inp, ora, g, bars = case
    ns, S = inp.block_tokens.shape
    g.inject_prefix(ora.caches)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    a = g.step(0.05)
    la = g.logits(ns * S)
    sm = g.smooth_state()
    sm["delta"].fill_(0.37)                    # ignored with alpha = 0
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    b = g.step_smooth(sm, 0.0, 0.05)
    assert np.array_equal(la, g.logits(ns * S))
    for key in ("tokens", "mask", "conf", "argmax", "n_committed"):
        assert np.array_equal(a[key], b[key]), key


def test_bad_arguments(case):
    wl, cfg, inp, ora, g, bars = case
    from paper_2510_08666_amd.binding import DinferError
    sm = g.smooth_state()
    with pytest.raises(DinferError):
        g.step_smooth(sm, -0.1, 0.5)
    small = dict(delta=sm["delta"], scratch=sm["scratch"][:4096])
    with pytest.raises(DinferError):
        g.step_smooth(small, 0.1, 0.5)
