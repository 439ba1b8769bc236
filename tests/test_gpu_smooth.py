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
        # more than 64 tokens: the contraction over the vocabulary in its many-token form (5 x 32 tokens: three
        # groups of 64, the last ragged), in both storage types.  (Above 64 tokens the LM head feeds the matrix cores
        # activations rounded to one bf16 plane; at the tiny preset's logit scale of 8 that rounding alone moves a
        # confidence by more than the bar, so the bf16 case runs at a scale of 2.)
        "many": W("many", tiny, 5, 32, 20, 60, threshold=0.9, seed_index=31),
        "many_bf16": W("many_bf16", sc(tiny, dtype="bf16", logit_scale=2.0), 5, 32, 20, 60, threshold=0.9, seed_index=31),
    }[name]


@pytest.fixture(scope="module", params=["c1", "c1_bf16", "pair", "odd_vocab", "many", "many_bf16"])
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


def _schedules(t, sched, target):
    """Appendix "IterSmooth", for step t of a block (0 first): the weight of what step t-1 retained, alpha_{t-1} =
    min(alpha_init + alpha_growth * (t-1), alpha_preset) (nothing is retained before step 0), and the decode
    threshold, which decays from its start value towards the target (linearly, floored at the target)."""
    a_init, a_growth, a_preset, th_start, th_decay = sched
    alpha = 0.0 if t == 0 else min(a_init + a_growth * (t - 1), a_preset)
    return np.float32(alpha), max(np.float32(th_start) - np.float32(th_decay) * np.float32(t), np.float32(target))


@pytest.mark.parametrize("steps_per_wait", [1, 5])
def test_block_under_the_schedules_equals_its_steps_one_by_one(case, steps_per_wait):
    """dinfer_generate_block_smooth against the same steps issued one at a time with the schedule values worked out
    here from the appendix: same kernels, so the same bits, and the same number of steps."""
    wl, cfg, inp, ora, g, bars = case
    ns, S = inp.block_tokens.shape
    sched, target = (0.1, 0.05, 0.3, 1.0, 0.2), 0.3
    g.inject_prefix(ora.caches)
    # one at a time
    sm = g.smooth_state()
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    manual, t = [], 0
    while True:
        alpha, tau = _schedules(t, sched, target)
        st = g.step_smooth(sm, float(alpha), float(tau))
        manual.append(st)
        t += 1
        if not st["mask"].any():
            break
        assert t < 4 * S
    delta_manual = sm["delta"].clone()
    # the loop
    sm2 = g.smooth_state()
    sm2["delta"].fill_(123.0)                   # needs no initial contents
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    n = g.ctx.generate_block_smooth(g.tokens, g.mask, g.prefix_len, g.page_table, target, sched, sm2["delta"],
                                    sm2["scratch"], g.conf, g.argmax, g.n_committed, 4 * S, steps_per_wait)
    g.torch.cuda.synchronize()
    got = g.state()
    assert n == len(manual), "steps: %d in the loop, %d one by one" % (n, len(manual))
    for key in ("tokens", "mask", "conf", "argmax", "n_committed"):
        assert np.array_equal(got[key], manual[-1][key]), key
    masked0 = np.array([[(int(inp.mask_bits[s]) >> i) & 1 for i in range(S)] for s in range(ns)], dtype=bool)
    assert g.torch.equal(sm2["delta"][g.torch.from_numpy(masked0).to(g.dev)],
                         delta_manual[g.torch.from_numpy(masked0).to(g.dev)])
    # the thresholds did decay: the block took more than one step, and fewer than one per position
    print("schedule block: %d steps for %d masked positions" % (n, int(masked0.sum())))
    assert 1 < n


def test_schedule_loop_bad_arguments(case):
    wl, cfg, inp, ora, g, bars = case
    from paper_2510_08666_amd.binding import DinferError
    sm = g.smooth_state()
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    args = (g.tokens, g.mask, g.prefix_len, g.page_table)
    tail = (sm["delta"], sm["scratch"], g.conf, g.argmax, g.n_committed)
    with pytest.raises(DinferError):      # start below the target
        g.ctx.generate_block_smooth(*args, 0.5, (0.1, 0.05, 0.3, 0.4, 0.1), *tail, 8)
    with pytest.raises(DinferError):      # preset below init
        g.ctx.generate_block_smooth(*args, 0.5, (0.3, 0.05, 0.1, 1.0, 0.1), *tail, 8)
    with pytest.raises(DinferError):      # too many steps
        g.ctx.generate_block_smooth(*args, 0.5, (0.1, 0.05, 0.3, 1.0, 0.1), *tail, 1000)
