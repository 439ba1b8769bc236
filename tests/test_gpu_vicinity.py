"""GPU parity of the step with vicinity KV-cache refresh (the look_back cached positions before the block are
recomputed with it and their K,V rows rewritten), through the C-ABI, element by element against the oracle."""
import numpy as np
import pytest

import dinfer_inputs as di
from harness import kv_close, GpuRun, OracleRun, bars_for, compare_logits, compare_step, make_case, max_abs_err

pytestmark = pytest.mark.gpu

LOOK_BACK = 16       # the window of the paper's experiments


def _variant(name):
    tiny = di.model_preset("tiny")
    W = di.Workload
    sc = di.configs.scaled
    return {
        "c1": W("c1", tiny, 1, 32, 64, 64, threshold=0.9, seed_index=1),
        "c1_bf16": W("c1_bf16", sc(tiny, dtype="bf16", logit_scale=1.0), 1, 32, 64, 64, threshold=0.9, seed_index=1),
        # ragged block and prefix
        "ragged": W("ragged", tiny, 1, 20, 50, 50, threshold=0.9, seed_index=6),
        # several sequences, block 64 half decided: 80 tokens per sequence, the many-token kernel forms
        "batch": W("batch", tiny, 5, 64, 17, 140, precommit=True, threshold=0.9, seed_index=7),
        "batch_bf16": W("batch_bf16", sc(tiny, dtype="bf16", logit_scale=1.0), 3, 64, 17, 140, precommit=True,
                        threshold=0.9, seed_index=8),
    }[name]


@pytest.fixture(scope="module", params=["c1", "c1_bf16", "ragged", "batch", "batch_bf16"])
def case(request):
    wl = _variant(request.param)
    cfg, w, inp = make_case(wl)
    ns, S = inp.block_tokens.shape
    cap = int(inp.prefix_len.max()) + 2 * S + 16
    ora = OracleRun(cfg, w, inp, cap)
    gpu = GpuRun(cfg, w, inp, ns * (S + LOOK_BACK), cap)
    yield wl, cfg, inp, ora, gpu, bars_for(cfg)
    gpu.close()


@pytest.mark.parametrize("look_back", [LOOK_BACK, 1])
def test_vicinity_step_matches_oracle(case, look_back):
    wl, cfg, inp, ora, g, bars = case
    ns, S = inp.block_tokens.shape
    run = look_back + S
    vic = np.stack([inp.prefix_tokens[s][int(inp.prefix_len[s]) - look_back:] for s in range(ns)])
    g.inject_prefix(ora.caches)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    probe = g.step_vicinity(vic, 2.0)
    tau = float(np.median(probe["conf"]))          # several positions commit
    g.inject_prefix(ora.caches)                    # the probe rewrote the neighbours' rows
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    got = g.step_vicinity(vic, tau)
    logits = g.logits(ns * run).reshape(ns, run, -1)[:, look_back:]
    routing = g.routing(ns * run).reshape(cfg.n_layers, ns, run, cfg.top_k)
    for s in range(ns):
        kc, vc = ora.caches[s]
        keep = kc.copy(), vc.copy()
        P = int(inp.prefix_len[s])
        ref, near = ora.step_vicinity_following(s, inp.block_tokens[s], vic[s], int(inp.mask_bits[s]), P, tau, 0,
                                                routing[:, s], bars)
        assert near <= max(1, cfg.n_layers * run // 4)
        compare_logits(ref["logits"], logits[s], bars)
        compare_step(ref, got["tokens"][s], got["mask"][s], got["conf"][s], got["argmax"][s], got["n_committed"][s],
                     inp.block_tokens[s], inp.mask_bits[s], tau, 0, bars, ref["logits"])
        for l in range(cfg.n_layers):
            k, v = g.read_kv(s, l, 0, P + S)
            # neighbours and block as the step rewrote them
            assert kv_close(k[P - look_back:], kc[l, P - look_back:P + S], bars)
            assert kv_close(v[P - look_back:], vc[l, P - look_back:P + S], bars)
            # everything before the neighbourhood untouched (bit for bit)
            ref_k, ref_v = keep[0][l, :P - look_back].astype(np.float32), keep[1][l, :P - look_back].astype(np.float32)
            if cfg.dtype == "bf16":
                ref_k, ref_v = di.bf16_to_f32(di.f32_to_bf16(ref_k)), di.bf16_to_f32(di.f32_to_bf16(ref_v))
            assert np.array_equal(k[:P - look_back], ref_k) and np.array_equal(v[:P - look_back], ref_v)
        # the neighbours' rows really moved (the prompt-only prefill had not seen the block)
        if look_back > 1:
            assert np.abs(kc[1, P - look_back:P] - keep[0][1, P - look_back:P]).max() > 1e-6
        kc[...], vc[...] = keep


def test_without_neighbours_equals_the_plain_step(case):
    wl, cfg, inp, ora, g, bars = case
    ns, S = inp.block_tokens.shape
    g.inject_prefix(ora.caches)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    a = g.step(0.05)
    la = g.logits(ns * S)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    b = g.step_vicinity(np.zeros((ns, 0), np.int32), 0.05)
    lb = g.logits(ns * S)
    assert np.array_equal(la, lb)
    for key in ("tokens", "mask", "conf", "argmax", "n_committed"):
        assert np.array_equal(a[key], b[key]), key


def test_bad_arguments(case):
    wl, cfg, inp, ora, g, bars = case
    ns, S = inp.block_tokens.shape
    from paper_2510_08666_amd.binding import DinferError
    with pytest.raises(DinferError):
        g.step_vicinity(np.zeros((ns, 65), np.int32), 0.5)          # window too long
    with pytest.raises(DinferError):
        g.step_vicinity(np.zeros((ns, 17), np.int32), 0.5)          # run exceeds max_tokens


def test_run_must_fit_position_table_and_page_row():
    """look_back + block_len positions beyond max_pos, or beyond what the page-table row holds, are refused before
    anything is launched (the token positions of such a run would leave the rotary table / the page-table row)."""
    from paper_2510_08666_amd.binding import DinferError
    wl = di.Workload("short", di.model_preset("tiny"), 1, 32, 40, 40, threshold=0.9, seed_index=31)
    cfg, w, inp = make_case(wl)
    vic = np.zeros((1, 40), np.int32)
    # max_pos 64 < 40 + 32
    g = GpuRun(cfg, w, inp, 128, 64)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    with pytest.raises(DinferError) as e:
        g.step_vicinity(vic, 0.5)
    assert e.value.code == -3
    g.close()
    # page-table row of 4 pages = 64 positions < 72
    g = GpuRun(cfg, w, inp, 128, 256)
    g.page_table = g.page_table[:, :4].contiguous()
    with pytest.raises(DinferError) as e:
        g.step_vicinity(vic, 0.5)
    assert e.value.code == -3
    g.close()


def test_debug_logits_takes_the_last_forward_whole(case):
    wl, cfg, inp, ora, g, bars = case
    ns, S = inp.block_tokens.shape
    from paper_2510_08666_amd.binding import DinferError
    g.inject_prefix(ora.caches)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    g.step(0.5)
    assert g.logits(ns * S).shape == (ns * S, cfg.vocab)
    if ns * S > 1:
        with pytest.raises(DinferError):
            g.logits(ns * S - 1)


def test_caller_side_warmup_then_vicinity(case):
    """The experimental configuration names `warmup_times` without defining it; it is taken as the number of steps
    at the start of a block that run without the vicinity refresh, which is the caller's choice of entry point per
    step.  Two plain steps, then two steps with the refresh, three commits each; the oracle does the same from the
    same start (teacher-forced on tokens and masks), and the caches of both sides agree at the end."""
    wl, cfg, inp, ora, g, bars = case
    ns, S = inp.block_tokens.shape
    look_back, fixed_k, warmup = LOOK_BACK, 3, 2
    vic = np.stack([inp.prefix_tokens[s][int(inp.prefix_len[s]) - look_back:] for s in range(ns)])
    keeps = [(kc.copy(), vc.copy()) for kc, vc in ora.caches]
    g.inject_prefix(ora.caches)
    tokens, masks = inp.block_tokens.copy(), inp.mask_bits.copy()
    for step in range(warmup + 2):
        g.set_state(tokens, masks, inp.prefix_len)
        if step < warmup:
            got = g.step(0.5, fixed_k)
            routing = g.routing().reshape(cfg.n_layers, ns, S, cfg.top_k)
        else:
            got = g.step_vicinity(vic, 0.5, fixed_k)
            routing = g.routing(ns * (look_back + S)).reshape(cfg.n_layers, ns, look_back + S, cfg.top_k)
        for s in range(ns):
            P = int(inp.prefix_len[s])
            if step < warmup:
                ref, _ = ora.step_following(s, tokens[s], int(masks[s]), P, 0.5, fixed_k, routing[:, s], bars)
            else:
                ref, _ = ora.step_vicinity_following(s, tokens[s], vic[s], int(masks[s]), P, 0.5, fixed_k,
                                                     routing[:, s], bars)
            compare_step(ref, got["tokens"][s], got["mask"][s], got["conf"][s], got["argmax"][s], got["n_committed"][s],
                         tokens[s], masks[s], 0.5, fixed_k, bars, ref["logits"])
        tokens, masks = got["tokens"].copy(), got["mask"].copy()
    for s in range(ns):
        P = int(inp.prefix_len[s])
        kc, vc = ora.caches[s]
        for l in range(cfg.n_layers):
            k, v = g.read_kv(s, l, 0, P + S)
            assert kv_close(k[P - look_back:], kc[l, P - look_back:P + S], bars)
            assert kv_close(v[P - look_back:], vc[l, P - look_back:P + S], bars)
        kc[...], vc[...] = keeps[s]
