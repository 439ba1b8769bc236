"""GPU parity at the benchmark's full LLaDA-MoE shapes (16 layers, hidden 2048, 64 experts top-8, vocab
157184, bf16), in the launch configuration bench.py times.

The cached prefix is a seeded synthetic K,V (same values on both sides): an oracle prefill of thousands of
tokens would take tens of minutes, and a step only ever reads the cache.  A real prefill at these shapes is
checked on a short prompt.  One weight set (14.7 GB) serves every case.
"""
import time

import numpy as np
import pytest

import dinfer_inputs as di
import oracle
from harness import kv_close, kv_err_ratio, GpuRun, bars_for, compare_logits, compare_step, check_routing, max_abs_err

pytestmark = pytest.mark.gpu

WEIGHT_SEED = di.BASE_SEED + 2


def log(msg):
    print("[llada %s] %s" % (time.strftime("%H:%M:%S"), msg), flush=True)


@pytest.fixture(scope="module")
def model():
    cfg = di.model_preset("llada_moe")
    t = time.time()
    w = di.make_weights(cfg, WEIGHT_SEED)
    log("weights generated in %.0f s" % (time.time() - t))
    return cfg, w, oracle.Oracle(cfg, w)


_shared = {}     # the packed device weights, uploaded by the first case and reused by the others


def gpu_run(model, inp, max_tokens, max_pos):
    cfg, w, _ = model
    t = time.time()
    g = GpuRun(cfg, w, inp, max_tokens, max_pos, weights_buffer=_shared.get("w"))
    if "w" not in _shared:
        _shared["w"] = g.ctx.weights
        log("weights uploaded and packed in %.0f s" % (time.time() - t))
    return g


class BigCase:
    """One workload on both sides, prefix K,V synthetic.  Oracle caches hold [L][cap][D] per sequence."""

    def __init__(self, model, wl, max_tokens=None, peaked=0):
        self.cfg, self.w, self.o = model
        self.wl = wl
        self.inp = di.make_workload_inputs(wl)
        self.ns, self.S = self.inp.block_tokens.shape
        self.bars = bars_for(self.cfg)
        max_pos = int(self.inp.prefix_len.max()) + max(self.S, wl.gen_len) + 16
        self.gpu = gpu_run(model, self.inp, max_tokens or max(self.ns * self.S, 64), max_pos)
        self.caches = []
        torch = self.gpu.torch
        for s in range(self.ns):
            P = int(self.inp.prefix_len[s])
            kc, vc = self.o.new_cache(P + max(self.S, wl.gen_len))
            if P:
                k, v = di.synthetic_prefix_kv(self.cfg, self.inp.seed, s, P, peaked=peaked)
                kc[:, :P], vc[:, :P] = k, v
                for l in range(self.cfg.n_layers):
                    self.gpu.ctx.kv_write(l, self.gpu.page_table[s], 0, torch.from_numpy(k[l]).to(self.gpu.dev),
                                          torch.from_numpy(v[l]).to(self.gpu.dev))
            self.caches.append((kc, vc))
        torch.cuda.synchronize()

    def oracle_step_following(self, s, tokens, mask, prefix_len, threshold, fixed_k, routing):
        kc, vc = self.caches[s]
        tr = oracle.Trace(self.cfg, len(tokens), forced_idx=routing)
        ref = self.o.step(tokens, mask, prefix_len, kc, vc, threshold, fixed_k, want_logits=True, trace=tr)
        self.router_stats = {}
        return ref, check_routing(tr, routing, self.cfg.top_k, self.bars, self.router_stats)

    def check_step(self, got, logits, routing, tokens, masks, prefix_len, threshold, fixed_k, seqs=None):
        """Compare the sequences in `seqs` (default all) of a GPU step against the oracle."""
        flagged, near_total = 0, 0
        for s in (range(self.ns) if seqs is None else seqs):
            t = time.time()
            ref, near = self.oracle_step_following(s, tokens[s], int(masks[s]), int(prefix_len[s]), threshold, fixed_k,
                                                   routing[:, s])
            worst = compare_logits(ref["logits"], logits[s], self.bars)
            rep = compare_step(ref, got["tokens"][s], got["mask"][s], got["conf"][s], got["argmax"][s],
                               got["n_committed"][s], tokens[s], masks[s], threshold, fixed_k, self.bars,
                               ref["logits"], logits[s])
            P = int(prefix_len[s])
            kc, vc = self.caches[s]
            kv_worst = 0.0
            for l in range(self.cfg.n_layers):
                k, v = self.gpu.read_kv(s, l, P, self.S)
                rk, rv = kv_err_ratio(k, kc[l, P:P + self.S], self.bars), kv_err_ratio(v, vc[l, P:P + self.S], self.bars)
                assert rk <= 1.0 and rv <= 1.0, "layer %d K,V error %.2f / %.2f of the bar" % (l, rk, rv)
                kv_worst = max(kv_worst, rk, rv)
            flagged += len(rep["flagged"])
            near_total += near
            log("%s seq %d: oracle step %.0f s, logits err %.2f of bar, K,V err %.2f of bar, conf rel err %.1e, "
                "flagged %s, router near-ties %d (worst gap %.2e), committed %d" % (
                    self.wl.name, s, time.time() - t, worst, kv_worst, rep["conf_rel_err"], rep["flagged"], near,
                    self.router_stats.get("router_worst_gap", 0.0), got["n_committed"][s]))
        return flagged, near_total

    def gpu_step(self, tokens, masks, prefix_len, threshold, fixed_k=0):
        g = self.gpu
        g.set_state(tokens, masks, prefix_len)
        got = g.step(threshold, fixed_k)
        logits = g.logits(self.ns * self.S).reshape(self.ns, self.S, -1)
        routing = g.routing().reshape(self.cfg.n_layers, self.ns, self.S, self.cfg.top_k)
        return got, logits, routing


def test_c2_batch1_step(model):
    """Configuration 2: batch 1, 512 cached positions, 32 masked positions, threshold 0.9."""
    c = BigCase(model, di.workload_preset(2))
    inp = c.inp
    got, logits, routing = c.gpu_step(inp.block_tokens, inp.mask_bits, inp.prefix_len, c.wl.threshold)
    c.check_step(got, logits, routing, inp.block_tokens, inp.mask_bits, inp.prefix_len, c.wl.threshold, 0)
    assert got["n_committed"][0] == 1      # random-init confidences are far below 0.9: the fallback commits one
    # a threshold inside the confidence distribution: several positions commit
    tau = float(np.median(got["conf"][0]))
    got2, logits2, routing2 = c.gpu_step(inp.block_tokens, inp.mask_bits, inp.prefix_len, tau)
    assert np.array_equal(logits2, logits), "same state, same bits"
    c.check_step(got2, logits2, routing2, inp.block_tokens, inp.mask_bits, inp.prefix_len, tau, 0)
    assert got2["n_committed"][0] > 1
    c.gpu.close()


@pytest.mark.parametrize("preset", [2, 3])
def test_split_sums_match_single_workgroup_sums_at_full_shapes(model, preset):
    """Configurations 2 and 3 in the launch shapes the benchmark times: 8 K slices per projection task, 8 x 8 waves
    per task of the fused down projection, and (configuration 3) 8 key splits per (query tile, head), each handing
    its partial to the workgroup that arrives last.  With the test switch on, one workgroup sums a task alone; the
    two results may differ by float32 summation order (and the bf16 re-rounding of activations) only."""
    from paper_2510_08666_amd import binding
    import dataclasses
    # A router near-tie may fall differently under the other summation order, and the logits of the two runs are
    # then not comparable: the comparison is made on the first of three seeded inputs whose routing agrees.
    base = di.workload_preset(preset)
    for seed_index in (base.seed_index, base.seed_index + 1000, base.seed_index + 2000):
        c = BigCase(model, dataclasses.replace(base, seed_index=seed_index))
        inp = c.inp
        got, logits, routing = c.gpu_step(inp.block_tokens, inp.mask_bits, inp.prefix_len, c.wl.threshold)
        binding.debug_single_slice(True)
        try:
            got1, logits1, routing1 = c.gpu_step(inp.block_tokens, inp.mask_bits, inp.prefix_len, c.wl.threshold)
        finally:
            binding.debug_single_slice(False)
        same_route = np.array_equal(np.sort(routing, axis=-1), np.sort(routing1, axis=-1))
        err = float(np.abs(logits - logits1).max()) / float(np.abs(logits).max())
        log("%s seed %d: single-slice vs split: max |dz| / max |z| = %.2e, routing identical: %s" % (
            c.wl.name, seed_index, err, same_route))
        c.gpu.close()
        if same_route:
            assert err <= 1e-3
            return
    raise AssertionError("routing differed between the split and the single-workgroup sums for all three inputs")


def test_c3_long_prefix_half_committed(model):
    """Configuration 3: 4096 cached positions, block of 64 with half the positions already decided,
    threshold 0.8."""
    c = BigCase(model, di.workload_preset(3))
    inp = c.inp
    got, logits, routing = c.gpu_step(inp.block_tokens, inp.mask_bits, inp.prefix_len, c.wl.threshold)
    c.check_step(got, logits, routing, inp.block_tokens, inp.mask_bits, inp.prefix_len, c.wl.threshold, 0)
    c.gpu.close()


def test_c3_peaked_attention(model):
    """Configuration 3's shapes with a sharply peaked softmax: in every layer 12 of the 4096 cached positions carry
    key rows 16 times as large as the rest (same values on both sides), spread over the key tiles of different
    waves and key splits.  A query's scores on them are ~N(0, 13^2) against ~N(0, 0.8^2) elsewhere, so its softmax
    sits on one or two of them: the running-maximum rescale across key tiles, the fold across waves and the merge
    across splits all see weights that differ by many orders of magnitude, which the flat synthetic prefix never
    produces.  Attention errors would show in the K,V rows of the following layers (compared in every layer) and in
    the logits."""
    wl = di.workload_preset(3)
    c = BigCase(model, wl, peaked=12)
    inp = c.inp
    P = int(inp.prefix_len[0])
    cells = set()
    for l in range(c.cfg.n_layers):
        for p in di.peaked_positions(inp.seed, 0, l, P, 12):
            cells.add((p // 32) % 40)          # (key split, wave) that owns the position's key tile: 5 splits x 8 waves
    assert len(cells) >= 30, "the enlarged keys do not cover the waves and splits"
    # the oracle's own attention is peaked: the largest softmax weight of a query is far above 1/4160
    got, logits, routing = c.gpu_step(inp.block_tokens, inp.mask_bits, inp.prefix_len, wl.threshold)
    c.check_step(got, logits, routing, inp.block_tokens, inp.mask_bits, inp.prefix_len, wl.threshold, 0)
    # and the result differs from the flat-prefix case by far more than the bars (the enlarged rows matter)
    flat = BigCase(model, wl)
    got_f, logits_f, _ = flat.gpu_step(inp.block_tokens, inp.mask_bits, inp.prefix_len, wl.threshold)
    moved = np.abs(logits_f - logits).max() / np.abs(logits).max()
    log("C3 peaked: logits moved by %.2f of their range against the flat prefix" % moved)
    assert moved > 10 * c.bars.logit_rel
    c.gpu.close()
    flat.gpu.close()


def test_c4_batch16_paged(model):
    """Configuration 4: 16 sequences, prefixes 256..2048 on scattered pages (512 block tokens: the many-token
    forms of the expert GEMMs and the LM head).  Every sequence is compared element by element against the
    oracle."""
    c = BigCase(model, di.workload_preset(4))
    inp = c.inp
    got, logits, routing = c.gpu_step(inp.block_tokens, inp.mask_bits, inp.prefix_len, c.wl.threshold)
    c.check_step(got, logits, routing, inp.block_tokens, inp.mask_bits, inp.prefix_len, c.wl.threshold, 0)
    for s in range(c.ns):
        assert got["n_committed"][s] == 1 and bin(int(got["mask"][s])).count("1") == c.S - 1
        i = int(np.argmax(got["conf"][s]))
        assert got["tokens"][s][i] == got["argmax"][s][i]
    cnt = c.gpu.ctx.debug_get(3, (c.cfg.n_experts,), c.gpu.torch.int32).cpu().numpy()
    log("C4 last-layer expert rows: min %d max %d mean %.1f" % (cnt.min(), cnt.max(), cnt.mean()))
    assert cnt.sum() == c.ns * c.S * c.cfg.top_k
    c.gpu.close()


def test_c5_first_block_fixed_k_and_refresh(model):
    """Configuration 5's loop on its first block: 256 cached positions, block of 64, exactly 8 steps of 8
    commits, then the refresh of the block.  Steps are compared teacher-forced (the oracle continues from the
    GPU's state after each step)."""
    wl = di.workload_preset(5)
    c = BigCase(model, wl)
    inp, g = c.inp, c.gpu
    tokens, masks = inp.block_tokens.copy(), inp.mask_bits.copy()
    n_steps = 0
    while masks.any():
        got, logits, routing = c.gpu_step(tokens, masks, inp.prefix_len, wl.threshold, wl.fixed_k)
        c.check_step(got, logits, routing, tokens, masks, inp.prefix_len, wl.threshold, wl.fixed_k)
        assert got["n_committed"][0] == 8
        assert int(got["mask"][0]) & ~int(masks[0]) == 0
        tokens, masks = got["tokens"].copy(), got["mask"].copy()
        n_steps += 1
    assert n_steps == 8
    # the library's loop does the same from the same start, without waiting between steps
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    assert g.generate_block(wl.threshold, wl.fixed_k, max_steps=64, masked_hint=64) == 8
    st = g.state()
    assert np.array_equal(st["tokens"], tokens) and not st["mask"].any()
    # refresh of the decoded block
    g.refresh()
    routing = g.routing().reshape(c.cfg.n_layers, 1, c.S, c.cfg.top_k)
    P = int(inp.prefix_len[0])
    assert g.prefix_len.cpu().numpy()[0] == P + c.S
    kc, vc = c.caches[0]
    tr = oracle.Trace(c.cfg, c.S, forced_idx=routing[:, 0])
    c.o.forward(tokens[0], P, kc, vc, tr)
    check_routing(tr, routing[:, 0], c.cfg.top_k, c.bars)
    for l in range(c.cfg.n_layers):
        k, v = g.read_kv(0, l, P, c.S)
        assert kv_close(k, kc[l, P:P + c.S], c.bars)
        assert kv_close(v, vc[l, P:P + c.S], c.bars)
    c.gpu.close()


def test_c2_vicinity_refresh_step(model):
    """Configuration 2 with the vicinity KV-cache refresh of the paper's experiments: the 16 cached positions
    before the block join the forward (48 tokens) and their K,V rows are rewritten."""
    look_back = 16
    wl = di.workload_preset(2)
    c = BigCase(model, wl, max_tokens=64)
    inp, g = c.inp, c.gpu
    S, P = c.S, int(inp.prefix_len[0])
    run = look_back + S
    vic = inp.prefix_tokens[0][P - look_back:][None, :]
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    got = g.step_vicinity(vic, wl.threshold)
    logits = g.logits(run)[look_back:]
    routing = g.routing(run)
    kc, vc = c.caches[0]
    keep_k = kc[:, :P - look_back].copy()
    tr = oracle.Trace(c.cfg, run, forced_idx=routing)
    t = time.time()
    ref = c.o.step_vicinity(inp.block_tokens[0], vic[0], int(inp.mask_bits[0]), P, kc, vc, wl.threshold, 0,
                            want_logits=True, trace=tr)
    near = check_routing(tr, routing, c.cfg.top_k, c.bars)
    worst = compare_logits(ref["logits"], logits, c.bars)
    rep = compare_step(ref, got["tokens"][0], got["mask"][0], got["conf"][0], got["argmax"][0], got["n_committed"][0],
                       inp.block_tokens[0], inp.mask_bits[0], wl.threshold, 0, c.bars, ref["logits"])
    for l in (0, c.cfg.n_layers - 1):
        k, v = g.read_kv(0, l, P - look_back, run)
        assert kv_close(k, kc[l, P - look_back:P + S], c.bars)
        assert kv_close(v, vc[l, P - look_back:P + S], c.bars)
        k0, _ = g.read_kv(0, l, 0, P - look_back)
        assert np.array_equal(k0, keep_k[l].astype(np.float32))     # synthetic prefix values are bf16-exact
    log("C2 vicinity: oracle %.0f s, logits err %.2f of bar, conf rel err %.1e, flagged %s, near-ties %d" %
        (time.time() - t, worst, rep["conf_rel_err"], rep["flagged"], near))
    c.gpu.close()


def test_c2_credit_decoding_steps(model):
    """Configuration 2 with credit decoding over three steps of a block (fixed 4 commits per step), teacher-forced
    like the tiny credit test.  With random-init weights the confidences are ~3e-4, so a boost is about one per
    cent: the case checks the credit lists, the recomputed listed logits and the exchanged softmax terms at the
    full vocabulary; the tiny cases check large boosts."""
    cfg, w, o = model
    wl = di.workload_preset(2)
    c = BigCase((cfg, w, o), wl)
    inp, g = c.inp, c.gpu
    S, P, V = c.S, int(inp.prefix_len[0]), cfg.vocab
    alpha, beta, gamma, fixed_k = 0.65, 0.7, 0.5, 4
    credit = g.credit_state()
    ora_credit = np.zeros((S, V))
    tokens, masks = inp.block_tokens.copy(), inp.mask_bits.copy()
    kc, vc = c.caches[0]
    boosted = False
    for step in range(3):
        g.set_state(tokens, masks, inp.prefix_len)
        got = g.step_credit(credit, 0.5, alpha, beta, gamma, fixed_k)
        routing = g.routing().reshape(cfg.n_layers, S, cfg.top_k)
        tr = oracle.Trace(cfg, S, forced_idx=routing)
        ref = o.step_credit(tokens[0], int(masks[0]), P, kc, vc, 0.5, ora_credit, alpha, beta, gamma, fixed_k,
                            want_logits=True, trace=tr)
        near = check_routing(tr, routing, cfg.top_k, c.bars)
        rep = compare_step(ref, got["tokens"][0], got["mask"][0], got["conf"][0], got["argmax"][0],
                           got["n_committed"][0], tokens[0], masks[0], 0.5, fixed_k, c.bars, ref["logits"])
        ids, val, n = (credit[k][0].cpu().numpy() for k in ("ids", "val", "n"))
        mine = np.zeros((S, V))
        for i in range(S):
            assert len(set(ids[i, :n[i]].tolist())) == n[i], "a token is listed twice"
            mine[i, ids[i, :n[i]]] = val[i, :n[i]]
        # the plain logits of the same forward (same expert sets): they decide which candidate a side may reward
        plain_ref = o.step(tokens[0], int(masks[0]), P, kc, vc, 2.0, want_logits=True,
                           trace=oracle.Trace(cfg, S, forced_idx=routing))
        plain, zp = plain_ref["conf"], plain_ref["logits"]
        masked = [i for i in range(S) if (int(masks[0]) >> i) & 1]
        tie_positions = []
        for i in masked:
            ids_g, ids_o = set(np.nonzero(mine[i])[0]), set(np.nonzero(ora_credit[i])[0])
            if ids_g != ids_o:
                # the two sides rewarded different top-1 candidates: only a near-tie of the plain logits allows that
                # (each logit within the logits' bar).  The oracle continues from the GPU's list at this position.
                allowed = 2 * c.bars.logit_rel * np.abs(zp[i]).max()
                for v in ids_g ^ ids_o:
                    assert zp[i].max() - zp[i, v] <= allowed, (step, i, int(v), float(zp[i].max() - zp[i, v]), allowed)
                tie_positions.append(i)
                ora_credit[i] = mine[i]
            else:
                nz = np.nonzero(mine[i])[0]
                assert 1 <= len(nz) <= step + 1, (step, i, len(nz))
                assert np.allclose(mine[i, nz], ora_credit[i, nz], rtol=5e-2), (step, i)
        assert len(tie_positions) <= max(2, len(masked) // 8), tie_positions
        for i in range(S):
            if i not in masked and step == 0:
                assert not mine[i].any()
        if step > 0 and np.median(ref["conf"][masked] / plain[masked]) > 1.005:
            boosted = True
        log("C2 credit step %d: conf rel err %.1e, flagged %s, near-ties %d, rewarded-candidate ties at %s, median "
            "enhanced/plain conf %.3f, max list length %d" % (step, rep["conf_rel_err"], rep["flagged"], near,
                                                              tie_positions,
                                                              float(np.median(ref["conf"][masked] / plain[masked])),
                                                              int(n.max())))
        tokens, masks = got["tokens"].copy(), got["mask"].copy()
    assert boosted
    c.gpu.close()


def test_c2_iteration_smoothing_steps(model):
    """Configuration 2 with iteration smoothing over two steps (fixed 4 commits per step).  Step 0 (alpha = 0, as
    the first step of a block) checks the expected embeddings the step leaves behind against the oracle's
    contraction over the full vocabulary.  With random-init weights the distributions are nearly uniform and the
    expected embedding is close to the mean embedding row, too small to move the logits past the bf16 tolerance;
    so step 1 is handed seeded embeddings of the scale of an embedding row (the retained embeddings are an input
    of the step on both sides) with alpha = 0.5."""
    cfg, w, o = model
    wl = di.workload_preset(2)
    c = BigCase((cfg, w, o), wl)
    inp, g = c.inp, c.gpu
    S, P, H = c.S, int(inp.prefix_len[0]), cfg.hidden
    fixed_k = 4
    sm = g.smooth_state()
    tokens, masks = inp.block_tokens.copy(), inp.mask_bits.copy()
    kc, vc = c.caches[0]
    rng = np.random.default_rng(di.BASE_SEED + 77)
    for step, alpha in enumerate((0.0, 0.5)):
        if step == 1:
            emb_scale = cfg.init_std           # standard deviation of the embedding matrix's entries
            sm["delta"].copy_(g.torch.from_numpy((emb_scale * rng.standard_normal((1, S, H))).astype(np.float32)))
        delta_in = sm["delta"].cpu().numpy().astype(np.float64)
        g.set_state(tokens, masks, inp.prefix_len)
        got = g.step_smooth(sm, alpha, 0.5, fixed_k)
        delta_out = sm["delta"].cpu().numpy()
        routing = g.routing().reshape(cfg.n_layers, S, cfg.top_k)
        tr = oracle.Trace(cfg, S, forced_idx=routing)
        d = np.ascontiguousarray(delta_in[0])
        keep = kc.copy(), vc.copy()
        ref = o.step_smooth(tokens[0], int(masks[0]), P, kc, vc, 0.5, alpha, d, fixed_k, want_logits=True, trace=tr)
        near = check_routing(tr, routing, cfg.top_k, c.bars)
        compare_logits(ref["logits"], g.logits(S), c.bars)
        rep = compare_step(ref, got["tokens"][0], got["mask"][0], got["conf"][0], got["argmax"][0],
                           got["n_committed"][0], tokens[0], masks[0], 0.5, fixed_k, c.bars, ref["logits"])
        worst = 0.0
        for i in range(S):
            if (int(masks[0]) >> i) & 1:
                err = np.abs(delta_out[0, i] - d[i]).max() / np.abs(d[i]).max()
                worst = max(worst, err)
                assert err <= 8e-2, (step, i, err)
            else:
                assert np.array_equal(delta_out[0, i], delta_in[0, i].astype(np.float32))
        moved = 0.0
        if step == 1:
            kc[...], vc[...] = keep
            plain = o.step(tokens[0], int(masks[0]), P, kc, vc, 2.0, want_logits=True)["logits"]
            moved = np.abs(plain - ref["logits"]).max() / np.abs(plain).max()
            assert moved > 3 * c.bars.logit_rel, moved
        log("C2 smoothing step %d: conf rel err %.1e, flagged %s, near-ties %d, expected-embedding rel err %.1e, "
            "logits moved by %.2f of their range" % (step, rep["conf_rel_err"], rep["flagged"], near, worst, moved))
        kc[...], vc[...] = keep
        tokens, masks = got["tokens"].copy(), got["mask"].copy()
    c.gpu.close()


def test_prefill_at_full_shapes(model):
    """A real prefill (bidirectional forward over the prompt) of 100 tokens at the full model shapes."""
    cfg, w, o = model
    wl = di.Workload("prefill100", cfg, 1, 32, 100, 100, seed_index=11)
    inp = di.make_workload_inputs(wl)
    bars = bars_for(cfg)
    g = gpu_run(model, inp, 128, 160)
    g.prefill()
    g.torch.cuda.synchronize()
    routing = g.routing(100)
    kc, vc = o.new_cache(160)
    tr = oracle.Trace(cfg, 100, forced_idx=routing)
    t = time.time()
    o.forward(inp.prefix_tokens[0], 0, kc, vc, tr)
    near = check_routing(tr, routing, cfg.top_k, bars)
    log("prefill 100 tokens: oracle %.0f s, router near-ties %d" % (time.time() - t, near))
    for l in range(cfg.n_layers):
        k, v = g.read_kv(0, l, 0, 100)
        assert kv_close(k, kc[l, :100], bars), l
        assert kv_close(v, vc[l, :100], bars), l
    g.close()
