"""GPU parity of the whole path at sizes the oracle finishes in seconds: the tiny fp32 configuration and
variants of it (bf16 storage, ragged blocks and prefixes, several sequences, pre-committed positions,
head_dim 128).  Every case runs through the C-ABI (ctypes binding) and is compared element by element."""
import numpy as np
import pytest

import dinfer_inputs as di
import oracle
from harness import kv_close, GpuRun, OracleRun, bars_for, compare_logits, compare_step, make_case, max_abs_err

pytestmark = pytest.mark.gpu


def _variant(name):
    tiny = di.model_preset("tiny")
    W = di.Workload
    sc = di.configs.scaled
    table = {
        # the benchmark's tiny configuration as stated
        "c1": W("c1", tiny, 1, 32, 64, 64, threshold=0.9, seed_index=1),
        # same, bf16 storage (exercises the bf16 MFMA path at a size the oracle handles)
        "c1_bf16": W("c1_bf16", sc(tiny, dtype="bf16", logit_scale=1.0), 1, 32, 64, 64, threshold=0.9, seed_index=1),
        # ragged: block of 20, prefix of 50 (neither a multiple of the page or tile size)
        "ragged": W("ragged", tiny, 1, 20, 50, 50, threshold=0.9, seed_index=6),
        # several sequences with different prefix lengths, block 64, half the positions already decided
        "batch": W("batch", tiny, 5, 64, 17, 140, precommit=True, threshold=0.9, seed_index=7),
        "batch_bf16": W("batch_bf16", sc(tiny, dtype="bf16", logit_scale=1.0), 3, 64, 17, 140, precommit=True, threshold=0.9,
                        seed_index=8),
        # head_dim 128, more experts than a wave-quarter, top-8, many tokens (token groups > 1)
        "wide": W("wide", sc(tiny, n_heads=2, head_dim=128, n_experts=64, top_k=8, moe_inter=128, vocab=1000),
                  9, 32, 5, 300, threshold=0.9, seed_index=9),
        "wide_bf16": W("wide_bf16", sc(tiny, n_heads=2, head_dim=128, n_experts=64, top_k=8, moe_inter=128,
                                       vocab=1000, dtype="bf16", logit_scale=1.0), 9, 32, 5, 300, threshold=0.9, seed_index=9),
        # hidden 1024: the K range of a projection task is shared by several workgroups (cross-workgroup sums,
        # last arrival runs the epilogue), with one and with two token tiles
        "deep": W("deep", sc(tiny, hidden=1024), 1, 32, 40, 40, threshold=0.9, seed_index=12),
        "deep_bf16": W("deep_bf16", sc(tiny, hidden=1024, dtype="bf16", logit_scale=1.0), 1, 64, 40, 40, threshold=0.9,
                       seed_index=13),
        # 896 tokens and 48 QKV tasks: the many-token projections take two token tiles per workgroup
        "dense2": W("dense2", sc(tiny, hidden=1024, n_heads=16, head_dim=64), 14, 64, 5, 40, threshold=0.9, seed_index=14),
        "dense2_bf16": W("dense2_bf16", sc(tiny, hidden=1024, n_heads=16, head_dim=64, dtype="bf16", logit_scale=1.0), 14, 64,
                         5, 40, threshold=0.9, seed_index=14),
        # the most sequences a call takes (64) with full blocks: 4096 tokens, experts with hundreds of rows (several row
        # groups per expert in the many-token expert GEMMs), 32 token groups in the LM head
        "max64": W("max64", tiny, 64, 64, 0, 70, precommit=True, threshold=0.9, seed_index=15),
        # short and long cached prefixes in one call: sequences use different numbers of attention key splits
        "longctx": W("longctx", tiny, 4, 32, 60, 1500, threshold=0.9, seed_index=22),
        "longctx_bf16": W("longctx_bf16", sc(tiny, dtype="bf16", logit_scale=1.0), 4, 32, 60, 1500, threshold=0.9, seed_index=22),
        # no prefix at all: the block attends to itself only
        "noprefix": W("noprefix", tiny, 2, 32, 0, 0, threshold=0.9, seed_index=10),
        # a skewed router (see _skew_router): three hot experts take most rows, eight more take the rest by the tie
        # rule, 53 stay empty.  32 tokens (records of the fused permutation, fused down projection over few experts),
        # 64 tokens, and 288 tokens (work list: the hot experts have up to three row groups, most experts none)
        "skew": W("skew", sc(tiny, n_heads=2, head_dim=128, n_experts=64, top_k=8, moe_inter=128, vocab=1000),
                  1, 32, 5, 40, threshold=0.9, seed_index=41),
        "skew_bf16": W("skew_bf16", sc(tiny, n_heads=2, head_dim=128, n_experts=64, top_k=8, moe_inter=128, vocab=1000,
                                       dtype="bf16", logit_scale=1.0), 2, 32, 5, 40, threshold=0.9, seed_index=42),
        "skew_many": W("skew_many", sc(tiny, n_heads=2, head_dim=128, n_experts=64, top_k=8, moe_inter=128, vocab=1000),
                       9, 32, 5, 300, threshold=0.9, seed_index=43),
    }
    return table[name]


CASES = ["c1", "c1_bf16", "ragged", "batch", "batch_bf16", "wide", "wide_bf16", "deep", "deep_bf16", "dense2", "dense2_bf16",
         "max64", "longctx", "longctx_bf16", "noprefix", "skew", "skew_bf16", "skew_many"]

HOT_EXPERTS = (5, 23, 40)


def _skew_router(cfg, w):
    """Router weights that send most rows to three experts: the rows of the hot experts are scaled by 16 (exact in
    either storage type), every other row is zero.  A cold expert's logit is then exactly 0 on both sides, a hot
    expert's is 16 times its usual value: a token takes the hot experts whose logits are positive and fills its
    top-k with the lowest-numbered cold experts (ties go to the lower id), so experts 0..7 and the three hot ones
    receive rows and the other 53 none."""
    for layer in w["layers"]:
        r = layer["w_router"]
        f = di.configs.bf16_to_f32(r) if cfg.dtype == "bf16" else r.astype(np.float32)
        g = np.zeros_like(f)
        for e in HOT_EXPERTS:
            g[e] = f[e] * 16.0
        layer["w_router"] = di.configs.f32_to_bf16(g) if cfg.dtype == "bf16" else g


class Case:
    def __init__(self, name):
        self.wl = _variant(name)
        self.cfg, self.w, self.inp = make_case(self.wl)
        if name.startswith("skew"):
            _skew_router(self.cfg, self.w)
        self.ns, self.S = self.inp.block_tokens.shape
        cap = int(self.inp.prefix_len.max()) + 2 * self.S + 16
        self.ora = OracleRun(self.cfg, self.w, self.inp, cap)
        total_prefix = int(sum(len(t) for t in self.inp.prefix_tokens))
        self.gpu = GpuRun(self.cfg, self.w, self.inp, max(self.ns * self.S, total_prefix, 1), cap)
        self.bars = bars_for(self.cfg)


@pytest.fixture(scope="module", params=CASES)
def case(request):
    c = Case(request.param)
    yield c
    c.gpu.close()


def test_kv_roundtrip(case):
    g, cfg = case.gpu, case.cfg
    rng = np.random.default_rng(1)
    torch = g.torch
    D = cfg.qkv_dim
    k = rng.standard_normal((37, D)).astype(np.float32)
    v = rng.standard_normal((37, D)).astype(np.float32)
    if cfg.dtype == "bf16":
        k, v = di.bf16_to_f32(di.f32_to_bf16(k)), di.bf16_to_f32(di.f32_to_bf16(v))
    row = g.page_table[0]
    first = 3
    n = min(37, int(case.inp.prefix_len[0]) + case.S - first)
    g.ctx.kv_write(cfg.n_layers - 1, row, first, torch.from_numpy(k[:n]).to(g.dev), torch.from_numpy(v[:n]).to(g.dev))
    k2, v2 = g.read_kv(0, cfg.n_layers - 1, first, n)
    assert np.array_equal(k2, k[:n]) and np.array_equal(v2, v[:n])


def test_prefill_matches_oracle(case):
    if case.inp.prefix_len.max() == 0:
        pytest.skip("no prompt")
    g = case.gpu
    g.prefill()
    g.torch.cuda.synchronize()
    lens = [len(t) for t in case.inp.prefix_tokens]
    routing = g.routing(sum(lens))
    at = 0
    for s in range(case.ns):
        P = lens[s]
        kc, vc = case.ora.caches[s]
        keep = kc.copy(), vc.copy()
        case.ora.forward_following(s, case.inp.prefix_tokens[s], 0, routing[:, at:at + P], case.bars)
        at += P
        for l in range(case.cfg.n_layers):
            k, v = g.read_kv(s, l, 0, P)
            assert kv_close(k, kc[l, :P], case.bars), (s, l)
            assert kv_close(v, vc[l, :P], case.bars), (s, l)
        kc[...], vc[...] = keep


def _run_step(case, threshold, fixed_k=0, tokens=None, masks=None):
    """Oracle prefix injected, then one step on both sides from the same state; compared per sequence."""
    g, inp = case.gpu, case.inp
    tokens = inp.block_tokens if tokens is None else tokens
    masks = inp.mask_bits if masks is None else masks
    g.inject_prefix(case.ora.caches)
    g.set_state(tokens, masks, inp.prefix_len)
    got = g.step(threshold, fixed_k)
    logits = g.logits(case.ns * case.S).reshape(case.ns, case.S, -1)
    routing = g.routing().reshape(case.cfg.n_layers, case.ns, case.S, case.cfg.top_k)
    reports = []
    for s in range(case.ns):
        kc, vc = case.ora.caches[s]
        P = int(inp.prefix_len[s])
        keep_k, keep_v = kc.copy(), vc.copy()
        ref, near = case.ora.step_following(s, tokens[s], int(masks[s]), P, threshold, fixed_k, routing[:, s],
                                            case.bars)
        assert near <= max(1, case.cfg.n_layers * case.S // 4), "too many router near-ties: %d" % near
        compare_logits(ref["logits"], logits[s], case.bars)
        rep = compare_step(ref, got["tokens"][s], got["mask"][s], got["conf"][s], got["argmax"][s],
                           got["n_committed"][s], tokens[s], masks[s], threshold, fixed_k, case.bars, ref["logits"],
                           logits[s])
        # K,V of the block positions as the step wrote them; prefix rows untouched
        for l in range(case.cfg.n_layers):
            k, v = g.read_kv(s, l, 0, P + case.S)
            assert kv_close(k[P:], kc[l, P:P + case.S], case.bars)
            assert kv_close(v[P:], vc[l, P:P + case.S], case.bars)
            if P:
                ref_k = keep_k[l, :P].astype(np.float32)
                ref_v = keep_v[l, :P].astype(np.float32)
                if case.cfg.dtype == "bf16":
                    ref_k, ref_v = di.bf16_to_f32(di.f32_to_bf16(ref_k)), di.bf16_to_f32(di.f32_to_bf16(ref_v))
                assert np.array_equal(k[:P], ref_k) and np.array_equal(v[:P], ref_v), "prefix KV changed"
        kc[...], vc[...] = keep_k, keep_v          # leave the oracle caches as the prefill made them
        reports.append((rep, ref))
    return got, reports


def test_step_as_configured(case):
    got, reports = _run_step(case, case.wl.threshold)
    for s, (rep, ref) in enumerate(reports):
        print("seq %d: flagged %s conf_err %.2e n_committed %d" % (s, rep["flagged"], rep["conf_err"], got["n_committed"][s]))


def test_step_threshold_at_median_confidence(case):
    """A threshold inside the confidence distribution, so that several positions commit at once."""
    probe = case.ora.step(0, case.inp.block_tokens[0], int(case.inp.mask_bits[0]), int(case.inp.prefix_len[0]), 2.0)
    kc, vc = case.ora.caches[0]
    masked = [i for i in range(case.S) if (int(case.inp.mask_bits[0]) >> i) & 1]
    tau = float(np.median(probe["conf"][masked]))
    got, reports = _run_step(case, tau)
    # (when the confidences of a sequence are all within rounding of each other - a fully masked block with
    # no prefix - which of them reach the threshold is not decidable; compare_step has flagged those)
    clear = sum(1 for i in masked if probe["conf"][i] >= tau * (1 + 10 * case.bars.conf_rel))
    if clear >= 2:
        assert got["n_committed"][0] >= clear


def test_step_fixed_k(case):
    got, reports = _run_step(case, 0.9, fixed_k=8)
    for s in range(case.ns):
        masked = bin(int(case.inp.mask_bits[s])).count("1")
        assert got["n_committed"][s] == min(8, masked)


def test_step_twice_is_bit_identical(case):
    """No atomics, fixed reduction orders: the same state gives the same bits."""
    g, inp = case.gpu, case.inp
    g.inject_prefix(case.ora.caches)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    a = g.step(case.wl.threshold)
    la = g.logits(case.ns * case.S)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    b = g.step(case.wl.threshold)
    lb = g.logits(case.ns * case.S)
    assert np.array_equal(a["conf"], b["conf"]) and np.array_equal(a["argmax"], b["argmax"])
    assert np.array_equal(a["tokens"], b["tokens"]) and np.array_equal(la, lb)


def test_split_sums_match_single_workgroup_sums(case):
    """Projections, router, fused down projection and attention normally share a task's sum among workgroups and
    hand the partials over through memory.  With the test switch on, one workgroup sums a task alone: the two
    results may differ by float32 summation order only (carried through the layers, and in bf16 storage through
    the re-rounding of activations to their two bf16 planes).  A partial that arrived late or stale would be off
    by a share of the sum (an eighth or more), two orders of magnitude above this bar."""
    from paper_2510_08666_amd import binding
    g, inp = case.gpu, case.inp
    T = case.ns * case.S
    g.inject_prefix(case.ora.caches)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    g.step(case.wl.threshold)
    la = g.logits(T)
    ids_a = g.ctx.debug_get(1, (case.cfg.n_layers, T, case.cfg.top_k), binding.torch.int32).cpu().numpy()
    binding.debug_single_slice(True)
    try:
        g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
        g.step(case.wl.threshold)
        lb = g.logits(T)
        ids_b = g.ctx.debug_get(1, (case.cfg.n_layers, T, case.cfg.top_k), binding.torch.int32).cpu().numpy()
    finally:
        binding.debug_single_slice(False)
    same_route = np.array_equal(np.sort(ids_a, axis=-1), np.sort(ids_b, axis=-1))
    scale = float(np.abs(la).max())
    err = float(np.abs(la - lb).max()) / scale
    print("single-slice vs split: max |dz| / max |z| = %.2e, routing identical: %s" % (err, same_route))
    if not same_route:
        pytest.skip("a router near-tie fell differently under the other summation order; logits are not comparable")
    assert err <= (1e-3 if case.cfg.dtype == "bf16" else 1e-4)


def test_skip_decided_rows(case):
    """decode.skip_decided: confidences and candidates of the undecided positions are the same bits as without it
    (a token's column of the matrix product does not depend on which other tokens share its tile), the decided
    positions' entries are left as they were, and the decoder commits the same."""
    from paper_2510_08666_amd import binding
    g, inp = case.gpu, case.inp
    g.inject_prefix(case.ora.caches)
    # every other position decided in every sequence (position 0 stays undecided), whatever the case's own mask
    full = (1 << case.S) - 1
    masks = np.array([((int(m) & 0x5555555555555555) | 1) & full for m in inp.mask_bits], dtype=np.uint64)
    toks = inp.block_tokens.copy()
    for s in range(case.ns):
        for i in range(case.S):
            if (int(masks[s]) >> i) & 1:
                toks[s, i] = case.cfg.mask_id
            elif toks[s, i] == case.cfg.mask_id:
                toks[s, i] = (7 * i + s) % (case.cfg.vocab - 1)
    g.set_state(toks, masks, inp.prefix_len)
    a = g.step(case.wl.threshold)
    g.set_state(toks, masks, inp.prefix_len)
    g.conf.fill_(-7.0)
    g.argmax.fill_(-7)
    dec = binding.Decode(float(case.wl.threshold), 0, 0, 0.0, 1)
    b = g.step(dec)
    for s in range(case.ns):
        for i in range(case.S):
            if (int(masks[s]) >> i) & 1:
                assert a["conf"][s, i] == b["conf"][s, i] and a["argmax"][s, i] == b["argmax"][s, i], (s, i)
            else:
                assert b["conf"][s, i] == -7.0 and b["argmax"][s, i] == -7, (s, i)
    for key in ("tokens", "mask", "n_committed"):
        assert np.array_equal(a[key], b[key]), key
    # nothing undecided at all: the row list is empty, nothing is computed, nothing is committed
    done = np.where(toks == case.cfg.mask_id, 3, toks)
    g.set_state(done, np.zeros(case.ns, dtype=np.uint64), inp.prefix_len)
    g.conf.fill_(-7.0)
    c = g.step(dec)
    assert np.array_equal(c["tokens"], done) and not c["mask"].any() and not c["n_committed"].any()
    assert (c["conf"] == -7.0).all()


def test_empty_mask_commits_nothing(case):
    g, inp = case.gpu, case.inp
    g.inject_prefix(case.ora.caches)
    toks = np.arange(case.ns * case.S, dtype=np.int32).reshape(case.ns, case.S) % (case.cfg.vocab - 1)
    masks = inp.mask_bits.copy()
    masks[0] = 0
    toks[1:] = inp.block_tokens[1:]
    g.set_state(toks, masks, inp.prefix_len)
    got = g.step(0.0)
    assert got["n_committed"][0] == 0 and got["mask"][0] == 0 and np.array_equal(got["tokens"][0], toks[0])
    for s in range(1, case.ns):   # threshold 0: everything masked commits
        assert got["mask"][s] == 0 and got["n_committed"][s] == bin(int(masks[s])).count("1")


def test_router_and_permutation(case):
    """Expert ids / weights of the last layer against the oracle's trace; permutation against the oracle's
    stable counting sort of the GPU's own routing (bit-exact)."""
    g, inp, cfg = case.gpu, case.inp, case.cfg
    torch = g.torch
    g.inject_prefix(case.ora.caches)
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    g.step(case.wl.threshold)
    T = case.ns * case.S
    idx = g.ctx.debug_get(1, (cfg.n_layers, T, cfg.top_k), torch.int32).cpu().numpy()[-1]
    wt = g.ctx.debug_get(2, (cfg.n_layers, T, cfg.top_k), torch.float32).cpu().numpy()[-1]
    cnt = g.ctx.debug_get(3, (cfg.n_experts,), torch.int32).cpu().numpy()
    off = g.ctx.debug_get(4, (cfg.n_experts + 1,), torch.int32).cpu().numpy()
    perm = g.ctx.debug_get(5, (T * cfg.top_k,), torch.int32).cpu().numpy()
    c2, o2, p2 = oracle.permutation(idx.reshape(-1), cfg.n_experts)
    assert np.array_equal(cnt, c2) and np.array_equal(off, o2) and np.array_equal(perm, p2)
    if case.wl.name.startswith("skew"):
        print("skewed router: rows per expert with rows", {int(e): int(n) for e, n in enumerate(cnt) if n})
        assert (cnt > 0).sum() <= 8 + len(HOT_EXPERTS) and cnt[list(HOT_EXPERTS)].sum() >= T
    mismatched = 0
    for s in range(case.ns):
        kc, vc = case.ora.caches[s]
        keep = kc.copy(), vc.copy()
        tr = oracle.Trace(cfg, case.S)
        case.ora.step(s, inp.block_tokens[s], int(inp.mask_bits[s]), int(inp.prefix_len[s]), case.wl.threshold, trace=tr)
        kc[...], vc[...] = keep
        for t in range(case.S):
            gi, gw = idx[s * case.S + t], wt[s * case.S + t]
            oi, ow = tr.topk_idx[-1, t], tr.topk_w[-1, t]
            if set(gi) != set(oi):
                mismatched += 1       # a near-tie at the k-th / (k+1)-th probability
                continue
            for j in range(cfg.top_k):
                assert abs(gw[j] - ow[list(oi).index(gi[j])]) <= (1e-5 if cfg.dtype == "f32" else 2e-2)
            assert abs(gw.sum() - 1.0) < 1e-5
    assert mismatched <= (0 if cfg.dtype == "f32" else max(1, T // 20))


def test_generate_block_teacher_forced(case):
    """The inner loop of Algorithm 1 on both sides.  After every step the GPU state is checked against the
    oracle's step from the same state; on a flagged divergence the oracle continues from the GPU's state."""
    g, inp = case.gpu, case.inp
    g.inject_prefix(case.ora.caches)
    probe = case.ora.step(0, inp.block_tokens[0], int(inp.mask_bits[0]), int(inp.prefix_len[0]), 2.0)
    kc, vc = case.ora.caches[0]
    tau = float(np.quantile(probe["conf"], 0.7))
    tokens, masks = inp.block_tokens.copy(), inp.mask_bits.copy()
    g.set_state(tokens, masks, inp.prefix_len)
    steps = 0
    while masks.any():
        got = g.step(tau)
        routing = g.routing().reshape(case.cfg.n_layers, case.ns, case.S, case.cfg.top_k)
        steps += 1
        for s in range(case.ns):
            ref, _ = case.ora.step_following(s, tokens[s], int(masks[s]), int(inp.prefix_len[s]), tau, 0,
                                             routing[:, s], case.bars)
            compare_step(ref, got["tokens"][s], got["mask"][s], got["conf"][s], got["argmax"][s],
                         got["n_committed"][s], tokens[s], masks[s], tau, 0, case.bars, ref["logits"])
        tokens, masks = got["tokens"].copy(), got["mask"].copy()
        assert steps <= case.S
    # the library's own loop from the same start reaches the same end state
    g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
    n = g.generate_block(tau, 0, max_steps=case.S)
    st = g.state()
    assert n == steps and not st["mask"].any() and np.array_equal(st["tokens"], tokens)
    # ... also when it enqueues several steps between two looks at the masks (the device skips the steps that find
    # nothing masked): same tokens, same confidences of the last real step, same count
    for per_wait in (3, 64):
        g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
        n2 = g.generate_block(tau, 0, max_steps=case.S, steps_per_wait=per_wait)
        st2 = g.state()
        assert n2 == steps and not st2["mask"].any() and np.array_equal(st2["tokens"], tokens)
        for key in ("conf", "argmax", "n_committed"):
            assert np.array_equal(st2[key], st[key]), key
    # max_steps cuts the loop short at the same point either way
    if steps > 2:
        for per_wait in (1, 4):
            g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
            assert g.generate_block(tau, 0, max_steps=2, steps_per_wait=per_wait) == 2
            assert g.state()["mask"].any()
        g.set_state(inp.block_tokens, inp.mask_bits, inp.prefix_len)
        assert g.generate_block(tau, 0, max_steps=case.S, steps_per_wait=8) == steps      # back to the decoded block
    # refresh: block K,V equal a forward over the final tokens, prefix length advances
    g.refresh()
    routing = g.routing().reshape(case.cfg.n_layers, case.ns, case.S, case.cfg.top_k)
    assert np.array_equal(g.prefix_len.cpu().numpy(), inp.prefix_len + case.S)
    for s in range(case.ns):
        P = int(inp.prefix_len[s])
        case.ora.forward_following(s, tokens[s], P, routing[:, s], case.bars)
        kc, vc = case.ora.caches[s]
        for l in range(case.cfg.n_layers):
            k, v = g.read_kv(s, l, P, case.S)
            assert kv_close(k, kc[l, P:P + case.S], case.bars)
            assert kv_close(v, vc[l, P:P + case.S], case.bars)


def test_fixed_k_generation_takes_ceil_steps(case):
    g, inp = case.gpu, case.inp
    g.inject_prefix(case.ora.caches)
    full = np.full_like(inp.block_tokens, case.cfg.mask_id)
    masks = np.full(case.ns, (1 << case.S) - 1, dtype=np.uint64)
    g.set_state(full, masks, inp.prefix_len)
    n = g.generate_block(0.9, 8, max_steps=64, masked_hint=case.S)
    assert n == (case.S + 7) // 8
    st = g.state()
    assert not st["mask"].any()
