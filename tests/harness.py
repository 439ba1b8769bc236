"""Shared plumbing of the GPU parity tests, the smoke check and the benchmark's baseline leg: run the same
seeded workload through the CPU oracle and through the HIP library, and compare under the stated bars.

Bars (block-denoising benchmark statement): committed ids and positions bit-exact except at positions
flagged as within `tau_margin` of the threshold or at an arg-max / most-confident near-tie; logits within
relative `logit_rel` of the row's largest |logit|; confidences within absolute `conf_abs`.
"""
import json
import os
from dataclasses import dataclass

import numpy as np

import dinfer_inputs as di
import oracle


@dataclass
class Bars:
    logit_rel: float
    conf_abs: float
    conf_rel: float      # extra, tighter than the stated bar when confidences are tiny
    tau_margin: float
    kv_abs: float
    router_rel: float    # two router probabilities closer than this (relative) count as a near-tie


# Worst margins seen, per test: every routing / K,V / logits / confidence comparison records how much of its bar it
# used, keyed by the running test.  conftest.py prints the table at the end of the session and writes it to
# the file named by DINFER_PARITY_STATS, so that the head-room under every bar is visible and not only "passed".
STATS = {}


def _record(key, value, where=None):
    test = os.environ.get("PYTEST_CURRENT_TEST", "(no test)").split(" ")[0]
    slot = STATS.setdefault(test, {})
    if value > slot.get(key, -1.0):
        slot[key] = float(value)
        if where is not None:
            slot[key + "_at"] = [int(x) for x in where]


def dump_stats(path=None):
    """Worst value per key over all tests, and the per-test table as JSON (if a path is given)."""
    worst = {}
    for test, slot in STATS.items():
        for k, v in slot.items():
            if not k.endswith("_at") and v > worst.get(k, (-1.0, ""))[0]:
                worst[k] = (v, test)
    if path:
        os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
        with open(path, "w") as f:
            json.dump({"worst": {k: {"value": v, "test": t} for k, (v, t) in worst.items()}, "per_test": STATS}, f,
                      indent=1)
    return worst


def bars_for(cfg):
    if cfg.dtype == "f32":
        # float32 kernels against the float64 oracle: rounding only
        return Bars(logit_rel=2e-4, conf_abs=2e-5, conf_rel=2e-3, tau_margin=1e-4, kv_abs=1e-4, router_rel=1e-4)
    # bf16 inputs, float32 accumulation.
    # router_rel: two experts' probabilities differ by the factor exp(h . (w_a - w_b)); an error dh of the normalised
    # row h moves that exponent by dh . (w_a - w_b), whose spread is sqrt(2) times that of a logit error dh . w_v
    # (router and LM-head weights have the same scale).  The logit errors measured at the full shapes have a standard
    # deviation of about 7e-3 (largest 0.037 over 5e6 logits), so the exponent moves by about 1e-2 (one sigma) and a
    # choice between experts can flip up to about 3.5 sigma = 3.5e-2 over the ~2000 routings of a step.  The
    # largest gap of a flipped choice seen over all full-shape cases is 1.26e-2; the bar is twice that.
    return Bars(logit_rel=2e-2, conf_abs=1e-3, conf_rel=8e-2, tau_margin=1e-3, kv_abs=3e-2, router_rel=2.5e-2)


class OracleRun:
    """Oracle state of a workload: one KV cache per sequence, prefilled from the prompt."""

    def __init__(self, cfg, weights, inp, cap):
        self.o = oracle.Oracle(cfg, weights)
        self.cfg, self.inp = cfg, inp
        self.caches = []
        for s, toks in enumerate(inp.prefix_tokens):
            kc, vc = self.o.new_cache(cap)
            if len(toks):
                self.o.forward(toks, 0, kc, vc)
            self.caches.append((kc, vc))

    def step(self, s, tokens, mask, prefix_len, threshold, fixed_k=0, want_logits=False, trace=None):
        kc, vc = self.caches[s]
        return self.o.step(tokens, mask, prefix_len, kc, vc, threshold, fixed_k, want_logits, trace)

    def step_following(self, s, tokens, mask, prefix_len, threshold, fixed_k, gpu_routing, bars, want_logits=True):
        """The oracle's step with the expert sets the HIP path chose (gpu_routing: [L][S][k]).  The top-k of
        the router is a discrete decision on floating-point values: where the oracle's own probabilities put
        the k-th and (k+1)-th within `router_rel`, either set is valid and the oracle follows the GPU so that
        the rest of the forward stays comparable; anywhere else the sets must be equal.  Returns
        (step result, number of (layer, token) routings that were near-ties)."""
        tr = oracle.Trace(self.cfg, len(tokens), forced_idx=gpu_routing)
        ref = self.step(s, tokens, mask, prefix_len, threshold, fixed_k, want_logits, tr)
        return ref, check_routing(tr, gpu_routing, self.cfg.top_k, bars)

    def step_vicinity_following(self, s, tokens, vicinity_tokens, mask, prefix_len, threshold, fixed_k, gpu_routing,
                                bars):
        """step_following for the vicinity-refresh step; gpu_routing: [L][look_back + S][k]."""
        kc, vc = self.caches[s]
        tr = oracle.Trace(self.cfg, len(vicinity_tokens) + len(tokens), forced_idx=gpu_routing)
        ref = self.o.step_vicinity(tokens, vicinity_tokens, mask, prefix_len, kc, vc, threshold, fixed_k, True, tr)
        return ref, check_routing(tr, gpu_routing, self.cfg.top_k, bars)

    def forward_following(self, s, tokens, prefix_len, gpu_routing, bars):
        """A forward without decoder (prefill, or the refresh of a decoded block) that follows the GPU's
        expert sets through router near-ties, as step_following does.  Writes K,V into sequence s's cache."""
        kc, vc = self.caches[s]
        tr = oracle.Trace(self.cfg, len(tokens), forced_idx=gpu_routing)
        self.o.forward(tokens, prefix_len, kc, vc, tr)
        return check_routing(tr, gpu_routing, self.cfg.top_k, bars)


class GpuRun:
    """The HIP library on the same workload.  Imports torch / the binding lazily (GPU machine only)."""

    def __init__(self, cfg, weights, inp, max_tokens, max_pos, weights_buffer=None):
        """weights_buffer: device tensor of an earlier GpuRun of the same model (skips the upload)."""
        import torch
        from paper_2510_08666_amd import binding
        self.torch, self.binding = torch, binding
        self.cfg, self.inp = cfg, inp
        self.dev = torch.device("cuda:0")
        self.ctx = binding.Context(cfg, inp.n_pages, max(1, len(inp.prefix_tokens)), max_tokens, max_pos,
                                   weights_buffer=weights_buffer)
        if weights_buffer is None:
            self.ctx.load_weights(weights)
        self.page_table = torch.from_numpy(inp.page_table).to(self.dev)
        self.prefix_len = torch.from_numpy(inp.prefix_len.astype(np.int32)).to(self.dev)
        self.tokens = torch.from_numpy(inp.block_tokens.copy()).to(self.dev)
        self.mask = torch.from_numpy(inp.mask_bits.view(np.int64).copy()).to(self.dev)
        ns, S = inp.block_tokens.shape
        self.conf = torch.zeros((ns, S), dtype=torch.float32, device=self.dev)
        self.argmax = torch.zeros((ns, S), dtype=torch.int32, device=self.dev)
        self.n_committed = torch.zeros(ns, dtype=torch.int32, device=self.dev)

    def prefill(self):
        torch = self.torch
        toks = torch.from_numpy(np.concatenate(self.inp.prefix_tokens).astype(np.int32)).to(self.dev)
        self.ctx.prefill(toks, [len(t) for t in self.inp.prefix_tokens], self.page_table)

    def inject_prefix(self, caches):
        """Write the oracle's prefix K,V into the pool, so that a step is judged apart from prefill error."""
        torch = self.torch
        for s, (kc, vc) in enumerate(caches):
            P = int(self.inp.prefix_len[s])
            if P == 0:
                continue
            for l in range(self.cfg.n_layers):
                k = torch.from_numpy(kc[l, :P].astype(np.float32)).to(self.dev)
                v = torch.from_numpy(vc[l, :P].astype(np.float32)).to(self.dev)
                self.ctx.kv_write(l, self.page_table[s], 0, k, v)
        torch.cuda.synchronize()

    def read_kv(self, s, layer, first, n):
        k, v = self.ctx.kv_read(layer, self.page_table[s], first, n)
        return k.cpu().numpy(), v.cpu().numpy()

    def set_state(self, tokens, masks, prefix_len=None):
        torch = self.torch
        self.tokens.copy_(torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)))
        self.mask.copy_(torch.from_numpy(np.asarray(masks, dtype=np.uint64).view(np.int64)))
        if prefix_len is not None:
            self.prefix_len.copy_(torch.from_numpy(np.asarray(prefix_len, dtype=np.int32)))

    def step(self, threshold, fixed_k=0):
        self.ctx.step(self.tokens, self.mask, self.prefix_len, self.page_table, threshold, fixed_k, self.conf,
                      self.argmax, self.n_committed)
        self.torch.cuda.synchronize()
        return self.state()

    def credit_state(self):
        """Fresh (empty) credit lists for every position of the block."""
        torch, cap = self.torch, self.binding.CREDIT_CAP
        ns, S = self.tokens.shape
        return dict(ids=torch.zeros((ns, S, cap), dtype=torch.int32, device=self.dev),
                    val=torch.zeros((ns, S, cap), dtype=torch.float32, device=self.dev),
                    n=torch.zeros((ns, S), dtype=torch.int32, device=self.dev))

    def step_credit(self, credit, threshold, alpha, beta, gamma, fixed_k=0):
        self.ctx.step_credit(self.tokens, self.mask, self.prefix_len, self.page_table, threshold, fixed_k, alpha, beta,
                             gamma, credit["ids"], credit["val"], credit["n"], self.conf, self.argmax, self.n_committed)
        self.torch.cuda.synchronize()
        return self.state()

    def smooth_state(self):
        """Zero expected embeddings [n_seq][S][H] and the scratch buffer of the smoothing step."""
        ns, S = self.tokens.shape
        return dict(delta=self.torch.zeros((ns, S, self.cfg.hidden), dtype=self.torch.float32, device=self.dev),
                    scratch=self.ctx.smooth_scratch(ns * S))

    def step_smooth(self, smooth, alpha, threshold, fixed_k=0):
        self.ctx.step_smooth(self.tokens, self.mask, self.prefix_len, self.page_table, threshold, fixed_k, alpha,
                             smooth["delta"], smooth["scratch"], self.conf, self.argmax, self.n_committed)
        self.torch.cuda.synchronize()
        return self.state()

    def step_vicinity(self, vicinity_tokens, threshold, fixed_k=0):
        """vicinity_tokens: [n_seq][look_back] ids of the cached positions right before each block."""
        vic = self.torch.from_numpy(np.ascontiguousarray(vicinity_tokens, dtype=np.int32)).to(self.dev)
        self.ctx.step_vicinity(self.tokens, vic, self.mask, self.prefix_len, self.page_table, threshold, fixed_k,
                               self.conf, self.argmax, self.n_committed)
        self.torch.cuda.synchronize()
        return self.state()

    def state(self):
        return dict(tokens=self.tokens.cpu().numpy(), mask=self.mask.cpu().numpy().view(np.uint64),
                    conf=self.conf.cpu().numpy(), argmax=self.argmax.cpu().numpy(),
                    n_committed=self.n_committed.cpu().numpy())

    def routing(self, T=None):
        """Expert ids of every layer of the last forward: [L][T][k]."""
        T = self.tokens.numel() if T is None else T
        shape = (self.cfg.n_layers, T, self.cfg.top_k)
        out = self.ctx.debug_get(1, shape, self.torch.int32)
        self.torch.cuda.synchronize()
        return out.cpu().numpy()

    def logits(self, n_rows):
        out = self.ctx.debug_logits(n_rows)
        self.torch.cuda.synchronize()
        return out.cpu().numpy()

    def refresh(self):
        self.ctx.refresh_block(self.tokens, self.prefix_len, self.page_table)
        self.torch.cuda.synchronize()

    def generate_block(self, threshold, fixed_k, max_steps, masked_hint=0, steps_per_wait=1):
        steps = self.ctx.generate_block(self.tokens, self.mask, self.prefix_len, self.page_table, threshold, fixed_k,
                                        self.conf, self.argmax, self.n_committed, max_steps, masked_hint, steps_per_wait)
        self.torch.cuda.synchronize()
        return steps

    def close(self):
        self.ctx.close()


def check_routing(trace, gpu_routing, top_k, bars, stats=None):
    """Every expert the GPU chose that the oracle did not (and vice versa) must sit within router_rel of the
    oracle's k-th largest probability.  Returns how many (layer, token) routings differed; `stats` (a dict)
    receives the largest relative gap seen."""
    flagged, worst, where = 0, 0.0, None
    L, T, _ = gpu_routing.shape
    for l in range(L):
        for t in range(T):
            mine, theirs = set(trace.topk_idx[l, t].tolist()), set(gpu_routing[l, t].tolist())
            assert len(theirs) == top_k, "GPU routing repeats an expert at layer %d token %d" % (l, t)
            if mine == theirs:
                continue
            p = trace.router_p[l, t]
            kth = np.sort(p)[::-1][top_k - 1]
            for e in mine ^ theirs:
                gap = abs(p[e] - kth) / kth
                if gap > worst:
                    worst, where = gap, (l, t, e)
            flagged += 1
    if stats is not None:
        stats["router_worst_gap"] = worst
        stats["router_worst_at"] = where
    _record("router_gap", worst, where)
    _record("router_gap_of_bar", worst / bars.router_rel)
    assert worst <= bars.router_rel, "routing differs beyond a near-tie (relative gap %.3g) at layer/token/expert %s" % (
        worst, where)
    return flagged


def max_abs_err(got, ref):
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max()) if np.size(ref) else 0.0


def kv_close(got, ref, bars):
    """Cached K or V rows [n][D] against the oracle's.  They are outputs of a linear layer computed with the same
    arithmetic as the logits (bf16 inputs, float32 accumulation), so they get the same relative bar, per row:
    max |got - ref| <= max(kv_abs, logit_rel * max |ref row|).  The absolute floor alone is too tight once a row
    holds values beyond 4, where bf16 storage and a 0.5 % activation error already add up to 0.03."""
    return kv_err_ratio(got, ref, bars) <= 1.0


def kv_err_ratio(got, ref, bars):
    """Worst row of kv_close: error / allowed."""
    if not np.size(ref):
        return 0.0
    err = np.abs(np.asarray(got, dtype=np.float64) - ref).max(axis=-1)
    allowed = np.maximum(bars.kv_abs, bars.logit_rel * np.abs(ref).max(axis=-1))
    ratio = float((err / allowed).max())
    _record("kv_err_of_bar", ratio)
    return ratio


def compare_logits(ref, got, bars):
    """Per row: max |got - ref| <= logit_rel * max(max |ref|, 1e-3).  Returns the worst ratio error/allowed."""
    worst = 0.0
    for i in range(ref.shape[0]):
        allowed = bars.logit_rel * max(np.abs(ref[i]).max(), 1e-3)
        err = np.abs(got[i].astype(np.float64) - ref[i]).max()
        worst = max(worst, err / allowed)
    _record("logits_err_of_bar", worst)
    assert worst <= 1.0, "logits off by %.3g x the allowed error" % worst
    return worst


def compare_step(ref, got_tokens, got_mask, got_conf, got_argmax, got_n, old_tokens, old_mask, threshold, fixed_k,
                 bars, ref_logits=None, got_logits=None):
    """One sequence, one step.  ref: the oracle's step result.  Returns dict(flagged=..., conf_err=...).

    Positions are flagged (and excused from bit-exactness) when the oracle's own numbers leave the decision
    within the stated bars: a confidence within tau_margin of the threshold; a most-confident / k-th most confident
    choice between positions whose oracle confidences are closer than the two confidence tolerances; an arg max
    whose oracle logit is below the oracle's top logit by no more than the logit errors of the two ids (with the
    HIP path's logits at hand, got_logits: their actual errors; otherwise the logits' bar, twice).  With
    got_logits the reported arg max must also be the first maximum of the HIP path's own logits, exactly."""
    S = len(ref["conf"])
    old_mask, got_mask = int(old_mask), int(got_mask)
    masked = [i for i in range(S) if (old_mask >> i) & 1]
    conf_o, conf_g = ref["conf"], got_conf.astype(np.float64)
    ctol = np.minimum(bars.conf_abs, bars.conf_rel * np.maximum(conf_o, 1e-30))
    cerr = np.abs(conf_g - conf_o)
    _record("conf_err_of_bar", float((cerr / ctol).max()))
    assert np.all(cerr <= ctol), "confidence error %.3g (allowed %.3g) at %d" % (
        cerr.max(), ctol[int(np.argmax(cerr / ctol))], int(np.argmax(cerr / ctol)))
    flagged = set()
    # candidate ids
    for i in range(S):
        if got_logits is not None:
            assert got_argmax[i] == int(np.argmax(got_logits[i])), "arg max at %d is not the first maximum of the logits" % i
        if got_argmax[i] != ref["argmax"][i]:
            assert ref_logits is not None, "arg max differs at %d and no logits to judge a tie" % i
            a, b = int(ref["argmax"][i]), int(got_argmax[i])
            gap = ref_logits[i, a] - ref_logits[i, b]
            if got_logits is not None:
                allowed = abs(float(got_logits[i, a]) - ref_logits[i, a]) + abs(float(got_logits[i, b]) - ref_logits[i, b])
            else:
                allowed = 2 * bars.logit_rel * max(np.abs(ref_logits[i]).max(), 1e-3)
            _record("argmax_tie_gap_of_logit_bar", gap / (bars.logit_rel * max(np.abs(ref_logits[i]).max(), 1e-3)))
            assert gap <= allowed, "arg max differs at %d beyond a near-tie (gap %.3g, allowed %.3g)" % (i, gap, allowed)
            flagged.add(i)
    # structural invariants that hold whatever the numbers are
    assert got_mask & ~old_mask == 0, "a decided position returned to the mask"
    sel_g = old_mask & ~got_mask
    sel_o = old_mask & ~ref["mask"]
    assert bin(sel_g).count("1") == int(got_n)
    assert (int(got_n) >= 1) == (old_mask != 0), "a step with masked positions must commit at least one"
    for i in range(S):
        if (sel_g >> i) & 1:
            assert got_tokens[i] == got_argmax[i]
        else:
            assert got_tokens[i] == old_tokens[i], "an uncommitted position changed"
    # which positions
    if sel_g != sel_o:
        if fixed_k > 0:
            # the k-th and (k+1)-th confidences may be a near-tie
            kth = sorted((conf_o[i] for i in masked), reverse=True)[min(fixed_k, len(masked)) - 1]
            near = {i for i in masked if abs(conf_o[i] - kth) <= 2 * ctol[i]}
        else:
            # a confidence can only end on the other side of the threshold if the oracle's lies within the
            # confidence tolerance of it, which is never more than the stated margin
            near = {i for i in masked if abs(conf_o[i] - threshold) <= min(bars.tau_margin, ctol[i])}
            if not any(conf_o[i] >= threshold + ctol[i] for i in masked):
                best = max(conf_o[i] for i in masked)
                near |= {i for i in masked if best - conf_o[i] <= 2 * ctol[i]}
        diff = {i for i in range(S) if ((sel_g ^ sel_o) >> i) & 1}
        assert diff <= near, "commit sets differ outside flagged positions: %s (flagged %s)" % (sorted(diff), sorted(near))
        flagged |= diff
    for i in range(S):
        if (sel_g >> i) & 1 and (sel_o >> i) & 1 and i not in flagged:
            assert got_tokens[i] == ref["tokens"][i]
    return dict(flagged=sorted(flagged), conf_err=float(cerr.max()), conf_rel_err=float((cerr / conf_o).max()))


def make_case(wl, seed=None, room=None, cfg=None):
    """Weights + inputs of a workload (optionally with a modified model config of the same shapes)."""
    cfg = cfg or wl.model
    seed = di.BASE_SEED + wl.seed_index if seed is None else seed
    weights = di.make_weights(cfg, seed)
    inp = di.make_workload_inputs(wl, seed, room)
    return cfg, weights, inp
