"""Pins of the oracle's hierarchical decoder (Appendix "Hierarchical decoding") and of the outer generation loop with
early termination (Section 3, system optimisations).  The paper gives hierarchical decoding in prose; the pins fix
the reading taken: the limits in which it is plain threshold decoding, a hand-worked example, the ideal case in which a
block of 2^k - 1 positions is decoded in k passes (1, 2, 4, ... commits), tie order, and the defining properties
checked by brute force over every mask of a short block."""
import itertools

import numpy as np
import pytest

import dinfer_inputs as di
import oracle


def runs(mask, S):
    out, i = [], 0
    while i < S:
        if (mask >> i) & 1:
            j = i
            while j + 1 < S and (mask >> (j + 1)) & 1:
                j += 1
            out.append((i, j))
            i = j + 1
        else:
            i += 1
    return out


def test_without_a_lower_boundary_it_is_threshold_decoding():
    """tau_low above every confidence: no region resolves on the lower boundary, what is left is the threshold rule
    with its at-least-one fallback."""
    rng = np.random.default_rng(3)
    for trial in range(200):
        S = int(rng.integers(1, 65))
        conf = rng.random(S)
        am = rng.integers(0, 1000, S).astype(np.int32)
        mask = int(rng.integers(0, 1 << 62)) & ((1 << S) - 1)
        tok = np.full(S, -7, dtype=np.int32)
        tau = float(rng.choice([0.3, 0.7, 0.95, 1.5]))
        assert_same(oracle.commit_hier(conf, am, mask, tok, tau, 2.0), oracle.commit(conf, am, mask, tok, tau))


def test_lower_boundary_equal_to_the_threshold_changes_nothing():
    """tau_low = tau_high: a region without a position at tau_high has none at tau_low either."""
    rng = np.random.default_rng(4)
    for trial in range(100):
        S = 32
        conf = rng.random(S)
        am = rng.integers(0, 1000, S).astype(np.int32)
        mask = int(rng.integers(0, 1 << 32))
        tok = np.zeros(S, dtype=np.int32)
        assert_same(oracle.commit_hier(conf, am, mask, tok, 0.8, 0.8), oracle.commit(conf, am, mask, tok, 0.8))


def assert_same(a, b):
    assert a[0] == b[0] and a[1] == b[1] and np.array_equal(a[2], b[2])


def test_hand_worked_example():
    """Block of 12; positions 0-4 and 7-10 are masked (two runs), 5, 6, 11 decided.
    run 0..4: 0.95 at position 1 reaches 0.92 -> committed; the run has a commit, the 0.7 at position 3 stays.
    run 7..10: nothing at 0.92; at least 0.62: positions 7 (0.80) and 10 (0.65); centre 8.5, distances 1.5 and 1.5:
    the more confident one, 7, is committed."""
    conf = np.array([0.1, 0.95, 0.2, 0.7, 0.3, 0.99, 0.99, 0.80, 0.5, 0.6, 0.65, 0.99])
    am = np.arange(100, 112).astype(np.int32)
    mask = 0b011110011111
    tok = np.full(12, -1, dtype=np.int32)
    n, m, t = oracle.commit_hier(conf, am, mask, tok, 0.92, 0.62)
    assert n == 2 and m == mask & ~((1 << 1) | (1 << 7))
    assert t[1] == 101 and t[7] == 107 and np.all(np.delete(t, [1, 7]) == -1)
    # the same with position 9 lifted to 0.63: it is closer to the centre (distance 0.5) and wins over 7
    conf[9] = 0.63
    n, m, t = oracle.commit_hier(conf, am, mask, tok, 0.92, 0.62)
    assert n == 2 and m == mask & ~((1 << 1) | (1 << 9))


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 6])
def test_ideal_case_takes_log_n_passes(k):
    """Every confidence between the two thresholds, block of 2^k - 1 masked positions: pass t commits the centres of
    the 2^(t-1) runs, which have length 2^(k-t+1) - 1, so the block is done after k passes."""
    S = (1 << k) - 1
    conf = np.full(S, 0.75)
    am = np.arange(S).astype(np.int32)
    tok = np.full(S, -1, dtype=np.int32)
    mask = (1 << S) - 1
    for t in range(1, k + 1):
        n, mask, tok = oracle.commit_hier(conf, am, mask, tok, 0.92, 0.62)
        assert n == 1 << (t - 1)
        length = (1 << (k - t)) - 1
        assert all(b - a + 1 == length for a, b in runs(mask, S))
    assert mask == 0 and np.array_equal(tok, am)


def test_tie_order():
    am = np.arange(4).astype(np.int32)
    tok = np.full(4, -1, dtype=np.int32)
    # run 0..3, centre 1.5: positions 1 and 2 are equally close; equal confidence -> the lower position
    n, m, _ = oracle.commit_hier(np.array([0.7, 0.7, 0.7, 0.7]), am, 0b1111, tok, 0.92, 0.62)
    assert (n, m) == (1, 0b1101)
    # the more confident of the two
    n, m, _ = oracle.commit_hier(np.array([0.9, 0.7, 0.71, 0.9]), am, 0b1111, tok, 0.92, 0.62)
    assert (n, m) == (1, 0b1011)
    # distance beats confidence
    n, m, _ = oracle.commit_hier(np.array([0.91, 0.1, 0.63, 0.1]), am, 0b1111, tok, 0.92, 0.62)
    assert (n, m) == (1, 0b1011)
    # nothing reaches the lower boundary: the single most confident position, lowest on ties
    n, m, _ = oracle.commit_hier(np.array([0.2, 0.5, 0.5, 0.1]), am, 0b1111, tok, 0.92, 0.62)
    assert (n, m) == (1, 0b1101)
    # boundaries are inclusive
    n, m, _ = oracle.commit_hier(np.array([0.92, 0.1, 0.62, 0.1]), am, 0b0101, tok, 0.92, 0.62)
    assert (n, m) == (2, 0)


def test_properties_by_brute_force():
    """Every mask of a block of 7 and confidences drawn from a small set (ties on purpose): the result is checked
    against the properties that define the rule, not against a second implementation of it."""
    S, hi, lo = 7, 0.92, 0.62
    levels = np.array([0.1, 0.5, 0.62, 0.7, 0.92, 0.97])
    rng = np.random.default_rng(11)
    am = (np.arange(S) + 50).astype(np.int32)
    for mask in range(1 << S):
        for trial in range(12):
            conf = levels[rng.integers(0, len(levels), S)]
            tok = np.full(S, -1, dtype=np.int32)
            n, m, t = oracle.commit_hier(conf, am, mask, tok, hi, lo)
            sel = mask & ~m
            assert m & ~mask == 0 and bin(sel).count("1") == n
            for i in range(S):
                assert t[i] == (am[i] if (sel >> i) & 1 else -1)
            if mask == 0:
                assert n == 0
                continue
            assert n >= 1
            picked_by_rule = 0
            for a, b in runs(mask, S):
                idx = list(range(a, b + 1))
                high = [i for i in idx if conf[i] >= hi]
                chosen = [i for i in idx if (sel >> i) & 1]
                if high:
                    assert chosen == high
                    picked_by_rule += len(high)
                    continue
                cands = [i for i in idx if conf[i] >= lo]
                if cands:
                    picked_by_rule += 1
                    assert len(chosen) == 1 and chosen[0] in cands
                    c = chosen[0]
                    for j in cands:       # nobody strictly closer to the centre; at equal distance nobody more confident
                        dj, dc = abs(2 * j - (a + b)), abs(2 * c - (a + b))
                        assert dj >= dc and (dj > dc or conf[j] < conf[c] or (conf[j] == conf[c] and j >= c))
            if picked_by_rule == 0:
                masked = [i for i in range(S) if (mask >> i) & 1]
                best = max(masked, key=lambda i: (conf[i], -i))
                assert sel == 1 << best
            else:
                assert n == picked_by_rule


@pytest.fixture(scope="module")
def tiny():
    wl = di.workload_preset(1)
    cfg = wl.model
    w = di.make_weights(cfg, di.BASE_SEED + 1)
    inp = di.make_workload_inputs(wl)
    o = oracle.Oracle(cfg, w)
    kc, vc = o.new_cache(200)
    o.forward(inp.prefix_tokens[0], 0, kc, vc)
    return wl, cfg, w, inp, o, kc, vc


def test_step_hier_is_the_step_with_the_other_commit_rule(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    plain = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 2.0, want_logits=True)
    q = np.sort(plain["conf"])
    hi, lo = float(q[-3]), float(q[len(q) // 2])
    k2, v2 = kc.copy(), vc.copy()
    r = o.step_hier(inp.block_tokens[0], int(inp.mask_bits[0]), 64, k2, v2, hi, lo, want_logits=True)
    assert np.array_equal(r["logits"], plain["logits"]) and np.array_equal(r["conf"], plain["conf"])
    n, m, t = oracle.commit_hier(plain["conf"], plain["argmax"], int(inp.mask_bits[0]), inp.block_tokens[0], hi, lo)
    assert (r["n_committed"], r["mask"]) == (n, m) and np.array_equal(r["tokens"], t)
    assert n >= 3


def test_generate_without_eos_is_the_block_loop(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    S, nb = 16, 3
    k1, v1 = kc.copy(), vc.copy()
    g = o.generate(S, nb, 64, k1, v1, 0.9, fixed_k=4)
    assert g["blocks"] == nb and np.all(g["steps"] == 4)
    k2, v2 = kc.copy(), vc.copy()
    for b in range(nb):
        blk = o.generate_block(np.full(S, cfg.mask_id, dtype=np.int32), (1 << S) - 1, 64 + b * S, k2, v2, 0.9, fixed_k=4)
        o.forward(blk["tokens"], 64 + b * S, k2, v2)
        assert np.array_equal(g["tokens"][b * S:(b + 1) * S], blk["tokens"])
    assert np.array_equal(k1, k2) and np.array_equal(v1, v2)
    assert np.array_equal(k1[:, :64], kc[:, :64])


def test_generate_stops_at_eos_and_fills_the_rest(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    S, nb = 16, 4
    free = o.generate(S, nb, 64, kc.copy(), vc.copy(), 0.9, fixed_k=4)
    tokens = free["tokens"].reshape(nb, S)
    # an id that a block after the first produces and no earlier block does (the random-init model repeats itself)
    b, eos = next((b, int(t)) for b in range(1, nb - 1) for t in tokens[b] if t not in tokens[:b])
    k1, v1 = kc.copy(), vc.copy()
    g = o.generate(S, nb, 64, k1, v1, 0.9, fixed_k=4, eos_id=eos)
    out = g["tokens"].reshape(nb, S)
    assert g["blocks"] == b + 1 and len(g["steps"]) == b + 1
    assert np.array_equal(out[:b + 1], tokens[:b + 1]) and np.all(out[b + 1:] == eos)
    assert np.all(k1[:, 64 + (b + 1) * S:] == 0), "no forward ran on the skipped blocks"
    # an id of block 0 stops after the first block
    g0 = o.generate(S, nb, 64, kc.copy(), vc.copy(), 0.9, fixed_k=4, eos_id=int(tokens[0][5]))
    assert g0["blocks"] == 1 and np.all(g0["tokens"][S:] == int(tokens[0][5]))
