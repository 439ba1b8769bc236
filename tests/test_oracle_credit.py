"""Pins of the oracle's credit decoding (Appendix "Credit decoding", equations 1 and 2): the limits in which it
reduces to plain decoding, closed forms of a single boosted logit and of the geometric credit recurrence, a
constructed case in which accumulated credit overturns the current arg max, and brute force over a tiny vocabulary
with library routines."""
import numpy as np
import pytest
from scipy.special import log1p, softmax

import dinfer_inputs as di
import oracle


def test_alpha_zero_is_plain_decoding_but_credits_still_accumulate():
    rng = np.random.default_rng(0)
    z = rng.standard_normal(50) * 2
    credit = np.zeros(50)
    conf, am, fused = oracle.credit_position(z, credit, 0.0, 0.9, 0.5)
    p = softmax(z)
    assert am == int(p.argmax()) and abs(conf - p.max()) < 1e-15 and np.array_equal(fused, z)
    assert credit[am] == pytest.approx(p.max() ** 0.5) and np.count_nonzero(credit) == 1


def test_first_step_closed_form():
    """From zero credit only the top-1 logit moves, by alpha*log(1 + p^gamma): its probability becomes
    p*b / (1 - p + p*b) with b = (1 + p^gamma)^alpha, and every other probability shrinks by the same factor."""
    z = np.array([0.3, 2.0, -1.0, 1.5, 0.0])
    alpha, beta, gamma = 0.65, 0.7, 0.4
    credit = np.zeros(5)
    conf, am, fused = oracle.credit_position(z, credit, alpha, beta, gamma)
    p = float(softmax(z)[1])
    b = (1.0 + p ** gamma) ** alpha
    assert am == 1 and conf == pytest.approx(p * b / (1.0 - p + p * b), rel=1e-14)
    assert conf > p                                   # a boost never lowers the leader
    assert np.array_equal(np.delete(fused, 1), np.delete(z, 1))


def test_credit_recurrence_is_geometric():
    """The same logits n times: C_n = p^gamma * (1 - beta^n) / (1 - beta) on the leader, zero elsewhere; and once the
    leader changes, the old credit decays as beta^m."""
    z = np.array([1.0, 0.2, -0.5])
    beta, gamma = 0.8, 0.5
    credit = np.zeros(3)
    p = float(softmax(z)[0])
    for n in range(1, 8):
        oracle.credit_position(z, credit, 0.0, beta, gamma)
        assert credit[0] == pytest.approx(p ** gamma * (1 - beta ** n) / (1 - beta), rel=1e-13)
        assert credit[1] == 0.0 and credit[2] == 0.0
    c7 = credit[0]
    z2 = np.array([0.0, 3.0, 0.0])
    for m in range(1, 4):
        oracle.credit_position(z2, credit, 0.0, beta, gamma)
        assert credit[0] == pytest.approx(c7 * beta ** m, rel=1e-13)


def test_accumulated_credit_overturns_a_narrow_lead():
    """Token 0 leads for five steps; then token 1 gets ahead by 0.05 in the logits.  With alpha = 1 token 0 keeps
    log(1 + C) >> 0.05 of prior, token 1 has only its first reward: the enhanced arg max stays token 0, while with
    alpha = 0 it follows the logits."""
    lead = np.array([2.0, 1.0, 0.0, 0.0])
    late = np.array([2.0, 2.05, 0.0, 0.0])
    for alpha, want in ((1.0, 0), (0.0, 1)):
        credit = np.zeros(4)
        for _ in range(5):
            oracle.credit_position(lead, credit, alpha, 0.9, 0.5)
        conf, am, fused = oracle.credit_position(late, credit, alpha, 0.9, 0.5)
        assert am == want
        assert credit[1] > 0 and credit[0] > 2 * credit[1]      # both were rewarded, token 0 five times


def test_ties_go_to_the_lower_id():
    z = np.array([1.0, 1.0, 0.0])
    credit = np.zeros(3)
    conf, am, _ = oracle.credit_position(z, credit, 0.5, 0.9, 0.5)
    assert am == 0 and credit[0] > 0 and credit[1] == 0


def test_brute_force_over_a_tiny_vocabulary():
    """Several steps with changing logits, redone with library routines on dense arrays."""
    rng = np.random.default_rng(3)
    V, alpha, beta, gamma = 12, 0.8, 0.85, 0.6
    credit = np.zeros(V)
    mine = np.zeros(V)
    for t in range(10):
        z = rng.standard_normal(V) * 1.5
        conf, am, fused = oracle.credit_position(z, credit, alpha, beta, gamma)
        p = softmax(z)
        mine *= beta
        mine[int(np.argmax(p))] += p.max() ** gamma
        q = softmax(z + alpha * log1p(mine))
        assert np.allclose(credit, mine, rtol=1e-13, atol=0)
        assert am == int(np.argmax(q)) and conf == pytest.approx(float(q.max()), rel=1e-13)


@pytest.fixture(scope="module")
def tiny():
    wl = di.workload_preset(1)
    cfg = wl.model
    w = di.make_weights(cfg, di.BASE_SEED + 1)
    inp = di.make_workload_inputs(wl)
    o = oracle.Oracle(cfg, w)
    kc, vc = o.new_cache(128)
    o.forward(inp.prefix_tokens[0], 0, kc, vc)
    return wl, cfg, inp, o, kc, vc


def test_step_with_alpha_zero_is_the_plain_step(tiny):
    wl, cfg, inp, o, kc, vc = tiny
    credit = np.zeros((wl.block_len, cfg.vocab))
    a = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.05, want_logits=True)
    b = o.step_credit(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.05, credit, 0.0, 0.9, 0.5,
                      want_logits=True)
    for key in ("tokens", "conf", "argmax", "logits"):
        assert np.array_equal(a[key], b[key]), key
    assert a["mask"] == b["mask"] and np.count_nonzero(credit) == wl.block_len


def test_step_touches_only_masked_rows_and_raises_their_confidence(tiny):
    wl, cfg, inp, o, kc, vc = tiny
    S = wl.block_len
    tokens = inp.block_tokens[0].copy()
    tokens[[2, 7]] = [11, 12]
    mask = int(inp.mask_bits[0]) & ~((1 << 2) | (1 << 7))
    credit = np.zeros((S, cfg.vocab))
    plain = o.step(tokens, mask, 64, kc.copy(), vc.copy(), 2.0)
    first = o.step_credit(tokens, mask, 64, kc.copy(), vc.copy(), 2.0, credit, 0.65, 0.7, 0.5)
    assert not credit[2].any() and not credit[7].any()
    assert first["conf"][2] == plain["conf"][2] and first["conf"][7] == plain["conf"][7]
    masked = [i for i in range(S) if (mask >> i) & 1]
    assert all(first["conf"][i] > plain["conf"][i] for i in masked)
    assert np.array_equal(first["argmax"], plain["argmax"])          # one boost of the leader keeps the leader
    # the threshold rule then acts on the enhanced confidences: more positions can pass the same threshold
    tau = float(np.median(plain["conf"][masked]))
    c2 = np.zeros((S, cfg.vocab))
    n_plain = o.step(tokens, mask, 64, kc.copy(), vc.copy(), tau)["n_committed"]
    n_credit = o.step_credit(tokens, mask, 64, kc.copy(), vc.copy(), tau, c2, 0.65, 0.7, 0.5)["n_committed"]
    assert n_credit >= n_plain
