"""Pins of the oracle's iteration smoothing (Appendix "IterSmooth": e_{t+1}[i] = e_mask + alpha_t * softmax(z_t[i]) .
W_emb on the positions that stay masked): the expected embedding against library routines and its one-hot limit,
the embedding addend through the linearity of the embedding stage, and the step's limits."""
import numpy as np
import pytest
from scipy.special import softmax

import dinfer_inputs as di
import oracle


@pytest.fixture(scope="module")
def tiny():
    wl = di.workload_preset(1)
    cfg = wl.model
    w = di.make_weights(cfg, di.BASE_SEED + 1)
    inp = di.make_workload_inputs(wl)
    o = oracle.Oracle(cfg, w)
    kc, vc = o.new_cache(128)
    o.forward(inp.prefix_tokens[0], 0, kc, vc)
    return wl, cfg, w, inp, o, kc, vc


def test_expected_embedding_is_the_probability_weighted_mean_of_embedding_rows(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    rng = np.random.default_rng(5)
    z = rng.standard_normal(cfg.vocab) * 3
    want = softmax(z) @ w["emb"].astype(np.float64)
    assert np.allclose(o.expected_embedding(z), want, rtol=1e-12, atol=1e-15)
    # a distribution concentrated on one token returns that token's embedding row
    z = np.full(cfg.vocab, -50.0)
    z[1234] = 50.0
    assert np.allclose(o.expected_embedding(z), w["emb"][1234], rtol=1e-12, atol=1e-30)
    # uniform logits: the mean row
    assert np.allclose(o.expected_embedding(np.zeros(cfg.vocab)), w["emb"].astype(np.float64).mean(0), rtol=1e-12)


def test_embedding_addend_enters_before_the_first_layer(tiny):
    """Adding W_emb[b] - W_emb[a] to the embedding of token a is the forward of token b (the stage is a sum)."""
    wl, cfg, w, inp, o, kc, vc = tiny
    emb = w["emb"].astype(np.float64)
    a = np.array([5, 17, 99, 400], dtype=np.int32)
    b = np.array([5, 2000, 98, 7], dtype=np.int32)
    k1, v1, k2, v2 = kc.copy(), vc.copy(), kc.copy(), vc.copy()
    h_b = o.forward(b, 64, k1, v1)
    h_a = o.forward_embedded(a, emb[b] - emb[a], 64, k2, v2)
    assert np.allclose(h_a, h_b, rtol=1e-9, atol=1e-12)
    assert np.allclose(k1, k2, atol=1e-12) and np.allclose(v1, v2, atol=1e-12)
    # and a zero addend is the plain forward, bit for bit
    k3, v3 = kc.copy(), vc.copy()
    assert np.array_equal(o.forward_embedded(b, np.zeros((4, cfg.hidden)), 64, k3, v3), h_b)


def test_first_step_is_the_plain_step_and_retains_the_expected_embeddings(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    S = wl.block_len
    tokens = inp.block_tokens[0].copy()
    tokens[4] = 77
    mask = int(inp.mask_bits[0]) & ~(1 << 4)
    delta = np.zeros((S, cfg.hidden))
    a = o.step(tokens, mask, 64, kc.copy(), vc.copy(), 0.05, want_logits=True)
    b = o.step_smooth(tokens, mask, 64, kc.copy(), vc.copy(), 0.05, 0.3, delta, want_logits=True)
    for key in ("tokens", "conf", "argmax", "logits"):
        assert np.array_equal(a[key], b[key]), key
    emb = w["emb"].astype(np.float64)
    for i in range(S):
        if i == 4:
            assert not delta[i].any()                       # decided before the step: nothing retained
        else:
            assert np.allclose(delta[i], softmax(a["logits"][i]) @ emb, rtol=1e-11, atol=1e-15)


def test_second_step_embeds_mask_plus_alpha_delta_on_masked_positions_only(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    S, H = wl.block_len, cfg.hidden
    rng = np.random.default_rng(2)
    delta = rng.standard_normal((S, H)) * 0.01
    tokens = inp.block_tokens[0].copy()
    tokens[[1, 30]] = [9, 10]
    mask = int(inp.mask_bits[0]) & ~((1 << 1) | (1 << 30))
    alpha = 0.25
    d2 = delta.copy()
    got = o.step_smooth(tokens, mask, 64, kc.copy(), vc.copy(), 2.0, alpha, d2, want_logits=True)
    add = alpha * delta
    add[[1, 30]] = 0.0
    hid = o.forward_embedded(tokens, add, 64, kc.copy(), vc.copy())
    assert np.array_equal(got["logits"], o.logits(hid))
    # alpha = 0 ignores what was retained
    d3 = delta.copy()
    zero = o.step_smooth(tokens, mask, 64, kc.copy(), vc.copy(), 2.0, 0.0, d3, want_logits=True)
    plain = o.step(tokens, mask, 64, kc.copy(), vc.copy(), 2.0, want_logits=True)
    assert np.array_equal(zero["logits"], plain["logits"])
    assert np.array_equal(d3[[1, 30]], delta[[1, 30]])        # rows of decided positions are left alone
    assert not np.allclose(got["logits"], plain["logits"])    # and the addend does matter
