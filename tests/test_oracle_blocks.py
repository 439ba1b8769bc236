"""Pins of the oracle's building blocks against closed forms, invariants, brute force and library routines.

Each test is chosen so that a plausible slip in oracle.c (dropped term, wrong sign or index, transposed
operand, wrong tie rule) makes it fail.
"""
import itertools

import numpy as np
import pytest

import dinfer_inputs as di
import oracle

rng = np.random.default_rng(20251008)


# ---------------------------------------------------------------- linear
def test_linear_is_x_times_w_transposed():
    W = rng.standard_normal((7, 5)).astype(np.float32)       # [out][in], non-square: a transposed read fails
    x = rng.standard_normal((3, 5))
    assert np.allclose(oracle.linear(W, x), x @ W.astype(np.float64).T, rtol=0, atol=1e-13)


def test_linear_reads_bf16_bit_patterns_exactly():
    Wf = rng.standard_normal((6, 9)).astype(np.float32)
    Wb = di.f32_to_bf16(Wf)
    x = rng.standard_normal((2, 9))
    assert np.allclose(oracle.linear(Wb, x), x @ di.bf16_to_f32(Wb).astype(np.float64).T, rtol=0, atol=1e-13)
    one = np.array([[0x3F80, 0x4000, 0xBF80]], dtype=np.uint16)   # 1.0, 2.0, -1.0
    assert oracle.linear(one, np.array([[1.0, 10.0, 100.0]]))[0, 0] == -79.0


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_unit_mean_square_and_scale_invariance():
    x = rng.standard_normal(64) * 3.0
    g = np.ones(64, dtype=np.float32)
    y = oracle.rmsnorm(x, g, 0.0)
    assert abs(np.mean(y * y) - 1.0) < 1e-12
    assert np.allclose(oracle.rmsnorm(5.0 * x, g, 0.0), y, atol=1e-12)
    # closed form on a hand-sized case: x = (3,4): mean square 12.5
    y2 = oracle.rmsnorm(np.array([3.0, 4.0]), np.array([1.0, 2.0], dtype=np.float32), 0.0)
    assert np.allclose(y2, [3.0 / np.sqrt(12.5), 8.0 / np.sqrt(12.5)], atol=1e-15)
    # eps enters under the root, next to the mean (not the sum)
    y3 = oracle.rmsnorm(np.array([3.0, 4.0]), np.ones(2, dtype=np.float32), 12.5)
    assert np.allclose(y3, [3.0 / 5.0, 4.0 / 5.0], atol=1e-15)


# ---------------------------------------------------------------- RoPE
def test_rope_identity_norm_and_closed_form():
    v = rng.standard_normal(8)
    assert np.array_equal(oracle.rope(v, 0, 10000.0), v)
    r = oracle.rope(v, 17, 10000.0)
    assert abs(np.linalg.norm(r) - np.linalg.norm(v)) < 1e-12
    # pair (j, j+hd/2); pair 0 turns by pos radians, pair j by pos * theta^(-2j/hd)
    e = np.zeros(4)
    e[0] = 1.0
    r = oracle.rope(e, 3, 100.0)
    assert np.allclose(r, [np.cos(3.0), 0.0, np.sin(3.0), 0.0], atol=1e-15)
    e = np.zeros(4)
    e[1] = 1.0
    r = oracle.rope(e, 3, 100.0)      # theta^(-2*1/4) = 0.1
    assert np.allclose(r, [0.0, np.cos(0.3), 0.0, np.sin(0.3)], atol=1e-15)


def test_rope_scores_depend_on_relative_position_only():
    q, k = rng.standard_normal(16), rng.standard_normal(16)
    a = oracle.rope(q, 5, 10000.0) @ oracle.rope(k, 2, 10000.0)
    b = oracle.rope(q, 105, 10000.0) @ oracle.rope(k, 102, 10000.0)
    assert abs(a - b) < 1e-12
    c = oracle.rope(q, 6, 10000.0) @ oracle.rope(k, 2, 10000.0)
    assert abs(a - c) > 1e-6


# ---------------------------------------------------------------- attention
def _attention_explicit(q, k, v, nh, hd):
    """sum_j exp(s_ij) v_j / sum_j exp(s_ij), no max subtraction."""
    out = np.zeros_like(q)
    for h in range(nh):
        sl = slice(h * hd, (h + 1) * hd)
        s = q[:, sl] @ k[:, sl].T / np.sqrt(hd)
        e = np.exp(s)
        out[:, sl] = (e @ v[:, sl]) / e.sum(axis=1, keepdims=True)
    return out


def test_attention_equals_explicit_softmax_formula():
    nh, hd, nq, nk = 3, 8, 5, 11
    q = rng.standard_normal((nq, nh * hd))
    k = rng.standard_normal((nk, nh * hd))
    v = rng.standard_normal((nk, nh * hd))
    assert np.allclose(oracle.attention(q, k, v, nh, hd), _attention_explicit(q, k, v, nh, hd), atol=1e-13)


def test_attention_special_cases_and_bidirectionality():
    nh, hd, nq, nk = 2, 4, 6, 9
    k = rng.standard_normal((nk, nh * hd))
    v = rng.standard_normal((nk, nh * hd))
    q0 = np.zeros((nq, nh * hd))
    assert np.allclose(oracle.attention(q0, k, v, nh, hd), np.tile(v.mean(axis=0), (nq, 1)), atol=1e-13)
    vsame = np.tile(rng.standard_normal(nh * hd), (nk, 1))
    q = rng.standard_normal((nq, nh * hd))
    assert np.allclose(oracle.attention(q, k, vsame, nh, hd), vsame[:nq], atol=1e-13)
    # no causal mask: the first query's output changes when the LAST key's value changes
    v2 = v.copy()
    v2[-1] += 1.0
    d = oracle.attention(q, k, v2, nh, hd) - oracle.attention(q, k, v, nh, hd)
    assert np.all(np.abs(d[0]) > 1e-6)
    # large scores do not overflow
    big = oracle.attention(q * 1e3, k, v, nh, hd)
    assert np.all(np.isfinite(big))


def test_attention_matches_torch_sdpa():
    torch = pytest.importorskip("torch")
    nh, hd, nq, nk = 4, 16, 7, 19
    q = rng.standard_normal((nq, nh * hd))
    k = rng.standard_normal((nk, nh * hd))
    v = rng.standard_normal((nk, nh * hd))
    tq = torch.from_numpy(q).view(nq, nh, hd).transpose(0, 1)
    tk = torch.from_numpy(k).view(nk, nh, hd).transpose(0, 1)
    tv = torch.from_numpy(v).view(nk, nh, hd).transpose(0, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).transpose(0, 1).reshape(nq, nh * hd)
    assert np.allclose(oracle.attention(q, k, v, nh, hd), ref.numpy(), atol=1e-12)


# ---------------------------------------------------------------- router / MoE
def test_router_topk_equals_full_sort_and_weights_sum_to_one():
    E, H = 8, 16
    for trial in range(20):
        W = rng.standard_normal((E, H)).astype(np.float32)
        h = rng.standard_normal(H)
        logits = W.astype(np.float64) @ h
        p = np.exp(logits - logits.max())
        p /= p.sum()
        order = sorted(range(E), key=lambda e: (-p[e], e))
        for k in (1, 2, 3, E):
            idx, wt = oracle.router(W, h, k, 1)
            assert list(idx) == order[:k]
            assert abs(wt.sum() - 1.0) < 1e-12
            assert np.allclose(wt, p[order[:k]] / p[order[:k]].sum(), atol=1e-14)
            idx2, wt2 = oracle.router(W, h, k, 0)
            assert list(idx2) == order[:k] and np.allclose(wt2, p[order[:k]], atol=1e-14)


def test_router_ties_go_to_lower_expert():
    W = np.zeros((6, 4), dtype=np.float32)       # all probabilities equal
    idx, wt = oracle.router(W, np.ones(4), 3, 1)
    assert list(idx) == [0, 1, 2] and np.allclose(wt, 1.0 / 3.0)
    W[4, 0] = 1.0
    idx, _ = oracle.router(W, np.ones(4), 3, 1)
    assert list(idx) == [4, 0, 1]


def _tiny_oracle(E, k, H=16, I=24, V=32, L=1, nh=2, hd=8, dtype="f32", norm_topk=1, seed=3):
    cfg = di.ModelConfig("t", n_layers=L, hidden=H, n_heads=nh, head_dim=hd, n_experts=E, top_k=k, moe_inter=I,
                         vocab=V, dtype=dtype, norm_topk=norm_topk, init_std=0.3)
    w = di.make_weights(cfg, seed)
    return oracle.Oracle(cfg, w), cfg, w


def _w64(a):
    return (di.bf16_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)


def _ffn_dense(lw, e, h):
    g = _w64(lw["w_gate"][e]) @ h
    u = _w64(lw["w_up"][e]) @ h
    return _w64(lw["w_down"][e]) @ ((g / (1.0 + np.exp(-g))) * u)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("norm_topk", [0, 1])
def test_moe_with_all_experts_selected_is_the_dense_mixture(dtype, norm_topk):
    E = 4
    o, cfg, w = _tiny_oracle(E, E, dtype=dtype, norm_topk=norm_topk)
    lw = w["layers"][0]
    h = rng.standard_normal(cfg.hidden)
    idx, wt = oracle.router(lw["w_router"], h, E, norm_topk)
    logits = _w64(lw["w_router"]) @ h
    p = np.exp(logits - logits.max())
    p /= p.sum()
    dense = sum(p[e] * _ffn_dense(lw, e, h) for e in range(E))
    assert np.allclose(oracle.moe_ffn(o, 0, h, idx, wt), dense, atol=1e-12)


def test_single_expert_moe_is_a_plain_swiglu_ffn():
    o, cfg, w = _tiny_oracle(1, 1)
    h = rng.standard_normal(cfg.hidden)
    idx, wt = oracle.router(w["layers"][0]["w_router"], h, 1, 1)
    assert list(idx) == [0] and wt[0] == 1.0
    assert np.allclose(oracle.moe_ffn(o, 0, h, idx, wt), _ffn_dense(w["layers"][0], 0, h), atol=1e-12)


def test_moe_uses_the_selected_experts_and_their_weights():
    o, cfg, w = _tiny_oracle(6, 2)
    h = rng.standard_normal(cfg.hidden)
    idx = np.array([5, 2], dtype=np.int32)
    wt = np.array([0.25, 0.75])
    want = 0.25 * _ffn_dense(w["layers"][0], 5, h) + 0.75 * _ffn_dense(w["layers"][0], 2, h)
    assert np.allclose(oracle.moe_ffn(o, 0, h, idx, wt), want, atol=1e-12)


# ---------------------------------------------------------------- permutation
def test_permutation_is_a_stable_counting_sort():
    E = 7
    for n in (0, 1, 5, 64, 257):
        ex = rng.integers(0, E, size=n).astype(np.int32)
        if n > 3:
            ex[ex == 3] = 2                       # an expert with no rows
        count, offset, perm = oracle.permutation(ex, E)
        assert offset[0] == 0 and offset[E] == n
        assert sorted(perm.tolist()) == list(range(n))
        for e in range(E):
            seg = perm[offset[e]:offset[e + 1]]
            assert count[e] == len(seg) == int((ex == e).sum())
            assert np.all(ex[seg] == e)
            assert np.all(np.diff(seg) > 0)
        assert np.array_equal(perm, np.argsort(ex, kind="stable"))


# ---------------------------------------------------------------- confidence
def test_confidence_bounds_ties_and_closed_forms():
    V = 50
    conf, am = oracle.confidence(np.zeros(V))
    assert conf == 1.0 / V and am == 0                      # all equal: 1/V, lowest id
    z = np.zeros(V)
    z[7] = z[31] = 2.0
    conf, am = oracle.confidence(z)
    assert am == 7
    assert abs(conf - np.e ** 2 / (2 * np.e ** 2 + (V - 2))) < 1e-15
    z = rng.standard_normal(V) * 4
    conf, am = oracle.confidence(z)
    p = np.exp(z) / np.exp(z).sum()
    assert am == int(np.argmax(p)) and abs(conf - p.max()) < 1e-14
    assert 1.0 / V <= conf <= 1.0
    z[11] = 1e4                                               # no overflow, conf -> 1
    conf, am = oracle.confidence(z)
    assert am == 11 and conf == 1.0


def test_confidence_matches_streaming_merge_in_any_tile_order():
    """A tile-by-tile (max, sum-exp) merge reaches the two-pass result: the form the HIP path relies on."""
    V = 1000
    z = rng.standard_normal(V) * 3
    conf, am = oracle.confidence(z)
    for order in (range(0, V, 64), reversed(range(0, V, 64))):
        m, s, best = -np.inf, 0.0, -1
        for a in order:
            t = z[a:a + 64]
            tm = t.max()
            ti = a + int(np.argmax(t))
            if tm > m or (tm == m and ti < best):
                s = s * np.exp(m - tm) + np.exp(t - tm).sum() if np.isfinite(m) else np.exp(t - tm).sum()
                m, best = tm, ti
            else:
                s += np.exp(t - m).sum()
        assert best == am and abs(1.0 / s - conf) < 1e-12


# ---------------------------------------------------------------- commit
def _commit_brute(conf, am, mask, tokens, tau, fixed_k):
    S = len(conf)
    masked = [i for i in range(S) if (mask >> i) & 1]
    if fixed_k > 0:
        sel = sorted(masked, key=lambda i: (-conf[i], i))[:fixed_k]
    else:
        sel = [i for i in masked if conf[i] >= tau]
        if not sel and masked:
            sel = [min(masked, key=lambda i: (-conf[i], i))]
    tok = list(tokens)
    for i in sel:
        tok[i] = am[i]
        mask &= ~(1 << i)
    return len(sel), mask, tok


def test_commit_brute_force_all_masks():
    S = 6
    for trial in range(6):
        conf = np.round(rng.random(S), 1 if trial % 2 else 3)      # coarse values: ties and conf == tau occur
        am = rng.integers(0, 100, size=S).astype(np.int32)
        tokens = rng.integers(100, 200, size=S).astype(np.int32)
        for mask in range(1 << S):
            for tau, fk in ((0.5, 0), (0.9, 0), (2.0, 0), (0.0, 0), (0.5, 1), (0.5, 2), (0.5, 8)):
                n, m2, t2 = oracle.commit(conf, am, mask, tokens, tau, fk)
                bn, bm, bt = _commit_brute(conf, am, mask, tokens, tau, fk)
                assert (n, m2, list(t2)) == (bn, bm, bt)
                assert m2 & ~mask == 0 and (n >= 1) == (mask != 0)
                assert bin(mask).count("1") - bin(m2).count("1") == n


def test_commit_threshold_is_at_or_above():
    conf = np.array([0.5, 0.25, 0.75])
    am = np.array([1, 2, 3], dtype=np.int32)
    n, m, tok = oracle.commit(conf, am, 0b111, [9, 9, 9], 0.5, 0)
    assert n == 2 and m == 0b010 and list(tok) == [1, 9, 3]


def test_commit_above_every_confidence_goes_in_descending_confidence_order():
    S = 9
    conf = rng.random(S)
    am = np.arange(S, dtype=np.int32) + 50
    mask, tokens, order = (1 << S) - 1, np.full(S, -1, dtype=np.int32), []
    while mask:
        n, m2, tokens = oracle.commit(conf, am, mask, tokens, 1.0, 0)
        assert n == 1
        order.append((mask ^ m2).bit_length() - 1)
        mask = m2
    assert order == list(np.argsort(-conf))
    assert np.array_equal(tokens, am)


def test_commit_fixed_k_empties_a_block_in_ceil_s_over_k_steps():
    S, k = 64, 8
    conf = rng.random(S)
    am = np.arange(S, dtype=np.int32)
    mask, tokens, steps = (1 << S) - 1, np.full(S, -1, dtype=np.int32), 0
    while mask:
        n, mask, tokens = oracle.commit(conf, am, mask, tokens, 0.9, k)
        assert n == k
        steps += 1
    assert steps == S // k and np.array_equal(tokens, am)


def test_commit_uses_all_64_bits():
    conf = np.zeros(64)
    conf[63] = 0.99
    n, m, tok = oracle.commit(conf, np.full(64, 7, dtype=np.int32), 1 << 63, np.zeros(64, dtype=np.int32), 0.9, 0)
    assert n == 1 and m == 0 and tok[63] == 7
    for trial in itertools.islice(itertools.count(), 3):
        mask = int(rng.integers(0, 1 << 62)) | (1 << 63)
        c = rng.random(64)
        assert oracle.commit(c, np.zeros(64, dtype=np.int32), mask, np.zeros(64, dtype=np.int32), 0.5, 0)[:2] == \
            _commit_brute(c, np.zeros(64, dtype=np.int32), mask, [0] * 64, 0.5, 0)[:2]
