"""Pins of the oracle's whole step: a torch-CPU library assembly of the same network, and the invariants
Algorithm 1 and the decoding rule imply (progress, monotone mask, frozen prefix, greedy limit)."""
import numpy as np
import pytest
import torch

import dinfer_inputs as di
import oracle


def _w(a):
    a = di.bf16_to_f32(a) if a.dtype == np.uint16 else a
    return torch.from_numpy(a.astype(np.float64))


def torch_forward(cfg, w, tokens, prefix_k, prefix_v):
    """The same pre-norm MoE transformer block stack from torch CPU library ops (matmul, softmax, topk,
    scaled_dot_product_attention without a mask, complex multiplication for the rotary embedding).
    prefix_k / prefix_v: [L][P][nh*hd] float64 tensors (already rotated keys).  Returns (hidden, logits, k, v)."""
    F = torch.nn.functional
    nh, hd, H = cfg.n_heads, cfg.head_dim, cfg.hidden
    T, P = len(tokens), prefix_k.shape[1]
    x = _w(w["emb"])[torch.as_tensor(np.asarray(tokens, dtype=np.int64))]
    pos = torch.arange(P, P + T, dtype=torch.float64)
    inv = cfg.rope_theta ** (-torch.arange(0, hd // 2, dtype=torch.float64) * 2.0 / hd)
    rot = torch.polar(torch.ones(T, hd // 2, dtype=torch.float64), pos[:, None] * inv[None, :])  # e^{i pos w_j}

    def rms(v, g):
        return v * torch.rsqrt((v * v).mean(-1, keepdim=True) + cfg.rms_eps) * torch.from_numpy(g.astype(np.float64))

    def rope(v):  # v [T][nh][hd]; pair (j, j+hd/2) is one complex number
        z = torch.complex(v[..., : hd // 2], v[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    ks, vs = [], []
    for l, lw in enumerate(w["layers"]):
        h = rms(x, lw["attn_gain"])
        q = rope((h @ _w(lw["wq"]).T).view(T, nh, hd))
        k = rope((h @ _w(lw["wk"]).T).view(T, nh, hd)).reshape(T, nh * hd)
        v = h @ _w(lw["wv"]).T
        kall = torch.cat([prefix_k[l], k]).view(P + T, nh, hd)
        vall = torch.cat([prefix_v[l], v]).view(P + T, nh, hd)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), kall.transpose(0, 1), vall.transpose(0, 1))
        x = x + a.transpose(0, 1).reshape(T, nh * hd) @ _w(lw["wo"]).T
        h = rms(x, lw["ffn_gain"])
        p = torch.softmax(h @ _w(lw["w_router"]).T, dim=-1)
        tw, ti = torch.topk(p, cfg.top_k, dim=-1)
        if cfg.norm_topk:
            tw = tw / tw.sum(-1, keepdim=True)
        wg, wu, wd = _w(lw["w_gate"]), _w(lw["w_up"]), _w(lw["w_down"])
        out = torch.zeros_like(x)
        for t in range(T):
            for j in range(cfg.top_k):
                e = int(ti[t, j])
                y = F.silu(wg[e] @ h[t]) * (wu[e] @ h[t])
                out[t] += tw[t, j] * (wd[e] @ y)
        x = x + out
        ks.append(k)
        vs.append(v)
    logits = cfg.logit_scale * (rms(x, w["final_gain"]) @ _w(w["lm_head"]).T)
    return x, logits, torch.stack(ks), torch.stack(vs)


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


def test_library_assembly_reproduces_prefill_and_step(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    P = int(inp.prefix_len[0])
    empty = torch.zeros(cfg.n_layers, 0, cfg.qkv_dim, dtype=torch.float64)
    hid, _, pk, pv = torch_forward(cfg, w, inp.prefix_tokens[0], empty, empty)
    assert np.allclose(kc[:, :P], pk.numpy(), atol=1e-10)
    assert np.allclose(vc[:, :P], pv.numpy(), atol=1e-10)
    k2, v2 = kc.copy(), vc.copy()
    tr = oracle.Trace(cfg, wl.block_len)
    r = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), P, k2, v2, wl.threshold, want_logits=True, trace=tr)
    hid, logits, bk, bv = torch_forward(cfg, w, inp.block_tokens[0], pk, pv)
    assert np.allclose(r["logits"], logits.numpy(), atol=1e-9)
    assert np.allclose(tr.resid[-1], hid.numpy(), atol=1e-10)
    assert np.allclose(k2[:, P:P + wl.block_len], bk.numpy(), atol=1e-10)
    assert np.allclose(v2[:, P:P + wl.block_len], bv.numpy(), atol=1e-10)
    p = torch.softmax(logits, -1)
    assert np.allclose(r["conf"], p.max(-1).values.numpy(), atol=1e-12)
    assert np.array_equal(r["argmax"], p.argmax(-1).numpy())


def test_library_assembly_bf16_weights():
    cfg = di.ModelConfig("t", n_layers=2, hidden=64, n_heads=2, head_dim=16, n_experts=4, top_k=2, moe_inter=48,
                         vocab=300, dtype="bf16", init_std=0.1)
    w = di.make_weights(cfg, 11)
    o = oracle.Oracle(cfg, w)
    kc, vc = o.new_cache(32)
    prompt = np.arange(10, 19, dtype=np.int32)
    o.forward(prompt, 0, kc, vc)
    empty = torch.zeros(cfg.n_layers, 0, cfg.qkv_dim, dtype=torch.float64)
    _, _, pk, pv = torch_forward(cfg, w, prompt, empty, empty)
    block = np.full(5, cfg.mask_id, dtype=np.int32)
    r = o.step(block, 0b11111, 9, kc, vc, 0.5, want_logits=True)
    _, logits, _, _ = torch_forward(cfg, w, block, pk, pv)
    assert np.allclose(r["logits"], logits.numpy(), atol=1e-9)


def test_step_leaves_prefix_kv_and_unmasked_tokens_alone(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    P = int(inp.prefix_len[0])
    k2, v2 = kc.copy(), vc.copy()
    tokens = inp.block_tokens[0].copy()
    tokens[[3, 9]] = [17, 99]                      # already decided positions
    mask = int(inp.mask_bits[0]) & ~((1 << 3) | (1 << 9))
    probe = o.step(tokens, mask, P, kc.copy(), vc.copy(), 2.0)
    tau = float(np.median(probe["conf"]))                  # about half of the masked positions reach it
    r = o.step(tokens, mask, P, k2, v2, tau)
    assert r["n_committed"] > 1
    assert np.array_equal(k2[:, :P], kc[:, :P]) and np.array_equal(v2[:, :P], vc[:, :P])
    assert np.array_equal(k2[:, P + 32:], kc[:, P + 32:])
    assert r["tokens"][3] == 17 and r["tokens"][9] == 99
    assert r["mask"] & ~mask == 0
    committed = mask & ~r["mask"]
    assert bin(committed).count("1") == r["n_committed"] >= 1
    for i in range(32):
        if (committed >> i) & 1:
            assert r["tokens"][i] == r["argmax"][i] and r["conf"][i] >= tau
        elif (mask >> i) & 1:
            assert r["tokens"][i] == cfg.mask_id and r["conf"][i] < tau
    assert np.all(r["conf"] >= 1.0 / cfg.vocab) and np.all(r["conf"] <= 1.0)


def test_step_falls_back_to_the_single_most_confident_position(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    r = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9)
    assert r["conf"].max() < 0.9 and r["n_committed"] == 1
    i = int(np.argmax(r["conf"]))
    assert r["mask"] == int(inp.mask_bits[0]) & ~(1 << i) and r["tokens"][i] == r["argmax"][i]


def test_empty_mask_is_a_no_op(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    tok = np.arange(32, dtype=np.int32)
    r = o.step(tok, 0, 64, kc.copy(), vc.copy(), 0.1)
    assert r["n_committed"] == 0 and r["mask"] == 0 and np.array_equal(r["tokens"], tok)


def test_threshold_one_is_one_token_per_step_greedy(tiny):
    """threshold 1.0 (no confidence reaches it): the block is decoded one position per step, each step taking
    the most confident remaining position of the re-run model."""
    wl, cfg, w, inp, o, kc, vc = tiny
    k2, v2 = kc.copy(), vc.copy()
    g = o.generate_block(inp.block_tokens[0], int(inp.mask_bits[0]), 64, k2, v2, 1.0, max_steps=64)
    assert g["steps"] == 32 and g["mask"] == 0 and np.all(g["committed_per_step"] == 1)
    # replay by hand
    tok, mask = inp.block_tokens[0].copy(), int(inp.mask_bits[0])
    k3, v3 = kc.copy(), vc.copy()
    for _ in range(32):
        r = o.step(tok, mask, 64, k3, v3, 1.0)
        masked = [i for i in range(32) if (mask >> i) & 1]
        best = max(masked, key=lambda i: (r["conf"][i], -i))
        assert r["mask"] == mask & ~(1 << best)
        tok, mask = r["tokens"], r["mask"]
    assert np.array_equal(tok, g["tokens"])


def test_generate_block_progress_and_fixed_k(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    g = o.generate_block(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.14, max_steps=64)
    assert g["mask"] == 0 and 1 <= g["steps"] <= 32
    assert g["committed_per_step"].sum() == 32 and np.all(g["committed_per_step"] >= 1)
    assert np.all(g["tokens"] != cfg.mask_id) or cfg.mask_id in g["tokens"]   # any id may be predicted
    f = o.generate_block(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9, fixed_k=8)
    assert f["steps"] == 4 and np.all(f["committed_per_step"] == 8) and f["mask"] == 0


def test_refresh_makes_cache_equal_to_recomputation_from_tokens(tiny):
    """After a block is decoded and refreshed, its cached K,V are those of a forward over its final tokens,
    and a later block sees the same cache whether it was built blockwise or the block is recomputed."""
    wl, cfg, w, inp, o, kc, vc = tiny
    k2, v2 = kc.copy(), vc.copy()
    g = o.generate_block(inp.block_tokens[0], int(inp.mask_bits[0]), 64, k2, v2, 0.9, fixed_k=8)
    o.forward(g["tokens"], 64, k2, v2)                       # refresh
    k3, v3 = kc.copy(), vc.copy()
    o.forward(g["tokens"], 64, k3, v3)                       # straight from the final tokens
    assert np.array_equal(k2, k3) and np.array_equal(v2, v3)
    assert not np.array_equal(k2[:, 64:96], kc[:, 64:96])


def test_zero_lm_head_gives_uniform_confidence_and_id_zero(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    w0 = dict(w)
    w0["lm_head"] = np.zeros_like(w["lm_head"])
    o0 = oracle.Oracle(cfg, w0)
    r = o0.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9)
    assert np.all(r["conf"] == 1.0 / cfg.vocab) and np.all(r["argmax"] == 0)
    assert r["n_committed"] == 1 and r["mask"] == int(inp.mask_bits[0]) & ~1    # ties -> lowest position


def test_planted_lm_head_row_commits_every_position(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    tr = oracle.Trace(cfg, 32)
    o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9, trace=tr)
    w1 = dict(w)
    lm = w["lm_head"].copy()
    # a row aligned with the (identical up to position) normalised final hidden states' mean, with a big norm
    hn = tr.resid[-1] / np.sqrt((tr.resid[-1] ** 2).mean(-1, keepdims=True))
    lm[1234] = (hn.mean(0) * 2.0).astype(np.float32)
    w1["lm_head"] = lm
    r = oracle.Oracle(cfg, w1).step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9)
    assert np.all(r["argmax"] == 1234) and r["n_committed"] == 32 and r["mask"] == 0
    assert np.all(r["tokens"] == 1234)


def test_logit_scale_multiplies_logits(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    r8 = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9, want_logits=True)
    o1 = oracle.Oracle(di.configs.scaled(cfg, logit_scale=1.0), w)
    r1 = o1.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9, want_logits=True)
    assert np.allclose(r8["logits"], 8.0 * r1["logits"], rtol=1e-13)


def test_a_sequence_does_not_depend_on_cache_capacity_or_other_rows(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    big_k, big_v = o.new_cache(300)
    big_k[:, :64], big_v[:, :64] = kc[:, :64], vc[:, :64]
    big_k[:, 96:], big_v[:, 96:] = 7.0, -7.0                 # garbage beyond the block must not be read
    a = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, big_k, big_v, 0.15)
    b = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.15)
    assert np.array_equal(a["conf"], b["conf"]) and a["mask"] == b["mask"]


def test_forced_routing_equal_to_own_choice_changes_nothing_and_other_choice_is_used(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    free = oracle.Trace(cfg, 32)
    a = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9, want_logits=True, trace=free)
    same = oracle.Trace(cfg, 32, forced_idx=free.topk_idx)
    b = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9, want_logits=True, trace=same)
    assert np.array_equal(a["logits"], b["logits"])
    assert np.allclose(free.router_p.sum(-1), 1.0, atol=1e-12)
    other = free.topk_idx.copy()
    other[1, 5] = [(other[1, 5, 0] + 3) % cfg.n_experts, (other[1, 5, 0] + 4) % cfg.n_experts]
    tr = oracle.Trace(cfg, 32, forced_idx=other)
    c = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9, want_logits=True, trace=tr)
    assert not np.allclose(c["logits"][5], a["logits"][5]) and np.array_equal(tr.topk_idx[0], free.topk_idx[0])
    # forcing the oracle's own sets in another order leaves the mixture (a sum) unchanged up to rounding
    swapped = oracle.Trace(cfg, 32, forced_idx=free.topk_idx[:, :, ::-1])
    d = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(), 0.9, want_logits=True, trace=swapped)
    assert np.allclose(d["logits"], a["logits"], atol=1e-11)
