"""Pins of the oracle's vicinity-refresh step (Section 2, KV-cache management: K and V are recomputed for the
block's tokens and their immediate neighbours): the plain step as the special case without neighbours, an
independent torch-CPU library assembly of the same forward, and the fixed point that a consistent cache is."""
import numpy as np
import pytest
import torch

import dinfer_inputs as di
import oracle
from test_oracle_step import torch_forward


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


def test_no_neighbours_is_the_plain_step(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    P = int(inp.prefix_len[0])
    k1, v1, k2, v2 = kc.copy(), vc.copy(), kc.copy(), vc.copy()
    a = o.step(inp.block_tokens[0], int(inp.mask_bits[0]), P, k1, v1, 0.05, want_logits=True)
    b = o.step_vicinity(inp.block_tokens[0], np.zeros(0, np.int32), int(inp.mask_bits[0]), P, k2, v2, 0.05,
                        want_logits=True)
    assert np.array_equal(a["logits"], b["logits"]) and np.array_equal(a["tokens"], b["tokens"])
    assert a["mask"] == b["mask"] and np.array_equal(k1, k2) and np.array_equal(v1, v2)


@pytest.mark.parametrize("look_back", [1, 16, 64])
def test_library_assembly_reproduces_the_vicinity_step(tiny, look_back):
    """torch CPU ops over the longer token run [P-look_back, P+S), with only the keys before it taken from the
    cache, give the same logits for the block and the same rewritten K,V rows."""
    wl, cfg, w, inp, o, kc, vc = tiny
    P, S = int(inp.prefix_len[0]), wl.block_len
    vic = inp.prefix_tokens[0][P - look_back:P]
    k2, v2 = kc.copy(), vc.copy()
    r = o.step_vicinity(inp.block_tokens[0], vic, int(inp.mask_bits[0]), P, k2, v2, wl.threshold, want_logits=True)
    before_k = torch.from_numpy(kc[:, :P - look_back].copy())
    before_v = torch.from_numpy(vc[:, :P - look_back].copy())
    tokens = np.concatenate([vic, inp.block_tokens[0]])
    _, logits, nk, nv = torch_forward(cfg, w, tokens, before_k, before_v)
    assert np.allclose(r["logits"], logits.numpy()[look_back:], atol=1e-9)
    assert np.allclose(k2[:, P - look_back:P + S], nk.numpy(), atol=1e-10)
    assert np.allclose(v2[:, P - look_back:P + S], nv.numpy(), atol=1e-10)
    # rows before the neighbourhood and after the block are not touched
    assert np.array_equal(k2[:, :P - look_back], kc[:, :P - look_back])
    assert np.array_equal(v2[:, P + S:], vc[:, P + S:])
    p = torch.softmax(logits[look_back:], -1)
    assert np.allclose(r["conf"], p.max(-1).values.numpy(), atol=1e-12)
    assert np.array_equal(r["argmax"], p.argmax(-1).numpy())
    # the neighbours' rows did change: the prompt-only prefill had not seen the block
    if look_back > 1:
        assert np.abs(k2[1, P - look_back:P] - kc[1, P - look_back:P]).max() > 1e-6


def test_consistent_cache_is_a_fixed_point(tiny):
    """If the cache comes from one bidirectional forward over prefix + block with the very same ids, recomputing
    the neighbours and the block reproduces it: nothing is stale."""
    wl, cfg, w, inp, o, _, _ = tiny
    P, S = int(inp.prefix_len[0]), 8
    ids = np.concatenate([inp.prefix_tokens[0], np.arange(100, 100 + S, dtype=np.int32)])
    kc, vc = o.new_cache(128)
    o.forward(ids, 0, kc, vc)
    k2, v2 = kc.copy(), vc.copy()
    r = o.step_vicinity(ids[P:], ids[P - 16:P], 0, P, k2, v2, 0.5)
    assert r["n_committed"] == 0 and np.array_equal(r["tokens"], ids[P:])
    assert np.allclose(k2, kc, atol=1e-11) and np.allclose(v2, vc, atol=1e-11)


def test_neighbourhood_must_lie_inside_the_prefix(tiny):
    wl, cfg, w, inp, o, kc, vc = tiny
    with pytest.raises(ValueError):
        o.step_vicinity(inp.block_tokens[0], np.zeros(70, np.int32), int(inp.mask_bits[0]), 64, kc.copy(), vc.copy(),
                        0.9)
