"""The seeded input generator: published SplitMix64 vectors, a pure-Python restatement, distribution."""
import numpy as np

import dinfer_inputs as di
from dinfer_inputs import generator as g

M64 = (1 << 64) - 1


def py_mix64(x):
    x = (x + 0x9E3779B97F4A7C15) & M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & M64
    return x ^ (x >> 31)


def test_mix64_published_vectors():
    # SplitMix64 seeded with 0: the first outputs of the reference generator (Vigna, splitmix64.c)
    golden = 0x9E3779B97F4A7C15
    assert g.mix64(0) == 0xE220A8397B1DCDAF
    assert g.mix64(golden) == 0x6E789E6AA1B965F4
    assert g.mix64(2 * golden) == 0x06C45D188009454F
    for x in (0, 1, 12345, M64, 0xDEADBEEF << 20):
        assert g.mix64(x) == py_mix64(x)


def test_normal_matches_python_restatement():
    key = g.stream_key(7, 3, 2, 1)
    a = g.normal(key, (64,), 0.02, "f32")
    scale = np.float32(0.02 / 209.02152998196777)
    for n in range(64):
        z = py_mix64((key + n) & M64)
        s = sum((z >> (8 * b)) & 0xFF for b in range(8))
        assert a[n] == np.float32(s - 1020) * scale


def test_normal_moments_and_bf16_rounding():
    key = g.stream_key(1, 2)
    a = g.normal(key, (1 << 20,), 0.02, "f32")
    assert abs(a.mean()) < 1e-4
    assert abs(a.std() - 0.02) < 2e-4
    b = g.normal(key, (1 << 20,), 0.02, "bf16")
    assert b.dtype == np.uint16
    wide = di.bf16_to_f32(b)
    assert np.all(np.abs(wide - a) <= np.abs(a) * 2.0 ** -8)
    assert np.array_equal(di.f32_to_bf16(a), b)
    # offsets address the same stream
    assert np.array_equal(g.normal(key, (100,), 0.02, "f32", first=1000), a[1000:1100])


def test_streams_differ():
    a = g.normal(g.stream_key(1, 2, 0), (256,), 0.02, "f32")
    b = g.normal(g.stream_key(1, 2, 1), (256,), 0.02, "f32")
    assert not np.array_equal(a, b)


def test_workload_presets():
    for i in range(1, 6):
        wl = di.workload_preset(i)
        inp = di.make_workload_inputs(wl)
        cfg = wl.model
        assert inp.block_tokens.shape == (wl.n_seq, wl.block_len)
        for s in range(wl.n_seq):
            assert wl.prefix_min <= inp.prefix_len[s] <= wl.prefix_max
            assert inp.prefix_tokens[s].max() < cfg.mask_id and inp.prefix_tokens[s].min() >= 0
            bits = int(inp.mask_bits[s])
            for p in range(wl.block_len):
                assert ((bits >> p) & 1) == (inp.block_tokens[s, p] == cfg.mask_id)
        used = []
        for s in range(wl.n_seq):
            need = (int(inp.prefix_len[s]) + max(wl.block_len, wl.gen_len) + 15) // 16
            used += list(inp.page_table[s, :need])
        assert len(set(used)) == len(used) and max(used) < inp.n_pages
    c3 = di.make_workload_inputs(di.workload_preset(3))
    frac = bin(int(c3.mask_bits[0])).count("1") / 64
    assert 0.25 < frac < 0.75
    c4 = di.make_workload_inputs(di.workload_preset(4))
    assert len(set(c4.prefix_len.tolist())) > 8


def test_tensor_shapes_and_gains():
    cfg = di.model_preset("tiny")
    w = di.make_weights(cfg, 5)
    assert w["emb"].shape == (4096, 256) and w["emb"].dtype == np.float32
    assert np.all(w["final_gain"] == 1.0)
    l0 = w["layers"][0]
    assert l0["w_gate"].shape == (8, 512, 256) and l0["w_down"].shape == (8, 256, 512)
    assert l0["wo"].shape == (256, 256) and l0["w_router"].shape == (8, 256)
    assert not np.array_equal(w["layers"][0]["wq"], w["layers"][1]["wq"])
