"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, sizes buffers and
rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import dinfer_inputs as di

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2510_08666_amd", "libdinfer.so")


@pytest.fixture(scope="module")
def binding():
    if not os.path.exists(LIB):
        pytest.fail("libdinfer.so is not built: run `python -m paper_2510_08666_amd.build`")
    from paper_2510_08666_amd import binding as b
    return b


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dinfer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dinfer_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(binding):
    names = declared_functions()
    assert len(names) >= 14
    raw = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(raw, n), n
    assert sorted(binding.EXPORTS) == names


def test_buffer_sizes(binding):
    cfg = di.model_preset("llada_moe")
    cc = binding.make_config(cfg, 8192)
    wb = binding.lib.dinfer_weights_bytes(cc)
    params = 2 * cfg.vocab * cfg.hidden + cfg.n_layers * (
        4 * cfg.hidden * cfg.qkv_dim + cfg.n_experts * cfg.hidden + 3 * cfg.n_experts * cfg.moe_inter * cfg.hidden)
    # packed layouts add no padding at these shapes; on top comes the transposed copy of the embedding matrix that
    # iteration smoothing contracts over (vocabulary padded to a multiple of 8192)
    emb_t = 2 * cfg.hidden * (-(-cfg.vocab // 8192) * 8192)
    assert 2 * params + emb_t <= wb <= 2 * params + emb_t + (1 << 20)
    kb = binding.lib.dinfer_kv_bytes(cc, 100)
    assert kb == cfg.n_layers * 100 * 2 * cfg.qkv_dim * 16 * 2
    assert binding.lib.dinfer_workspace_bytes(cc, 16, 512) > 0
    assert binding.lib.dinfer_workspace_bytes(cc, 65, 512) == 0
    assert binding.lib.dinfer_workspace_bytes(cc, 1, 0) == 0


def test_bad_configs_are_rejected(binding):
    tiny = di.model_preset("tiny")
    for kw in (dict(head_dim=32), dict(hidden=100), dict(n_experts=65), dict(top_k=9), dict(top_k=0),
               dict(moe_inter=96), dict(vocab=1)):
        cc = binding.make_config(di.configs.scaled(tiny, **kw), 128)
        assert binding.lib.dinfer_weights_bytes(cc) == 0, kw
        assert binding.last_error() != ""
    cc = binding.make_config(tiny, 128)
    cc.page_size = 32
    assert binding.lib.dinfer_kv_bytes(cc, 4) == 0
    cc = binding.make_config(tiny, 128)
    cc.mask_id = tiny.vocab
    assert binding.lib.dinfer_weights_bytes(cc) == 0


def test_create_rejects_null_and_misaligned_buffers(binding):
    cc = binding.make_config(di.model_preset("tiny"), 128)
    h = ctypes.c_void_p()
    rc = binding.lib.dinfer_create(cc, None, 0, None, 1, None, 0, 1, 32, None, ctypes.byref(h))
    assert rc == -1 and not h.value
    rc = binding.lib.dinfer_create(cc, 0x1008, 1 << 40, 0x2000, 1, 0x3000, 1 << 40, 1, 32, None, ctypes.byref(h))
    assert rc == -1 and "aligned" in binding.last_error()
    rc = binding.lib.dinfer_create(cc, 0x1000, 16, 0x2000, 1, 0x3000, 16, 1, 32, None, ctypes.byref(h))
    assert rc == -3                                              # buffers too small: nothing is touched
    assert binding.lib.dinfer_step(None, 1, 32, None, None, None, None, 1, None, None, None, None, None) == -1
    assert binding.lib.dinfer_set_tensor(None, 0, 0, None, 0, None) == -1
