"""Shape presets of the benchmark configurations and the seeded tensors that fill them.

Weights are approximately N(0, 0.02^2) from the seed, norm gains are 1.0, token
ids are uniform on [0, vocab-1) (the last id is the mask id), as the
configurations of the block-denoising benchmark state.  Every weight matrix is
stored row-major as [out_features][in_features].
"""
from dataclasses import dataclass, field, replace
from typing import List

import numpy as np

from . import generator as g

BASE_SEED = 20251008
PAGE_SIZE = 16

# Global tensors, then per-layer tensors.  The position in these tuples is the stream id.
TENSOR_NAMES = ("emb", "lm_head", "final_gain")
LAYER_TENSOR_NAMES = (
    "attn_gain", "wq", "wk", "wv", "wo",
    "ffn_gain", "w_router", "w_gate", "w_up", "w_down",
)


@dataclass(frozen=True)
class ModelConfig:
    name: str
    n_layers: int
    hidden: int
    n_heads: int
    head_dim: int
    n_experts: int
    top_k: int
    moe_inter: int
    vocab: int
    dtype: str = "bf16"          # storage type of weights / activations / KV: "f32" or "bf16"
    norm_topk: int = 1
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    logit_scale: float = 1.0
    init_std: float = 0.02

    @property
    def mask_id(self):
        return self.vocab - 1

    @property
    def qkv_dim(self):
        return self.n_heads * self.head_dim


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelConfig
    n_seq: int
    block_len: int
    prefix_min: int
    prefix_max: int               # prefix length uniform on [prefix_min, prefix_max]
    precommit: bool = False       # Bernoulli(1/2) of the block positions already hold a token
    threshold: float = 0.9
    fixed_k: int = 0              # >0: commit exactly this many per step
    gen_len: int = 0              # >0: whole generation loop of this many tokens
    seed_index: int = 0


def model_preset(name):
    if name == "tiny":
        return ModelConfig("tiny", n_layers=2, hidden=256, n_heads=4, head_dim=64, n_experts=8, top_k=2,
                           moe_inter=512, vocab=4096, dtype="f32", logit_scale=8.0)
    if name == "llada_moe":
        return ModelConfig("llada_moe", n_layers=16, hidden=2048, n_heads=16, head_dim=128, n_experts=64,
                           top_k=8, moe_inter=1024, vocab=157184, dtype="bf16")
    raise KeyError(name)


def workload_preset(index):
    """index 1..5 = the five benchmark configurations, in their stated order."""
    tiny, big = model_preset("tiny"), model_preset("llada_moe")
    table = {
        1: Workload("C1-tiny-fp32", tiny, 1, 32, 64, 64, threshold=0.9, seed_index=1),
        2: Workload("C2-llada-moe-b1-p512-s32", big, 1, 32, 512, 512, threshold=0.9, seed_index=2),
        3: Workload("C3-llada-moe-b1-p4096-s64", big, 1, 64, 4096, 4096, precommit=True, threshold=0.8,
                    seed_index=3),
        4: Workload("C4-llada-moe-b16-paged", big, 16, 32, 256, 2048, threshold=0.9, seed_index=4),
        5: Workload("C5-llada-moe-generate-1024", big, 1, 64, 256, 256, fixed_k=8, gen_len=1024, seed_index=5),
    }
    return table[index]


def tensor_shape(cfg, name):
    H, D, E, I, V = cfg.hidden, cfg.qkv_dim, cfg.n_experts, cfg.moe_inter, cfg.vocab
    return {
        "emb": (V, H), "lm_head": (V, H), "final_gain": (H,),
        "attn_gain": (H,), "wq": (D, H), "wk": (D, H), "wv": (D, H), "wo": (H, D),
        "ffn_gain": (H,), "w_router": (E, H), "w_gate": (E, I, H), "w_up": (E, I, H), "w_down": (E, H, I),
    }[name]


def bf16_to_f32(a):
    """uint16 bfloat16 bit patterns -> float32 (exact)."""
    return (a.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16(a):
    """float32 -> uint16 bfloat16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def make_tensor(cfg, seed, name, layer=0):
    """One weight tensor by name.  Gains are ones (float32); matrices are N(0, init_std^2) in cfg.dtype."""
    shape = tensor_shape(cfg, name)
    if name.endswith("gain"):
        return np.ones(shape, dtype=np.float32)
    if name in TENSOR_NAMES:
        tid = TENSOR_NAMES.index(name)
    else:
        tid = 16 + LAYER_TENSOR_NAMES.index(name)
    return g.normal(g.stream_key(seed, tid, layer), shape, cfg.init_std, cfg.dtype)


def make_weights(cfg, seed):
    """All weights: {'emb','lm_head','final_gain', 'layers': [ {name: array} ]}."""
    w = {n: make_tensor(cfg, seed, n) for n in TENSOR_NAMES}
    w["layers"] = [{n: make_tensor(cfg, seed, n, layer) for n in LAYER_TENSOR_NAMES}
                   for layer in range(cfg.n_layers)]
    return w


@dataclass
class WorkloadInputs:
    prefix_tokens: List[np.ndarray]           # per sequence, int32[P_s]
    block_tokens: np.ndarray                  # int32[n_seq][S]; mask_id where still masked
    mask_bits: np.ndarray                     # uint64[n_seq]; bit i set = position i masked
    prefix_len: np.ndarray                    # int32[n_seq]
    page_table: np.ndarray                    # int32[n_seq][pt_stride]
    n_pages: int
    seed: int = 0
    extra: dict = field(default_factory=dict)


def _permutation(key, n):
    """Seeded Fisher-Yates shuffle of 0..n-1."""
    p = np.arange(n, dtype=np.int32)
    r = g.uniform_ids(key, n, 1 << 31)
    for i in range(n - 1, 0, -1):
        j = int(r[i]) % (i + 1)
        p[i], p[j] = p[j], p[i]
    return p


def make_workload_inputs(wl, seed=None, room=None):
    """Token ids, mask bitmap, prefix lengths and a scattered page table for a workload.

    `room` = positions each sequence's page list must hold beyond its prefix (default: one block,
    or the whole generation length for a generation-loop workload).
    """
    cfg = wl.model
    seed = BASE_SEED + wl.seed_index if seed is None else seed
    S, ns = wl.block_len, wl.n_seq
    if room is None:
        room = max(S, wl.gen_len)
    span = wl.prefix_max - wl.prefix_min + 1
    plen = wl.prefix_min + g.uniform_ids(g.stream_key(seed, 100), ns, span)
    prefix = [g.uniform_ids(g.stream_key(seed, 101, s), int(plen[s]), cfg.vocab - 1) for s in range(ns)]
    block = np.full((ns, S), cfg.mask_id, dtype=np.int32)
    bits = np.zeros(ns, dtype=np.uint64)
    for s in range(ns):
        if wl.precommit:
            keep = g.bernoulli_bits(g.stream_key(seed, 102, s), S)      # 1 = still masked
            ids = g.uniform_ids(g.stream_key(seed, 103, s), S, cfg.vocab - 1)
            block[s] = np.where(keep == 1, cfg.mask_id, ids)
        else:
            keep = np.ones(S, dtype=np.uint8)
        b = 0
        for i in range(S):
            if keep[i]:
                b |= 1 << i
        bits[s] = np.uint64(b)
    pages_per_seq = [(int(plen[s]) + room + PAGE_SIZE - 1) // PAGE_SIZE for s in range(ns)]
    n_pages = sum(pages_per_seq)
    perm = _permutation(g.stream_key(seed, 104), n_pages)
    stride = max(pages_per_seq)
    table = np.zeros((ns, stride), dtype=np.int32)
    at = 0
    for s in range(ns):
        table[s, :pages_per_seq[s]] = perm[at:at + pages_per_seq[s]]
        at += pages_per_seq[s]
    return WorkloadInputs(prefix, block, bits, plen.astype(np.int32), table, n_pages, seed)


KV_STD = 0.9   # std of a key / value element of the random-init LLaDA-MoE-shaped model (0.02 * sqrt(2048))


def synthetic_prefix_kv(cfg, seed, s, length, std=KV_STD, peaked=0):
    """Seeded stand-in for the cached prefix of sequence s: K,V rows ~ N(0, std^2), every value representable
    in bfloat16 (so that a bf16 and a float64 consumer see the same numbers).  Returns float32 [L][length][D].

    peaked > 0: in every layer that many seeded positions (peaked_positions) carry key rows 16 times and value rows
    4 times as large (powers of two: still exact in bfloat16).  Their attention scores dominate, so every query's
    softmax is sharply peaked on a few cached keys that sit in different key tiles, instead of nearly flat."""
    D = cfg.qkv_dim
    k = bf16_to_f32(g.normal(g.stream_key(seed, 200, s), (cfg.n_layers, length, D), std, "bf16"))
    v = bf16_to_f32(g.normal(g.stream_key(seed, 201, s), (cfg.n_layers, length, D), std, "bf16"))
    if peaked:
        for layer in range(cfg.n_layers):
            pos = peaked_positions(seed, s, layer, length, peaked)
            k[layer, pos] *= 16.0
            v[layer, pos] *= 4.0
    return k, v


def peaked_positions(seed, s, layer, length, n):
    """The n distinct cached positions of (sequence s, layer) that synthetic_prefix_kv(peaked=n) enlarges."""
    draws = g.uniform_ids(g.stream_key(seed, 202 + layer, s), 4 * n, length)
    pos = []
    for p in draws:
        if int(p) not in pos:
            pos.append(int(p))
        if len(pos) == n:
            break
    return np.array(sorted(pos), dtype=np.int64)


def scaled(cfg, **kw):
    """Copy of a model config with fields replaced (test variants)."""
    return replace(cfg, **kw)
