"""ctypes front end of the CPU oracle (oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; the HIP library and its Python binding never do.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, "oracle.c"), os.path.join(_HERE, "oracle.h")]
_LIB = os.path.join(_HERE, "liboracle.so")

c_i32, c_f64, c_vp = ctypes.c_int32, ctypes.c_double, ctypes.c_void_p


def build(force=False):
    """Compile oracle.c with gcc: -O2, OpenMP, no fast-math."""
    newest = max(os.path.getmtime(s) for s in _SRC)
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-std=c11", "-O2", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC",
                               "-o", tmp, _SRC[0], "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class CConfig(ctypes.Structure):
    _fields_ = [(n, c_i32) for n in ("n_layers", "hidden", "n_heads", "head_dim", "n_experts", "top_k",
                                     "moe_inter", "vocab", "wdtype", "norm_topk")] + \
               [(n, c_f64) for n in ("rms_eps", "rope_theta", "logit_scale")]


class CLayer(ctypes.Structure):
    _fields_ = [(n, c_vp) for n in ("attn_gain", "wq", "wk", "wv", "wo", "ffn_gain", "w_router", "w_gate",
                                    "w_up", "w_down")]


class CWeights(ctypes.Structure):
    _fields_ = [("emb", c_vp), ("lm_head", c_vp), ("final_gain", c_vp), ("layers", ctypes.POINTER(CLayer))]


class CTrace(ctypes.Structure):
    _fields_ = [(n, c_vp) for n in ("topk_idx", "topk_w", "resid", "attn_out", "router_p", "forced_idx")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        P = ctypes.POINTER
        L.oracle_rmsnorm.argtypes = [c_vp, c_vp, c_i32, c_f64, c_vp]
        L.oracle_rope.argtypes = [c_vp, c_i32, c_i32, c_f64]
        L.oracle_linear.argtypes = [c_i32, c_vp, c_i32, c_i32, c_vp, c_i32, c_vp]
        L.oracle_attention.argtypes = [c_vp, c_i32, c_vp, c_vp, c_i32, c_i32, c_i32, c_vp]
        L.oracle_router.argtypes = [c_i32, c_vp, c_i32, c_i32, c_vp, c_i32, c_i32, c_vp, c_vp]
        L.oracle_moe_ffn.argtypes = [P(CConfig), P(CLayer), c_vp, c_vp, c_vp, c_vp]
        L.oracle_permutation.argtypes = [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp]
        L.oracle_confidence.argtypes = [c_vp, c_i32, c_vp, c_vp]
        L.oracle_commit.argtypes = [c_vp, c_vp, c_i32, c_vp, c_vp, c_f64, c_i32]
        L.oracle_commit.restype = c_i32
        L.oracle_forward.argtypes = [P(CConfig), P(CWeights), c_i32, c_vp, c_i32, c_vp, c_vp, c_i32, c_vp,
                                     P(CTrace)]
        L.oracle_forward.restype = c_i32
        L.oracle_logits.argtypes = [P(CConfig), P(CWeights), c_vp, c_i32, c_vp]
        L.oracle_step.argtypes = [P(CConfig), P(CWeights), c_i32, c_vp, c_vp, c_i32, c_vp, c_vp, c_i32, c_f64,
                                  c_i32, c_vp, c_vp, c_vp, P(CTrace)]
        L.oracle_step.restype = c_i32
        L.oracle_expected_embedding.argtypes = [P(CConfig), P(CWeights), c_vp, c_vp]
        L.oracle_expected_embedding.restype = None
        L.oracle_forward_embedded.argtypes = [P(CConfig), P(CWeights), c_i32, c_vp, c_vp, c_i32, c_vp, c_vp, c_i32, c_vp,
                                              P(CTrace)]
        L.oracle_forward_embedded.restype = c_i32
        L.oracle_step_smooth.argtypes = [P(CConfig), P(CWeights), c_i32, c_vp, c_vp, c_i32, c_vp, c_vp, c_i32, c_f64,
                                         c_i32, c_f64, c_vp, c_vp, c_vp, c_vp, P(CTrace)]
        L.oracle_step_smooth.restype = c_i32
        L.oracle_credit_position.argtypes = [c_vp, c_i32, c_vp, c_f64, c_f64, c_f64, c_vp, c_vp, c_vp]
        L.oracle_credit_position.restype = None
        L.oracle_step_credit.argtypes = [P(CConfig), P(CWeights), c_i32, c_vp, c_vp, c_i32, c_vp, c_vp, c_i32, c_f64,
                                         c_i32, c_vp, c_f64, c_f64, c_f64, c_vp, c_vp, c_vp, P(CTrace)]
        L.oracle_step_credit.restype = c_i32
        L.oracle_step_vicinity.argtypes = [P(CConfig), P(CWeights), c_i32, c_i32, c_vp, c_vp, c_vp, c_i32, c_vp, c_vp,
                                           c_i32, c_f64, c_i32, c_vp, c_vp, c_vp, P(CTrace)]
        L.oracle_step_vicinity.restype = c_i32
        L.oracle_generate_block.argtypes = [P(CConfig), P(CWeights), c_i32, c_vp, c_vp, c_i32, c_vp, c_vp,
                                            c_i32, c_f64, c_i32, c_i32, c_vp]
        L.oracle_generate_block.restype = c_i32
        L.oracle_commit_hier.argtypes = [c_vp, c_vp, c_i32, c_vp, c_vp, c_f64, c_f64]
        L.oracle_commit_hier.restype = c_i32
        L.oracle_step_hier.argtypes = [P(CConfig), P(CWeights), c_i32, c_vp, c_vp, c_i32, c_vp, c_vp, c_i32, c_f64,
                                       c_f64, c_vp, c_vp, c_vp, P(CTrace)]
        L.oracle_step_hier.restype = c_i32
        L.oracle_generate.argtypes = [P(CConfig), P(CWeights), c_i32, c_i32, c_i32, c_vp, c_vp, c_i32, c_f64, c_i32,
                                      c_i32, c_i32, c_vp, c_vp]
        L.oracle_generate.restype = c_i32
        L.oracle_num_threads.restype = c_i32
        for f in (L.oracle_rmsnorm, L.oracle_rope, L.oracle_linear, L.oracle_attention, L.oracle_router,
                  L.oracle_moe_ffn, L.oracle_permutation, L.oracle_confidence, L.oracle_logits):
            f.restype = None
        _lib = L
    return _lib


def _wdtype(a):
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError("weights must be float32 or uint16 (bfloat16 bit patterns), got %s" % a.dtype)


def _p(a):
    return a.ctypes.data if a is not None else None


def f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


class Trace:
    """Intermediates of one forward over n_tok tokens."""

    def __init__(self, cfg, n_tok, forced_idx=None):
        """forced_idx: optional int32 [L][n_tok][k] expert ids the forward must use (see oracle.h)."""
        L, H, D, K = cfg.n_layers, cfg.hidden, cfg.n_heads * cfg.head_dim, cfg.top_k
        self.topk_idx = np.zeros((L, n_tok, K), dtype=np.int32)
        self.topk_w = np.zeros((L, n_tok, K), dtype=np.float64)
        self.resid = np.zeros((L + 1, n_tok, H), dtype=np.float64)
        self.attn_out = np.zeros((L, n_tok, D), dtype=np.float64)
        self.router_p = np.zeros((L, n_tok, cfg.n_experts), dtype=np.float64)
        self.forced_idx = None
        if forced_idx is not None:
            self.forced_idx = np.ascontiguousarray(forced_idx, dtype=np.int32)
            assert self.forced_idx.shape == (L, n_tok, K)
            assert self.forced_idx.min() >= 0 and self.forced_idx.max() < cfg.n_experts
        self.c = CTrace(_p(self.topk_idx), _p(self.topk_w), _p(self.resid), _p(self.attn_out), _p(self.router_p),
                        _p(self.forced_idx))


class Oracle:
    """The oracle bound to one model configuration and one set of weights (numpy arrays, kept alive here).

    `cfg` needs the ModelConfig fields; `weights` is the dict layout of dinfer_inputs.make_weights.
    """

    def __init__(self, cfg, weights):
        self.cfg = cfg
        self.w = weights
        wd = _wdtype(weights["emb"])
        self.ccfg = CConfig(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.head_dim, cfg.n_experts, cfg.top_k,
                            cfg.moe_inter, cfg.vocab, wd, cfg.norm_topk, cfg.rms_eps, cfg.rope_theta,
                            cfg.logit_scale)
        self._layers = (CLayer * cfg.n_layers)()
        for i, lw in enumerate(weights["layers"]):
            for name, _ in CLayer._fields_:
                a = lw[name]
                if not name.endswith("gain") and _wdtype(a) != wd:
                    raise TypeError("mixed weight dtypes")
                if not a.flags["C_CONTIGUOUS"]:
                    raise ValueError("weights must be contiguous")
                setattr(self._layers[i], name, a.ctypes.data)
        self.cw = CWeights(_p(weights["emb"]), _p(weights["lm_head"]), _p(weights["final_gain"]), self._layers)
        self.D = cfg.n_heads * cfg.head_dim

    def new_cache(self, cap):
        shape = (self.cfg.n_layers, cap, self.D)
        return np.zeros(shape, dtype=np.float64), np.zeros(shape, dtype=np.float64)

    def forward(self, tokens, prefix_len, kc, vc, trace=None):
        """Forward of `tokens` at positions prefix_len.. ; writes their K,V rows; returns hidden [n][H].
        With the block's final ids this is the KV refresh of a decoded block; with prefix_len = 0 and the
        prompt as tokens it is the prefill."""
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        n = tokens.shape[0]
        hidden = np.zeros((n, self.cfg.hidden), dtype=np.float64)
        rc = lib().oracle_forward(self.ccfg, self.cw, n, _p(tokens), int(prefix_len), _p(kc), _p(vc),
                                  kc.shape[1], _p(hidden), trace.c if trace else None)
        if rc != 0:
            raise ValueError("oracle_forward failed: %d" % rc)
        return hidden

    def logits(self, hidden):
        hidden = f64(hidden)
        out = np.zeros((hidden.shape[0], self.cfg.vocab), dtype=np.float64)
        lib().oracle_logits(self.ccfg, self.cw, _p(hidden), hidden.shape[0], _p(out))
        return out

    def step(self, block_tokens, mask, prefix_len, kc, vc, threshold, fixed_k=0, want_logits=False, trace=None):
        """One denoising step.  Returns dict(tokens, mask, n_committed, conf, argmax[, logits])."""
        tok = np.array(block_tokens, dtype=np.int32)
        S = tok.shape[0]
        m = np.array([mask], dtype=np.uint64)
        conf = np.zeros(S, dtype=np.float64)
        am = np.zeros(S, dtype=np.int32)
        logits = np.zeros((S, self.cfg.vocab), dtype=np.float64) if want_logits else None
        n = lib().oracle_step(self.ccfg, self.cw, S, _p(tok), _p(m), int(prefix_len), _p(kc), _p(vc),
                              kc.shape[1], float(threshold), int(fixed_k), _p(conf), _p(am), _p(logits),
                              trace.c if trace else None)
        if n < 0:
            raise ValueError("oracle_step failed")
        r = dict(tokens=tok, mask=int(m[0]), n_committed=int(n), conf=conf, argmax=am)
        if want_logits:
            r["logits"] = logits
        return r

    def expected_embedding(self, logits):
        """softmax(logits) . W_emb for one position: float64 [H]."""
        logits = f64(logits)
        out = np.zeros(self.cfg.hidden)
        lib().oracle_expected_embedding(self.ccfg, self.cw, _p(logits), _p(out))
        return out

    def forward_embedded(self, tokens, emb_add, prefix_len, kc, vc, trace=None):
        """forward() with emb_add [n_tok][H] added to the token embeddings."""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        add = f64(emb_add)
        hidden = np.zeros((tok.shape[0], self.cfg.hidden))
        rc = lib().oracle_forward_embedded(self.ccfg, self.cw, tok.shape[0], _p(tok), _p(add), int(prefix_len), _p(kc),
                                           _p(vc), kc.shape[1], _p(hidden), trace.c if trace else None)
        if rc != 0:
            raise ValueError("oracle_forward_embedded failed (%d)" % rc)
        return hidden

    def step_smooth(self, block_tokens, mask, prefix_len, kc, vc, threshold, alpha, delta, fixed_k=0, want_logits=False,
                    trace=None):
        """One denoising step with iteration smoothing.  delta: float64 [S][H], in (previous step's expected
        embeddings) and out (this step's, rows of the positions masked at the start)."""
        tok = np.array(block_tokens, dtype=np.int32)
        S = tok.shape[0]
        assert delta.dtype == np.float64 and delta.shape == (S, self.cfg.hidden) and delta.flags.c_contiguous
        m = np.array([mask], dtype=np.uint64)
        conf = np.zeros(S, dtype=np.float64)
        am = np.zeros(S, dtype=np.int32)
        logits = np.zeros((S, self.cfg.vocab), dtype=np.float64) if want_logits else None
        n = lib().oracle_step_smooth(self.ccfg, self.cw, S, _p(tok), _p(m), int(prefix_len), _p(kc), _p(vc),
                                     kc.shape[1], float(threshold), int(fixed_k), float(alpha), _p(delta), _p(conf),
                                     _p(am), _p(logits), trace.c if trace else None)
        if n < 0:
            raise ValueError("oracle_step_smooth failed")
        r = dict(tokens=tok, mask=int(m[0]), n_committed=int(n), conf=conf, argmax=am)
        if want_logits:
            r["logits"] = logits
        return r

    def step_credit(self, block_tokens, mask, prefix_len, kc, vc, threshold, credit, alpha, beta, gamma, fixed_k=0,
                    want_logits=False, trace=None):
        """One denoising step with credit decoding.  credit: float64 [S][V], updated in place (rows of positions
        masked at the start of the step).  Returns the dict of step(); conf / argmax are those of the enhanced
        distribution, logits (if wanted) the fused logits of the masked rows."""
        tok = np.array(block_tokens, dtype=np.int32)
        S = tok.shape[0]
        assert credit.dtype == np.float64 and credit.shape == (S, self.cfg.vocab) and credit.flags.c_contiguous
        m = np.array([mask], dtype=np.uint64)
        conf = np.zeros(S, dtype=np.float64)
        am = np.zeros(S, dtype=np.int32)
        logits = np.zeros((S, self.cfg.vocab), dtype=np.float64) if want_logits else None
        n = lib().oracle_step_credit(self.ccfg, self.cw, S, _p(tok), _p(m), int(prefix_len), _p(kc), _p(vc),
                                     kc.shape[1], float(threshold), int(fixed_k), _p(credit), float(alpha),
                                     float(beta), float(gamma), _p(conf), _p(am), _p(logits),
                                     trace.c if trace else None)
        if n < 0:
            raise ValueError("oracle_step_credit failed")
        r = dict(tokens=tok, mask=int(m[0]), n_committed=int(n), conf=conf, argmax=am)
        if want_logits:
            r["logits"] = logits
        return r

    def step_vicinity(self, block_tokens, vicinity_tokens, mask, prefix_len, kc, vc, threshold, fixed_k=0,
                      want_logits=False, trace=None):
        """One denoising step that also recomputes K,V of the len(vicinity_tokens) cached positions before the
        block (vicinity KV-cache refresh).  Returns the same dict as step()."""
        tok = np.array(block_tokens, dtype=np.int32)
        vic = np.ascontiguousarray(vicinity_tokens, dtype=np.int32)
        S = tok.shape[0]
        m = np.array([mask], dtype=np.uint64)
        conf = np.zeros(S, dtype=np.float64)
        am = np.zeros(S, dtype=np.int32)
        logits = np.zeros((S, self.cfg.vocab), dtype=np.float64) if want_logits else None
        n = lib().oracle_step_vicinity(self.ccfg, self.cw, S, int(vic.shape[0]), _p(tok), _p(vic), _p(m),
                                       int(prefix_len), _p(kc), _p(vc), kc.shape[1], float(threshold), int(fixed_k),
                                       _p(conf), _p(am), _p(logits), trace.c if trace else None)
        if n < 0:
            raise ValueError("oracle_step_vicinity failed")
        r = dict(tokens=tok, mask=int(m[0]), n_committed=int(n), conf=conf, argmax=am)
        if want_logits:
            r["logits"] = logits
        return r

    def step_hier(self, block_tokens, mask, prefix_len, kc, vc, tau_high, tau_low, want_logits=False, trace=None):
        """One denoising step with the hierarchical decoder.  Returns what step() returns."""
        tok = np.array(block_tokens, dtype=np.int32)
        S = tok.shape[0]
        m = np.array([mask], dtype=np.uint64)
        conf = np.zeros(S, dtype=np.float64)
        am = np.zeros(S, dtype=np.int32)
        logits = np.zeros((S, self.cfg.vocab), dtype=np.float64) if want_logits else None
        n = lib().oracle_step_hier(self.ccfg, self.cw, S, _p(tok), _p(m), int(prefix_len), _p(kc), _p(vc), kc.shape[1],
                                   float(tau_high), float(tau_low), _p(conf), _p(am), _p(logits),
                                   trace.c if trace else None)
        if n < 0:
            raise ValueError("oracle_step_hier failed")
        r = dict(tokens=tok, mask=int(m[0]), n_committed=int(n), conf=conf, argmax=am)
        if want_logits:
            r["logits"] = logits
        return r

    def generate(self, block_len, n_blocks, prefix_len, kc, vc, threshold, fixed_k=0, eos_id=-1):
        """Outer loop over blocks with early termination.  Returns dict(tokens [n_blocks*block_len], blocks, steps)."""
        out = np.zeros(n_blocks * block_len, dtype=np.int32)
        steps = np.zeros(n_blocks, dtype=np.int32)
        done = lib().oracle_generate(self.ccfg, self.cw, int(block_len), int(n_blocks), int(prefix_len), _p(kc), _p(vc),
                                     kc.shape[1], float(threshold), int(fixed_k), int(self.cfg.mask_id), int(eos_id),
                                     _p(out), _p(steps))
        if done < 0:
            raise ValueError("oracle_generate failed")
        return dict(tokens=out, blocks=int(done), steps=steps[:done].copy())

    def generate_block(self, block_tokens, mask, prefix_len, kc, vc, threshold, fixed_k=0, max_steps=64):
        tok = np.array(block_tokens, dtype=np.int32)
        m = np.array([mask], dtype=np.uint64)
        per = np.zeros(max_steps, dtype=np.int32)
        steps = lib().oracle_generate_block(self.ccfg, self.cw, tok.shape[0], _p(tok), _p(m), int(prefix_len),
                                            _p(kc), _p(vc), kc.shape[1], float(threshold), int(fixed_k),
                                            int(max_steps), _p(per))
        if steps < 0:
            raise ValueError("oracle_generate_block failed")
        return dict(tokens=tok, mask=int(m[0]), steps=int(steps), committed_per_step=per[:steps].copy())


# ---- building blocks, for the pins ----

def credit_position(logits, credit, alpha, beta, gamma):
    """Credit decoding of one position; credit (float64 [V]) is updated in place.  Returns (conf, argmax, fused)."""
    logits = f64(logits)
    assert credit.dtype == np.float64 and credit.flags.c_contiguous
    conf = np.zeros(1)
    am = np.zeros(1, dtype=np.int32)
    fused = np.zeros_like(logits)
    lib().oracle_credit_position(_p(logits), logits.shape[0], _p(credit), float(alpha), float(beta), float(gamma),
                                 _p(conf), _p(am), _p(fused))
    return float(conf[0]), int(am[0]), fused


def rmsnorm(x, gain, eps):
    x = f64(x)
    gain = np.ascontiguousarray(gain, dtype=np.float32)
    out = np.zeros_like(x)
    lib().oracle_rmsnorm(_p(x), _p(gain), x.shape[0], float(eps), _p(out))
    return out


def rope(vec, pos, theta):
    v = f64(vec).copy()
    lib().oracle_rope(_p(v), v.shape[0], int(pos), float(theta))
    return v


def linear(W, x):
    W = np.ascontiguousarray(W)
    x = f64(x)
    out = np.zeros((x.shape[0], W.shape[0]), dtype=np.float64)
    lib().oracle_linear(_wdtype(W), _p(W), W.shape[0], W.shape[1], _p(x), x.shape[0], _p(out))
    return out


def attention(q, k, v, n_heads, head_dim):
    q, k, v = f64(q), f64(k), f64(v)
    out = np.zeros_like(q)
    lib().oracle_attention(_p(q), q.shape[0], _p(k), _p(v), k.shape[0], n_heads, head_dim, _p(out))
    return out


def router(w_router, h, top_k, norm_topk):
    w_router = np.ascontiguousarray(w_router)
    h = f64(h)
    idx = np.zeros(top_k, dtype=np.int32)
    wt = np.zeros(top_k, dtype=np.float64)
    lib().oracle_router(_wdtype(w_router), _p(w_router), w_router.shape[0], w_router.shape[1], _p(h), top_k,
                        int(norm_topk), _p(idx), _p(wt))
    return idx, wt


def moe_ffn(oracle, layer, h, idx, wt):
    h = f64(h)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    wt = f64(wt)
    out = np.zeros(oracle.cfg.hidden, dtype=np.float64)
    lib().oracle_moe_ffn(oracle.ccfg, ctypes.byref(oracle._layers[layer]), _p(h), _p(idx), _p(wt), _p(out))
    return out


def permutation(expert_of_pair, n_experts):
    e = np.ascontiguousarray(expert_of_pair, dtype=np.int32)
    count = np.zeros(n_experts, dtype=np.int32)
    offset = np.zeros(n_experts + 1, dtype=np.int32)
    perm = np.zeros(e.shape[0], dtype=np.int32)
    lib().oracle_permutation(_p(e), e.shape[0], n_experts, _p(count), _p(offset), _p(perm))
    return count, offset, perm


def confidence(logits_row):
    z = f64(logits_row)
    conf = ctypes.c_double()
    am = ctypes.c_int32()
    lib().oracle_confidence(_p(z), z.shape[0], ctypes.byref(conf), ctypes.byref(am))
    return conf.value, am.value


def commit(conf, argmax, mask, tokens, threshold, fixed_k=0):
    conf = f64(conf)
    am = np.ascontiguousarray(argmax, dtype=np.int32)
    tok = np.array(tokens, dtype=np.int32)
    m = np.array([mask], dtype=np.uint64)
    n = lib().oracle_commit(_p(conf), _p(am), conf.shape[0], _p(m), _p(tok), float(threshold), int(fixed_k))
    return int(n), int(m[0]), tok


def commit_hier(conf, argmax, mask, tokens, tau_high, tau_low):
    conf = f64(conf)
    am = np.ascontiguousarray(argmax, dtype=np.int32)
    tok = np.array(tokens, dtype=np.int32)
    m = np.array([mask], dtype=np.uint64)
    n = lib().oracle_commit_hier(_p(conf), _p(am), conf.shape[0], _p(m), _p(tok), float(tau_high), float(tau_low))
    return int(n), int(m[0]), tok


def num_threads():
    return int(lib().oracle_num_threads())
