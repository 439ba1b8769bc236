"""ctypes binding of libdinfer.so: the same entry points as include/dinfer.h, argument marshalling only.

Every step of the path runs inside the HIP library; nothing here computes.  PyTorch is used only to own
device memory and to name the stream.  Importing this module without the built library raises.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DINFER_LIB") or os.path.join(_HERE, "libdinfer.so")   # DINFER_LIB: another build of it

c_i32, c_u64, c_f32, c_vp, c_sz = ctypes.c_int32, ctypes.c_uint64, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t

F32, BF16 = 0, 1
(T_EMB, T_LM_HEAD, T_FINAL_GAIN, T_ATTN_GAIN, T_WQ, T_WK, T_WV, T_WO, T_FFN_GAIN, T_ROUTER, T_GATE, T_UP,
 T_DOWN) = range(13)
TENSOR_IDS = {"emb": T_EMB, "lm_head": T_LM_HEAD, "final_gain": T_FINAL_GAIN, "attn_gain": T_ATTN_GAIN, "wq": T_WQ,
              "wk": T_WK, "wv": T_WV, "wo": T_WO, "ffn_gain": T_FFN_GAIN, "w_router": T_ROUTER, "w_gate": T_GATE,
              "w_up": T_UP, "w_down": T_DOWN}

EXPORTS = ["dinfer_weights_bytes", "dinfer_kv_bytes", "dinfer_workspace_bytes", "dinfer_create", "dinfer_destroy",
           "dinfer_last_error", "dinfer_set_tensor", "dinfer_prefill", "dinfer_step", "dinfer_step_vicinity", "dinfer_step_credit", "dinfer_step_smooth", "dinfer_step_smooth_static", "dinfer_smooth_scratch_bytes",
           "dinfer_refresh_block", "dinfer_commit", "dinfer_generate",
           "dinfer_generate_block", "dinfer_kv_write", "dinfer_kv_read", "dinfer_debug_logits", "dinfer_debug_get",
           "dinfer_profile_every", "dinfer_profile_start", "dinfer_profile_stop", "dinfer_stream_read", "dinfer_debug_trace",
           "dinfer_debug_single_slice", "dinfer_generate_block_smooth"]
(STAGE_QKV, STAGE_ATTENTION, STAGE_OPROJ, STAGE_EXPERT_GATE_UP, STAGE_EXPERT_DOWN, STAGE_LM_HEAD,
 STAGE_ROUTER) = range(7)


class Config(ctypes.Structure):
    _fields_ = [(n, c_i32) for n in ("n_layers", "hidden", "n_heads", "head_dim", "n_experts", "top_k", "moe_inter",
                                     "vocab", "dtype", "page_size", "mask_id", "norm_topk", "max_pos")] + \
               [(n, c_f32) for n in ("rms_eps", "rope_theta", "logit_scale")]


class Decode(ctypes.Structure):
    _fields_ = [("threshold", c_f32), ("fixed_k", c_i32), ("hierarchical", c_i32), ("lower_bound", c_f32),
                ("skip_decided", c_i32)]


def _decode(threshold, fixed_k):
    """A Decode passes through; otherwise threshold decoding (or fixed-k when fixed_k > 0)."""
    if isinstance(threshold, Decode):
        return threshold
    return Decode(float(threshold), int(fixed_k), 0, 0.0, 0)


def hierarchical(threshold, lower_bound):
    """Decoder settings of hierarchical decoding."""
    return Decode(float(threshold), 0, 1, float(lower_bound), 0)


class Credit(ctypes.Structure):
    _fields_ = [("alpha", c_f32), ("beta", c_f32), ("gamma", c_f32)]


class SmoothSchedule(ctypes.Structure):
    _fields_ = [("alpha_init", c_f32), ("alpha_growth", c_f32), ("alpha_preset", c_f32), ("threshold_start", c_f32),
                ("threshold_decay", c_f32)]


CREDIT_CAP = 64


def commit(d_conf, d_argmax, d_block_tokens, d_mask, decode, d_n_committed):
    """The decoder alone on given confidences and candidate ids ([n_seq][block_len] device tensors)."""
    n_seq, block_len = d_block_tokens.shape
    _check(lib.dinfer_commit(_ptr(d_conf), _ptr(d_argmax), n_seq, block_len, _ptr(d_block_tokens), _ptr(d_mask),
                             ctypes.byref(decode), _ptr(d_n_committed), _stream()))


class DinferError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("dinfer error %d: %s" % (code, msg))
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libdinfer.so is not built (run `python -m paper_2510_08666_amd.build`); "
                          "there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER
    L.dinfer_weights_bytes.restype = c_sz
    L.dinfer_weights_bytes.argtypes = [P(Config)]
    L.dinfer_kv_bytes.restype = c_sz
    L.dinfer_kv_bytes.argtypes = [P(Config), c_i32]
    L.dinfer_workspace_bytes.restype = c_sz
    L.dinfer_workspace_bytes.argtypes = [P(Config), c_i32, c_i32]
    L.dinfer_create.restype = c_i32
    L.dinfer_create.argtypes = [P(Config), c_vp, c_sz, c_vp, c_i32, c_vp, c_sz, c_i32, c_i32, c_vp, P(c_vp)]
    L.dinfer_destroy.restype = None
    L.dinfer_destroy.argtypes = [c_vp]
    L.dinfer_last_error.restype = ctypes.c_char_p
    L.dinfer_last_error.argtypes = []
    L.dinfer_set_tensor.restype = c_i32
    L.dinfer_set_tensor.argtypes = [c_vp, c_i32, c_i32, c_vp, c_sz, c_vp]
    L.dinfer_prefill.restype = c_i32
    L.dinfer_prefill.argtypes = [c_vp, c_i32, c_vp, c_vp, c_vp, c_i32, c_vp]
    L.dinfer_step.restype = c_i32
    L.dinfer_step.argtypes = [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_i32, P(Decode), c_vp, c_vp, c_vp, c_vp]
    L.dinfer_smooth_scratch_bytes.restype = c_sz
    L.dinfer_smooth_scratch_bytes.argtypes = [P(Config), c_i32]
    L.dinfer_step_smooth.restype = c_i32
    L.dinfer_step_smooth.argtypes = [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_i32, P(Decode), c_f32, c_vp, c_vp, c_sz,
                                     c_vp, c_vp, c_vp, c_vp]
    L.dinfer_generate_block_smooth.restype = c_i32
    L.dinfer_generate_block_smooth.argtypes = [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_i32, P(Decode),
                                               P(SmoothSchedule), c_vp, c_vp, c_sz, c_vp, c_vp, c_vp, c_i32, c_i32,
                                               P(c_i32), c_vp]
    L.dinfer_step_smooth_static.restype = c_i32
    L.dinfer_step_smooth_static.argtypes = [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_i32, P(Decode), c_f32, c_vp,
                                            c_vp, c_vp, c_vp, c_vp]
    L.dinfer_step_credit.restype = c_i32
    L.dinfer_step_credit.argtypes = [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_i32, P(Decode), P(Credit), c_vp, c_vp,
                                     c_vp, c_vp, c_vp, c_vp, c_vp]
    L.dinfer_step_vicinity.restype = c_i32
    L.dinfer_step_vicinity.argtypes = [c_vp, c_i32, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_vp, c_i32, P(Decode), c_vp,
                                       c_vp, c_vp, c_vp]
    L.dinfer_refresh_block.restype = c_i32
    L.dinfer_refresh_block.argtypes = [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_i32, c_vp]
    L.dinfer_generate_block.restype = c_i32
    L.dinfer_generate_block.argtypes = [c_vp, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_i32, P(Decode), c_vp, c_vp, c_vp,
                                        c_i32, c_i32, c_i32, P(c_i32), c_vp]
    L.dinfer_commit.restype = c_i32
    L.dinfer_commit.argtypes = [c_vp, c_vp, c_i32, c_i32, c_vp, c_vp, P(Decode), c_vp, c_vp]
    L.dinfer_generate.restype = c_i32
    L.dinfer_generate.argtypes = [c_vp, c_i32, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp, c_vp, c_i32, P(Decode), c_i32, c_i32,
                                  c_vp, c_vp, c_vp, c_vp, P(c_i32), c_vp]
    L.dinfer_kv_write.restype = c_i32
    L.dinfer_kv_write.argtypes = [c_vp, c_i32, c_vp, c_i32, c_i32, c_vp, c_vp, c_vp]
    L.dinfer_kv_read.restype = c_i32
    L.dinfer_kv_read.argtypes = [c_vp, c_i32, c_vp, c_i32, c_i32, c_vp, c_vp, c_vp]
    L.dinfer_debug_logits.restype = c_i32
    L.dinfer_debug_logits.argtypes = [c_vp, c_i32, c_vp, c_vp]
    L.dinfer_debug_single_slice.restype = c_i32
    L.dinfer_debug_single_slice.argtypes = [c_i32]
    L.dinfer_debug_get.restype = c_i32
    L.dinfer_debug_get.argtypes = [c_vp, c_i32, c_vp, c_sz, c_vp]
    L.dinfer_profile_every.restype = c_i32
    L.dinfer_profile_every.argtypes = [c_vp, c_i32]
    L.dinfer_profile_start.restype = c_i32
    L.dinfer_profile_start.argtypes = [c_vp, c_i32]
    L.dinfer_profile_stop.restype = c_i32
    L.dinfer_profile_stop.argtypes = [c_vp, P(c_i32), P(c_f32)]
    L.dinfer_debug_trace.restype = c_i32
    L.dinfer_debug_trace.argtypes = [c_i32, c_vp, c_sz]
    L.dinfer_stream_read.restype = c_i32
    L.dinfer_stream_read.argtypes = [c_vp, c_sz, c_vp, c_vp]
    return L


lib = _load()


def last_error():
    return lib.dinfer_last_error().decode()


def _check(rc):
    if rc != 0:
        raise DinferError(rc, last_error())


def make_config(cfg, max_pos):
    """dinfer_config from an object with the model fields (n_layers, hidden, ..., dtype 'f32'|'bf16')."""
    return Config(cfg.n_layers, cfg.hidden, cfg.n_heads, cfg.head_dim, cfg.n_experts, cfg.top_k, cfg.moe_inter,
                  cfg.vocab, BF16 if cfg.dtype == "bf16" else F32, 16, cfg.mask_id, cfg.norm_topk, int(max_pos),
                  cfg.rms_eps, cfg.rope_theta, cfg.logit_scale)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def debug_single_slice(on):
    """Test switch: while on, no contraction shares a task's sum among workgroups."""
    _check(lib.dinfer_debug_single_slice(1 if on else 0))


def debug_trace(unit, n_wgs):
    """Phase timestamps [n_wgs][8] (uint64, 10 ns ticks) of a library built with DINFER_TRACE=<kernel id>."""
    import numpy as np
    out = np.zeros((n_wgs, 8), dtype=np.uint64)
    _check(lib.dinfer_debug_trace(int(unit), out.ctypes.data, out.nbytes))
    return out


def stream_read(d_buf, nbytes, d_sink):
    """One pass of the streaming-read probe over the first nbytes of a device tensor."""
    _check(lib.dinfer_stream_read(_ptr(d_buf), int(nbytes), _ptr(d_sink), _stream()))


class Context:
    """A dinfer context plus the three device buffers it lives in (allocated through torch)."""

    def __init__(self, cfg, n_pages, max_seqs, max_tokens, max_pos, device="cuda:0", weights_buffer=None):
        """weights_buffer: the `weights` tensor of another Context of the same configuration whose tensors are
        already loaded (the packed weights are position independent, so contexts may share them)."""
        self.cfg = cfg
        self.device = torch.device(device)
        self.ccfg = make_config(cfg, max_pos)
        wb = lib.dinfer_weights_bytes(self.ccfg)
        kb = lib.dinfer_kv_bytes(self.ccfg, n_pages)
        sb = lib.dinfer_workspace_bytes(self.ccfg, max_seqs, max_tokens)
        if wb == 0 or kb == 0 or sb == 0:
            raise DinferError(-1, last_error())
        self.n_pages, self.max_seqs, self.max_tokens = n_pages, max_seqs, max_tokens
        if weights_buffer is not None:
            if weights_buffer.numel() < wb or weights_buffer.device != self.device:
                raise ValueError("weights_buffer does not fit this configuration")
            self.weights = weights_buffer
        else:
            self.weights = torch.empty(wb, dtype=torch.uint8, device=self.device)
        self.kv = torch.empty(kb, dtype=torch.uint8, device=self.device)
        self.ws = torch.empty(sb, dtype=torch.uint8, device=self.device)
        h = c_vp()
        _check(lib.dinfer_create(self.ccfg, _ptr(self.weights), self.weights.numel(), _ptr(self.kv), n_pages, _ptr(self.ws), sb, max_seqs,
                                 max_tokens, _stream(), ctypes.byref(h)))
        self.h = h

    def close(self):
        if self.h:
            torch.cuda.synchronize(self.device)
            lib.dinfer_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- weights
    def set_tensor(self, name, layer, array):
        """Upload one tensor given as a numpy array (float32, or uint16 bfloat16 bit patterns)."""
        a = np.ascontiguousarray(array)
        d = torch.from_numpy(a.reshape(-1).view(np.uint8)).to(self.device)
        _check(lib.dinfer_set_tensor(self.h, TENSOR_IDS[name], layer, _ptr(d), a.nbytes, _stream()))
        torch.cuda.current_stream().synchronize()     # d is released after the pack kernel has read it

    def load_weights(self, weights):
        for n in ("emb", "lm_head", "final_gain"):
            self.set_tensor(n, 0, weights[n])
        for l, lw in enumerate(weights["layers"]):
            for n, a in lw.items():
                self.set_tensor(n, l, a)

    # ---- the path
    def prefill(self, d_tokens, lens, d_page_table):
        h_lens = (c_i32 * len(lens))(*[int(x) for x in lens])
        _check(lib.dinfer_prefill(self.h, len(lens), _ptr(d_tokens), ctypes.cast(h_lens, c_vp), _ptr(d_page_table),
                                  d_page_table.shape[1], _stream()))

    def step(self, d_block_tokens, d_mask, d_prefix_len, d_page_table, threshold, fixed_k, d_conf, d_argmax,
             d_n_committed):
        n_seq, block_len = d_block_tokens.shape
        dec = _decode(threshold, fixed_k)
        _check(lib.dinfer_step(self.h, n_seq, block_len, _ptr(d_block_tokens), _ptr(d_mask), _ptr(d_prefix_len),
                               _ptr(d_page_table), d_page_table.shape[1], ctypes.byref(dec), _ptr(d_conf),
                               _ptr(d_argmax), _ptr(d_n_committed), _stream()))

    def smooth_scratch(self, max_tokens):
        """Device scratch buffer for step_smooth with up to max_tokens block tokens."""
        n = lib.dinfer_smooth_scratch_bytes(ctypes.byref(self.ccfg), int(max_tokens))
        if n == 0:
            raise DinferError(-1, "dinfer_smooth_scratch_bytes: unsupported size")
        return torch.empty(n, dtype=torch.uint8, device=self.device)

    def step_smooth(self, d_block_tokens, d_mask, d_prefix_len, d_page_table, threshold, fixed_k, alpha, d_delta,
                    d_scratch, d_conf, d_argmax, d_n_committed):
        n_seq, block_len = d_block_tokens.shape
        dec = _decode(threshold, fixed_k)
        _check(lib.dinfer_step_smooth(self.h, n_seq, block_len, _ptr(d_block_tokens), _ptr(d_mask), _ptr(d_prefix_len),
                                      _ptr(d_page_table), d_page_table.shape[1], ctypes.byref(dec), float(alpha),
                                      _ptr(d_delta), _ptr(d_scratch), d_scratch.numel(), _ptr(d_conf), _ptr(d_argmax),
                                      _ptr(d_n_committed), _stream()))

    def step_smooth_static(self, d_block_tokens, d_mask, d_prefix_len, d_page_table, threshold, fixed_k, alpha, d_delta,
                           d_conf, d_argmax, d_n_committed):
        """step_smooth with the library's own static scratch: the call allocates nothing."""
        n_seq, block_len = d_block_tokens.shape
        dec = _decode(threshold, fixed_k)
        _check(lib.dinfer_step_smooth_static(self.h, n_seq, block_len, _ptr(d_block_tokens), _ptr(d_mask),
                                             _ptr(d_prefix_len), _ptr(d_page_table), d_page_table.shape[1],
                                             ctypes.byref(dec), float(alpha), _ptr(d_delta), _ptr(d_conf),
                                             _ptr(d_argmax), _ptr(d_n_committed), _stream()))

    def step_credit(self, d_block_tokens, d_mask, d_prefix_len, d_page_table, threshold, fixed_k, alpha, beta, gamma,
                    d_credit_ids, d_credit_val, d_credit_n, d_conf, d_argmax, d_n_committed):
        n_seq, block_len = d_block_tokens.shape
        dec = _decode(threshold, fixed_k)
        cr = Credit(float(alpha), float(beta), float(gamma))
        _check(lib.dinfer_step_credit(self.h, n_seq, block_len, _ptr(d_block_tokens), _ptr(d_mask), _ptr(d_prefix_len),
                                      _ptr(d_page_table), d_page_table.shape[1], ctypes.byref(dec), ctypes.byref(cr),
                                      _ptr(d_credit_ids), _ptr(d_credit_val), _ptr(d_credit_n), _ptr(d_conf),
                                      _ptr(d_argmax), _ptr(d_n_committed), _stream()))

    def step_vicinity(self, d_block_tokens, d_vicinity_tokens, d_mask, d_prefix_len, d_page_table, threshold, fixed_k,
                      d_conf, d_argmax, d_n_committed):
        n_seq, block_len = d_block_tokens.shape
        look_back = d_vicinity_tokens.shape[1]
        dec = _decode(threshold, fixed_k)
        _check(lib.dinfer_step_vicinity(self.h, n_seq, block_len, look_back, _ptr(d_block_tokens),
                                        _ptr(d_vicinity_tokens), _ptr(d_mask), _ptr(d_prefix_len), _ptr(d_page_table),
                                        d_page_table.shape[1], ctypes.byref(dec), _ptr(d_conf), _ptr(d_argmax),
                                        _ptr(d_n_committed), _stream()))

    def refresh_block(self, d_block_tokens, d_prefix_len, d_page_table):
        n_seq, block_len = d_block_tokens.shape
        _check(lib.dinfer_refresh_block(self.h, n_seq, block_len, _ptr(d_block_tokens), _ptr(d_prefix_len),
                                        _ptr(d_page_table), d_page_table.shape[1], _stream()))

    def generate_block(self, d_block_tokens, d_mask, d_prefix_len, d_page_table, threshold, fixed_k, d_conf, d_argmax,
                       d_n_committed, max_steps, masked_hint=0, steps_per_wait=1):
        """The inner loop over the steps of a block; returns the number of steps that ran.  steps_per_wait: steps
        enqueued between two host waits when the step count depends on the data."""
        n_seq, block_len = d_block_tokens.shape
        dec = _decode(threshold, fixed_k)
        steps = c_i32(0)
        _check(lib.dinfer_generate_block(self.h, n_seq, block_len, _ptr(d_block_tokens), _ptr(d_mask),
                                         _ptr(d_prefix_len), _ptr(d_page_table), d_page_table.shape[1],
                                         ctypes.byref(dec), _ptr(d_conf), _ptr(d_argmax), _ptr(d_n_committed),
                                         int(max_steps), int(masked_hint), int(steps_per_wait), ctypes.byref(steps),
                                         _stream()))
        return steps.value

    def generate_block_smooth(self, d_block_tokens, d_mask, d_prefix_len, d_page_table, threshold, schedule, d_delta,
                              d_scratch, d_conf, d_argmax, d_n_committed, max_steps, steps_per_wait=1):
        """A block denoised with iteration smoothing; schedule = (alpha_init, alpha_growth, alpha_preset,
        threshold_start, threshold_decay).  Returns the number of steps that ran."""
        n_seq, block_len = d_block_tokens.shape
        dec = _decode(threshold, 0)
        sch = SmoothSchedule(*[float(v) for v in schedule])
        steps = c_i32(0)
        _check(lib.dinfer_generate_block_smooth(self.h, n_seq, block_len, _ptr(d_block_tokens), _ptr(d_mask),
                                                _ptr(d_prefix_len), _ptr(d_page_table), d_page_table.shape[1],
                                                ctypes.byref(dec), ctypes.byref(sch), _ptr(d_delta), _ptr(d_scratch),
                                                d_scratch.numel(), _ptr(d_conf), _ptr(d_argmax), _ptr(d_n_committed),
                                                int(max_steps), int(steps_per_wait), ctypes.byref(steps), _stream()))
        return steps.value

    def generate(self, d_out, d_block_tokens, d_mask, d_prefix_len, d_page_table, threshold, fixed_k, eos_id,
                 d_finished, d_conf, d_argmax, d_n_committed, steps_per_wait=1):
        """Outer loop over the blocks of d_out [n_seq][n_blocks * block_len]; returns the blocks that were run."""
        n_seq, block_len = d_block_tokens.shape
        n_blocks = d_out.shape[1] // block_len
        assert d_out.shape[1] == n_blocks * block_len and d_out.is_contiguous()
        dec = _decode(threshold, fixed_k)
        run = c_i32(0)
        _check(lib.dinfer_generate(self.h, n_seq, block_len, n_blocks, _ptr(d_out), _ptr(d_block_tokens), _ptr(d_mask),
                                   _ptr(d_prefix_len), _ptr(d_page_table), d_page_table.shape[1], ctypes.byref(dec),
                                   int(eos_id), int(steps_per_wait), _ptr(d_finished), _ptr(d_conf), _ptr(d_argmax),
                                   _ptr(d_n_committed), ctypes.byref(run), _stream()))
        return run.value

    # ---- KV rows in and out, test hooks
    def kv_write(self, layer, d_page_row, first_pos, d_k, d_v):
        _check(lib.dinfer_kv_write(self.h, layer, _ptr(d_page_row), first_pos, d_k.shape[0], _ptr(d_k), _ptr(d_v),
                                   _stream()))

    def kv_read(self, layer, d_page_row, first_pos, n_pos):
        D = self.cfg.n_heads * self.cfg.head_dim
        k = torch.empty((n_pos, D), dtype=torch.float32, device=self.device)
        v = torch.empty((n_pos, D), dtype=torch.float32, device=self.device)
        _check(lib.dinfer_kv_read(self.h, layer, _ptr(d_page_row), first_pos, n_pos, _ptr(k), _ptr(v), _stream()))
        return k, v

    def debug_logits(self, n_rows):
        out = torch.empty((n_rows, self.cfg.vocab), dtype=torch.float32, device=self.device)
        _check(lib.dinfer_debug_logits(self.h, n_rows, _ptr(out), _stream()))
        return out

    def profile_every(self, n_forwards):
        _check(lib.dinfer_profile_every(self.h, n_forwards))

    def profile_start(self, stage):
        _check(lib.dinfer_profile_start(self.h, stage))

    def profile_stop(self):
        """(launches recorded, summed milliseconds) of the profiled stage."""
        n, ms = c_i32(0), c_f32(0.0)
        _check(lib.dinfer_profile_stop(self.h, ctypes.byref(n), ctypes.byref(ms)))
        return n.value, ms.value

    def debug_get(self, what, shape, dtype):
        out = torch.empty(shape, dtype=dtype, device=self.device)
        _check(lib.dinfer_debug_get(self.h, what, _ptr(out), out.numel() * out.element_size(), _stream()))
        return out
