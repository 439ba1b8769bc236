// C-ABI of the dinfer library: argument checks, buffer carving, and the launch sequence of one forward.
#include "../../include/dinfer.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <vector>

#include "gemm.hpp"
#include "kernels.hpp"

using namespace dinfer;

// Scratch of dinfer_step_smooth_static: device memory that exists from the moment the library is loaded until the
// process ends, one copy per GPU.  In host code this name is only a handle for hipGetSymbolAddress; kernels and
// copies get the device address kept in g_static_scratch.
static __device__ __align__(256) unsigned char scratch[DINFER_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
void* g_static_scratch[MAX_DEVICES];   // device address of `scratch` on each GPU, resolved with that GPU current

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                        \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) return fail(DINFER_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

constexpr int MAX_LOOP_STEPS = 256;   // steps one dinfer_generate_block call can take (a block has at most 64 positions)

// Every kernel enqueued while a LiveScope exists is handed `word` (see step_is_dead in common.hpp).
struct LiveScope {
  explicit LiveScope(const int32_t* word) { set_live_word(word); }
  ~LiveScope() { set_live_word(nullptr); }
};

// Address of the static scratch array on the current device (*dev_out).  Resolved once per device.
int static_scratch_of_current_device(void** out, int* dev_out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(DINFER_EUNSUPPORTED, "device ordinal %d", dev);
  if (!g_static_scratch[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(DINFER_EHIP, "hipGetSymbolAddress returned a null address");
    g_static_scratch[dev] = p;
  }
  *out = g_static_scratch[dev];
  if (dev_out) *dev_out = dev;
  return DINFER_OK;
}

struct LayerW {
  size_t attn_gain, wqkv, wo, ffn_gain, router, gate_up, down;   // byte offsets into d_weights
};
struct WeightMap {
  size_t emb, emb_t, lm_head, final_gain;   // emb_t: the embedding matrix transposed and packed (iteration smoothing)
  std::vector<LayerW> layers;
  size_t total;
};

struct Carve {   // bump allocator over a byte range
  size_t at = 0;
  size_t take(size_t bytes) {
    const size_t o = at;
    at = align_up(at + bytes);
    return o;
  }
};

int check_config(const dinfer_config* c) {
  if (!c) return fail(DINFER_EINVAL, "config is null");
  if (c->dtype != DINFER_F32 && c->dtype != DINFER_BF16) return fail(DINFER_EINVAL, "dtype %d", c->dtype);
  if (c->n_layers < 1 || c->hidden < 64 || c->n_heads < 1 || c->n_experts < 1 || c->top_k < 1 || c->moe_inter < 64 ||
      c->vocab < 2 || c->max_pos < 1)
    return fail(DINFER_EINVAL, "non-positive or too small dimension");
  if (c->page_size != PAGE) return fail(DINFER_EUNSUPPORTED, "page_size must be %d", PAGE);
  if (c->head_dim != 64 && c->head_dim != 128) return fail(DINFER_EUNSUPPORTED, "head_dim must be 64 or 128");
  if (c->hidden % 64 || c->moe_inter % 64 || (c->n_heads * c->head_dim) % 64)
    return fail(DINFER_EUNSUPPORTED, "hidden, moe_inter and n_heads*head_dim must be multiples of 64");
  if (c->hidden > 4096) return fail(DINFER_EUNSUPPORTED, "hidden > 4096");
  if (c->n_experts > MAX_EXPERTS) return fail(DINFER_EUNSUPPORTED, "n_experts > %d", MAX_EXPERTS);
  if (c->top_k > MAX_TOPK || c->top_k > c->n_experts) return fail(DINFER_EINVAL, "top_k %d out of range", c->top_k);
  if (c->mask_id < 0 || c->mask_id >= c->vocab) return fail(DINFER_EINVAL, "mask_id out of range");
  if (c->max_pos > ATTN_MAX_PAGES * PAGE) return fail(DINFER_EUNSUPPORTED, "max_pos > %d", ATTN_MAX_PAGES * PAGE);
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return fail(DINFER_EINVAL, "rms_eps / rope_theta");
  return DINFER_OK;
}

WeightMap map_weights(const dinfer_config& c) {
  const bool bf = c.dtype == DINFER_BF16;
  const size_t es = bf ? 2 : 4;
  const int H = c.hidden, D = c.n_heads * c.head_dim, I = c.moe_inter, E = c.n_experts, V = c.vocab;
  WeightMap m;
  Carve cv;
  m.emb = cv.take((size_t)V * H * es);
  m.emb_t = cv.take((size_t)packed_bytes(bf, H / 64, smooth_kpad(bf, V)));
  m.lm_head = cv.take((size_t)packed_bytes(bf, (V + 63) / 64, H));
  m.final_gain = cv.take((size_t)H * 4);
  m.layers.resize(c.n_layers);
  for (auto& l : m.layers) {
    l.attn_gain = cv.take((size_t)H * 4);
    l.wqkv = cv.take((size_t)packed_bytes(bf, 3 * D / 64, H));
    l.wo = cv.take((size_t)packed_bytes(bf, H / 64, D));
    l.ffn_gain = cv.take((size_t)H * 4);
    l.router = cv.take((size_t)packed_bytes(bf, 1, H));   // one task: experts 0-31 and 32-63
    l.gate_up = cv.take((size_t)E * packed_bytes(bf, I / 32, H));
    l.down = cv.take((size_t)E * packed_bytes(bf, H / 64, I));
  }
  m.total = cv.at;
  return m;
}

// Key splits the attention grid offers per (query tile, head): what the longest possible sequence (key_bound keys)
// would use under the rule of attn_splits_for (common.hpp), but no more than it takes to give every compute unit
// one workgroup (a workgroup fills a compute unit's LDS, so more of them only queue up: measured at 16 sequences
// with up to 5 splits each, 85 us against 43 without splits); every sequence then uses its own count.
int attn_splits(int n_qtiles, int n_heads, int key_bound) {
  int s = attn_splits_for(key_bound);
  const int cover = (256 + n_qtiles * n_heads - 1) / (n_qtiles * n_heads);
  return s > cover ? cover : s;
}

struct Workspace {
  size_t cos_tab, sin_tab, tok_seq, tok_pos, seq_nkeys, qtile, x, xn, ssq, ssq_a, tk_part, tickets, tickets_bytes, attn_tickets, attn_tickets_bytes, rinv_f, q, a, attn_part, topk_idx, topk_w, cnt, off,
      perm, pos_of_pair, work, run_tokens, run_base, n_finished, loop_flags, loop_steps, lm_rows, y, o, lm_part, lm_stats, conf, argmax, total;
};

Workspace map_workspace(const dinfer_config& c, int max_seqs, int max_tokens) {
  const size_t es = c.dtype == DINFER_BF16 ? 2 : 4;
  const int H = c.hidden, D = c.n_heads * c.head_dim, I = c.moe_inter, K = c.top_k;
  const size_t T = (size_t)max_tokens;
  const int max_qtiles = max_tokens / TILE + max_seqs;
  Workspace w;
  Carve cv;
  w.cos_tab = cv.take((size_t)c.max_pos * (c.head_dim / 2) * 4);
  w.sin_tab = cv.take((size_t)c.max_pos * (c.head_dim / 2) * 4);
  w.tok_seq = cv.take(T * 4);
  w.tok_pos = cv.take(T * 4);
  w.seq_nkeys = cv.take((size_t)max_seqs * 4);
  w.qtile = cv.take((size_t)max_qtiles * 3 * 4);
  w.x = cv.take(T * H * 4);
  w.rinv_f = cv.take(T * 4);   // 1/rms of the residual rows entering the expert half
  const size_t planes = c.dtype == DINFER_BF16 ? 2 : 1;   // stored bf16 activations are hi + lo planes
  w.xn = cv.take(planes * T * H * es);   // normalised-input planes of the residual rows
  w.ssq = cv.take((size_t)(H / 64) * T * 4);     // sums of squares of the rows entering the expert half, per task
  w.ssq_a = cv.take((size_t)(H / 64) * T * 4);   // ... of the rows entering the attention half / the LM head
  {
    // cross-workgroup split-K scratch: units (tasks) x slices x [2 * token tiles * 16][64] floats, for one and
    // two token tiles, over the QKV projection (K = H), the output projection (K = D) and the router
    const bool bf = c.dtype == DINFER_BF16;
    size_t most = 0;
    for (int tt = 1; tt <= 2; ++tt) {
      const size_t tile = (size_t)2 * tt * 16 * WAVE * 4;
      const size_t qkv = (size_t)(3 * D / 64) * gemm_slices(bf, H, tt * TILE) * tile;
      const size_t opr = (size_t)(H / 64) * gemm_slices(bf, D, tt * TILE) * tile;
      const size_t smooth = (size_t)(H / 64) * SMOOTH_SLICES * tile;   // expected-embedding contraction
      const size_t down = (size_t)(H / 64) * down_fused_slices() * tile;   // fused down projection
      most = down > most ? down : most;
      most = qkv > most ? qkv : most;
      most = opr > most ? opr : most;
      most = smooth > most ? smooth : most;
    }
    w.tk_part = cv.take(most);
    const int units = 3 * D / 64 > H / 64 ? 3 * D / 64 : H / 64;
    w.tickets_bytes = (size_t)units * 4;
    w.tickets = cv.take(w.tickets_bytes);
  }
  w.q = cv.take(planes * T * D * es);
  w.a = cv.take(planes * T * D * es);
  size_t part = 0;   // the split policy depends on the number of query tiles only
  for (int nq = 1; nq <= max_qtiles; ++nq) {
    const size_t p = attn_part_floats(nq, c.n_heads, attn_splits(nq, c.n_heads, c.max_pos), c.head_dim);
    if (p > part) part = p;
  }
  w.attn_part = cv.take(part * 4);
  w.attn_tickets_bytes = (size_t)max_qtiles * c.n_heads * 4;   // one arrival counter per (query tile, head)
  w.attn_tickets = cv.take(w.attn_tickets_bytes);
  w.topk_idx = cv.take((size_t)c.n_layers * T * K * 4);   // kept per layer (tests read the routing back)
  w.topk_w = cv.take((size_t)c.n_layers * T * K * 4);
  w.cnt = cv.take((size_t)MAX_EXPERTS * 4);
  w.off = cv.take((size_t)OFF_INTS * 4);   // offsets, then the lists of experts with rows (gemm.hpp)
  w.perm = cv.take(T * K * 4);
  w.pos_of_pair = cv.take(T * K * 4);
  w.run_tokens = cv.take(T * 4);                 // token run and start positions of a vicinity-refresh forward
  w.run_base = cv.take((size_t)max_seqs * 4);
  w.n_finished = cv.take(4);                     // generation loop: sequences that have produced the end-of-sequence id
  w.loop_flags = cv.take((size_t)(MAX_LOOP_STEPS + 1) * 4);   // inner loop: "step i is still needed" words
  w.loop_steps = cv.take(4);                     // inner loop: steps that ran
  w.lm_rows = cv.take((size_t)(1 + T) * 4);      // LM head: rows of the undecided positions
  w.work = cv.take((size_t)(1 + expert_work_items(MAX_EXPERTS, (int)(T * K))) * 4);
  w.y = cv.take(planes * T * K * I * es);
  w.o = cv.take(T * K * H * 4);
  w.lm_part = cv.take((size_t)lm_head_waves(c.vocab) * T * 4 * 4);
  w.lm_stats = cv.take(T * 2 * 4);
  w.conf = cv.take(T * 4);
  w.argmax = cv.take(T * 4);
  w.total = cv.at;
  return w;
}

}  // namespace

struct dinfer_ctx {
  dinfer_config cfg;
  bool bf16;
  char* weights;
  char* kv;
  char* ws;
  int n_pages, max_seqs, max_tokens;
  WeightMap wm;
  Workspace wsm;
  KvGeom geom;
  size_t kv_layer_bytes;
  int last_T;   // tokens of the last forward (debug hooks)
  int last_n_ssq;   // shares the last forward left per row in ssq_a (statistics of the rows the LM head reads)
  int device;   // GPU that was current at dinfer_create: owner of the three buffers
  uint64_t* h_mask_pinned;
  // optional per-launch timing of one stage (dinfer_profile_start / _stop)
  int prof_stage;
  size_t prof_n;
  int prof_every;      // launches of every prof_every-th forward are bracketed
  int64_t prof_fwd;    // forwards since dinfer_profile_start
  bool prof_sampled;   // the current forward is one of them
  std::vector<hipEvent_t> prof_ev;   // start/stop pairs
};

namespace {

template <typename T> T* at(char* base, size_t off) { return reinterpret_cast<T*>(base + off); }

constexpr size_t PROF_MAX_LAUNCHES = 8192;

int check_decode(const dinfer_decode* d) {
  if (!d) return fail(DINFER_EINVAL, "decode is null");
  if (d->fixed_k < 0 || d->fixed_k > 64) return fail(DINFER_EINVAL, "fixed_k %d", d->fixed_k);
  if (d->hierarchical) {
    if (d->fixed_k > 0) return fail(DINFER_EINVAL, "hierarchical decoding with fixed_k %d", d->fixed_k);
    if (!(d->lower_bound <= d->threshold)) return fail(DINFER_EINVAL, "lower_bound %g above threshold %g",
                                                        (double)d->lower_bound, (double)d->threshold);
  }
  return DINFER_OK;
}
CommitRule commit_rule(const dinfer_decode* d) {
  return CommitRule{d->threshold, d->fixed_k, d->hierarchical != 0 ? 1 : 0, d->lower_bound};
}

// Brackets the launches of one stage with an event pair when that stage is being profiled.
struct StageTimer {
  dinfer_ctx* c;
  hipStream_t st;
  bool on;
  StageTimer(dinfer_ctx* c_, int stage, hipStream_t st_) : c(c_), st(st_), on(false) {
    if (c->prof_stage == stage && c->prof_sampled && c->prof_n < PROF_MAX_LAUNCHES) {
      on = true;
      (void)hipEventRecord(c->prof_ev[2 * c->prof_n], st);
    }
  }
  ~StageTimer() {
    if (on) {
      (void)hipEventRecord(c->prof_ev[2 * c->prof_n + 1], st);
      ++c->prof_n;
    }
  }
};

// One forward over the packed tokens of `span`.  with_head: final norm into h (ready for the LM head).
int forward(dinfer_ctx* c, const SeqSpan& span, const int32_t* d_tokens, const int32_t* d_base,
            const int32_t* d_page_table, int pt_stride, bool with_head, hipStream_t st,
            const SmoothIn* smooth = nullptr) {
  const dinfer_config& f = c->cfg;
  const bool bf = c->bf16;
  const int T = span.off[span.n_seq];
  const int H = f.hidden, D = f.n_heads * f.head_dim;
  char* ws = c->ws;
  const Workspace& w = c->wsm;
  if (c->prof_stage >= 0) c->prof_sampled = c->prof_fwd++ % c->prof_every == 0;
  int n_qtiles = 0;
  for (int s = 0; s < span.n_seq; ++s) n_qtiles += (span.off[s + 1] - span.off[s] + TILE - 1) / TILE;
  FwdMeta meta{at<int32_t>(ws, w.tok_seq), at<int32_t>(ws, w.tok_pos), at<int32_t>(ws, w.seq_nkeys),
               at<int32_t>(ws, w.qtile)};
  const int limit = f.max_pos < pt_stride * PAGE ? f.max_pos : pt_stride * PAGE;
  float* x = at<float>(ws, w.x);
  float* ssq_a = at<float>(ws, w.ssq_a);
  float* rinv_f = at<float>(ws, w.rinv_f);
  // Up to 32 tokens the down projection sums a token's experts itself and leaves the residual row, its planes for
  // the next norm and one share of its sum of squares per task; larger forwards run the combine kernel.  (With two
  // token tiles every wave of the fused form fetches twice the activation operands per weight byte, and the
  // separate kernels are faster: measured at 64 tokens, 251 against 259 steps/s.)
  // (the fused kernel needs its 64 wave shares, each within two experts; under the single-slice test switch the
  // down projection takes the unfused route, which has no sum across workgroups)
  const bool fused_down = T <= TILE && !single_slice();
  int n_ssq_a = 1;
  const int64_t q_plane = (int64_t)c->max_tokens * D;
  for (int l = 0; l < f.n_layers; ++l) {
    const LayerW& lw = c->wm.layers[l];
    char* kv_layer = c->kv + (size_t)l * c->kv_layer_bytes;
    int32_t* topk_idx = at<int32_t>(ws, w.topk_idx) + (size_t)l * T * f.top_k;
    float* topk_w = at<float>(ws, w.topk_w) + (size_t)l * T * f.top_k;
    void* xn = ws + w.xn;
    float* tk_part = at<float>(ws, w.tk_part);
    int32_t* tickets = at<int32_t>(ws, w.tickets);
    if (l == 0)
      launch_embed(bf, d_tokens, c->weights + c->wm.emb, T, H, f.vocab, x, ssq_a, at<float>(c->weights, lw.attn_gain),
                   xn, smooth, span, d_base, limit, at<int32_t>(ws, w.tok_seq), at<int32_t>(ws, w.tok_pos),
                   at<int32_t>(ws, w.seq_nkeys), at<int32_t>(ws, w.qtile), st);
    else if (!fused_down)
      launch_combine(bf, x, at<float>(ws, w.o), topk_w - (size_t)T * f.top_k, f.top_k, T, H, ssq_a,
                     at<float>(c->weights, lw.attn_gain), xn, st);
    QkvArgs qa{c->weights + lw.wqkv, xn, RowNorm{ssq_a, n_ssq_a, f.rms_eps}, ws + w.q, q_plane, kv_layer, c->geom, meta,
               d_page_table, pt_stride, at<float>(ws, w.cos_tab), at<float>(ws, w.sin_tab), T, H, tk_part, tickets};
    {
      StageTimer tm(c, DINFER_STAGE_QKV, st);
      launch_qkv(bf, qa, st);
#ifdef DINFER_TRACE
      if (DINFER_TRACE == 1 && getenv("DINFER_TRACE_REPEAT")) launch_qkv(bf, qa, st);   // second launch: warm caches
#endif
    }
    AttnArgs aa{ws + w.q, q_plane, kv_layer, c->geom, meta, d_page_table, pt_stride, n_qtiles,
                single_slice() ? 1 : attn_splits(n_qtiles, f.n_heads, limit), at<float>(ws, w.attn_part), at<int32_t>(ws, w.attn_tickets),
                ws + w.a, T, oproj_prefetch_plan(bf, c->weights + lw.wo, D, H, T)};
    {
      StageTimer tm(c, DINFER_STAGE_ATTENTION, st);
      launch_attention(bf, aa, st);
    }
    OprojArgs oa{c->weights + lw.wo, ws + w.a, x, at<float>(c->weights, lw.ffn_gain), xn,
                 at<float>(ws, w.ssq), T, D, H, tk_part, tickets};
    {
      StageTimer tm(c, DINFER_STAGE_OPROJ, st);
      launch_oproj(bf, oa, st);
    }
    RouterArgs ra{c->weights + lw.router, xn, at<float>(ws, w.ssq), f.rms_eps, T, H, f.n_experts, f.top_k,
                  f.norm_topk, rinv_f, topk_idx, topk_w, at<int32_t>(ws, w.cnt), at<int32_t>(ws, w.off),
                  at<int32_t>(ws, w.perm), at<int32_t>(ws, w.pos_of_pair), at<int32_t>(ws, w.work), tk_part, tickets};
    {
      StageTimer tm(c, DINFER_STAGE_ROUTER, st);
      launch_router(bf, ra, st);
    }
    ExpertArgs ea{c->weights + lw.gate_up, c->weights + lw.down, xn, rinv_f,
                  ws + w.y, at<float>(ws, w.o), at<int32_t>(ws, w.cnt), at<int32_t>(ws, w.off),
                  at<int32_t>(ws, w.perm), at<int32_t>(ws, w.work), T, H, f.moe_inter, f.n_experts, f.top_k,
                  fused_down ? topk_w : nullptr, topk_idx, at<int32_t>(ws, w.pos_of_pair)};
    {
      StageTimer tm(c, DINFER_STAGE_EXPERT_GATE_UP, st);
      launch_expert_gate_up(bf, ea, st);
    }
    {
      StageTimer tm(c, DINFER_STAGE_EXPERT_DOWN, st);
      if (fused_down) {
        // the gain of the norm that reads the new rows: the next layer's attention norm, or the final norm
        const float* next_gain = l + 1 < f.n_layers ? at<float>(c->weights, c->wm.layers[l + 1].attn_gain)
                                                    : at<float>(c->weights, c->wm.final_gain);
        OprojArgs res{nullptr, nullptr, x, next_gain, xn, ssq_a, T, 0, H, tk_part, tickets};
        launch_expert_down_fused(bf, ea, res, st);
        n_ssq_a = H / 64;
      } else {
        launch_expert_down(bf, ea, st);
      }
    }
  }
  // many tokens: the last layer's expert outputs are folded into the residual here, with the final norm's gain
  if (!fused_down)
    launch_combine(bf, x, at<float>(ws, w.o), at<float>(ws, w.topk_w) + (size_t)(f.n_layers - 1) * T * f.top_k, f.top_k,
                   T, H, ssq_a, at<float>(c->weights, c->wm.final_gain), ws + w.xn, st);
  c->last_n_ssq = n_ssq_a;
  (void)with_head;
  c->last_T = T;
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int check_block_args(dinfer_ctx* c, int n_seq, int block_len, const void* tokens, const void* prefix_len,
                     const void* page_table, int pt_stride) {
  if (!c) return fail(DINFER_EINVAL, "context is null");
  if (!tokens || !prefix_len || !page_table) return fail(DINFER_EINVAL, "null device pointer");
  if (n_seq < 1 || n_seq > c->max_seqs) return fail(DINFER_EINVAL, "n_seq %d outside [1, %d]", n_seq, c->max_seqs);
  if (block_len < 1 || block_len > 64) return fail(DINFER_EINVAL, "block_len %d outside [1, 64]", block_len);
  if ((int64_t)n_seq * block_len > c->max_tokens)
    return fail(DINFER_ENOSPACE, "n_seq*block_len %d exceeds max_tokens %d", n_seq * block_len, c->max_tokens);
  if (pt_stride < (block_len + PAGE - 1) / PAGE) return fail(DINFER_ENOSPACE, "page table row too short");
  if (block_len > c->cfg.max_pos) return fail(DINFER_ENOSPACE, "block_len exceeds max_pos");
  return DINFER_OK;
}

SeqSpan uniform_span(int n_seq, int len) {
  SeqSpan s;
  s.n_seq = n_seq;
  for (int i = 0; i <= n_seq; ++i) s.off[i] = i * len;
  return s;
}

}  // namespace

extern "C" {

const char* dinfer_last_error(void) { return g_err; }

size_t dinfer_weights_bytes(const dinfer_config* cfg) {
  if (check_config(cfg) != DINFER_OK) return 0;
  return map_weights(*cfg).total;
}

size_t dinfer_kv_bytes(const dinfer_config* cfg, int32_t n_pages) {
  if (check_config(cfg) != DINFER_OK || n_pages < 1) return 0;
  const size_t es = cfg->dtype == DINFER_BF16 ? 2 : 4;
  return (size_t)cfg->n_layers * n_pages * 2 * cfg->n_heads * PAGE * cfg->head_dim * es;
}

size_t dinfer_workspace_bytes(const dinfer_config* cfg, int32_t max_seqs, int32_t max_tokens) {
  if (check_config(cfg) != DINFER_OK || max_seqs < 1 || max_seqs > MAX_SEQS || max_tokens < 1) return 0;
  if ((int64_t)max_tokens * cfg->top_k > permute_max_pairs()) return 0;
  return map_workspace(*cfg, max_seqs, max_tokens).total;
}

int dinfer_create(const dinfer_config* cfg, void* d_weights, size_t weights_bytes, void* d_kv_pool, int32_t n_pages,
                  void* d_workspace, size_t workspace_bytes, int32_t max_seqs, int32_t max_tokens, void* stream,
                  dinfer_ctx** out) {
  if (!out) return fail(DINFER_EINVAL, "out is null");
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc != DINFER_OK) return rc;
  if (!d_weights || !d_kv_pool || !d_workspace) return fail(DINFER_EINVAL, "null device buffer");
  if (((uintptr_t)d_weights | (uintptr_t)d_kv_pool | (uintptr_t)d_workspace) & 255)
    return fail(DINFER_EINVAL, "device buffers must be 256-byte aligned");
  if (n_pages < 1) return fail(DINFER_EINVAL, "n_pages < 1");
  if (max_seqs < 1 || max_seqs > MAX_SEQS) return fail(DINFER_EINVAL, "max_seqs outside [1, %d]", MAX_SEQS);
  if (max_tokens < 1) return fail(DINFER_EINVAL, "max_tokens < 1");
  if ((int64_t)max_tokens * cfg->top_k > permute_max_pairs())
    return fail(DINFER_EUNSUPPORTED, "max_tokens * top_k exceeds %d routed pairs per forward", permute_max_pairs());
  dinfer_ctx* c = new (std::nothrow) dinfer_ctx();
  if (!c) return fail(DINFER_EINVAL, "out of host memory");
  c->cfg = *cfg;
  c->bf16 = cfg->dtype == DINFER_BF16;
  c->wm = map_weights(*cfg);
  c->wsm = map_workspace(*cfg, max_seqs, max_tokens);
  if (weights_bytes < c->wm.total || workspace_bytes < c->wsm.total) {
    rc = fail(DINFER_ENOSPACE, "weights buffer %zu < %zu or workspace %zu < %zu", weights_bytes, c->wm.total,
              workspace_bytes, c->wsm.total);
    delete c;
    return rc;
  }
  c->weights = (char*)d_weights;
  c->kv = (char*)d_kv_pool;
  c->ws = (char*)d_workspace;
  c->n_pages = n_pages;
  c->max_seqs = max_seqs;
  c->max_tokens = max_tokens;
  const size_t es = c->bf16 ? 2 : 4;
  c->geom.n_heads = cfg->n_heads;
  c->geom.head_dim = cfg->head_dim;
  c->geom.n_pages = n_pages;
  c->geom.kblk = 32 / (int)es;
  c->geom.page_stride = (int64_t)2 * cfg->n_heads * PAGE * cfg->head_dim;
  c->geom.layer_stride = c->geom.page_stride * n_pages;
  c->kv_layer_bytes = (size_t)c->geom.layer_stride * es;
  c->last_T = 0;
  c->last_n_ssq = 1;
  {
    // set-up is the place for everything that may allocate: the static scratch of this GPU is resolved here, so
    // that dinfer_step_smooth_static finds its address ready
    void* unused = nullptr;
    rc = static_scratch_of_current_device(&unused, &c->device);
    if (rc != DINFER_OK) {
      delete c;
      return rc;
    }
  }
  c->prof_stage = -1;
  c->prof_n = 0;
  c->prof_every = 1;
  c->prof_fwd = 0;
  c->prof_sampled = true;
  c->h_mask_pinned = nullptr;
  if (hipHostMalloc((void**)&c->h_mask_pinned, MAX_SEQS * sizeof(uint64_t), hipHostMallocDefault) != hipSuccess) {
    delete c;
    return fail(DINFER_EHIP, "hipHostMalloc failed");
  }
  if (!configure_kernels() || !configure_attention() || !configure_permute() || !configure_wide()) {
    (void)hipHostFree(c->h_mask_pinned);
    delete c;
    return fail(DINFER_EHIP, "the runtime refused the kernels' LDS sizes");
  }
  // the arrival counters start at zero and every kernel that uses them leaves them at zero
  if (hipMemsetAsync(c->ws + c->wsm.tickets, 0, c->wsm.tickets_bytes, (hipStream_t)stream) != hipSuccess ||
      hipMemsetAsync(c->ws + c->wsm.attn_tickets, 0, c->wsm.attn_tickets_bytes, (hipStream_t)stream) != hipSuccess ||
      hipMemsetAsync(c->ws + c->wsm.off, 0, (size_t)OFF_INTS * 4, (hipStream_t)stream) != hipSuccess) {
    (void)hipHostFree(c->h_mask_pinned);
    delete c;
    return fail(DINFER_EHIP, "clearing the workspace failed");
  }
  launch_rope_table(at<float>(c->ws, c->wsm.cos_tab), at<float>(c->ws, c->wsm.sin_tab), cfg->max_pos, cfg->head_dim,
                    cfg->rope_theta, (hipStream_t)stream);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    rc = fail(DINFER_EHIP, "rotary table launch: %s", hipGetErrorString(e));
    (void)hipHostFree(c->h_mask_pinned);
    delete c;
    return rc;
  }
  *out = c;
  return DINFER_OK;
}

void dinfer_destroy(dinfer_ctx* ctx) {
  if (!ctx) return;
  for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
  if (ctx->h_mask_pinned) (void)hipHostFree(ctx->h_mask_pinned);
  delete ctx;
}

int dinfer_set_tensor(dinfer_ctx* c, int32_t tensor_id, int32_t layer, const void* d_src, size_t bytes, void* stream) {
  if (!c || !d_src) return fail(DINFER_EINVAL, "null argument");
  if (tensor_id < 0 || tensor_id >= DINFER_T_COUNT) return fail(DINFER_EINVAL, "tensor id %d", tensor_id);
  const dinfer_config& f = c->cfg;
  const bool per_layer = tensor_id >= DINFER_T_ATTN_GAIN;
  if (per_layer && (layer < 0 || layer >= f.n_layers)) return fail(DINFER_EINVAL, "layer %d", layer);
  const bool bf = c->bf16;
  const size_t es = bf ? 2 : 4;
  const int H = f.hidden, D = f.n_heads * f.head_dim, I = f.moe_inter, E = f.n_experts, V = f.vocab;
  hipStream_t st = (hipStream_t)stream;
  const LayerW* lw = per_layer ? &c->wm.layers[layer] : nullptr;
  size_t want = 0;
  switch (tensor_id) {
    case DINFER_T_EMB: want = (size_t)V * H * es; break;
    case DINFER_T_LM_HEAD: want = (size_t)V * H * es; break;
    case DINFER_T_FINAL_GAIN: case DINFER_T_ATTN_GAIN: case DINFER_T_FFN_GAIN: want = (size_t)H * 4; break;
    case DINFER_T_WQ: case DINFER_T_WK: case DINFER_T_WV: case DINFER_T_WO: want = (size_t)D * H * es; break;
    case DINFER_T_ROUTER: want = (size_t)E * H * es; break;
    default: want = (size_t)E * I * H * es; break;
  }
  if (bytes != want) return fail(DINFER_EINVAL, "tensor %d: %zu bytes given, %zu expected", tensor_id, bytes, want);
  char* W = c->weights;
  const size_t qk_bytes = (size_t)packed_bytes(bf, D / 64, H);
  switch (tensor_id) {
    case DINFER_T_EMB:
      HIP_TRY(hipMemcpyAsync(W + c->wm.emb, d_src, bytes, hipMemcpyDeviceToDevice, st));
      launch_pack_transposed(bf, d_src, W + c->wm.emb_t, V, H, smooth_kpad(bf, V), st);
      break;
    case DINFER_T_LM_HEAD: launch_pack(bf, d_src, W + c->wm.lm_head, 1, V, H, (V + 63) / 64, PACK_ADJACENT, 0, st); break;
    case DINFER_T_FINAL_GAIN: HIP_TRY(hipMemcpyAsync(W + c->wm.final_gain, d_src, bytes, hipMemcpyDeviceToDevice, st)); break;
    case DINFER_T_ATTN_GAIN: HIP_TRY(hipMemcpyAsync(W + lw->attn_gain, d_src, bytes, hipMemcpyDeviceToDevice, st)); break;
    case DINFER_T_FFN_GAIN: HIP_TRY(hipMemcpyAsync(W + lw->ffn_gain, d_src, bytes, hipMemcpyDeviceToDevice, st)); break;
    case DINFER_T_WQ: launch_pack(bf, d_src, W + lw->wqkv, 1, D, H, D / 64, PACK_ROPE_PAIR, f.head_dim, st); break;
    case DINFER_T_WK: launch_pack(bf, d_src, W + lw->wqkv + qk_bytes, 1, D, H, D / 64, PACK_ROPE_PAIR, f.head_dim, st); break;
    case DINFER_T_WV: launch_pack(bf, d_src, W + lw->wqkv + 2 * qk_bytes, 1, D, H, D / 64, PACK_ADJACENT, 0, st); break;
    case DINFER_T_WO: launch_pack(bf, d_src, W + lw->wo, 1, H, D, H / 64, PACK_ADJACENT, 0, st); break;
    case DINFER_T_ROUTER: launch_pack(bf, d_src, W + lw->router, 1, E, H, 1, PACK_ADJACENT, 0, st); break;
    case DINFER_T_GATE: launch_pack(bf, d_src, W + lw->gate_up, E, I, H, I / 32, PACK_HALF0, 0, st); break;
    case DINFER_T_UP: launch_pack(bf, d_src, W + lw->gate_up, E, I, H, I / 32, PACK_HALF1, 0, st); break;
    case DINFER_T_DOWN: launch_pack(bf, d_src, W + lw->down, E, H, I, H / 64, PACK_ADJACENT, 0, st); break;
  }
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_prefill(dinfer_ctx* c, int32_t n_seq, const int32_t* d_tokens, const int32_t* h_lens,
                   const int32_t* d_page_table, int32_t pt_stride, void* stream) {
  if (!c) return fail(DINFER_EINVAL, "context is null");
  if (!d_tokens || !h_lens || !d_page_table) return fail(DINFER_EINVAL, "null pointer");
  if (n_seq < 1 || n_seq > c->max_seqs) return fail(DINFER_EINVAL, "n_seq %d outside [1, %d]", n_seq, c->max_seqs);
  SeqSpan span;
  span.n_seq = n_seq;
  span.off[0] = 0;
  int qtiles = 0;
  for (int s = 0; s < n_seq; ++s) {
    if (h_lens[s] < 1 || h_lens[s] > c->cfg.max_pos) return fail(DINFER_EINVAL, "prompt length %d", h_lens[s]);
    if (pt_stride * PAGE < h_lens[s]) return fail(DINFER_ENOSPACE, "page table row too short for prompt %d", s);
    span.off[s + 1] = span.off[s] + h_lens[s];
    qtiles += (h_lens[s] + TILE - 1) / TILE;
  }
  if (span.off[n_seq] > c->max_tokens || qtiles > c->max_tokens / TILE + c->max_seqs)
    return fail(DINFER_ENOSPACE, "prefill of %d tokens exceeds max_tokens %d", span.off[n_seq], c->max_tokens);
  return forward(c, span, d_tokens, nullptr, d_page_table, pt_stride, false, (hipStream_t)stream);
}

// One plain step.  live / next_live / steps: the words of a loop of steps enqueued ahead of the host (null for a
// single step).
static int step_impl(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                     const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                     const dinfer_decode* decode, float* d_conf, int32_t* d_argmax, int32_t* d_n_committed,
                     hipStream_t st, const int32_t* live, int32_t* next_live, int32_t* steps) {
  int rc = check_block_args(c, n_seq, block_len, d_block_tokens, d_prefix_len, d_page_table, pt_stride);
  if (rc != DINFER_OK) return rc;
  if (!d_mask || !decode || !d_conf || !d_argmax || !d_n_committed) return fail(DINFER_EINVAL, "null pointer");
  if ((rc = check_decode(decode)) != DINFER_OK) return rc;
  LiveScope scope(live);
  rc = forward(c, uniform_span(n_seq, block_len), d_block_tokens, d_prefix_len, d_page_table, pt_stride, true, st);
  if (rc != DINFER_OK) return rc;
  const dinfer_config& f = c->cfg;
  const int T = n_seq * block_len;
  LmArgs la{c->weights + c->wm.lm_head, c->ws + c->wsm.xn,
            RowNorm{at<float>(c->ws, c->wsm.ssq_a), c->last_n_ssq, f.rms_eps}, T, f.hidden, f.vocab, f.logit_scale,
            at<float>(c->ws, c->wsm.lm_part), nullptr};
  const bool skip = decode->skip_decided != 0;
  if (skip && T > 2 * TILE) {   // with few tokens the LM head is bound by its weight stream: rows cost nothing there
    int32_t* rows = at<int32_t>(c->ws, c->wsm.lm_rows);
    launch_lm_rows(d_mask, n_seq, block_len, rows, st);
    la.rows = rows;
  }
  {
    StageTimer tm(c, DINFER_STAGE_LM_HEAD, st);
    launch_lm_head(c->bf16, la, st);
  }
  launch_lm_merge(la.part, lm_head_parts(f.vocab, T), T, d_conf, d_argmax, nullptr, st, skip ? d_mask : nullptr, block_len);
  launch_commit(d_conf, d_argmax, n_seq, block_len, block_len, 0, d_block_tokens, d_mask, commit_rule(decode), d_n_committed,
                nullptr, nullptr, st, next_live, steps);
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_step(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride, const dinfer_decode* decode,
                float* d_conf, int32_t* d_argmax, int32_t* d_n_committed, void* stream) {
  return step_impl(c, n_seq, block_len, d_block_tokens, d_mask, d_prefix_len, d_page_table, pt_stride, decode, d_conf,
                   d_argmax, d_n_committed, (hipStream_t)stream, nullptr, nullptr, nullptr);
}

size_t dinfer_smooth_scratch_bytes(const dinfer_config* cfg, int32_t max_tokens) {
  if (check_config(cfg) != DINFER_OK || max_tokens < 1) return 0;
  const bool bf = cfg->dtype == DINFER_BF16;
  const size_t planes = bf ? 2 : 1, es = bf ? 2 : 4;
  return align_up((size_t)max_tokens * cfg->vocab * 4) + align_up(planes * max_tokens * smooth_kpad(bf, cfg->vocab) * es);
}

// live / next_live / steps: as in step_impl.
static int smooth_impl(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                       const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                       const dinfer_decode* decode, float alpha, float* d_delta, void* d_scratch, size_t scratch_bytes,
                       float* d_conf, int32_t* d_argmax, int32_t* d_n_committed, hipStream_t st, const int32_t* live,
                       int32_t* next_live, int32_t* steps) {
  int rc = check_block_args(c, n_seq, block_len, d_block_tokens, d_prefix_len, d_page_table, pt_stride);
  if (rc != DINFER_OK) return rc;
  if (!d_mask || !decode || !d_conf || !d_argmax || !d_n_committed || !d_delta || !d_scratch)
    return fail(DINFER_EINVAL, "null pointer");
  if ((rc = check_decode(decode)) != DINFER_OK) return rc;
  if (!(alpha >= 0.f)) return fail(DINFER_EINVAL, "alpha must be >= 0");
  const dinfer_config& f = c->cfg;
  const int T = n_seq * block_len;
  if ((uintptr_t)d_scratch & 255) return fail(DINFER_EINVAL, "scratch must be 256-byte aligned");
  const size_t need = dinfer_smooth_scratch_bytes(&f, T);
  if (scratch_bytes < need) return fail(DINFER_ENOSPACE, "smoothing scratch %zu < %zu bytes", scratch_bytes, need);
  LiveScope scope(live);
  float* logits = (float*)d_scratch;
  void* probs = (char*)d_scratch + align_up((size_t)T * f.vocab * 4);
  SmoothIn sin{d_delta, alpha, d_mask, block_len};
  rc = forward(c, uniform_span(n_seq, block_len), d_block_tokens, d_prefix_len, d_page_table, pt_stride, true, st,
               alpha > 0.f ? &sin : nullptr);
  if (rc != DINFER_OK) return rc;
  float* stats = at<float>(c->ws, c->wsm.lm_stats);
  // this variant keeps the logits of the block (T x vocab float32): the second contraction over the vocabulary
  // needs the normalised probabilities, which exist only once the row's maximum and sum are known
  LmArgs la{c->weights + c->wm.lm_head, c->ws + c->wsm.xn,
            RowNorm{at<float>(c->ws, c->wsm.ssq_a), c->last_n_ssq, f.rms_eps}, T, f.hidden, f.vocab, f.logit_scale,
            at<float>(c->ws, c->wsm.lm_part), logits};
  {
    StageTimer tm(c, DINFER_STAGE_LM_HEAD, st);
    launch_lm_head(c->bf16, la, st);
  }
  launch_lm_merge(la.part, lm_head_parts(f.vocab, T), T, d_conf, d_argmax, stats, st);
  SmoothArgs sa{c->weights + c->wm.emb_t, logits, stats, probs, d_mask, block_len, d_delta, T, f.hidden, f.vocab,
                at<float>(c->ws, c->wsm.tk_part), at<int32_t>(c->ws, c->wsm.tickets)};
  launch_expected_embedding(c->bf16, sa, st);
  launch_commit(d_conf, d_argmax, n_seq, block_len, block_len, 0, d_block_tokens, d_mask, commit_rule(decode), d_n_committed,
                nullptr, nullptr, st, next_live, steps);
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_step_smooth(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                       const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                       const dinfer_decode* decode, float alpha, float* d_delta, void* d_scratch, size_t scratch_bytes,
                       float* d_conf, int32_t* d_argmax, int32_t* d_n_committed, void* stream) {
  return smooth_impl(c, n_seq, block_len, d_block_tokens, d_mask, d_prefix_len, d_page_table, pt_stride, decode, alpha,
                     d_delta, d_scratch, scratch_bytes, d_conf, d_argmax, d_n_committed, (hipStream_t)stream, nullptr,
                     nullptr, nullptr);
}

int dinfer_step_smooth_static(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                              const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                              const dinfer_decode* decode, float alpha, float* d_delta, float* d_conf, int32_t* d_argmax,
                              int32_t* d_n_committed, void* stream) {
  int rc = check_block_args(c, n_seq, block_len, d_block_tokens, d_prefix_len, d_page_table, pt_stride);
  if (rc != DINFER_OK) return rc;
  const size_t need = dinfer_smooth_scratch_bytes(&c->cfg, n_seq * block_len);
  if (need == 0) return fail(DINFER_EINVAL, "bad configuration");
  if (need > (size_t)DINFER_STATIC_SCRATCH_BYTES)
    return fail(DINFER_ENOSPACE, "%d block tokens of a %d-id vocabulary need %zu bytes of scratch; the static scratch holds %zu",
                n_seq * block_len, c->cfg.vocab, need, (size_t)DINFER_STATIC_SCRATCH_BYTES);
  void* p = nullptr;
  int dev = -1;
  if ((rc = static_scratch_of_current_device(&p, &dev)) != DINFER_OK) return rc;   // a look-up: resolved at dinfer_create
  if (dev != c->device)
    return fail(DINFER_EINVAL, "the context was created on device %d, the current device is %d", c->device, dev);
  return dinfer_step_smooth(c, n_seq, block_len, d_block_tokens, d_mask, d_prefix_len, d_page_table, pt_stride, decode,
                            alpha, d_delta, p, (size_t)DINFER_STATIC_SCRATCH_BYTES, d_conf, d_argmax, d_n_committed,
                            stream);
}

int dinfer_step_credit(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                       const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                       const dinfer_decode* decode, const dinfer_credit* credit, int32_t* d_credit_ids,
                       float* d_credit_val, int32_t* d_credit_n, float* d_conf, int32_t* d_argmax,
                       int32_t* d_n_committed, void* stream) {
  int rc = check_block_args(c, n_seq, block_len, d_block_tokens, d_prefix_len, d_page_table, pt_stride);
  if (rc != DINFER_OK) return rc;
  if (!d_mask || !decode || !d_conf || !d_argmax || !d_n_committed) return fail(DINFER_EINVAL, "null pointer");
  if (!credit || !d_credit_ids || !d_credit_val || !d_credit_n) return fail(DINFER_EINVAL, "null pointer");
  if ((rc = check_decode(decode)) != DINFER_OK) return rc;
  if (!(credit->alpha >= 0.f) || !(credit->beta >= 0.f && credit->beta <= 1.f) ||
      !(credit->gamma > 0.f && credit->gamma <= 1.f))
    return fail(DINFER_EINVAL, "credit parameters: alpha >= 0, 0 <= beta <= 1, 0 < gamma <= 1");
  hipStream_t st = (hipStream_t)stream;
  rc = forward(c, uniform_span(n_seq, block_len), d_block_tokens, d_prefix_len, d_page_table, pt_stride, true, st);
  if (rc != DINFER_OK) return rc;
  const dinfer_config& f = c->cfg;
  const int T = n_seq * block_len;
  float* stats = at<float>(c->ws, c->wsm.lm_stats);
  LmArgs la{c->weights + c->wm.lm_head, c->ws + c->wsm.xn,
            RowNorm{at<float>(c->ws, c->wsm.ssq_a), c->last_n_ssq, f.rms_eps}, T, f.hidden, f.vocab, f.logit_scale,
            at<float>(c->ws, c->wsm.lm_part), nullptr};
  {
    StageTimer tm(c, DINFER_STAGE_LM_HEAD, st);
    launch_lm_head(c->bf16, la, st);
  }
  launch_lm_merge(la.part, lm_head_parts(f.vocab, T), T, d_conf, d_argmax, stats, st);
  launch_credit(c->bf16, la.w, la.xn, la.norm, T, f.hidden, f.vocab, f.logit_scale, stats, d_mask, block_len,
                credit->alpha, credit->beta, credit->gamma, d_credit_ids, d_credit_val, d_credit_n, d_conf, d_argmax, st);
  launch_commit(d_conf, d_argmax, n_seq, block_len, block_len, 0, d_block_tokens, d_mask, commit_rule(decode), d_n_committed, nullptr, nullptr, st);
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_step_vicinity(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t look_back, int32_t* d_block_tokens,
                         const int32_t* d_vicinity_tokens, uint64_t* d_mask, const int32_t* d_prefix_len,
                         const int32_t* d_page_table, int32_t pt_stride, const dinfer_decode* decode, float* d_conf,
                         int32_t* d_argmax, int32_t* d_n_committed, void* stream) {
  int rc = check_block_args(c, n_seq, block_len, d_block_tokens, d_prefix_len, d_page_table, pt_stride);
  if (rc != DINFER_OK) return rc;
  if (!d_mask || !decode || !d_conf || !d_argmax || !d_n_committed) return fail(DINFER_EINVAL, "null pointer");
  if ((rc = check_decode(decode)) != DINFER_OK) return rc;
  if (look_back < 0 || look_back > 64) return fail(DINFER_EINVAL, "look_back %d outside [0, 64]", look_back);
  if (look_back > 0 && !d_vicinity_tokens) return fail(DINFER_EINVAL, "null pointer");
  const int run = look_back + block_len;
  if ((int64_t)n_seq * run > c->max_tokens)
    return fail(DINFER_ENOSPACE, "n_seq*(look_back+block_len) %d exceeds max_tokens %d", n_seq * run, c->max_tokens);
  // the run of look_back + block_len positions must fit the rotary table and the page-table row like a block does
  if (run > c->cfg.max_pos || (int64_t)pt_stride * PAGE < run)
    return fail(DINFER_ENOSPACE, "look_back+block_len %d exceeds max_pos %d or the page-table row (%d positions)", run,
                c->cfg.max_pos, pt_stride * PAGE);
  hipStream_t st = (hipStream_t)stream;
  const dinfer_config& f = c->cfg;
  int32_t* run_tokens = at<int32_t>(c->ws, c->wsm.run_tokens);
  int32_t* run_base = at<int32_t>(c->ws, c->wsm.run_base);
  launch_vicinity_pack(n_seq, block_len, look_back, d_block_tokens, d_vicinity_tokens, d_prefix_len, run_tokens, run_base,
                       st);
  rc = forward(c, uniform_span(n_seq, run), run_tokens, run_base, d_page_table, pt_stride, true, st);
  if (rc != DINFER_OK) return rc;
  const int T = n_seq * run;
  float* conf_rows = at<float>(c->ws, c->wsm.conf);
  int32_t* argmax_rows = at<int32_t>(c->ws, c->wsm.argmax);
  LmArgs la{c->weights + c->wm.lm_head, c->ws + c->wsm.xn,
            RowNorm{at<float>(c->ws, c->wsm.ssq_a), c->last_n_ssq, f.rms_eps}, T, f.hidden, f.vocab, f.logit_scale,
            at<float>(c->ws, c->wsm.lm_part), nullptr};
  {
    StageTimer tm(c, DINFER_STAGE_LM_HEAD, st);
    launch_lm_head(c->bf16, la, st);
  }
  launch_lm_merge(la.part, lm_head_parts(f.vocab, T), T, conf_rows, argmax_rows, nullptr, st);
  launch_commit(conf_rows, argmax_rows, n_seq, block_len, run, look_back, d_block_tokens, d_mask, commit_rule(decode), d_n_committed, d_conf, d_argmax, st);
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_refresh_block(dinfer_ctx* c, int32_t n_seq, int32_t block_len, const int32_t* d_block_tokens,
                         int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride, void* stream) {
  int rc = check_block_args(c, n_seq, block_len, d_block_tokens, d_prefix_len, d_page_table, pt_stride);
  if (rc != DINFER_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  rc = forward(c, uniform_span(n_seq, block_len), d_block_tokens, d_prefix_len, d_page_table, pt_stride, false, st);
  if (rc != DINFER_OK) return rc;
  launch_add_i32(d_prefix_len, n_seq, block_len, st);
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_generate_block(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                          const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                          const dinfer_decode* decode, float* d_conf, int32_t* d_argmax, int32_t* d_n_committed,
                          int32_t max_steps, int32_t h_masked_hint, int32_t steps_per_wait, int32_t* h_steps_taken,
                          void* stream) {
  if (max_steps < 1 || max_steps > MAX_LOOP_STEPS) return fail(DINFER_EINVAL, "max_steps %d outside [1, %d]", max_steps, MAX_LOOP_STEPS);
  if (!decode) return fail(DINFER_EINVAL, "decode is null");
  if (steps_per_wait < 0) return fail(DINFER_EINVAL, "steps_per_wait %d", steps_per_wait);
  hipStream_t st = (hipStream_t)stream;
  int steps = 0;
  if (decode->fixed_k > 0 && h_masked_hint > 0) {
    int n = (h_masked_hint + decode->fixed_k - 1) / decode->fixed_k;
    if (n > max_steps) n = max_steps;
    for (; steps < n; ++steps) {
      int rc = dinfer_step(c, n_seq, block_len, d_block_tokens, d_mask, d_prefix_len, d_page_table, pt_stride, decode,
                           d_conf, d_argmax, d_n_committed, stream);
      if (rc != DINFER_OK) return rc;
    }
  } else {
    // The number of steps depends on the data.  Steps are enqueued steps_per_wait at a time without waiting; the
    // device keeps one "still needed" word per step, raised by the decoder of the step before it, and a step whose
    // word is zero costs only the launches of its kernels.  The host waits once per batch to read the word of the
    // next step and the number of steps that ran.
    if (!c || !d_mask || n_seq < 1 || n_seq > c->max_seqs) return fail(DINFER_EINVAL, "bad argument");
    const int batch = steps_per_wait > 0 ? steps_per_wait : 1;
    int32_t* flags = at<int32_t>(c->ws, c->wsm.loop_flags);
    int32_t* d_steps = at<int32_t>(c->ws, c->wsm.loop_steps);
    int32_t* h_words = reinterpret_cast<int32_t*>(c->h_mask_pinned);
    launch_loop_begin(d_mask, n_seq, flags, max_steps + 1, d_steps, st);
    int enq = 0;
    while (enq < max_steps) {
      const int n = batch < max_steps - enq ? batch : max_steps - enq;
      for (int i = 0; i < n; ++i) {
        int rc = step_impl(c, n_seq, block_len, d_block_tokens, d_mask, d_prefix_len, d_page_table, pt_stride, decode,
                           d_conf, d_argmax, d_n_committed, st, flags + enq + i, flags + enq + i + 1, d_steps);
        if (rc != DINFER_OK) return rc;
      }
      enq += n;
      HIP_TRY(hipMemcpyAsync(h_words, flags + enq, sizeof(int32_t), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipMemcpyAsync(h_words + 1, d_steps, sizeof(int32_t), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      steps = h_words[1];
      if (h_words[0] == 0) break;
    }
  }
  if (h_steps_taken) *h_steps_taken = steps;
  return DINFER_OK;
}

int dinfer_generate_block_smooth(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens,
                                 uint64_t* d_mask, const int32_t* d_prefix_len, const int32_t* d_page_table,
                                 int32_t pt_stride, const dinfer_decode* decode, const dinfer_smooth_schedule* sched,
                                 float* d_delta, void* d_scratch, size_t scratch_bytes, float* d_conf, int32_t* d_argmax,
                                 int32_t* d_n_committed, int32_t max_steps, int32_t steps_per_wait,
                                 int32_t* h_steps_taken, void* stream) {
  if (max_steps < 1 || max_steps > MAX_LOOP_STEPS) return fail(DINFER_EINVAL, "max_steps %d outside [1, %d]", max_steps, MAX_LOOP_STEPS);
  if (!c || !decode || !sched || !d_mask) return fail(DINFER_EINVAL, "null argument");
  if (n_seq < 1 || n_seq > c->max_seqs) return fail(DINFER_EINVAL, "n_seq %d outside [1, %d]", n_seq, c->max_seqs);
  if (steps_per_wait < 0) return fail(DINFER_EINVAL, "steps_per_wait %d", steps_per_wait);
  if (decode->fixed_k > 0) return fail(DINFER_EINVAL, "the threshold schedule needs a threshold decoder (fixed_k == 0)");
  if (!(sched->alpha_init >= 0.f) || !(sched->alpha_growth >= 0.f) || !(sched->alpha_preset >= sched->alpha_init))
    return fail(DINFER_EINVAL, "schedule: 0 <= alpha_init <= alpha_preset, alpha_growth >= 0");
  if (!(sched->threshold_decay >= 0.f) || !(sched->threshold_start >= decode->threshold) || !(sched->threshold_start <= 1.f))
    return fail(DINFER_EINVAL, "schedule: decode->threshold <= threshold_start <= 1, threshold_decay >= 0");
  hipStream_t st = (hipStream_t)stream;
  const int batch = steps_per_wait > 0 ? steps_per_wait : 1;
  int32_t* flags = at<int32_t>(c->ws, c->wsm.loop_flags);
  int32_t* d_steps = at<int32_t>(c->ws, c->wsm.loop_steps);
  int32_t* h_words = reinterpret_cast<int32_t*>(c->h_mask_pinned);
  launch_loop_begin(d_mask, n_seq, flags, max_steps + 1, d_steps, st);
  int enq = 0, steps = 0;
  while (enq < max_steps) {
    const int n = batch < max_steps - enq ? batch : max_steps - enq;
    for (int i = 0; i < n; ++i) {
      // Step t of the block (t = 0 first).  Steps only ever get skipped once every mask is empty, so the index
      // of an enqueued step is also the number of steps that ran before it.
      const int t = enq + i;
      dinfer_decode d = *decode;
      const float tau = sched->threshold_start - sched->threshold_decay * (float)t;
      d.threshold = tau > decode->threshold ? tau : decode->threshold;
      if (d.hierarchical && d.lower_bound > d.threshold) d.lower_bound = d.threshold;
      float alpha = 0.f;   // the first step has nothing retained
      if (t > 0) {
        alpha = sched->alpha_init + sched->alpha_growth * (float)(t - 1);
        if (alpha > sched->alpha_preset) alpha = sched->alpha_preset;
      }
      int rc = smooth_impl(c, n_seq, block_len, d_block_tokens, d_mask, d_prefix_len, d_page_table, pt_stride, &d, alpha,
                           d_delta, d_scratch, scratch_bytes, d_conf, d_argmax, d_n_committed, st, flags + t,
                           flags + t + 1, d_steps);
      if (rc != DINFER_OK) return rc;
    }
    enq += n;
    HIP_TRY(hipMemcpyAsync(h_words, flags + enq, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(h_words + 1, d_steps, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    steps = h_words[1];
    if (h_words[0] == 0) break;
  }
  if (h_steps_taken) *h_steps_taken = steps;
  return DINFER_OK;
}

int dinfer_commit(const float* d_conf, const int32_t* d_argmax, int32_t n_seq, int32_t block_len,
                  int32_t* d_block_tokens, uint64_t* d_mask, const dinfer_decode* decode, int32_t* d_n_committed,
                  void* stream) {
  if (!d_conf || !d_argmax || !d_block_tokens || !d_mask || !d_n_committed) return fail(DINFER_EINVAL, "null pointer");
  if (n_seq < 1 || block_len < 1 || block_len > 64) return fail(DINFER_EINVAL, "n_seq %d block_len %d", n_seq, block_len);
  int rc = check_decode(decode);
  if (rc != DINFER_OK) return rc;
  launch_commit(d_conf, d_argmax, n_seq, block_len, block_len, 0, d_block_tokens, d_mask, commit_rule(decode),
                d_n_committed, nullptr, nullptr, (hipStream_t)stream);
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_generate(dinfer_ctx* c, int32_t n_seq, int32_t block_len, int32_t n_blocks, int32_t* d_out,
                    int32_t* d_block_tokens, uint64_t* d_mask, int32_t* d_prefix_len, const int32_t* d_page_table,
                    int32_t pt_stride, const dinfer_decode* decode, int32_t eos_id, int32_t steps_per_wait,
                    int32_t* d_finished, float* d_conf, int32_t* d_argmax, int32_t* d_n_committed, int32_t* h_blocks_run,
                    void* stream) {
  int rc = check_block_args(c, n_seq, block_len, d_block_tokens, d_prefix_len, d_page_table, pt_stride);
  if (rc != DINFER_OK) return rc;
  if (!d_out || !d_mask || !d_finished || !d_conf || !d_argmax || !d_n_committed) return fail(DINFER_EINVAL, "null pointer");
  if (n_blocks < 1) return fail(DINFER_EINVAL, "n_blocks %d", n_blocks);
  if (eos_id >= c->cfg.vocab) return fail(DINFER_EINVAL, "eos_id %d outside the vocabulary", eos_id);
  if ((rc = check_decode(decode)) != DINFER_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  int32_t* d_count = at<int32_t>(c->ws, c->wsm.n_finished);
  int32_t* h_count = reinterpret_cast<int32_t*>(c->h_mask_pinned);
  int b = 0;
  for (; b < n_blocks; ++b) {
    launch_block_begin(n_seq, block_len, c->cfg.mask_id, eos_id, d_finished, b == 0, d_block_tokens, d_mask, st);
    rc = dinfer_generate_block(c, n_seq, block_len, d_block_tokens, d_mask, d_prefix_len, d_page_table, pt_stride, decode,
                               d_conf, d_argmax, d_n_committed, block_len, block_len, steps_per_wait, nullptr, stream);
    if (rc != DINFER_OK) return rc;
    rc = dinfer_refresh_block(c, n_seq, block_len, d_block_tokens, d_prefix_len, d_page_table, pt_stride, stream);
    if (rc != DINFER_OK) return rc;
    launch_block_end(n_seq, block_len, n_blocks, b, eos_id, d_block_tokens, d_out, d_finished, d_count, st);
    if (eos_id >= 0) {   // without an end-of-sequence id nothing can stop the loop: no wait at all
      HIP_TRY(hipMemcpyAsync(h_count, d_count, sizeof(int32_t), hipMemcpyDeviceToHost, st));
      HIP_TRY(hipStreamSynchronize(st));
      if (*h_count >= n_seq) {
        ++b;
        break;
      }
    }
  }
  launch_fill_blocks(n_seq, block_len, n_blocks, b, eos_id, d_out, st);
  HIP_TRY(hipGetLastError());
  if (h_blocks_run) *h_blocks_run = b;
  return DINFER_OK;
}

static int kv_copy(dinfer_ctx* c, bool to_pool, int32_t layer, const int32_t* d_page_row, int32_t first_pos,
                   int32_t n_pos, float* d_k, float* d_v, void* stream) {
  if (!c || !d_page_row || !d_k || !d_v) return fail(DINFER_EINVAL, "null argument");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(DINFER_EINVAL, "layer %d", layer);
  if (first_pos < 0 || n_pos < 1 || first_pos + n_pos > c->cfg.max_pos) return fail(DINFER_EINVAL, "position range");
  launch_kv_copy(c->bf16, to_pool, c->kv + (size_t)layer * c->kv_layer_bytes, c->geom, d_page_row, first_pos, n_pos, d_k,
                 d_v, (hipStream_t)stream);
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_kv_write(dinfer_ctx* c, int32_t layer, const int32_t* d_page_row, int32_t first_pos, int32_t n_pos,
                    const float* d_k, const float* d_v, void* stream) {
  return kv_copy(c, true, layer, d_page_row, first_pos, n_pos, const_cast<float*>(d_k), const_cast<float*>(d_v), stream);
}

int dinfer_kv_read(dinfer_ctx* c, int32_t layer, const int32_t* d_page_row, int32_t first_pos, int32_t n_pos,
                   float* d_k, float* d_v, void* stream) {
  return kv_copy(c, false, layer, d_page_row, first_pos, n_pos, d_k, d_v, stream);
}

int dinfer_stream_read(const void* d_buf, size_t bytes, float* d_sink, void* stream) {
  if (!d_buf || !d_sink) return fail(DINFER_EINVAL, "null argument");
  if (((uintptr_t)d_buf & 15) || bytes < (256u << 10)) return fail(DINFER_EINVAL, "buffer must be 16-byte aligned, >= 256 KiB");
  launch_stream_read(d_buf, bytes, d_sink, (hipStream_t)stream);
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_profile_every(dinfer_ctx* c, int32_t n_forwards) {
  if (!c) return fail(DINFER_EINVAL, "context is null");
  if (n_forwards < 1) return fail(DINFER_EINVAL, "profile every %d forwards", n_forwards);
  c->prof_every = n_forwards;
  return DINFER_OK;
}

int dinfer_profile_start(dinfer_ctx* c, int32_t stage) {
  if (!c) return fail(DINFER_EINVAL, "context is null");
  if (stage < 0 || stage >= DINFER_STAGE_COUNT) return fail(DINFER_EINVAL, "stage %d", stage);
  while (c->prof_ev.size() < 2 * PROF_MAX_LAUNCHES) {
    hipEvent_t e;
    HIP_TRY(hipEventCreate(&e));
    c->prof_ev.push_back(e);
  }
  c->prof_stage = stage;
  c->prof_n = 0;
  c->prof_fwd = 0;
  // the running totals of experts with rows (dinfer_debug_get 6) start over with the profile
  HIP_TRY(hipMemset(at<int32_t>(c->ws, c->wsm.off) + STAT_ACTIVE_SUM, 0, 2 * sizeof(int32_t)));
  return DINFER_OK;
}

int dinfer_profile_stop(dinfer_ctx* c, int32_t* n_launches, float* total_ms) {
  if (!c || !n_launches || !total_ms) return fail(DINFER_EINVAL, "null argument");
  if (c->prof_stage < 0) return fail(DINFER_EINVAL, "no profile running");
  float sum = 0.f;
  for (size_t i = 0; i < c->prof_n; ++i) {
    HIP_TRY(hipEventSynchronize(c->prof_ev[2 * i + 1]));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
    sum += ms;
  }
  *n_launches = (int32_t)c->prof_n;
  *total_ms = sum;
  c->prof_stage = -1;
  c->prof_n = 0;
  return DINFER_OK;
}

int dinfer_debug_logits(dinfer_ctx* c, int32_t n_rows, float* d_out, void* stream) {
  if (!c || !d_out) return fail(DINFER_EINVAL, "null argument");
  // the normalised-input planes are laid out for last_T rows: the kernel must be run over exactly those
  if (n_rows != c->last_T) return fail(DINFER_EINVAL, "n_rows %d is not the last forward's %d rows", n_rows, c->last_T);
  const dinfer_config& f = c->cfg;
  LmArgs la{c->weights + c->wm.lm_head, c->ws + c->wsm.xn,
            RowNorm{at<float>(c->ws, c->wsm.ssq_a), c->last_n_ssq, f.rms_eps}, n_rows, f.hidden, f.vocab, f.logit_scale,
            at<float>(c->ws, c->wsm.lm_part), d_out};
  launch_lm_head(c->bf16, la, (hipStream_t)stream);
  HIP_TRY(hipGetLastError());
  return DINFER_OK;
}

int dinfer_debug_get(dinfer_ctx* c, int32_t what, void* d_out, size_t bytes, void* stream) {
  if (!c || !d_out) return fail(DINFER_EINVAL, "null argument");
  const dinfer_config& f = c->cfg;
  const size_t T = (size_t)c->last_T;
  size_t off = 0, want = 0;
  switch (what) {
    case 0: off = c->wsm.x; want = T * f.hidden * 4; break;
    case 1: off = c->wsm.topk_idx; want = (size_t)f.n_layers * T * f.top_k * 4; break;
    case 2: off = c->wsm.topk_w; want = (size_t)f.n_layers * T * f.top_k * 4; break;
    case 3: off = c->wsm.cnt; want = (size_t)f.n_experts * 4; break;
    case 4: off = c->wsm.off; want = (size_t)(f.n_experts + 1) * 4; break;
    case 5: off = c->wsm.perm; want = T * f.top_k * 4; break;
    case 6: off = c->wsm.off + (size_t)STAT_ACTIVE_SUM * 4; want = 8; break;
    default: return fail(DINFER_EINVAL, "what %d", what);
  }
  if (bytes != want || want == 0) return fail(DINFER_EINVAL, "%zu bytes given, %zu expected", bytes, want);
  HIP_TRY(hipMemcpyAsync(d_out, c->ws + off, want, hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return DINFER_OK;
}

int dinfer_debug_single_slice(int32_t on) {
  set_single_slice(on != 0);
  return DINFER_OK;
}

int dinfer_debug_trace(int32_t unit, void* h_out, size_t bytes) {
  if (!h_out) return fail(DINFER_EINVAL, "null argument");
  const int r = unit == 0   ? trace_read_gemm(h_out, bytes)
                : unit == 1 ? trace_read_attention(h_out, bytes)
                : unit == 2 ? trace_read_wide(h_out, bytes)
                            : -2;
  if (r == -1) return fail(DINFER_EINVAL, "library built without DINFER_TRACE, or buffer too large");
  if (r != 0) return fail(DINFER_EINVAL, "trace read failed (%d)", r);
  return DINFER_OK;
}

}  // extern "C"
