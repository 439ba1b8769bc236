// Host-callable launchers of the dinfer kernels.  Every launcher only enqueues work on `st`; none waits.
// `bf16` selects the element type (false: float32) of weights, activations fed to the MFMAs and the KV pool.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.hpp"

namespace dinfer {

// The "is this step still needed" word of the forward being enqueued on this host thread (see step_is_dead in
// common.hpp): set by the step entry points around a forward, handed to every kernel by its launcher.
void set_live_word(const int32_t* d_live);
const int32_t* live_word();
// Test switch (process-wide): while on, no contraction shares a task's sum among workgroups -- projections, router
// and attention run with one K slice / key split, the expert down projection unfused.
void set_single_slice(bool on);
bool single_slice();

// ---- weight packing (pack.hip) ----
enum PackMode { PACK_ADJACENT = 0, PACK_ROPE_PAIR = 1, PACK_HALF0 = 2, PACK_HALF1 = 3 };
// src: [batch][N][K] row-major; dst: [batch][n_tasks][K/KS][2][64][16 B]
void launch_pack(bool bf16, const void* src, void* dst, int batch, int N, int K, int n_tasks, int mode,
                 int head_dim, hipStream_t st);
int64_t packed_bytes(bool bf16, int n_tasks, int K);
// src [V][H] row-major -> the packed layout of its transpose ([H] output features, contraction over V padded to Kpad)
void launch_pack_transposed(bool bf16, const void* src, void* dst, int V, int H, int Kpad, hipStream_t st);

// ---- forward pieces ----
struct FwdMeta {            // device arrays describing the tokens of one forward
  const int32_t* tok_seq;   // [T]
  const int32_t* tok_pos;   // [T] absolute position
  const int32_t* seq_nkeys; // [n_seq] keys visible to the sequence = base + its tokens in this forward
  const int32_t* qtile;     // [n_qtiles][3]: sequence, first packed token, valid rows
};

void launch_rope_table(float* cos_tab, float* sin_tab, int max_pos, int head_dim, float theta, hipStream_t st);
// Normalised-input planes: whoever produces a residual row x[t] also stores x[t] * gain (gain of the RMSNorm
// that follows; the row's 1/rms factor is NOT applied) as a k-major activation matrix [T][H] (act_index in
// common.hpp).  The consumers feed it to the matrix cores and apply 1/rms in their epilogues.
// Row statistics travel as shares of the row's sum of squares, ssq[n_ssq][T] (row_rinv in common.hpp): one share
// per 64-feature task where a projection epilogue produced the row, a single share from the kernels below.
struct RowNorm {
  const float* ssq;
  int n_ssq;
  float eps;
};
// x[t] = emb[token[t]];  ssq[t] = sum(x[t]^2);  xn[t] = planes of x[t] * gain
// Iteration smoothing: a position that is still masked (bit of its sequence's mask, uniform blocks of block_len
// tokens) is embedded as emb[token] + alpha * delta[t].  Pass null for a plain embedding.
// The launch also writes the forward's token bookkeeping (FwdMeta's arrays) from `span` and the sequences' first
// positions d_base (device, or null for 0): `limit` = positions a sequence may use (rotary table and page-table
// row); a first position that would leave it is pulled back so that no later kernel indexes outside its buffers.
struct SmoothIn {
  const float* delta;       // [T][H]
  float alpha;
  const uint64_t* mask;     // [n_seq]
  int block_len;
};
void launch_embed(bool bf16, const int32_t* tokens, const void* emb, int T, int H, int V, float* x,
                  float* ssq, const float* gain, void* xn, const SmoothIn* smooth, const SeqSpan& span,
                  const int32_t* d_base, int limit, int32_t* tok_seq, int32_t* tok_pos, int32_t* seq_nkeys,
                  int32_t* qtile, hipStream_t st);
// x[t] += sum_j topk_w[t][j] * O[t*k+j];  ssq[t] and xn[t] as above, of the updated row
void launch_combine(bool bf16, float* x, const float* O, const float* topk_w, int top_k,
                    int T, int H, float* ssq, const float* gain, void* xn, hipStream_t st);

// Cross-workgroup split-K scratch shared by the projections and the router (see gemm.hip): `part` holds the
// workgroup sums, `tickets` one arrival counter per (task, token group), all zero between launches.
int gemm_slices(bool bf16, int K, int T);   // workgroups that share one task's K range for T tokens

struct QkvArgs {
  const void* w;            // packed fused QKV
  const void* xn;           // [T][H] normalised-input planes (attention gain)
  RowNorm norm;             // statistics of the residual rows
  void* q;                  // [T][D] (hi / lo planes)
  int64_t q_plane;
  void* kv_layer;           // pool base of this layer
  KvGeom geom;
  FwdMeta meta;
  const int32_t* page_table;
  int pt_stride;
  const float* cos_tab;
  const float* sin_tab;
  int T, H;
  float* part;
  int32_t* tickets;
};
void launch_qkv(bool bf16, const QkvArgs& a, hipStream_t st);

// Queries are stored row-major as Planes<E>::N planes (see common.hpp), q_plane elements apart; the attention
// output is a k-major activation matrix [T][D].
// Weights of a later split-K launch, brought into the L2s ahead of time.  Lines that ordinary loads bring into a
// die's L2 stay there while the big weight streams pass (non-temporal loads do not displace them), and a launch's
// workgroup i always runs on die i mod 8: so while attention runs with a few workgroups (batch 1: 16 of them on a
// chip of 256 compute units), extra workgroups of the same launch read, with ordinary loads, exactly the bytes that
// the output projection's workgroups on the same die will stream, and that launch finds them in its L2.
// Region i = [base + i * region_bytes, + region_bytes) is what workgroup i of the later launch streams; it is fetched
// by a workgroup whose index in its own launch is congruent to i modulo 8.
// (Measured at batch 1: output projection 8.06 -> 7.24 us, attention 11.2 -> 11.4.  The same for the next layer's
// QKV weights, 3 MB per die fetched beside the router: QKV 11.9 -> 10.5 us, but attention, the router and the LM
// head lose 1.1, 1.5 and 4 us to the lines it displaces; not done.)
struct L2Prefetch {
  const char* base;        // null: nothing to fetch
  uint32_t region_bytes;   // a multiple of 16
  int32_t n_regions;
};
// The plan for the split-K form of the output projection over T tokens (base null where it takes another form).
L2Prefetch oproj_prefetch_plan(bool bf16, const void* w, int D, int H, int T);

struct AttnArgs {
  const void* q;            // [T][D]
  int64_t q_plane;
  const void* kv_layer;
  KvGeom geom;
  FwdMeta meta;
  const int32_t* page_table;
  int pt_stride;
  int n_qtiles, n_splits;
  float* part;              // partial results, see attention.hip
  int32_t* tickets;         // [n_qtiles][n_heads] arrival counters, zero between launches
  void* out;                // [T][D] k-major
  int T;
  L2Prefetch pf;            // fetched by extra workgroups of the launch when it has few of its own (see L2Prefetch)
};
size_t attn_part_floats(int n_qtiles, int n_heads, int n_splits, int head_dim);
void launch_attention(bool bf16, const AttnArgs& a, hipStream_t st);

// x += a . Wo^T; the new rows also leave as normalised-input planes (FFN gain) and, per 64-feature task, their
// share of the row's sum of squares: ssq[H/64][T].
struct OprojArgs {
  const void* w;            // packed output projection
  const void* a;            // [T][D] attention output, k-major
  float* x;                 // [T][H] residual stream, updated in place
  const float* gain;        // [H] FFN norm gain
  void* xn;
  float* ssq;
  int T, D, H;
  float* part;
  int32_t* tickets;
};
void launch_oproj(bool bf16, const OprojArgs& a, hipStream_t st);

// Iteration smoothing: delta[t] = softmax(logits[t]) . W_emb for the rows of positions that are still masked.
//   probs: scratch for the probabilities as a k-major activation matrix [T][Kpad]; logits [T][V] float32;
//   stats [T][2] = (largest logit, sum exp(z - max)) of every row; w_emb_t: launch_pack_transposed's layout.
constexpr int SMOOTH_SLICES = 16;     // workgroups that share the vocabulary range of one 64-column task
int smooth_kpad(bool bf16, int V);    // the vocabulary rounded up so that every wave of every slice gets whole bursts
struct SmoothArgs {
  const void* w_emb_t;
  const float* logits;
  const float* stats;
  void* probs;
  const uint64_t* mask;
  int block_len;
  float* delta;             // [T][H] in/out
  int T, H, V;
  float* part;
  int32_t* tickets;
};
void launch_expected_embedding(bool bf16, const SmoothArgs& a, hipStream_t st);
void launch_prob_planes(bool bf16, const float* logits, const float* stats, int T, int V, int Kpad, void* probs,
                        hipStream_t st);
// Router logits on the matrix cores + softmax + top-k (ties to the lower expert id, weights renormalised when
// norm_topk); rinv[t] from the sums of squares above; for T <= 64 also the token->expert permutation
// (otherwise launch_permute is issued behind it).
struct RouterArgs {
  const void* w;            // packed router weights (one task)
  const void* xn;           // [T][H] normalised-input planes (FFN gain)
  const float* ssq;         // [H/64][T]
  float eps;
  int T, H, E, top_k, norm_topk;
  float* rinv;              // [T] out: 1/rms of the residual rows
  int32_t* topk_idx;        // [T][top_k] out
  float* topk_w;            // [T][top_k] out
  int32_t* cnt;             // [E], off [E+1], perm [T*top_k], pos_of_pair [T*top_k]: out
  int32_t* off;
  int32_t* perm;
  int32_t* pos_of_pair;
  int32_t* work;            // [1 + expert_work_items]: work list of the many-token expert GEMMs (T > 64 only)
  float* part;
  int32_t* tickets;
};
void launch_router(bool bf16, const RouterArgs& a, hipStream_t st);
void launch_permute(const int32_t* topk_idx, int n_pairs, int E, int32_t* cnt, int32_t* off, int32_t* perm,
                    int32_t* pos_of_pair, int32_t* work, hipStream_t st);
// Work items (expert, group of 128 rows) the many-token expert GEMMs can be handed for n_pairs routed pairs.
inline int expert_work_items(int E, int n_pairs) { return E + n_pairs / (4 * TILE); }
int permute_max_pairs();      // most (token, slot) pairs one forward may route
bool configure_permute();

struct ExpertArgs {
  const void* w_gate_up;    // packed [E][I/32 tasks]
  const void* w_down;       // packed [E][H/64 tasks]
  const void* xn;           // [T][H] normalised-input planes (FFN gain)
  const float* rinv;        // [T]
  void* y;                  // [T*k][I] k-major
  float* o;                 // [T*k][H], row = token*top_k + slot (many-token form only)
  const int32_t* cnt;
  const int32_t* off;
  const int32_t* perm;
  const int32_t* work;      // see RouterArgs
  int T, H, I, E, top_k;
  // at most 32 tokens: the down projection is fused with the combine (launch_expert_down_fused); the expert
  // intermediate then carries the routing weight, taken from topk_w [T][top_k] (null: not applied)
  const float* topk_w;
  const int32_t* topk_idx;  // [T][top_k]
  const int32_t* pos_of_pair;
};
void launch_expert_gate_up(bool bf16, const ExpertArgs& a, hipStream_t st);   // picks the form by a.T
void launch_expert_down(bool bf16, const ExpertArgs& a, hipStream_t st);
// x += sum over a token's experts of (weighted intermediate) . Wd^T, then as launch_oproj: normalised-input planes
// with the gain of the norm that follows, sums of squares per task.  At most 32 tokens (one token tile).
void launch_expert_down_fused(bool bf16, const ExpertArgs& a, const OprojArgs& res, hipStream_t st);
int down_fused_slices();      // workgroups that share one task's sum (workspace sizing)
void launch_expert_gate_up_wide(bool bf16, const ExpertArgs& a, hipStream_t st);   // many-token forms (wide.hip)
void launch_expert_down_wide(bool bf16, const ExpertArgs& a, hipStream_t st);

struct LmArgs {
  const void* w;            // packed LM head
  const void* xn;           // [T][H] normalised-input planes (final gain)
  RowNorm norm;             // statistics of the residual rows
  int T, H, V;
  float scale;
  float* part;              // [lm_head_parts(V, T)][T][4]: max, sum-exp, argmax bits, unused
  float* logits_out;        // debug: [T][V] or null
  const int32_t* rows = nullptr;   // null: every row.  Else [1 + T]: rows[0] = n, rows[1 .. n] = the token rows to take,
                                   // ascending (forwards of more than 64 tokens only; smaller ones take every row)
};
// rows[0] = number of undecided positions over all sequences, rows[1 ..] = their token rows n_seq-major, ascending.
void launch_lm_rows(const uint64_t* mask, int n_seq, int block_len, int32_t* rows, hipStream_t st);
int lm_head_waves(int V);          // upper bound of partials per token row (workspace sizing)
int lm_head_parts(int V, int T);   // partials per token row launch_lm_head writes for T tokens
void launch_lm_head(bool bf16, const LmArgs& a, hipStream_t st);        // picks the form by a.T
void launch_lm_head_wide(bool bf16, const LmArgs& a, hipStream_t st);
int lm_head_wide_parts(int V);
// stats (may be null): [T][2] = the row's largest logit and sum exp(z - max)
// mask (may be null) with block_len: rows of decided positions are left alone.
void launch_lm_merge(const float* part, int n_lm_waves, int T, float* conf, int32_t* argmax, float* stats,
                     hipStream_t st, const uint64_t* mask = nullptr, int block_len = 0);
// Credit decoding of the masked rows: conf / argmax hold the plain values on entry and the enhanced ones on return.
void launch_credit(bool bf16, const void* w_lm, const void* xn, RowNorm norm, int T, int H, int V, float scale,
                   const float* stats, const uint64_t* mask, int block_len, float alpha, float beta, float gamma,
                   int32_t* cred_ids, float* cred_val, int32_t* cred_n, float* conf, int32_t* argmax, hipStream_t st);
// conf / argmax: one row per forward token, position i of sequence s at row s*row_stride + row_off + i;
// conf_out / argmax_out (may be null): the block's values, compact [n_seq][block_len].
// rule: threshold / fixed_k as in the decoder settings of the C interface; hier != 0 selects the hierarchical
// rule with lower boundary tau_low.
struct CommitRule {
  float threshold;
  int fixed_k;
  int hier;
  float tau_low;
};
// next_live / steps (may be null): see launch_loop_begin.
void launch_commit(const float* conf, const int32_t* argmax, int n_seq, int block_len, int row_stride, int row_off,
                   int32_t* tokens, uint64_t* mask, CommitRule rule, int32_t* n_committed, float* conf_out,
                   int32_t* argmax_out, hipStream_t st, int32_t* next_live = nullptr, int32_t* steps = nullptr);
// Loop of steps enqueued without waiting for the masks: step i runs only if flags[i] != 0 (set_live_word), its
// decoder raises flags[i + 1] if a masked position remains and adds one to steps[0].
void launch_loop_begin(const uint64_t* mask, int n_seq, int32_t* flags, int n_flags, int32_t* steps, hipStream_t st);
// Generation loop over blocks: start of a block (ids = mask_id and a full mask, or eos_id and an empty mask for a
// finished sequence; `first` clears the finished flags instead of reading them); end of a block (copy into out[s][block_index], mark sequences whose block holds eos_id,
// count the finished ones into n_finished[0]); fill of the blocks from first_block on with eos_id.
void launch_block_begin(int n_seq, int block_len, int mask_id, int eos_id, int32_t* finished, bool first,
                        int32_t* block_tokens, uint64_t* mask, hipStream_t st);
void launch_block_end(int n_seq, int block_len, int n_blocks, int block_index, int eos_id, const int32_t* block_tokens,
                      int32_t* out, int32_t* finished, int32_t* n_finished, hipStream_t st);
void launch_fill_blocks(int n_seq, int block_len, int n_blocks, int first_block, int eos_id, int32_t* out,
                        hipStream_t st);
void launch_vicinity_pack(int n_seq, int block_len, int look_back, const int32_t* block_tokens,
                          const int32_t* vicinity_tokens, const int32_t* prefix_len, int32_t* run_tokens,
                          int32_t* run_base, hipStream_t st);
void launch_add_i32(int32_t* a, int n, int v, hipStream_t st);

void launch_kv_copy(bool bf16, bool to_pool, void* kv_layer, KvGeom geom, const int32_t* page_row, int first_pos,
                    int n_pos, float* k, float* v, hipStream_t st);

void launch_stream_read(const void* buf, size_t bytes, float* sink, hipStream_t st);

bool configure_kernels();     // one-time function attributes (dynamic LDS limits); false if the runtime refuses
bool configure_attention();
bool configure_wide();

// In-kernel phase timestamps of builds with -DDINFER_TRACE (see common.hpp); return -1 in ordinary builds.
int trace_read_gemm(void* h_out, size_t bytes);
int trace_read_attention(void* h_out, size_t bytes);
int trace_read_wide(void* h_out, size_t bytes);

}  // namespace dinfer
