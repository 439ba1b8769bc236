/*
 * dinfer: the block-denoising hot path of diffusion-LLM inference on one MI355X (gfx950).
 *
 * One call of dinfer_step is one iteration of the inner loop of the paper's Algorithm 1 (blockwise dLLM
 * inference): a model forward on the active block with a KV cache (bidirectional attention of the block
 * over the cached prefix plus the block itself, Section 2), then the decoder (threshold decoding, Section 2,
 * with a commit-at-least-one fallback so that the loop of Algorithm 1 terminates).  dinfer_generate_block
 * is that inner loop; dinfer_refresh_block is the cache update of a fully decoded block (Section 2,
 * "KV-cache management"); dinfer_prefill builds the prompt's cache.
 *
 * Conventions for every entry point
 *  - All `d_` pointers are DEVICE pointers, `h_` pointers are HOST pointers.  The caller owns every buffer;
 *    the library allocates no device memory and keeps only the pointers given to dinfer_create.
 *  - `stream` is a hipStream_t passed as void*; work is enqueued on it and the call returns without waiting
 *    (dinfer_generate_block in threshold mode waits once per batch of steps, see there).  Outputs are valid
 *    after the caller synchronises the stream.
 *  - Return value: 0 on success, a negative DINFER_E* code otherwise.  Nothing is launched when an argument
 *    is rejected.  dinfer_last_error() returns a thread-local description of the last failure.
 *  - Calls on one context must not overlap: the workspace is shared state.
 *
 * Model: pre-norm transformer, RMSNorm, rotary embedding (rotate-half pairing), multi-head attention,
 * softmax top-k router over SwiGLU experts, untied embedding / LM head.  Limits: head_dim 64 or 128,
 * hidden, n_heads*head_dim and moe_inter multiples of 64, n_experts <= 64, top_k <= 8, block_len <= 64.
 */
#ifndef DINFER_H
#define DINFER_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { DINFER_F32 = 0, DINFER_BF16 = 1 };

enum {
  DINFER_OK = 0,
  DINFER_EINVAL = -1,      /* null pointer, size or shape out of range */
  DINFER_EUNSUPPORTED = -2,/* a shape the kernels are not built for */
  DINFER_ENOSPACE = -3,    /* workspace, page table or KV pool too small */
  DINFER_EHIP = -4         /* a HIP call failed; see dinfer_last_error */
};

/* Tensor ids for dinfer_set_tensor.  Every matrix is given row-major as [out_features][in_features] in the
 * configuration's dtype; gains are float32. */
enum {
  DINFER_T_EMB = 0,        /* [vocab][hidden] */
  DINFER_T_LM_HEAD = 1,    /* [vocab][hidden] */
  DINFER_T_FINAL_GAIN = 2, /* [hidden] float32 */
  DINFER_T_ATTN_GAIN = 3,  /* [hidden] float32, per layer */
  DINFER_T_WQ = 4,         /* [n_heads*head_dim][hidden], per layer */
  DINFER_T_WK = 5,
  DINFER_T_WV = 6,
  DINFER_T_WO = 7,         /* [hidden][n_heads*head_dim], per layer */
  DINFER_T_FFN_GAIN = 8,   /* [hidden] float32, per layer */
  DINFER_T_ROUTER = 9,     /* [n_experts][hidden], per layer */
  DINFER_T_GATE = 10,      /* [n_experts][moe_inter][hidden], per layer */
  DINFER_T_UP = 11,        /* [n_experts][moe_inter][hidden], per layer */
  DINFER_T_DOWN = 12,      /* [n_experts][hidden][moe_inter], per layer */
  DINFER_T_COUNT = 13
};

typedef struct dinfer_config {
  int32_t n_layers, hidden, n_heads, head_dim, n_experts, top_k, moe_inter, vocab;
  int32_t dtype;      /* DINFER_F32 or DINFER_BF16: storage of weights, activations fed to the matrix cores
                         and the KV cache; accumulation is always float32 */
  int32_t page_size;  /* tokens per KV page; must be 16 */
  int32_t mask_id;    /* id that marks an undecided position (Algorithm 1) */
  int32_t norm_topk;  /* 1: the k selected router probabilities are renormalised to sum to 1 */
  int32_t max_pos;    /* positions 0..max_pos-1 may be used (size of the rotary table) */
  float rms_eps, rope_theta, logit_scale;
} dinfer_config;

/* Decoder settings.  fixed_k == 0: commit every masked position whose confidence is at or above
 * `threshold`, or the single most confident one if none is.  fixed_k > 0: commit the fixed_k most confident
 * masked positions (all that remain if fewer).  Ties go to the lower position.
 *
 * hierarchical != 0 (with fixed_k == 0) selects hierarchical decoding (Appendix "Hierarchical decoding"; the
 * experiments use threshold 0.92 and lower boundary 0.62).  The paper describes it in prose; this library takes it
 * as: (1) every masked position at or above `threshold` is committed; (2) in every maximal run of consecutive
 * masked positions in which (1) committed nothing, the position closest to the centre of the run among those at
 * or above `lower_bound` is committed (at equal distance the more confident one, then the lower position), so
 * that runs are split near their middle and the next step works on the halves; (3) if nothing was committed at
 * all, the single most confident masked position is.  lower_bound <= threshold. */
typedef struct dinfer_decode {
  float threshold;
  int32_t fixed_k;
  int32_t hierarchical;
  float lower_bound;
  int32_t skip_decided;   /* dinfer_step, dinfer_generate_block, dinfer_generate: 1 = confidence and candidate id are
                             worked out only for the positions that were undecided when the step began (the only
                             ones the decoder reads); the d_conf / d_argmax entries of the others are left as they
                             were.  With more than 64 tokens the LM head then skips the decided rows' matrix work.
                             The other step variants ignore the field. */
} dinfer_decode;

typedef struct dinfer_ctx dinfer_ctx;

/* Sizes of the three device buffers the caller must allocate (256-byte aligned).  0 on a bad config. */
size_t dinfer_weights_bytes(const dinfer_config* cfg);
size_t dinfer_kv_bytes(const dinfer_config* cfg, int32_t n_pages);
/* max_seqs <= 64 sequences per call, max_tokens = most tokens one forward processes over all sequences
 * (the block for a step, the prompt for a prefill); max_tokens * top_k may not exceed 65535 routed pairs. */
size_t dinfer_workspace_bytes(const dinfer_config* cfg, int32_t max_seqs, int32_t max_tokens);

/* Validates the configuration, records the buffers, builds the rotary table in the workspace (enqueued on
 * `stream`).  The KV pool is laid out by the library; its contents are opaque (dinfer_kv_read/_write move
 * rows in and out).  *out is freed by dinfer_destroy (host memory only). */
int dinfer_create(const dinfer_config* cfg, void* d_weights, size_t weights_bytes, void* d_kv_pool,
                  int32_t n_pages, void* d_workspace, size_t workspace_bytes, int32_t max_seqs,
                  int32_t max_tokens, void* stream, dinfer_ctx** out);
void dinfer_destroy(dinfer_ctx* ctx);
const char* dinfer_last_error(void);

/* Copies one tensor (layer ignored for the three global ones) from `d_src`, row-major as listed above, into
 * the library's packed layout inside d_weights.  `bytes` must equal the tensor's size. */
int dinfer_set_tensor(dinfer_ctx* ctx, int32_t tensor_id, int32_t layer, const void* d_src, size_t bytes,
                      void* stream);

/* Prompt prefill: a bidirectional forward over each sequence's prompt alone, writing K,V of positions
 * 0..len-1 into the pages of its page-table row.  (The paper does not describe prefill for a diffusion model; this
 * is the reading taken here: the prompt attends to itself only, since the blocks after it do not exist yet.)  d_tokens: the prompts back to back (sum of lens);
 * h_lens: [n_seq] on the host; d_page_table: [n_seq][pt_stride] page ids. */
int dinfer_prefill(dinfer_ctx* ctx, int32_t n_seq, const int32_t* d_tokens, const int32_t* h_lens,
                   const int32_t* d_page_table, int32_t pt_stride, void* stream);

/* One denoising step (Algorithm 1, steps 3 and 4) for n_seq sequences, each with a block of block_len
 * positions that follows its d_prefix_len[s] cached positions.
 *   d_block_tokens [n_seq][block_len] in/out: mask_id at undecided positions; committed positions receive
 *                  their id.
 *   d_mask         [n_seq] in/out: bit i set = position i undecided.  Bits only ever get cleared.
 *   d_prefix_len   [n_seq] in: cached positions before the block.  Their K,V pages are only read.
 *   d_page_table   [n_seq][pt_stride]: page ids; must cover prefix_len + block_len positions.  K,V of the
 *                  block's positions are (re)written every step.
 *   d_conf, d_argmax [n_seq][block_len] out: confidence (largest softmax probability of the position's
 *                  logits) and candidate id (lowest id on ties) of every position.
 *   d_n_committed  [n_seq] out.
 * A sequence whose mask is empty commits nothing. */
int dinfer_step(dinfer_ctx* ctx, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                const dinfer_decode* decode, float* d_conf, int32_t* d_argmax, int32_t* d_n_committed,
                void* stream);

/* The decoder alone, on confidences and candidate ids the caller provides (all device pointers, [n_seq][block_len];
 * block_len <= 64, n_seq >= 1): applies `decode` to d_block_tokens / d_mask as the last stage of dinfer_step does
 * and writes d_n_committed [n_seq].  Needs no context. */
int dinfer_commit(const float* d_conf, const int32_t* d_argmax, int32_t n_seq, int32_t block_len,
                  int32_t* d_block_tokens, uint64_t* d_mask, const dinfer_decode* decode, int32_t* d_n_committed,
                  void* stream);

/* The step with iteration smoothing (Appendix "IterSmooth").  Positions that are still masked are not embedded as
 * the bare mask token: e_t[i] = e_mask + alpha * delta[i], where delta[i] = softmax(z_{t-1}[i]) . W_emb is the
 * expected INPUT embedding under the distribution the previous step predicted for the position (the embedding
 * matrix is not tied to the LM head).  alpha is this step's mixing weight min(alpha_init + alpha_growth * t,
 * alpha_preset), computed by the caller (0 on the first step of a block, or to ignore what was retained).
 *   d_delta   [n_seq][block_len][hidden] float32, in/out, kept by the caller across the steps of a block: on return
 *             the rows of the positions that were masked when the step began hold this step's expected embeddings;
 *             other rows are left alone.
 *   d_scratch device buffer of at least dinfer_smooth_scratch_bytes(cfg, n_seq * block_len) bytes, 256-byte
 *             aligned, contents irrelevant: this variant stores the block's logits there (the second contraction
 *             over the vocabulary needs normalised probabilities).
 * Any token count the context takes; above 64 tokens the contraction over the vocabulary runs in the many-token
 * form, in which every group of 64 tokens streams the whole embedding matrix again.  Everything else as in
 * dinfer_step. */
size_t dinfer_smooth_scratch_bytes(const dinfer_config* cfg, int32_t max_tokens);
int dinfer_step_smooth(dinfer_ctx* ctx, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                       const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                       const dinfer_decode* decode, float alpha, float* d_delta, void* d_scratch,
                       size_t scratch_bytes, float* d_conf, int32_t* d_argmax, int32_t* d_n_committed, void* stream);

/* A block denoised with iteration smoothing under the two schedules of Appendix "IterSmooth": the inner loop of
 * Algorithm 1 with dinfer_step_smooth as its step.  Step t = 0, 1, ... of the block uses
 *   mixing weight  alpha = 0 for t = 0 (nothing is retained yet), else min(alpha_init + alpha_growth * (t-1),
 *                  alpha_preset): the weight alpha_{t-1} that the appendix attaches to the expected embeddings
 *                  which step t-1 left for step t;
 *   threshold      max(threshold_start - threshold_decay * t, decode->threshold): decays from threshold_start
 *                  (1.0 in the appendix) to the decoder's own threshold as its target.  The appendix names no
 *                  curve; this is a linear one.  A hierarchical lower bound above the step's threshold is lowered
 *                  to it.
 * decode->fixed_k must be 0.  d_delta [n_seq][block_len][hidden] needs no initial contents.  Steps are enqueued
 * steps_per_wait at a time and the host waits once per batch, as in dinfer_generate_block's threshold mode (the
 * schedules are functions of the step index, which the host knows without waiting);
 * max_steps <= 256; scratch as in dinfer_step_smooth. */
typedef struct {
  float alpha_init, alpha_growth, alpha_preset;
  float threshold_start, threshold_decay;
} dinfer_smooth_schedule;
int dinfer_generate_block_smooth(dinfer_ctx* ctx, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens,
                                 uint64_t* d_mask, const int32_t* d_prefix_len, const int32_t* d_page_table,
                                 int32_t pt_stride, const dinfer_decode* decode, const dinfer_smooth_schedule* sched,
                                 float* d_delta, void* d_scratch, size_t scratch_bytes, float* d_conf, int32_t* d_argmax,
                                 int32_t* d_n_committed, int32_t max_steps, int32_t steps_per_wait,
                                 int32_t* h_steps_taken, void* stream);

/* dinfer_step_smooth for callers that cannot allocate device memory or hand over a scratch buffer (code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation): the logits and probability planes live in a
 * device array that is part of the library image, DINFER_STATIC_SCRATCH_BYTES per GPU, held from the moment the
 * library is loaded until the process ends.  The call allocates nothing and frees nothing; everything else is
 * dinfer_step_smooth (same kernels, same results bit for bit).
 *  - n_seq * block_len tokens are accepted while dinfer_smooth_scratch_bytes(cfg, n_seq * block_len) fits the array
 *    (e.g. 37 block tokens at a vocabulary of 157184 in bf16); more is refused with DINFER_ENOSPACE.
 *  - The array's address is looked up once per GPU, at dinfer_create; the context must be used with the GPU that was
 *    current then (DINFER_EINVAL otherwise).
 *  - All calls on one GPU share the array, whatever their context: calls that overlap on one GPU (different streams
 *    or threads) race.  Nothing in it has to start at zero: every call overwrites all the rows it reads, so the
 *    previous call's contents, of any size, do no harm. */
#define DINFER_STATIC_SCRATCH_BYTES (48u << 20)
int dinfer_step_smooth_static(dinfer_ctx* ctx, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens,
                              uint64_t* d_mask, const int32_t* d_prefix_len, const int32_t* d_page_table,
                              int32_t pt_stride, const dinfer_decode* decode, float alpha, float* d_delta,
                              float* d_conf, int32_t* d_argmax, int32_t* d_n_committed, void* stream);

/* The step with credit decoding (Appendix "Credit decoding").  Every undecided position keeps a credit per token,
 * C_t[v] = beta * C_{t-1}[v] + (v == top-1 candidate of step t ? p_t(v)^gamma : 0)          (equation 1)
 * and the decoder sees softmax(logits + alpha * log(1 + C_t)) instead of softmax(logits)     (equation 2):
 * d_conf / d_argmax report the largest probability of that enhanced distribution and its id (lowest id on
 * ties), and the threshold / fixed-k rule of `decode` acts on them.  Positions already decided report the
 * plain values and their credits are left alone.
 * Credit state, device memory owned by the caller and carried across the steps of one block: a token can only
 * hold credit if it was the top-1 candidate at some step, so a position stores a list of at most
 * DINFER_CREDIT_CAP (id, credit) entries:
 *   d_credit_ids [n_seq][block_len][DINFER_CREDIT_CAP] int32, d_credit_val same shape float32,
 *   d_credit_n   [n_seq][block_len] int32 entries in use.  Zero d_credit_n to start a block.
 * A block takes at most block_len <= 64 steps, so the list cannot overflow inside one; if a caller keeps state
 * longer, the entry with the smallest credit is replaced.
 * alpha >= 0, 0 <= beta <= 1, 0 < gamma <= 1.  Everything else as in dinfer_step. */
#define DINFER_CREDIT_CAP 64
typedef struct {
  float alpha, beta, gamma;
} dinfer_credit;
int dinfer_step_credit(dinfer_ctx* ctx, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens, uint64_t* d_mask,
                       const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                       const dinfer_decode* decode, const dinfer_credit* credit, int32_t* d_credit_ids,
                       float* d_credit_val, int32_t* d_credit_n, float* d_conf, int32_t* d_argmax,
                       int32_t* d_n_committed, void* stream);

/* The step with vicinity KV-cache refresh (Section 2, KV-cache management: during denoising K and V are
 * recomputed for the masked tokens and their immediate neighbours; the paper's experiments use a window of 16).
 * The look_back cached positions before each block join the forward: d_vicinity_tokens [n_seq][look_back] holds
 * their ids (positions prefix_len-look_back .. prefix_len-1); they are embedded again, attend to every key like
 * the block's positions, and their K,V rows in the prefix pages are OVERWRITTEN.  Logits, confidence and the
 * commit concern the block only; every other argument is as in dinfer_step.  There is no look-ahead part: the
 * block attends to its prefix and itself, positions after it do not exist here.
 * 0 <= look_back <= 64; the caller guarantees d_prefix_len[s] >= look_back for every sequence (a shorter prefix
 * keeps all accesses in bounds but misplaces the block); n_seq * (look_back + block_len) <= max_tokens, and
 * look_back + block_len positions must fit max_pos and the page-table row (DINFER_ENOSPACE otherwise).
 * look_back = 0 is dinfer_step. */
int dinfer_step_vicinity(dinfer_ctx* ctx, int32_t n_seq, int32_t block_len, int32_t look_back,
                         int32_t* d_block_tokens, const int32_t* d_vicinity_tokens, uint64_t* d_mask,
                         const int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride,
                         const dinfer_decode* decode, float* d_conf, int32_t* d_argmax, int32_t* d_n_committed,
                         void* stream);

/* Cache update of a decoded block: the same forward without LM head and decoder over the block's final
 * ids, leaving the block's K,V final, then d_prefix_len[s] += block_len. */
int dinfer_refresh_block(dinfer_ctx* ctx, int32_t n_seq, int32_t block_len, const int32_t* d_block_tokens,
                         int32_t* d_prefix_len, const int32_t* d_page_table, int32_t pt_stride, void* stream);

/* The outer loop of Algorithm 1 with early termination (Section 3, system optimisations, diffusion iterations):
 * n_blocks blocks of block_len positions are generated one after the other behind the cached prefix; every block
 * starts fully masked, is denoised by the inner loop (dinfer_generate_block: with decode->fixed_k > 0 its
 * ceil(block_len / fixed_k) steps are enqueued without waiting) and is then run through dinfer_refresh_block.
 * Once a decoded block of a sequence contains eos_id (negative: never) the sequence is finished: its remaining
 * blocks are filled with eos_id and commit nothing; when every sequence is finished the loop stops.  The host
 * waits once per block to read the count of finished sequences (and, with threshold decoding, once per
 * steps_per_wait steps inside a block: see dinfer_generate_block).
 *   d_out          [n_seq][n_blocks * block_len] out: the generated ids.
 *   d_block_tokens [n_seq][block_len], d_mask [n_seq], d_conf, d_argmax, d_n_committed: working buffers as in
 *                  dinfer_step (contents on return: those of the last step).
 *   d_finished     [n_seq] int32 out: 1 for a sequence that produced eos_id.
 *   d_prefix_len   [n_seq] in/out: advanced by block_len for every block that was run, for every sequence (a
 *                  finished sequence rides along in the batch; its rows of eos_id are cached like any others).
 *   *h_blocks_run  (host, may be NULL): blocks that were run before the loop stopped. */
int dinfer_generate(dinfer_ctx* ctx, int32_t n_seq, int32_t block_len, int32_t n_blocks, int32_t* d_out,
                    int32_t* d_block_tokens, uint64_t* d_mask, int32_t* d_prefix_len, const int32_t* d_page_table,
                    int32_t pt_stride, const dinfer_decode* decode, int32_t eos_id, int32_t steps_per_wait,
                    int32_t* d_finished, float* d_conf, int32_t* d_argmax, int32_t* d_n_committed, int32_t* h_blocks_run,
                    void* stream);

/* The inner loop of Algorithm 1: steps until every mask is empty or max_steps (at most 256) were taken.
 *  - fixed_k > 0 and h_masked_hint > 0 (the caller's count of undecided positions per sequence, the same for
 *    all): exactly ceil(h_masked_hint / fixed_k) steps are enqueued without waiting.
 *  - otherwise the number of steps depends on the data.  Steps are enqueued steps_per_wait at a time (0 or 1: one
 *    at a time) without waiting for their outcome, and the host waits once per such batch (Section 3, "Diffusion
 *    iterations": iterations are launched back to back; "Parallel decoding": the decoder runs on the device and
 *    nothing is copied to the host between iterations).  The device itself knows whether a step is still needed:
 *    the decoder of every step records whether a masked position remains, and the kernels of a step that finds
 *    nothing masked return at once -- such a step changes nothing, writes no output and is not counted.  A batch
 *    can therefore run up to steps_per_wait - 1 such empty steps behind the last real one (about a tenth of a
 *    real step each); the results are the same for every steps_per_wait.
 * *h_steps_taken (host, may be NULL) receives the number of steps that ran. */
int dinfer_generate_block(dinfer_ctx* ctx, int32_t n_seq, int32_t block_len, int32_t* d_block_tokens,
                          uint64_t* d_mask, const int32_t* d_prefix_len, const int32_t* d_page_table,
                          int32_t pt_stride, const dinfer_decode* decode, float* d_conf, int32_t* d_argmax,
                          int32_t* d_n_committed, int32_t max_steps, int32_t h_masked_hint, int32_t steps_per_wait,
                          int32_t* h_steps_taken, void* stream);

/* Moves K,V rows of one layer and one sequence between the pool and plain float32 arrays
 * d_k, d_v: [n_pos][n_heads*head_dim] for positions first_pos .. first_pos+n_pos-1 (keys as stored, i.e.
 * after the rotary embedding).  d_page_row: that sequence's page-table row. */
int dinfer_kv_write(dinfer_ctx* ctx, int32_t layer, const int32_t* d_page_row, int32_t first_pos,
                    int32_t n_pos, const float* d_k, const float* d_v, void* stream);
int dinfer_kv_read(dinfer_ctx* ctx, int32_t layer, const int32_t* d_page_row, int32_t first_pos, int32_t n_pos,
                   float* d_k, float* d_v, void* stream);

/* Test hooks.  dinfer_debug_logits recomputes the logits of the last forward's rows (n_rows must equal their
 * number) through the LM-head kernel's arithmetic and stores them: d_out [n_rows][vocab] float32.  dinfer_debug_get copies
 * an intermediate of the last forward: what = 0 residual stream leaving the last layer [T][hidden] f32;
 * 1 router expert ids of every layer [n_layers][T][top_k] i32; 2 their mixture weights, same shape, f32;
 * and of the last layer: 3 expert row counts [n_experts] i32; 4 expert offsets [n_experts+1] i32;
 * 5 permutation [T*top_k] i32; 6 two running totals since the last dinfer_profile_start [2] i32: experts that
 * received rows, summed over every layer of every forward, and the number of such (layer, forward) pairs. */
int dinfer_debug_logits(dinfer_ctx* ctx, int32_t n_rows, float* d_out, void* stream);
int dinfer_debug_get(dinfer_ctx* ctx, int32_t what, void* d_out, size_t bytes, void* stream);
/* Process-wide test switch.  While on (on != 0), no contraction shares a task's sum among workgroups: the
 * projections, the router and attention run with a single K slice / key split and the expert down projection takes
 * its unfused route (per-pair outputs, then the weighted combine), so no partial sum crosses workgroups.  Results then differ from the default path by float32 summation order only; the
 * tests compare the two to check that the cross-workgroup hand-off delivers every partial.  Not for concurrent use. */
int dinfer_debug_single_slice(int32_t on);

/* Per-launch timing of one stage of the forward, for benchmarks: between dinfer_profile_start and
 * dinfer_profile_stop every launch of that stage is bracketed by a HIP event pair on the caller's stream
 * (at most 8192 launches are recorded).  _stop waits for the recorded events and returns their count and
 * the summed elapsed milliseconds.  An event pair costs the stream a few microseconds around the launch it
 * brackets, so a benchmark that times whole steps as well samples: dinfer_profile_every(ctx, n), called before
 * _start, makes the profile bracket the launches of every n-th forward only (n >= 1; 1, the default, is every
 * forward; the setting stays until it is changed). */
enum {
  DINFER_STAGE_QKV = 0,
  DINFER_STAGE_ATTENTION = 1,
  DINFER_STAGE_OPROJ = 2,
  DINFER_STAGE_EXPERT_GATE_UP = 3,
  DINFER_STAGE_EXPERT_DOWN = 4,
  DINFER_STAGE_LM_HEAD = 5,
  DINFER_STAGE_ROUTER = 6,   /* RMSNorm statistics + router + top-k + permutation */
  DINFER_STAGE_COUNT = 7
};
int dinfer_profile_every(dinfer_ctx* ctx, int32_t n_forwards);
int dinfer_profile_start(dinfer_ctx* ctx, int32_t stage);
int dinfer_profile_stop(dinfer_ctx* ctx, int32_t* n_launches, float* total_ms);

/* Benchmark utility: one kernel that reads the first `bytes` (rounded down to 256 KiB) of d_buf once, with the
 * access pattern of the library's weight streams, and stores nothing (d_sink: one float, never written for
 * finite data).  Its duration gives the practical HBM read ceiling the weight-streaming kernels are judged
 * against.  d_buf: device, 16-byte aligned. */
int dinfer_stream_read(const void* d_buf, size_t bytes, float* d_sink, void* stream);

/* Profiling aid of libraries built with -DDINFER_TRACE=<kernel id>: copies the phase timestamps (100 MHz wall
 * clock, [workgroup][8 slots] of uint64) that the chosen kernel's last launch left, to the HOST buffer h_out
 * (synchronous).  unit: 0 = GEMM kernels, 1 = attention, 2 = many-token GEMM forms.  Ordinary builds return DINFER_EINVAL. */
int dinfer_debug_trace(int32_t unit, void* h_out, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif
