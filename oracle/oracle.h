/*
 * CPU oracle of one block denoising step of a MoE diffusion LLM.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain statement of what the
 * step computes; the tests, the smoke check and the benchmark's cpu_baseline
 * leg call it to judge the HIP library.  The product never calls it and it
 * shares no code with the HIP path.
 *
 * All arithmetic is IEEE double.  Weights are read as the stored values
 * (float32, or bfloat16 bit patterns widened exactly); no intermediate is
 * rounded to a narrower type.  Every weight matrix is row-major
 * [out_features][in_features].
 *
 * What is computed follows the paper's Algorithm 1 (inner loop: forward on
 * the active block with a KV cache, then decode), Section 2 (bidirectional
 * attention; threshold decoding; block-level KV reuse with a refresh of the
 * block once it is fully decoded) and the benchmark configuration for what
 * the paper leaves open (pre-norm transformer, RoPE, softmax top-k router,
 * SwiGLU experts, min-1 fallback, fixed-k variant).
 *
 * Parity pins: tests/test_oracle_*.py.  Unpinned: agreement with trained
 * LLaDA-MoE outputs (needs weights that are not available): "parity unpinned".
 */
#ifndef DINFER_ORACLE_H
#define DINFER_ORACLE_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t n_layers, hidden, n_heads, head_dim, n_experts, top_k, moe_inter, vocab;
  int32_t wdtype;    /* 0: float32 weights, 1: bfloat16 bit patterns */
  int32_t norm_topk; /* 1: renormalise the k selected router probabilities */
  double rms_eps, rope_theta, logit_scale;
} oracle_config;

typedef struct {
  const float* attn_gain; /* [H] */
  const void* wq;         /* [nh*hd][H] */
  const void* wk;
  const void* wv;
  const void* wo;         /* [H][nh*hd] */
  const float* ffn_gain;  /* [H] */
  const void* w_router;   /* [E][H] */
  const void* w_gate;     /* [E][I][H] */
  const void* w_up;       /* [E][I][H] */
  const void* w_down;     /* [E][H][I] */
} oracle_layer;

typedef struct {
  const void* emb;         /* [V][H] */
  const void* lm_head;     /* [V][H] */
  const float* final_gain; /* [H] */
  const oracle_layer* layers;
} oracle_weights;

/* Optional intermediates of a forward; any pointer may be NULL. */
typedef struct {
  int32_t* topk_idx; /* [L][T][k] expert ids in selection order */
  double* topk_w;    /* [L][T][k] their mixture weights */
  double* resid;     /* [L+1][T][H] residual stream entering layer l; [L] = leaving the last layer */
  double* attn_out;  /* [L][T][nh*hd] attention output before the output projection */
  double* router_p;  /* [L][T][E] router probabilities */
  /* INPUT, normally NULL: [L][T][k] expert ids to use instead of the oracle's own top-k.  Tests use it to
   * follow the HIP path through a near-tie of the k-th and (k+1)-th probability, where either choice is
   * valid; topk_idx still reports the oracle's own choice so that the two can be compared. */
  const int32_t* forced_idx;
} oracle_trace;

/* ---- building blocks (exported so that each can be pinned on its own) ---- */
void oracle_rmsnorm(const double* x, const float* gain, int n, double eps, double* out);
void oracle_rope(double* vec, int head_dim, int pos, double theta);
void oracle_linear(int wdtype, const void* W, int n_out, int n_in, const double* x, int n_tok, double* out);
void oracle_attention(const double* q, int n_q, const double* k, const double* v, int n_keys, int n_heads,
                      int head_dim, double* out);
void oracle_router_probs(int wdtype, const void* w_router, int n_experts, int hidden, const double* h, double* p);
void oracle_router(int wdtype, const void* w_router, int n_experts, int hidden, const double* h, int top_k,
                   int norm_topk, int32_t* idx, double* weight);
void oracle_moe_ffn(const oracle_config* c, const oracle_layer* l, const double* h, const int32_t* idx,
                    const double* weight, double* out);
void oracle_permutation(const int32_t* expert_of_pair, int n_pairs, int n_experts, int32_t* count,
                        int32_t* offset, int32_t* perm);
void oracle_confidence(const double* logits, int vocab, double* conf, int32_t* argmax);
int32_t oracle_commit(const double* conf, const int32_t* argmax, int block_len, uint64_t* mask,
                      int32_t* tokens, double threshold, int fixed_k);

/* Credit decoding (Appendix, "Credit decoding", equations 1 and 2) for ONE position.  logits [V] are the model's;
 * credit [V] is C_{t-1} on entry and C_t on return:
 *   p = softmax(logits),  v* = arg max p (lowest id on ties),
 *   C_t[v] = beta * C_{t-1}[v] + (v == v* ? p[v*]^gamma : 0),
 *   fused[v] = logits[v] + alpha * log(1 + C_t[v]),  enhanced distribution = softmax(fused).
 * conf / argmax: the largest enhanced probability and its id (lowest id on ties).  fused_out may be NULL. */
void oracle_credit_position(const double* logits, int vocab, double* credit, double alpha, double beta, double gamma,
                            double* conf, int32_t* argmax, double* fused_out);

/* ---- the step ---- */

/* Forward of n_tok tokens placed at positions prefix_len .. prefix_len+n_tok-1 of one sequence.
 * kcache/vcache: [L][cache_cap][nh*hd]; rows [0,prefix_len) are read, rows of the new tokens are
 * written, nothing else is touched.  hidden_out: [n_tok][H], the residual stream after the last layer. */
int oracle_forward(const oracle_config* c, const oracle_weights* w, int n_tok, const int32_t* tokens,
                   int prefix_len, double* kcache, double* vcache, int cache_cap, double* hidden_out,
                   const oracle_trace* trace);

/* The same forward with emb_add [n_tok][H] (may be NULL) added to the token embeddings before the first layer. */
int oracle_forward_embedded(const oracle_config* c, const oracle_weights* w, int n_tok, const int32_t* tokens,
                            const double* emb_add, int prefix_len, double* kcache, double* vcache, int cache_cap,
                            double* hidden_out, const oracle_trace* trace);

/* logits[t][v] = logit_scale * RMSNorm(hidden[t]; final_gain) . lm_head[v] */
void oracle_logits(const oracle_config* c, const oracle_weights* w, const double* hidden, int n_tok,
                   double* logits);

/* One denoising step of one sequence: forward, logits, confidence, commit.
 * conf/argmax: [block_len] (defined for every position); logits_out may be NULL, else [block_len][V].
 * Returns the number of positions committed. */
int32_t oracle_step(const oracle_config* c, const oracle_weights* w, int block_len, int32_t* block_tokens,
                    uint64_t* mask, int prefix_len, double* kcache, double* vcache, int cache_cap,
                    double threshold, int fixed_k, double* conf, int32_t* argmax, double* logits_out,
                    const oracle_trace* trace);

/* The step with vicinity KV-cache refresh (Section 2, KV-cache management: during denoising K and V are recomputed
 * for the masked tokens and for their immediate neighbours).  The look_back cached positions before the block
 * (ids in vicinity_tokens[look_back], positions prefix_len-look_back .. prefix_len-1) join the forward: they
 * are embedded again, attend to every key like the block's positions, and their K,V rows in the cache are
 * overwritten.  Logits, confidence and the commit concern the block's positions only.  Positions after the block
 * do not exist in this formulation (the block attends to the prefix and itself), so there is no look-ahead part.
 * Requires 0 <= look_back <= prefix_len.  The trace (if any) covers look_back + block_len tokens. */
int32_t oracle_step_vicinity(const oracle_config* c, const oracle_weights* w, int block_len, int look_back,
                             int32_t* block_tokens, const int32_t* vicinity_tokens, uint64_t* mask, int prefix_len,
                             double* kcache, double* vcache, int cache_cap, double threshold, int fixed_k,
                             double* conf, int32_t* argmax, double* logits_out, const oracle_trace* trace);

/* Iteration smoothing (Appendix "IterSmooth").  delta [H] = softmax(logits) . W_emb: the expected input embedding
 * under the position's predicted distribution (the input embedding matrix is used: it is not tied to the LM head). */
void oracle_expected_embedding(const oracle_config* c, const oracle_weights* w, const double* logits, double* delta);

/* One denoising step with iteration smoothing.  delta: [block_len][H], kept by the caller across the steps of a
 * block (zero at its start).  On entry it holds the expected embeddings the previous step retained; a position that
 * is still masked is embedded as e_mask + alpha * delta[i] (alpha = this step's mixing weight
 * min(alpha_init + alpha_growth * t, alpha_preset), computed by the caller), every other position as its token's
 * embedding.  On return the rows of the positions that were masked at the start of the step hold the expected
 * embeddings of this step's logits.  Everything else as oracle_step. */
int32_t oracle_step_smooth(const oracle_config* c, const oracle_weights* w, int block_len, int32_t* block_tokens,
                           uint64_t* mask, int prefix_len, double* kcache, double* vcache, int cache_cap,
                           double threshold, int fixed_k, double alpha, double* delta, double* conf, int32_t* argmax,
                           double* logits_out, const oracle_trace* trace);

/* One denoising step with credit decoding: as oracle_step, but the decoder sees the enhanced distribution.
 * credit: [block_len][V], kept by the caller across the steps of one block (zero at its start); only the rows of
 * positions that are still masked when the step begins are updated and fused, the other positions report the
 * plain confidence and arg max.  logits_out (may be NULL) receives the FUSED logits of the masked rows and the
 * plain logits of the others. */
int32_t oracle_step_credit(const oracle_config* c, const oracle_weights* w, int block_len, int32_t* block_tokens,
                           uint64_t* mask, int prefix_len, double* kcache, double* vcache, int cache_cap,
                           double threshold, int fixed_k, double* credit, double alpha, double beta, double gamma,
                           double* conf, int32_t* argmax, double* logits_out, const oracle_trace* trace);

/* Repeats oracle_step until the mask is empty (at most max_steps); returns steps taken.
 * committed_per_step (may be NULL): [max_steps]. */
int32_t oracle_generate_block(const oracle_config* c, const oracle_weights* w, int block_len,
                              int32_t* block_tokens, uint64_t* mask, int prefix_len, double* kcache,
                              double* vcache, int cache_cap, double threshold, int fixed_k, int max_steps,
                              int32_t* committed_per_step);

/* Hierarchical decoding (Appendix "Hierarchical decoding"): the commit rule on given confidences, and the step
 * that uses it in place of oracle_commit.  See oracle.c for the reading of the paper's prose. */
int32_t oracle_commit_hier(const double* conf, const int32_t* argmax, int block_len, uint64_t* mask,
                           int32_t* tokens, double tau_high, double tau_low);
int32_t oracle_step_hier(const oracle_config* c, const oracle_weights* w, int block_len, int32_t* block_tokens,
                         uint64_t* mask, int prefix_len, double* kcache, double* vcache, int cache_cap,
                         double tau_high, double tau_low, double* conf, int32_t* argmax, double* logits_out,
                         const oracle_trace* trace);

/* Outer loop of Algorithm 1 over n_blocks blocks (each starts as block_len times mask_id) with early termination
 * at eos_id (Section 3, system optimisations; negative: none); out
 * [n_blocks * block_len]; steps_per_block (may be NULL) [n_blocks]; returns the blocks decoded. */
int32_t oracle_generate(const oracle_config* c, const oracle_weights* w, int block_len, int n_blocks, int prefix_len,
                        double* kcache, double* vcache, int cache_cap, double threshold, int fixed_k, int32_t mask_id,
                        int32_t eos_id, int32_t* out, int32_t* steps_per_block);

int oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
