/*
 * CPU oracle of one block denoising step of a MoE diffusion LLM: see oracle.h.
 * TEST INFRASTRUCTURE ONLY; plain loops in IEEE double, in the order the step is defined.
 */
#include "oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Stored weight element i of tensor W as a double (exact widening). */
static inline double wval(int wdtype, const void* W, size_t i) {
  if (wdtype == 0) return (double)((const float*)W)[i];
  union { uint32_t u; float f; } v;
  v.u = (uint32_t)((const uint16_t*)W)[i] << 16;
  return (double)v.f;
}

/* sum_k w[row][k] * x[k] */
static double dot_row(int wdtype, const void* W, size_t row, int n_in, const double* x) {
  double acc = 0.0;
  const size_t base = row * (size_t)n_in;
  if (wdtype == 0) {
    const float* w = (const float*)W + base;
#pragma omp simd reduction(+ : acc)
    for (int k = 0; k < n_in; ++k) acc += (double)w[k] * x[k];
  } else {
    const uint16_t* w = (const uint16_t*)W + base;
#pragma omp simd reduction(+ : acc)
    for (int k = 0; k < n_in; ++k) {
      union { uint32_t u; float f; } v;
      v.u = (uint32_t)w[k] << 16;
      acc += (double)v.f * x[k];
    }
  }
  return acc;
}

/* RMSNorm: out = x / sqrt(mean(x^2) + eps) * gain */
void oracle_rmsnorm(const double* x, const float* gain, int n, double eps, double* out) {
  double ss = 0.0;
  for (int i = 0; i < n; ++i) ss += x[i] * x[i];
  const double r = 1.0 / sqrt(ss / n + eps);
  for (int i = 0; i < n; ++i) out[i] = x[i] * r * (double)gain[i];
}

/* Rotary embedding, rotate-half pairing (j, j + hd/2), angle = pos * theta^(-2j/hd). */
void oracle_rope(double* vec, int head_dim, int pos, double theta) {
  const int half = head_dim / 2;
  for (int j = 0; j < half; ++j) {
    const double ang = (double)pos * pow(theta, -2.0 * j / head_dim);
    const double c = cos(ang), s = sin(ang);
    const double a = vec[j], b = vec[j + half];
    vec[j] = a * c - b * s;
    vec[j + half] = b * c + a * s;
  }
}

/* out[t][n] = sum_k x[t][k] * W[n][k] */
void oracle_linear(int wdtype, const void* W, int n_out, int n_in, const double* x, int n_tok, double* out) {
#pragma omp parallel for schedule(static)
  for (int n = 0; n < n_out; ++n)
    for (int t = 0; t < n_tok; ++t) out[(size_t)t * n_out + n] = dot_row(wdtype, W, (size_t)n, n_in, x + (size_t)t * n_in);
}

/* Bidirectional attention: every query sees every one of the n_keys keys (Section 2: dLLMs use
 * bidirectional attention).  q: [n_q][nh*hd], k, v: [n_keys][nh*hd], out: [n_q][nh*hd]. */
void oracle_attention(const double* q, int n_q, const double* k, const double* v, int n_keys, int n_heads,
                      int head_dim, double* out) {
  const int D = n_heads * head_dim;
  const double scale = 1.0 / sqrt((double)head_dim);
#pragma omp parallel for collapse(2) schedule(static)
  for (int i = 0; i < n_q; ++i) {
    for (int h = 0; h < n_heads; ++h) {
      double* s = (double*)malloc(sizeof(double) * (size_t)n_keys);
      const double* qi = q + (size_t)i * D + h * head_dim;
      double m = -INFINITY;
      for (int j = 0; j < n_keys; ++j) {
        const double* kj = k + (size_t)j * D + h * head_dim;
        double acc = 0.0;
        for (int d = 0; d < head_dim; ++d) acc += qi[d] * kj[d];
        s[j] = acc * scale;
        if (s[j] > m) m = s[j];
      }
      double z = 0.0;
      for (int j = 0; j < n_keys; ++j) {
        s[j] = exp(s[j] - m);
        z += s[j];
      }
      double* o = out + (size_t)i * D + h * head_dim;
      for (int d = 0; d < head_dim; ++d) o[d] = 0.0;
      for (int j = 0; j < n_keys; ++j) {
        const double p = s[j] / z;
        const double* vj = v + (size_t)j * D + h * head_dim;
        for (int d = 0; d < head_dim; ++d) o[d] += p * vj[d];
      }
      free(s);
    }
  }
}

/* Router probabilities: softmax over all experts of h . w_router[e]. */
void oracle_router_probs(int wdtype, const void* w_router, int n_experts, int hidden, const double* h, double* p) {
  double m = -INFINITY;
  for (int e = 0; e < n_experts; ++e) {
    p[e] = dot_row(wdtype, w_router, (size_t)e, hidden, h);
    if (p[e] > m) m = p[e];
  }
  double z = 0.0;
  for (int e = 0; e < n_experts; ++e) {
    p[e] = exp(p[e] - m);
    z += p[e];
  }
  for (int e = 0; e < n_experts; ++e) p[e] /= z;
}

/* Router: the k largest probabilities (ties -> lower expert id), in selection order; weights
 * renormalised to sum 1 when norm_topk. */
void oracle_router(int wdtype, const void* w_router, int n_experts, int hidden, const double* h, int top_k,
                   int norm_topk, int32_t* idx, double* weight) {
  double* p = (double*)malloc(sizeof(double) * (size_t)n_experts);
  oracle_router_probs(wdtype, w_router, n_experts, hidden, h, p);
  double sel = 0.0;
  for (int j = 0; j < top_k; ++j) {
    int best = -1;
    for (int e = 0; e < n_experts; ++e) {
      int taken = 0;
      for (int i = 0; i < j; ++i) taken |= (idx[i] == e);
      if (!taken && (best < 0 || p[e] > p[best])) best = e;
    }
    idx[j] = best;
    weight[j] = p[best];
    sel += p[best];
  }
  if (norm_topk)
    for (int j = 0; j < top_k; ++j) weight[j] /= sel;
  free(p);
}

static inline double silu(double x) { return x / (1.0 + exp(-x)); }

/* out[H] = sum_j weight[j] * ( (silu(h Wg_e) * (h Wu_e)) Wd_e ),  e = idx[j] */
void oracle_moe_ffn(const oracle_config* c, const oracle_layer* l, const double* h, const int32_t* idx,
                    const double* weight, double* out) {
  const int H = c->hidden, I = c->moe_inter;
  double* y = (double*)malloc(sizeof(double) * (size_t)I);
  for (int n = 0; n < H; ++n) out[n] = 0.0;
  for (int j = 0; j < c->top_k; ++j) {
    const size_t e = (size_t)idx[j];
    for (int f = 0; f < I; ++f) {
      const double gate = dot_row(c->wdtype, l->w_gate, e * I + f, H, h);
      const double up = dot_row(c->wdtype, l->w_up, e * I + f, H, h);
      y[f] = silu(gate) * up;
    }
    for (int n = 0; n < H; ++n) out[n] += weight[j] * dot_row(c->wdtype, l->w_down, e * H + n, I, y);
  }
  free(y);
}

/* Stable counting sort of (token, slot) pairs by expert: count[E], offset[E+1], perm[n_pairs] where
 * perm[offset[e] + r] is the r-th pair (in pair order) routed to expert e. */
void oracle_permutation(const int32_t* expert_of_pair, int n_pairs, int n_experts, int32_t* count,
                        int32_t* offset, int32_t* perm) {
  for (int e = 0; e < n_experts; ++e) count[e] = 0;
  for (int p = 0; p < n_pairs; ++p) count[expert_of_pair[p]]++;
  offset[0] = 0;
  for (int e = 0; e < n_experts; ++e) offset[e + 1] = offset[e] + count[e];
  int32_t* fill = (int32_t*)calloc((size_t)(n_experts > 0 ? n_experts : 1), sizeof(int32_t));
  for (int p = 0; p < n_pairs; ++p) {
    const int e = expert_of_pair[p];
    perm[offset[e] + fill[e]++] = p;
  }
  free(fill);
}

int oracle_forward(const oracle_config* c, const oracle_weights* w, int n_tok, const int32_t* tokens,
                   int prefix_len, double* kcache, double* vcache, int cache_cap, double* hidden_out,
                   const oracle_trace* trace) {
  return oracle_forward_embedded(c, w, n_tok, tokens, NULL, prefix_len, kcache, vcache, cache_cap, hidden_out, trace);
}

int oracle_forward_embedded(const oracle_config* c, const oracle_weights* w, int n_tok, const int32_t* tokens,
                            const double* emb_add, int prefix_len, double* kcache, double* vcache, int cache_cap,
                            double* hidden_out, const oracle_trace* trace) {
  const int H = c->hidden, D = c->n_heads * c->head_dim, hd = c->head_dim, K = c->top_k;
  if (prefix_len < 0 || n_tok <= 0 || prefix_len + n_tok > cache_cap) return -1;
  for (int t = 0; t < n_tok; ++t)
    if (tokens[t] < 0 || tokens[t] >= c->vocab) return -2;
  if (c->n_experts > 64 || c->top_k > 64) return -3;

  double* x = hidden_out; /* residual stream [n_tok][H] */
  double* hn = (double*)malloc(sizeof(double) * (size_t)n_tok * H);
  double* q = (double*)malloc(sizeof(double) * (size_t)n_tok * D);
  double* a = (double*)malloc(sizeof(double) * (size_t)n_tok * D);
  double* proj = (double*)malloc(sizeof(double) * (size_t)n_tok * H);

  /* the sequence is first embedded (masked positions carry the mask id and embed its row) */
  for (int t = 0; t < n_tok; ++t)
    for (int i = 0; i < H; ++i) x[(size_t)t * H + i] = wval(c->wdtype, w->emb, (size_t)tokens[t] * H + i);
  /* iteration smoothing: what the previous iteration retained for a position is added to its embedding */
  if (emb_add)
    for (size_t i = 0; i < (size_t)n_tok * H; ++i) x[i] += emb_add[i];

  for (int l = 0; l < c->n_layers; ++l) {
    const oracle_layer* L = &w->layers[l];
    double* kc = kcache + (size_t)l * cache_cap * D;
    double* vc = vcache + (size_t)l * cache_cap * D;
    if (trace && trace->resid) memcpy(trace->resid + (size_t)l * n_tok * H, x, sizeof(double) * (size_t)n_tok * H);

    /* attention half: x += Attn(RMSNorm(x)) Wo */
    for (int t = 0; t < n_tok; ++t) oracle_rmsnorm(x + (size_t)t * H, L->attn_gain, H, c->rms_eps, hn + (size_t)t * H);
    oracle_linear(c->wdtype, L->wq, D, H, hn, n_tok, q);
    /* K and V of the block's tokens are recomputed and placed after the cached prefix */
    oracle_linear(c->wdtype, L->wk, D, H, hn, n_tok, kc + (size_t)prefix_len * D);
    oracle_linear(c->wdtype, L->wv, D, H, hn, n_tok, vc + (size_t)prefix_len * D);
    for (int t = 0; t < n_tok; ++t)
      for (int h = 0; h < c->n_heads; ++h) {
        oracle_rope(q + (size_t)t * D + h * hd, hd, prefix_len + t, c->rope_theta);
        oracle_rope(kc + (size_t)(prefix_len + t) * D + h * hd, hd, prefix_len + t, c->rope_theta);
      }
    oracle_attention(q, n_tok, kc, vc, prefix_len + n_tok, c->n_heads, hd, a);
    if (trace && trace->attn_out) memcpy(trace->attn_out + (size_t)l * n_tok * D, a, sizeof(double) * (size_t)n_tok * D);
    oracle_linear(c->wdtype, L->wo, H, D, a, n_tok, proj);
    for (size_t i = 0; i < (size_t)n_tok * H; ++i) x[i] += proj[i];

    /* MoE half: x += sum over the token's top-k experts of weight * SwiGLU-FFN_e(RMSNorm(x)) */
    for (int t = 0; t < n_tok; ++t) oracle_rmsnorm(x + (size_t)t * H, L->ffn_gain, H, c->rms_eps, hn + (size_t)t * H);
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < n_tok; ++t) {
      int32_t idx[64];
      double wt[64];
      oracle_router(c->wdtype, L->w_router, c->n_experts, H, hn + (size_t)t * H, K, c->norm_topk, idx, wt);
      if (trace && trace->topk_idx) memcpy(trace->topk_idx + ((size_t)l * n_tok + t) * K, idx, sizeof(int32_t) * K);
      if (trace && trace->topk_w) memcpy(trace->topk_w + ((size_t)l * n_tok + t) * K, wt, sizeof(double) * K);
      if (trace && (trace->router_p || trace->forced_idx)) {
        double p[64];
        oracle_router_probs(c->wdtype, L->w_router, c->n_experts, H, hn + (size_t)t * H, p);
        if (trace->router_p) memcpy(trace->router_p + ((size_t)l * n_tok + t) * c->n_experts, p, sizeof(double) * c->n_experts);
        if (trace->forced_idx) {
          /* the caller dictates the expert set (to follow another implementation through a near-tie);
           * the mixture weights are still this oracle's own probabilities of those experts */
          double sel = 0.0;
          for (int j = 0; j < K; ++j) {
            idx[j] = trace->forced_idx[((size_t)l * n_tok + t) * K + j];
            wt[j] = p[idx[j]];
            sel += wt[j];
          }
          if (c->norm_topk)
            for (int j = 0; j < K; ++j) wt[j] /= sel;
        }
      }
      oracle_moe_ffn(c, L, hn + (size_t)t * H, idx, wt, proj + (size_t)t * H);
    }
    for (size_t i = 0; i < (size_t)n_tok * H; ++i) x[i] += proj[i];
  }
  if (trace && trace->resid)
    memcpy(trace->resid + (size_t)c->n_layers * n_tok * H, x, sizeof(double) * (size_t)n_tok * H);
  free(hn);
  free(q);
  free(a);
  free(proj);
  return 0;
}

void oracle_logits(const oracle_config* c, const oracle_weights* w, const double* hidden, int n_tok,
                   double* logits) {
  const int H = c->hidden;
  double* hn = (double*)malloc(sizeof(double) * (size_t)n_tok * H);
  for (int t = 0; t < n_tok; ++t) oracle_rmsnorm(hidden + (size_t)t * H, w->final_gain, H, c->rms_eps, hn + (size_t)t * H);
  oracle_linear(c->wdtype, w->lm_head, c->vocab, H, hn, n_tok, logits);
  for (size_t i = 0; i < (size_t)n_tok * c->vocab; ++i) logits[i] *= c->logit_scale;
  free(hn);
}

/* Confidence of a position = the largest softmax probability of its logits row; the candidate id is
 * the arg max (lowest id on ties).  conf = exp(z_max - z_max) / sum_v exp(z_v - z_max). */
void oracle_confidence(const double* logits, int vocab, double* conf, int32_t* argmax) {
  int best = 0;
  for (int v = 1; v < vocab; ++v)
    if (logits[v] > logits[best]) best = v;
  double z = 0.0;
  for (int v = 0; v < vocab; ++v) z += exp(logits[v] - logits[best]);
  *conf = 1.0 / z;
  *argmax = best;
}

/* Credit decoding for one position (Appendix "Credit decoding", equations 1 and 2), written out densely over the
 * vocabulary: discount every credit, reward the current top-1 token with its probability to the power gamma, add
 * alpha * log(1 + credit) to the logits and take the softmax of that. */
void oracle_credit_position(const double* logits, int vocab, double* credit, double alpha, double beta, double gamma,
                            double* conf, int32_t* argmax, double* fused_out) {
  double p_top;
  int32_t v_top;
  oracle_confidence(logits, vocab, &p_top, &v_top);               /* p = softmax(logits), v* and p[v*] */
  for (int v = 0; v < vocab; ++v) credit[v] *= beta;              /* equation 1 */
  credit[v_top] += pow(p_top, gamma);
  double* fused = fused_out ? fused_out : (double*)malloc(sizeof(double) * (size_t)vocab);
  for (int v = 0; v < vocab; ++v) fused[v] = logits[v] + alpha * log(1.0 + credit[v]);   /* equation 2 */
  oracle_confidence(fused, vocab, conf, argmax);                  /* largest enhanced probability */
  if (!fused_out) free(fused);
}

/* Decoder (Section 2, threshold decoding): among masked positions commit those whose confidence
 * reaches the threshold; if there is none, commit the single most confident one (lowest position on
 * ties) so that every step makes progress.  fixed_k > 0 instead commits the fixed_k most confident
 * masked positions (all of them if fewer remain).  Committed positions take their candidate id and
 * leave the mask; nothing else changes. */
int32_t oracle_commit(const double* conf, const int32_t* argmax, int block_len, uint64_t* mask,
                      int32_t* tokens, double threshold, int fixed_k) {
  const uint64_t old = *mask;
  uint64_t sel = 0;
  if (fixed_k > 0) {
    for (int r = 0; r < fixed_k; ++r) {
      int best = -1;
      for (int i = 0; i < block_len; ++i) {
        if (!((old >> i) & 1) || ((sel >> i) & 1)) continue;
        if (best < 0 || conf[i] > conf[best]) best = i;
      }
      if (best < 0) break;
      sel |= (uint64_t)1 << best;
    }
  } else {
    int best = -1;
    for (int i = 0; i < block_len; ++i) {
      if (!((old >> i) & 1)) continue;
      if (conf[i] >= threshold) sel |= (uint64_t)1 << i;
      if (best < 0 || conf[i] > conf[best]) best = i;
    }
    if (sel == 0 && best >= 0) sel = (uint64_t)1 << best;
  }
  int32_t n = 0;
  for (int i = 0; i < block_len; ++i)
    if ((sel >> i) & 1) {
      tokens[i] = argmax[i];
      ++n;
    }
  *mask = old & ~sel;
  return n;
}

/* Decoder (Appendix "Hierarchical decoding"; thresholds from the experimental configuration: decoding
 * threshold 0.92, lower boundary 0.62).  The paper gives the method in prose only; this is the reading taken:
 *   1. every masked position whose confidence reaches tau_high is committed;
 *   2. the regions of a step are the maximal runs of consecutive masked positions (as masked when the step
 *      starts).  A region in which step 1 committed nothing tries to resolve one position: among its positions
 *      whose confidence reaches tau_low, the one closest to the centre of the run (on equal distance the more
 *      confident one, then the lower position).  Committing near the centre splits the run, so the regions of the
 *      next step are the halves: the recursion runs over the forward passes;
 *   3. if steps 1 and 2 committed nothing at all, the single most confident masked position is committed (lowest
 *      position on ties), as in oracle_commit, so that the loop of Algorithm 1 ends. */
int32_t oracle_commit_hier(const double* conf, const int32_t* argmax, int block_len, uint64_t* mask,
                           int32_t* tokens, double tau_high, double tau_low) {
  const uint64_t old = *mask;
  uint64_t sel = 0;
  int a = 0;
  while (a < block_len) {
    if (!((old >> a) & 1)) {
      ++a;
      continue;
    }
    int b = a;                                     /* the run is a .. b inclusive */
    while (b + 1 < block_len && ((old >> (b + 1)) & 1)) ++b;
    int high = 0;
    for (int i = a; i <= b; ++i)
      if (conf[i] >= tau_high) {
        sel |= (uint64_t)1 << i;
        high = 1;
      }
    if (!high) {
      int best = -1, best_dist = 0;
      for (int i = a; i <= b; ++i) {
        if (conf[i] < tau_low) continue;
        int dist = 2 * i - (a + b);                /* twice the distance to the centre (a + b) / 2 */
        if (dist < 0) dist = -dist;
        if (best < 0 || dist < best_dist || (dist == best_dist && conf[i] > conf[best])) {
          best = i;
          best_dist = dist;
        }
      }
      if (best >= 0) sel |= (uint64_t)1 << best;
    }
    a = b + 1;
  }
  if (sel == 0) {
    int best = -1;
    for (int i = 0; i < block_len; ++i)
      if (((old >> i) & 1) && (best < 0 || conf[i] > conf[best])) best = i;
    if (best >= 0) sel = (uint64_t)1 << best;
  }
  int32_t n = 0;
  for (int i = 0; i < block_len; ++i)
    if ((sel >> i) & 1) {
      tokens[i] = argmax[i];
      ++n;
    }
  *mask = old & ~sel;
  return n;
}

int32_t oracle_step_hier(const oracle_config* c, const oracle_weights* w, int block_len, int32_t* block_tokens,
                         uint64_t* mask, int prefix_len, double* kcache, double* vcache, int cache_cap,
                         double tau_high, double tau_low, double* conf, int32_t* argmax, double* logits_out,
                         const oracle_trace* trace) {
  const int V = c->vocab;
  double* hidden = (double*)malloc(sizeof(double) * (size_t)block_len * c->hidden);
  double* logits = logits_out ? logits_out : (double*)malloc(sizeof(double) * (size_t)block_len * V);
  int32_t n = -1;
  if (oracle_forward(c, w, block_len, block_tokens, prefix_len, kcache, vcache, cache_cap, hidden, trace) == 0) {
    oracle_logits(c, w, hidden, block_len, logits);
    for (int i = 0; i < block_len; ++i) oracle_confidence(logits + (size_t)i * V, V, &conf[i], &argmax[i]);
    n = oracle_commit_hier(conf, argmax, block_len, mask, block_tokens, tau_high, tau_low);
  }
  if (!logits_out) free(logits);
  free(hidden);
  return n;
}

int32_t oracle_step(const oracle_config* c, const oracle_weights* w, int block_len, int32_t* block_tokens,
                    uint64_t* mask, int prefix_len, double* kcache, double* vcache, int cache_cap,
                    double threshold, int fixed_k, double* conf, int32_t* argmax, double* logits_out,
                    const oracle_trace* trace) {
  const int V = c->vocab;
  double* hidden = (double*)malloc(sizeof(double) * (size_t)block_len * c->hidden);
  double* logits = logits_out ? logits_out : (double*)malloc(sizeof(double) * (size_t)block_len * V);
  int32_t n = -1;
  if (oracle_forward(c, w, block_len, block_tokens, prefix_len, kcache, vcache, cache_cap, hidden, trace) == 0) {
    oracle_logits(c, w, hidden, block_len, logits);
    for (int i = 0; i < block_len; ++i) oracle_confidence(logits + (size_t)i * V, V, &conf[i], &argmax[i]);
    n = oracle_commit(conf, argmax, block_len, mask, block_tokens, threshold, fixed_k);
  }
  if (!logits_out) free(logits);
  free(hidden);
  return n;
}

/* Expected embedding of one position (Appendix "IterSmooth"): p = softmax(logits), delta = p . W_emb. */
void oracle_expected_embedding(const oracle_config* c, const oracle_weights* w, const double* logits, double* delta) {
  const int V = c->vocab, H = c->hidden;
  double m = logits[0];
  for (int v = 1; v < V; ++v)
    if (logits[v] > m) m = logits[v];
  double z = 0.0;
  for (int v = 0; v < V; ++v) z += exp(logits[v] - m);
  for (int i = 0; i < H; ++i) delta[i] = 0.0;
  for (int v = 0; v < V; ++v) {
    const double p = exp(logits[v] - m) / z;
    for (int i = 0; i < H; ++i) delta[i] += p * wval(c->wdtype, w->emb, (size_t)v * H + i);
  }
}

int32_t oracle_step_smooth(const oracle_config* c, const oracle_weights* w, int block_len, int32_t* block_tokens,
                           uint64_t* mask, int prefix_len, double* kcache, double* vcache, int cache_cap,
                           double threshold, int fixed_k, double alpha, double* delta, double* conf, int32_t* argmax,
                           double* logits_out, const oracle_trace* trace) {
  const int V = c->vocab, H = c->hidden;
  double* hidden = (double*)malloc(sizeof(double) * (size_t)block_len * H);
  double* add = (double*)calloc((size_t)block_len * H, sizeof(double));
  double* logits = logits_out ? logits_out : (double*)malloc(sizeof(double) * (size_t)block_len * V);
  /* e_t[i] = e_mask + alpha_t * delta_{t-1}[i] on the positions that are still masked, plain embeddings elsewhere */
  for (int i = 0; i < block_len; ++i)
    if ((*mask >> i) & 1)
      for (int j = 0; j < H; ++j) add[(size_t)i * H + j] = alpha * delta[(size_t)i * H + j];
  int32_t n = -1;
  if (oracle_forward_embedded(c, w, block_len, block_tokens, add, prefix_len, kcache, vcache, cache_cap, hidden, trace) == 0) {
    oracle_logits(c, w, hidden, block_len, logits);
    for (int i = 0; i < block_len; ++i) oracle_confidence(logits + (size_t)i * V, V, &conf[i], &argmax[i]);
    /* what this iteration retains for the next one: the expected embedding of every position that was masked */
    for (int i = 0; i < block_len; ++i)
      if ((*mask >> i) & 1) oracle_expected_embedding(c, w, logits + (size_t)i * V, delta + (size_t)i * H);
    n = oracle_commit(conf, argmax, block_len, mask, block_tokens, threshold, fixed_k);
  }
  if (!logits_out) free(logits);
  free(add);
  free(hidden);
  return n;
}

int32_t oracle_step_credit(const oracle_config* c, const oracle_weights* w, int block_len, int32_t* block_tokens,
                           uint64_t* mask, int prefix_len, double* kcache, double* vcache, int cache_cap,
                           double threshold, int fixed_k, double* credit, double alpha, double beta, double gamma,
                           double* conf, int32_t* argmax, double* logits_out, const oracle_trace* trace) {
  const int V = c->vocab;
  double* hidden = (double*)malloc(sizeof(double) * (size_t)block_len * c->hidden);
  double* logits = logits_out ? logits_out : (double*)malloc(sizeof(double) * (size_t)block_len * V);
  double* fused = (double*)malloc(sizeof(double) * (size_t)V);
  int32_t n = -1;
  if (oracle_forward(c, w, block_len, block_tokens, prefix_len, kcache, vcache, cache_cap, hidden, trace) == 0) {
    oracle_logits(c, w, hidden, block_len, logits);
    for (int i = 0; i < block_len; ++i) {
      double* row = logits + (size_t)i * V;
      if ((*mask >> i) & 1) {
        oracle_credit_position(row, V, credit + (size_t)i * V, alpha, beta, gamma, &conf[i], &argmax[i], fused);
        for (int v = 0; v < V; ++v) row[v] = fused[v];
      } else {
        oracle_confidence(row, V, &conf[i], &argmax[i]);
      }
    }
    n = oracle_commit(conf, argmax, block_len, mask, block_tokens, threshold, fixed_k);
  }
  free(fused);
  if (!logits_out) free(logits);
  free(hidden);
  return n;
}

int32_t oracle_step_vicinity(const oracle_config* c, const oracle_weights* w, int block_len, int look_back,
                             int32_t* block_tokens, const int32_t* vicinity_tokens, uint64_t* mask, int prefix_len,
                             double* kcache, double* vcache, int cache_cap, double threshold, int fixed_k,
                             double* conf, int32_t* argmax, double* logits_out, const oracle_trace* trace) {
  if (look_back < 0 || look_back > prefix_len) return -1;
  const int V = c->vocab, n = look_back + block_len;
  int32_t* tokens = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
  double* hidden = (double*)malloc(sizeof(double) * (size_t)n * c->hidden);
  double* logits = logits_out ? logits_out : (double*)malloc(sizeof(double) * (size_t)block_len * V);
  for (int i = 0; i < look_back; ++i) tokens[i] = vicinity_tokens[i];
  for (int i = 0; i < block_len; ++i) tokens[look_back + i] = block_tokens[i];
  int32_t committed = -1;
  /* the neighbours are simply the first tokens of a longer forward that starts look_back positions earlier */
  if (oracle_forward(c, w, n, tokens, prefix_len - look_back, kcache, vcache, cache_cap, hidden, trace) == 0) {
    oracle_logits(c, w, hidden + (size_t)look_back * c->hidden, block_len, logits);
    for (int i = 0; i < block_len; ++i) oracle_confidence(logits + (size_t)i * V, V, &conf[i], &argmax[i]);
    committed = oracle_commit(conf, argmax, block_len, mask, block_tokens, threshold, fixed_k);
  }
  if (!logits_out) free(logits);
  free(hidden);
  free(tokens);
  return committed;
}

int32_t oracle_generate_block(const oracle_config* c, const oracle_weights* w, int block_len,
                              int32_t* block_tokens, uint64_t* mask, int prefix_len, double* kcache,
                              double* vcache, int cache_cap, double threshold, int fixed_k, int max_steps,
                              int32_t* committed_per_step) {
  double* conf = (double*)malloc(sizeof(double) * (size_t)block_len);
  int32_t* am = (int32_t*)malloc(sizeof(int32_t) * (size_t)block_len);
  int32_t steps = 0;
  while (*mask != 0 && steps < max_steps) {
    const int32_t n = oracle_step(c, w, block_len, block_tokens, mask, prefix_len, kcache, vcache, cache_cap,
                                  threshold, fixed_k, conf, am, NULL, NULL);
    if (n < 0) {
      steps = -1;
      break;
    }
    if (committed_per_step) committed_per_step[steps] = n;
    ++steps;
  }
  free(conf);
  free(am);
  return steps;
}

/* The outer loop of Algorithm 1 for one sequence whose prompt is cached: block after block starts fully masked,
 * is denoised by oracle_generate_block and, once decoded, is run through the forward again so that its K,V are
 * those of its final ids.  Early termination (Section 3, system optimisations, diffusion iterations): once a
 * decoded block contains eos_id the loop stops and the remaining blocks are filled with eos_id (eos_id < 0: never).
 * out [n_blocks * block_len]; returns the number of blocks that were decoded, -1 on failure. */
int32_t oracle_generate(const oracle_config* c, const oracle_weights* w, int block_len, int n_blocks, int prefix_len,
                        double* kcache, double* vcache, int cache_cap, double threshold, int fixed_k, int32_t mask_id,
                        int32_t eos_id, int32_t* out, int32_t* steps_per_block) {
  double* hidden = (double*)malloc(sizeof(double) * (size_t)block_len * c->hidden);
  int32_t done = 0;
  int stop = 0;
  for (int b = 0; b < n_blocks; ++b) {
    int32_t* blk = out + (size_t)b * block_len;
    if (stop) {
      for (int i = 0; i < block_len; ++i) blk[i] = eos_id;
      continue;
    }
    for (int i = 0; i < block_len; ++i) blk[i] = mask_id;
    uint64_t mask = block_len == 64 ? ~(uint64_t)0 : (((uint64_t)1 << block_len) - 1);
    const int P = prefix_len + b * block_len;
    const int32_t steps = oracle_generate_block(c, w, block_len, blk, &mask, P, kcache, vcache, cache_cap, threshold,
                                                fixed_k, block_len, NULL);
    if (steps < 0 || mask != 0 || oracle_forward(c, w, block_len, blk, P, kcache, vcache, cache_cap, hidden, NULL) != 0) {
      done = -1;
      break;
    }
    if (steps_per_block) steps_per_block[b] = steps;
    ++done;
    for (int i = 0; i < block_len; ++i)
      if (eos_id >= 0 && blk[i] == eos_id) stop = 1;
  }
  free(hidden);
  return done;
}
