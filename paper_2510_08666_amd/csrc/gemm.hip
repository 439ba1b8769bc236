// The dense contractions of the step as weight-streaming MFMA kernels (core in gemm.hpp):
//   QKV projection + rotary embedding + KV-page write, output projection + residual,
//   routed-expert grouped GEMMs (gate/up + SwiGLU, down), LM head + streaming max / arg max / sum-exp.
#include "gemm.hpp"
#include "kernels.hpp"

namespace dinfer {

// ------------------------------------------------------------------------------------------------
// Split-K kernel for the attention-side projections: one workgroup per (token group, task); its KSPLIT
// waves each stream a K slice of the task's weights, partial tiles are summed through LDS in wave order
// (deterministic), wave 0 runs the epilogue.
// ------------------------------------------------------------------------------------------------
template <typename E> struct QkvEpi {
  E* q;
  int64_t q_plane;
  E* kv_layer;
  KvGeom geom;
  const int32_t* tok_seq;
  const int32_t* tok_pos;
  const int32_t* page_table;
  int pt_stride;
  const float* cos_tab;
  const float* sin_tab;
  int D;   // n_heads * head_dim

  __device__ void operator()(int task, int tok, bool valid, int half, const f32x16& a0, const f32x16& a1) const {
    if (!valid) return;
    const int hd = geom.head_dim;
    const int per_head = hd / 64;
    const int qk_tasks = geom.n_heads * per_head;
    const int pos = tok_pos[tok];
    const int page = safe_page(geom, page_table[(int64_t)tok_seq[tok] * pt_stride + pos / PAGE]);
    const int slot = pos % PAGE;
    if (task < 2 * qk_tasks) {
      // rotary pair: a0 holds feature j of the head, a1 feature j + hd/2
      const bool is_k = task >= qk_tasks;
      const int r = is_k ? task - qk_tasks : task;
      const int head = r / per_head, jt = r % per_head;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int j0 = jt * TILE + acc_row(4 * g, half);   // 4 consecutive features j0..j0+3
        float lo[4], hi[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float c = cos_tab[(int64_t)pos * (hd / 2) + j0 + i];
          const float s = sin_tab[(int64_t)pos * (hd / 2) + j0 + i];
          const float a = a0[4 * g + i], b = a1[4 * g + i];
          lo[i] = a * c - b * s;
          hi[i] = b * c + a * s;
        }
        if (is_k) {
          E* dst = kv_layer + kv_k_index(geom, page, head, slot, j0);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            dst[i] = from_f32<E>(lo[i]);
            dst[hd / 2 + i] = from_f32<E>(hi[i]);
          }
        } else {
          const int64_t dst = (int64_t)tok * D + head * hd + j0;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            store_act<E>(q, dst + i, q_plane, lo[i]);
            store_act<E>(q, dst + hd / 2 + i, q_plane, hi[i]);
          }
        }
      }
    } else {
      const int t = task - 2 * qk_tasks;   // adjacent tiles 2t, 2t+1 of V
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int f0 = (2 * t) * TILE + acc_row(v, half);
        const int f1 = f0 + TILE;
        kv_layer[kv_v_index(geom, page, f0 / hd, slot, f0 % hd)] = from_f32<E>(a0[v]);
        kv_layer[kv_v_index(geom, page, f1 / hd, slot, f1 % hd)] = from_f32<E>(a1[v]);
      }
    }
  }
};

struct ResidualEpi {
  float* x;
  int H;
  __device__ void operator()(int task, int tok, bool valid, int half, const f32x16& a0, const f32x16& a1) const {
    if (!valid) return;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float* p0 = x + (int64_t)tok * H + (2 * task) * TILE + acc_row(4 * g, half);
      float* p1 = p0 + TILE;
      f32x4 r0 = *reinterpret_cast<f32x4*>(p0), r1 = *reinterpret_cast<f32x4*>(p1);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        r0[i] += a0[4 * g + i];
        r1[i] += a1[4 * g + i];
      }
      *reinterpret_cast<f32x4*>(p0) = r0;
      *reinterpret_cast<f32x4*>(p1) = r1;
    }
  }
};

// Router: the single task holds experts 0-31 (tile 0) and 32-63 (tile 1).  A token's 64 probabilities sit in
// the two lanes l and l^32; softmax and the k selection rounds combine the pair with one shuffle each.
struct RouterEpi {
  int n_exp, top_k, norm_topk;
  int32_t* topk_idx;
  float* topk_w;
  __device__ void operator()(int /*task*/, int tok, bool valid, int half, const f32x16& a0, const f32x16& a1) const {
    float p[32];
    int id[32];
    float m = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) {      // ids ascend with the index within each lane
      id[v] = acc_row(v, half);
      id[16 + v] = TILE + acc_row(v, half);
      p[v] = id[v] < n_exp ? a0[v] : -INFINITY;
      p[16 + v] = id[16 + v] < n_exp ? a1[v] : -INFINITY;
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) m = fmaxf(m, p[i]);
    m = fmaxf(m, __shfl_xor(m, 32, WAVE));
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      p[i] = id[i] < n_exp ? expf(p[i] - m) : 0.f;
      sum += p[i];
    }
    sum += __shfl_xor(sum, 32, WAVE);
    const float inv = 1.f / sum;
#pragma unroll
    for (int i = 0; i < 32; ++i) p[i] = id[i] < n_exp ? p[i] * inv : -1.f;
    float wsel[MAX_TOPK];
    int isel[MAX_TOPK];
    float sel_sum = 0.f;
#pragma unroll
    for (int j = 0; j < MAX_TOPK; ++j) {
      if (j < top_k) {
        float bv = -1.f;
        int bi = 0x7fffffff, slot = 0;
#pragma unroll
        for (int i = 0; i < 32; ++i)
          if (p[i] > bv) {
            bv = p[i];
            bi = id[i];
            slot = i;
          }
        const float ov = __shfl_xor(bv, 32, WAVE);
        const int oi = __shfl_xor(bi, 32, WAVE);
        const bool mine = bv > ov || (bv == ov && bi < oi);
        wsel[j] = mine ? bv : ov;
        isel[j] = mine ? bi : oi;
        sel_sum += wsel[j];
        if (mine) {
#pragma unroll
          for (int i = 0; i < 32; ++i)
            if (i == slot) p[i] = -1.f;
        }
      }
    }
    if (valid && half == 0) {
#pragma unroll
      for (int j = 0; j < MAX_TOPK; ++j)
        if (j < top_k) {
          topk_idx[tok * top_k + j] = isel[j];
          topk_w[tok * top_k + j] = norm_topk ? wsel[j] / sel_sum : wsel[j];
        }
    }
  }
};

template <typename E, int TT, int KSPLIT, class Epi>
__global__ __launch_bounds__(KSPLIT * WAVE) void gemm_ksplit_kernel(const E* __restrict__ W, int ksteps,
                                                                     const E* __restrict__ X, int64_t plane,
                                                                     int T, int K, Epi epi) {
  extern __shared__ float red[];   // [KSPLIT-1][2*TT*16][64]
  constexpr int G = ET<E>::G;
  const int task = blockIdx.y, group = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int tok0 = group * TT * TILE;
  const E* bp[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int tok = min(tok0 + t * TILE + (lane & 31), T - 1);
    bp[t] = X + (int64_t)tok * K + half * G;
  }
  f32x16 acc0[TT], acc1[TT];
  zero_acc<TT>(acc0);
  zero_acc<TT>(acc1);
  const int per = (ksteps + KSPLIT - 1) / KSPLIT;
  const int ks0 = wave * per, ks1 = min(ksteps, ks0 + per);
  if (ks0 < ks1)
    stream_task<E, TT, (TT == 1 ? 8 : 4)>(W + (int64_t)task * task_stride_elems<E>(ksteps), ks0, ks1, bp, plane, acc0,
                                          acc1);
  if (KSPLIT > 1) {
    if (wave > 0) {
      float* r = red + (int64_t)(wave - 1) * (2 * TT * 16) * WAVE + lane;
#pragma unroll
      for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          r[(t * 32 + v) * WAVE] = acc0[t][v];
          r[(t * 32 + 16 + v) * WAVE] = acc1[t][v];
        }
    }
    __syncthreads();
    if (wave == 0) {
      for (int w = 1; w < KSPLIT; ++w) {
        const float* r = red + (int64_t)(w - 1) * (2 * TT * 16) * WAVE + lane;
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            acc0[t][v] += r[(t * 32 + v) * WAVE];
            acc1[t][v] += r[(t * 32 + 16 + v) * WAVE];
          }
      }
    }
  }
  if (wave == 0) {
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      const int tok = tok0 + t * TILE + (lane & 31);
      epi(task, tok, tok < T, half, acc0[t], acc1[t]);
    }
  }
}

template <int TT, int KSPLIT> constexpr size_t ksplit_lds() { return (size_t)(KSPLIT - 1) * 2 * TT * 16 * WAVE * 4; }

template <typename E, class Epi>
static void launch_ksplit(const E* W, int ksteps, const E* X, int64_t plane, int T, int K, int n_tasks,
                          const Epi& epi, hipStream_t st) {
  if (T <= 32) {
    gemm_ksplit_kernel<E, 1, 8, Epi><<<dim3(1, n_tasks), 8 * WAVE, ksplit_lds<1, 8>(), st>>>(W, ksteps, X, plane, T, K, epi);
  } else if (T <= 64) {
    gemm_ksplit_kernel<E, 2, 4, Epi><<<dim3(1, n_tasks), 4 * WAVE, ksplit_lds<2, 4>(), st>>>(W, ksteps, X, plane, T, K, epi);
  } else {
    const int groups = (T + 4 * TILE - 1) / (4 * TILE);
    gemm_ksplit_kernel<E, 4, 4, Epi><<<dim3(groups, n_tasks), 4 * WAVE, ksplit_lds<4, 4>(), st>>>(W, ksteps, X, plane, T, K, epi);
  }
}

template <typename E, class Epi> static void configure_ksplit() {
  (void)hipFuncSetAttribute((const void*)gemm_ksplit_kernel<E, 1, 8, Epi>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)ksplit_lds<1, 8>());
  (void)hipFuncSetAttribute((const void*)gemm_ksplit_kernel<E, 2, 4, Epi>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)ksplit_lds<2, 4>());
  (void)hipFuncSetAttribute((const void*)gemm_ksplit_kernel<E, 4, 4, Epi>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)ksplit_lds<4, 4>());
}

template <typename E> static void launch_qkv_t(const QkvArgs& a, hipStream_t st) {
  const int D = a.geom.n_heads * a.geom.head_dim;
  QkvEpi<E> epi{(E*)a.q, a.q_plane, (E*)a.kv_layer, a.geom, a.meta.tok_seq, a.meta.tok_pos, a.page_table, a.pt_stride,
                a.cos_tab, a.sin_tab, D};
  launch_ksplit<E>((const E*)a.w, a.H / ET<E>::KS, (const E*)a.h, a.act_plane, a.T, a.H, 3 * D / 64, epi, st);
}
void launch_qkv(bool bf16, const QkvArgs& a, hipStream_t st) {
  if (bf16) launch_qkv_t<bf16_t>(a, st);
  else launch_qkv_t<float>(a, st);
}

void launch_oproj(bool bf16, const void* w, const void* a, int64_t act_plane, float* x, int T, int D, int H,
                  hipStream_t st) {
  ResidualEpi epi{x, H};
  if (bf16) launch_ksplit<bf16_t>((const bf16_t*)w, D / 16, (const bf16_t*)a, act_plane, T, D, H / 64, epi, st);
  else launch_ksplit<float>((const float*)w, D / 8, (const float*)a, act_plane, T, D, H / 64, epi, st);
}

void launch_router(bool bf16, const void* w_router_packed, const void* h, int64_t h_plane, int T, int H, int E,
                   int top_k, int norm_topk, int32_t* topk_idx, float* topk_w, hipStream_t st) {
  RouterEpi epi{E, top_k, norm_topk, topk_idx, topk_w};
  if (bf16) launch_ksplit<bf16_t>((const bf16_t*)w_router_packed, H / 16, (const bf16_t*)h, h_plane, T, H, 1, epi, st);
  else launch_ksplit<float>((const float*)w_router_packed, H / 8, (const float*)h, h_plane, T, H, 1, epi, st);
}

// ------------------------------------------------------------------------------------------------
// Routed experts.  Rows of expert e are the pairs perm[off[e] .. off[e]+cnt[e]) (pair = token*top_k + slot).
// One wave per (expert, task, row group); experts without rows exit at once.
//   GEMM 1: task = 32 gate features + the same 32 up features;  y = silu(gate) * up   -> Y[sorted row][I]
//   GEMM 2: task = 64 adjacent output features of the down projection                  -> O[sorted row][H]
// ------------------------------------------------------------------------------------------------
__device__ inline float silu_f(float x) { return x / (1.f + __expf(-x)); }

template <typename E, int TT>
__global__ __launch_bounds__(256) void expert_gemm1_kernel(const E* __restrict__ W, const E* __restrict__ Hn,
                                                            E* __restrict__ Y, const int32_t* __restrict__ cnt,
                                                            const int32_t* __restrict__ off,
                                                            const int32_t* __restrict__ perm, int H, int I,
                                                            int top_k, int64_t h_plane, int64_t y_plane) {
  constexpr int G = ET<E>::G;
  const int e = blockIdx.y, group = blockIdx.z;
  const int n_rows = cnt[e];
  const int row0 = group * TT * TILE;
  if (row0 >= n_rows) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int task = blockIdx.x * 4 + wave;
  const int n_tasks = I / TILE;
  if (task >= n_tasks) return;
  const int base = off[e];
  const E* bp[TT];
  int row[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    row[t] = row0 + t * TILE + (lane & 31);
    const int pair = perm[base + min(row[t], n_rows - 1)];
    bp[t] = Hn + (int64_t)(pair / top_k) * H + half * G;
  }
  f32x16 acc0[TT], acc1[TT];
  zero_acc<TT>(acc0);
  zero_acc<TT>(acc1);
  const int ksteps = H / ET<E>::KS;
  stream_task<E, TT, (TT == 1 ? 8 : 4)>(W + ((int64_t)e * n_tasks + task) * task_stride_elems<E>(ksteps), 0, ksteps, bp, h_plane, acc0,
                        acc1);
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    if (row[t] < n_rows) {
      E* yrow = Y + (int64_t)(base + row[t]) * I + task * TILE;
#pragma unroll
      for (int v = 0; v < 16; ++v) store_act<E>(yrow, acc_row(v, half), y_plane, silu_f(acc0[t][v]) * acc1[t][v]);
    }
  }
}

template <typename E, int TT>
__global__ __launch_bounds__(256) void expert_gemm2_kernel(const E* __restrict__ W, const E* __restrict__ Y,
                                                            float* __restrict__ O, const int32_t* __restrict__ cnt,
                                                            const int32_t* __restrict__ off, int H, int I,
                                                            int64_t y_plane) {
  constexpr int G = ET<E>::G;
  const int e = blockIdx.y, group = blockIdx.z;
  const int n_rows = cnt[e];
  const int row0 = group * TT * TILE;
  if (row0 >= n_rows) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int task = blockIdx.x * 4 + wave;
  const int n_tasks = H / (2 * TILE);
  if (task >= n_tasks) return;
  const int base = off[e];
  const E* bp[TT];
  int row[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    row[t] = row0 + t * TILE + (lane & 31);
    bp[t] = Y + (int64_t)(base + min(row[t], n_rows - 1)) * I + half * G;
  }
  f32x16 acc0[TT], acc1[TT];
  zero_acc<TT>(acc0);
  zero_acc<TT>(acc1);
  const int ksteps = I / ET<E>::KS;
  stream_task<E, TT, (TT == 1 ? 8 : 4)>(W + ((int64_t)e * n_tasks + task) * task_stride_elems<E>(ksteps), 0, ksteps, bp, y_plane, acc0,
                        acc1);
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    if (row[t] < n_rows) {
      float* orow = O + (int64_t)(base + row[t]) * H + (2 * task) * TILE;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 r0, r1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          r0[i] = acc0[t][4 * g + i];
          r1[i] = acc1[t][4 * g + i];
        }
        *reinterpret_cast<f32x4*>(orow + acc_row(4 * g, half)) = r0;
        *reinterpret_cast<f32x4*>(orow + TILE + acc_row(4 * g, half)) = r1;
      }
    }
  }
}

template <typename E, int TT> static void launch_gate_up_t(const ExpertArgs& a, int groups, hipStream_t st) {
  const int t1 = a.I / TILE;
  expert_gemm1_kernel<E, TT><<<dim3((t1 + 3) / 4, a.E, groups), 256, 0, st>>>(
      (const E*)a.w_gate_up, (const E*)a.h, (E*)a.y, a.cnt, a.off, a.perm, a.H, a.I, a.top_k, a.h_plane, a.y_plane);
}
template <typename E, int TT> static void launch_down_t(const ExpertArgs& a, int groups, hipStream_t st) {
  const int t2 = a.H / (2 * TILE);
  expert_gemm2_kernel<E, TT><<<dim3((t2 + 3) / 4, a.E, groups), 256, 0, st>>>(
      (const E*)a.w_down, (const E*)a.y, a.o, a.cnt, a.off, a.H, a.I, a.y_plane);
}

// An expert can receive at most T rows (a token selects an expert at most once): T fixes the row tiling.
#define DINFER_EXPERT_DISPATCH(FN)                                                              \
  if (a.T <= 32) {                                                                              \
    if (bf16) FN<bf16_t, 1>(a, 1, st); else FN<float, 1>(a, 1, st);                             \
  } else if (a.T <= 64) {                                                                       \
    if (bf16) FN<bf16_t, 2>(a, 1, st); else FN<float, 2>(a, 1, st);                             \
  } else {                                                                                      \
    const int groups = (a.T + 4 * TILE - 1) / (4 * TILE);                                       \
    if (bf16) FN<bf16_t, 4>(a, groups, st); else FN<float, 4>(a, groups, st);                   \
  }

void launch_expert_gate_up(bool bf16, const ExpertArgs& a, hipStream_t st) { DINFER_EXPERT_DISPATCH(launch_gate_up_t) }
void launch_expert_down(bool bf16, const ExpertArgs& a, hipStream_t st) { DINFER_EXPERT_DISPATCH(launch_down_t) }

// ------------------------------------------------------------------------------------------------
// LM head fused with the confidence reduction.  Each wave walks tasks (64 vocabulary ids each) and keeps,
// per token column, the running maximum logit, its lowest id, and sum exp(z - max); logits are never stored
// (unless the debug pointer is set).  One partial (max, sum, id) per (wave, token) is written at the end.
// ------------------------------------------------------------------------------------------------
template <typename E, int TT>
__global__ __launch_bounds__(256) void lm_head_kernel(const E* __restrict__ W, const E* __restrict__ Hn, int T,
                                                       int H, int V, float scale, float* __restrict__ part,
                                                       int n_waves, float* __restrict__ logits_out, int64_t plane) {
  constexpr int G = ET<E>::G;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63, half = lane >> 5;
  const int group = blockIdx.y;
  const int tok0 = group * TT * TILE;
  const int n_tasks = (V + 2 * TILE - 1) / (2 * TILE);
  const int ksteps = H / ET<E>::KS;
  const E* bp[TT];
  float m[TT], s[TT];
  int best[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int tok = min(tok0 + t * TILE + (lane & 31), T - 1);
    bp[t] = Hn + (int64_t)tok * H + half * G;
    m[t] = -INFINITY;
    s[t] = 0.f;
    best[t] = 0x7fffffff;
  }
  for (int task = wave; task < n_tasks; task += n_waves) {
    f32x16 acc0[TT], acc1[TT];
    zero_acc<TT>(acc0);
    zero_acc<TT>(acc1);
    stream_task<E, TT, (TT == 1 ? 8 : 4)>(W + (int64_t)task * task_stride_elems<E>(ksteps), 0, ksteps, bp, plane, acc0, acc1);
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      const int tok = tok0 + t * TILE + (lane & 31);
      // this lane's 32 logits of the task, ids ascending within each tile
      float z[32];
      int id[32];
      float tm = -INFINITY;
      int ti = 0x7fffffff;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        id[v] = (2 * task) * TILE + acc_row(v, half);
        id[16 + v] = id[v] + TILE;
        z[v] = id[v] < V ? acc0[t][v] * scale : -INFINITY;
        z[16 + v] = id[16 + v] < V ? acc1[t][v] * scale : -INFINITY;
      }
#pragma unroll
      for (int v = 0; v < 32; ++v)
        if (z[v] > tm) {          // ids ascend with v, so strict '>' keeps the lowest id
          tm = z[v];
          ti = id[v];
        }
      if (logits_out && tok < T) {
#pragma unroll
        for (int v = 0; v < 32; ++v)
          if (id[v] < V) logits_out[(int64_t)tok * V + id[v]] = z[v];
      }
      if (tm > m[t] || (tm == m[t] && ti < best[t])) {
        s[t] *= __expf(m[t] - tm);      // exp(-inf) = 0 on the first task
        m[t] = tm;
        best[t] = ti;
      }
      if (m[t] > -INFINITY) {
#pragma unroll
        for (int v = 0; v < 32; ++v) s[t] += __expf(z[v] - m[t]);
      }
    }
  }
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    // fold the two half-waves (same token, other rows)
    const float om = __shfl_xor(m[t], 32, WAVE), os = __shfl_xor(s[t], 32, WAVE);
    const int ob = __shfl_xor(best[t], 32, WAVE);
    float M = m[t], S = s[t];
    int B = best[t];
    if (om > M || (om == M && ob < B)) {
      S = (M > -INFINITY ? S * __expf(M - om) : 0.f) + os;
      M = om;
      B = ob;
    } else if (om > -INFINITY) {
      S += os * __expf(om - M);
    }
    const int tok = tok0 + t * TILE + (lane & 31);
    if (half == 0 && tok < T) {
      float* p = part + ((int64_t)wave * T + tok) * 4;
      p[0] = M;
      p[1] = S;
      p[2] = __int_as_float(B);
      p[3] = 0.f;
    }
  }
}

int lm_head_waves(int V) {
  const int n_tasks = (V + 63) / 64;
  int wgs = (n_tasks + 3) / 4;          // one task per wave while that keeps the partial table small
  if (wgs > 768) wgs = 768;
  if (wgs < 1) wgs = 1;
  return wgs * 4;
}

template <typename E> static void launch_lm_t(const LmArgs& a, hipStream_t st) {
  const int wgs = a.n_lm_waves / 4;
  if (a.T <= 32) {
    lm_head_kernel<E, 1><<<dim3(wgs, 1), 256, 0, st>>>((const E*)a.w, (const E*)a.h, a.T, a.H, a.V, a.scale, a.part,
                                                        a.n_lm_waves, a.logits_out, a.act_plane);
  } else if (a.T <= 64) {
    lm_head_kernel<E, 2><<<dim3(wgs, 1), 256, 0, st>>>((const E*)a.w, (const E*)a.h, a.T, a.H, a.V, a.scale, a.part,
                                                        a.n_lm_waves, a.logits_out, a.act_plane);
  } else {
    // token groups of 128 rows: the partials of group g live in rows [g*128, ...) of the same table
    const int groups = (a.T + 4 * TILE - 1) / (4 * TILE);
    lm_head_kernel<E, 4><<<dim3(wgs, groups), 256, 0, st>>>((const E*)a.w, (const E*)a.h, a.T, a.H, a.V, a.scale,
                                                             a.part, a.n_lm_waves, a.logits_out, a.act_plane);
  }
}
void launch_lm_head(bool bf16, const LmArgs& a, hipStream_t st) {
  if (bf16) launch_lm_t<bf16_t>(a, st);
  else launch_lm_t<float>(a, st);
}

void configure_kernels() {
  configure_ksplit<bf16_t, QkvEpi<bf16_t>>();
  configure_ksplit<float, QkvEpi<float>>();
  configure_ksplit<bf16_t, ResidualEpi>();
  configure_ksplit<float, ResidualEpi>();
  configure_ksplit<bf16_t, RouterEpi>();
  configure_ksplit<float, RouterEpi>();
}

}  // namespace dinfer
