// The dense contractions of the step as weight-streaming MFMA kernels (core in gemm.hpp):
//   QKV projection + rotary embedding + KV-page write, output projection + residual,
//   router + top-k (+ token->expert permutation), routed-expert grouped GEMMs (gate/up + SwiGLU, down),
//   LM head + streaming max / arg max / sum-exp.
// RMSNorm is never materialised.  Whoever produces a residual row also stores it multiplied by the gain of the
// norm that follows, as MFMA-ready planes ("normalised-input planes", without the 1/rms factor); the consumers
// feed those planes to the matrix cores and scale their accumulators by the row's 1/rms in the epilogue.
#include "gemm.hpp"
#include "kernels.hpp"
#include "wide_stream.hpp"

namespace dinfer {

// ------------------------------------------------------------------------------------------------
// Split-K kernel for the attention-side projections.  A task (64 output features) of one token group is shared
// by `slices` workgroups of KW waves; every wave streams its own K range.  The partial tiles of a workgroup are
// summed through LDS in wave order; with more than one slice the workgroup sums go to global memory and the
// workgroup that arrives last adds them in slice order (so the result does not depend on scheduling) and runs
// the epilogue.  At small token counts the host picks the slices so that a wave's whole K range is in flight at
// once: these kernels are bound by memory latency, not bandwidth, and every further dependent round trip
// costs microseconds.
// ------------------------------------------------------------------------------------------------
// Epilogues receive, for one token (lane) and one accumulator tile pair, PER consecutive accumulator registers
// v0 .. v0+PER-1 of tile 0 (a0) and tile 1 (a1): rows acc_row(v0, half) .. +PER-1 of each tile, which are PER
// consecutive features (v0 is a multiple of PER, PER divides 4).  apply() returns the lane's contribution to the
// row statistic of the epilogue (ROWSUM), which the kernel sums over the task and hands to row_sum().
template <typename E> struct QkvEpi {
  static constexpr bool ROWSUM = false;
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
  RowNorm norm;        // statistics of the tokens' residual rows
  int T, H;
  int D;               // n_heads * head_dim

  // What the epilogue needs from memory besides the accumulators.  prefetch() runs before the weight stream
  // starts and issues only loads whose addresses are known then; prefetch2() runs behind the stream and issues
  // the loads that depend on the first ones, so that they are under way while the partial sums are folded.
  template <int PER> struct Pre {
    int pos, seq, page, tok;
    float r;
    float c[PER], s[PER];
  };
  template <int PER> __device__ Pre<PER> prefetch(int, int tok, bool valid, int, int) const {
    Pre<PER> p;
    const int t = valid ? tok : 0;
    p.pos = tok_pos[t];
    p.seq = tok_seq[t];
    p.tok = t;
    return p;
  }
  template <int PER> __device__ void prefetch2(Pre<PER>& p, int task, int half, int v0) const {
    const int hd = geom.head_dim;
    p.r = row_rinv(norm.ssq, norm.n_ssq, T, p.tok, H, norm.eps);   // up to 32 loads: kept behind the weight stream
    p.page = page_table[(int64_t)p.seq * pt_stride + p.pos / PAGE];
    const int j0 = (task % (hd / 64)) * TILE + acc_row(v0, half);
    const bool rot = task < 2 * geom.n_heads * (hd / 64);
    if constexpr (PER == 4) {   // j0 is a multiple of 4: one 16-byte load per table
      const f32x4 c4 = *reinterpret_cast<const f32x4*>(cos_tab + (int64_t)p.pos * (hd / 2) + (rot ? j0 : 0));
      const f32x4 s4 = *reinterpret_cast<const f32x4*>(sin_tab + (int64_t)p.pos * (hd / 2) + (rot ? j0 : 0));
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p.c[i] = rot ? c4[i] : 1.f;
        p.s[i] = rot ? s4[i] : 0.f;
      }
    } else {
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        p.c[i] = rot ? cos_tab[(int64_t)p.pos * (hd / 2) + j0 + i] : 1.f;
        p.s[i] = rot ? sin_tab[(int64_t)p.pos * (hd / 2) + j0 + i] : 0.f;
      }
    }
  }

  template <int PER>
  __device__ float apply(const Pre<PER>& pre, int task, int tok, bool valid, int half, int v0, const float (&a0)[PER],
                         const float (&a1)[PER]) const {
    if (!valid) return 0.f;
    const int hd = geom.head_dim;
    const int per_head = hd / 64;
    const int qk_tasks = geom.n_heads * per_head;
    const int page = safe_page(geom, pre.page);
    const int slot = pre.pos % PAGE;
    const float r = pre.r;
    const int row0 = acc_row(v0, half);
    if (task < 2 * qk_tasks) {
      // rotary pair: a0 holds feature j of the head, a1 feature j + hd/2
      const bool is_k = task >= qk_tasks;
      const int rr = is_k ? task - qk_tasks : task;
      const int head = rr / per_head, jt = rr % per_head;
      const int j0 = jt * TILE + row0;
      float lo[PER], hi[PER];
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const float a = a0[i] * r, b = a1[i] * r;
        lo[i] = a * pre.c[i] - b * pre.s[i];
        hi[i] = b * pre.c[i] + a * pre.s[i];
      }
      if (is_k) {
        // (PER consecutive features starting at a multiple of PER stay inside one 32-byte block of the K layout)
        E* dst = kv_layer + kv_k_index(geom, page, head, slot, j0);
        E* dst_hi = kv_layer + kv_k_index(geom, page, head, slot, j0 + hd / 2);
        if constexpr (PER == 4) {
          store_elems4<E>(dst, f32x4{lo[0], lo[1], lo[2], lo[3]});
          store_elems4<E>(dst_hi, f32x4{hi[0], hi[1], hi[2], hi[3]});
        } else {
#pragma unroll
          for (int i = 0; i < PER; ++i) {
            dst[i] = from_f32<E>(lo[i]);
            dst_hi[i] = from_f32<E>(hi[i]);
          }
        }
      } else {
        const int64_t dst = (int64_t)tok * D + head * hd + j0;
        if constexpr (PER == 4) {
          store_act4<E>(q, dst, q_plane, f32x4{lo[0], lo[1], lo[2], lo[3]});
          store_act4<E>(q, dst + hd / 2, q_plane, f32x4{hi[0], hi[1], hi[2], hi[3]});
        } else {
#pragma unroll
          for (int i = 0; i < PER; ++i) {
            store_act<E>(q, dst + i, q_plane, lo[i]);
            store_act<E>(q, dst + hd / 2 + i, q_plane, hi[i]);
          }
        }
      }
    } else {
      const int t = task - 2 * qk_tasks;   // adjacent tiles 2t, 2t+1 of V
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int f0 = (2 * t) * TILE + row0 + i;
        const int f1 = f0 + TILE;
        kv_layer[kv_v_index(geom, page, f0 / hd, slot, f0 % hd)] = from_f32<E>(a0[i] * r);
        kv_layer[kv_v_index(geom, page, f1 / hd, slot, f1 % hd)] = from_f32<E>(a1[i] * r);
      }
    }
    return 0.f;
  }
  __device__ void row_sum(int, int, float) const {}
};

// x += result; the new row also goes out as normalised-input planes for the expert half (times its norm's gain),
// and the task's share of the row's sum of squares to ssq[task][token].
template <typename E> struct ResidualEpi {
  static constexpr bool ROWSUM = true;
  float* x;
  int H;
  const float* gain;   // [H] gain of the norm that follows
  E* xn;               // [T][H] k-major planes
  float* ssq;          // [H/64][T]
  int T;

  template <int PER> struct Pre {
    float x0[PER], x1[PER], g0[PER], g1[PER];
  };
  template <int PER> __device__ Pre<PER> prefetch(int task, int tok, bool valid, int half, int v0) const {
    Pre<PER> p;
    const int col = (2 * task) * TILE + acc_row(v0, half);
    const float* p0 = x + (int64_t)(valid ? tok : 0) * H + col;
    if constexpr (PER == 4) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(p0), b = *reinterpret_cast<const f32x4*>(p0 + TILE);
      const f32x4 c = *reinterpret_cast<const f32x4*>(gain + col), d = *reinterpret_cast<const f32x4*>(gain + col + TILE);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p.x0[i] = a[i];
        p.x1[i] = b[i];
        p.g0[i] = c[i];
        p.g1[i] = d[i];
      }
      return p;
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      p.x0[i] = p0[i];
      p.x1[i] = p0[TILE + i];
      p.g0[i] = gain[col + i];
      p.g1[i] = gain[col + TILE + i];
    }
    return p;
  }
  template <int PER> __device__ void prefetch2(Pre<PER>&, int, int, int) const {}

  template <int PER>
  __device__ float apply(const Pre<PER>& pre, int task, int tok, bool valid, int half, int v0, const float (&a0)[PER],
                         const float (&a1)[PER]) const {
    if (!valid) return 0.f;
    const int col = (2 * task) * TILE + acc_row(v0, half);
    float* p0 = x + (int64_t)tok * H + col;
    float ss = 0.f;
    if constexpr (PER == 4) {
      f32x4 n0, n1, m0, m1;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        n0[i] = pre.x0[i] + a0[i];
        n1[i] = pre.x1[i] + a1[i];
        m0[i] = n0[i] * pre.g0[i];
        m1[i] = n1[i] * pre.g1[i];
        ss += n0[i] * n0[i] + n1[i] * n1[i];
      }
      *reinterpret_cast<f32x4*>(p0) = n0;
      *reinterpret_cast<f32x4*>(p0 + TILE) = n1;
      store_actk4<E>(xn, T, tok, col, m0);
      store_actk4<E>(xn, T, tok, col + TILE, m1);
      return ss;
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const float n0 = pre.x0[i] + a0[i], n1 = pre.x1[i] + a1[i];
      p0[i] = n0;
      p0[TILE + i] = n1;
      store_actk<E>(xn, T, tok, col + i, n0 * pre.g0[i]);
      store_actk<E>(xn, T, tok, col + TILE + i, n1 * pre.g1[i]);
      ss += n0 * n0 + n1 * n1;
    }
    return ss;
  }
  __device__ void row_sum(int task, int tok, float s) const { ssq[(int64_t)task * T + tok] = s; }
};

// Iteration smoothing: the contraction of the probabilities with the embedding matrix; a row of a position that
// is still masked receives the expected embedding, the other rows are left alone.
struct SmoothEpi {
  static constexpr bool ROWSUM = false;
  float* delta;         // [T][H]
  int H;
  const uint64_t* mask;
  int block_len;
  template <int PER> struct Pre {
    bool on;
  };
  template <int PER> __device__ Pre<PER> prefetch(int, int tok, bool valid, int, int) const {
    Pre<PER> p;
    p.on = valid && ((mask[tok / block_len] >> (tok % block_len)) & 1ull);
    return p;
  }
  template <int PER> __device__ void prefetch2(Pre<PER>&, int, int, int) const {}
  template <int PER>
  __device__ float apply(const Pre<PER>& pre, int task, int tok, bool, int half, int v0, const float (&a0)[PER],
                         const float (&a1)[PER]) const {
    if (!pre.on) return 0.f;
    float* p0 = delta + (int64_t)tok * H + (2 * task) * TILE + acc_row(v0, half);
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      p0[i] = a0[i];
      p0[TILE + i] = a1[i];
    }
    return 0.f;
  }
  __device__ void row_sum(int, int, float) const {}
};

// Every wave leaves its partial accumulators in LDS: red[wave][t*32 + tile*16 + v][lane].
template <int TT, int ROWS>
__device__ inline void spill_partials(float* red, int wave, int lane, const f32x16 (&acc0)[TT], const f32x16 (&acc1)[TT]) {
  float* r = red + (int64_t)wave * ROWS * WAVE + lane;
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      r[(t * 32 + v) * WAVE] = acc0[t][v];
      r[(t * 32 + 16 + v) * WAVE] = acc1[t][v];
    }
}

// Sum over the KW waves' partials in LDS: wave w takes accumulator registers w*PER .. w*PER+PER-1 of both tiles.
template <int TT, int KW, int PER>
__device__ inline void fold_partials(const float* red, int lane, int v0, float (&a0)[TT][PER], float (&a1)[TT][PER]) {
  constexpr int ROWS = 2 * TT * 16;
#pragma unroll
  for (int t = 0; t < TT; ++t) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      a0[t][i] = 0.f;
      a1[t][i] = 0.f;
    }
    for (int w = 0; w < KW; ++w) {
      const float* r = red + ((int64_t)w * ROWS + t * 32 + v0) * WAVE + lane;
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        a0[t][i] += r[i * WAVE];
        a1[t][i] += r[(16 + i) * WAVE];
      }
    }
  }
}

// The workgroup's sums leave for / come back from the cross-workgroup buffer.  A thread holds PER consecutive
// accumulator registers (v0 .. v0+PER-1) of each tile; they travel as one PER-float piece:
//   part[unit][slice][token tile][weight tile][v0 / PER][lane][PER]
// Writer and reader are the same (wave, lane) of their workgroups, so each reads what its counterpart wrote.
template <int TT, int PER> __device__ inline uint32_t slice_piece(int64_t unit_slice, int t, int tile, int v0, int lane) {
  return (uint32_t)(((((unit_slice * TT + t) * 2 + tile) * (16 / PER) + v0 / PER) * WAVE + lane) * PER * sizeof(float));
}
template <int TT, int PER>
__device__ inline void put_slice(float* part, int64_t unit_slice, int lane, int v0, const float (&a0)[TT][PER],
                                 const float (&a1)[TT][PER]) {
  const buf_rsrc r = coherent_buffer(part);
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    coherent_store_n<PER>(r, slice_piece<TT, PER>(unit_slice, t, 0, v0, lane), a0[t]);
    coherent_store_n<PER>(r, slice_piece<TT, PER>(unit_slice, t, 1, v0, lane), a1[t]);
  }
}
// The loads of CH slices are issued together before any of them is added (a loop that loads and adds slice by
// slice pays one memory round trip per slice); the sum still runs in slice order.
template <int TT, int PER, int CH = 4>
__device__ inline void sum_slices(const float* part, int64_t unit, int n_slices, int lane, int v0, float (&a0)[TT][PER],
                                  float (&a1)[TT][PER]) {
  const buf_rsrc r = coherent_buffer(part);
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      a0[t][i] = 0.f;
      a1[t][i] = 0.f;
    }
  for (int s0 = 0; s0 < n_slices; s0 += CH) {
    float b0[CH][TT][PER], b1[CH][TT][PER];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int64_t us = unit * n_slices + min(s0 + c, n_slices - 1);
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        coherent_load_n<PER>(r, slice_piece<TT, PER>(us, t, 0, v0, lane), b0[c][t]);
        coherent_load_n<PER>(r, slice_piece<TT, PER>(us, t, 1, v0, lane), b1[c][t]);
      }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const bool on = s0 + c < n_slices;
#pragma unroll
      for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int i = 0; i < PER; ++i) {
          a0[t][i] += on ? b0[c][t][i] : 0.f;
          a1[t][i] += on ? b1[c][t][i] : 0.f;
        }
    }
  }
}

template <typename E, int TT, int KW, class Epi>
__global__ __launch_bounds__(KW * WAVE) void gemm_ksplit_kernel(const E* __restrict__ W, int ksteps,
                                                                 const E* __restrict__ B, int T, int K,
                                                                 float* __restrict__ part, int32_t* __restrict__ tickets,
                                                                 Epi epi, const int32_t* __restrict__ live) {
  if (step_is_dead(live)) return;
  extern __shared__ float red[];   // [KW][2*TT*16][64]
  __shared__ int32_t s_flag;
  constexpr int ROWS = 2 * TT * 16, PER = 16 / KW;
  [[maybe_unused]] constexpr int KID = Epi::ROWSUM ? 2 : 1;
  const int slice = blockIdx.x, n_slices = gridDim.x, task = blockIdx.y, group = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int tok0 = group * TT * TILE;
  TRACE_MARK(KID, 0);
  const int v0 = wave * PER;
  typename Epi::template Pre<PER> pre[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int tok = tok0 + t * TILE + (lane & 31);
    pre[t] = epi.template prefetch<PER>(task, tok, tok < T, half, v0);
  }
  f32x16 acc0[TT], acc1[TT];
  zero_acc<TT>(acc0);
  zero_acc<TT>(acc1);
  const int per = (ksteps + n_slices * KW - 1) / (n_slices * KW);
  const int ks0 = min(ksteps, (slice * KW + wave) * per), ks1 = min(ksteps, ks0 + per);
  PlaneLoader<E, TT> ld;
#pragma unroll
  for (int t = 0; t < TT; ++t) ld.set(t, B, T, min(tok0 + t * TILE + (lane & 31), T - 1), half);
  stream_task<E, TT, (TT == 1 ? 8 : 4)>(W + (int64_t)task * task_stride_elems<E>(ksteps), ks0, ks1, ld, acc0, acc1);
  TRACE_MARK(KID, 1);
#pragma unroll
  for (int t = 0; t < TT; ++t) epi.template prefetch2<PER>(pre[t], task, half, v0);
  spill_partials<TT, ROWS>(red, wave, lane, acc0, acc1);
  __syncthreads();
  TRACE_MARK(KID, 2);
  float a0[TT][PER], a1[TT][PER];
  fold_partials<TT, KW, PER>(red, lane, v0, a0, a1);
  if (n_slices > 1) {
    const int64_t unit = (int64_t)task * gridDim.z + group;
    put_slice<TT, PER>(part, unit * n_slices + slice, lane, v0, a0, a1);
    if (!last_arrival(tickets + unit, n_slices, &s_flag)) return;
    TRACE_MARK(KID, 3);
    sum_slices<TT, PER>(part, unit, n_slices, lane, v0, a0, a1);
  }
  float ss[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int tok = tok0 + t * TILE + (lane & 31);
    ss[t] = epi.template apply<PER>(pre[t], task, tok, tok < T, half, v0, a0[t], a1[t]);
  }
  if (Epi::ROWSUM) {
    // the task's row statistic: both half-waves of a column, then the KW waves in order
    __syncthreads();   // the partials in `red` are consumed
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      const float s2 = ss[t] + __shfl_xor(ss[t], 32, WAVE);
      if (half == 0) red[(wave * TT + t) * TILE + lane] = s2;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < TT * TILE; i += KW * WAVE) {
      float s = 0.f;
      for (int w = 0; w < KW; ++w) s += red[w * TT * TILE + i];
      const int tok = tok0 + i;
      if (tok < T) epi.row_sum(task, tok, s);
    }
  }
  TRACE_MARK(KID, 4);
}

template <int TT, int KW> constexpr size_t ksplit_lds() { return (size_t)KW * 2 * TT * 16 * WAVE * 4; }

// K slices (workgroups) per task: as many as leave every wave exactly one burst of k-steps (8 with one token
// tile, 4 with two), when K divides that way; one otherwise and whenever there are several token groups.
int gemm_slices(bool bf16, int K, int T) {
  if (T > 2 * TILE) return 1;
  const int ksteps = K / (bf16 ? 16 : 8);
  const int burst = 4 * (T <= TILE ? 8 : 4);   // KW = 4 waves
  return ksteps % burst == 0 ? ksteps / burst : 1;
}

// Slices a launch uses of those gemm_slices() allows (the workspace is sized for the latter): a hand-off among
// fewer workgroups is cheaper, so a projection with many tasks takes only as many slices as bring the launch to
// about half a workgroup per compute unit (measured at 32 tokens, K = 2048: the QKV projection, 96 tasks, 12.3 us
// with 2 slices against 13.1 with 4 and 14.9 with 1; the output projection, 32 tasks, 8.1 us with 4 slices, 10.0
// with 2, 13.4 with 1).
static int ksplit_slices(bool bf16, int K, int T, int n_tasks) {
  const int most = gemm_slices(bf16, K, T);
  int s = 1;
  while (s < most && s * n_tasks < 128) s *= 2;
  return most % s == 0 ? s : most;
}

template <typename E, class Epi>
static void launch_ksplit(bool bf16, const E* W, int ksteps, const E* B, int T, int K, int n_tasks,
                          float* part, int32_t* tickets, const Epi& epi, hipStream_t st, int forced_slices = 0) {
  const int slices = forced_slices ? forced_slices : single_slice() ? 1 : ksplit_slices(bf16, K, T, n_tasks);
  if (T <= 32) {
    gemm_ksplit_kernel<E, 1, 4, Epi><<<dim3(slices, n_tasks, 1), 4 * WAVE, ksplit_lds<1, 4>(), st>>>(W, ksteps, B, T, K, part, tickets, epi, live_word());
  } else if (T <= 64) {
    gemm_ksplit_kernel<E, 2, 4, Epi><<<dim3(slices, n_tasks, 1), 4 * WAVE, ksplit_lds<2, 4>(), st>>>(W, ksteps, B, T, K, part, tickets, epi, live_word());
  } else {
    const int groups = (T + 4 * TILE - 1) / (4 * TILE);
    gemm_ksplit_kernel<E, 4, 4, Epi><<<dim3(forced_slices ? forced_slices : 1, n_tasks, groups), 4 * WAVE, ksplit_lds<4, 4>(), st>>>(W, ksteps, B, T, K, part, tickets, epi, live_word());
  }
}

// Static + dynamic LDS of these kernels can pass the 64 KiB default: opt in to the 160 KiB LDS of gfx950
// (dynamic limit = what the kernel's static LDS leaves).  Returns false if the runtime refuses.
static bool opt_in_lds(const void* fn) {
  hipFuncAttributes fa;
  if (hipFuncGetAttributes(&fa, fn) != hipSuccess) return false;
  const int room = 160 * 1024 - (int)fa.sharedSizeBytes;
  return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, room) == hipSuccess;
}
template <typename E, class Epi> static bool configure_ksplit() {
  return opt_in_lds((const void*)gemm_ksplit_kernel<E, 1, 4, Epi>) &&
         opt_in_lds((const void*)gemm_ksplit_kernel<E, 2, 4, Epi>) &&
         opt_in_lds((const void*)gemm_ksplit_kernel<E, 4, 4, Epi>);
}

// ------------------------------------------------------------------------------------------------
// Down projection of the routed experts fused with the weighted combine, the residual add and the statistics of
// the norm that follows, for at most 32 tokens.  The sum over a token's k experts is a contraction like any other:
//   x[t][f] += sum_e sum_i  y[e][t][i] * Wd[e][f][i]      (y already carries the routing weight; y[e][t] = 0
//                                                           for tokens that were not routed to expert e)
// so a task (64 output features) runs over the "long K" of all experts that received rows, 64 k-steps each, with
// the token tile as the MFMA columns: a lane whose token is not among an expert's rows feeds zeros.  The long K is
// cut into pieces for n_slices x KW waves; wave sums are folded through LDS, workgroup sums through the
// cross-workgroup hand-off of the split-K kernel, in fixed order, and the last workgroup of a task runs the
// residual epilogue.  No per-(token, expert) output rows are stored and no separate combine pass runs; and because
// the work is cut by weight bytes, a layer that touches 8 experts fills the chip as well as one that touches 60.
// ------------------------------------------------------------------------------------------------
template <typename E, int TT, int KW, int PF>
__global__ __launch_bounds__(KW * WAVE) void expert_down_fused_kernel(const E* __restrict__ W, const E* __restrict__ Y,
                                                                       int64_t y_rows, const int32_t* __restrict__ off,
                                                                       const int32_t* __restrict__ topk_idx,
                                                                       const int32_t* __restrict__ pos_of_pair, int T,
                                                                       int I, int top_k, int n_tasks,
                                                                       float* __restrict__ part,
                                                                       int32_t* __restrict__ tickets, ResidualEpi<E> epi, const int32_t* __restrict__ live) {
  if (step_is_dead(live)) return;
  typedef typename ET<E>::vec vec;
  extern __shared__ float red[];   // [KW][2*TT*16][64]
  __shared__ int32_t s_flag;
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N, ROWS = 2 * TT * 16;
  constexpr int EW = 4, PER = 16 / EW;   // the first EW waves run the epilogue, four accumulator registers each
  static_assert(KW >= EW && MAX_EXPERTS <= WAVE, "epilogue waves; one lane per listed expert");
  constexpr int64_t STEP = 2 * WAVE * G;
  const int slice = blockIdx.x, n_slices = gridDim.x, task = blockIdx.y;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  TRACE_MARK(5, 0);
  TRACE_MARK_WAVE(55, 0, KW);
  // Everything the first loads hang on is requested at once, so that a workgroup is two memory round trips away
  // from its first weights however busy the memory system already is: the list of experts with rows (one per
  // lane) and their number, and this lane's tokens -- which experts they were routed to, where those rows sit in Y.
  const int listed = off[ACTIVE_LIST + lane];
  const int n_act = __builtin_amdgcn_readfirstlane(off[ACTIVE_LIST + MAX_EXPERTS]);
  int my_e[TT][MAX_TOPK], my_row[TT][MAX_TOPK];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int tok = min(t * TILE + col, T - 1);
#pragma unroll
    for (int j = 0; j < MAX_TOPK; ++j) {
      const int jj = min(j, top_k - 1);
      my_e[t][j] = topk_idx[tok * top_k + jj];
      my_row[t][j] = pos_of_pair[tok * top_k + jj];
    }
  }
  // The long K: experts with rows in list order, ksteps_e k-steps each, in groups of PF k-steps; this wave's
  // contiguous share [g0, g1).  A share is never longer than one expert's groups, so it meets at most two experts.
  const int ksteps_e = I / KS, groups_e = ksteps_e / PF, total = n_act * groups_e;
  const int units = n_slices * KW, per = (total + units - 1) / units;
  const int g0 = min(total, (slice * KW + wave) * per), g1 = min(total, g0 + per);
  const int i0 = g0 / groups_e;
  const int e_first = __builtin_amdgcn_readlane(listed, min(i0, MAX_EXPERTS - 1));
  const int e_second = __builtin_amdgcn_readlane(listed, min(i0 + 1, MAX_EXPERTS - 1));
  const E* wbase = W + (int64_t)task * task_stride_elems<E>(ksteps_e) + lane * G;
  const int64_t wexpert = (int64_t)n_tasks * task_stride_elems<E>(ksteps_e);
  auto weights_of = [&](int g) { return wbase + (g / groups_e == i0 ? e_first : e_second) * wexpert + (g % groups_e) * PF * STEP; };
  // Which Y row this lane reads for group g (byte offset of its first k-step) and how far it moves per k-step.
  // Y is read through a buffer descriptor with hardware range checking: a lane whose token was not routed to the
  // group's expert is given an offset past the end, for which the load returns zeros without touching memory --
  // exactly the operand such a token contributes.
  const __amdgpu_buffer_rsrc_t ybuf = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<E*>(Y), 0, (uint32_t)(y_rows * I * NP * sizeof(E)), 0x00020000);
  constexpr uint32_t ROW_BYTES = NP * KS * sizeof(E), PAST_END = 0x80000000u;
  const uint32_t ykstride = (uint32_t)y_rows * ROW_BYTES;
  auto rows_of = [&](int g, uint32_t (&yoff)[TT], uint32_t (&ystep)[TT]) {
    const int e = g / groups_e == i0 ? e_first : e_second, kk = (g % groups_e) * PF;
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      int row = -1;
#pragma unroll
      for (int j = 0; j < MAX_TOPK; ++j) row = (j < top_k && my_e[t][j] == e) ? my_row[t][j] : row;
      yoff[t] = row >= 0 ? ((uint32_t)kk * (uint32_t)y_rows + row) * ROW_BYTES + half * 16 : PAST_END;
      ystep[t] = row >= 0 ? ykstride : 0;
    }
  };
  f32x16 acc0[TT], acc1[TT];
  zero_acc<TT>(acc0);
  zero_acc<TT>(acc1);
  vec a0[PF], a1[PF], yr[PF][TT][NP];
  auto issue_w = [&](int i, const E* wp) {
    a0[i] = load16_stream<E>(wp + i * STEP);
    a1[i] = load16_stream<E>(wp + i * STEP + WAVE * G);
  };
  auto issue_y = [&](int i, const uint32_t (&yoff)[TT], const uint32_t (&ystep)[TT]) {
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int q = 0; q < NP; ++q)
        yr[i][t][q] = __builtin_bit_cast(vec, __builtin_amdgcn_raw_buffer_load_b128(
                                                  ybuf, yoff[t] + i * ystep[t] + q * (uint32_t)(KS * sizeof(E)), 0, 0));
  };
  auto use = [&](int i) {
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        mfma32(acc0[t], a0[i], yr[i][t][q]);
        mfma32(acc1[t], a1[i], yr[i][t][q]);
      }
  };
  if (g0 < g1) {
    {
      const E* wp = weights_of(g0);
      TRACE_MARK_WAVE(55, 1, KW);
#pragma unroll
      for (int i = 0; i < PF; ++i) issue_w(i, wp);
      uint32_t yoff[TT], ystep[TT];
      rows_of(g0, yoff, ystep);
#pragma unroll
      for (int i = 0; i < PF; ++i) issue_y(i, yoff, ystep);
    }
    auto group = [&](int g) {
      if (g == g0 + 1) TRACE_MARK(5, 5);
      if (g == g0 + 2) TRACE_MARK(5, 6);
      if (g == g0 + 4) TRACE_MARK(5, 7);
      if (g == g0) TRACE_MARK_WAVE(55, 2, KW);
      if (g == g0 + 1) TRACE_MARK_WAVE(55, 3, KW);
      if (g == g0 + 3) TRACE_MARK_WAVE(55, 4, KW);
      const E* wn = weights_of(g + 1);
      uint32_t yn[TT], ynstep[TT];
      rows_of(g + 1, yn, ynstep);
      // k-step by k-step: multiply, then request the same slot of the next group.  The scheduling barriers keep
      // the compiler from collecting the requests at the end of the iteration (it then waits for all of them at
      // the top of the next one and the memory pipe idles while the group is multiplied).
#pragma unroll
      for (int i = 0; i < PF; ++i) {
        use(i);
        __builtin_amdgcn_sched_barrier(0);
        issue_w(i, wn);
        issue_y(i, yn, ynstep);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // The first group stands in front of the loop: it meets the loads in the prologue's order (all weights, then
    // all rows), the later ones in the order the groups leave them (slot by slot), and wait counts at the top of a
    // loop that is entered both ways are the smaller of the two: slot 0 then waited for half the group in flight.
    if (g0 + 1 < g1) {
      group(g0);
      for (int g = g0 + 1; g + 1 < g1; ++g) group(g);
    }
#pragma unroll
    for (int i = 0; i < PF; ++i) use(i);
  }
  // Epilogue by the first EW waves (the others only keep the workgroup's barriers company).
  const bool worker = wave < EW;
  const int v0 = (worker ? wave : 0) * PER;
  typename ResidualEpi<E>::template Pre<PER> pre[TT];
  if (worker) {
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      const int tok = t * TILE + col;
      pre[t] = epi.template prefetch<PER>(task, tok, tok < T, half, v0);
    }
  }
  TRACE_MARK(5, 1);
  TRACE_MARK_WAVE(55, 5, KW);
  spill_partials<TT, ROWS>(red, wave, lane, acc0, acc1);
  __syncthreads();
  TRACE_MARK(5, 2);
  float s0[TT][PER], s1[TT][PER];
  if (worker) fold_partials<TT, KW, PER>(red, lane, v0, s0, s1);
  if (n_slices > 1) {
    if (worker) put_slice<TT, PER>(part, (int64_t)task * n_slices + slice, lane, v0, s0, s1);
    if (!last_arrival(tickets + task, n_slices, &s_flag)) return;
    TRACE_MARK(5, 3);
    if (worker) sum_slices<TT, PER, 8>(part, task, n_slices, lane, v0, s0, s1);
  }
  float ss[TT];
  if (worker) {
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      const int tok = t * TILE + col;
      ss[t] = epi.template apply<PER>(pre[t], task, tok, tok < T, half, v0, s0[t], s1[t]);
    }
  }
  __syncthreads();   // the partials in `red` are consumed
  if (worker) {
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      const float s2 = ss[t] + __shfl_xor(ss[t], 32, WAVE);
      if (half == 0) red[(wave * TT + t) * TILE + lane] = s2;
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < TT * TILE; i += KW * WAVE) {
    float s = 0.f;
    for (int w = 0; w < EW; ++w) s += red[w * TT * TILE + i];
    if (i < T) epi.row_sum(task, i, s);
  }
  TRACE_MARK(5, 4);
}

// ------------------------------------------------------------------------------------------------
// Dense projections over many token rows (more than 64).  A workgroup takes TASKS (four or two) tasks and WT token
// tiles; its TASKS * KH waves are KH teams, each team with its own share of the K range, its own LDS staging area for the
// activation fragments (wide_stream.hpp) and one wave per task, which streams that task's weights once and keeps
// the accumulators of 64 features x WT*32 rows.  The teams' sums are folded through LDS at the end and team 0
// runs the epilogue (those of the split-K kernel, called for four accumulator registers at a time).  KH > 1 puts
// several waves on every SIMD, so that one multiplies while another waits for LDS or memory, without asking the
// launch for more workgroups than there are (task, token) tiles.
// Grid (task groups, token groups): with a multiple of eight task groups the workgroups of one die always take the
// same tasks, so the weights (a few MB per die) are read from HBM once and then served by that die's L2.
// ------------------------------------------------------------------------------------------------
// Measured at 512 tokens (QKV / output projection, microseconds): one team 58 / 34, two teams 58 / 34 before and
// 41 / 29 after the epilogue stores were widened, four teams of one token tile 94 / 37; four token tiles per
// workgroup 102 / 95 (too few workgroups); two tasks per workgroup 57 / 19 (the output projection, with 32 tasks,
// then fills the chip with 256 workgroups).
constexpr int DENSE_PRE = 2, DENSE_KH = 2, DENSE_WT = 2;
constexpr int DENSE_FILL = 160;   // workgroups a launch with DENSE_WT token tiles must keep, else one tile each

template <typename E, int KID, int WT, int DENSE_TASKS> constexpr size_t dense_lds() {
  const size_t stage = DENSE_KH * wide_lds<E, KID, WT>();
  const size_t fold = (size_t)(DENSE_KH - 1) * DENSE_TASKS * 2 * WT * 16 * WAVE * 4;
  return stage > fold ? stage : fold;
}

template <typename E, int WT, int DENSE_TASKS, class Epi>
__global__ __launch_bounds__(DENSE_TASKS * DENSE_KH * WAVE) void gemm_dense_kernel(const E* __restrict__ W, int ksteps,
                                                                                  const E* __restrict__ B, int T,
                                                                                  int n_tasks, Epi epi, const int32_t* __restrict__ live) {
  if (step_is_dead(live)) return;
  typedef typename ET<E>::vec vec;
  extern __shared__ __align__(16) char lds_raw[];   // 16-byte aligned: staged fragments move as 128-bit LDS accesses
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N, PER = 4;
  constexpr int KID = Epi::ROWSUM ? 13 : 12;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int team = wave / DENSE_TASKS, rank = wave % DENSE_TASKS;
  const int slot = blockIdx.x * DENSE_TASKS + rank, task = min(slot, n_tasks - 1);
  const int tok0 = blockIdx.y * WT * TILE;
  const int nt = min(WT, (T - tok0 + TILE - 1) / TILE);
  const int chunks = ksteps / WKC / DENSE_KH;          // per team
  const int ks0 = team * chunks * WKC;
  vec* sb = reinterpret_cast<vec*>(lds_raw + team * wide_lds<E, KID, WT>());
  const E* brow = B + (int64_t)ks0 * T * (NP * KS) + (int64_t)min(tok0 + (rank % WT) * TILE + col, T - 1) * (NP * KS) + half * G;
  f32x16 acc0[WT], acc1[WT];
  zero_acc<WT>(acc0);
  zero_acc<WT>(acc1);
  wide_stream<E, WT, DENSE_TASKS, DENSE_PRE, KID>(
      W + (int64_t)task * task_stride_elems<E>(ksteps) + (int64_t)ks0 * (2 * WAVE * G) + lane * G, chunks, [&] { return brow; },
      (int64_t)T * (NP * KS), sb, nt, acc0, acc1, rank);
  if (DENSE_KH > 1) {
    // fold: team h > 0 leaves its sums at red[h-1][rank][t*32 + tile*16 + v][lane], team 0 adds them up
    float* red = reinterpret_cast<float*>(lds_raw);
    __syncthreads();   // the staging areas are done with
    if (team > 0) {
      float* r = red + ((int64_t)((team - 1) * DENSE_TASKS + rank) * (2 * WT * 16)) * WAVE + lane;
#pragma unroll
      for (int t = 0; t < WT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          r[(t * 32 + v) * WAVE] = acc0[t][v];
          r[(t * 32 + 16 + v) * WAVE] = acc1[t][v];
        }
    }
    __syncthreads();
    if (team > 0) return;
    for (int h = 1; h < DENSE_KH; ++h) {
      const float* r = red + ((int64_t)((h - 1) * DENSE_TASKS + rank) * (2 * WT * 16)) * WAVE + lane;
#pragma unroll
      for (int t = 0; t < WT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          acc0[t][v] += r[(t * 32 + v) * WAVE];
          acc1[t][v] += r[(t * 32 + 16 + v) * WAVE];
        }
    }
  }
  if (slot >= n_tasks) return;
  // Epilogue in three sweeps over the (tile, register group) pairs, so that the loads of one sweep are all in flight
  // together: what is addressed by the token, what is addressed by what those loads return, then the arithmetic.
  constexpr int NG = 16 / PER;
  typename Epi::template Pre<PER> pre[WT][NG];
#pragma unroll
  for (int t = 0; t < WT; ++t)
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const int tok = tok0 + t * TILE + col;
      pre[t][g] = epi.template prefetch<PER>(task, tok, t < nt && tok < T, half, g * PER);
    }
#pragma unroll
  for (int t = 0; t < WT; ++t)
#pragma unroll
    for (int g = 0; g < NG; ++g) epi.template prefetch2<PER>(pre[t][g], task, half, g * PER);
#pragma unroll
  for (int t = 0; t < WT; ++t) {
    const int tok = tok0 + t * TILE + col;
    const bool valid = t < nt && tok < T;
    float ss = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      float a0[PER], a1[PER];
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        a0[i] = acc0[t][g * PER + i];
        a1[i] = acc1[t][g * PER + i];
      }
      ss += epi.template apply<PER>(pre[t][g], task, tok, valid, half, g * PER, a0, a1);
    }
    if (Epi::ROWSUM) {   // the wave holds the whole task: the row statistic is the sum over its two half-waves
      ss += __shfl_xor(ss, 32, WAVE);
      if (half == 0 && valid) epi.row_sum(task, tok, ss);
    }
  }
  TRACE_MARK(KID, 7);
}

// True when the dense form takes the call (many rows, K a whole number of staged chunks per team).
// (Above 64 tokens.  With two token tiles the split-K form of the QKV projection used to hand 12.6 MB of partial
// sums between workgroups, 8 slices per task, and the dense form was faster, 19.1 against 27.9 us; with the two
// slices that ksplit_slices() now gives a launch of 96 tasks it takes 14.9 us.  For the output projection, a third
// of the weights, split-K was ahead all along, 11.5 against 17.1.)
static bool dense_applies(int T, int ksteps) { return T > 2 * TILE && ksteps % (WKC * DENSE_KH) == 0; }

template <typename E, int WT, int TASKS, class Epi>
static void launch_dense_as(const E* W, int ksteps, const E* B, int T, int n_tasks, const Epi& epi, hipStream_t st) {
  constexpr int KID = Epi::ROWSUM ? 13 : 12;
  gemm_dense_kernel<E, WT, TASKS, Epi><<<dim3((n_tasks + TASKS - 1) / TASKS, (T + WT * TILE - 1) / (WT * TILE)),
                                        TASKS * DENSE_KH * WAVE, dense_lds<E, KID, WT, TASKS>(), st>>>(W, ksteps, B, T,
                                                                                                    n_tasks, epi, live_word());
}
// More tasks and token tiles per workgroup cut the operand traffic, but only while the launch still fills the chip.
template <typename E, class Epi>
static void launch_dense(const E* W, int ksteps, const E* B, int T, int n_tasks, const Epi& epi, hipStream_t st) {
  auto wgs = [&](int tasks, int wt) { return ((n_tasks + tasks - 1) / tasks) * ((T + wt * TILE - 1) / (wt * TILE)); };
  if (wgs(4, DENSE_WT) >= DENSE_FILL) launch_dense_as<E, DENSE_WT, 4, Epi>(W, ksteps, B, T, n_tasks, epi, st);
  else if (wgs(4, 1) >= DENSE_FILL) launch_dense_as<E, 1, 4, Epi>(W, ksteps, B, T, n_tasks, epi, st);
  else launch_dense_as<E, 1, 2, Epi>(W, ksteps, B, T, n_tasks, epi, st);
}

template <typename E, class Epi> static bool configure_dense() {
  return opt_in_lds((const void*)gemm_dense_kernel<E, DENSE_WT, 4, Epi>) && opt_in_lds((const void*)gemm_dense_kernel<E, 1, 4, Epi>) &&
         opt_in_lds((const void*)gemm_dense_kernel<E, 1, 2, Epi>);
}

template <typename E> static void launch_qkv_t(bool bf16, const QkvArgs& a, hipStream_t st) {
  const int D = a.geom.n_heads * a.geom.head_dim;
  QkvEpi<E> epi{(E*)a.q, a.q_plane, (E*)a.kv_layer, a.geom, a.meta.tok_seq, a.meta.tok_pos, a.page_table,
                a.pt_stride, a.cos_tab, a.sin_tab, a.norm, a.T, a.H, D};
  if (dense_applies(a.T, a.H / ET<E>::KS))
    launch_dense<E>((const E*)a.w, a.H / ET<E>::KS, (const E*)a.xn, a.T, 3 * D / 64, epi, st);
  else
    launch_ksplit<E>(bf16, (const E*)a.w, a.H / ET<E>::KS, (const E*)a.xn, a.T, a.H, 3 * D / 64, a.part,
                     a.tickets, epi, st);
}
void launch_qkv(bool bf16, const QkvArgs& a, hipStream_t st) {
  if (bf16) launch_qkv_t<bf16_t>(true, a, st);
  else launch_qkv_t<float>(false, a, st);
}

template <typename E> static void launch_oproj_t(bool bf16, const OprojArgs& a, hipStream_t st) {
  ResidualEpi<E> epi{a.x, a.H, a.gain, (E*)a.xn, a.ssq, a.T};
  if (dense_applies(a.T, a.D / ET<E>::KS))
    launch_dense<E>((const E*)a.w, a.D / ET<E>::KS, (const E*)a.a, a.T, a.H / 64, epi, st);
  else
    launch_ksplit<E>(bf16, (const E*)a.w, a.D / ET<E>::KS, (const E*)a.a, a.T, a.D, a.H / 64, a.part, a.tickets,
                     epi, st);
}
// What the workgroups of the split-K launch stream: workgroup (slice, task) has index task * slices + slice and takes
// the slice's share of the task's k-steps, 2 KB of packed weights each, so region i starts at i * region_bytes.
L2Prefetch oproj_prefetch_plan(bool bf16, const void* w, int D, int H, int T) {
  const int ksteps = D / (bf16 ? 16 : 8), n_tasks = H / 64;
  if (T > 2 * TILE || single_slice()) return L2Prefetch{nullptr, 0, 0};   // more tokens: the dense form
  const int slices = ksplit_slices(bf16, D, T, n_tasks);
  if (ksteps % (slices * 4) != 0) return L2Prefetch{nullptr, 0, 0};       // slices of unequal length
  return L2Prefetch{(const char*)w, (uint32_t)(ksteps / slices) * 2048u, n_tasks * slices};
}
void launch_oproj(bool bf16, const OprojArgs& a, hipStream_t st) {
  if (bf16) launch_oproj_t<bf16_t>(true, a, st);
  else launch_oproj_t<float>(false, a, st);
}

int smooth_kpad(bool bf16, int V) {
  const int unit = (bf16 ? 16 : 8) * 4 * 8 * SMOOTH_SLICES;   // k-step x waves x burst x slices
  return (V + unit - 1) / unit * unit;
}
template <typename E> static void launch_smooth_t(bool bf16, const SmoothArgs& a, hipStream_t st) {
  const int Kpad = smooth_kpad(bf16, a.V);
  SmoothEpi epi{a.delta, a.H, a.mask, a.block_len};
  // More than 64 tokens: the shared-operand form, with the most token tiles per workgroup whatever the fill -- every
  // token group streams the whole transposed embedding matrix, so fewer, larger groups move fewer bytes.
  if (dense_applies(a.T, Kpad / ET<E>::KS))
    launch_dense_as<E, DENSE_WT, 4, SmoothEpi>((const E*)a.w_emb_t, Kpad / ET<E>::KS, (const E*)a.probs, a.T, a.H / 64, epi, st);
  else
    launch_ksplit<E>(bf16, (const E*)a.w_emb_t, Kpad / ET<E>::KS, (const E*)a.probs, a.T, Kpad, a.H / 64, a.part,
                     a.tickets, epi, st, SMOOTH_SLICES);
}
void launch_expected_embedding(bool bf16, const SmoothArgs& a, hipStream_t st) {
  launch_prob_planes(bf16, a.logits, a.stats, a.T, a.V, smooth_kpad(bf16, a.V), a.probs, st);
  if (bf16) launch_smooth_t<bf16_t>(true, a, st);
  else launch_smooth_t<float>(false, a, st);
}

// ------------------------------------------------------------------------------------------------
// Router.  The single weight task holds experts 0-31 (tile 0) and 32-63 (tile 1); per token group its K range is
// shared by `slices` workgroups of KW waves exactly as in the split-K kernel above.  The workgroup that holds the
// complete sums turns them into logits[token][expert] (times the row's 1/rms, which it derives from the per-task
// sums of squares the output projection left), then groups of 16 lanes (4 experts per lane) take one token each
// through softmax and the k selection rounds (ties to the lower expert id).  With a single token group the same
// workgroup goes on to build the token->expert permutation.
// ------------------------------------------------------------------------------------------------
// Cross-lane moves inside rows of 16 lanes on the data-parallel-primitive path (no LDS round trip).  The four
// controls below form a butterfly: after them every lane of a 16-lane group holds the group's result, provided
// the combining step is symmetric.
template <int CTRL> __device__ inline int dpp_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true); }
template <int CTRL> __device__ inline float dpp_f(float v) { return __int_as_float(dpp_i<CTRL>(__float_as_int(v))); }
constexpr int DPP_SWAP1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int DPP_SWAP2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i <- lane 7-i of its group of 8
constexpr int DPP_MIRROR = 0x140;       // lane i <- lane 15-i of its row
__device__ inline float group16_max(float v) {
  v = fmaxf(v, dpp_f<DPP_SWAP1>(v));
  v = fmaxf(v, dpp_f<DPP_SWAP2>(v));
  v = fmaxf(v, dpp_f<DPP_HALF_MIRROR>(v));
  return fmaxf(v, dpp_f<DPP_MIRROR>(v));
}
// Sum over the group in a fixed tree; every lane ends with the same bits (each step adds the same two values on
// both sides, and float addition commutes).
__device__ inline float group16_sum(float v) {
  v += dpp_f<DPP_SWAP1>(v);
  v += dpp_f<DPP_SWAP2>(v);
  v += dpp_f<DPP_HALF_MIRROR>(v);
  return v + dpp_f<DPP_MIRROR>(v);
}
__device__ inline int group16_min(int v) {
  v = min(v, dpp_i<DPP_SWAP1>(v));
  v = min(v, dpp_i<DPP_SWAP2>(v));
  v = min(v, dpp_i<DPP_HALF_MIRROR>(v));
  return min(v, dpp_i<DPP_MIRROR>(v));
}
// Largest value of the group and the lowest id that holds it: the largest value first, then the lowest id among
// the lanes whose own best equals it (two plain butterflies instead of one with a compound comparison).
__device__ inline void group16_argmax(float& bv, int& bi) {
  const float mx = group16_max(bv);
  bi = group16_min(bv == mx ? bi : 0x7fffffff);
  bv = mx;
}

// Token->expert permutation of at most 8*64 pairs whose expert ids sit in LDS (s_idx): a stable counting sort.
// A wave takes 64 consecutive pairs (a chunk).  The chunk's 64 ballots "which lanes go to expert e" are formed all
// at once by OR-ing lane bits into s_ballot[chunk][e]; a pair's rank inside its chunk is the number of set bits
// below its lane in its expert's ballot, the chunk's count for expert e the population of ballot e.  Lane e of
// wave 0 then turns the per-chunk counts into offsets.  s_ballot: [8][MAX_EXPERTS] 64-bit words, s_cc:
// [8][MAX_EXPERTS] ints.  A wave owns chunks wave and wave + n_waves (at least 4 waves, at most 8 chunks).
__device__ inline void ballot_permute_small(const int32_t* s_idx, int n_pairs, int n_exp, int32_t* __restrict__ cnt,
                                            int32_t* __restrict__ off, int32_t* __restrict__ perm,
                                            int32_t* __restrict__ pos_of_pair, unsigned long long* s_ballot,
                                            int32_t* s_cc) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n_waves = blockDim.x >> 6;
  const int n_chunks = (n_pairs + WAVE - 1) / WAVE;
  const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  for (int i = threadIdx.x; i < n_chunks * MAX_EXPERTS; i += blockDim.x) s_ballot[i] = 0ull;
  __syncthreads();
  int my_e[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = wave + i * n_waves;
    const int p = c * WAVE + lane;
    my_e[i] = (c < n_chunks && p < n_pairs) ? s_idx[p] : -1;
    if (my_e[i] >= 0) atomicOr(&s_ballot[c * MAX_EXPERTS + my_e[i]], 1ull << lane);
  }
  __syncthreads();
  int my_rank[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = wave + i * n_waves;
    my_rank[i] = my_e[i] >= 0 ? __popcll(s_ballot[c * MAX_EXPERTS + my_e[i]] & below) : 0;
    if (c < n_chunks) s_cc[c * MAX_EXPERTS + lane] = __popcll(s_ballot[c * MAX_EXPERTS + lane]);   // lane = expert id
  }
  __syncthreads();
  if (wave == 0) {
    int tot = 0;
    for (int c = 0; c < n_chunks; ++c) tot += s_cc[c * MAX_EXPERTS + lane];
    if (lane >= n_exp) tot = 0;
    int incl = tot;   // inclusive scan over the lanes (experts)
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
      const int up = __shfl_up(incl, o, WAVE);
      if (lane >= o) incl += up;
    }
    const int start = incl - tot;
    if (lane < n_exp) {
      cnt[lane] = tot;
      off[lane] = start;
      if (lane == n_exp - 1) off[n_exp] = incl;
    }
    const uint64_t has_rows = __ballot(tot > 0);          // dense list of the experts with rows (ACTIVE_LIST)
    if (tot > 0) {
      const int at = __popcll(has_rows & below);
      off[ACTIVE_LIST + at] = lane;
      *reinterpret_cast<int4*>(off + ACTIVE_RECORDS + 4 * at) = make_int4(lane, start, tot, 0);
    }
    if (lane == 0) {
      off[ACTIVE_LIST + MAX_EXPERTS] = __popcll(has_rows);
      off[STAT_ACTIVE_SUM] += __popcll(has_rows);
      off[STAT_PERMUTATIONS] += 1;
    }
    int run = start;                                      // chunk c of expert `lane` starts at run
    for (int c = 0; c < n_chunks; ++c) {
      const int n = s_cc[c * MAX_EXPERTS + lane];
      s_cc[c * MAX_EXPERTS + lane] = run;
      run += n;
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = wave + i * n_waves;
    if (c < n_chunks && my_e[i] >= 0) {
      const int p = c * WAVE + lane;
      const int r = s_cc[c * MAX_EXPERTS + my_e[i]] + my_rank[i];
      perm[r] = p;
      pos_of_pair[p] = r;
    }
  }
}

template <typename E, int TT, int KW>
__global__ __launch_bounds__(KW * WAVE) void router_kernel(const E* __restrict__ W, const E* __restrict__ xn,
                                                            const float* __restrict__ ssq, int n_ssq,
                                                            float eps, int T, int H, int n_exp, int top_k, int norm_topk,
                                                            float* __restrict__ rinv, int32_t* __restrict__ topk_idx,
                                                            float* __restrict__ topk_w, int fuse_permute,
                                                            int32_t* __restrict__ cnt, int32_t* __restrict__ off,
                                                            int32_t* __restrict__ perm,
                                                            int32_t* __restrict__ pos_of_pair, float* __restrict__ part,
                                                            int32_t* __restrict__ tickets, const int32_t* __restrict__ live) {
  if (step_is_dead(live)) return;
  extern __shared__ float red[];   // [KW][2*TT*16][64] partials
  constexpr int ROWS = 2 * TT * 16, NTOK = TT * TILE, NTHREADS = KW * WAVE, PER = 16 / KW;
  constexpr int SS_PARTS = NTHREADS / NTOK;                       // threads per token for the sums of squares
  constexpr int SS_PER = (MAX_HIDDEN / 64 + SS_PARTS - 1) / SS_PARTS;
  constexpr int LOGIT_STRIDE = MAX_EXPERTS + 1;   // padded: the transposed writes spread over the banks
  __shared__ float s_logit[NTOK * LOGIT_STRIDE];
  __shared__ float s_ssp[SS_PARTS * NTOK];
  __shared__ float s_rinv[NTOK];
  __shared__ int32_t s_idx[NTOK * MAX_TOPK];
  __shared__ unsigned long long s_ballot[8 * MAX_EXPERTS];
  __shared__ int32_t s_cc[8 * MAX_EXPERTS];
  __shared__ int32_t s_flag;
  const int slice = blockIdx.x, n_slices = gridDim.x, group = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5;
  const int tok0 = group * NTOK;
  const int ksteps = H / ET<E>::KS;
  TRACE_MARK(3, 0);
  // shares of the rows' sums of squares (one per 64-feature task of the producer), loaded before the stream
  float ssv[SS_PER];
  {
    const int tok = min(tok0 + (int)threadIdx.x % NTOK, T - 1), part0 = threadIdx.x / NTOK;
#pragma unroll
    for (int i = 0; i < SS_PER; ++i) {
      const int j = part0 + i * SS_PARTS;
      ssv[i] = j < n_ssq ? ssq[(int64_t)j * T + tok] : 0.f;
    }
  }
  f32x16 acc0[TT], acc1[TT];
  zero_acc<TT>(acc0);
  zero_acc<TT>(acc1);
  PlaneLoader<E, TT> ld;
#pragma unroll
  for (int t = 0; t < TT; ++t) ld.set(t, xn, T, min(tok0 + t * TILE + (lane & 31), T - 1), half);
  const int per = (ksteps + n_slices * KW - 1) / (n_slices * KW);
  const int ks0 = min(ksteps, (slice * KW + wave) * per), ks1 = min(ksteps, ks0 + per);
  stream_task<E, TT, (TT == 1 ? 8 : 4), false>(W, ks0, ks1, ld, acc0, acc1);
  TRACE_MARK(3, 1);
  spill_partials<TT, ROWS>(red, wave, lane, acc0, acc1);
  {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < SS_PER; ++i) s += ssv[i];
    s_ssp[threadIdx.x] = s;     // [part][token]
  }
  __syncthreads();
  TRACE_MARK(3, 2);
  const int v0 = wave * PER;
  float a0[TT][PER], a1[TT][PER];
  fold_partials<TT, KW, PER>(red, lane, v0, a0, a1);
  if (n_slices > 1) {
    put_slice<TT, PER>(part, (int64_t)group * n_slices + slice, lane, v0, a0, a1);
    if (!last_arrival(tickets + group, n_slices, &s_flag)) return;
    sum_slices<TT, PER>(part, group, n_slices, lane, v0, a0, a1);
  }
  if (threadIdx.x < NTOK) {
    float row_ss = 0.f;
    for (int q = 0; q < SS_PARTS; ++q) row_ss += s_ssp[q * NTOK + threadIdx.x];
    const float r = rsqrtf(row_ss / H + eps);
    s_rinv[threadIdx.x] = r;
    if (tok0 + (int)threadIdx.x < T) rinv[tok0 + threadIdx.x] = r;
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    const int tl = t * TILE + (lane & 31);
    const float r = s_rinv[tl];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      s_logit[tl * LOGIT_STRIDE + acc_row(v0 + i, half)] = a0[t][i] * r;
      s_logit[tl * LOGIT_STRIDE + TILE + acc_row(v0 + i, half)] = a1[t][i] * r;
    }
  }
  __syncthreads();
  TRACE_MARK(3, 3);
  // 16 lanes per token, 4 consecutive experts per lane
  const int grp = threadIdx.x >> 4, sub = threadIdx.x & 15;
  for (int tl = grp; tl < NTOK; tl += NTHREADS / 16) {
    float p[4];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = 4 * sub + i < n_exp ? s_logit[tl * LOGIT_STRIDE + 4 * sub + i] : -INFINITY;
      m = fmaxf(m, p[i]);
    }
    m = group16_max(m);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      p[i] = 4 * sub + i < n_exp ? expf(p[i] - m) : 0.f;
      sum += p[i];
    }
    const float inv = 1.f / group16_sum(sum);
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = 4 * sub + i < n_exp ? p[i] * inv : -1.f;
    float wsel = 0.f, sel_sum = 0.f;   // lane j of the group keeps the j-th selection
    int isel = 0;
    for (int j = 0; j < top_k; ++j) {
      float bv = -1.f;
      int bi = 0x7fffffff;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (p[i] > bv) {               // ids ascend with i: strict '>' keeps the lowest id
          bv = p[i];
          bi = 4 * sub + i;
        }
      group16_argmax(bv, bi);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (4 * sub + i == bi) p[i] = -1.f;
      if (sub == j) {
        wsel = bv;
        isel = bi;
      }
      sel_sum += bv;
    }
    if (sub < top_k) {
      const int tok = tok0 + tl;
      if (tok < T) {
        topk_idx[tok * top_k + sub] = isel;
        topk_w[tok * top_k + sub] = norm_topk ? wsel / sel_sum : wsel;
      }
      s_idx[tl * top_k + sub] = tok < T ? isel : -1;
    }
  }
  TRACE_MARK(3, 4);
  if (!fuse_permute) return;
  __syncthreads();
  ballot_permute_small(s_idx, T * top_k, n_exp, cnt, off, perm, pos_of_pair, s_ballot, s_cc);
  TRACE_MARK(3, 5);
}

// Workgroups that share the router's K range: as for the projections, with 8 waves per workgroup.
static int router_slices(bool bf16, int K, int T) {
  if (T > 2 * TILE || single_slice()) return 1;
  const int ksteps = K / (bf16 ? 16 : 8);
  const int burst = 8 * (T <= TILE ? 8 : 4);
  return ksteps % burst == 0 ? ksteps / burst : 1;
}

template <typename E> static void launch_router_t(bool bf16, const RouterArgs& a, hipStream_t st) {
  const E* W = (const E*)a.w;
  const int slices = router_slices(bf16, a.H, a.T);
  if (a.T <= 32) {
    router_kernel<E, 1, 8><<<dim3(slices, 1), 8 * WAVE, ksplit_lds<1, 8>(), st>>>(
        W, (const E*)a.xn, a.ssq, a.H / 64, a.eps, a.T, a.H, a.E, a.top_k, a.norm_topk, a.rinv, a.topk_idx,
        a.topk_w, 1, a.cnt, a.off, a.perm, a.pos_of_pair, a.part, a.tickets, live_word());
  } else if (a.T <= 64) {
    router_kernel<E, 2, 8><<<dim3(slices, 1), 8 * WAVE, ksplit_lds<2, 8>(), st>>>(
        W, (const E*)a.xn, a.ssq, a.H / 64, a.eps, a.T, a.H, a.E, a.top_k, a.norm_topk, a.rinv, a.topk_idx,
        a.topk_w, 1, a.cnt, a.off, a.perm, a.pos_of_pair, a.part, a.tickets, live_word());
  } else {
    const int groups = (a.T + TILE - 1) / TILE;   // 32 tokens per workgroup: one round of the top-k lanes, more workgroups
    router_kernel<E, 1, 8><<<dim3(1, groups), 8 * WAVE, ksplit_lds<1, 8>(), st>>>(
        W, (const E*)a.xn, a.ssq, a.H / 64, a.eps, a.T, a.H, a.E, a.top_k, a.norm_topk, a.rinv, a.topk_idx,
        a.topk_w, 0, a.cnt, a.off, a.perm, a.pos_of_pair, a.part, a.tickets, live_word());
    launch_permute(a.topk_idx, a.T * a.top_k, a.E, a.cnt, a.off, a.perm, a.pos_of_pair, a.work, st);
  }
}
void launch_router(bool bf16, const RouterArgs& a, hipStream_t st) {
  if (bf16) launch_router_t<bf16_t>(true, a, st);
  else launch_router_t<float>(false, a, st);
}

// Fused down projection: DOWN_SLICES workgroups of DOWN_KW waves share a task's long K.
constexpr int DOWN_SLICES = 8, DOWN_KW = 8;
int down_fused_slices() { return DOWN_SLICES; }
template <typename E> static void launch_down_fused_t(const ExpertArgs& a, const OprojArgs& r, hipStream_t st) {
  ResidualEpi<E> epi{r.x, r.H, r.gain, (E*)r.xn, r.ssq, r.T};
  const int n_tasks = a.H / 64, ksteps_e = a.I / ET<E>::KS;
  const dim3 grid(DOWN_SLICES, n_tasks);
  const E *w = (const E*)a.w_down, *y = (const E*)a.y;
  const int64_t y_rows = (int64_t)a.T * a.top_k;
  if (ksteps_e % 8 == 0)
    expert_down_fused_kernel<E, 1, DOWN_KW, 8><<<grid, DOWN_KW * WAVE, ksplit_lds<1, DOWN_KW>(), st>>>(
        w, y, y_rows, a.off, a.topk_idx, a.pos_of_pair, a.T, a.I, a.top_k, n_tasks, r.part, r.tickets, epi, live_word());
  else
    expert_down_fused_kernel<E, 1, DOWN_KW, 4><<<grid, DOWN_KW * WAVE, ksplit_lds<1, DOWN_KW>(), st>>>(
        w, y, y_rows, a.off, a.topk_idx, a.pos_of_pair, a.T, a.I, a.top_k, n_tasks, r.part, r.tickets, epi, live_word());
}
void launch_expert_down_fused(bool bf16, const ExpertArgs& a, const OprojArgs& res, hipStream_t st) {
  if (bf16) launch_down_fused_t<bf16_t>(a, res, st);
  else launch_down_fused_t<float>(a, res, st);
}

// The routed-expert GEMMs and the LM head live in wide.hip (shared-operand forms for every token count).
void launch_expert_gate_up(bool bf16, const ExpertArgs& a, hipStream_t st) { launch_expert_gate_up_wide(bf16, a, st); }
void launch_expert_down(bool bf16, const ExpertArgs& a, hipStream_t st) { launch_expert_down_wide(bf16, a, st); }
int lm_head_waves(int V) { return lm_head_wide_parts(V); }
int lm_head_parts(int V, int) { return lm_head_wide_parts(V); }
void launch_lm_head(bool bf16, const LmArgs& a, hipStream_t st) { launch_lm_head_wide(bf16, a, st); }

bool configure_kernels() {
  bool ok = configure_ksplit<bf16_t, QkvEpi<bf16_t>>() && configure_ksplit<float, QkvEpi<float>>() &&
            configure_ksplit<bf16_t, ResidualEpi<bf16_t>>() && configure_ksplit<float, ResidualEpi<float>>() &&
            configure_ksplit<bf16_t, SmoothEpi>() && configure_ksplit<float, SmoothEpi>();
  ok = ok && configure_dense<bf16_t, QkvEpi<bf16_t>>() && configure_dense<float, QkvEpi<float>>() &&
       configure_dense<bf16_t, ResidualEpi<bf16_t>>() && configure_dense<float, ResidualEpi<float>>() &&
       configure_dense<bf16_t, SmoothEpi>() && configure_dense<float, SmoothEpi>();
  ok = ok && opt_in_lds((const void*)expert_down_fused_kernel<bf16_t, 1, DOWN_KW, 8>) &&
       opt_in_lds((const void*)expert_down_fused_kernel<bf16_t, 1, DOWN_KW, 4>) &&
       opt_in_lds((const void*)expert_down_fused_kernel<float, 1, DOWN_KW, 8>) &&
       opt_in_lds((const void*)expert_down_fused_kernel<float, 1, DOWN_KW, 4>);
  ok = ok && opt_in_lds((const void*)router_kernel<bf16_t, 1, 8>) && opt_in_lds((const void*)router_kernel<float, 1, 8>) &&
       opt_in_lds((const void*)router_kernel<bf16_t, 2, 8>) && opt_in_lds((const void*)router_kernel<float, 2, 8>);
  (void)hipGetLastError();
  return ok;
}

TRACE_READER(trace_read_gemm)

}  // namespace dinfer
