// Many-token forms (more than 64 tokens in a forward) of the weight-streaming contractions: routed-expert
// grouped GEMMs and the LM head.  With hundreds of token rows a wave that fetched its own activation operands
// would pull several times more bytes through the L2 than it streams weights from HBM, so here a workgroup of
// eight waves shares them (wide_stream.hpp): the workgroup covers 128 token rows (four 32-row tiles) and eight
// tasks (512 output features).  The accumulators of a wave (64 features x 128 rows) stay in registers for the
// whole K range: there is no split of K and no fold.
#include "kernels.hpp"
#include "wide_stream.hpp"

namespace dinfer {

constexpr int WT = 4;      // token tiles per workgroup
// Waves (= tasks) per workgroup and weight chunks in flight per wave.  Eight waves put two on every SIMD, so one
// computes while the other waits for LDS or memory, and the activation fragments are shared by eight tasks.
// (Measured at 512 tokens: four waves with the whole register file behind a six-chunk weight prefetch are slower
// for the expert GEMMs, 173 against 141 microseconds.)
constexpr int EXPERT_WW = 8, EXPERT_PRE = 2;
#ifndef LM_WW_N
#define LM_WW_N 8
#endif
#ifndef LM_PRE_N
#define LM_PRE_N 2
#endif
constexpr int LM_WW = LM_WW_N, LM_PRE = LM_PRE_N;
constexpr int XCDS = 8;      // accelerator dies, each with its own L2; workgroup i of a launch runs on die i % 8

__device__ inline float silu_w(float x) { return x / (1.f + __expf(-x)); }

// ------------------------------------------------------------------------------------------------
// Routed experts, rows of expert e = pairs perm[off[e] .. off[e]+cnt[e]).  Grid (tasks / 8, work items): a work item
// is an (expert, group of up to 128 rows) pair; the permutation kernel lists them heaviest first.
//   GEMM 1: task = 32 gate features + the same 32 up features;  y = silu(gate) * up  -> Y[sorted row][I]
//   GEMM 2: task = 64 adjacent output features of the down projection                -> O[token*top_k + slot][H]
// ------------------------------------------------------------------------------------------------
template <typename E>
__global__ __launch_bounds__(EXPERT_WW * WAVE) void expert_gemm1_wide_kernel(const E* __restrict__ W, const E* __restrict__ xn,
                                                                       const float* __restrict__ rinv,
                                                                       E* __restrict__ Y, const int32_t* __restrict__ cnt,
                                                                       const int32_t* __restrict__ off,
                                                                       const int32_t* __restrict__ perm,
                                                                       const int32_t* __restrict__ work, int T, int H,
                                                                       int I, int top_k) {
  typedef typename ET<E>::vec vec;
  extern __shared__ char lds_raw[];
  vec* sb = reinterpret_cast<vec*>(lds_raw);
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N;
  if ((int)blockIdx.y >= work[0]) return;   // uniform over the block
  const int item = work[1 + blockIdx.y], e = item >> 16;
  const int n_rows = cnt[e], row0 = (item & 0xffff) * WT * TILE;
  const int nt = min(WT, (n_rows - row0 + TILE - 1) / TILE);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int n_tasks = I / TILE, task = min((int)blockIdx.x * EXPERT_WW + wave, n_tasks - 1);
  const int base = off[e];
  const int ksteps = H / KS;
  int tok[WT];
  float r[WT];
#pragma unroll
  for (int t = 0; t < WT; ++t) {
    tok[t] = perm[base + min(row0 + t * TILE + col, n_rows - 1)] / top_k;
    r[t] = rinv[tok[t]];
  }
  int stage_tok = tok[0];
#pragma unroll
  for (int t = 1; t < WT; ++t)
    if (wave % WT == t) stage_tok = tok[t];
  const E* brow = xn + (int64_t)stage_tok * (NP * KS) + half * G;
  f32x16 acc0[WT], acc1[WT];
  zero_acc<WT>(acc0);
  zero_acc<WT>(acc1);
  wide_stream<E, WT, EXPERT_WW, EXPERT_PRE, 10>(W + ((int64_t)e * n_tasks + task) * task_stride_elems<E>(ksteps) + lane * G, ksteps / WKC, brow,
                 (int64_t)T * (NP * KS), sb, nt, acc0, acc1);
  if ((int)blockIdx.x * EXPERT_WW + wave >= n_tasks) return;
#pragma unroll
  for (int t = 0; t < WT; ++t) {
    const int row = row0 + t * TILE + col;
    if (t < nt && row < n_rows) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {   // accumulator registers 4g .. 4g+3 are four consecutive features
        f32x4 y;
#pragma unroll
        for (int i = 0; i < 4; ++i) y[i] = silu_w(acc0[t][4 * g + i] * r[t]) * (acc1[t][4 * g + i] * r[t]);
        store_actk4<E>(Y, (int64_t)T * top_k, base + row, task * TILE + acc_row(4 * g, half), y);
      }
    }
  }
}

template <typename E>
__global__ __launch_bounds__(EXPERT_WW * WAVE) void expert_gemm2_wide_kernel(const E* __restrict__ W, const E* __restrict__ Y,
                                                                       float* __restrict__ O, const int32_t* __restrict__ cnt,
                                                                       const int32_t* __restrict__ off,
                                                                       const int32_t* __restrict__ perm,
                                                                       const int32_t* __restrict__ work, int n_pairs,
                                                                       int H, int I) {
  typedef typename ET<E>::vec vec;
  extern __shared__ char lds_raw[];
  vec* sb = reinterpret_cast<vec*>(lds_raw);
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N;
  if ((int)blockIdx.y >= work[0]) return;
  const int item = work[1 + blockIdx.y], e = item >> 16;
  const int n_rows = cnt[e], row0 = (item & 0xffff) * WT * TILE;
  const int nt = min(WT, (n_rows - row0 + TILE - 1) / TILE);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int n_tasks = H / (2 * TILE), task = min((int)blockIdx.x * EXPERT_WW + wave, n_tasks - 1);
  const int base = off[e];
  const int ksteps = I / KS;
  int pair[WT];
#pragma unroll
  for (int t = 0; t < WT; ++t) pair[t] = perm[base + min(row0 + t * TILE + col, n_rows - 1)];
  const E* brow = Y + (int64_t)(base + min(row0 + (wave % WT) * TILE + col, n_rows - 1)) * (NP * KS) + half * G;
  f32x16 acc0[WT], acc1[WT];
  zero_acc<WT>(acc0);
  zero_acc<WT>(acc1);
  wide_stream<E, WT, EXPERT_WW, EXPERT_PRE, 11>(W + ((int64_t)e * n_tasks + task) * task_stride_elems<E>(ksteps) + lane * G, ksteps / WKC, brow,
                 (int64_t)n_pairs * (NP * KS), sb, nt, acc0, acc1);
  if ((int)blockIdx.x * EXPERT_WW + wave >= n_tasks) return;
#pragma unroll
  for (int t = 0; t < WT; ++t) {
    if (t < nt && row0 + t * TILE + col < n_rows) {
      float* orow = O + (int64_t)pair[t] * H + (2 * task) * TILE;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 a, b;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          a[i] = acc0[t][4 * g + i];
          b[i] = acc1[t][4 * g + i];
        }
        *reinterpret_cast<f32x4*>(orow + acc_row(4 * g, half)) = a;
        *reinterpret_cast<f32x4*>(orow + TILE + acc_row(4 * g, half)) = b;
      }
    }
  }
}

template <typename E> static void launch_gate_up_wide_t(const ExpertArgs& a, hipStream_t st) {
  const int n_tasks = a.I / TILE;
  expert_gemm1_wide_kernel<E><<<dim3((n_tasks + EXPERT_WW - 1) / EXPERT_WW, expert_work_items(a.E, a.T * a.top_k)),
                                EXPERT_WW * WAVE, wide_lds<E, 10, WT>(), st>>>(
      (const E*)a.w_gate_up, (const E*)a.xn, a.rinv, (E*)a.y, a.cnt, a.off, a.perm, a.work, a.T, a.H, a.I, a.top_k);
}
template <typename E> static void launch_down_wide_t(const ExpertArgs& a, hipStream_t st) {
  const int n_tasks = a.H / (2 * TILE);
  expert_gemm2_wide_kernel<E><<<dim3((n_tasks + EXPERT_WW - 1) / EXPERT_WW, expert_work_items(a.E, a.T * a.top_k)),
                                EXPERT_WW * WAVE, wide_lds<E, 11, WT>(), st>>>(
      (const E*)a.w_down, (const E*)a.y, a.o, a.cnt, a.off, a.perm, a.work, a.T * a.top_k, a.H, a.I);
}
void launch_expert_gate_up_wide(bool bf16, const ExpertArgs& a, hipStream_t st) {
  if (bf16) launch_gate_up_wide_t<bf16_t>(a, st);
  else launch_gate_up_wide_t<float>(a, st);
}
void launch_expert_down_wide(bool bf16, const ExpertArgs& a, hipStream_t st) {
  if (bf16) launch_down_wide_t<bf16_t>(a, st);
  else launch_down_wide_t<float>(a, st);
}

// ------------------------------------------------------------------------------------------------
// LM head fused with the confidence reduction, many-token form.  A workgroup takes one task group (8 tasks = 512
// vocabulary ids) and one group of 128 tokens; a wave turns its accumulators (64 vocabulary ids x 128 tokens) into
// one (max, sum-exp, lowest arg max) partial per token: part[task group * 8 + wave][token].  Logits are never
// stored (unless the debug pointer is set).
// The token groups of one task group stream the same weights.  Workgroups go to the dies in turn, so the launch is
// one-dimensional and workgroup i = die (i % 8), turn (i / 8): consecutive turns of ONE die take the token groups
// of one task group, which then run side by side behind the same L2 (measured at 512 tokens: 0.88 GB fetched from
// HBM per launch for 0.64 GB of weights, where four separate passes would fetch 2.6 GB).
// ------------------------------------------------------------------------------------------------
template <typename E, int WT, int KID, int WW>
__global__ __launch_bounds__(WW * WAVE) void lm_head_wide_kernel(const E* __restrict__ W, const E* __restrict__ xn,
                                                                  const float* __restrict__ rinv, int T, int H, int V,
                                                                  float scale, float* __restrict__ part,
                                                                  float* __restrict__ logits_out) {
  typedef typename ET<E>::vec vec;
  extern __shared__ char lds_raw[];
  vec* sb = reinterpret_cast<vec*>(lds_raw);
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int groups = (T + WT * TILE - 1) / (WT * TILE);
  const int turn = blockIdx.x / XCDS;
  const int tgroup = (turn / groups) * XCDS + blockIdx.x % XCDS;
  const int n_tasks = (V + 2 * TILE - 1) / (2 * TILE);
  if (tgroup * WW >= n_tasks) return;   // uniform over the workgroup
  const int tok0 = (turn % groups) * WT * TILE;
  const int nt = min(WT, (T - tok0 + TILE - 1) / TILE);
  const int slot = tgroup * WW + wave, task = min(slot, n_tasks - 1);
  const int ksteps = H / KS;
  float zs[WT];
#pragma unroll
  for (int t = 0; t < WT; ++t) zs[t] = rinv[min(tok0 + t * TILE + col, T - 1)] * scale;
  const E* brow = xn + (int64_t)min(tok0 + (wave % WT) * TILE + col, T - 1) * (NP * KS) + half * G;
  f32x16 acc0[WT], acc1[WT];
  zero_acc<WT>(acc0);
  zero_acc<WT>(acc1);
  wide_stream<E, WT, WW, LM_PRE, KID>(W + (int64_t)task * task_stride_elems<E>(ksteps) + lane * G, ksteps / WKC, brow, (int64_t)T * (NP * KS),
                 sb, nt, acc0, acc1);
#pragma unroll
  for (int t = 0; t < WT; ++t) {
    const int tok = tok0 + t * TILE + col;
    float m = -INFINITY, sum = 0.f;
    int best = 0x7fffffff;
    if (t < nt && slot < n_tasks) {
      float z[32];
#pragma unroll
      for (int i = 0; i < 32; ++i) {   // ids ascend with i inside each tile; tile 1 follows tile 0
        const int id = (2 * task + (i >> 4)) * TILE + acc_row(i & 15, half);
        const float a = i < 16 ? acc0[t][i & 15] : acc1[t][i & 15];
        z[i] = id < V ? a * zs[t] : -INFINITY;
        if (z[i] > m) {                // strict '>' keeps the lowest id
          m = z[i];
          best = id;
        }
        if (logits_out && tok < T && id < V) logits_out[(int64_t)tok * V + id] = z[i];
      }
      if (m > -INFINITY) {
#pragma unroll
        for (int i = 0; i < 32; ++i) sum += __expf(z[i] - m);
      }
    }
    // fold the two half-waves (same token, other rows)
    const float om = __shfl_xor(m, 32, WAVE), os = __shfl_xor(sum, 32, WAVE);
    const int ob = __shfl_xor(best, 32, WAVE);
    float M = m, S = sum;
    int B = best;
    if (om > M || (om == M && ob < B)) {
      S = (M > -INFINITY ? S * __expf(M - om) : 0.f) + os;
      M = om;
      B = ob;
    } else if (om > -INFINITY) {
      S += os * __expf(om - M);
    }
    if (half == 0 && tok < T && t < nt) {
      float* p = part + ((int64_t)slot * T + tok) * 4;
      p[0] = M;
      p[1] = S;
      p[2] = __int_as_float(B);
      p[3] = 0.f;
    }
  }
}

int lm_head_wide_parts(int V) { return ((V + 63) / 64 + LM_WW - 1) / LM_WW * LM_WW; }

// Up to 64 tokens: two token tiles per workgroup and both activation planes (trace id 14): there the weight stream
// is the bound, and sharing the activation fragments of eight tasks relieves the address unit, which would
// otherwise take every lane's own activation row one by one.  More tokens: four tiles, high plane only (id 9).
template <typename E> static void launch_lm_wide_t(const LmArgs& a, hipStream_t st) {
  if (a.T <= 2 * TILE) {   // four tasks per workgroup: 614 work units spread more evenly over 256 compute units than 307
    const int tgroups = lm_head_wide_parts(a.V) / 4;
    lm_head_wide_kernel<E, 2, 14, 4><<<(tgroups + XCDS - 1) / XCDS * XCDS, 4 * WAVE, wide_lds<E, 14, 2>(), st>>>(
        (const E*)a.w, (const E*)a.xn, a.rinv, a.T, a.H, a.V, a.scale, a.part, a.logits_out);
    return;
  }
  const int tgroups = lm_head_wide_parts(a.V) / LM_WW;
  const int groups = (a.T + WT * TILE - 1) / (WT * TILE);
  lm_head_wide_kernel<E, WT, 9, LM_WW><<<(tgroups + XCDS - 1) / XCDS * XCDS * groups, LM_WW * WAVE, wide_lds<E, 9, WT>(), st>>>(
      (const E*)a.w, (const E*)a.xn, a.rinv, a.T, a.H, a.V, a.scale, a.part, a.logits_out);
}
void launch_lm_head_wide(bool bf16, const LmArgs& a, hipStream_t st) {
  if (bf16) launch_lm_wide_t<bf16_t>(a, st);
  else launch_lm_wide_t<float>(a, st);
}

bool configure_wide() {
  const void* fns[6] = {(const void*)expert_gemm1_wide_kernel<bf16_t>, (const void*)expert_gemm1_wide_kernel<float>,
                        (const void*)expert_gemm2_wide_kernel<bf16_t>, (const void*)expert_gemm2_wide_kernel<float>,
                        (const void*)lm_head_wide_kernel<bf16_t, WT, 9, LM_WW>, (const void*)lm_head_wide_kernel<float, WT, 9, LM_WW>};
  for (const void* f : fns)
    if (hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess) return false;
  return true;
}

TRACE_READER(trace_read_wide)

}  // namespace dinfer
