// The weight-streaming contractions with the most bytes: routed-expert grouped GEMMs and the LM head, in the
// shared-operand form of wide_stream.hpp for every token count.  A workgroup takes a few tasks (64 output features
// each) and 1, 2 or 4 tiles of 32 token rows; each wave streams the whole K range of one task and keeps its
// accumulators in registers (no split of K, no fold), and the activation fragments go through LDS once per
// workgroup.  With hundreds of token rows a wave that fetched its own activation operands would pull several
// times more bytes through the L2 than it streams weights from HBM; with few rows it still keeps the compute
// unit's address path busy with 64 separate rows per load.  Above 64 tokens: 8 tasks x 128 rows per workgroup.
#include "kernels.hpp"
#include "wide_stream.hpp"

namespace dinfer {

constexpr int WT = 4;      // token tiles per workgroup above 64 tokens
// Waves (= tasks) per workgroup and weight chunks in flight per wave.  Eight waves put two on every SIMD, so one
// computes while the other waits for LDS or memory, and the activation fragments are shared by eight tasks.
// (Measured at 512 tokens: four waves with two, four or six weight chunks in flight are slower for the expert
// GEMMs, 131 to 134 against 120 microseconds; four waves in the LM head, 450 against 352.)
constexpr int EXPERT_WW = 8, EXPERT_PRE = 2;
constexpr int LM_WW = 8, LM_PRE = 2;
// Tasks per workgroup of the LM head up to 32 tokens.  All workgroups of these launches are resident at once and
// the dispatcher deals them evenly, so a launch lasts as long as the compute units with one workgroup more than the
// others: 614 workgroups of four tasks put 3 MB on some units and 2 MB on others (112 us), 1228 of two tasks 2.5 or
// 2 MB (108 us).
constexpr int LM_SMALL_WW = 2;
constexpr int XCDS = 8;      // accelerator dies, each with its own L2; workgroup i of a launch runs on die i % 8

__device__ inline float silu_w(float x) { return x / (1.f + __expf(-x)); }

// ------------------------------------------------------------------------------------------------
// Routed experts, rows of expert e = pairs perm[off[e] .. off[e]+cnt[e]).  Grid (tasks / 8, work items): a work item
// is an (expert, group of up to 128 rows) pair; the permutation kernel lists them heaviest first.
//   GEMM 1: task = 32 gate features + the same 32 up features;  y = silu(gate) * up  -> Y[sorted row][I]
//   GEMM 2: task = 64 adjacent output features of the down projection                -> O[token*top_k + slot][H]
// ------------------------------------------------------------------------------------------------
// What a workgroup of the expert GEMMs works on.  RECORDS: the y-th expert with rows, from the records the router's
// fused permutation leaves (at most 64 tokens, one row group per expert); otherwise the y-th item of the work list.
struct ExpertItem {
  int e, base, n_rows, row0;
};
template <int WT, bool RECORDS>
__device__ inline bool expert_item(const int32_t* __restrict__ cnt, const int32_t* __restrict__ off,
                                   const int32_t* __restrict__ work, ExpertItem& it) {
  if constexpr (RECORDS) {
    if ((int)blockIdx.y >= off[ACTIVE_LIST + MAX_EXPERTS]) return false;   // uniform over the block
    const int4 rec = *reinterpret_cast<const int4*>(off + ACTIVE_RECORDS + 4 * blockIdx.y);
    it = ExpertItem{rec.x, rec.y, rec.z, 0};
  } else {
    if ((int)blockIdx.y >= work[0]) return false;
    const int item = work[1 + blockIdx.y], e = item >> 16;
    it = ExpertItem{e, off[e], cnt[e], (item & 0xffff) * WT * TILE};
  }
  return true;
}

template <typename E, int WT, int WW, int KID, bool RECORDS>
__global__ __launch_bounds__(WW * WAVE) __attribute__((amdgpu_waves_per_eu(2))) void expert_gemm1_wide_kernel(const E* __restrict__ W, const E* __restrict__ xn,
                                                                      const float* __restrict__ rinv, E* __restrict__ Y,
                                                                      const int32_t* __restrict__ cnt,
                                                                      const int32_t* __restrict__ off,
                                                                      const int32_t* __restrict__ perm,
                                                                      const int32_t* __restrict__ work, int T, int H, int I,
                                                                      int top_k, const float* __restrict__ topk_w, const int32_t* __restrict__ live) {
  if (step_is_dead(live)) return;
  typedef typename ET<E>::vec vec;
  extern __shared__ __align__(16) char lds_raw[];   // 16-byte aligned: staged fragments move as 128-bit LDS accesses
  vec* sb = reinterpret_cast<vec*>(lds_raw);
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N;
  ExpertItem it;
  if (!expert_item<WT, RECORDS>(cnt, off, work, it)) return;
  const int e = it.e, base = it.base, n_rows = it.n_rows, row0 = it.row0;
  const int nt = min(WT, (n_rows - row0 + TILE - 1) / TILE);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int n_tasks = I / TILE, task = min((int)blockIdx.x * WW + wave, n_tasks - 1);
  const int ksteps = H / KS;
  float r[WT], wgt[WT];
  // the token rows hang on the permutation: that chain is resolved while the first weights are in flight
  auto brow = [&]() {
    int tok[WT];
#pragma unroll
    for (int t = 0; t < WT; ++t) {
      const int pair = perm[base + min(row0 + t * TILE + col, n_rows - 1)];
      tok[t] = pair / top_k;
      r[t] = rinv[tok[t]];
      wgt[t] = topk_w ? topk_w[pair] : 1.f;   // the routing weight, when the down projection sums the experts itself
    }
    int stage_tok = tok[0];
#pragma unroll
    for (int t = 1; t < WT; ++t)
      if (wave % WT == t) stage_tok = tok[t];
    return xn + (int64_t)stage_tok * (NP * KS) + half * G;
  };
  f32x16 acc0[WT], acc1[WT];
  zero_acc<WT>(acc0);
  zero_acc<WT>(acc1);
  wide_stream<E, WT, WW, EXPERT_PRE, KID>(W + ((int64_t)e * n_tasks + task) * task_stride_elems<E>(ksteps) + lane * G,
                                          ksteps / WKC, brow, (int64_t)T * (NP * KS), sb, nt, acc0, acc1);
  if ((int)blockIdx.x * WW + wave >= n_tasks) return;
#pragma unroll
  for (int t = 0; t < WT; ++t) {
    const int row = row0 + t * TILE + col;
    if (t < nt && row < n_rows) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {   // accumulator registers 4g .. 4g+3 are four consecutive features
        f32x4 y;
#pragma unroll
        for (int i = 0; i < 4; ++i) y[i] = silu_w(acc0[t][4 * g + i] * r[t]) * (acc1[t][4 * g + i] * r[t]) * wgt[t];
        store_actk4<E>(Y, (int64_t)T * top_k, base + row, task * TILE + acc_row(4 * g, half), y);
      }
    }
  }
}

template <typename E, int WT, int WW, int KID, bool RECORDS>
__global__ __launch_bounds__(WW * WAVE) __attribute__((amdgpu_waves_per_eu(2))) void expert_gemm2_wide_kernel(const E* __restrict__ W, const E* __restrict__ Y,
                                                                      float* __restrict__ O, const int32_t* __restrict__ cnt,
                                                                      const int32_t* __restrict__ off,
                                                                      const int32_t* __restrict__ perm,
                                                                      const int32_t* __restrict__ work, int n_pairs, int H,
                                                                      int I, const int32_t* __restrict__ live) {
  if (step_is_dead(live)) return;
  typedef typename ET<E>::vec vec;
  extern __shared__ __align__(16) char lds_raw[];   // 16-byte aligned: staged fragments move as 128-bit LDS accesses
  vec* sb = reinterpret_cast<vec*>(lds_raw);
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N;
  ExpertItem it;
  if (!expert_item<WT, RECORDS>(cnt, off, work, it)) return;
  const int e = it.e, base = it.base, n_rows = it.n_rows, row0 = it.row0;
  const int nt = min(WT, (n_rows - row0 + TILE - 1) / TILE);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int n_tasks = H / (2 * TILE), task = min((int)blockIdx.x * WW + wave, n_tasks - 1);
  const int ksteps = I / KS;
  int pair[WT];
#pragma unroll
  for (int t = 0; t < WT; ++t) pair[t] = perm[base + min(row0 + t * TILE + col, n_rows - 1)];   // for the epilogue
  auto brow = [&]() { return Y + (int64_t)(base + min(row0 + (wave % WT) * TILE + col, n_rows - 1)) * (NP * KS) + half * G; };
  f32x16 acc0[WT], acc1[WT];
  zero_acc<WT>(acc0);
  zero_acc<WT>(acc1);
  wide_stream<E, WT, WW, EXPERT_PRE, KID>(W + ((int64_t)e * n_tasks + task) * task_stride_elems<E>(ksteps) + lane * G,
                                          ksteps / WKC, brow, (int64_t)n_pairs * (NP * KS), sb, nt, acc0, acc1);
  if ((int)blockIdx.x * WW + wave >= n_tasks) return;
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

// Up to 32 / 64 tokens: one / two token tiles and SMALL_WW tasks per workgroup, experts from the router's records
// (trace ids 16 .. 19); more: four tiles, eight tasks, the work list of the permutation kernel (ids 10, 11).
// (Measured, gate/up + down in microseconds: two tasks 69.8 + 37.6 at 32 tokens and 86.6 + 49.2 at 64; four tasks
// 68.9 + 38.9 and 88.1 + 50.7; the earlier per-wave-operand kernels, whose four waves split K, 72.9 + 38.6 and
// 100.5 + 55.2.  Four or six weight chunks in flight per wave instead of two: 71.9 + 39.4 at 32 tokens, 90.8 + 53.0
// at 64.)
constexpr int SMALL_WW = 2;
// The gate/up projection of up to 32 tokens takes one task per workgroup: with 49 to 56 experts touched, 16
// two-task workgroups per expert are 3.1 to 3.5 per compute unit, so some units carry four (2 MB) and the launch
// lasts as long as those; 32 one-task workgroups per expert put 1.75 MB on the fullest unit (78 -> 70 us for such
// layers, 69.1 -> 65.7 us on average at batch 1, though every workgroup now stages the activation rows for itself).
constexpr int GU1_WW = 1;

template <typename E> static void launch_gate_up_wide_t(const ExpertArgs& a, hipStream_t st) {
  const int n_tasks = a.I / TILE;
  const E *w = (const E*)a.w_gate_up, *xn = (const E*)a.xn;
  if (a.T <= TILE) {
    expert_gemm1_wide_kernel<E, 1, GU1_WW, 16, true><<<dim3((n_tasks + GU1_WW - 1) / GU1_WW, a.E), GU1_WW * WAVE,
                                                         wide_lds<E, 16, 1>(), st>>>(
        w, xn, a.rinv, (E*)a.y, a.cnt, a.off, a.perm, a.work, a.T, a.H, a.I, a.top_k, a.topk_w, live_word());
  } else if (a.T <= 2 * TILE) {
    expert_gemm1_wide_kernel<E, 2, SMALL_WW, 17, true><<<dim3((n_tasks + SMALL_WW - 1) / SMALL_WW, a.E), SMALL_WW * WAVE,
                                                         wide_lds<E, 17, 2>(), st>>>(
        w, xn, a.rinv, (E*)a.y, a.cnt, a.off, a.perm, a.work, a.T, a.H, a.I, a.top_k, a.topk_w, live_word());
  } else {
    expert_gemm1_wide_kernel<E, WT, EXPERT_WW, 10, false>
        <<<dim3((n_tasks + EXPERT_WW - 1) / EXPERT_WW, expert_work_items(a.E, a.T * a.top_k)), EXPERT_WW * WAVE,
           wide_lds<E, 10, WT>(), st>>>(w, xn, a.rinv, (E*)a.y, a.cnt, a.off, a.perm, a.work, a.T, a.H, a.I, a.top_k,
                                        a.topk_w, live_word());
  }
}
template <typename E> static void launch_down_wide_t(const ExpertArgs& a, hipStream_t st) {
  const int n_tasks = a.H / (2 * TILE), n_pairs = a.T * a.top_k;
  const E *w = (const E*)a.w_down, *y = (const E*)a.y;
  if (a.T <= TILE) {
    expert_gemm2_wide_kernel<E, 1, SMALL_WW, 18, true><<<dim3((n_tasks + SMALL_WW - 1) / SMALL_WW, a.E), SMALL_WW * WAVE,
                                                         wide_lds<E, 18, 1>(), st>>>(
        w, y, a.o, a.cnt, a.off, a.perm, a.work, n_pairs, a.H, a.I, live_word());
  } else if (a.T <= 2 * TILE) {
    expert_gemm2_wide_kernel<E, 2, SMALL_WW, 19, true><<<dim3((n_tasks + SMALL_WW - 1) / SMALL_WW, a.E), SMALL_WW * WAVE,
                                                         wide_lds<E, 19, 2>(), st>>>(
        w, y, a.o, a.cnt, a.off, a.perm, a.work, n_pairs, a.H, a.I, live_word());
  } else {
    expert_gemm2_wide_kernel<E, WT, EXPERT_WW, 11, false>
        <<<dim3((n_tasks + EXPERT_WW - 1) / EXPERT_WW, expert_work_items(a.E, n_pairs)), EXPERT_WW * WAVE,
           wide_lds<E, 11, WT>(), st>>>(w, y, a.o, a.cnt, a.off, a.perm, a.work, n_pairs, a.H, a.I, live_word());
  }
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
                                                                  RowNorm norm, int T, int H, int V,
                                                                  float scale, float* __restrict__ part,
                                                                  float* __restrict__ logits_out,
                                                                  const int32_t* __restrict__ rows,
                                                                  const int32_t* __restrict__ live) {
  if (step_is_dead(live)) return;
  typedef typename ET<E>::vec vec;
  extern __shared__ __align__(16) char lds_raw[];   // 16-byte aligned: staged fragments move as 128-bit LDS accesses
  vec* sb = reinterpret_cast<vec*>(lds_raw);
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  // With a row list the workgroup's 128 "tokens" are entries of the list, and the token groups are counted from
  // the list's length: the grid is sized for all T rows, and the workgroups left over at its end return at once.
  const int n_rows = rows ? min(rows[0], T) : T;
  if (n_rows == 0) return;              // uniform over the workgroup
  const int groups = (n_rows + WT * TILE - 1) / (WT * TILE);
  const int turn = blockIdx.x / XCDS;
  const int tgroup = (turn / groups) * XCDS + blockIdx.x % XCDS;
  const int n_tasks = (V + 2 * TILE - 1) / (2 * TILE);
  if (tgroup * WW >= n_tasks) return;   // uniform over the workgroup
  const int tok0 = (turn % groups) * WT * TILE;
  const int nt = min(WT, (n_rows - tok0 + TILE - 1) / TILE);
  const int slot = tgroup * WW + wave, task = min(slot, n_tasks - 1);
  const int ksteps = H / KS;
  auto row_of = [&](int i) { return rows ? min(max(rows[1 + min(i, n_rows - 1)], 0), T - 1) : min(i, T - 1); };
  int tok_of[WT];
  float zs[WT];
#pragma unroll
  for (int t = 0; t < WT; ++t) {
    tok_of[t] = row_of(tok0 + t * TILE + col);
    zs[t] = row_rinv(norm.ssq, norm.n_ssq, T, tok_of[t], H, norm.eps) * scale;
  }
  const E* brow = xn + (int64_t)row_of(tok0 + (wave % WT) * TILE + col) * (NP * KS) + half * G;
  f32x16 acc0[WT], acc1[WT];
  zero_acc<WT>(acc0);
  zero_acc<WT>(acc1);
  wide_stream<E, WT, WW, LM_PRE, KID>(W + (int64_t)task * task_stride_elems<E>(ksteps) + lane * G, ksteps / WKC, [&] { return brow; }, (int64_t)T * (NP * KS),
                 sb, nt, acc0, acc1);
#pragma unroll
  for (int t = 0; t < WT; ++t) {
    const bool listed = tok0 + t * TILE + col < n_rows;
    const int tok = listed ? tok_of[t] : T;     // T: no row
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
  if (a.T <= TILE) {   // one token tile (trace id 15)
    const int tgroups = lm_head_wide_parts(a.V) / LM_SMALL_WW;
    lm_head_wide_kernel<E, 1, 15, LM_SMALL_WW><<<(tgroups + XCDS - 1) / XCDS * XCDS, LM_SMALL_WW * WAVE, wide_lds<E, 15, 1>(), st>>>(
        (const E*)a.w, (const E*)a.xn, a.norm, a.T, a.H, a.V, a.scale, a.part, a.logits_out, a.rows, live_word());
    return;
  }
  if (a.T <= 2 * TILE) {   // four tasks per workgroup (two: 144 against 119 us, the activation fragments of 64 rows are shared by too few)
    const int tgroups = lm_head_wide_parts(a.V) / 4;
    lm_head_wide_kernel<E, 2, 14, 4><<<(tgroups + XCDS - 1) / XCDS * XCDS, 4 * WAVE, wide_lds<E, 14, 2>(), st>>>(
        (const E*)a.w, (const E*)a.xn, a.norm, a.T, a.H, a.V, a.scale, a.part, a.logits_out, a.rows, live_word());
    return;
  }
  const int tgroups = lm_head_wide_parts(a.V) / LM_WW;
  const int groups = (a.T + WT * TILE - 1) / (WT * TILE);
  lm_head_wide_kernel<E, WT, 9, LM_WW><<<(tgroups + XCDS - 1) / XCDS * XCDS * groups, LM_WW * WAVE, wide_lds<E, 9, WT>(), st>>>(
      (const E*)a.w, (const E*)a.xn, a.norm, a.T, a.H, a.V, a.scale, a.part, a.logits_out, a.rows, live_word());
}
void launch_lm_head_wide(bool bf16, const LmArgs& a, hipStream_t st) {
  if (bf16) launch_lm_wide_t<bf16_t>(a, st);
  else launch_lm_wide_t<float>(a, st);
}

bool configure_wide() {
  const void* fns[6] = {(const void*)expert_gemm1_wide_kernel<bf16_t, WT, EXPERT_WW, 10, false>,
                        (const void*)expert_gemm1_wide_kernel<float, WT, EXPERT_WW, 10, false>,
                        (const void*)expert_gemm2_wide_kernel<bf16_t, WT, EXPERT_WW, 11, false>,
                        (const void*)expert_gemm2_wide_kernel<float, WT, EXPERT_WW, 11, false>,
                        (const void*)lm_head_wide_kernel<bf16_t, WT, 9, LM_WW>, (const void*)lm_head_wide_kernel<float, WT, 9, LM_WW>};
  for (const void* f : fns)
    if (hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess) return false;
  return true;
}

TRACE_READER(trace_read_wide)

}  // namespace dinfer
