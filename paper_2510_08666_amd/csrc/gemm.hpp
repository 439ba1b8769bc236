// Weight-streaming GEMM core for skinny activations (a block of 32-512 tokens against a large weight
// matrix).  Weights are the MFMA "A" operand and are read exactly once, straight from HBM into registers,
// from a tile-packed layout in which every load of a wave is one contiguous KiB; the activations are the
// "B" operand (tokens along the 32 columns).
//
// Packed layout of a weight matrix [N][K]:  [task][kstep][2][64 lanes][16 bytes]
//   a task is a pair of 32-feature tiles that one wave accumulates together (the pairing is chosen per
//   matrix so that the epilogue finds its partner values in the same lane: rotary pairs, gate/up, ...);
//   lane l of a tile holds feature l%32 and the G input features  kstep*KS + (l/32)*G ... +G.
//
// The B operand comes from a Loader:
//   Raw  issue(t, ks)                 start the loads of token tile t, k-step ks; the data is not touched
//   void finish(raw, t, ks, out[NP])  turn them into the NP MFMA operands (hi / lo planes for bf16)
// Keeping the two apart lets the pipeline below issue loads PF k-steps ahead of their use.
#pragma once
#include "common.hpp"

namespace dinfer {

template <typename E> __host__ __device__ constexpr int64_t task_stride_elems(int ksteps) {
  return (int64_t)ksteps * 2 * WAVE * ET<E>::G;
}

// Activations stored k-major (see act_index in common.hpp): normalised-input planes of the residual stream,
// attention output, expert intermediate.
template <typename E, int TT> struct PlaneLoader {
  typedef typename ET<E>::vec vec;
  static constexpr int NP = Planes<E>::N, KS = ET<E>::KS, G = ET<E>::G;
  struct Raw {
    vec p[NP];
  };
  const E* bp[TT];   // this lane's row in k-step 0, hi plane, + (lane/32)*G
  int64_t kstride;   // elements from one k-step to the next = n_rows * NP * KS
  __device__ void set(int t, const E* base, int64_t n_rows, int64_t row, int half) {
    bp[t] = base + row * (NP * KS) + half * G;
    kstride = n_rows * (NP * KS);
  }
  __device__ Raw issue(int t, int ks) const {
    Raw r;
#pragma unroll
    for (int q = 0; q < NP; ++q) r.p[q] = load16<E>(bp[t] + ks * kstride + q * KS);
    return r;
  }
  __device__ void finish(const Raw& r, int, int, vec (&out)[NP]) {
#pragma unroll
    for (int q = 0; q < NP; ++q) out[q] = r.p[q];
  }
};

// Software-pipelined core: PF k-steps of loads are always in flight.  The loop body is straight-line (no
// predicated loads), so the compiler can count outstanding loads exactly and every MFMA waits only for its own
// operands; n must be a positive multiple of PF.
// STREAM: the weights are read once per launch and loaded non-temporally (false where several token groups read the
// same weights again, as in the router).
template <typename E, int TT, int PF, bool STREAM, class Loader>
__device__ inline void stream_steps(const E* __restrict__ wp, Loader& ld, int ks0, int n, f32x16 (&acc0)[TT],
                                    f32x16 (&acc1)[TT]) {
  typedef typename ET<E>::vec vec;
  constexpr int G = ET<E>::G, NP = Planes<E>::N;
  constexpr int64_t STEP = 2 * WAVE * G;   // elements of packed weights per k-step
  auto wload = [](const E* p) { return STREAM ? load16_stream<E>(p) : load16<E>(p); };
  vec a0[PF], a1[PF];
  typename Loader::Raw raw[PF][TT];
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    a0[i] = wload(wp + i * STEP);
    a1[i] = wload(wp + i * STEP + WAVE * G);
  }
#pragma unroll
  for (int i = 0; i < PF; ++i)
#pragma unroll
    for (int t = 0; t < TT; ++t) raw[i][t] = ld.issue(t, ks0 + i);
  auto burst = [&](int s) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        vec b[NP];
        ld.finish(raw[i][t], t, ks0 + s + i, b);
#pragma unroll
        for (int q = 0; q < NP; ++q) {
          mfma32(acc0[t], a0[i], b[q]);
          mfma32(acc1[t], a1[i], b[q]);
        }
      }
      const int nx = s + i + PF;
      a0[i] = wload(wp + nx * STEP);
      a1[i] = wload(wp + nx * STEP + WAVE * G);
#pragma unroll
      for (int t = 0; t < TT; ++t) raw[i][t] = ld.issue(t, ks0 + nx);
    }
  };
  // The first burst stands in front of the loop: it meets the loads in the prologue's order (all weights, then all
  // activation fragments), the later ones slot by slot, and the wait counts at the top of a loop entered both ways
  // are the smaller of the two.
  if (PF < n) {
    burst(0);
    for (int s = PF; s + PF < n; s += PF) burst(s);
  }
#pragma unroll
  for (int i = 0; i < PF; ++i)
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      vec b[NP];
      ld.finish(raw[i][t], t, ks0 + n - PF + i, b);
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        mfma32(acc0[t], a0[i], b[q]);
        mfma32(acc1[t], a1[i], b[q]);
      }
    }
}

// Accumulate k-steps [ks0, ks1) of one task for TT token tiles; wtask = packed weights of the task (k-step 0).
// The prefetch depth follows the step count (a wave-uniform choice): PFMAX when it divides, else 4, else 1.
template <typename E, int TT, int PFMAX, bool STREAM = true, class Loader>
__device__ inline void stream_task(const E* __restrict__ wtask, int ks0, int ks1, Loader& ld, f32x16 (&acc0)[TT],
                                   f32x16 (&acc1)[TT]) {
  constexpr int G = ET<E>::G;
  const int lane = threadIdx.x & (WAVE - 1);
  const E* wp = wtask + (int64_t)ks0 * (2 * WAVE * G) + lane * G;
  const int n = ks1 - ks0;
  if (n <= 0) return;
  if (PFMAX > 4 && n % PFMAX == 0) stream_steps<E, TT, PFMAX, STREAM>(wp, ld, ks0, n, acc0, acc1);
  else if (n % 4 == 0) stream_steps<E, TT, 4, STREAM>(wp, ld, ks0, n, acc0, acc1);
  else stream_steps<E, TT, 1, STREAM>(wp, ld, ks0, n, acc0, acc1);
}

template <int TT> __device__ inline void zero_acc(f32x16 (&a)[TT]) {
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) a[t][v] = 0.f;
}

// The offset array is followed by the list of experts that received at least one row: off[ACTIVE_LIST + i] is
// the i-th such expert (ascending), off[ACTIVE_LIST + MAX_EXPERTS] their number.  The grouped GEMMs index their
// grid through it, so that workgroups of experts without rows sit at the end of the grid instead of leaving
// holes in the dispatch order.
constexpr int ACTIVE_LIST = MAX_EXPERTS + 1;
// ... and by one 16-byte record per listed expert, {expert, first sorted row, rows, 0}, at off[ACTIVE_RECORDS + 4*i]:
// everything a grouped-GEMM workgroup needs to know about its expert in a single load.
constexpr int ACTIVE_RECORDS = 2 * MAX_EXPERTS + 4;
// ... and by two running totals for benchmarks: experts with rows summed over the permutations built so far, and the
// number of permutations (one per layer and forward); dinfer_profile_start clears them.
constexpr int STAT_ACTIVE_SUM = ACTIVE_RECORDS + 4 * MAX_EXPERTS;
constexpr int STAT_PERMUTATIONS = STAT_ACTIVE_SUM + 1;
constexpr int OFF_INTS = STAT_PERMUTATIONS + 1;   // size of the offset array with everything behind it

}  // namespace dinfer
