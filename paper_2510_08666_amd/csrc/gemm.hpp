// Weight-streaming GEMM core for skinny activations (a block of 32-512 tokens against a large weight
// matrix).  Weights are the MFMA "A" operand and are read exactly once, straight from HBM into registers,
// from a tile-packed layout in which every load of a wave is one contiguous KiB; the activations are the
// "B" operand (tokens along the 32 columns).
//
// Packed layout of a weight matrix [N][K]:  [task][kstep][2][64 lanes][16 bytes]
//   a task is a pair of 32-feature tiles that one wave accumulates together (the pairing is chosen per
//   matrix so that the epilogue finds its partner values in the same lane: rotary pairs, gate/up, ...);
//   lane l of a tile holds feature l%32 and the G input features  kstep*KS + (l/32)*G ... +G.
#pragma once
#include "common.hpp"

namespace dinfer {

template <typename E> __host__ __device__ constexpr int64_t task_stride_elems(int ksteps) {
  return (int64_t)ksteps * 2 * WAVE * ET<E>::G;
}

// Software-pipelined core: PF k-steps of loads are always in flight.  The loop body is straight-line (no
// predicated loads), so the compiler can count outstanding loads exactly and every MFMA waits only for its own
// operands; n must be a positive multiple of PF.
template <typename E, int TT, int PF>
__device__ inline void stream_steps(const E* __restrict__ wp, const E* const (&bp)[TT], int64_t plane, int ks0, int n,
                                    f32x16 (&acc0)[TT], f32x16 (&acc1)[TT]) {
  typedef typename ET<E>::vec vec;
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N;
  constexpr int64_t STEP = 2 * WAVE * G;   // elements of packed weights per k-step
  vec a0[PF], a1[PF], b[PF][TT][NP];
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    a0[i] = load16<E>(wp + i * STEP);
    a1[i] = load16<E>(wp + i * STEP + WAVE * G);
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int q = 0; q < NP; ++q) b[i][t][q] = load16<E>(bp[t] + q * plane + (int64_t)(ks0 + i) * KS);
  }
  for (int s = 0; s + PF < n; s += PF) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {
#pragma unroll
      for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int q = 0; q < NP; ++q) {
          mfma32(acc0[t], a0[i], b[i][t][q]);
          mfma32(acc1[t], a1[i], b[i][t][q]);
        }
      const int nx = s + i + PF;
      a0[i] = load16<E>(wp + nx * STEP);
      a1[i] = load16<E>(wp + nx * STEP + WAVE * G);
#pragma unroll
      for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int q = 0; q < NP; ++q) b[i][t][q] = load16<E>(bp[t] + q * plane + (int64_t)(ks0 + nx) * KS);
    }
  }
#pragma unroll
  for (int i = 0; i < PF; ++i)
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        mfma32(acc0[t], a0[i], b[i][t][q]);
        mfma32(acc1[t], a1[i], b[i][t][q]);
      }
}

// Accumulate k-steps [ks0, ks1) of one task for TT token tiles.
//   wtask : packed weights of the task (k-step 0), bp[tt]: this lane's activation row + (lane/32)*G in the
//   hi plane; the lo plane (bf16 only) sits `plane` elements further.
// The prefetch depth follows the step count (a wave-uniform choice): PFMAX when it divides, else 4, else 1.
template <typename E, int TT, int PFMAX>
__device__ inline void stream_task(const E* __restrict__ wtask, int ks0, int ks1, const E* const (&bp)[TT],
                                   int64_t plane, f32x16 (&acc0)[TT], f32x16 (&acc1)[TT]) {
  constexpr int G = ET<E>::G;
  const int lane = threadIdx.x & (WAVE - 1);
  const E* wp = wtask + (int64_t)ks0 * (2 * WAVE * G) + lane * G;
  const int n = ks1 - ks0;
  if (n <= 0) return;
  if (PFMAX > 4 && n % PFMAX == 0) stream_steps<E, TT, PFMAX>(wp, bp, plane, ks0, n, acc0, acc1);
  else if (n % 4 == 0) stream_steps<E, TT, 4>(wp, bp, plane, ks0, n, acc0, acc1);
  else stream_steps<E, TT, 1>(wp, bp, plane, ks0, n, acc0, acc1);
}

template <int TT> __device__ inline void zero_acc(f32x16 (&a)[TT]) {
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) a[t][v] = 0.f;
}

}  // namespace dinfer
