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

// Accumulate k-steps [ks0, ks1) of one task for TT token tiles.
//   wtask : packed weights of the task (k-step 0), bp[tt]: this lane's activation row + (lane/32)*G in the
//   hi plane; the lo plane (bf16 only) sits `plane` elements further.
template <typename E, int TT, int PF>
__device__ inline void stream_task(const E* __restrict__ wtask, int ks0, int ks1, const E* const (&bp)[TT],
                                   int64_t plane, f32x16 (&acc0)[TT], f32x16 (&acc1)[TT]) {
  typedef typename ET<E>::vec vec;
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = Planes<E>::N;
  const int lane = threadIdx.x & (WAVE - 1);
  const E* wp = wtask + (int64_t)ks0 * (2 * WAVE * G) + lane * G;
  const int n = ks1 - ks0;
  vec a0[PF], a1[PF], b[PF][TT][NP];
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    if (i < n) {
      a0[i] = load16<E>(wp + (int64_t)i * (2 * WAVE * G));
      a1[i] = load16<E>(wp + (int64_t)i * (2 * WAVE * G) + WAVE * G);
#pragma unroll
      for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int q = 0; q < NP; ++q) b[i][t][q] = load16<E>(bp[t] + q * plane + (int64_t)(ks0 + i) * KS);
    }
  }
  for (int s = 0; s < n; s += PF) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      if (s + i < n) {
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
          for (int q = 0; q < NP; ++q) {
            mfma32(acc0[t], a0[i], b[i][t][q]);
            mfma32(acc1[t], a1[i], b[i][t][q]);
          }
        const int nx = s + i + PF;
        if (nx < n) {
          a0[i] = load16<E>(wp + (int64_t)nx * (2 * WAVE * G));
          a1[i] = load16<E>(wp + (int64_t)nx * (2 * WAVE * G) + WAVE * G);
#pragma unroll
          for (int t = 0; t < TT; ++t)
#pragma unroll
            for (int q = 0; q < NP; ++q) b[i][t][q] = load16<E>(bp[t] + q * plane + (int64_t)(ks0 + nx) * KS);
        }
      }
    }
  }
}

template <int TT> __device__ inline void zero_acc(f32x16 (&a)[TT]) {
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) a[t][v] = 0.f;
}

}  // namespace dinfer
