// Re-layout of a row-major weight matrix [N][K] into the tile-packed stream the GEMM kernels read
// (layout described in gemm.hpp).  Run once per tensor at load time.
#include "gemm.hpp"
#include "kernels.hpp"

namespace dinfer {

// Source tile (of 32 features) that lands in slot `which` of `task`.
__device__ inline int src_tile_of(int mode, int task, int which, int head_dim) {
  switch (mode) {
    case PACK_ADJACENT: return 2 * task + which;
    case PACK_ROPE_PAIR: {   // rotary partner features j and j + head_dim/2 of one head share a task
      const int per_head = head_dim / 64;
      const int head = task / per_head, jt = task % per_head;
      return head * (head_dim / 32) + jt + which * per_head;
    }
    default: return task;    // PACK_HALF0 / PACK_HALF1: one source matrix fills one slot of every task
  }
}

template <typename E>
__global__ __launch_bounds__(256) void pack_kernel(const E* __restrict__ src, E* __restrict__ dst, int N, int K,
                                                    int n_tasks, int mode, int head_dim) {
  constexpr int G = ET<E>::G, KS = ET<E>::KS;
  const int ksteps = K / KS;
  const int lane = threadIdx.x & 63;
  const int64_t chunk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);      // (task, kstep, which)
  const int64_t per_batch = (int64_t)n_tasks * ksteps * 2;
  if (chunk >= per_batch) return;
  const int which = (int)(chunk & 1);
  const int ks = (int)((chunk >> 1) % ksteps);
  const int task = (int)((chunk >> 1) / ksteps);
  if ((mode == PACK_HALF0 && which != 0) || (mode == PACK_HALF1 && which != 1)) return;
  const int b = blockIdx.y;
  const int feature = src_tile_of(mode, task, which, head_dim) * TILE + (lane & 31);
  const int k = ks * KS + (lane >> 5) * G;
  typename ET<E>::vec v;
  if (feature < N) {
    v = load16<E>(src + ((int64_t)b * N + feature) * K + k);
  } else {
#pragma unroll
    for (int i = 0; i < G; ++i) v[i] = (E)0.f;
  }
  E* d = dst + (int64_t)b * n_tasks * task_stride_elems<E>(ksteps) + (chunk * WAVE + lane) * G;
  *reinterpret_cast<typename ET<E>::vec*>(d) = v;
}

// The embedding matrix [V][H] as the A operand of (probabilities) . W_emb: output features are the H embedding
// columns, the contraction runs over the vocabulary, padded with zeros to Kpad.  dst: [H/64][Kpad/KS][2][64][16 B].
template <typename E>
__global__ __launch_bounds__(256) void pack_transposed_kernel(const E* __restrict__ src, E* __restrict__ dst, int V, int H,
                                                               int Kpad) {
  constexpr int G = ET<E>::G, KS = ET<E>::KS;
  const int ksteps = Kpad / KS;
  const int lane = threadIdx.x & 63;
  const int64_t chunk = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);      // (task, kstep, which)
  if (chunk >= (int64_t)(H / 64) * ksteps * 2) return;
  const int which = (int)(chunk & 1);
  const int ks = (int)((chunk >> 1) % ksteps);
  const int task = (int)((chunk >> 1) / ksteps);
  const int feature = (2 * task + which) * TILE + (lane & 31);
  const int k = ks * KS + (lane >> 5) * G;
  typename ET<E>::vec v;
#pragma unroll
  for (int i = 0; i < G; ++i) v[i] = k + i < V ? src[(int64_t)(k + i) * H + feature] : (E)0.f;
  *reinterpret_cast<typename ET<E>::vec*>(dst + (chunk * WAVE + lane) * G) = v;
}
void launch_pack_transposed(bool bf16, const void* src, void* dst, int V, int H, int Kpad, hipStream_t st) {
  const int ks = bf16 ? 16 : 8;
  const int64_t chunks = (int64_t)(H / 64) * (Kpad / ks) * 2;
  if (bf16)
    pack_transposed_kernel<bf16_t><<<(unsigned)((chunks + 3) / 4), 256, 0, st>>>((const bf16_t*)src, (bf16_t*)dst, V, H, Kpad);
  else
    pack_transposed_kernel<float><<<(unsigned)((chunks + 3) / 4), 256, 0, st>>>((const float*)src, (float*)dst, V, H, Kpad);
}

int64_t packed_bytes(bool bf16, int n_tasks, int K) {
  const int ks = bf16 ? 16 : 8;
  return (int64_t)n_tasks * (K / ks) * 2 * WAVE * 16;
}

void launch_pack(bool bf16, const void* src, void* dst, int batch, int N, int K, int n_tasks, int mode,
                 int head_dim, hipStream_t st) {
  const int ks = bf16 ? 16 : 8;
  const int64_t chunks = (int64_t)n_tasks * (K / ks) * 2;
  dim3 grid((unsigned)((chunks + 3) / 4), batch);
  if (bf16)
    pack_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)src, (bf16_t*)dst, N, K, n_tasks, mode, head_dim);
  else
    pack_kernel<float><<<grid, 256, 0, st>>>((const float*)src, (float*)dst, N, K, n_tasks, mode, head_dim);
}

}  // namespace dinfer
