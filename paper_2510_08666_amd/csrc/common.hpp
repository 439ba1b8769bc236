// Shared device helpers of the dinfer HIP library (gfx950 only): element types, MFMA wrappers,
// wave-level reductions, and the structs passed from the host side to the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dinfer {

typedef __bf16 bf16_t;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int WAVE = 64;
constexpr int TILE = 32;        // features per weight tile = tokens per token tile (32x32 MFMA)
constexpr int PAGE = 16;        // tokens per KV page
constexpr int MAX_SEQS = 64;
constexpr int MAX_TOPK = 8;
constexpr int MAX_EXPERTS = 64;
constexpr int MAX_HIDDEN = 4096;
constexpr int CREDIT_CAP = 64;   // credited tokens a position can hold (= DINFER_CREDIT_CAP of the C header)
constexpr int ATTN_MAX_PAGES = 2048;   // pages of one sequence the attention kernel stages in LDS (32768 positions)

// Per element type: G = elements in one 16-byte lane chunk; one MFMA k-step covers KS = 2*G input features.
template <typename E> struct ET;
template <> struct ET<float> {
  static constexpr int G = 4, KS = 8;
  typedef f32x4 vec;
};
template <> struct ET<bf16_t> {
  static constexpr int G = 8, KS = 16;
  typedef bf16x8 vec;
};

__device__ inline float to_f32(float v) { return v; }
__device__ inline float to_f32(bf16_t v) { return (float)v; }
template <typename E> __device__ inline E from_f32(float v);
template <> __device__ inline float from_f32<float>(float v) { return v; }
template <> __device__ inline bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }   // round to nearest even

// Activations that feed the matrix cores as bf16 are kept as TWO bf16 planes, hi = bf16(v) and
// lo = bf16(v - hi), so that hi + lo carries ~16 mantissa bits: at small token counts the MFMA units idle
// behind the weight stream, and a second MFMA per weight tile buys back the precision that a single bf16
// rounding of every GEMM input would cost.  float32 activations need one plane.
template <typename E> struct Planes { static constexpr int N = 1; };
template <> struct Planes<bf16_t> { static constexpr int N = 2; };

template <typename E> __device__ inline void store_act(E* base, int64_t idx, int64_t plane, float v);
template <> __device__ inline void store_act<float>(float* base, int64_t idx, int64_t, float v) { base[idx] = v; }
template <> __device__ inline void store_act<bf16_t>(bf16_t* base, int64_t idx, int64_t plane, float v) {
  const bf16_t hi = (bf16_t)v;
  base[idx] = hi;
  base[idx + plane] = (bf16_t)(v - (float)hi);
}

// Four consecutive activations at once (idx a multiple of 4).
template <typename E> __device__ inline void store_act4(E* base, int64_t idx, int64_t plane, const f32x4& v);
template <> __device__ inline void store_act4<float>(float* base, int64_t idx, int64_t, const f32x4& v) {
  *reinterpret_cast<f32x4*>(base + idx) = v;
}
template <> __device__ inline void store_act4<bf16_t>(bf16_t* base, int64_t idx, int64_t plane, const f32x4& v) {
  bf16x4 hi, lo;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    hi[i] = (bf16_t)v[i];
    lo[i] = (bf16_t)(v[i] - (float)hi[i]);
  }
  *reinterpret_cast<bf16x4*>(base + idx) = hi;
  *reinterpret_cast<bf16x4*>(base + idx + plane) = lo;
}

// Stored activation matrices [n_rows][K] that feed the matrix cores as the B operand are kept "k-major":
//   [K / KS][n_rows][Planes<E>::N][KS]
// so that what a wave loads for one MFMA k-step (32 rows x 2 half-lanes x 16 bytes, both planes) is one
// contiguous piece for consecutive rows, and a handful of cache lines for gathered rows.
template <typename E> __device__ inline int64_t act_index(int64_t n_rows, int64_t row, int col) {
  constexpr int KS = ET<E>::KS, NP = Planes<E>::N;
  return ((int64_t)(col / KS) * n_rows + row) * (NP * KS) + col % KS;
}
template <typename E> __device__ inline void store_actk(E* base, int64_t n_rows, int64_t row, int col, float v) {
  store_act<E>(base, act_index<E>(n_rows, row, col), ET<E>::KS, v);
}
template <typename E> __device__ inline void store_actk4(E* base, int64_t n_rows, int64_t row, int col, const f32x4& v) {
  store_act4<E>(base, act_index<E>(n_rows, row, col), ET<E>::KS, v);   // col a multiple of 4
}

// Four consecutive stored elements at once (dst 8- or 16-byte aligned): one store instruction instead of four,
// which matters where every lane addresses a row of its own and the address unit takes the lanes one by one.
template <typename E> __device__ inline void store_elems4(E* dst, const f32x4& v);
template <> __device__ inline void store_elems4<float>(float* dst, const f32x4& v) { *reinterpret_cast<f32x4*>(dst) = v; }
template <> __device__ inline void store_elems4<bf16_t>(bf16_t* dst, const f32x4& v) {
  bf16x4 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = (bf16_t)v[i];
  *reinterpret_cast<bf16x4*>(dst) = o;
}

// acc[32 x 32] += A[32 x KS] * B[KS x 32].  Lane l supplies row (A) / column (B) l%32 and the G consecutive
// k values that start at (l/32)*G; result: lane l holds column l%32, rows 8*(v/4) + 4*(l/32) + v%4.
__device__ inline void mfma32(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}
__device__ inline void mfma32(f32x16& acc, const f32x4& a, const f32x4& b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[0], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[1], b[1], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2], b[2], acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[3], b[3], acc, 0, 0, 0);
}

// Row of accumulator register v within the 32-row tile, for a lane in half `half` (= lane / 32).
__device__ inline int acc_row(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

template <typename E> __device__ inline typename ET<E>::vec load16(const E* p) {
  return *reinterpret_cast<const typename ET<E>::vec*>(p);
}
// Weights are read once per forward: a streaming (non-temporal) load keeps them from evicting the activations
// that the same kernel re-reads from the L2 many times.
template <typename E> __device__ inline typename ET<E>::vec load16_stream(const E* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const typename ET<E>::vec*>(p));
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// 1/rms of residual row `tok` from the shares of its sum of squares that the row's producer left: ssq[n_ssq][T]
// (one share per 64-feature task of a projection epilogue, or a single share holding the whole sum).  The shares
// are added in index order, so every consumer of a row derives the same bits.
__device__ inline float row_rinv(const float* __restrict__ ssq, int n_ssq, int T, int tok, int H, float eps) {
  if (n_ssq == 1) return rsqrtf(ssq[tok] / H + eps);
  float s = 0.f;
  for (int j0 = 0; j0 < n_ssq; j0 += 32) {   // 32 independent loads at a time
    float v[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = ssq[(int64_t)min(j0 + i, n_ssq - 1) * T + tok];
#pragma unroll
    for (int i = 0; i < 32; ++i) s += j0 + i < n_ssq ? v[i] : 0.f;
  }
  return rsqrtf(s / H + eps);
}

// Data handed from one workgroup to another INSIDE a kernel goes through device-coherent accesses (they bypass
// the per-XCD L2, which is not coherent across the chip): no cache-wide write-back or invalidate is needed then.
__device__ inline void coherent_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float coherent_load(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The same device-coherent accesses for N = 1, 2 or 4 consecutive floats at once, through a buffer descriptor
// (cache policy sc1, what the compiler emits for the agent-scope accesses above).  off: byte offset from the
// descriptor's base, a multiple of 4 * N.
typedef __amdgpu_buffer_rsrc_t buf_rsrc;
__device__ inline buf_rsrc coherent_buffer(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
constexpr int COHERENT_AUX = 0x10;   // sc1
template <int N> __device__ inline void coherent_store_n(buf_rsrc r, uint32_t off, const float (&v)[N]) {
  static_assert(N == 1 || N == 2 || N == 4, "1, 2 or 4 floats");
  if constexpr (N == 4)
    __builtin_amdgcn_raw_buffer_store_b128(u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])},
                                           r, off, 0, COHERENT_AUX);
  else if constexpr (N == 2)
    __builtin_amdgcn_raw_buffer_store_b64(u32x2{__float_as_uint(v[0]), __float_as_uint(v[1])}, r, off, 0, COHERENT_AUX);
  else
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v[0]), r, off, 0, COHERENT_AUX);
}
template <int N> __device__ inline void coherent_load_n(buf_rsrc r, uint32_t off, float (&v)[N]) {
  static_assert(N == 1 || N == 2 || N == 4, "1, 2 or 4 floats");
  if constexpr (N == 4) {
    const u32x4 b = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, COHERENT_AUX);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(b[i]);
  } else if constexpr (N == 2) {
    const u32x2 b = __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, COHERENT_AUX);
    v[0] = __uint_as_float(b[0]);
    v[1] = __uint_as_float(b[1]);
  } else {
    v[0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, off, 0, COHERENT_AUX));
  }
}

// Completion ticket over the n workgroups that share the counter *c (zero before the first arrives): true in every
// thread of the workgroup that arrives last, which has then reset the counter for the next use.  What the other
// n-1 workgroups wrote with coherent_store before their call can be read with coherent_load afterwards: every
// thread waits for its own stores to complete, then one thread counts the arrival.  Nothing spins, so the order
// in which workgroups are scheduled does not matter.  Every thread of the workgroup must call.
__device__ inline bool last_arrival(int32_t* c, int n, int32_t* s_flag) {
  // vmcnt(0): this thread's write-through stores have been acknowledged.  As inline assembly with a memory clobber,
  // so that the compiler can neither sink a store below the wait nor hoist a later load above it.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const int last = atomicAdd(c, 1) == n - 1;
    if (last) atomicExch(c, 0);
    *s_flag = last;
  }
  __syncthreads();
  const bool last = *s_flag != 0;
  asm volatile("" ::: "memory");   // the partials are read only after the ticket has been seen
  return last;
}

// Index of the first workgroup that fetches region 0 in a launch whose first n_real workgroups do other work: the
// next multiple of 8, so that fetching workgroup first + i runs on the die of the later launch's workgroup i.
__host__ __device__ inline int l2_prefetch_first(int n_real) { return (n_real + 7) / 8 * 8; }
// Every thread of the workgroup reads its share of [p, p + bytes) with ordinary 16-byte loads and drops the data: the
// lines are then in this die's L2 (bytes: a multiple of 16).
__device__ inline void l2_fetch(const char* __restrict__ p, uint32_t bytes) {
  const uint32_t step = blockDim.x * 16;
  uint32_t acc = 0;
#pragma unroll 8
  for (uint32_t o = threadIdx.x * 16; o < bytes; o += step) {
    const u32x4 v = *reinterpret_cast<const u32x4*>(p + o);
    acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  asm volatile("" ::"v"(acc));   // the loads have a use, nothing is stored
}

// Steps that are enqueued before the host knows whether they are still needed (the inner loop of blockwise
// decoding without a host round trip per step) carry the address of a word that is zero once every mask was
// already empty when the step began: every kernel of such a step returns at once.  Null: an ordinary step.
__device__ inline bool step_is_dead(const int32_t* live) { return live != nullptr && *live == 0; }

// Which sequence a forward's packed tokens belong to: sequence s owns tokens [off[s], off[s+1]).
struct SeqSpan {
  int32_t n_seq;
  int32_t off[MAX_SEQS + 1];
};

// Where the KV pool keeps things.  Pool: [layer][page][K|V][head][PAGE*head_dim] elements.
// K part of a (page, head): [head_dim / kblk][slot][kblk] with kblk elements = 32 bytes, one k-step of the
// QK^T product: the 16 slots of a page lie next to each other for every k-step, so a wave's load of one k-step
// for the 32 keys of a tile touches two runs of 512 contiguous bytes (8 cache lines) instead of 32 rows.
// V part: [head_dim][slot] (transposed, so that the PV product finds the keys of one page contiguous per feature).
struct KvGeom {
  int64_t layer_stride;   // elements
  int64_t page_stride;    // elements = 2 * n_heads * PAGE * head_dim
  int32_t n_heads, head_dim;
  int32_t n_pages;
  int32_t kblk;           // elements in 32 bytes: 16 (bf16) or 8 (float)
};
// Page ids come from the caller's page table: keep every access inside the pool whatever they hold.
__device__ inline int safe_page(const KvGeom& g, int id) { return min(max(id, 0), g.n_pages - 1); }
__device__ inline int64_t kv_k_index(const KvGeom& g, int page, int head, int slot, int d) {
  return (int64_t)page * g.page_stride + (int64_t)head * PAGE * g.head_dim +
         ((int64_t)(d / g.kblk) * PAGE + slot) * g.kblk + d % g.kblk;
}
__device__ inline int64_t kv_v_index(const KvGeom& g, int page, int head, int slot, int d) {
  return (int64_t)page * g.page_stride + (int64_t)g.n_heads * PAGE * g.head_dim +
         ((int64_t)head * g.head_dim + d) * PAGE + slot;
}

// Attention: workgroups (splits) that share the keys of one (head, query tile) of a sequence with n_keys keys.  The
// key tiles (32 keys) of a pair are dealt round-robin to the 8 waves of its splits, and a wave holds the loads of two
// tiles at a time; its third tile costs another memory round trip (about 3 us at batch 1, where nothing else hides
// it).  Up to 24 tiles one workgroup takes the pair (at most three tiles per wave, no hand-off between workgroups);
// beyond, one split per 16 tiles, so that every wave has its whole share in flight at once.  The splits of a pair
// hand their partial results to whichever of them finishes last (arrival ticket), which merges them: no second
// kernel.  The host offers at most ATTN_MAX_SPLITS splits per pair; a sequence uses what its own key count asks for
// and the other workgroups exit at once.  Host (largest possible key count, for the grid and the workspace) and
// kernels (the sequence's own count) use the same rule.
constexpr int ATTN_MAX_SPLITS = 16;
__host__ __device__ inline int attn_splits_for(int n_keys) {
  const int tiles = (n_keys + 31) / 32;
  if (tiles <= 24) return 1;
  const int s = (tiles + 15) / 16;
  return s > ATTN_MAX_SPLITS ? ATTN_MAX_SPLITS : s;
}

// Optional in-kernel phase timestamps (builds with -DDINFER_TRACE=<kernel id> only): thread 0 of every workgroup
// of the chosen kernel stores the 100 MHz wall clock at each mark.  Kernel ids: 1 QKV, 2 O-proj, 3 router,
// 4 expert GEMM 1, 5 expert GEMM 2, 6 LM head, 7 attention, 8 combine, 9 / 10 / 11 many-token LM head / expert GEMM 1 /
// expert GEMM 2, 12 / 13 many-token QKV / output projection, 14 LM head of 33 to 64 tokens.
#ifdef DINFER_TRACE
constexpr int TRACE_WGS = 8192, TRACE_SLOTS = 8;
static __device__ unsigned long long g_trace[TRACE_WGS * TRACE_SLOTS];
#define TRACE_MARK(kid, slot)                                                                          \
  do {                                                                                                 \
    if ((kid) == DINFER_TRACE && threadIdx.x == 0) {                                                   \
      const unsigned wg_ = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;             \
      if (wg_ < (unsigned)TRACE_WGS) g_trace[wg_ * TRACE_SLOTS + (slot)] = wall_clock64();             \
    }                                                                                                  \
  } while (0)
// Per-wave variant: lane 0 of every wave marks, record index = workgroup * waves + wave.
#define TRACE_MARK_WAVE(kid, slot, n_waves)                                                            \
  do {                                                                                                 \
    if ((kid) == DINFER_TRACE && (threadIdx.x & 63) == 0) {                                            \
      const unsigned wg_ = ((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * (n_waves) + (threadIdx.x >> 6); \
      if (wg_ < (unsigned)TRACE_WGS) g_trace[wg_ * TRACE_SLOTS + (slot)] = wall_clock64();             \
    }                                                                                                  \
  } while (0)
#define TRACE_READER(name)                                                                             \
  int name(void* h_out, size_t bytes) {                                                                \
    if (bytes > sizeof(unsigned long long) * TRACE_WGS * TRACE_SLOTS) return -1;                       \
    return (int)hipMemcpyFromSymbol(h_out, HIP_SYMBOL(g_trace), bytes);                                \
  }
#else
#define TRACE_MARK(kid, slot) do {} while (0)
#define TRACE_MARK_WAVE(kid, slot, n_waves) do {} while (0)
#define TRACE_READER(name) int name(void*, size_t) { return -1; }
#endif

}  // namespace dinfer
