// Shared-operand weight streaming for forwards with many token rows: a workgroup of WW waves covers WW tasks
// (64 output features each) and WT tiles of 32 token rows.  Each wave streams the weights of its task from memory
// into registers for the whole K range; the activation fragments of the WT token tiles go through LDS, staged
// chunk by chunk (WKC k-steps) and double buffered, so that every fragment is fetched once per workgroup.
#pragma once
#include <type_traits>

#include "gemm.hpp"

namespace dinfer {

constexpr int WKC = 4;     // k-steps per staged chunk
// LDS fragments read ahead of the matrix instructions that use them (pinned by scheduling barriers, see the chunk
// body), and the chunks of activation fragments a wave holds in registers on their way to LDS: two everywhere
// except in the many-token expert GEMMs (trace ids 10, 11), whose 128 accumulator registers and two activation
// planes leave room for one only (with two, the pinned read-ahead spills and they run at half speed).
constexpr int WIDE_FD = 4;
template <int KID> constexpr int wide_bdepth() { return (KID == 10 || KID == 11) ? 1 : 2; }

// Planes of the activations a kernel (by its trace id) feeds to the matrix cores.  The LM head with hundreds of
// token rows is bound by the matrix cores, and its rounding error is not carried into later layers: it takes the
// high bf16 plane only, that is activations rounded to bf16 as in the paper's arithmetic (bf16 inputs, float32
// accumulation); the low plane would double its matrix work.  The expert GEMMs stay bound by their weight streams
// and keep both planes (one plane: 7 % faster, but the error carried through 16 layers reaches the test bars).
template <typename E, int KID> struct WidePlanes { static constexpr int N = Planes<E>::N; };
template <> struct WidePlanes<bf16_t, 9> { static constexpr int N = 1; };

template <int N, class F, int I = 0> __device__ inline void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, F, I + 1>(static_cast<F&&>(f));
  }
}

template <typename E, int KID, int WT> constexpr size_t wide_lds() { return (size_t)2 * WKC * WT * WidePlanes<E, KID>::N * WAVE * 16; }

// Accumulate all n_chunks * WKC k-steps.  wp: this wave's task (k-step 0) + lane * G.  brow_of(): the k-major
// activation row this lane stages (row of token tile `wave % WT`) + (lane / 32) * G; bkstride: its k-step stride.
// sb: LDS [2][WKC][WT][planes][64] operand vectors.  NT: token tiles that hold rows.  wave: 0 .. WW-1, the
// wave's rank among the WW waves that share sb (every wave of the workgroup must make the call: it holds the
// workgroup's barriers).
// Pipeline per chunk c: barrier; the fragments of chunk c+1 go from registers to LDS buffer (c+1)&1 and the
// loads of chunk c+3 take their place; chunk c is multiplied out of buffer c&1; the weights of chunk c+WPRE are
// requested.  Loads past the end are clamped to the last chunk (never used), so the loop body has no branch
// around a load.  A wave stays within 256 registers, so that the eight waves of a workgroup fit on a compute unit.
template <typename E, int WT, int NT, int WW, int WPRE, int KID, class BRow>
__device__ inline void wide_stream_nt(const E* __restrict__ wp, int n_chunks, BRow&& brow_of, int64_t bkstride,
                                      typename ET<E>::vec* sb, f32x16 (&acc0)[WT], f32x16 (&acc1)[WT], int wave) {
  typedef typename ET<E>::vec vec;
  constexpr int G = ET<E>::G, KS = ET<E>::KS, NP = WidePlanes<E, KID>::N;   // planes used; the rows hold Planes<E>::N
  constexpr int64_t STEP = 2 * WAVE * G;
  // Weights that are streamed once (experts, LM head) are loaded non-temporally; those of the dense projections
  // (kernel ids 12, 13: a few MB that every token group reads again) must stay in the L2.
  auto wload = [](const E* p) { return (KID == 12 || KID == 13) ? load16<E>(p) : load16_stream<E>(p); };
  static_assert(WPRE % 2 == 0, "buffer parities are taken from the unrolled index");
  static_assert(WW % WT == 0 && (WKC * WT) % WW == 0, "every wave stages whole k-steps of one token tile");
  const int lane = threadIdx.x & 63;
  const int last = n_chunks - 1;
  TRACE_MARK(KID, 0);
  constexpr int SKS = WKC * WT / WW;               // k-steps of a chunk this wave stages (of token tile wave % WT)
  const int st = wave % WT, sk0 = (wave / WT) * SKS;
  vec wa0[WPRE][WKC], wa1[WPRE][WKC];
  constexpr int BD = wide_bdepth<KID>();
  vec bset[BD][SKS][NP];                           // fragments of the next BD chunks, on their way to LDS
  auto sb_at = [&](int buf, int ks, int t, int q) -> vec& { return sb[((((buf * WKC + ks) * WT + t) * NP + q) * WAVE) + lane]; };
  // Prologue: the weights of the first WPRE chunks are requested before anything else, since they hang on nothing;
  // brow_of() then resolves the activation row this lane stages (for the experts a chain of dependent loads through
  // the permutation), and the fragments of chunks 0 (to LDS), 1 and 2 (to registers) follow.
#pragma unroll
  for (int i = 0; i < WPRE; ++i) {
    const int c = min(i, last);
#pragma unroll
    for (int ks = 0; ks < WKC; ++ks) {
      wa0[i][ks] = wload(wp + (int64_t)(c * WKC + ks) * STEP);
      wa1[i][ks] = wload(wp + (int64_t)(c * WKC + ks) * STEP + WAVE * G);
    }
  }
  const E* __restrict__ brow = brow_of();
  {
    vec b0[SKS][NP];
    const int c1 = min(1, last), c2 = min(2, last);
#pragma unroll
    for (int ks = 0; ks < SKS; ++ks)
#pragma unroll
      for (int q = 0; q < NP; ++q) b0[ks][q] = load16<E>(brow + (int64_t)(sk0 + ks) * bkstride + q * KS);
#pragma unroll
    for (int ks = 0; ks < SKS; ++ks)
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        bset[1 % BD][ks][q] = load16<E>(brow + (int64_t)(c1 * WKC + sk0 + ks) * bkstride + q * KS);
        if constexpr (BD == 2) bset[0][ks][q] = load16<E>(brow + (int64_t)(c2 * WKC + sk0 + ks) * bkstride + q * KS);
      }
#pragma unroll
    for (int ks = 0; ks < SKS; ++ks)
#pragma unroll
      for (int q = 0; q < NP; ++q) sb_at(0, sk0 + ks, st, q) = b0[ks][q];
  }
  // One chunk; i = c % WPRE picks the weight registers and the LDS buffer parities at compile time.
  auto chunk = [&](auto I, int c) {
    constexpr int i = decltype(I)::value;
    __syncthreads();
    if (c == 0) TRACE_MARK(KID, 1);
    if (c == 1) TRACE_MARK(KID, 2);
    if (c == 2) TRACE_MARK(KID, 3);
    if (c == 16) TRACE_MARK(KID, 4);
    if (c == 17) TRACE_MARK(KID, 5);
    constexpr int nb = (i + 1) & 1, cb = i & 1;   // WPRE is even: parities of c+1 and c
#pragma unroll
    for (int ks = 0; ks < SKS; ++ks)
#pragma unroll
      for (int q = 0; q < NP; ++q) sb_at(nb, sk0 + ks, st, q) = bset[nb % BD][ks][q];
    const int cn = min(c + 1 + BD, last);
#pragma unroll
    for (int ks = 0; ks < SKS; ++ks)
#pragma unroll
      for (int q = 0; q < NP; ++q)
        bset[nb % BD][ks][q] = load16<E>(brow + (int64_t)(cn * WKC + sk0 + ks) * bkstride + q * KS);
    // Fragment pipeline: the LDS read of fragment f + FD is issued before the matrix instructions of fragment f, and
    // a scheduling barrier keeps the compiler from sinking it back next to its use (left alone it keeps only two
    // reads in flight and the matrix pipe waits for LDS after every four instructions; measured at 512 tokens: LM
    // head 362 -> 322 us, QKV 41.7 -> 38.7 us, expert gate/up 118 -> 113 us).  Fragments in the order (k-step, token tile, plane).
    constexpr int F = WKC * NT * NP;
    constexpr int FD = WIDE_FD < F ? WIDE_FD : F;
    vec ring[FD];
    auto frag = [&](int f) -> vec& { return sb_at(cb, f / (NT * NP), (f / NP) % NT, f % NP); };
    static_for<FD>([&](auto J) { ring[decltype(J)::value] = frag(decltype(J)::value); });
    static_for<F>([&](auto Fi) {
      constexpr int f = decltype(Fi)::value, ks = f / (NT * NP), t = (f / NP) % NT;
      const vec b = ring[f % FD];
      if constexpr (f + FD < F) ring[f % FD] = frag(f + FD);
      __builtin_amdgcn_sched_barrier(0);
      mfma32(acc0[t], wa0[i][ks], b);
      mfma32(acc1[t], wa1[i][ks], b);
    });
    const int cw = min(c + WPRE, last);
#pragma unroll
    for (int ks = 0; ks < WKC; ++ks) {
      wa0[i][ks] = wload(wp + (int64_t)(cw * WKC + ks) * STEP);
      wa1[i][ks] = wload(wp + (int64_t)(cw * WKC + ks) * STEP + WAVE * G);
    }
  };
  // Whole rounds of WPRE chunks run without a test between the chunks: a branch there gives the compiler a path from
  // one chunk straight back to the loop top, for which it drains every load in flight at each iteration.
  // The first round stands in front of the loop: the prologue leaves the loads in another order than a round does
  // (all weights first, then the fragments), and the wait counts the compiler puts at the loop top are the smaller
  // of what its two ways in allow -- entered straight from the prologue, every chunk waited until all but four of
  // the loads in flight had returned, the weights requested one chunk earlier included, and a wave had one chunk
  // of weights under way instead of WPRE.
  int c0 = 0;
  if (n_chunks >= WPRE) {
    static_for<WPRE>([&](auto I) { chunk(I, decltype(I)::value); });
    for (c0 = WPRE; c0 + WPRE <= n_chunks; c0 += WPRE) static_for<WPRE>([&](auto I) { chunk(I, c0 + decltype(I)::value); });
  }
  static_for<WPRE - 1>([&](auto I) {
    if (c0 + decltype(I)::value < n_chunks) chunk(I, c0 + decltype(I)::value);   // uniform over the workgroup
  });
  TRACE_MARK(KID, 6);
}

// nt: token tiles that hold rows (the others are skipped); the tile count is a compile-time constant of the loop.
// brow: a callable that returns the activation row pointer the lane stages (see wide_stream_nt).
template <typename E, int WT, int WW, int WPRE, int KID, class BRow>
__device__ inline void wide_stream(const E* __restrict__ wp, int n_chunks, BRow&& brow, int64_t bkstride,
                                   typename ET<E>::vec* sb, int nt, f32x16 (&acc0)[WT], f32x16 (&acc1)[WT],
                                   int wave = threadIdx.x >> 6) {
  if constexpr (WT >= 4) {
    if (nt >= 4) return wide_stream_nt<E, WT, 4, WW, WPRE, KID>(wp, n_chunks, brow, bkstride, sb, acc0, acc1, wave);
    if (nt == 3) return wide_stream_nt<E, WT, 3, WW, WPRE, KID>(wp, n_chunks, brow, bkstride, sb, acc0, acc1, wave);
  }
  if constexpr (WT >= 2) {
    if (nt >= 2) return wide_stream_nt<E, WT, 2, WW, WPRE, KID>(wp, n_chunks, brow, bkstride, sb, acc0, acc1, wave);
  }
  wide_stream_nt<E, WT, 1, WW, WPRE, KID>(wp, n_chunks, brow, bkstride, sb, acc0, acc1, wave);
}

}  // namespace dinfer
