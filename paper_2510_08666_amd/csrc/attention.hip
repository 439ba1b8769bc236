// Bidirectional (non-causal) attention of a tile of 32 query tokens over every key of its sequence: the
// cached prefix pages plus the tokens of this forward, read through the page table.
//
// Work split: grid (split, head, query tile), ATTN_WAVES waves per workgroup.  A sequence uses as many of the
// grid's splits as its own key count asks for (attn_splits_for; the other workgroups exit at once), and its key
// tiles (32 keys) are dealt round-robin to the waves of those splits.  Each wave keeps its own online-softmax
// state; the waves of a workgroup are folded through LDS in wave order, each wave finishing its share of the
// output rows.  With one split the workgroup writes the normalised output itself; otherwise it leaves one
// partial (unnormalised output, max, sum) and takes an arrival ticket of its (query tile, head); the workgroup
// that arrives last folds the partials in split order and writes the output.
//
// MFMA mapping (32x32 tiles):  S^T[key][query] = K_tile . Q^T   (A = K rows, B = Q columns), so a lane owns
// one query column and softmax statistics are per lane;  O^T[d][query] += V^T_tile . P^T  (A = V^T rows read
// from the transposed V page, B = P^T taken from the S^T accumulator registers without any shuffle).
#include "gemm.hpp"
#include "kernels.hpp"

namespace dinfer {

constexpr int ATTN_WAVES = 8;
constexpr int ATTN_FETCH_MAX_OWN = 64;   // launches with at most this many workgroups of their own also fetch AttnArgs::pf

size_t attn_part_floats(int n_qtiles, int n_heads, int n_splits, int head_dim) {
  return (size_t)n_qtiles * n_heads * n_splits * TILE * (head_dim + 2);
}

// B operand of the PV product for k-step s2: the G probabilities this lane holds for that step's keys, and
// the matching A operand (V^T of those keys for feature row d).  Keys of accumulator register v sit at
// tile-local index acc_row(v, half).
template <typename E> struct PvStep;
template <> struct PvStep<bf16_t> {
  // step s2 in {0,1}: registers 8*s2 .. 8*s2+7 -> keys 16*s2 + {4h..4h+3, 8+4h..8+4h+3}
  static constexpr int STEPS = 2;
  // plane 0: bf16(p); plane 1: bf16(p - plane 0)
  __device__ static bf16x8 p_vec(const float (&p)[16], int s2, int plane) {
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bf16_t hi = (bf16_t)p[8 * s2 + i];
      r[i] = plane == 0 ? hi : (bf16_t)(p[8 * s2 + i] - (float)hi);
    }
    return r;
  }
  // vrow: V^T row of feature d inside the page of this step (16 slots contiguous)
  __device__ static bf16x8 v_vec(const bf16_t* vrow, int half, int /*s2*/) {
    const bf16x4 lo = *reinterpret_cast<const bf16x4*>(vrow + 4 * half);
    const bf16x4 hi = *reinterpret_cast<const bf16x4*>(vrow + 8 + 4 * half);
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      r[i] = lo[i];
      r[4 + i] = hi[i];
    }
    return r;
  }
  __device__ static int page_of_step(int s2) { return s2; }
  __device__ static int key_of(int s2, int half, int i) { return 16 * s2 + (i < 4 ? 4 * half + i : 8 + 4 * half + i - 4); }
};
template <> struct PvStep<float> {
  // step s2 in {0..3}: registers 4*s2 .. 4*s2+3 -> keys 8*s2 + 4h + {0..3}
  static constexpr int STEPS = 4;
  __device__ static f32x4 p_vec(const float (&p)[16], int s2, int /*plane*/) {
    f32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = p[4 * s2 + i];
    return r;
  }
  __device__ static f32x4 v_vec(const float* vrow, int half, int s2) {
    return *reinterpret_cast<const f32x4*>(vrow + 8 * (s2 & 1) + 4 * half);
  }
  __device__ static int page_of_step(int s2) { return s2 >> 1; }
  __device__ static int key_of(int s2, int half, int i) { return 8 * s2 + 4 * half + i; }
};

template <typename E, int HD>
__global__ __launch_bounds__(ATTN_WAVES * WAVE) void attention_kernel(const E* __restrict__ Q, int64_t q_plane,
                                                         const E* __restrict__ kv_layer, KvGeom geom, FwdMeta meta,
                                                         const int32_t* __restrict__ page_table, int pt_stride,
                                                         int n_splits, float* __restrict__ part,
                                                         int32_t* __restrict__ tickets, E* __restrict__ out,
                                                         int T_out, int n_qtiles, L2Prefetch pf,
                                                         const int32_t* __restrict__ live) {
  if (step_is_dead(live)) return;
  if ((int)blockIdx.z >= n_qtiles) {
    // not an attention workgroup: one that fetches a region of a later launch's weights into this die's L2
    const int index = (int)((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x);
    const int region = index - l2_prefetch_first(n_qtiles * gridDim.y * gridDim.x);
    if (region >= 0 && region < pf.n_regions) l2_fetch(pf.base + (size_t)region * pf.region_bytes, pf.region_bytes);
    return;
  }
  typedef typename ET<E>::vec vec;
  constexpr int G = ET<E>::G, KS = ET<E>::KS, DSTEPS = HD / KS, DT = HD / TILE, NP = Planes<E>::N;
  const int split = blockIdx.x, head = blockIdx.y, qt = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
  const int seq = meta.qtile[qt * 3 + 0], tok0 = meta.qtile[qt * 3 + 1], nvalid = meta.qtile[qt * 3 + 2];
  const int n_keys = meta.seq_nkeys[seq];
  const int my_splits = min(attn_splits_for(n_keys), n_splits);   // splits this sequence uses of those the grid offers
  if (split >= my_splits) return;                                  // uniform over the workgroup
  const int D = geom.n_heads * HD;
  const float scale = rsqrtf((float)HD);
  TRACE_MARK(7, 0);
  // The sequence's page-table row goes to LDS first: a tile's K / V addresses then need no global round trip
  // of their own, and the loads of the next tile can be issued at once.
  __shared__ int32_t pt[ATTN_MAX_PAGES];
  {
    const int32_t* row = page_table + (int64_t)seq * pt_stride;
    const int n_pages_used = (n_keys + PAGE - 1) / PAGE;       // <= pt_stride, <= ATTN_MAX_PAGES (host checks)
    for (int i = threadIdx.x; i < n_pages_used; i += blockDim.x) pt[i] = row[i];
  }

  // Q^T operand (queries and probabilities enter the MFMAs as hi + lo planes when E is bf16, like every
  // activation): all waves use the same query tile, so it is staged once in LDS in operand order
  // [head_dim k-step][plane][lane] and read from there in the tile loop instead of living in registers.
  __shared__ vec qs[DSTEPS * NP * WAVE];
  {
    const E* qrow = Q + (int64_t)(tok0 + min(col, nvalid - 1)) * D + head * HD + half * G;
    for (int i = wave; i < DSTEPS * NP; i += ATTN_WAVES)
      qs[i * WAVE + lane] = load16<E>(qrow + (i % NP) * q_plane + (i / NP) * KS);
  }
  __syncthreads();
  TRACE_MARK(7, 1);
  f32x16 o[DT];
  zero_acc<DT>(o);
  float m_run = -INFINITY, l_run = 0.f;

  const int n_ktiles = (n_keys + TILE - 1) / TILE;
  const int stride = my_splits * ATTN_WAVES;             // key tiles are dealt round-robin to all its waves
  const int kt0 = split * ATTN_WAVES + wave;
  // K rows and V^T rows of one key tile, loaded straight into MFMA operand registers
  struct TileRegs {
    vec k[DSTEPS];
    vec v[PvStep<E>::STEPS][DT];
  };
  auto load_tile = [&](int kt, TileRegs& r) {
    const int key = min(kt * TILE + col, n_keys - 1);
    const E* krow = kv_layer + kv_k_index(geom, safe_page(geom, pt[key / PAGE]), head, key % PAGE, 0) + half * G;
#pragma unroll
    for (int s = 0; s < DSTEPS; ++s) r.k[s] = load16<E>(krow + s * (PAGE * KS));   // k-step s of this slot
#pragma unroll
    for (int s2 = 0; s2 < PvStep<E>::STEPS; ++s2) {
      const int pkey = min(kt * TILE + PvStep<E>::page_of_step(s2) * PAGE, n_keys - 1);
      const int page = safe_page(geom, pt[pkey / PAGE]);
#pragma unroll
      for (int t = 0; t < DT; ++t)
        r.v[s2][t] = PvStep<E>::v_vec(kv_layer + kv_v_index(geom, page, head, 0, t * TILE + col), half, s2);
    }
  };
  // Softmax statistics live in the log2 domain (scores times scale * log2(e), one fused multiply-add in front of
  // the exponential).  A lane's reference maximum m_run moves only when a tile's maximum passes it by more than
  // REF_SLACK: probabilities are then bounded by 2^REF_SLACK instead of 1, which float32 sums and the bf16
  // hi + lo planes hold just as well, and the 64 output registers are rescaled only in the rare tile where some
  // lane's reference moves (a wave-uniform branch), not in every tile.
  constexpr float REF_SLACK = 6.f;
  const float c2 = scale * 1.44269504088896341f;
  auto use_tile = [&](TileRegs& cur, int kt) {
    // ---- S^T = K . Q^T  (the compiler barrier keeps the query reads inside the loop: hoisted, they would
    // occupy the 64 registers that staging them in LDS is meant to free)
    asm volatile("" ::: "memory");
    f32x16 sacc;
#pragma unroll
    for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
    {
      // the query fragments are read from LDS QD ahead of the matrix instructions that use them; the scheduling
      // barrier keeps the compiler from moving the reads back next to their use
      constexpr int QF = DSTEPS * NP, QD = 3;
      vec ring[QD];
#pragma unroll
      for (int f = 0; f < QD; ++f) ring[f] = qs[f * WAVE + lane];
#pragma unroll
      for (int f = 0; f < QF; ++f) {
        const vec b = ring[f % QD];
        if (f + QD < QF) ring[f % QD] = qs[(f + QD) * WAVE + lane];
        __builtin_amdgcn_sched_barrier(0);
        mfma32(sacc, cur.k[f / NP], b);
      }
    }
    if ((kt + 1) * TILE > n_keys) {
      // the sequence's last, ragged tile (wave-uniform, at most once per wave; the empty asm keeps it a branch):
      // scores of slots past the last key become -inf, and their V entries, which may hold anything (NaN * 0
      // would poison the sum), become 0
      asm volatile("" ::: "memory");
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (kt * TILE + acc_row(v, half) >= n_keys) sacc[v] = -INFINITY;
#pragma unroll
      for (int s2 = 0; s2 < PvStep<E>::STEPS; ++s2)
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
          for (int i = 0; i < G; ++i)
            if (kt * TILE + PvStep<E>::key_of(s2, half, i) >= n_keys) cur.v[s2][t][i] = (E)0.f;
    }
    float mx = sacc[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sacc[v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));      // the other half-wave holds the column's other 16 keys
    const float mt = mx * c2;                       // finite: a key tile always holds at least one valid key
    const bool moves = mt > m_run + REF_SLACK;      // (m_run = -inf before the wave's first tile)
    if (__builtin_amdgcn_ballot_w64(moves)) {
      const float m_new = moves ? mt : m_run;
      const float alpha = moves ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;
      l_run *= alpha;
      m_run = m_new;
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[t][v] *= alpha;
    }
    float p[16];
    float psum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      p[v] = __builtin_amdgcn_exp2f(fmaf(sacc[v], c2, -m_run));
      psum += p[v];
    }
    l_run += psum;
    // ---- O^T += V^T . P^T
#pragma unroll
    for (int s2 = 0; s2 < PvStep<E>::STEPS; ++s2) {
      vec pv[NP];
#pragma unroll
      for (int pl = 0; pl < NP; ++pl) pv[pl] = PvStep<E>::p_vec(p, s2, pl);
#pragma unroll
      for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) mfma32(o[t], cur.v[s2][t], pv[pl]);
    }
  };
  // Two tile buffers that swap roles (the loop is unrolled by two, so no registers are copied): the next tile's
  // loads are issued before this tile is used, clamped, so that no branch surrounds loads and the compiler can
  // count them; a wave's last turn re-reads its own tile.
  TileRegs ta, tb;
  if (kt0 < n_ktiles) load_tile(kt0, ta);
  for (int kt = kt0; kt < n_ktiles; kt += 2 * stride) {
    load_tile(min(kt + stride, n_ktiles - 1), tb);
    use_tile(ta, kt);
    if (kt + stride >= n_ktiles) break;
    load_tile(min(kt + 2 * stride, n_ktiles - 1), ta);
    use_tile(tb, kt + stride);
  }
  TRACE_MARK(7, 2);
  // ---- fold the waves through LDS (lane-major, conflict free): every wave leaves its state, then wave w
  // finishes RPW of the DT*16 accumulator registers, summed over the waves in wave order
  extern __shared__ float lds[];                       // [ATTN_WAVES][DT*16 + 2][64 lanes]
  constexpr int PW = (DT * 16 + 2) * WAVE, RPW = DT * 16 / ATTN_WAVES;
  static_assert(RPW % 4 == 0, "a wave finishes whole groups of four accumulator registers");
  {
    float* pb = lds + wave * PW + lane;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) pb[(t * 16 + v) * WAVE] = o[t][v];
    pb[(DT * 16) * WAVE] = m_run;
    pb[(DT * 16 + 1) * WAVE] = l_run + __shfl_xor(l_run, 32, WAVE);
  }
  __syncthreads();
  TRACE_MARK(7, 3);
  float M = -INFINITY;
#pragma unroll
  for (int w = 0; w < ATTN_WAVES; ++w) M = fmaxf(M, lds[w * PW + (DT * 16) * WAVE + lane]);
  float L = 0.f;
  float r[RPW];
#pragma unroll
  for (int i = 0; i < RPW; ++i) r[i] = 0.f;
#pragma unroll
  for (int w = 0; w < ATTN_WAVES; ++w) {
    const float* pb = lds + w * PW + lane;
    const float mw = pb[(DT * 16) * WAVE];
    const float sw = mw > -INFINITY ? __builtin_amdgcn_exp2f(mw - M) : 0.f;   // a wave that saw no key tile contributes nothing
    L += sw * pb[(DT * 16 + 1) * WAVE];
#pragma unroll
    for (int i = 0; i < RPW; ++i) r[i] += sw * pb[(wave * RPW + i) * WAVE];
  }
  if (my_splits == 1) {
    // the whole key range was here: normalise and write the attention output
    if (col < nvalid) {
      const float inv = 1.f / L;
#pragma unroll
      for (int i4 = 0; i4 < RPW / 4; ++i4) {   // four accumulator registers = four consecutive features
        const int g = wave * RPW + 4 * i4;
        const f32x4 o = {r[4 * i4] * inv, r[4 * i4 + 1] * inv, r[4 * i4 + 2] * inv, r[4 * i4 + 3] * inv};
        store_actk4<E>(out, T_out, tok0 + col, head * HD + (g / 16) * TILE + acc_row(g % 16, half), o);
      }
    }
    TRACE_MARK(7, 4);
    return;
  }
  // partial of this split: O [32 q][HD] (unnormalised), m [32], l [32], handed over with device-coherent stores
  const int pair = qt * geom.n_heads + head;
  const buf_rsrc pr = coherent_buffer(part);
  const uint32_t pair_bytes = (uint32_t)pair * n_splits * TILE * (HD + 2) * 4, part_bytes = TILE * (HD + 2) * 4;
  {
    const uint32_t pb = pair_bytes + split * part_bytes;
#pragma unroll
    for (int i4 = 0; i4 < RPW / 4; ++i4) {
      const int g = wave * RPW + 4 * i4;
      const float v4[4] = {r[4 * i4], r[4 * i4 + 1], r[4 * i4 + 2], r[4 * i4 + 3]};
      coherent_store_n<4>(pr, pb + (col * HD + (g / 16) * TILE + acc_row(g % 16, half)) * 4, v4);
    }
    if (wave == 0 && half == 0) {
      const float mv[1] = {M}, lv[1] = {L};
      coherent_store_n<1>(pr, pb + (TILE * HD + col) * 4, mv);
      coherent_store_n<1>(pr, pb + (TILE * HD + TILE + col) * 4, lv);
    }
  }
  __shared__ int32_t s_flag;
  if (!last_arrival(tickets + pair, my_splits, &s_flag)) return;
  // Last to arrive: fold the partials in split order.  A thread takes a (query, 4 consecutive features) item.
  for (int item = threadIdx.x; item < TILE * HD / 4; item += ATTN_WAVES * WAVE) {
    const int q = item / (HD / 4), d = (item % (HD / 4)) * 4;
    if (q >= nvalid) continue;
    float mp[ATTN_MAX_SPLITS], lp[ATTN_MAX_SPLITS], op[ATTN_MAX_SPLITS][4];
#pragma unroll
    for (int p = 0; p < ATTN_MAX_SPLITS; ++p) {   // all loads first (clamped: the unused ones repeat the last part)
      const uint32_t pb = pair_bytes + min(p, my_splits - 1) * part_bytes;
      float t1[1], t2[1];
      coherent_load_n<1>(pr, pb + (TILE * HD + q) * 4, t1);
      coherent_load_n<1>(pr, pb + (TILE * HD + TILE + q) * 4, t2);
      coherent_load_n<4>(pr, pb + (q * HD + d) * 4, op[p]);
      mp[p] = t1[0];
      lp[p] = t2[0];
    }
    float Mx = -INFINITY;
#pragma unroll
    for (int p = 0; p < ATTN_MAX_SPLITS; ++p) Mx = p < my_splits ? fmaxf(Mx, mp[p]) : Mx;
    float Ls = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < ATTN_MAX_SPLITS; ++p) {
      if (p < my_splits && mp[p] > -INFINITY) {   // (a split whose waves saw no key tile contributes nothing)
        const float w = __builtin_amdgcn_exp2f(mp[p] - Mx);
        Ls += w * lp[p];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] += w * op[p][i];
      }
    }
    const float inv = 1.f / Ls;
    f32x4 res;
#pragma unroll
    for (int i = 0; i < 4; ++i) res[i] = acc[i] * inv;
    store_actk4<E>(out, T_out, tok0 + q, head * HD + d, res);
  }
}

template <int HD> constexpr size_t attn_lds() { return (size_t)ATTN_WAVES * ((HD / TILE) * 16 + 2) * WAVE * 4; }

template <typename E, int HD> static void launch_attention_t(const AttnArgs& a, hipStream_t st) {
  // With few workgroups of its own the launch gets layers of the grid behind the query tiles that fetch a.pf (a
  // workgroup fills a compute unit, so with many of its own the fetching ones would only queue up behind them).
  const int per_layer = a.n_splits * a.geom.n_heads, real = per_layer * a.n_qtiles;
  const bool fetch = a.pf.base != nullptr && real <= ATTN_FETCH_MAX_OWN;
  const int last = fetch ? l2_prefetch_first(real) + a.pf.n_regions : real;   // one past the last index in use
  attention_kernel<E, HD><<<dim3(a.n_splits, a.geom.n_heads, (last + per_layer - 1) / per_layer), ATTN_WAVES * WAVE,
                            attn_lds<HD>(), st>>>(
      (const E*)a.q, a.q_plane, (const E*)a.kv_layer, a.geom, a.meta, a.page_table, a.pt_stride, a.n_splits, a.part,
      a.tickets, (E*)a.out, a.T, a.n_qtiles, fetch ? a.pf : L2Prefetch{nullptr, 0, 0}, live_word());
}

bool configure_attention() {
  const void* fns[4] = {(const void*)attention_kernel<bf16_t, 128>, (const void*)attention_kernel<float, 128>,
                        (const void*)attention_kernel<bf16_t, 64>, (const void*)attention_kernel<float, 64>};
  bool ok = true;
  for (const void* fn : fns)
    ok = ok && hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_lds<128>()) == hipSuccess;
  (void)hipGetLastError();
  return ok;
}

void launch_attention(bool bf16, const AttnArgs& a, hipStream_t st) {
  const int hd = a.geom.head_dim;
  if (bf16) {
    if (hd == 128) launch_attention_t<bf16_t, 128>(a, st);
    else launch_attention_t<bf16_t, 64>(a, st);
  } else {
    if (hd == 128) launch_attention_t<float, 128>(a, st);
    else launch_attention_t<float, 64>(a, st);
  }
}

TRACE_READER(trace_read_attention)

}  // namespace dinfer
