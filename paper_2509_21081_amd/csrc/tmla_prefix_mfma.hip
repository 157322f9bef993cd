// Naive shared-prefix flash-decode on the matrix cores (paper Algorithm 1 step 4).
//
// Per head, all B*S_q queries attend the same expanded K/V, so queries are batched on the MFMA
// column axis and every K/V tile is fetched once per workgroup.  The expanded cache is stored in
// MFMA operand order (see typhoon_mla.h), so a 32-token block is 12 K fragments + 8 V fragments of
// 1 KiB each that are copied verbatim.  A wavefront owns 64 queries (two 32-column blocks): the
// Q^T fragments stay in registers, S^T = K Q^T gives every lane 16 scores of one query, the
// probabilities become the B operand of O^T = V^T P^T without any cross-lane traffic.
//
// Two workgroup shapes (4 wavefronts each):
//   * query-split : the wavefronts own 4 x 64 different queries and share each K/V block through
//     LDS (register-staged double buffer).  Used when a head has more than 128 queries; this is
//     the MFMA-bound regime (intensity = number of queries per fetched byte).
//   * token-split : all wavefronts own the same <= 64 queries and stream disjoint token blocks
//     straight from global memory into registers (no LDS, no barriers in the loop); their partial
//     softmaxes are merged through LDS at the end.  Used for small batches, the HBM-bound regime.
// Split-K over the prefix comes on top (grid.z); each workgroup writes a normalised partial
// output and its natural-log LSE for the combine step.
#include "tmla_common.hpp"
#include "tmla_lds_asm.hpp"
#include "tmla_mfma.hpp"

namespace tmla {

struct PrefixArgs {
  const __bf16* q;    // [M, H, 192]
  const __bf16* pk;   // expanded K, operand order
  const __bf16* pv;   // expanded V, operand order
  float* o;           // [np_split, rows, 128]
  float* lse;         // [np_split, rows]
  int M, H, Ls, ntb, blocks_per_split;
  int64_t rows;
  float c;            // sm_scale * log2(e)
};

__device__ inline void load_q_frags(const PrefixArgs& a, int h, int q0, int n, int g,
                                    bf16x8 (&qf)[2][12]) {
#pragma unroll
  for (int nb = 0; nb < 2; nb++) {
    const int qi = q0 + nb * 32 + n;
    const __bf16* p = a.q + ((size_t)qi * a.H + h) * D_QK + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 12; ks++) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[nb][ks] = (qi < a.M) ? *(const bf16x8*)(p + 16 * ks) : z;
    }
  }
}

// ------------------------------------------------------------------ query-split workgroup
// Eight wavefronts (two per SIMD, so one wavefront's softmax overlaps the other's MFMAs), each
// owning 32 queries of the head; K/V blocks stream global -> LDS through a ring of QS_NSLOT
// blocks shared by all of them.  Per wavefront the work on block i is
//     scores (MFMA)  ->  softmax (VALU) side by side with P V of block i-1 (MFMA).
constexpr int QS_BLOCK_BYTES = (K_BLK_ELEMS + V_BLK_ELEMS) * 2;  // 20480 = 20 x 1 KiB
constexpr int QS_NSLOT = 7;
constexpr int QS_LDS_BYTES = QS_NSLOT * QS_BLOCK_BYTES;           // 143360
constexpr int QS_AHEAD = QS_NSLOT - 2;   // blocks in flight beyond the two being worked on
constexpr int QS_WAVES = 8;
constexpr int QS_QUERIES = QS_WAVES * 32;

// scores of one 32-token block for this wavefront's 32 queries: K_block(32 x 192) Q^T, with the
// K fragments read from the LDS block whose lane address is `ka`
__device__ inline f32x16 qs_scores(uint32_t ka, const bf16x8 (&qf)[12]) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 sacc;
  bf16x8 f[2][4];
  static_for<4>([&](auto j) { f[0][j] = lds_read_b128<1024 * decltype(j)::value>(ka); });
  static_for<3>([&](auto grp) {
    constexpr int G = decltype(grp)::value;
    constexpr int cur = G & 1, nxt = cur ^ 1;
    if constexpr (G + 1 < 3) {
      static_for<4>([&](auto j) {
        f[nxt][j] = lds_read_b128<1024 * (4 * (G + 1) + decltype(j)::value)>(ka);
      });
      lgkm_wait<4>(f[cur][0], f[cur][1], f[cur][2], f[cur][3]);
    } else {
      lgkm_wait<0>(f[cur][0], f[cur][1], f[cur][2], f[cur][3]);
    }
    static_for<4>([&](auto j) {
      constexpr int ks = 4 * G + decltype(j)::value;
      if constexpr (ks == 0) sacc = mfma32(f[cur][j], qf[ks], zero);
      else sacc = mfma32(f[cur][j], qf[ks], sacc);
    });
  });
  return sacc;
}

// o += V_block^T P^T, V fragments from the LDS block whose lane address is `ka`
__device__ inline void qs_pv(uint32_t ka, const bf16x8 (&p)[2], f32x16 (&o)[4]) {
  bf16x8 vf[8];
  static_for<8>([&](auto j) {
    vf[j] = lds_read_b128<K_BLK_ELEMS * 2 + 1024 * decltype(j)::value>(ka);
  });
  lgkm_wait<4>(vf[0], vf[1], vf[2], vf[3]);
#pragma unroll
  for (int db = 0; db < 4; db++) o[db] = mfma32(vf[db], p[0], o[db]);
  lgkm_wait<0>(vf[4], vf[5], vf[6], vf[7]);
#pragma unroll
  for (int db = 0; db < 4; db++) o[db] = mfma32(vf[4 + db], p[1], o[db]);
}

template <int PER_BLOCK>
__device__ inline void qs_wait_pending(int pending) {
  if (pending >= 4) vm_wait<4 * PER_BLOCK>();
  else if (pending == 3) vm_wait<3 * PER_BLOCK>();
  else if (pending == 2) vm_wait<2 * PER_BLOCK>();
  else if (pending == 1) vm_wait<PER_BLOCK>();
  else vm_wait<0>();
}

__global__ void __launch_bounds__(QS_WAVES * 64, 1) prefix_attn_query_split_kernel(PrefixArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int h = blockIdx.x, mb = blockIdx.y, sp = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qi = mb * QS_QUERIES + wave * 32 + n;   // this lane's query

  const int tb0 = sp * a.blocks_per_split;
  const int tb1 = min(a.ntb, tb0 + a.blocks_per_split);
  const int nblk = tb1 - tb0;
  // the very last block of the prefix may be partial; it is handled after the pipelined loop
  const bool has_tail = (tb1 == a.ntb) && (a.Ls % TOK_BLK != 0) && nblk > 0;
  const int nfull = has_tail ? nblk - 1 : nblk;
  const uint32_t smem_addr = lds_addr(smem) + lane * 16;

  // transfers per block: wavefronts 0-3 move K fragments w, w+4, w+8; wavefronts 4-7 move V
  // fragments w-4 and w
  const bool k_mover = wave < 4;
  const char* src = k_mover
      ? (const char*)(a.pk + ((size_t)h * a.ntb + tb0) * K_BLK_ELEMS) + wave * 1024 + lane * 16
      : (const char*)(a.pv + ((size_t)h * a.ntb + tb0) * V_BLK_ELEMS) + (wave - 4) * 1024 + lane * 16;
  auto issue = [&](int i) {
    char* slot = smem + (i % QS_NSLOT) * QS_BLOCK_BYTES;
    if (k_mover) {
      const char* s0 = src + (size_t)i * (K_BLK_ELEMS * 2);
      char* dst = slot + wave * 1024;
      dma16(s0, dst);
      dma16(s0 + 4096, dst + 4096);
      dma16(s0 + 8192, dst + 8192);
    } else {
      const char* s0 = src + (size_t)i * (V_BLK_ELEMS * 2);
      char* dst = slot + K_BLK_ELEMS * 2 + (wave - 4) * 1024;
      dma16(s0, dst);
      dma16(s0 + 4096, dst + 4096);
    }
  };
#pragma unroll
  for (int i = 0; i < QS_AHEAD; i++)
    if (i < nblk) issue(i);

  bf16x8 qf[12];
  {
    const __bf16* p = a.q + ((size_t)qi * a.H + h) * D_QK + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 12; ks++) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[ks] = (qi < a.M) ? *(const bf16x8*)(p + 16 * ks) : z;
    }
  }
#pragma unroll
  for (int ks = 0; ks < 12; ks += 4)
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(qf[ks]), "+v"(qf[ks + 1]), "+v"(qf[ks + 2]), "+v"(qf[ks + 3])::"memory");

  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int v = 0; v < 16; v++) o[db][v] = 0.f;
  float m = -INFINITY, l = 0.f;

  // Block i may be read once (a) this wavefront's transfers of it are done and (b) the barrier
  // has been passed by everyone after their own wait.  Called exactly once per block, in order;
  // after it, everybody has also finished reading block i-2, whose slot is refilled.
  auto sync_and_refill = [&](int i) {
    const int newest = min(nblk - 1, i + QS_AHEAD - 1);   // newest block issued so far
    if (k_mover) qs_wait_pending<3>(newest - i);
    else qs_wait_pending<2>(newest - i);
    raw_barrier();
    if (i + QS_AHEAD < nblk) issue(i + QS_AHEAD);
  };
  auto blk_addr = [&](int i) { return smem_addr + (i % QS_NSLOT) * QS_BLOCK_BYTES; };
  auto rescale_o = [&](float alpha, bool resc) {
    if (resc) {
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int v = 0; v < 16; v++) o[db][v] *= alpha;
    }
  };

  // One pipeline phase for full block i: its scores (matrix core), then its softmax (vector
  // ALU) side by side with P V of block i-1 (matrix core), which uses the previous phase's P.
  // The two wavefronts that share a SIMD (w and w+4) run the same work in a different order so
  // that one is on the matrix core while the other is on the vector ALU:
  //   wavefronts 0-3, period i:  scores(i)     -> softmax(i)   -> P V(i-1)
  //   wavefronts 4-7, period i:  softmax(i-1)  -> scores(i)    -> P V(i-1)
  // Both read K of block i and V of block i-1 in period i, so the ring bookkeeping is the same,
  // and both call sync_and_refill exactly once per block.
  const int tail_limit = a.Ls - (tb0 + nblk - 1) * TOK_BLK;   // valid tokens of a partial tail
  bf16x8 p_a[2], p_b[2];
  bool resc;
  if (wave < 4) {
    auto phase = [&](int i, bf16x8 (&p_out)[2], const bf16x8 (&p_in)[2]) {
      sync_and_refill(i);
      f32x16 s = qs_scores(blk_addr(i), qf);
      const float alpha = softmax_block<false>(s, m, l, a.c, 32, g, p_out[0], p_out[1], resc);
      if (i > 0) qs_pv(blk_addr(i - 1), p_in, o);
      rescale_o(alpha, resc);
    };
    for (int i = 0; i < nfull; i += 2) {
      phase(i, p_a, p_b);
      if (i + 1 < nfull) phase(i + 1, p_b, p_a);
    }
    if (has_tail) sync_and_refill(nblk - 1);
    if (nfull > 0) {
      if (nfull & 1) qs_pv(blk_addr(nfull - 1), p_a, o);
      else qs_pv(blk_addr(nfull - 1), p_b, o);
    }
  } else {
    f32x16 s_hold;
    if (nfull > 0) {
      sync_and_refill(0);
      s_hold = qs_scores(blk_addr(0), qf);
    }
    for (int i = 1; i < nfull; i++) {
      sync_and_refill(i);
      const float alpha = softmax_block<false>(s_hold, m, l, a.c, 32, g, p_a[0], p_a[1], resc);
      rescale_o(alpha, resc);
      s_hold = qs_scores(blk_addr(i), qf);
      qs_pv(blk_addr(i - 1), p_a, o);
    }
    if (has_tail) sync_and_refill(nblk - 1);
    if (nfull > 0) {
      const float alpha = softmax_block<false>(s_hold, m, l, a.c, 32, g, p_a[0], p_a[1], resc);
      rescale_o(alpha, resc);
      qs_pv(blk_addr(nfull - 1), p_a, o);
    }
  }
  if (has_tail) {   // partial last block of the prefix: plain masked pass
    const int i = nblk - 1;
    f32x16 s = qs_scores(blk_addr(i), qf);
    const float alpha = softmax_block<true>(s, m, l, a.c, tail_limit, g, p_a[0], p_a[1], resc);
    rescale_o(alpha, resc);
    qs_pv(blk_addr(i), p_a, o);
  }

  const float lt = sum_halves(l);
  if (qi >= a.M) return;
  const size_t row = (size_t)sp * a.rows + (size_t)qi * a.H + h;
  if (lt > 0.f) {
    const float inv = 1.f / lt;
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int v4 = 0; v4 < 4; v4++) {
        float4 w = make_float4(o[db][4 * v4] * inv, o[db][4 * v4 + 1] * inv,
                               o[db][4 * v4 + 2] * inv, o[db][4 * v4 + 3] * inv);
        *(float4*)(a.o + row * D_V + 32 * db + 8 * v4 + 4 * g) = w;
      }
    if (g == 0) a.lse[row] = (m + fast_log2(lt)) * LN2;
  } else if (g == 0) {
    a.lse[row] = -INFINITY;
  }
}

// ------------------------------------------------------------------ token-split workgroup
constexpr int TS_ROW_FLOATS = 132;  // 128 + 4 padding: conflict-free 16-byte LDS accesses
constexpr int TS_MERGE_BYTES = 4 * 64 * TS_ROW_FLOATS * 4 + 2 * 4 * 64 * 4;  // O regions + m, l
constexpr int TS_BLOCK_BYTES = (K_BLK_ELEMS + V_BLK_ELEMS) * 2;  // 20480 = 20 x 1 KiB
constexpr int TS_RING_BYTES = 4 * 2 * TS_BLOCK_BYTES;             // two blocks per wavefront
constexpr int TS_LDS_BYTES = TS_RING_BYTES > TS_MERGE_BYTES ? TS_RING_BYTES : TS_MERGE_BYTES;

// One 32-token block against this wavefront's 64 queries, operands read from an LDS copy of the
// block (K fragments at [0, 12 KiB), V fragments behind them).
__device__ inline void ts_block(uint32_t blk, int lane, const bf16x8 (&qf)[2][12],
                                f32x16 (&o)[4][2], float (&m)[2], float (&l)[2], float c,
                                int limit, int g) {
  const uint32_t ka = blk + lane * 16;
  f32x16 sacc[2];
#pragma unroll
  for (int nb = 0; nb < 2; nb++)
#pragma unroll
    for (int v = 0; v < 16; v++) sacc[nb][v] = 0.f;
  {
    bf16x8 f[2][4];
    static_for<4>([&](auto j) { f[0][j] = lds_read_b128<1024 * decltype(j)::value>(ka); });
    static_for<3>([&](auto grp) {
      constexpr int G = decltype(grp)::value;
      constexpr int cur = G & 1, nxt = cur ^ 1;
      if constexpr (G + 1 < 3) {
        static_for<4>([&](auto j) {
          f[nxt][j] = lds_read_b128<1024 * (4 * (G + 1) + decltype(j)::value)>(ka);
        });
        lgkm_wait<4>(f[cur][0], f[cur][1], f[cur][2], f[cur][3]);
      } else {
        lgkm_wait<0>(f[cur][0], f[cur][1], f[cur][2], f[cur][3]);
      }
      static_for<4>([&](auto j) {
        constexpr int ks = 4 * G + decltype(j)::value;
        sacc[0] = mfma32(f[cur][j], qf[0][ks], sacc[0]);
        sacc[1] = mfma32(f[cur][j], qf[1][ks], sacc[1]);
      });
    });
  }
  // the V fragments are requested before the softmax so their latency hides under it
  bf16x8 vf[8];
  static_for<8>([&](auto j) {
    vf[j] = lds_read_b128<K_BLK_ELEMS * 2 + 1024 * decltype(j)::value>(ka);
  });
  bf16x8 p[2][2];
#pragma unroll
  for (int nb = 0; nb < 2; nb++) {
    bool rescale;
    const float alpha =
        softmax_block(sacc[nb], m[nb], l[nb], c, limit, g, p[nb][0], p[nb][1], rescale);
    if (rescale) {
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int v = 0; v < 16; v++) o[db][nb][v] *= alpha;
    }
  }
  lgkm_wait<0>(vf[0], vf[1], vf[2], vf[3]);
  lgkm_wait<0>(vf[4], vf[5], vf[6], vf[7]);
#pragma unroll
  for (int kk = 0; kk < 2; kk++)
#pragma unroll
    for (int db = 0; db < 4; db++) {
      o[db][0] = mfma32(vf[kk * 4 + db], p[0][kk], o[db][0]);
      o[db][1] = mfma32(vf[kk * 4 + db], p[1][kk], o[db][1]);
    }
}

__global__ void __launch_bounds__(256, 1) prefix_attn_token_split_kernel(PrefixArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int h = blockIdx.x, mb = blockIdx.y, sp = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int q0 = mb * 64;

  bf16x8 qf[2][12];
  load_q_frags(a, h, q0, n, g, qf);
  // resident before the streamed loads start: no wait on them inside the loop
#pragma unroll
  for (int nb = 0; nb < 2; nb++)
#pragma unroll
    for (int ks = 0; ks < 12; ks += 4)
      asm volatile("s_waitcnt vmcnt(0)"
                   : "+v"(qf[nb][ks]), "+v"(qf[nb][ks + 1]), "+v"(qf[nb][ks + 2]),
                     "+v"(qf[nb][ks + 3])::"memory");

  const int tb0 = sp * a.blocks_per_split;
  const int tb1 = min(a.ntb, tb0 + a.blocks_per_split);
  const __bf16* kbase = a.pk + ((size_t)h * a.ntb) * K_BLK_ELEMS + lane * 8;
  const __bf16* vbase = a.pv + ((size_t)h * a.ntb) * V_BLK_ELEMS + lane * 8;

  f32x16 o[4][2];
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int nb = 0; nb < 2; nb++)
#pragma unroll
      for (int v = 0; v < 16; v++) o[db][nb][v] = 0.f;
  float m[2] = {-INFINITY, -INFINITY}, l[2] = {0.f, 0.f};

  // wavefront w streams blocks tb0 + w, tb0 + w + 4, ... through its private two-slot LDS ring
  char* ring = smem + wave * (2 * TS_BLOCK_BYTES);
  const uint32_t ring_addr = lds_addr(ring);
  auto issue = [&](int tb, int slot) {
    char* dst = ring + slot * TS_BLOCK_BYTES;
    const __bf16* ks = kbase + (size_t)tb * K_BLK_ELEMS;
    const __bf16* vs = vbase + (size_t)tb * V_BLK_ELEMS;
#pragma unroll
    for (int f = 0; f < 12; f++) dma16(ks + f * 512, dst + f * 1024);
#pragma unroll
    for (int f = 0; f < 8; f++) dma16(vs + f * 512, dst + K_BLK_ELEMS * 2 + f * 1024);
  };
  const int first = tb0 + wave;
  const int nmine = first < tb1 ? (tb1 - first + 3) / 4 : 0;
  if (nmine > 0) issue(first, 0);
  if (nmine > 1) issue(first + 4, 1);
  for (int j = 0; j < nmine; j++) {
    if (j + 1 < nmine) vm_wait<20>();   // block j has landed, block j+1 may still be in flight
    else vm_wait<0>();
    const int tb = first + 4 * j;
    ts_block(ring_addr + (j & 1) * TS_BLOCK_BYTES, lane, qf, o, m, l, a.c,
             min(32, a.Ls - tb * TOK_BLK), g);
    if (j + 2 < nmine) issue(tb + 8, j & 1);
  }
  __syncthreads();   // the merge buffers below alias every wavefront's ring

  // merge the four wavefronts' partial softmaxes (same queries, disjoint tokens)
  float* sm_o = (float*)smem;                                   // [4][64][132]
  float* sm_m = (float*)(smem + 4 * 64 * TS_ROW_FLOATS * 4);    // [4][64]
  float* sm_l = sm_m + 4 * 64;                                  // [4][64]
  float lt[2];
#pragma unroll
  for (int nb = 0; nb < 2; nb++) {
    lt[nb] = sum_halves(l[nb]);
    if (g == 0) {
      sm_m[wave * 64 + nb * 32 + n] = m[nb];
      sm_l[wave * 64 + nb * 32 + n] = lt[nb];
    }
  }
  __syncthreads();
#pragma unroll
  for (int nb = 0; nb < 2; nb++) {
    const int qq = nb * 32 + n;
    float ms = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; w++) ms = fmaxf(ms, sm_m[w * 64 + qq]);
    float lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; w++) {
      const float mw = sm_m[w * 64 + qq];
      lsum += (mw == -INFINITY) ? 0.f : sm_l[w * 64 + qq] * fast_exp2(mw - ms);
    }
    const float f = (m[nb] == -INFINITY || !(lsum > 0.f)) ? 0.f : fast_exp2(m[nb] - ms) / lsum;
    float* dst = sm_o + ((size_t)wave * 64 + qq) * TS_ROW_FLOATS;
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int v4 = 0; v4 < 4; v4++) {
        float4 w4 = make_float4(o[db][nb][4 * v4] * f, o[db][nb][4 * v4 + 1] * f,
                                o[db][nb][4 * v4 + 2] * f, o[db][nb][4 * v4 + 3] * f);
        *(float4*)(dst + 32 * db + 8 * v4 + 4 * g) = w4;
      }
  }
  __syncthreads();
  for (int idx = tid; idx < 64 * 32; idx += 256) {
    const int qq = idx >> 5, c4 = idx & 31;
    const int qi = q0 + qq;
    if (qi >= a.M) continue;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int w = 0; w < 4; w++) {
      const float4 x = *(const float4*)(sm_o + ((size_t)w * 64 + qq) * TS_ROW_FLOATS + c4 * 4);
      acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    const size_t row = (size_t)sp * a.rows + (size_t)qi * a.H + h;
    *(float4*)(a.o + row * D_V + c4 * 4) = acc;
  }
  if (tid < 64 && q0 + tid < a.M) {
    float ms = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; w++) ms = fmaxf(ms, sm_m[w * 64 + tid]);
    float lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; w++) {
      const float mw = sm_m[w * 64 + tid];
      lsum += (mw == -INFINITY) ? 0.f : sm_l[w * 64 + tid] * fast_exp2(mw - ms);
    }
    const size_t row = (size_t)sp * a.rows + (size_t)(q0 + tid) * a.H + h;
    a.lse[row] = (lsum > 0.f) ? (ms + fast_log2(lsum)) * LN2 : -INFINITY;
  }
}

int mfma_prefix_attention(const Plan& p, const DecodeArgs& d) {
  if (p.np_split <= 0) return TMLA_OK;
  PrefixArgs a;
  a.q = (const __bf16*)d.q;
  a.pk = (const __bf16*)d.prefix_k;
  a.pv = (const __bf16*)d.prefix_v;
  a.o = (float*)(d.ws + p.off_naive_o);
  a.lse = (float*)(d.ws + p.off_naive_lse);
  a.M = p.B * p.Sq; a.H = p.H; a.Ls = p.Ls;
  a.ntb = (p.Ls + TOK_BLK - 1) / TOK_BLK;
  a.blocks_per_split = p.p_chunk / TOK_BLK;
  a.rows = p.rows;
  a.c = d.sm_scale * LOG2E;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)prefix_attn_query_split_kernel,
                            hipFuncAttributeMaxDynamicSharedMemorySize, QS_LDS_BYTES) != hipSuccess ||
        hipFuncSetAttribute((const void*)prefix_attn_token_split_kernel,
                            hipFuncAttributeMaxDynamicSharedMemorySize, TS_LDS_BYTES) != hipSuccess)
      return TMLA_ERR_HIP;
    attr_set = true;
  }
  if (a.M > 128) {
    dim3 grid(p.H, (a.M + QS_QUERIES - 1) / QS_QUERIES, p.np_split);
    hipLaunchKernelGGL(prefix_attn_query_split_kernel, grid, dim3(QS_WAVES * 64), QS_LDS_BYTES,
                       d.stream, a);
  } else {
    dim3 grid(p.H, (a.M + 63) / 64, p.np_split);
    hipLaunchKernelGGL(prefix_attn_token_split_kernel, grid, dim3(256), TS_LDS_BYTES, d.stream, a);
  }
  return TMLA_OK;
}

}  // namespace tmla
