// Naive shared-prefix flash-decode on the matrix cores (paper Algorithm 1 step 4).
//
// Per head, all B*S_q queries attend the same expanded K/V, so queries are batched on the MFMA
// column axis and every K/V tile is fetched once per workgroup.  The expanded cache is stored in
// MFMA operand order (see typhoon_mla.h), so a 32-token block is 12 K fragments + 8 V fragments of
// 1 KiB each that are copied verbatim.  A wavefront owns 64 queries (two 32-column blocks): the
// Q^T fragments stay in registers, S^T = K Q^T gives every lane 16 scores of one query, the
// probabilities become the B operand of O^T = V^T P^T without any cross-lane traffic.
//
// Three workgroup shapes; every K/V block goes global -> LDS with global_load_lds transfers
// (no staging registers):
//   * pipelined   : four wavefronts own 4 x 64 different queries of a head and share each block
//     through LDS rings (K and V separately, all 160 KiB); one hand-laid instruction stream per
//     wavefront overlaps the scores of block t+1, the softmax of block t and P V of block t-1.
//     Used when a head has more than 128 queries: the MFMA-bound regime (intensity = number of
//     queries per fetched byte).
//   * query-split : the same split of the queries over eight wavefronts (two per SIMD) with
//     moving exponent references, scheduled by the compiler; kept as the debug alternative.
//   * token-split : all four wavefronts own the same <= 64 queries and stream disjoint token
//     blocks, each through a private two-slot LDS ring (no barriers in the loop); their partial
//     softmaxes are merged through LDS at the end.  Used for small batches, the HBM-bound regime,
//     and (PAGED) for the expanded paged suffix of naive_only mode.
// Split-K over the prefix comes on top (grid.z); each workgroup writes a normalised partial
// output and its natural-log LSE for the combine step.
#include <type_traits>

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
  // paged per-request suffix (naive_only, Table 1 row "naive"): grid.y = request
  const int32_t* block_table;
  const int32_t* lens;
  int max_blocks, page_shift;   // 32-token blocks per cache page = 1 << page_shift
  int Sq, first_slot;           // partial slot of chunk 0
};

__device__ inline void load_q_frags(const PrefixArgs& a, int h, int q0, int n, int g,
                                    bf16x8 (&qf)[2][12], int q_end = 0x7fffffff) {
#pragma unroll
  for (int nb = 0; nb < 2; nb++) {
    const int qi = q0 + nb * 32 + n;
    const __bf16* p = a.q + ((size_t)qi * a.H + h) * D_QK + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 12; ks++) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[nb][ks] = (qi < a.M && qi < q_end) ? *(const bf16x8*)(p + 16 * ks) : z;
    }
  }
}

// ------------------------------------------------------------------ query-split workgroup
// 256 queries of a head per workgroup; K/V blocks stream global -> LDS through a ring of QS_NSLOT
// blocks shared by all wavefronts.  Per wavefront the work on block i is
//     scores (MFMA)  ->  softmax (VALU) side by side with P V of block i-1 (MFMA).
// Template NB = 32-query column blocks per wavefront:
//   NB = 1: eight wavefronts (two per SIMD) x 32 queries, every LDS fragment feeds one MFMA;
//   NB = 2: four wavefronts x 64 queries, every LDS fragment feeds two MFMAs (half the LDS
//           traffic per flop, but the whole register file of a SIMD for one wavefront).
constexpr int QS_BLOCK_BYTES = (K_BLK_ELEMS + V_BLK_ELEMS) * 2;  // 20480 = 20 x 1 KiB
constexpr int QS_NSLOT = 7;
constexpr int QS_LDS_BYTES = QS_NSLOT * QS_BLOCK_BYTES;           // 143360
constexpr int QS_AHEAD = 4;   // blocks issued ahead of the pair being synchronised
constexpr int QS_QUERIES = 256;

// scores of one 32-token block for this wavefront's queries: K_block(32 x 192) Q^T, with the
// K fragments read from the LDS block whose lane address is `ka`
template <int NB>
__device__ inline void qs_scores(uint32_t ka, const bf16x8 (&qf)[NB][12], f32x16 (&sacc)[NB]) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
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
#pragma unroll
      for (int nb = 0; nb < NB; nb++) {
        if constexpr (ks == 0) sacc[nb] = mfma32(f[cur][j], qf[nb][ks], zero);
        else sacc[nb] = mfma32(f[cur][j], qf[nb][ks], sacc[nb]);
      }
    });
  });
}

// o += V_block^T P^T, V fragments from the LDS block whose lane address is `ka`
template <int NB>
__device__ inline void qs_pv(uint32_t ka, const bf16x8 (&p)[NB][2], f32x16 (&o)[4][NB]) {
  bf16x8 vf[8];
  static_for<8>([&](auto j) {
    vf[j] = lds_read_b128<K_BLK_ELEMS * 2 + 1024 * decltype(j)::value>(ka);
  });
  lgkm_wait<4>(vf[0], vf[1], vf[2], vf[3]);
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int nb = 0; nb < NB; nb++) o[db][nb] = mfma32(vf[db], p[nb][0], o[db][nb]);
  lgkm_wait<0>(vf[4], vf[5], vf[6], vf[7]);
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int nb = 0; nb < NB; nb++) o[db][nb] = mfma32(vf[4 + db], p[nb][1], o[db][nb]);
}

template <int PER_BLOCK>
__device__ inline void qs_wait_pending(int pending) {
  if (pending >= 4) vm_wait<4 * PER_BLOCK>();
  else if (pending == 3) vm_wait<3 * PER_BLOCK>();
  else if (pending == 2) vm_wait<2 * PER_BLOCK>();
  else if (pending == 1) vm_wait<PER_BLOCK>();
  else vm_wait<0>();
}

template <int NB>
__global__ void __launch_bounds__(512 / NB, 1) prefix_attn_query_split_kernel(PrefixArgs a) {
  constexpr int NWAVE = 8 / NB;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int h = blockIdx.x, mb = blockIdx.y, sp = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q0 = mb * QS_QUERIES + wave * (32 * NB);   // first query of this wavefront

  const int tb0 = sp * a.blocks_per_split;
  const int tb1 = min(a.ntb, tb0 + a.blocks_per_split);
  const int nblk = tb1 - tb0;
  // the very last block of the prefix may be partial; it is handled after the pipelined loop
  const bool has_tail = (tb1 == a.ntb) && (a.Ls % TOK_BLK != 0) && nblk > 0;
  const int nfull = has_tail ? nblk - 1 : nblk;
  const uint32_t smem_addr = lds_addr(smem) + lane * 16;

  // 20 transfers of 1 KiB per block (fragments 0-11 = K, 12-19 = V), spread over the wavefronts:
  //   8 wavefronts: 0-3 move K fragments w, w+4, w+8; 4-7 move V fragments w-4, w
  //   4 wavefronts: each moves K fragments w, w+4, w+8 and V fragments w, w+4
  const bool k_mover = NWAVE == 4 || wave < 4;
  const bool v_mover = NWAVE == 4 || wave >= 4;
  const int wq = wave & 3;
  const char* ksrc = (const char*)(a.pk + ((size_t)h * a.ntb + tb0) * K_BLK_ELEMS) + wq * 1024 + lane * 16;
  const char* vsrc = (const char*)(a.pv + ((size_t)h * a.ntb + tb0) * V_BLK_ELEMS) + wq * 1024 + lane * 16;
  auto issue = [&](int i) __attribute__((always_inline)) {
    char* slot = smem + (i % QS_NSLOT) * QS_BLOCK_BYTES;
    if (k_mover) {
      const char* s0 = ksrc + (size_t)i * (K_BLK_ELEMS * 2);
      char* dst = slot + wq * 1024;
      dma16_stream(s0, dst);
      dma16_stream(s0 + 4096, dst + 4096);
      dma16_stream(s0 + 8192, dst + 8192);
    }
    if (v_mover) {
      const char* s0 = vsrc + (size_t)i * (V_BLK_ELEMS * 2);
      char* dst = slot + K_BLK_ELEMS * 2 + wq * 1024;
      dma16_stream(s0, dst);
      dma16_stream(s0 + 4096, dst + 4096);
    }
  };
#pragma unroll
  for (int i = 0; i < QS_AHEAD; i++)
    if (i < nblk) issue(i);

  bf16x8 qf[NB][12];
#pragma unroll
  for (int nb = 0; nb < NB; nb++) {
    const int qi = q0 + nb * 32 + n;
    const __bf16* p = a.q + ((size_t)qi * a.H + h) * D_QK + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 12; ks++) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[nb][ks] = (qi < a.M) ? *(const bf16x8*)(p + 16 * ks) : z;
    }
  }
#pragma unroll
  for (int nb = 0; nb < NB; nb++)
#pragma unroll
    for (int ks = 0; ks < 12; ks += 4)
      if constexpr (NB == 2)   // one wavefront per SIMD: park the fragments in accumulator registers
        asm volatile("s_waitcnt vmcnt(0)"
                     : "+a"(qf[nb][ks]), "+a"(qf[nb][ks + 1]), "+a"(qf[nb][ks + 2]),
                       "+a"(qf[nb][ks + 3])::"memory");
      else
        asm volatile("s_waitcnt vmcnt(0)"
                     : "+v"(qf[nb][ks]), "+v"(qf[nb][ks + 1]), "+v"(qf[nb][ks + 2]),
                       "+v"(qf[nb][ks + 3])::"memory");

  f32x16 o[4][NB];
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
      for (int v = 0; v < 16; v++) o[db][nb][v] = 0.f;
  float m[NB], l[NB];
#pragma unroll
  for (int nb = 0; nb < NB; nb++) { m[nb] = -INFINITY; l[nb] = 0.f; }

  // Blocks are synchronised in pairs (i even): blocks i and i+1 may be read once (a) this
  // wavefront's transfers of them are done and (b) the barrier has been passed by everyone after
  // their own wait.  Called once per pair, in order; after it everybody has also finished the
  // previous pair's period, which was the last reader of blocks i-3 and i-2 (7 slots: three
  // blocks in use -- V of i-1, K/V of i and i+1 -- and four in flight), so i+4 and i+5 are issued.
  auto sync_pair = [&](int i) __attribute__((always_inline)) {
    const int newest = min(nblk - 1, i + QS_AHEAD - 1);   // newest block issued so far
    const int pending = newest - min(nblk - 1, i + 1);    // blocks issued after the pair
    if (NWAVE == 4) qs_wait_pending<5>(pending);
    else if (k_mover) qs_wait_pending<3>(pending);
    else qs_wait_pending<2>(pending);
    raw_barrier();
    if (i + QS_AHEAD < nblk) issue(i + QS_AHEAD);
    if (i + QS_AHEAD + 1 < nblk) issue(i + QS_AHEAD + 1);
  };
  auto blk_addr = [&](int i) { return smem_addr + (i % QS_NSLOT) * QS_BLOCK_BYTES; };
  // softmax of the scores `s` (all column blocks) into `p`, then rescale of the outputs
  float alpha[NB];
  bool resc[NB];
  auto softmax_all = [&](f32x16 (&s)[NB], bf16x8 (&p)[NB][2], auto mask_tag, int limit)
                         __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < NB; nb++) {
      if constexpr (decltype(mask_tag)::value)
        alpha[nb] = softmax_block<true>(s[nb], m[nb], l[nb], a.c, limit, g, p[nb][0], p[nb][1],
                                        resc[nb]);
      else
        alpha[nb] = softmax_block_fast(s[nb], m[nb], l[nb], a.c, g, p[nb][0], p[nb][1], resc[nb]);
    }
  };
  auto rescale_o = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
      if (resc[nb]) {
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
          for (int v = 0; v < 16; v++) o[db][nb][v] *= alpha[nb];
      }
  };

  // With two wavefronts per SIMD (NB = 1), the pair (w, w+4) runs the same work in a different
  // order so that one is on the matrix core while the other is on the vector ALU:
  //   first group, period i:   scores(i)     -> softmax(i)   -> P V(i-1)
  //   second group, period i:  softmax(i-1)  -> scores(i)    -> P V(i-1)
  // Both read K of block i and V of block i-1 in period i, so the ring bookkeeping is the same,
  // and both call sync_pair exactly once per pair of blocks.
  const int tail_limit = a.Ls - (tb0 + nblk - 1) * TOK_BLK;   // valid tokens of a partial tail
  bf16x8 p_a[NB][2], p_b[NB][2];
  if (NWAVE == 4 || wave < 4) {
    auto phase = [&](int i, bf16x8 (&p_out)[NB][2], const bf16x8 (&p_in)[NB][2])
                     __attribute__((always_inline)) {
      if ((i & 1) == 0) sync_pair(i);
      f32x16 s[NB];
      qs_scores<NB>(blk_addr(i), qf, s);
      softmax_all(s, p_out, std::false_type{}, 32);
      if (i > 0) qs_pv<NB>(blk_addr(i - 1), p_in, o);
      rescale_o();
    };
    for (int i = 0; i < nfull; i += 2) {
      phase(i, p_a, p_b);
      if (i + 1 < nfull) phase(i + 1, p_b, p_a);
    }
    if (has_tail && (nfull & 1) == 0) sync_pair(nfull);
    if (nfull > 0) {
      if (nfull & 1) qs_pv<NB>(blk_addr(nfull - 1), p_a, o);
      else qs_pv<NB>(blk_addr(nfull - 1), p_b, o);
    }
  } else {
    f32x16 s_hold[NB];
    if (nfull > 0) {
      sync_pair(0);
      qs_scores<NB>(blk_addr(0), qf, s_hold);
    }
    for (int i = 1; i < nfull; i++) {
      if ((i & 1) == 0) sync_pair(i);
      softmax_all(s_hold, p_a, std::false_type{}, 32);
      rescale_o();
      qs_scores<NB>(blk_addr(i), qf, s_hold);
      qs_pv<NB>(blk_addr(i - 1), p_a, o);
    }
    if (has_tail && (nfull & 1) == 0) sync_pair(nfull);
    if (nfull > 0) {
      softmax_all(s_hold, p_a, std::false_type{}, 32);
      rescale_o();
      qs_pv<NB>(blk_addr(nfull - 1), p_a, o);
    }
  }
  if (has_tail) {   // partial last block of the prefix: plain masked pass
    const int i = nblk - 1;
    f32x16 s[NB];
    qs_scores<NB>(blk_addr(i), qf, s);
    softmax_all(s, p_a, std::true_type{}, tail_limit);
    rescale_o();
    qs_pv<NB>(blk_addr(i), p_a, o);
  }

#pragma unroll
  for (int nb = 0; nb < NB; nb++) {
    const int qi = q0 + nb * 32 + n;
    const float lt = sum_halves(l[nb]);
    if (qi >= a.M) continue;
    const size_t row = (size_t)sp * a.rows + (size_t)qi * a.H + h;
    if (lt > 0.f) {
      const float inv = 1.f / lt;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int v4 = 0; v4 < 4; v4++) {
          float4 w = make_float4(o[db][nb][4 * v4] * inv, o[db][nb][4 * v4 + 1] * inv,
                                 o[db][nb][4 * v4 + 2] * inv, o[db][nb][4 * v4 + 3] * inv);
          *(float4*)(a.o + row * D_V + 32 * db + 8 * v4 + 4 * g) = w;
        }
      if (g == 0) a.lse[row] = (m[nb] + fast_log2(lt)) * LN2;
    } else if (g == 0) {
      a.lse[row] = -INFINITY;
    }
  }
}

// ------------------------------------------------------------------ pipelined workgroup
// 256 queries of a head per workgroup, four wavefronts (one per SIMD) of 64 queries each, so
// every K/V fragment read from LDS feeds two MFMAs.  The instruction stream of a wavefront is
// laid out by hand as one software pipeline: in period t it issues
//     matrix core : scores of block t+1 (24 MFMAs), then P V of block t-1 (16 MFMAs)
//     vector ALU  : softmax of block t, cut into 32 slices of three instructions, one slice
//                   behind each of the first 32 MFMAs
//     LDS         : one fragment read per MFMA pair, PL_D pairs ahead of its use (the reads run
//                   on into the next period's first K fragments)
//     global->LDS : this wavefront's five transfers of the period, one behind each of five MFMAs
// so the vector work, the LDS latency and the transfer issue all hide under the matrix core.
// K and V stream through separate rings because V of a block is needed two periods after its K:
// period t issues K of block t + PL_AHEAD and V of block t + PL_AHEAD - 3 ("group" t + PL_AHEAD).
// At the top of period t every wavefront waits for its own transfers of group t+2 and passes
// the barrier; then K(t+1), the head of K(t+2) and V(t-1) are complete for everybody, and all
// wavefronts have left period t-1, the last reader of K(t) and V(t-2), whose slots group
// t + PL_AHEAD reuses.
constexpr int PL_AHEAD = 8;
constexpr int PL_NK = PL_AHEAD;                                   // K ring slots
constexpr int PL_NV = 8;                                          // V ring slots (7 needed)
constexpr int PL_K_BYTES = K_BLK_ELEMS * 2;                       // 12288
constexpr int PL_V_BYTES = V_BLK_ELEMS * 2;                       // 8192
constexpr int PL_V_BASE = PL_NK * PL_K_BYTES;                     // 98304
constexpr int PL_LDS_BYTES = PL_V_BASE + PL_NV * PL_V_BYTES;      // 163840 = all of LDS
static_assert((PL_NK & (PL_NK - 1)) == 0 && (PL_NV & (PL_NV - 1)) == 0, "slot = block & (n - 1)");
constexpr int PL_D = 6;                                           // fragment reads in flight
constexpr int PL_QUERIES = 256;
constexpr int PL_OUT_ROW = 132;   // floats per row of the epilogue's LDS tile: 128 + 4 of padding
static_assert(4 * 64 * PL_OUT_ROW * 4 <= PL_LDS_BYTES, "epilogue tiles fit the idle rings");
#define PL_SB() __builtin_amdgcn_sched_barrier(0)

// The MFMAs of the pipelined loop are written in assembly to fix where their operands live:
// scores accumulate in vector registers (the softmax reads them), outputs and the resident Q
// fragments in accumulation registers (only the matrix core touches them), so no copies between
// the two register files appear in the loop.  The assembler cannot see that these statements
// are MFMAs: every vector-ALU read of their results below is either a whole period away or
// preceded by pl_mfma_drain().
__device__ inline void pl_mfma_s_first(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
__device__ inline void pl_mfma_s(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}
__device__ inline void pl_mfma_o(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
// The same, behind a wait for outstanding fragment reads.  The reads return in order and one is
// issued per quantum, PL_D quanta ahead of its use; waiting once per PL_WG quanta until at most
// PL_D - PL_WG of them are in flight makes the fragments of the whole group valid (a wait costs
// a lone wavefront an issue slot like any other instruction).
#ifndef PL_WG
#define PL_WG 4
#endif
constexpr int PL_WAIT = PL_D - PL_WG;
static_assert(PL_WAIT >= 0 && 20 % PL_WG == 0, "a period's 20 quanta are waited for in whole groups");
__device__ inline void pl_mfma_s_first_w(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(%3)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0"
               : "=&v"(d) : "v"(a), "a"(b), "n"(PL_WAIT));
}
__device__ inline void pl_mfma_s_w(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(%3)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
               : "+v"(d) : "v"(a), "a"(b), "n"(PL_WAIT));
}
__device__ inline void pl_mfma_o_w(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(%3)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
               : "+a"(d) : "v"(a), "v"(b), "n"(PL_WAIT));
}
// An output MFMA with one global -> LDS transfer behind it.  M0 (the transfer's LDS address) is
// set in front of the MFMA, which then fills the wait state the hardware wants between a write
// of M0 and its use; set next to the transfer it costs an idle issue slot.  Same contract as
// dma16_scalar_base: wave-uniform base and LDS address, 32-bit per-lane offset.
// STREAM: non-temporal transfer (data nobody else reads).
template <bool WAIT, bool STREAM>
__device__ inline void pl_mfma_o_dma(f32x16& d, const bf16x8& a, const bf16x8& b,
                                     uint32_t lane_off, const void* base, uint32_t lds) {
  const uint64_t u = (uint64_t)base;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  base = (const void*)(((uint64_t)hi << 32) | lo);
  lds = __builtin_amdgcn_readfirstlane(lds);
#define PL_MFMA_DMA_W(POLICY)                                                                   \
  asm volatile("s_mov_b32 m0, %5\n\ts_waitcnt lgkmcnt(%6)\n\t"                                  \
               "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\tglobal_load_lds_dwordx4 %3, %4" POLICY \
               : "+a"(d) : "v"(a), "v"(b), "v"(lane_off), "s"(base), "s"(lds), "n"(PL_WAIT)      \
               : "memory")
#define PL_MFMA_DMA(POLICY)                                                                     \
  asm volatile("s_mov_b32 m0, %5\n\t"                                                           \
               "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\tglobal_load_lds_dwordx4 %3, %4" POLICY \
               : "+a"(d) : "v"(a), "v"(b), "v"(lane_off), "s"(base), "s"(lds) : "memory")
  if constexpr (WAIT && STREAM) PL_MFMA_DMA_W(TMLA_STREAM_POLICY);
  else if constexpr (WAIT) PL_MFMA_DMA_W("");
  else if constexpr (STREAM) PL_MFMA_DMA(TMLA_STREAM_POLICY);
  else PL_MFMA_DMA("");
#undef PL_MFMA_DMA_W
#undef PL_MFMA_DMA
}
// enough idle issue slots for the last MFMA (16 passes) to have written its result
__device__ inline void pl_mfma_drain() {
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");
}
__global__ void __launch_bounds__(256, 1) prefix_attn_pipelined_kernel(PrefixArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int h = blockIdx.x, mb = blockIdx.y, sp = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q0 = mb * PL_QUERIES + wave * 64;   // first query of this wavefront

  const int tb0 = sp * a.blocks_per_split;
  const int tb1 = min(a.ntb, tb0 + a.blocks_per_split);
  const int nblk = tb1 - tb0;
  // the very last block of the prefix may be partial; it gets a masked pass after the loop
  const bool has_tail = (tb1 == a.ntb) && (a.Ls % TOK_BLK != 0) && nblk > 0;
  const int nfull = has_tail ? nblk - 1 : nblk;
  const int tail_limit = a.Ls - (tb0 + nblk - 1) * TOK_BLK;   // valid tokens of a partial tail
  const uint32_t lane_addr = lds_addr(smem) + lane * 16;

  bf16x8 qf[2][12];
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
#pragma unroll
  for (int nb = 0; nb < 2; nb++)
#pragma unroll
    for (int ks = 0; ks < 12; ks += 4)
      asm volatile("s_waitcnt vmcnt(0)"
                   : "+a"(qf[nb][ks]), "+a"(qf[nb][ks + 1]), "+a"(qf[nb][ks + 2]),
                     "+a"(qf[nb][ks + 3])::"memory");

  // transfers: fragment f of a block is moved by wavefront f % 4 (K: 12 fragments, V: 8)
  const char* kbase = (const char*)(a.pk + ((size_t)h * a.ntb + tb0) * K_BLK_ELEMS);
  const char* vbase = (const char*)(a.pv + ((size_t)h * a.ntb + tb0) * V_BLK_ELEMS);
  // The RoPE part of a key (fragments 8 .. 11 of a block) is the same for every head: all heads
  // take it from head 0's blocks, so that it is fetched from HBM once and served from cache to
  // the other heads (a fifth of the expanded cache's bytes), with the ordinary cache policy.
  const char* rbase = (const char*)(a.pk + (size_t)tb0 * K_BLK_ELEMS);
  const uint32_t lds_base = lds_addr(smem) + wave * 1024;
  uint32_t lane_off[3];   // fragment w, w + 4, w + 8 of a block
#pragma unroll
  for (int f = 0; f < 3; f++) lane_off[f] = f * 4096 + wave * 1024 + lane * 16;
  using GUARD = std::true_type;
  using NOGUARD = std::false_type;
  auto dma_k = [&](int k, int f, auto guard_tag) __attribute__((always_inline)) {
    if (!decltype(guard_tag)::value || k < nblk) {
      if (f == 2)
        dma16_scalar_base<false>(lane_off[f], rbase + (size_t)k * PL_K_BYTES,
                                 lds_base + (k & (PL_NK - 1)) * PL_K_BYTES + f * 4096);
      else
        dma16_scalar_base<true>(lane_off[f], kbase + (size_t)k * PL_K_BYTES,
                                lds_base + (k & (PL_NK - 1)) * PL_K_BYTES + f * 4096);
    }
  };
  auto dma_v = [&](int kv, int f, auto guard_tag) __attribute__((always_inline)) {
    if (!decltype(guard_tag)::value || (kv >= 0 && kv < nblk))
      dma16_scalar_base(lane_off[f], vbase + (size_t)kv * PL_V_BYTES,
               lds_base + PL_V_BASE + (kv & (PL_NV - 1)) * PL_V_BYTES + f * 4096);
  };
  f32x16 o[4][2];
  // Softmax bookkeeping.  The exponent reference m of a query is fixed before the walk over the
  // split and never moved inside the loop: the result does not depend on the reference
  // (numerator and denominator share it), only the float range does.  The first walk takes the
  // maximum of the query's scores over the first block; scores more than ~2^7 (log2 units) above
  // that would overflow, which shows as a denominator that is not a moderate finite number and
  // is checked once at the end.  Then (rare) the exact maxima over the whole split are formed in
  // a scores-only pass and the split is walked again with those.
  float m[2] = {0.f, 0.f}, l[2] = {0.f, 0.f}, lt[2] = {0.f, 0.f};
  float m_exact[2] = {0.f, 0.f};
  const float c = a.c;

  // top of period t: groups t+3 .. t+PL_AHEAD-1 may still be in flight, group t+2 must have
  // landed.  Group k holds three transfers of K(k) if k < nblk and two of V(k-3) if
  // 0 <= k-3 < nblk.
  auto sync = [&](int t, auto steady_tag) __attribute__((always_inline)) {
    static_assert(PL_AHEAD == 8, "the waits below assume five groups in flight");
    if constexpr (decltype(steady_tag)::value) {
      vm_wait<25>();
    } else {
      const int lo = t + 3, hi = t + PL_AHEAD - 1;
      const int nk = max(0, min(hi, nblk - 1) - max(lo, 0) + 1);
      const int nv = max(0, min(hi, nblk + 2) - max(lo, 3) + 1);
      const int pend = 3 * nk + 2 * nv;
      if (pend >= 25) vm_wait<25>();
      else if (pend >= 20) vm_wait<20>();
      else if (pend >= 15) vm_wait<15>();
      else if (pend >= 10) vm_wait<10>();
      else if (pend >= 5) vm_wait<5>();
      else vm_wait<0>();
    }
    raw_barrier();
  };

  bf16x8 fr[8];          // fragment ring: fragment j of period t lives in fr[(4 (t & 1) + j) % 8]
  f32x16 sb[2][2];       // scores of blocks of even / odd index
  bf16x8 pb[2][2][2];    // probabilities of blocks of even / odd index

  // Period t = 0 .. nfull.  The instruction stream is the same for every period; at the two ends
  // some of it runs on data that is not there, arranged to be harmless:
  //   * scores of a block t+1 > nfull multiply whatever the ring holds; nobody reads them;
  //   * the softmax pieces of block t = nfull (the partial tail, or nothing) produce
  //     probabilities nobody reads, and their sum is dropped;
  //   * P V of block -1 (period 0) multiplies the all-zero initial probabilities with the K
  //     fragments of block 0 standing in for V, which adds exact zeros.
  // STEADY: 2 <= t and t + PL_AHEAD < nblk -- every block and transfer the period touches exists,
  // so the guards and the count of transfers in flight are compile-time facts.
  auto period = [&](int t, auto par_tag, auto steady_tag) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par_tag)::value;
    constexpr bool STEADY = decltype(steady_tag)::value;
    f32x16 (&s_in)[2] = sb[PAR];
    f32x16 (&s_out)[2] = sb[PAR ^ 1];
    bf16x8 (&p_out)[2][2] = pb[PAR];
    bf16x8 (&p_in)[2][2] = pb[PAR ^ 1];

    sync(t, steady_tag);
    const uint32_t ka1 = lane_addr + ((t + 1) & (PL_NK - 1)) * PL_K_BYTES;   // K(t+1)
    const uint32_t ka2 = lane_addr + ((t + 2) & (PL_NK - 1)) * PL_K_BYTES;   // K(t+2)
    const uint32_t va =                                                // V(t-1), or K(0)
        lane_addr + (STEADY || t >= 1 ? PL_V_BASE + ((t - 1) & (PL_NV - 1)) * PL_V_BYTES : 0);
    const int kg = t + PL_AHEAD;      // group issued in this period

    float xa = 0.f, xb = 0.f, ea = 0.f, eb = 0.f;
    // denominators of block t, per column block; the two probabilities of a packed pair go to
    // separate sums (a temporary for their sum lands in the register next to the packed pair,
    // and the write behind the conversion then costs a wait state)
    float sum[2] = {0.f, 0.f}, sum_b[2] = {0.f, 0.f};
    // The softmax of block t, two scores (one packed pair of probabilities) per quantum, spread
    // so that no instruction waits for the one before it and no transcendental directly follows
    // an MFMA (either would cost idle issue slots):
    //   behind the first MFMA of quantum j : arguments of pair j
    //   behind the second MFMA             : pack the pair of quantum j-1 and add it to the
    //                                        denominator; e_a(j), e_b(j) = exp2
    // Pair k = elements 2 (k % 8), 2 (k % 8) + 1 of column block k / 8.  The empty statements pin
    // every piece where it is written (the results are only used much later, and would
    // otherwise be moved down there).  (Summing the denominators on the matrix core instead -- a
    // 32 x 16 matrix of ones times P^T, four more MFMAs per block for 32 additions less -- was 2 %
    // slower: the kernel runs at the clock the power limit allows, and MFMAs are what draws it.)
    auto part1 = [&](auto j_tag) __attribute__((always_inline)) {
      constexpr int j = decltype(j_tag)::value;
      if constexpr (j < 16) {
        constexpr int nb = j / 8, v0 = 2 * (j % 8);
        xa = __builtin_fmaf(s_in[nb][v0], c, -m[nb]);
        xb = __builtin_fmaf(s_in[nb][v0 + 1], c, -m[nb]);
        asm volatile("" : "+v"(xa), "+v"(xb));
      }
    };
    auto part2 = [&](auto j_tag) __attribute__((always_inline)) {
      constexpr int j = decltype(j_tag)::value;
      if constexpr (j >= 1 && j <= 16) {
        constexpr int nb = (j - 1) / 8, v0 = 2 * ((j - 1) % 8);
        const bf16x2 pk = {(__bf16)ea, (__bf16)eb};
        p_out[nb][v0 / 8][v0 % 8] = pk[0];
        p_out[nb][v0 / 8][v0 % 8 + 1] = pk[1];
        asm volatile("" : "+v"(p_out[nb][v0 / 8]));
        PL_SB();
      }
      if constexpr (j >= 1 && j <= 16) {
        constexpr int nbp = (j - 1) / 8;
        sum[nbp] += ea;
        sum_b[nbp] += eb;
        asm volatile("" : "+v"(sum[nbp]), "+v"(sum_b[nbp]));
        PL_SB();
      }
      if constexpr (j < 16) {
        ea = fast_exp2(xa);
        asm volatile("" : "+v"(ea));
        PL_SB();
        eb = fast_exp2(xb);
        asm volatile("" : "+v"(eb));
      }
    };
    auto dma = [&](auto i_tag) __attribute__((always_inline)) {
      constexpr int i = decltype(i_tag)::value;
      if constexpr (i < 3) dma_k(kg, i, std::integral_constant<bool, !STEADY>{});
      else dma_v(kg - 3, i - 3, std::integral_constant<bool, !STEADY>{});
    };

    // Quantum j: two MFMAs on fragment j (one per column block of queries).  A wavefront issues
    // in order and the matrix core takes one MFMA per ~32 cycles, so whatever stands between two
    // MFMAs beyond ~24 cycles of issue time leaves the matrix core idle: the other work is dealt
    // out evenly -- behind the first MFMA the two score arguments and the request for fragment
    // j + PL_D, behind the second the pack and the two exponentials; the transfers and the
    // denominator MFMAs go to the last quanta, which carry no softmax work.
    static_for<20>([&](auto j_tag) {
      constexpr int j = decltype(j_tag)::value;
      constexpr int cur = (4 * PAR + j) % 8;
      static_for<2>([&](auto nb_tag) {
        constexpr int nb = decltype(nb_tag)::value;
        // (the first MFMA of a group of PL_WG quanta waits for the group's fragments)
        constexpr bool wait_here = nb == 0 && j % PL_WG == 0;
        // the period's five transfers ride behind the MFMAs of quanta 16 .. 18; in the steady
        // state (no guards) each is fused with its MFMA
        constexpr int d = 2 * (j - 16) + nb;
        constexpr bool has_dma = d >= 0 && d < 5;
        constexpr bool fused_dma = STEADY && has_dma;
        if constexpr (j == 0) {
          if constexpr (wait_here) pl_mfma_s_first_w(s_out[nb], fr[cur], qf[nb][j]);
          else pl_mfma_s_first(s_out[nb], fr[cur], qf[nb][j]);
        } else if constexpr (j < 12) {
          if constexpr (wait_here) pl_mfma_s_w(s_out[nb], fr[cur], qf[nb][j]);
          else pl_mfma_s(s_out[nb], fr[cur], qf[nb][j]);
        } else {
          constexpr int kk = (j - 12) / 4, db = (j - 12) % 4;
          if constexpr (fused_dma) {
            // transfer d of the group: K fragments w, w + 4, w + 8 of block kg, then V fragments
            // w, w + 4 of block kg - 3
            if constexpr (d < 2)
              pl_mfma_o_dma<wait_here, true>(o[db][nb], fr[cur], p_in[nb][kk], lane_off[d],
                                             kbase + (size_t)kg * PL_K_BYTES,
                                             lds_base + (kg & (PL_NK - 1)) * PL_K_BYTES + d * 4096);
            else if constexpr (d == 2)
              pl_mfma_o_dma<wait_here, false>(o[db][nb], fr[cur], p_in[nb][kk], lane_off[d],
                                              rbase + (size_t)kg * PL_K_BYTES,
                                              lds_base + (kg & (PL_NK - 1)) * PL_K_BYTES + d * 4096);
            else
              pl_mfma_o_dma<wait_here, true>(o[db][nb], fr[cur], p_in[nb][kk], lane_off[d - 3],
                                       vbase + (size_t)(kg - 3) * PL_V_BYTES,
                                       lds_base + PL_V_BASE + ((kg - 3) & (PL_NV - 1)) * PL_V_BYTES +
                                           (d - 3) * 4096);
          } else if constexpr (wait_here) {
            pl_mfma_o_w(o[db][nb], fr[cur], p_in[nb][kk]);
          } else {
            pl_mfma_o(o[db][nb], fr[cur], p_in[nb][kk]);
          }
        }
        PL_SB();
        if constexpr (nb == 0) {
          part1(j_tag);
          constexpr int jn = j + PL_D;
          constexpr int nxt = (4 * PAR + jn) % 8;
          if constexpr (jn < 12) fr[nxt] = lds_read_b128<1024 * jn>(ka1);
          else if constexpr (jn < 20) fr[nxt] = lds_read_b128<1024 * (jn - 12)>(va);
          else fr[nxt] = lds_read_b128<1024 * (jn - 20)>(ka2);
        } else {
          part2(j_tag);
        }
        if constexpr (has_dma && !fused_dma) dma(std::integral_constant<int, has_dma ? d : 0>{});
        PL_SB();
      });
    });
    // Control flow joins below and at the top of the next period, and register copies may be
    // placed there; the last MFMAs must have written their results before any such copy.  The
    // steady-state periods follow each other without a join, and nothing reads this period's
    // last results before the next period is well under way (the generated code is checked for
    // that, across the loop's back edge as well).
#ifndef PL_STEADY_DRAIN
    if constexpr (!STEADY)
#endif
      pl_mfma_drain();
    if (STEADY || t < nfull) {
      l[0] += sum[0] + sum_b[0];
      l[1] += sum[1] + sum_b[1];
    }
  };

  // maximum of this lane's query over the first `limit` tokens of a block of scores, scaled
  auto block_max = [&](const f32x16& s, int limit) __attribute__((always_inline)) {
    float mx = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; v++)
      if (acc_row(v, g) < limit) mx = fmaxf(mx, s[v]);
    return max_halves(mx) * c;
  };

  using P0 = std::integral_constant<int, 0>;
  using P1 = std::integral_constant<int, 1>;

  // Scores-only pass over the split: the exact maximum of every query's scores (rare path, plain
  // double buffering of K through the ring, one barrier per block).
  auto exact_maxima = [&]() __attribute__((always_inline)) {
    float mx[2] = {-INFINITY, -INFINITY};
    dma_k(0, 0, GUARD{}); dma_k(0, 1, GUARD{}); dma_k(0, 2, GUARD{});
    for (int bk = 0; bk < nblk; bk++) {
      if (bk + 1 < nblk) {
        dma_k(bk + 1, 0, GUARD{}); dma_k(bk + 1, 1, GUARD{}); dma_k(bk + 1, 2, GUARD{});
        vm_wait<3>();
      } else {
        vm_wait<0>();
      }
      raw_barrier();
      const uint32_t ka = lane_addr + (bk & (PL_NK - 1)) * PL_K_BYTES;
      static_for<12>([&](auto j_tag) {
        constexpr int j = decltype(j_tag)::value;
        fr[j % 8] = lds_read_b128<1024 * j>(ka);
        lgkm_wait<0>(fr[j % 8]);
        static_for<2>([&](auto nb_tag) {
          constexpr int nb = decltype(nb_tag)::value;
          if constexpr (j == 0) pl_mfma_s_first(sb[0][nb], fr[j % 8], qf[nb][j]);
          else pl_mfma_s(sb[0][nb], fr[j % 8], qf[nb][j]);
        });
      });
      pl_mfma_drain();
      const int lim = (has_tail && bk == nblk - 1) ? tail_limit : 32;
#pragma unroll
      for (int nb = 0; nb < 2; nb++)
#pragma unroll
        for (int v = 0; v < 16; v++)
          if (acc_row(v, g) < lim) mx[nb] = fmaxf(mx[nb], sb[0][nb][v]);
    }
    m_exact[0] = max_halves(mx[0]) * c;
    m_exact[1] = max_halves(mx[1]) * c;
    raw_barrier();   // everybody is done reading before the next walk refills the ring
  };

  for (int attempt = 0;; attempt++) {
    // (the zeros are pinned: moved down next to the first MFMA that reads them, or re-created
    // there because they are known to be zero, the register writes would sit closer to that MFMA
    // than the hardware allows without wait states, which nobody inserts in front of an MFMA
    // written in assembly)
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
      for (int nb = 0; nb < 2; nb++)
#pragma unroll
        for (int v = 0; v < 16; v++) o[db][nb][v] = 0.f;
    asm volatile("" : "+a"(o[0][0]), "+a"(o[1][0]), "+a"(o[2][0]), "+a"(o[3][0]), "+a"(o[0][1]),
                      "+a"(o[1][1]), "+a"(o[2][1]), "+a"(o[3][1]));
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
      for (int e = 0; e < 8; e++) (&pb[0][0][0])[i][e] = (__bf16)0.f;
    asm volatile("" : "+v"(pb[0][0][0]), "+v"(pb[0][0][1]), "+v"(pb[0][1][0]), "+v"(pb[0][1][1]),
                      "+v"(pb[1][0][0]), "+v"(pb[1][0][1]), "+v"(pb[1][1][0]), "+v"(pb[1][1][1]));
    l[0] = l[1] = 0.f;
    for (int k = 0; k < PL_AHEAD - 1; k++) {
      dma_k(k, 0, GUARD{}); dma_k(k, 1, GUARD{}); dma_k(k, 2, GUARD{});
      dma_v(k - 3, 0, GUARD{}); dma_v(k - 3, 1, GUARD{});
    }

    if (nblk > 0) {
      // before period 0: the scores of block 0 and from them the exponent references, the first
      // fragments of K(1), group PL_AHEAD - 1
      sync(-1, NOGUARD{});
      {
        const uint32_t ka0 = lane_addr, ka1 = lane_addr + PL_K_BYTES;
        static_for<12>([&](auto j_tag) {
          constexpr int j = decltype(j_tag)::value;
          fr[j % 8] = lds_read_b128<1024 * j>(ka0);
          lgkm_wait<0>(fr[j % 8]);
          static_for<2>([&](auto nb_tag) {
            constexpr int nb = decltype(nb_tag)::value;
            if constexpr (j == 0) pl_mfma_s_first(sb[0][nb], fr[j % 8], qf[nb][j]);
            else pl_mfma_s(sb[0][nb], fr[j % 8], qf[nb][j]);
          });
        });
        static_for<PL_D>([&](auto j_tag) {
          constexpr int j = decltype(j_tag)::value;
          fr[j] = lds_read_b128<1024 * j>(ka1);
        });
        const int k = PL_AHEAD - 1;
        dma_k(k, 0, GUARD{}); dma_k(k, 1, GUARD{}); dma_k(k, 2, GUARD{});
        dma_v(k - 3, 0, GUARD{}); dma_v(k - 3, 1, GUARD{});
        pl_mfma_drain();
        if (attempt == 0) {
          const int limit0 = nfull > 0 ? 32 : tail_limit;
          m[0] = block_max(sb[0][0], limit0);
          m[1] = block_max(sb[0][1], limit0);
        } else {
          m[0] = m_exact[0];
          m[1] = m_exact[1];
        }
      }
      using ST = std::true_type;
      using GN = std::false_type;
      period(0, P0{}, GN{});
      if (1 <= nfull) period(1, P1{}, GN{});
      int t = 2;
      for (; t + 1 + PL_AHEAD < nblk; t += 2) {
        period(t, P0{}, ST{});
        period(t + 1, P1{}, ST{});
      }
      for (; t <= nfull; t += 2) {
        period(t, P0{}, GN{});
        if (t + 1 <= nfull) period(t + 1, P1{}, GN{});
      }
      lgkm_wait<0>();
      pl_mfma_drain();
    }
    if (has_tail) {
      // The scores of the partial last block were formed by the loop's last period (or above, if
      // the block is the only one).  Masked probabilities against the same references, then P V.
      vm_wait<0>();
      raw_barrier();
      auto tail = [&](auto par_tag) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_tag)::value;
        bf16x8 pt[2][2];
  #pragma unroll
        for (int nb = 0; nb < 2; nb++)
  #pragma unroll
          for (int v = 0; v < 16; v++) {
            const float e = acc_row(v, g) < tail_limit
                                ? fast_exp2(__builtin_fmaf(sb[PAR][nb][v], c, -m[nb])) : 0.f;
            l[nb] += e;
            pt[nb][v / 8][v % 8] = (__bf16)e;
          }
        // packed before the fragment reads, i.e. well in front of the MFMAs that read them
        asm volatile("s_nop 3" : "+v"(pt[0][0]), "+v"(pt[0][1]), "+v"(pt[1][0]), "+v"(pt[1][1]));
        const uint32_t va = lane_addr + PL_V_BASE + ((nblk - 1) & (PL_NV - 1)) * PL_V_BYTES;
        bf16x8 vf[8];
        static_for<8>([&](auto j) { vf[j] = lds_read_b128<1024 * decltype(j)::value>(va); });
        lgkm_wait<0>(vf[0], vf[1], vf[2], vf[3]);
        lgkm_wait<0>(vf[4], vf[5], vf[6], vf[7]);
  #pragma unroll
        for (int kk = 0; kk < 2; kk++)
  #pragma unroll
          for (int db = 0; db < 4; db++)
  #pragma unroll
            for (int nb = 0; nb < 2; nb++) pl_mfma_o(o[db][nb], vf[kk * 4 + db], pt[nb][kk]);
        pl_mfma_drain();
      };
      if (nfull & 1) tail(P1{});
      else tail(P0{});
    }


    lt[0] = sum_halves(l[0]);
    lt[1] = sum_halves(l[1]);
    if (attempt == 1) break;
    // a denominator that is not a moderate finite number: the references did not hold
    const bool bad_lane = !(lt[0] < 0x1p100f) || !(lt[1] < 0x1p100f);
    const bool bad_wave = __builtin_amdgcn_ballot_w64(bad_lane) != 0;
    int* flags = (int*)smem;
    __syncthreads();   // every transfer has landed and every ring read is done
    if (lane == 0) flags[wave] = bad_wave ? 1 : 0;
    __syncthreads();
    const int bad_wg = flags[0] | flags[1] | flags[2] | flags[3];
    __syncthreads();   // the flags are read before the ring is written again
    if (__builtin_amdgcn_readfirstlane(bad_wg) == 0) break;
    exact_maxima();
  }

  // Epilogue.  As MFMA output a lane holds 16-byte pieces of its query's partial row, 32 bytes
  // apart from its neighbour's: stored that way every instruction scatters 64 pieces of 32 B
  // over 32 rows, and the burst of all workgroups at once took 10 us of a launch.  The rings are
  // idle now (every transfer has landed, everyone is past the last barrier), so each wavefront
  // turns its 64 x 128 tile around in a private LDS region and 32 lanes store one row's 512
  // contiguous bytes.  A row that saw nothing (l = 0) is left unwritten: its LSE is -inf.
  {
    // (after a second walk nobody has met at a barrier yet: the other wavefronts may still be
    // reading the rings, and their last transfers may still be landing)
    vm_wait<0>();
    lgkm_wait<0>();
    raw_barrier();
    float* tile = (float*)smem + wave * (64 * PL_OUT_ROW);
    bool row_ok[2];
#pragma unroll
    for (int nb = 0; nb < 2; nb++) {
      const int qi = q0 + nb * 32 + n;
      row_ok[nb] = qi < a.M && lt[nb] > 0.f;
      const float inv = row_ok[nb] ? 1.f / lt[nb] : 0.f;
#pragma unroll
      for (int db = 0; db < 4; db++)
#pragma unroll
        for (int v4 = 0; v4 < 4; v4++) {
          const float4 w = make_float4(o[db][nb][4 * v4] * inv, o[db][nb][4 * v4 + 1] * inv,
                                       o[db][nb][4 * v4 + 2] * inv, o[db][nb][4 * v4 + 3] * inv);
          *(float4*)(tile + (nb * 32 + n) * PL_OUT_ROW + 32 * db + 8 * v4 + 4 * g) = w;
        }
      if (qi < a.M && g == 0) {
        const size_t row = (size_t)sp * a.rows + (size_t)qi * a.H + h;
        a.lse[row] = row_ok[nb] ? (m[nb] + fast_log2(lt[nb])) * LN2 : -INFINITY;
      }
    }
    // which of this wavefront's 64 rows are written: one bit per row, from the lanes that own them
    const uint64_t ok0 = __builtin_amdgcn_ballot_w64(row_ok[0] && g == 0);
    const uint64_t ok1 = __builtin_amdgcn_ballot_w64(row_ok[1] && g == 0);
    const uint64_t ok = (ok0 & 0xffffffffull) | (ok1 << 32);
    // (each wavefront reads back only what it wrote itself: no barrier)
#pragma unroll 4
    for (int i = 0; i < 32; i++) {
      const int r = 2 * i + g;                       // row of the tile: query q0 + r
      const float4 w = *(const float4*)(tile + r * PL_OUT_ROW + 4 * n);
      if ((ok >> r) & 1) {
        const size_t row = (size_t)sp * a.rows + (size_t)(q0 + r) * a.H + h;
        *(float4*)(a.o + row * D_V + 4 * n) = w;
      }
    }
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
                                const int (&limit)[2], int g, int nvalid = 32) {
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
        softmax_block(sacc[nb], m[nb], l[nb], c, limit[nb], g, p[nb][0], p[nb][1], rescale);
    if (rescale) {
#pragma unroll
      for (int db = 0; db < 4; db++) {
        // the accumulators live in accumulation registers, which the vector ALU cannot address;
        // routing them through these statements keeps their copies inside the rare branch
        // (otherwise the copies out are hoisted and run for every block)
        asm volatile("" : "+a"(o[db][nb]));
#pragma unroll
        for (int v = 0; v < 16; v++) o[db][nb][v] *= alpha;
        asm volatile("" : "+a"(o[db][nb]));
      }
    }
  }
  lgkm_wait<0>(vf[0], vf[1], vf[2], vf[3]);
  lgkm_wait<0>(vf[4], vf[5], vf[6], vf[7]);
  if (nvalid < 32) {
    // a partial block of a paged cache: what lies behind its last token is not ours and need not
    // be finite, and 0 * NaN would poison the product, so those V entries are cleared (element e
    // of fragment kk holds token 16 kk + 8 (e / 4) + 4 g + e % 4, the order of the probabilities)
#pragma unroll
    for (int kk = 0; kk < 2; kk++)
#pragma unroll
      for (int e = 0; e < 8; e++)
        if (acc_row(8 * kk + e, g) >= nvalid) {
#pragma unroll
          for (int db = 0; db < 4; db++) vf[kk * 4 + db][e] = (__bf16)0.f;
        }
  }
#pragma unroll
  for (int kk = 0; kk < 2; kk++)
#pragma unroll
    for (int db = 0; db < 4; db++) {
      o[db][0] = mfma32(vf[kk * 4 + db], p[0][kk], o[db][0]);
      o[db][1] = mfma32(vf[kk * 4 + db], p[1][kk], o[db][1]);
    }
}

// PAGED = false: the shared prefix, query block mb of all M queries, token split sp.
// PAGED = true: the expanded paged suffix of request mb (naive_only mode): its S_q <= 64 queries,
// token chunk sp of its own suffix, 32-token blocks located through the block table, causal mask
// inside the suffix.  Same streaming and merge; grid.y = request.
template <bool PAGED>
__global__ void __launch_bounds__(256, 1) prefix_attn_token_split_kernel(PrefixArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int h = blockIdx.x, mb = blockIdx.y, sp = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int q0 = PAGED ? mb * a.Sq : mb * 64;
  const int q_end = PAGED ? q0 + a.Sq : a.M;
  const int slot = PAGED ? a.first_slot + sp : sp;
  int len = a.Ls;               // tokens this workgroup's queries can see at most
  const int32_t* bt = nullptr;
  if (PAGED) {
    len = a.lens[mb];
    bt = a.block_table + (size_t)mb * a.max_blocks;
  }

  const int tb0 = sp * a.blocks_per_split;
  const int tb1 = min(PAGED ? (len + TOK_BLK - 1) / TOK_BLK : a.ntb, tb0 + a.blocks_per_split);
  const __bf16* kbase = a.pk + ((size_t)h * a.ntb) * K_BLK_ELEMS + lane * 8;
  const __bf16* vbase = a.pv + ((size_t)h * a.ntb) * V_BLK_ELEMS + lane * 8;
  // the RoPE part of the keys is the same for every head: taken from head 0's blocks, fetched
  // from HBM once and served from cache to the other heads
  const __bf16* rbase = a.pk + lane * 8;

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
  auto issue = [&](int tb, int rslot) {
    char* dst = ring + rslot * TS_BLOCK_BYTES;
    size_t ptb = tb;            // physical 32-token block
    if (PAGED) {
      // scalar load: a vector load here would have to be waited for with vmcnt(0)
      const int page = scalar_load_i32(bt + (tb >> a.page_shift));
      ptb = ((size_t)page << a.page_shift) + (tb & ((1 << a.page_shift) - 1));
    }
    const __bf16* ks = kbase + ptb * K_BLK_ELEMS;
    const __bf16* rs = rbase + ptb * K_BLK_ELEMS;
    const __bf16* vs = vbase + ptb * V_BLK_ELEMS;
#pragma unroll
    for (int f = 0; f < 8; f++) dma16_stream(ks + f * 512, dst + f * 1024);
#pragma unroll
    for (int f = 8; f < 12; f++) dma16(rs + f * 512, dst + f * 1024);
#pragma unroll
    for (int f = 0; f < 8; f++) dma16_stream(vs + f * 512, dst + K_BLK_ELEMS * 2 + f * 1024);
  };
  const int first = tb0 + wave;
  const int nmine = first < tb1 ? (tb1 - first + 3) / 4 : 0;
  if (nmine > 0) issue(first, 0);
  if (nmine > 1) issue(first + 4, 1);
  // The queries are requested behind the first two blocks, so their latency runs alongside the
  // stream's instead of in front of it, and waited for together with those blocks: resident
  // from here on, no wait on them inside the loop.
  bf16x8 qf[2][12];
  load_q_frags(a, h, q0, n, g, qf, q_end);
#pragma unroll
  for (int nb = 0; nb < 2; nb++)
#pragma unroll
    for (int ks = 0; ks < 12; ks += 4)
      asm volatile("s_waitcnt vmcnt(0)"
                   : "+v"(qf[nb][ks]), "+v"(qf[nb][ks + 1]), "+v"(qf[nb][ks + 2]),
                     "+v"(qf[nb][ks + 3])::"memory");
  for (int j = 0; j < nmine; j++) {
    if (j + 1 < nmine) vm_wait<20>();   // block j has landed, block j+1 may still be in flight
    else vm_wait<0>();
    const int tb = first + 4 * j;
    int limit[2];
#pragma unroll
    for (int nb = 0; nb < 2; nb++) {
      // PAGED: query s = nb * 32 + n of the request sees suffix tokens j <= len - S_q + s
      const int vis = PAGED ? len - a.Sq + nb * 32 + n + 1 : len;
      limit[nb] = min(32, vis - tb * TOK_BLK);
    }
    ts_block(ring_addr + (j & 1) * TS_BLOCK_BYTES, lane, qf, o, m, l, a.c, limit, g,
             PAGED ? min(32, len - tb * TOK_BLK) : 32);
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
    if (qi >= q_end) continue;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int w = 0; w < 4; w++) {
      const float4 x = *(const float4*)(sm_o + ((size_t)w * 64 + qq) * TS_ROW_FLOATS + c4 * 4);
      acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    const size_t row = (size_t)slot * a.rows + (size_t)qi * a.H + h;
    *(float4*)(a.o + row * D_V + c4 * 4) = acc;
  }
  if (tid < 64 && q0 + tid < q_end) {
    float ms = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; w++) ms = fmaxf(ms, sm_m[w * 64 + tid]);
    float lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; w++) {
      const float mw = sm_m[w * 64 + tid];
      lsum += (mw == -INFINITY) ? 0.f : sm_l[w * 64 + tid] * fast_exp2(mw - ms);
    }
    const size_t row = (size_t)slot * a.rows + (size_t)(q0 + tid) * a.H + h;
    a.lse[row] = (lsum > 0.f) ? (ms + fast_log2(lsum)) * LN2 : -INFINITY;
  }
}

int mfma_prefix_attention(const Plan& p, const DecodeArgs& d) {
  if (p.np_split <= 0) return TMLA_OK;
  PrefixArgs a = {};
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
  static LdsOptIn lds_pl, lds_qs, lds_ts;
  if (a.M > PIPELINED_MIN_M && !(debug_flags() & 0x400)) {
    if (lds_pl.ensure((const void*)prefix_attn_pipelined_kernel, PL_LDS_BYTES) != hipSuccess)
      return TMLA_ERR_HIP;
    dim3 grid(p.H, (a.M + PL_QUERIES - 1) / PL_QUERIES, p.np_split);
    hipLaunchKernelGGL(prefix_attn_pipelined_kernel, grid, dim3(256), PL_LDS_BYTES, d.stream, a);
  } else if (a.M > PIPELINED_MIN_M) {
    if (lds_qs.ensure((const void*)prefix_attn_query_split_kernel<1>, QS_LDS_BYTES) != hipSuccess)
      return TMLA_ERR_HIP;
    dim3 grid(p.H, (a.M + QS_QUERIES - 1) / QS_QUERIES, p.np_split);
    // NB = 1 measured faster than NB = 2 on every configuration: vector-ALU and matrix-core
    // instructions of a SIMD issue serially, so hiding LDS and barrier latency with a second
    // wavefront pays more than halving the LDS traffic
    hipLaunchKernelGGL(prefix_attn_query_split_kernel<1>, grid, dim3(512), QS_LDS_BYTES, d.stream,
                       a);
  } else {
    if (lds_ts.ensure((const void*)prefix_attn_token_split_kernel<false>, TS_LDS_BYTES) != hipSuccess)
      return TMLA_ERR_HIP;
    dim3 grid(p.H, (a.M + 63) / 64, p.np_split);
    hipLaunchKernelGGL(prefix_attn_token_split_kernel<false>, grid, dim3(256), TS_LDS_BYTES, d.stream, a);
  }
  return TMLA_OK;
}

// Naive attention over each request's own expanded paged suffix (naive_only mode): chunks of
// p.ns_chunk tokens, partial slots [np_split, np_split + ns_chunks).
int mfma_naive_suffix_attention(const Plan& p, const DecodeArgs& d) {
  if (p.ns_chunks <= 0 || p.rows == 0) return TMLA_OK;
  if (p.Sq > 64) return TMLA_ERR_UNSUPPORTED;
  PrefixArgs a = {};
  a.q = (const __bf16*)d.q;
  a.pk = (const __bf16*)d.suffix_k_pool;
  a.pv = (const __bf16*)d.suffix_v_pool;
  a.o = (float*)(d.ws + p.off_naive_o);
  a.lse = (float*)(d.ws + p.off_naive_lse);
  a.M = p.B * p.Sq; a.H = p.H; a.Ls = 0;
  a.ntb = (int)(((int64_t)d.num_blocks * d.block_size) / TOK_BLK);
  a.blocks_per_split = p.ns_chunk / TOK_BLK;
  a.rows = p.rows;
  a.c = d.sm_scale * LOG2E;
  a.block_table = d.block_table; a.lens = d.suffix_lens; a.max_blocks = d.max_blocks;
  a.page_shift = d.block_size == 64 ? 1 : 2;
  a.Sq = p.Sq; a.first_slot = p.np_split;
  static LdsOptIn lds;
  if (lds.ensure((const void*)prefix_attn_token_split_kernel<true>, TS_LDS_BYTES) != hipSuccess)
    return TMLA_ERR_HIP;
  dim3 grid(p.H, p.B, p.ns_chunks);
  hipLaunchKernelGGL(prefix_attn_token_split_kernel<true>, grid, dim3(256), TS_LDS_BYTES, d.stream, a);
  return TMLA_OK;
}

}  // namespace tmla
