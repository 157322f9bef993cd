// Absorb-formulation flash-decode over latent cache rows for requests with 128 or more query rows
// (S_q * H >= 128; paper Algorithm 1 step 6): 128 query rows per workgroup, 64 tokens per step.
//
// A compute unit fetches cache tiles at a limited rate (about 25 B/ns of data that is not yet in
// its L2), and with 64 query rows per workgroup a step's two tiles take longer to fetch than its
// MFMAs take to run.  Here every fetched tile meets twice as many query rows, so the arithmetic
// of a step (136 MFMAs per wavefront) outlasts the fetch of the next one.
//
// The two matrix products of a step want different work splits, so the four wavefronts change
// roles inside a step and hand the probabilities over through LDS:
//   scores   S^T = C Q_abs^T : wavefront w takes query block w (32 rows) and all 64 tokens:
//            72 MFMAs, the two tiles alternating (two independent accumulation chains).  All
//            scores of a query sit in one wavefront, so maxima and denominators need no exchange;
//   outputs  O^T += C_N^T P^T: wavefront (qp, lh) takes query blocks 2 qp, 2 qp + 1 and latent
//            columns [256 lh, 256 lh + 256): 64 MFMAs, every transposed cache fragment read from
//            LDS feeds two of them.
// One step: barrier A (the step's tiles have landed, everyone is done with the previous step),
// scores with the next step's transfers between the MFMAs, exponentials, probabilities -> LDS,
// barrier C, outputs.
//
// Exponent references are fixed for a whole walk over the chunk (the result does not depend on
// the reference, only the float range does): the first walk takes the maxima of step 0; if a
// denominator ends up outside a moderate finite range, the exact maxima are formed in a
// scores-only pass and the chunk is walked again with those.
//
// LDS is filled to the last byte: four tiles of 36864 B and 16 KiB of probabilities.  The tile
// therefore has no padding: latent row r at r * 1024, chunk c (16 B) in slot c ^ f(r) with
// f(r) = ((r & 3) << 2) | ((r >> 2) & 3) -- a bijection on any 16 consecutive rows, which keeps
// the 16-byte reads of the score product (16 rows, one chunk) on distinct banks, and whose high
// two bits differ among four consecutive rows, which does the same for the transposing reads
// (4 rows x 64 B).  The rope part (32 rows x 128 B) keeps chunk c of row r in slot
// c ^ ((r >> 1) & 7).  XOR-ing a compile-time chunk index into a per-lane offset commutes with
// the swizzle, so one address register per pattern serves all fragments.
#include "tmla_absorb_tile.hpp"

namespace tmla {

constexpr int A128_MAIN_BYTES = 32 * 1024;
constexpr int A128_TILE_BYTES = A128_MAIN_BYTES + 32 * 128;   // 36864
constexpr int A128_P_OFF = 4 * A128_TILE_BYTES;               // 147456
constexpr int A128_P_BYTES = 4 * 4096;                        // [query block][k-step][lane] 16 B
constexpr int A128_LDS_BYTES = A128_P_OFF + A128_P_BYTES;     // 163840 = all of LDS
static_assert(A128_LDS_BYTES <= 163840, "LDS layout");

// With 256 accumulation registers of outputs and 144 vector registers of query fragments per
// lane the register file is full, so the MFMAs are written in assembly to fix where their
// operands live (outputs in accumulation registers, everything else in vector registers; left
// to the allocator, outputs wander between the files and spill).  The assembler does not see
// that these statements are MFMAs: every vector-ALU read of their results is preceded by
// a128_drain(), and no vector-ALU instruction writes an operand right in front of them.
__device__ inline void a128_mfma_s_first(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b));
}
__device__ inline void a128_mfma_s(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b));
}
__device__ inline void a128_mfma_o(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
// The same behind a wait for LDS reads (at most N still in flight): one statement, so that
// nothing is put between the wait and the MFMA.
template <int N>
__device__ inline void a128_mfma_s_first_w(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(%3)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0"
               : "=&v"(d) : "v"(a), "v"(b), "n"(N));
}
template <int N>
__device__ inline void a128_mfma_s_w(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(%3)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
               : "+v"(d) : "v"(a), "v"(b), "n"(N));
}
template <int N>
__device__ inline void a128_mfma_o_w(f32x16& d, const bf16x8& a, const bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(%3)\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0"
               : "+a"(d) : "v"(a), "v"(b), "n"(N));
}
// enough idle issue slots for the last MFMA (16 passes) to have written its result
__device__ inline void a128_drain() {
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");
}

struct Absorb128Args {
  AbsorbArgs a;
  int nqg, n_lat, B;
};

// HAS_PREFIX: the launch has work items over the shared latent prefix (absorb_only mode).  Those
// rows are read by every request and must stay cached, and a per-transfer choice of the cache
// policy is a branch in the hot loop (-13 % at 64 heads), so such a launch uses ordinary
// transfers throughout; a launch over suffix rows alone streams them with the non-temporal hint.
template <bool HAS_PREFIX>
__global__ void __launch_bounds__(256, 1) absorb128_kernel(Absorb128Args args) {
  const AbsorbArgs& a = args.a;
  // (the alignment makes the low address bits of every tile zero, which the XOR addressing needs)
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // Workgroups that read the same tokens (the query groups of one request chunk) get ids 8 apart:
  // hardware deals consecutive ids round-robin over the 8 XCDs, so they share an L2.
  int item, qg, b;
  {
    const int id = blockIdx.x, x = id & 7, sl = id >> 3;
    qg = sl % args.nqg;
    const int j = (sl / args.nqg) * 8 + x;
    if (j >= args.n_lat * args.B) return;
    item = j % args.n_lat;
    b = j / args.n_lat;
    if (args.a.order) b = args.a.order[b];
  }
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qb = wave;                       // score product
  const int qp = wave & 1, lh = wave >> 1;   // output product

  // ---- which tokens
  int t0, t1;
  const bool is_prefix = HAS_PREFIX && item < a.ap_chunks;
  int len = 0;
  if (is_prefix) {
    t0 = item * a.ap_chunk;
    t1 = min(a.Ls, t0 + a.ap_chunk);
  } else {
    len = a.lens[b];
    t0 = (item - a.ap_chunks) * a.as_chunk;
    t1 = min(len, t0 + a.as_chunk);
  }
  const int r_own = (qg * 4 + qb) * 32 + n;   // the query row whose scores this lane holds
  int vis_q = t1;
  if (!is_prefix) {
    const int s = r_own < a.R ? r_own / a.H : 0;
    vis_q = max(0, min(len, len - a.Sq + s + 1));
  }
  if (t1 <= t0) {   // empty chunk (workgroup-uniform): only the LSEs are defined
    if (g == 0 && r_own < a.R)
      a.lat_lse[(size_t)item * a.rows + (int64_t)b * a.R + r_own] = -INFINITY;
    return;
  }
  const int nstep = (t1 - t0 + 63) / 64;

  // ---- tile streaming: global -> LDS
  const int32_t* bt = a.block_table + (size_t)b * a.max_blocks;
  const int first_blk = is_prefix ? 0 : t0 / a.block_size;
  int bt_cache = 0;
  if (!is_prefix) {
    const int nblk_chunk = (t1 - 1) / a.block_size - first_blk + 1;
    bt_cache = (lane < nblk_chunk) ? bt[first_blk + lane] : 0;
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(bt_cache)::"memory");
  }
  // A tile is filled by 36 wavefront-wide 1 KiB transfers, nine per wavefront: latent rows
  // wave + 4 K (K < 8; f(row) = (wave << 2) | (K & 3), uniform per transfer) and the rope parts of
  // rows 8 wave .. 8 wave + 7.  Rows past the end of the chunk repeat its last row (masked).
  // (the per-lane offsets are formed at every transfer from the lane number: registers are
  // scarcer here than vector-ALU slots)
  const int lane16 = lane << 4;
  // (scalar base + 32-bit lane offset: no 64-bit vector arithmetic per transfer; dst = LDS address)
  auto issue_part = [&](auto k_tag, const RowSrc& s, uint32_t dst) __attribute__((always_inline)) {
    constexpr int K = decltype(k_tag)::value;
    if constexpr (K < 8) {
      const int r = wave + 4 * K;
      const int rr = min(r, s.last);
      if (s.stream)
        dma16_scalar_base<true>(lane16 ^ (((wave << 2) | (K & 3)) << 4),
                                s.lat + (size_t)rr * s.lat_stride, dst, r * 1024);
      else
        dma16_scalar_base<false>(lane16 ^ (((wave << 2) | (K & 3)) << 4),
                                 s.lat + (size_t)rr * s.lat_stride, dst, r * 1024);
    } else {
      const int rope_row = 8 * wave + (lane >> 3);
      const int rope_ch = ((lane & 7) ^ ((rope_row >> 1) & 7)) << 4;
      const int rr = min(rope_row, s.last);
      if (s.stream)
        dma16_scalar_base<true>(rr * s.rope_stride + rope_ch, s.rope, dst,
                                A128_MAIN_BYTES + wave * 1024);
      else
        dma16_scalar_base<false>(rr * s.rope_stride + rope_ch, s.rope, dst,
                                 A128_MAIN_BYTES + wave * 1024);
    }
  };
  auto issue_all = [&](const RowSrc& s, uint32_t dst) __attribute__((always_inline)) {
    static_for<9>([&](auto k) { issue_part(k, s, dst); });
  };
  // The two tiles (32 tokens each) of step `step`, tokens t0 + 64 * step ...  Suffix chunks start
  // on a 64-token boundary and cache blocks hold a multiple of 64 tokens, so one block-table
  // entry serves a step.  A second tile past the end of the chunk is filled with the chunk's
  // last row: all its scores are masked.
  const int bs_shift = __builtin_ctz((unsigned)a.block_size);
  auto step_src = [&](int step, RowSrc& s0, RowSrc& s1) __attribute__((always_inline)) {
    const int tok0 = t0 + step * 64;
    s0.last = t1 - 1 - tok0;              // >= 0 for every step of the chunk
    s0.stream = !HAS_PREFIX;
    if (is_prefix) {
      s0.lat = (const char*)a.pc + (size_t)tok0 * (D_L * 2);
      s0.rope = (const char*)a.pr + (size_t)tok0 * (D_R * 2);
      s0.lat_stride = D_L * 2;
      s0.rope_stride = D_R * 2;
    } else {
      const int bi = __builtin_amdgcn_readfirstlane((tok0 >> bs_shift) - first_blk);
      const int blk = bi < 64 ? __builtin_amdgcn_readlane(bt_cache, bi)
                              : scalar_load_i32(bt + first_blk + bi);
      s0.lat = (const char*)(a.pool +
                             (((size_t)blk << bs_shift) + (tok0 & (a.block_size - 1))) * D_ROW);
      s0.rope = s0.lat + D_L * 2;
      s0.lat_stride = s0.rope_stride = D_ROW * 2;
    }
    s1 = s0;
    const int adv = s0.last >= 32 ? 32 : s0.last;   // rows to the second tile (or to the last row)
    s1.lat += (size_t)adv * s0.lat_stride;
    s1.rope += (size_t)adv * s0.rope_stride;
    s1.last = s0.last >= 32 ? s0.last - 32 : 0;
  };
  auto issue_step = [&](int step) __attribute__((always_inline)) {
    RowSrc s0, s1;
    step_src(step, s0, s1);
    const uint32_t dst = lds_addr(smem) + ((step & 1) * 2) * A128_TILE_BYTES;
    issue_all(s0, dst);
    issue_all(s1, dst + A128_TILE_BYTES);
  };

  // ---- per-lane LDS byte offsets inside a tile
  const uint32_t smem_base = lds_addr(smem);
  //   score product: row n, chunk 2 ks + g -> (s0 ^ ((ks & 7) << 5)) + 256 (ks >> 3)   (ks < 32)
  //                  rope chunk 2 k + g    -> r0 ^ (k << 5)
  const int fn = ((n & 3) << 2) | ((n >> 2) & 3);
  const uint32_t s0_off = n * 1024 + ((g ^ fn) << 4);
  const uint32_t r0_off = A128_MAIN_BYTES + n * 128 + ((g ^ ((n >> 1) & 7)) << 4);
  //   output product (transposing 8-byte reads; 16-lane group j = lane / 16, r = lane % 16):
  //     token row 16 kk + 8 half + 4 g + r / 4   (f = ((r / 4) << 2) | (2 half + g)),
  //     latent columns 256 lh + 32 mb + 16 (j % 2) + 4 (r % 4) .. + 3
  //     -> (v ^ ((mb & 3) << 6)) + 256 (mb >> 2) + 16384 kk (+ the tile)
  const int j16 = lane >> 4, r16 = lane & 15, rq = r16 >> 2;
  const int cx = 2 * (j16 & 1) + ((r16 & 3) >> 1);
  const uint32_t v_lo = (4 * g + rq) * 1024 + 64 * rq + ((cx ^ g) << 4) + 8 * (r16 & 1) + 512 * lh;
  //     (eight rows further down the swizzle differs in bit 1 of the slot: v_hi = (v_lo + 8192) ^ 32)
  float* const lbuf = (float*)(smem + A128_P_OFF);   // [query block][n] after the last step

  // ---- absorbed query fragments of the own query block (B operand of the score product):
  // row n, elements 16 ks + 8 g .. + 7.  Rows past the request's last one repeat it.
  issue_step(0);
  bf16x8 qf[36];
  {
    const int64_t row = (int64_t)b * a.R + min(r_own, a.R - 1);
    const __bf16* qrow = a.qabs + row * D_ROW + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 36; ks++) qf[ks] = *(const bf16x8*)(qrow + 16 * ks);
#pragma unroll
    for (int ks = 0; ks < 36; ks += 4)
      asm volatile("" : "+v"(qf[ks]), "+v"(qf[ks + 1]), "+v"(qf[ks + 2]), "+v"(qf[ks + 3]));
  }

  // The 72 MFMAs of a step's score product: 36 pairs, one k-step each with the two tiles
  // alternating (two accumulation chains).  Latent k-steps are taken in the order
  // ks = 8 hi + k7, k7 outermost: the four k-steps with equal k7 share their address registers
  // (s0 ^ (k7 << 5), one per tile) and differ in the immediate offset, so a fragment costs one
  // LDS instruction and no address arithmetic.  Fragments travel through a ring of eight
  // registers, six reads ahead; `between(G)` runs behind group G of four MFMAs.
  auto scores = [&](uint32_t sbase, f32x16 (&sacc)[2], auto&& between) __attribute__((always_inline)) {
    constexpr int NF = 72, AHEAD = 6;
    bf16x8 fr[8];
    uint32_t xa[2] = {0, 0};   // addresses of the k7 group (or rope k-step) being requested
    auto rd = [&](auto i_) __attribute__((always_inline)) {
      constexpr int i = decltype(i_)::value;
      constexpr int P = i >> 1, th = i & 1;
      if constexpr (P < 32) {
        constexpr int k7 = P >> 2, hi = P & 3;
        if constexpr (hi == 0 && th == 0) {
          xa[0] = (sbase + s0_off) ^ (k7 << 5);
          xa[1] = (sbase + A128_TILE_BYTES + s0_off) ^ (k7 << 5);
        }
        fr[i % 8] = lds_read_b128<256 * hi>(xa[th]);
      } else {
        if constexpr (th == 0) xa[0] = (sbase + r0_off) ^ ((P - 32) << 5);
        fr[i % 8] = lds_read_b128<th * A128_TILE_BYTES>(xa[0]);
      }
    };
    static_for<AHEAD>([&](auto i_) { rd(i_); });
    static_for<NF>([&](auto i_) {
      constexpr int i = decltype(i_)::value;
      constexpr int P = i >> 1;
      constexpr int KS = P < 32 ? 8 * (P & 3) + (P >> 2) : P;   // the k-step of this pair
      if constexpr (i + AHEAD < NF) rd(std::integral_constant<int, i + AHEAD>{});
      constexpr int later = NF - 1 - i < AHEAD ? NF - 1 - i : AHEAD;   // younger requests
      if constexpr (i < 2) a128_mfma_s_first_w<later>(sacc[i & 1], fr[i % 8], qf[KS]);
      else a128_mfma_s_w<later>(sacc[i & 1], fr[i % 8], qf[KS]);
      if constexpr (i % 4 == 3) between(std::integral_constant<int, i / 4>{});
    });
    a128_drain();
  };
  // scores of tokens this lane's query must not see -> -inf
  auto mask = [&](int step, f32x16 (&sacc)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int th = 0; th < 2; th++) {
      // element v is token 8 (v / 4) + 4 g + v % 4 of the tile
      const int lim_g = min(32, vis_q - (t0 + step * 64 + th * 32)) - 4 * g;
      if (lim_g < 28) {
#pragma unroll
        for (int v = 0; v < 16; v++)
          if (8 * (v / 4) + v % 4 >= lim_g) sacc[th][v] = -INFINITY;
      }
    }
  };
  auto row_max = [&](const f32x16 (&sacc)[2]) __attribute__((always_inline)) {
    float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
    for (int v = 1; v < 16; v++) mx = fmaxf(mx, fmaxf(sacc[0][v], sacc[1][v]));
    return max_halves(mx) * a.c;
  };

  float m = -INFINITY;   // exponent reference of this lane's query (log2 units)
  float ll[4];           // denominators of column n in the four query blocks

  // A walk over the chunk with references fixed at its start: in the first attempt from step 0
  // (already on its way), in the second (`exact`) the exact maxima.  One copy of the code for
  // both, and the outputs leave in one place behind the loop: with two inlined walks the
  // compiler merges their epilogues and hands 256 accumulation registers over through scratch
  // memory (40 000 cycles per workgroup).
  f32x16 o[8][2];   // [latent block of the own half][query block of the own pair]
  for (int attempt = 0;; attempt++) {
    const bool exact = attempt == 1;
    if (exact) issue_step(0);
#pragma unroll
    for (int mb = 0; mb < 8; mb++)
#pragma unroll
      for (int q = 0; q < 2; q++)
#pragma unroll
        for (int v = 0; v < 16; v++) o[mb][q][v] = 0.f;
#pragma unroll
    for (int mb = 0; mb < 8; mb++) asm volatile("" : "+a"(o[mb][0]), "+a"(o[mb][1]));
    float m_use = (m == -INFINITY) ? 0.f : m;
    float l = 0.f;

    for (int step = 0; step < nstep; step++) {
      vm_wait<0>();
      raw_barrier();   // A
      const bool do_pf = step + 1 < nstep;
      RowSrc pf0, pf1;
      if (do_pf) step_src(step + 1, pf0, pf1);
      const uint32_t pf_dst = smem_base + (((step + 1) & 1) * 2) * A128_TILE_BYTES;
      const uint32_t sbase = smem_base + ((step & 1) * 2) * A128_TILE_BYTES;

      // ---- scores; the next step's transfers one behind every group of four MFMAs
      f32x16 sacc[2];
      scores(sbase, sacc, [&](auto grp) __attribute__((always_inline)) {
        constexpr int G = decltype(grp)::value;
        if (do_pf) {
          if constexpr (G < 9) issue_part(std::integral_constant<int, G>{}, pf0, pf_dst);
          else issue_part(std::integral_constant<int, G - 9>{}, pf1, pf_dst + A128_TILE_BYTES);
        }
      });
      mask(step, sacc);
      if (!exact && step == 0) {
        m = row_max(sacc);
        m_use = (m == -INFINITY) ? 0.f : m;
      }

      // ---- probabilities -> LDS: fragment 2 th + kk holds tokens 16 kk .. + 15 of tile th
      {
        float sum = 0.f;
#pragma unroll
        for (int th = 0; th < 2; th++) {
          bf16x8 p0, p1;
#pragma unroll
          for (int v = 0; v < 8; v++) {
            const float p = fast_exp2(__builtin_fmaf(sacc[th][v], a.c, -m_use));
            sum += p;
            p0[v] = (__bf16)p;
          }
#pragma unroll
          for (int v = 0; v < 8; v++) {
            const float p = fast_exp2(__builtin_fmaf(sacc[th][8 + v], a.c, -m_use));
            sum += p;
            p1[v] = (__bf16)p;
          }
          if (th == 0) {
            const uint32_t p_wr = smem_base + A128_P_OFF + qb * 4096 + lane16;
            lds_write_b128<0>(p_wr, p0);
            lds_write_b128<1024>(p_wr, p1);
          } else {
            const uint32_t p_wr = smem_base + A128_P_OFF + qb * 4096 + lane16;
            lds_write_b128<2048>(p_wr, p0);
            lds_write_b128<3072>(p_wr, p1);
          }
        }
        l += sum;
        // (pinned: otherwise the additions sink behind the output product, with all 32
        // probabilities kept in registers until then)
        asm volatile("" : "+v"(l));
      }
      // Transposed cache fragments: one group per latent block mb (4 k-steps, lo and hi half
      // each), double buffered.  The first group does not depend on the probabilities and is
      // requested before barrier C (the probability writes were issued earlier and complete
      // first); the requests of group mb + 1 are dealt out one behind every MFMA of group mb, so
      // that no burst of LDS instructions keeps the wavefront from feeding the matrix core.
      const uint32_t va = sbase + v_lo, vh = (va + 8192) ^ 32;
      short4v trf[2][8];   // [buffer][2 ks + half]
      auto rdv = [&](auto mb_, auto r_) __attribute__((always_inline)) {
        constexpr int MB = decltype(mb_)::value;
        constexpr int R = decltype(r_)::value;
        constexpr int ks = R >> 1, thp = ks >> 1, kk = ks & 1;
        constexpr int off = thp * A128_TILE_BYTES + kk * 16384 + 256 * (MB >> 2);
        trf[MB & 1][R] = lds_read_tr16_b64<off>(((R & 1) ? vh : va) ^ ((MB & 3) << 6));
      };
      static_for<8>([&](auto r_) { rdv(std::integral_constant<int, 0>{}, r_); });
      lgkm_wait<8>();
      raw_barrier();   // C

      // ---- outputs: own latent half, all 64 tokens, own pair of query blocks
      {
        // k-step ks = 2 * th + kk; probability fragments [ks][query block of the pair]
        bf16x8 pf[4][2];
        const uint32_t p_rd = smem_base + A128_P_OFF + (2 * qp) * 4096 + lane16;
        static_for<4>([&](auto ks_) {
          constexpr int ks = decltype(ks_)::value;
          pf[ks][0] = lds_read_b128<ks * 1024>(p_rd);
          pf[ks][1] = lds_read_b128<4096 + ks * 1024>(p_rd);
        });
        static_for<4>([&](auto ks_) {
          constexpr int ks = decltype(ks_)::value;
          lgkm_wait<0>(pf[ks][0], pf[ks][1]);
        });
        static_for<8>([&](auto mb_) {
          constexpr int mb = decltype(mb_)::value;
          constexpr int cur = mb & 1;
          static_for<8>([&](auto i_) {
            constexpr int i = decltype(i_)::value;   // MFMA i: k-step i / 2, query block i % 2
            constexpr int ks = i >> 1, q = i & 1;
            // requests behind those of fragment ks: 6 - 2 ks of this group, i of the next
            constexpr int later = mb + 1 < 8 ? 6 : 6 - 2 * ks;
            if constexpr (q == 0)
              a128_mfma_o_w<later>(o[mb][q], join_tr(trf[cur][2 * ks], trf[cur][2 * ks + 1]), pf[ks][q]);
            else
              a128_mfma_o(o[mb][q], join_tr(trf[cur][2 * ks], trf[cur][2 * ks + 1]), pf[ks][q]);
            if constexpr (mb + 1 < 8) rdv(std::integral_constant<int, mb + 1>{}, i_);
          });
        });
      }
      // (behind the loop the register allocator may store accumulators to scratch right away;
      // the last MFMAs must have written them by then)
      if (step + 1 == nstep) a128_drain();
    }

    // ---- denominators: the score owners publish theirs, everybody reads all four blocks
    raw_barrier();   // everyone is past its last read of the probabilities
    {
      const float lt = sum_halves(l);
      if (g == 0) lbuf[qb * 32 + n] = lt;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; q++) ll[q] = lbuf[q * 32 + n];
    __syncthreads();   // read before the next walk (or nothing) writes the region again
    if (exact) break;
    // a denominator that is not a moderate finite number: the references did not hold.  Every
    // wavefront reads the same four vectors, so the verdict is the same in all of them.
    {
      const bool bad = !(ll[0] < 0x1p100f) || !(ll[1] < 0x1p100f) || !(ll[2] < 0x1p100f) ||
                       !(ll[3] < 0x1p100f);
      if (__builtin_amdgcn_ballot_w64(bad) == 0) break;
    }
    // exact maxima of every query over the chunk: scores-only pass, one step at a time
    float mx = -INFINITY;
    for (int step = 0; step < nstep; step++) {
      raw_barrier();   // everyone is done with the tiles of the step before
      issue_step(step);
      vm_wait<0>();
      raw_barrier();
      f32x16 sacc[2];
      scores(smem_base + ((step & 1) * 2) * A128_TILE_BYTES, sacc, [](auto) {});
      mask(step, sacc);
      mx = fmaxf(mx, row_max(sacc));
    }
    m = mx;
    raw_barrier();
  }

  {
    // Outputs, normalised, go out through LDS (the tiles are no longer needed): a lane holds
    // 8-byte pieces of its query's row, 16 bytes apart from its neighbour's; turned around, 32
    // lanes write the 512 bytes a row has in this wavefront's latent half in one piece.  Rows
    // whose denominator is zero get zeros (their LSE says that nothing is there).
    constexpr int ST_ROW = 528;   // 512 + 16: rows stay 16-byte aligned
    char* mine = smem + wave * (32 * ST_ROW);
    const int rr = lane >> 5, ch = lane & 31;
#pragma unroll
    for (int q = 0; q < 2; q++) {
      const float lt = ll[2 * qp + q];
      const float inv = lt > 0.f ? 1.f / lt : 0.f;
#pragma unroll
      for (int mb = 0; mb < 8; mb++)
#pragma unroll
        for (int v4 = 0; v4 < 4; v4++) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; e++) w[e] = (__bf16)(o[mb][q][4 * v4 + e] * inv);
          *(bf16x4*)(mine + n * ST_ROW + (32 * mb + 8 * v4 + 4 * g) * 2) = w;
        }
      // (each wavefront reads back only what it wrote itself: no barrier)
      const int row0 = (qg * 4 + 2 * qp + q) * 32;
#pragma unroll
      for (int i = 0; i < 16; i++) {
        const int r = 2 * i + rr;
        const bf16x8 w = *(const bf16x8*)(mine + r * ST_ROW + ch * 16);
        if (row0 + r < a.R)
          *(bf16x8*)(a.lat_o + ((size_t)item * a.rows + (int64_t)b * a.R + row0 + r) * D_L +
                     256 * lh + ch * 8) = w;
      }
    }
    if (g == 0 && r_own < a.R) {
      const float lt = ll[qb];
      a.lat_lse[(size_t)item * a.rows + (int64_t)b * a.R + r_own] =
          lt > 0.f ? (m + fast_log2(lt)) * LN2 : -INFINITY;
    }
  }
}

int mfma_absorb128_attention(const Plan& p, const DecodeArgs& d, const AbsorbArgs& a) {
  static LdsOptIn lds[2];
  auto kernel = a.ap_chunks > 0 ? absorb128_kernel<true> : absorb128_kernel<false>;
  if (lds[a.ap_chunks > 0].ensure((const void*)kernel, A128_LDS_BYTES) != hipSuccess) return TMLA_ERR_HIP;
  Absorb128Args args;
  args.a = a;
  args.nqg = (a.R + 127) / 128;
  args.n_lat = p.n_lat;
  args.B = p.B;
  const long long units = (long long)p.n_lat * p.B;
  const long long wgs = 8LL * args.nqg * ((units + 7) / 8);
  if (wgs > 0x7fffffffLL) return TMLA_ERR_UNSUPPORTED;
  args.a.order = suffix_request_order(p, d, wgs);
  hipLaunchKernelGGL(kernel, dim3((unsigned)wgs), dim3(256), A128_LDS_BYTES, d.stream, args);
  return TMLA_OK;
}

}  // namespace tmla
