// Absorb-formulation flash-decode over latent cache rows for requests with more than 32 query
// rows (S_q * H > 32; paper Algorithm 1 step 6): 64 query rows per workgroup, 64 tokens per step.
//
// The two matrix products of a step want different work splits, so the four wavefronts change
// roles inside a step and hand the probabilities over through LDS:
//   scores   S^T = C Q_abs^T : wavefront (qb, th) takes query block qb (32 rows) and token half th
//            (32 of the step's 64 tokens): 36 MFMAs, every score computed exactly once;
//   outputs  O^T += C_N^T P^T: wavefront w takes latent columns [128 w, 128 w + 128) for all 64
//            queries and all 64 tokens, so each transposed cache fragment read from LDS feeds
//            two MFMAs (one per query block): 32 MFMAs for 32 transposing reads.
// The LDS, not the matrix cores, bounds this kernel.  Cycle stamps per step (64 rows x 64 tokens,
// 68 MFMAs per wavefront): score product ~1000 cycles (one 1 KiB fragment per MFMA), exponentials
// and hand-over ~900, output product ~1350, barriers ~400 -- and the 72 global-to-LDS transfers of
// the next step's tiles add ~1900 more wherever in the step they are issued (spread over the
// score MFMAs, taken in turns by the wavefronts, or all inside the exponentials phase): a
// transfer occupies the LDS for ~26 cycles per KiB while the fragment reads wait.  Hence the care
// to read each fragment once and the conflict-free tile layout.
//
// One step:
//   barrier A   the step's two tiles have landed; everyone is done with the previous step
//   scores of the own (query block, token half), local row maxima -> LDS; the transfers of the
//   next step are issued between the MFMAs
//   barrier B   all four maxima vectors visible: every wavefront derives the same new exponent
//   references for both query blocks (lazy update, see tmla_mfma.hpp), rescales what it owns,
//   exponentiates its scores and writes them as bf16 B-operand fragments -> LDS
//   barrier C   every wavefront reads the 8 probability fragments (4 k-steps x 2 query blocks)
//   and accumulates its latent quarter.
// The denominators stay split by token half until the end and are summed through LDS.
//
// The chunk is first walked with FIXED exponent references: they are set once, to the maxima of
// step 0, so from step 1 on the maxima, their exchange, barrier B and the rescale all disappear
// (the result does not depend on the reference, only the float range does: scores about 2^7
// log2-units above the first step's maximum overflow).  If the denominators end up outside a
// moderate finite range, the workgroup walks the chunk again with the lazy moving references
// described above.
#include "tmla_absorb_tile.hpp"

namespace tmla {

constexpr int A64_P_BYTES = 4 * 2048;                      // probability fragments [wave][kk][lane]
constexpr int A64_P_OFF = AB_NSLOT * AB_TILE_BYTES;        // 155648
constexpr int A64_LDS_BYTES = A64_P_OFF + A64_P_BYTES;     // 163840 = all of LDS
// row maxima [query n][wave]: 16 bytes behind the chunks of row n of ring slot 0, which no
// transfer writes
constexpr int A64_MAX_OFF = 1024;
static_assert(AB_ROW_BYTES >= A64_MAX_OFF + 16 && A64_LDS_BYTES <= 163840, "LDS layout");

struct Absorb64Args {
  AbsorbArgs a;
  int nqg, n_lat, B;
  int moving_only;   // debug: skip the walk with fixed references
};

// HAS_PREFIX: the launch has work items over the shared latent prefix (absorb_only mode).  Those
// rows are read by every request and must stay cached, and a per-transfer choice of the cache
// policy is a branch in the hot loop (-13 % at 64 heads), so such a launch uses ordinary
// transfers throughout; a launch over suffix rows alone streams them with the non-temporal hint.
template <bool HAS_PREFIX>
__global__ void __launch_bounds__(256, 1) absorb64_kernel(Absorb64Args args) {
  const AbsorbArgs& a = args.a;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // Workgroups that read the same tokens (the query groups of one request chunk) get ids 8 apart:
  // hardware deals consecutive ids round-robin over the 8 XCDs, so they share an L2 and run at
  // the same time, and the second reader of a tile finds it there.
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
  const int qb = wave & 1, th = wave >> 1;

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
  // lane (n, g) of wavefront (qb, th) scores query row r_own; when it accumulates outputs it
  // holds rows r_blk[0], r_blk[1] (column n of either query block)
  const int r_own = (qg * 2 + qb) * 32 + n;
  int vis_q = t1;
  if (!is_prefix) {
    const int s = r_own < a.R ? r_own / a.H : 0;
    vis_q = max(0, min(len, len - a.Sq + s + 1));
  }
  if (t1 <= t0) {   // empty chunk (workgroup-uniform): only the LSEs are defined
    if (th == 0 && g == 0 && r_own < a.R)
      a.lat_lse[(size_t)item * a.rows + (int64_t)b * a.R + r_own] = -INFINITY;
    return;
  }
  const int nstep = (t1 - t0 + 63) / 64;

  // ---- tile streaming: global -> LDS (see tmla_absorb_tile.hpp)
  const int32_t* bt = a.block_table + (size_t)b * a.max_blocks;
  const int first_blk = is_prefix ? 0 : t0 / a.block_size;
  int bt_cache = 0;
  if (!is_prefix) {
    const int nblk_chunk = (t1 - 1) / a.block_size - first_blk + 1;
    bt_cache = (lane < nblk_chunk) ? bt[first_blk + lane] : 0;
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(bt_cache)::"memory");
  }
  const DmaLane dl = dma_lane(wave, lane);
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

  // per-lane LDS byte offsets inside a tile (layout in tmla_absorb_tile.hpp)
  const uint32_t smem_base = lds_addr(smem);
  const TileLane tl = tile_lane(lane);
  const uint32_t v_lo = tl.v_lo + 256 * wave, v_hi = tl.v_hi + 256 * wave;   // own latent quarter
  const uint32_t p_wr = smem_base + A64_P_OFF + wave * 2048 + lane * 16;
  const uint32_t p_rd = smem_base + A64_P_OFF + lane * 16;
  const uint32_t mx_rd = smem_base + n * AB_ROW_BYTES + A64_MAX_OFF;
  const uint32_t mx_wr = mx_rd + wave * 4;

  // ---- absorbed query fragments of the own query block (B operand of the score product),
  // staged like cache tiles in slots 2 and 3 while step 0 streams into slots 0 and 1
  {
    const int64_t req_row0 = (int64_t)b * a.R;
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int blk_row0 = (qg * 2 + j) * 32;
      RowSrc qs;
      qs.stream = false;
      qs.last = min(31, a.R - 1 - blk_row0);
      int64_t first = req_row0 + blk_row0;
      if (qs.last < 0) {   // block entirely past the request's rows: any valid row will do
        qs.last = 0;
        first = req_row0 + a.R - 1;
      }
      qs.lat = (const char*)(a.qabs + first * D_ROW);
      qs.rope = qs.lat + D_L * 2;
      qs.lat_stride = qs.rope_stride = D_ROW * 2;
      issue_all(qs, smem + (2 + j) * AB_TILE_BYTES, dl);
    }
  }
  {
    RowSrc s0, s1;
    step_src(0, s0, s1);
    issue_all(s0, smem, dl);
    issue_all(s1, smem + AB_TILE_BYTES, dl);
  }
  vm_wait<2 * AB_DMA_PER_WAVE>();
  raw_barrier();
  bf16x8 qf[36];
  {
    const uint32_t qa = smem_base + (2 + qb) * AB_TILE_BYTES;
    static_for<32>([&](auto ks) {
      qf[decltype(ks)::value] = tile_score_frag<decltype(ks)::value>(qa, tl);
    });
    static_for<4>([&](auto k) {
      qf[32 + decltype(k)::value] = lds_read_b128<0>(qa + tl.r_off[decltype(k)::value]);
    });
#pragma unroll
    for (int ks = 0; ks < 36; ks += 4)
      lgkm_wait<0>(qf[ks], qf[ks + 1], qf[ks + 2], qf[ks + 3]);
  }
  // (barrier A of step 0 also tells that every wavefront has its fragments: slots 2, 3 are free)

  // A walk over the chunk: the first attempt with fixed references (unless the debug switch asks
  // for moving ones), its step 0 already on its way (issued above with the query blocks); a
  // second one with moving references if the fixed ones did not hold.  One copy of the code for
  // both and one epilogue behind the loop (written as a lambda inlined once per variant, every
  // trip around the step loop and the hand-over of the accumulators to the merged epilogues
  // cost extra).
  f32x16 o[4][2];   // [latent block of the own quarter][query block]
  float m[2];       // exponent references of column n in either query block
  f32x4 ll;         // denominators [query block + 2 * token half] of column n
  for (int attempt = 0;; attempt++) {
    const bool fixed = attempt == 0 && !args.moving_only;
    if (attempt > 0) {
      RowSrc s0, s1;
      step_src(0, s0, s1);
      issue_all(s0, smem, dl);
      issue_all(s1, smem + AB_TILE_BYTES, dl);
    }
  #pragma unroll
    for (int mb = 0; mb < 4; mb++)
  #pragma unroll
      for (int q = 0; q < 2; q++)
  #pragma unroll
        for (int v = 0; v < 16; v++) o[mb][q][v] = 0.f;
    m[0] = m[1] = -INFINITY;
    float m_use[2] = {0.f, 0.f};           // the same, 0 where no token is visible
    float l = 0.f;                         // denominator part: own query block, own token half

    for (int step = 0; step < nstep; step++) {
      vm_wait<0>();
      raw_barrier();   // A
      const bool do_pf = step + 1 < nstep;
      RowSrc pf0, pf1;
      if (do_pf) step_src(step + 1, pf0, pf1);
      char* pf_dst = smem + (((step + 1) & 1) * 2) * AB_TILE_BYTES;
      const uint32_t sbase = smem_base + ((step & 1) * 2) * AB_TILE_BYTES;   // the step's two tiles

      // ---- scores: own token half, own query block
      const uint32_t tbase = sbase + th * AB_TILE_BYTES;
      f32x16 sacc;
  #pragma unroll
      for (int v = 0; v < 16; v++) sacc[v] = 0.f;
      {
        // 9 groups of 4 k-steps (the last one is the rope part); three fragment buffers in
        // rotation keep two groups of LDS reads in flight behind the one feeding the MFMAs
        bf16x8 f[3][4];
        auto rd = [&](auto gsel, auto dsel) __attribute__((always_inline)) {
          constexpr int G = decltype(gsel)::value;
          constexpr int D = decltype(dsel)::value;
          if constexpr (G < 8) {
            static_for<4>([&](auto j) {
              f[D][j] = tile_score_frag<4 * G + decltype(j)::value>(tbase, tl);
            });
          } else {
            static_for<4>([&](auto j) {
              f[D][j] = lds_read_b128<0>(tbase + tl.r_off[decltype(j)::value]);
            });
          }
        };
        rd(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        rd(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{});
        static_for<9>([&](auto grp) {
          constexpr int G = decltype(grp)::value;
          constexpr int cur = G % 3;
          if constexpr (G + 2 < 9) {
            rd(std::integral_constant<int, G + 2>{}, std::integral_constant<int, (G + 2) % 3>{});
            lgkm_wait<8>(f[cur][0], f[cur][1], f[cur][2], f[cur][3]);
          } else if constexpr (G + 1 < 9) {
            lgkm_wait<4>(f[cur][0], f[cur][1], f[cur][2], f[cur][3]);
          } else {
            lgkm_wait<0>(f[cur][0], f[cur][1], f[cur][2], f[cur][3]);
          }
          static_for<4>([&](auto j) {
            sacc = mfma32(f[cur][j], qf[4 * G + decltype(j)::value], sacc);
          });
          // The next step's transfers.  A transfer holds up the issuing wavefront while the
          // memory pipeline takes it, and longer when other wavefronts present theirs at the same
          // time, so the wavefronts take turns: wavefront w issues in groups w and w + 4 (a whole
          // tile each), wavefront 0, which has three groups (0, 4, 8), a third of its 18 in each.
          if (do_pf) {
            if constexpr (G == 0 || G == 4 || G == 8) {
              if (wave == 0) {
                static_for<6>([&](auto i_) {
                  constexpr int k = (G / 4) * 6 + decltype(i_)::value;   // 0 .. 17
                  if constexpr (k < 9) issue_part<k>(pf0, pf_dst, dl);
                  else issue_part<k - 9>(pf1, pf_dst + AB_TILE_BYTES, dl);
                });
              }
            } else if constexpr (G < 4) {
              if (wave == G) issue_all(pf0, pf_dst, dl);
            } else {
              if (wave == G - 4) issue_all(pf1, pf_dst + AB_TILE_BYTES, dl);
            }
          }
        });
      }

      // ---- local maxima -> LDS
      const int limit = min(32, vis_q - (t0 + step * 64 + th * 32));
      if (limit < 32) {
  #pragma unroll
        for (int v = 0; v < 16; v++)
          if (acc_row(v, g) >= limit) sacc[v] = -INFINITY;
      }
      if (!fixed || step == 0) {
        {
          float mx = sacc[0];
#pragma unroll
          for (int v = 1; v < 16; v++) mx = fmaxf(mx, sacc[v]);
          mx = max_halves(mx) * a.c;
          if (g == 0) lds_write_b32(mx_wr, mx);
        }
        lgkm_wait<0>();
        raw_barrier();   // B

        // ---- common exponent references
        f32x4 mm = lds_read_f32x4(mx_rd);   // [wave] = [qb + 2 * th]
        lgkm_wait<0>(mm);
        float alpha[2];
        bool grow = false;
#pragma unroll
        for (int q = 0; q < 2; q++) {
          const float bm = fmaxf(mm[q], mm[q + 2]);
          const float m_new = (bm > m[q] + RESCALE_TAU) ? bm : m[q];
          m_use[q] = (m_new == -INFINITY) ? 0.f : m_new;
          grow = grow || (m_new > m[q]);
          alpha[q] = m[q] - m_use[q];   // exponent of the rescale factor (m = -inf -> factor 0)
          m[q] = m_new;
        }
        // (in step 0 every accumulator is still zero: nothing to rescale)
        if (!fixed && step > 0 && __builtin_amdgcn_ballot_w64(grow) != 0) {
          alpha[0] = fast_exp2(alpha[0]);
          alpha[1] = fast_exp2(alpha[1]);
          l *= alpha[qb];
#pragma unroll
          for (int mb = 0; mb < 4; mb++)
#pragma unroll
            for (int q = 0; q < 2; q++) {
              // the accumulators live in accumulation registers, which the vector ALU cannot
              // address; routing them through this statement keeps their copies inside the rare
              // branch (otherwise the copies out are hoisted and run in every step)
              asm volatile("" : "+a"(o[mb][q]));
#pragma unroll
              for (int v = 0; v < 16; v++) o[mb][q][v] *= alpha[q];
              asm volatile("" : "+a"(o[mb][q]));
            }
        }
      }
      // ---- probabilities -> LDS
      {
        const float mu = m_use[qb];
        bf16x8 p0, p1;
        float sum = 0.f;
  #pragma unroll
        for (int v = 0; v < 8; v++) {
          const float p = fast_exp2(__builtin_fmaf(sacc[v], a.c, -mu));
          sum += p;
          p0[v] = (__bf16)p;
        }
  #pragma unroll
        for (int v = 0; v < 8; v++) {
          const float p = fast_exp2(__builtin_fmaf(sacc[8 + v], a.c, -mu));
          sum += p;
          p1[v] = (__bf16)p;
        }
        l += sum;
        lds_write_b128<0>(p_wr, p0);
        lds_write_b128<1024>(p_wr, p1);
      }
      // the first group of transposed cache fragments does not depend on the probabilities: it is
      // requested before barrier C (the probability writes were issued earlier and complete first)
      const uint32_t va = sbase + v_lo, vh = sbase + v_hi;
      short4v lo[2][4], hi[2][4];
      auto rdv = [&](auto grp_, auto buf_) __attribute__((always_inline)) {
        constexpr int G = decltype(grp_)::value;   // = mb
        constexpr int D = decltype(buf_)::value;
        static_for<4>([&](auto ks_) {
          constexpr int ks = decltype(ks_)::value;
          constexpr int thp = ks >> 1, kk = ks & 1;
          constexpr int off = thp * AB_TILE_BYTES + (16 * kk) * AB_ROW_BYTES + 64 * G;
          lo[D][ks] = lds_read_tr16_b64<off>(va);
          hi[D][ks] = lds_read_tr16_b64<off>(vh);
        });
      };
      rdv(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
      lgkm_wait<8>();
      raw_barrier();   // C

      // ---- outputs: own latent quarter, all 64 tokens, both query blocks
      {
        // k-step ks = 2 * th' + kk: 16 tokens of tile th'; probability fragments [ks][query block]
        bf16x8 pf[4][2];
        static_for<4>([&](auto ks_) {
          constexpr int ks = decltype(ks_)::value;
          constexpr int thp = ks >> 1, kk = ks & 1;
          pf[ks][0] = lds_read_b128<(0 + 2 * thp) * 2048 + kk * 1024>(p_rd);
          pf[ks][1] = lds_read_b128<(1 + 2 * thp) * 2048 + kk * 1024>(p_rd);
        });
        // transposed cache fragments: one group per latent block mb (4 k-steps, 8 reads), double
        // buffered; each fragment feeds the MFMAs of both query blocks
        static_for<4>([&](auto ks_) {
          constexpr int ks = decltype(ks_)::value;
          lgkm_wait<0>(pf[ks][0], pf[ks][1]);
        });
        static_for<4>([&](auto mb_) {
          constexpr int mb = decltype(mb_)::value;
          constexpr int cur = mb & 1, nxt = cur ^ 1;
          if constexpr (mb + 1 < 4) {
            rdv(std::integral_constant<int, mb + 1>{}, std::integral_constant<int, nxt>{});
            lgkm_wait<8>(lo[cur][0], lo[cur][1], lo[cur][2], lo[cur][3]);
            lgkm_wait<8>(hi[cur][0], hi[cur][1], hi[cur][2], hi[cur][3]);
          } else {
            lgkm_wait<0>(lo[cur][0], lo[cur][1], lo[cur][2], lo[cur][3]);
            lgkm_wait<0>(hi[cur][0], hi[cur][1], hi[cur][2], hi[cur][3]);
          }
          static_for<4>([&](auto ks_) {
            constexpr int ks = decltype(ks_)::value;
            const bf16x8 af = join_tr(lo[cur][ks], hi[cur][ks]);
            o[mb][0] = mfma32(af, pf[ks][0], o[mb][0]);
            o[mb][1] = mfma32(af, pf[ks][1], o[mb][1]);
          });
        });
      }
    }

    // ---- denominators: sum the two token halves of either query block through LDS
    raw_barrier();   // everyone is past its last read of the maxima buffer
    {
      const float lh = sum_halves(l);
      if (g == 0) lds_write_b32(mx_wr, lh);
    }
    lgkm_wait<0>();
    raw_barrier();
    ll = lds_read_f32x4(mx_rd);
    lgkm_wait<0>(ll);
    if (!fixed) break;
    // a denominator that is not a moderate finite number: the fixed references did not hold.
    // Every wavefront reads the same four vectors, so the verdict is the same in all of them.
    const bool bad = !(ll[0] + ll[2] < 0x1p100f) || !(ll[1] + ll[3] < 0x1p100f);
    if (__builtin_amdgcn_ballot_w64(bad) == 0) break;
    raw_barrier();   // everyone has read the denominators before the next walk's maxima land there
  }
  {
  #pragma unroll
    for (int q = 0; q < 2; q++) {
      const int r_local = (qg * 2 + q) * 32 + n;
      if (r_local >= a.R) continue;
      const int64_t row = (int64_t)b * a.R + r_local;
      const float lt = ll[q] + ll[q + 2];
      float* l_dst = a.lat_lse + (size_t)item * a.rows + row;
      if (lt > 0.f) {
        const float inv = 1.f / lt;
        __bf16* o_dst = a.lat_o + ((size_t)item * a.rows + row) * D_L + 128 * wave + 4 * g;
  #pragma unroll
        for (int mb = 0; mb < 4; mb++)
  #pragma unroll
          for (int v4 = 0; v4 < 4; v4++) {
            bf16x4 w;
  #pragma unroll
            for (int e = 0; e < 4; e++) w[e] = (__bf16)(o[mb][q][4 * v4 + e] * inv);
            *(bf16x4*)(o_dst + 32 * mb + 8 * v4) = w;
          }
        if (wave == q && g == 0) *l_dst = (m[q] + fast_log2(lt)) * LN2;
      } else if (wave == q && g == 0) {
        *l_dst = -INFINITY;   // the causal mask hid every token of this chunk from this query
      }
    }
  }
}

int mfma_absorb64_attention(const Plan& p, const DecodeArgs& d, const AbsorbArgs& a) {
  static LdsOptIn lds[2];
  auto kernel = a.ap_chunks > 0 ? absorb64_kernel<true> : absorb64_kernel<false>;
  if (lds[a.ap_chunks > 0].ensure((const void*)kernel, A64_LDS_BYTES) != hipSuccess) return TMLA_ERR_HIP;
  Absorb64Args args;
  args.a = a;
  args.nqg = (a.R + 63) / 64;
  args.n_lat = p.n_lat;
  args.B = p.B;
  args.moving_only = (debug_flags() & 0x800) != 0;
  const long long units = (long long)p.n_lat * p.B;
  const long long wgs = 8LL * args.nqg * ((units + 7) / 8);
  if (wgs > 0x7fffffffLL) return TMLA_ERR_UNSUPPORTED;
  args.a.order = suffix_request_order(p, d, wgs);
  hipLaunchKernelGGL(kernel, dim3((unsigned)wgs), dim3(256), A64_LDS_BYTES, d.stream, args);
  return TMLA_OK;
}

}  // namespace tmla
