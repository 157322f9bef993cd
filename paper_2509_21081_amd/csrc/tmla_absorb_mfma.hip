// Absorb-formulation flash-decode over latent cache rows on the matrix cores
// (paper Algorithm 1 step 6; the absorbed queries of step 5 arrive precomputed, the W_UV
// up-projection of step 7 is applied after the split partials are merged because it is linear).
//
// One workgroup = one request x one token chunk x up to 128 of its S_q*H query rows.  Each
// 576-wide cache row is read from HBM once per workgroup (fully coalesced 1152-byte rows) into
// an LDS tile of 32 tokens, and serves both products:
//   S^T  = C   Q_abs^T   (tokens x queries, k = 576): A operand = token-major rows (ds_read_b128)
//   O^T += C_N^T P^T     (latent x queries, k = tokens): A operand = the same tile read through
//                         the transposing LDS load (ds_read_b64_tr_b16), no second copy.
// Queries sit on the MFMA column axis, so softmax statistics are per-lane and P^T feeds the second
// product straight from the accumulator registers.
//
// Wavefront roles (template NQB = query blocks of 32 rows per workgroup, NQB * NLP = 4):
//   NQB = 4: four wavefronts own 4 x 32 query rows and all 512 latent columns each (not built:
//            it needs more registers than a wavefront has)
//   NQB = 2: 2 x 32 query rows, two wavefronts per block own 256 latent columns each
//   NQB = 1: 32 query rows (H = 16 with S_q <= 2), four wavefronts own 128 latent columns each;
//            the scores are recomputed per wavefront, which the HBM-bound small-H case affords.
#include <type_traits>
#include <utility>

#include "tmla_absorb_tile.hpp"

namespace tmla {

// HAS_PREFIX: the launch has work items over the shared latent prefix (absorb_only mode); then
// every transfer is an ordinary one (see the 64-row kernel), else the suffix rows are streamed.
template <int NQB, bool HAS_PREFIX>
__global__ void __launch_bounds__(256, 1) absorb_attn_kernel(AbsorbArgs a) {
  constexpr int NLP = 4 / NQB;
  constexpr int MBW = 16 / NLP;  // 32-latent blocks owned by a wavefront
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int item = blockIdx.x, qg = blockIdx.y;
  const int b = a.order ? a.order[blockIdx.z] : blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: transfer bookkeeping is SALU
  const int qb = wave % NQB, lp = wave / NQB;
  const int r_local = (qg * NQB + qb) * 32 + n;   // this lane's query row within the request
  const bool q_valid = r_local < a.R;
  const int64_t row = (int64_t)b * a.R + r_local; // global output row (b, s, h)

  // ---- which tokens
  int t0, t1, vis_q;
  const bool is_prefix = HAS_PREFIX && item < a.ap_chunks;
  if (is_prefix) {
    t0 = item * a.ap_chunk;
    t1 = min(a.Ls, t0 + a.ap_chunk);
    vis_q = t1;
  } else {
    const int len = a.lens[b];
    t0 = (item - a.ap_chunks) * a.as_chunk;
    t1 = min(len, t0 + a.as_chunk);
    const int s = q_valid ? r_local / a.H : 0;
    vis_q = max(0, min(len, len - a.Sq + s + 1));
  }
  __bf16* o_dst = a.lat_o + ((size_t)item * a.rows + row) * D_L;
  float* l_dst = a.lat_lse + (size_t)item * a.rows + row;
  if (t1 <= t0) {   // empty chunk (workgroup-uniform)
    if (q_valid && lp == 0 && g == 0) *l_dst = -INFINITY;
    return;
  }
  const int ntile = (t1 - t0 + 31) / 32;

  // ---- tile streaming: global -> LDS.
  // The physical blocks of this chunk are fetched once, one entry per lane (a chunk spans at most
  // 64 blocks here, longer ones fall back to a scalar load per tile), and picked with v_readlane:
  // no memory latency on the tile-issue path.
  const int32_t* bt = a.block_table + (size_t)b * a.max_blocks;
  const int first_blk = is_prefix ? 0 : t0 / a.block_size;
  int bt_cache = 0;
  if (!is_prefix) {
    const int nblk_chunk = (t1 - 1) / a.block_size - first_blk + 1;
    bt_cache = (lane < nblk_chunk) ? bt[first_blk + lane] : 0;
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(bt_cache)::"memory");
  }
  const DmaLane dl = dma_lane(wave, lane);
  auto tile_src = [&](int tile) __attribute__((always_inline)) {
    RowSrc s;
    const int tok0 = t0 + tile * 32;
    s.last = t1 - 1 - tok0;              // last valid row of this tile (>= 0)
    s.stream = !HAS_PREFIX;
    if (is_prefix) {
      s.lat = (const char*)a.pc + (size_t)tok0 * (D_L * 2);
      s.rope = (const char*)a.pr + (size_t)tok0 * (D_R * 2);
      s.lat_stride = D_L * 2;
      s.rope_stride = D_R * 2;
    } else {
      const int bi = __builtin_amdgcn_readfirstlane(tok0 / a.block_size - first_blk);
      const int blk = bi < 64 ? __builtin_amdgcn_readlane(bt_cache, bi)
                              : scalar_load_i32(bt + first_blk + bi);
      s.lat = (const char*)(a.pool + ((size_t)blk * a.block_size + tok0 % a.block_size) * D_ROW);
      s.rope = s.lat + D_L * 2;
      s.lat_stride = s.rope_stride = D_ROW * 2;
    }
    return s;
  };
  auto slot_ptr = [&](int tile) __attribute__((always_inline)) {
    return smem + (tile % AB_NSLOT) * AB_TILE_BYTES;
  };

  // per-lane LDS byte offsets inside a tile (tmla_absorb_tile.hpp)
  const uint32_t smem_base = lds_addr(smem);
  const TileLane tl = tile_lane(lane);
  const uint32_t v_lo = tl.v_lo + 64 * (lp * MBW), v_hi = tl.v_hi + 64 * (lp * MBW);

  // ---- absorbed query fragments (B operand): 36 k-steps of 16.
  // The NQB blocks of 32 absorbed-query rows are staged like cache tiles (same transfers, same
  // layout) in the last NQB ring slots, and every wavefront picks its block's fragments with the
  // score-product read pattern: the rows are fetched once per workgroup with full 1 KiB
  // transfers instead of once per wavefront with 32-byte pieces.  The first tiles of the chunk
  // stream into the other slots meanwhile.
  constexpr int NPRE = AB_NSLOT - NQB;   // tiles issued next to the query blocks
  {
    const int64_t req_row0 = (int64_t)b * a.R;
#pragma unroll
    for (int j = 0; j < NQB; j++) {
      const int blk_row0 = (qg * NQB + j) * 32;
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
      issue_all(qs, smem + (NPRE + j) * AB_TILE_BYTES, dl);
    }
  }
#pragma unroll
  for (int t = 0; t < NPRE; t++)
    if (t < ntile) issue_all(tile_src(t), slot_ptr(t), dl);
  {
    const int pre = min(ntile, NPRE);    // tiles in flight behind the query blocks
    if (pre >= 3) vm_wait<3 * AB_DMA_PER_WAVE>();
    else if (pre == 2) vm_wait<2 * AB_DMA_PER_WAVE>();
    else vm_wait<AB_DMA_PER_WAVE>();
  }
  raw_barrier();
  bf16x8 qf[36];
  {
    const uint32_t qa = smem_base + (NPRE + qb) * AB_TILE_BYTES;
    static_for<32>([&](auto ks) { qf[decltype(ks)::value] = tile_score_frag<decltype(ks)::value>(qa, tl); });
    static_for<4>([&](auto k) { qf[32 + decltype(k)::value] = lds_read_b128<0>(qa + tl.r_off[decltype(k)::value]); });
#pragma unroll
    for (int ks = 0; ks < 36; ks += 4)
      lgkm_wait<0>(qf[ks], qf[ks + 1], qf[ks + 2], qf[ks + 3]);
  }
  raw_barrier();   // the query slots may now be overwritten by tiles
#pragma unroll
  for (int t = NPRE; t < AB_NSLOT - 1; t++)
    if (t < ntile) issue_all(tile_src(t), slot_ptr(t), dl);

  f32x16 o[MBW];
#pragma unroll
  for (int mb = 0; mb < MBW; mb++)
#pragma unroll
    for (int v = 0; v < 16; v++) o[mb][v] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int tile = 0; tile < ntile; tile++) {
    // this wavefront's transfers of `tile` are complete once at most the transfers of the
    // following (up to two) tiles remain in flight
    const int ahead = ntile - 1 - tile;
    if (ahead >= 2) vm_wait<2 * AB_DMA_PER_WAVE>();
    else if (ahead == 1) vm_wait<AB_DMA_PER_WAVE>();
    else vm_wait<0>();
    raw_barrier();   // everyone's part of `tile` has landed; everyone is done with tile - 1
    // The four wavefronts run the same instruction stream; leaving the barrier together they
    // would present their transfers and LDS reads at the same cycle and queue behind each
    // other.  A skew of 32 cycles per wavefront (one MFMA) keeps them apart.
    if (wave & 1) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    if (wave & 2) asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    // the tile three ahead goes into the slot freed by the barrier; its transfers are spread
    // over the score product (one per group of four MFMAs) so that the wavefront never sits
    // behind a full memory-instruction queue
    const int pf = tile + AB_NSLOT - 1;
    const bool do_pf = pf < ntile;
    RowSrc pf_src;
    if (do_pf) pf_src = tile_src(pf);
    char* pf_dst = slot_ptr(pf);

    const uint32_t tbase = smem_base + (tile % AB_NSLOT) * AB_TILE_BYTES;
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
        if (do_pf) issue_part<G>(pf_src, pf_dst, dl);
      });
    }
    const int limit = min(32, vis_q - (t0 + tile * 32));
    bf16x8 p[2];
    bool rescale;
    const float alpha = softmax_block(sacc, m, l, a.c, limit, g, p[0], p[1], rescale);
    if (rescale) {
      // (the asm statements keep the accumulator <-> vector register copies inside this branch)
#pragma unroll
      for (int mb = 0; mb < MBW; mb++) {
        asm volatile("" : "+a"(o[mb]));
#pragma unroll
        for (int v = 0; v < 16; v++) o[mb][v] *= alpha;
        asm volatile("" : "+a"(o[mb]));
      }
    }
    {
      // step st = 2*mb + kk; groups of 4 steps (8 transposing reads), double buffered
      const uint32_t va = tbase + v_lo, vh = tbase + v_hi;
      constexpr int NSTEP = 2 * MBW, NGRP = NSTEP / 4;
      short4v lo[2][4], hi[2][4];
      static_for<4>([&](auto j) {
        constexpr int st = decltype(j)::value;
        constexpr int off = (16 * (st & 1)) * AB_ROW_BYTES + 64 * (st >> 1);
        lo[0][st] = lds_read_tr16_b64<off>(va);
        hi[0][st] = lds_read_tr16_b64<off>(vh);
      });
      static_for<NGRP>([&](auto grp) {
        constexpr int G = decltype(grp)::value;
        constexpr int cur = G & 1, nxt = cur ^ 1;
        if constexpr (G + 1 < NGRP) {
          static_for<4>([&](auto j) {
            constexpr int st = 4 * (G + 1) + decltype(j)::value;
            constexpr int off = (16 * (st & 1)) * AB_ROW_BYTES + 64 * (st >> 1);
            lo[nxt][decltype(j)::value] = lds_read_tr16_b64<off>(va);
            hi[nxt][decltype(j)::value] = lds_read_tr16_b64<off>(vh);
          });
          lgkm_wait<8>(lo[cur][0], lo[cur][1], lo[cur][2], lo[cur][3]);
          lgkm_wait<8>(hi[cur][0], hi[cur][1], hi[cur][2], hi[cur][3]);
        } else {
          lgkm_wait<0>(lo[cur][0], lo[cur][1], lo[cur][2], lo[cur][3]);
          lgkm_wait<0>(hi[cur][0], hi[cur][1], hi[cur][2], hi[cur][3]);
        }
        static_for<4>([&](auto j) {
          constexpr int st = 4 * G + decltype(j)::value;
          o[st >> 1] = mfma32(join_tr(lo[cur][decltype(j)::value], hi[cur][decltype(j)::value]),
                              p[st & 1], o[st >> 1]);
        });
      });
    }
  }

  const float lt = sum_halves(l);
  if (!q_valid) return;
  if (lt > 0.f) {
    const float inv = 1.f / lt;
#pragma unroll
    for (int mb = 0; mb < MBW; mb++)
#pragma unroll
      for (int v4 = 0; v4 < 4; v4++) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; e++) w[e] = (__bf16)(o[mb][4 * v4 + e] * inv);
        *(bf16x4*)(o_dst + 32 * (lp * MBW + mb) + 8 * v4 + 4 * g) = w;
      }
    if (lp == 0 && g == 0) *l_dst = (m + fast_log2(lt)) * LN2;
  } else if (lp == 0 && g == 0) {
    *l_dst = -INFINITY;   // causal mask hid every token of this chunk from this query
  }
}

// rank of every request by (suffix length descending, index ascending); order[rank] = request.
// One wavefront per request: its lanes compare 64 other requests at a time and count
// (a thread per request walking all lengths one by one is bound by the latency of each read:
// 25 us for 512 requests).
__global__ void __launch_bounds__(256) suffix_order_kernel(const int32_t* lens, int B,
                                                           int32_t* order) {
  const int lane = threadIdx.x & 63;
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= B) return;   // wavefront-uniform
  const int mine = lens[b];
  // per-lane counts first (independent loads, several in flight), one reduction at the end
  int rank = 0;
#pragma unroll 8
  for (int i = lane; i < B; i += 64) {
    const int other = lens[i];
    rank += (other > mine || (other == mine && i < b)) ? 1 : 0;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) rank += __shfl_xor(rank, off);
  if (lane == 0) order[rank] = b;
}

// Workgroups are handed to the compute units in index order, each unit taking the next one when
// it is free.  When there are more workgroups than units and the suffix lengths differ, the
// pass ends with a few units working on late long requests while the rest idle; starting the
// longest requests first evens that out.  Debug flags:
// bit 14 orders whatever the grid size, bit 15 never orders.
constexpr int ORDER_MAX_BATCH = 4096;   // the ranking is quadratic in the batch size
const int32_t* suffix_request_order(const Plan& p, const DecodeArgs& d, long long wgs) {
  if (p.as_chunks <= 0 || !d.suffix_lens || p.B < 2 || p.B > ORDER_MAX_BATCH) return nullptr;
  if (debug_flags() & 0x8000) return nullptr;
  if (wgs <= NUM_CU && !(debug_flags() & 0x4000)) return nullptr;
  int32_t* order = (int32_t*)(d.ws + p.off_order);
  hipLaunchKernelGGL(suffix_order_kernel, dim3((p.B + 3) / 4), dim3(256), 0, d.stream,
                     d.suffix_lens, p.B, order);
  return order;
}

int mfma_absorb_attention(const Plan& p, const DecodeArgs& d) {
  if (p.n_lat <= 0 || p.rows == 0) return TMLA_OK;
  if (p.Sq * p.H <= 16) return mfma_absorb16_attention(p, d);
  AbsorbArgs a;
  a.qabs = (const __bf16*)(d.ws + p.off_qabs);
  a.pc = (const __bf16*)d.prefix_ckv;
  a.pr = (const __bf16*)d.prefix_krope;
  a.pool = (const __bf16*)d.suffix_pool;
  a.block_table = d.block_table;
  a.lens = d.suffix_lens;
  a.order = nullptr;
  a.lat_o = (__bf16*)(d.ws + p.off_lat_o);
  a.lat_lse = (float*)(d.ws + p.off_lat_lse);
  a.Sq = p.Sq; a.H = p.H; a.R = p.Sq * p.H; a.Ls = p.Ls;
  a.ap_chunks = p.ap_chunks; a.ap_chunk = p.ap_chunk; a.as_chunk = p.as_chunk;
  a.max_blocks = d.max_blocks; a.block_size = d.block_size;
  a.rows = p.rows;
  a.c = d.sm_scale * LOG2E;
  // 128 rows per workgroup when the request has whole blocks of them and the grid still covers
  // the chip (measured against the 64-row kernel at L_n = 256 ... 4096: 4 to 25 % less time).
  // Debug flags: bit 12 keeps the 64-row kernel, bit 13 takes the 128-row kernel whatever the
  // grid size.
  if (a.R % 128 == 0 && !(debug_flags() & 0x1000) &&
      ((debug_flags() & 0x2000) || (long long)p.n_lat * p.B * (a.R / 128) >= NUM_CU))
    return mfma_absorb128_attention(p, d, a);
  if (a.R > 32) return mfma_absorb64_attention(p, d, a);
  static LdsOptIn lds[2];
  auto kernel = a.ap_chunks > 0 ? absorb_attn_kernel<1, true> : absorb_attn_kernel<1, false>;
  if (lds[a.ap_chunks > 0].ensure((const void*)kernel, AB_LDS_BYTES) != hipSuccess) return TMLA_ERR_HIP;
  dim3 grid(p.n_lat, 1, p.B);
  a.order = suffix_request_order(p, d, (long long)p.n_lat * p.B);
  hipLaunchKernelGGL(kernel, grid, dim3(256), AB_LDS_BYTES, d.stream, a);
  return TMLA_OK;
}

}  // namespace tmla
