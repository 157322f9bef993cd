// Absorb-formulation flash-decode for requests with at most 16 query rows (S_q * H <= 16: one
// tensor-parallel rank's head share), paper Algorithm 1 step 6.  This is the HBM-bound case
// (about 30 FLOP per cache byte), so the design minimises everything except the cache stream:
//
//   * v_mfma_f32_16x16x32_bf16 with the 16 queries on the column axis: no padding to 32 columns;
//   * every wavefront is an independent worker with a private 32-token LDS tile: it streams its
//     own contiguous share of the request's tokens (global -> LDS), reads the tile once for the
//     scores and once (transposed) for P V, and never synchronises with the other wavefronts.
//     Each cache row is therefore read from LDS exactly twice per workgroup, and the latency of
//     a wavefront's tile load is hidden by the other three wavefronts of the compute unit;
//   * the wavefronts of a workgroup cover up to four consecutive plan items (token chunks) of
//     one request; the span is divided evenly among them at run time so that requests shorter
//     than the planned span still use all four.  Each writes its own latent partial + LSE.
//
// MFMA 16x16x32 operand layout (lane = n + 16*q, n in [0,16), q in [0,4)):
//   A (16 x 32): row n, k = 8*q + e;   B (32 x 16): column n, k = 8*q + e;
//   D (16 x 16): column n, rows 4*q + v, v in [0,4).
#include <type_traits>

#include "tmla_common.hpp"
#include "tmla_lds_asm.hpp"
#include "tmla_mfma.hpp"

namespace tmla {

struct Absorb16Args {
  const __bf16* qabs;        // [rows, 576]
  const __bf16* pc;          // prefix latent [Ls, 512]  (absorb_only)
  const __bf16* pr;          // prefix rope   [Ls, 64]
  const __bf16* pool;        // [num_blocks, block_size, 576]
  const int32_t* block_table;
  const int32_t* lens;
  const int32_t* order;      // blockIdx.y -> request, or nullptr (identity)
  __bf16* lat_o;             // [n_lat, rows, 512]
  float* lat_lse;            // [n_lat, rows]
  int Sq, H, R, Ls, ap_chunks, ap_chunk, as_chunks, as_chunk, ap_groups, max_blocks, block_size;
  int64_t rows;
  float c;                   // sm_scale * log2(e)
};

// private tile layout: latent rows at r * 1056 with the 16-byte chunk c in slot
// c ^ ((r >> 3) & 1), then 32 x 128 B of rope with chunk c of row r in slot c ^ ((r >> 1) & 7).
// The LDS has 64 four-byte banks; a 16-byte read is served 16 lanes at a time, an 8-byte
// transposing read 32 lanes at a time.  The row stride is 8 banks mod 64: the transposing reads
// of the output product (8 rows x 32 B per 32 lanes) cover the banks exactly, and the score
// product's 16 rows x 16 B per 16 lanes do so because rows r and r + 8 sit in different halves
// of a 32-byte pair.  Rope rows of equal parity share 32 banks; the swizzle separates the eight
// of them that a 16-lane group reads.
constexpr int A16_ROW_BYTES = 1056;
constexpr int A16_MAIN_BYTES = 32 * A16_ROW_BYTES;
constexpr int A16_TILE_BYTES = A16_MAIN_BYTES + 32 * 128;   // 37888
constexpr int A16_LDS_BYTES = 4 * A16_TILE_BYTES;

__device__ inline f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// max / sum over the four lanes n, n+16, n+32, n+48 (all four end up with the result)
__device__ inline float max_quads(float x) {
  int xi = __float_as_int(x);
  auto r = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
  x = fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
  return max_halves(x);
}
__device__ inline float sum_quads(float x) {
  int xi = __float_as_int(x);
  auto r = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
  x = __int_as_float(r[0]) + __int_as_float(r[1]);
  return sum_halves(x);
}

__global__ void __launch_bounds__(256, 1) absorb16_kernel(Absorb16Args a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int grp = blockIdx.x, b = a.order ? a.order[blockIdx.y] : blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 15, q4 = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool q_valid = n < a.R;
  const int64_t row = (int64_t)b * a.R + n;

  // ---- the span of this workgroup and this wavefront's share of it
  const bool is_prefix = grp < a.ap_groups;
  int first_item, nparts, span0, span1, len = 0;
  if (is_prefix) {
    first_item = 4 * grp;
    nparts = min(4, a.ap_chunks - first_item);
    span0 = first_item * a.ap_chunk;
    span1 = min(a.Ls, span0 + nparts * a.ap_chunk);
  } else {
    const int sg = grp - a.ap_groups;
    len = a.lens[b];
    nparts = min(4, a.as_chunks - 4 * sg);
    span0 = 4 * sg * a.as_chunk;
    span1 = min(len, span0 + nparts * a.as_chunk);
    first_item = a.ap_chunks + 4 * sg;
  }
  if (wave >= nparts) return;   // no barriers below: wavefronts are independent
  const int item = first_item + wave;
  __bf16* o_dst = a.lat_o + ((size_t)item * a.rows + row) * D_L + 4 * q4;
  float* l_dst = a.lat_lse + (size_t)item * a.rows + row;
  const int span = max(0, span1 - span0);
  const int part = ((span + nparts - 1) / nparts + 31) & ~31;   // tokens per wavefront, tile aligned
  const int t0 = __builtin_amdgcn_readfirstlane(span0 + wave * part);
  const int t1 = __builtin_amdgcn_readfirstlane(min(span1, t0 + part));
  int vis_q = t1;
  if (!is_prefix) {
    const int s = q_valid ? n / a.H : 0;
    vis_q = max(0, min(len, len - a.Sq + s + 1));
  }
  if (t1 <= t0) {
    if (q_valid && q4 == 0) *l_dst = -INFINITY;
    return;
  }
  const int ntile = (t1 - t0 + 31) / 32;

  // ---- tile streaming into this wavefront's private slot: 32 latent rows + 4 rope groups
  char* slot = smem + wave * A16_TILE_BYTES;
  // physical blocks of this wavefront's token range: one entry per lane, picked with v_readlane
  // (ranges longer than 64 blocks fall back to a scalar load per tile)
  const int32_t* bt = a.block_table + (size_t)b * a.max_blocks;
  const int first_blk = is_prefix ? 0 : t0 / a.block_size;
  int bt_cache = 0;
  if (!is_prefix) {
    const int nblk_mine = (t1 - 1) / a.block_size - first_blk + 1;
    bt_cache = (lane < nblk_mine) ? bt[first_blk + lane] : 0;
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(bt_cache)::"memory");
  }
  const int lane_off0 = lane << 4, lane_off1 = (lane ^ 1) << 4;
  const int rope_ch = ((lane & 7) ^ (lane >> 4)) << 4;   // rope group 0; odd groups: ^ 64
  auto issue_tile = [&](int tile, auto prefix_tag) __attribute__((always_inline)) {
    constexpr bool PREFIX = decltype(prefix_tag)::value;
    const int tok0 = t0 + tile * 32;
    const int last = t1 - 1 - tok0;      // last valid row of this tile (>= 0)
    const char* base;
    if constexpr (PREFIX) {
      base = (const char*)a.pc + (size_t)tok0 * (D_L * 2);
    } else {
      const int bi = __builtin_amdgcn_readfirstlane(tok0 / a.block_size - first_blk);
      const int blk = bi < 64 ? __builtin_amdgcn_readlane(bt_cache, bi)
                              : scalar_load_i32(bt + first_blk + bi);
      base = (const char*)(a.pool + ((size_t)blk * a.block_size + tok0 % a.block_size) * D_ROW);
    }
    constexpr int row_bytes = PREFIX ? D_L * 2 : D_ROW * 2;
#pragma unroll
    for (int r = 0; r < 32; r++) {
      const int rr = min(r, last);
      const int loff = ((r >> 3) & 1) ? lane_off1 : lane_off0;
      // (the shared latent prefix is read by every request: default policy; a request's own
      // rows are streamed)
      if constexpr (PREFIX) dma16(base + (size_t)rr * row_bytes + loff, slot + r * A16_ROW_BYTES);
      else dma16_stream(base + (size_t)rr * row_bytes + loff, slot + r * A16_ROW_BYTES);
    }
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int rr = min(8 * j + (lane >> 3), last);
      const char* src;
      if constexpr (PREFIX)
        src = (const char*)a.pr + (size_t)(tok0 + rr) * (D_R * 2) + (rope_ch ^ ((j & 1) << 6));
      else
        src = base + (size_t)rr * row_bytes + D_L * 2 + (rope_ch ^ ((j & 1) << 6));
      if constexpr (PREFIX) dma16(src, slot + A16_MAIN_BYTES + j * 1024);
      else dma16_stream(src, slot + A16_MAIN_BYTES + j * 1024);
    }
  };
  auto issue = [&](int tile) __attribute__((always_inline)) {
    if (is_prefix) issue_tile(tile, std::true_type{});
    else issue_tile(tile, std::false_type{});
  };
  issue(0);

  // ---- absorbed query fragments (B operand): 18 k-steps of 32
  bf16x8 qf[18];
  {
    const __bf16* qp = a.qabs + row * D_ROW + 8 * q4;
#pragma unroll
    for (int ks = 0; ks < 18; ks++) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[ks] = q_valid ? *(const bf16x8*)(qp + 32 * ks) : z;
    }
  }
#pragma unroll
  for (int ks = 0; ks < 18; ks += 3)
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(qf[ks]), "+v"(qf[ks + 1]), "+v"(qf[ks + 2])::"memory");

  // ---- per-lane LDS addresses
  //   scores, latent k-step ks < 16, token block mb: row 16*mb + n, chunk 4*ks + q4
  //       -> (16*mb + n)*1056 + ((q4 ^ sw) * 16) + 64*ks,  sw = (n >> 3) & 1 (16*mb does not change it)
  //   rope k-step k < 2: chunk c = 4*k + q4 in slot c ^ ((row >> 1) & 7), the same for row n
  //       and row 16 + n
  const uint32_t tbase = lds_addr(slot);
  const uint32_t s_addr = tbase + n * A16_ROW_BYTES + ((q4 ^ ((n >> 3) & 1)) << 4);
  uint32_t r_addr[2];
#pragma unroll
  for (int k = 0; k < 2; k++)
    r_addr[k] = tbase + A16_MAIN_BYTES + n * 128 + (((4 * k + q4) ^ ((n >> 1) & 7)) << 4);
  //   P V (transposing read inside the 16-lane group q4, r = lane % 16):
  //     token row 16*half + 4*q4 + r/4, latent 16*mb + 4*(r%4); row swizzle bit = q4 >> 1
  const uint32_t v_addr = tbase + (4 * q4 + (n >> 2)) * A16_ROW_BYTES +
                          ((((n & 3) >> 1) ^ (q4 >> 1)) << 4) + 8 * (n & 1);

  f32x4 o[32];
#pragma unroll
  for (int mb = 0; mb < 32; mb++)
#pragma unroll
    for (int v = 0; v < 4; v++) o[mb][v] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int tile = 0; tile < ntile; tile++) {
    vm_wait<0>();   // this wavefront's own transfers of the tile (nothing else is in flight)
    // ---- scores: two 16-token blocks x 18 k-steps
    f32x4 sacc[2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int v = 0; v < 4; v++) sacc[i][v] = 0.f;
    {
      // groups of 2 k-steps = 4 fragments (2 token blocks each), double buffered; 9 groups,
      // the last one is the rope part
      bf16x8 f[2][4];
      auto rd = [&](auto gsel, auto dsts) {
        constexpr int G = decltype(gsel)::value;
        constexpr int D = decltype(dsts)::value;
        if constexpr (G < 8) {
          f[D][0] = lds_read_b128<64 * (2 * G)>(s_addr);
          f[D][1] = lds_read_b128<64 * (2 * G) + 16 * A16_ROW_BYTES>(s_addr);
          f[D][2] = lds_read_b128<64 * (2 * G + 1)>(s_addr);
          f[D][3] = lds_read_b128<64 * (2 * G + 1) + 16 * A16_ROW_BYTES>(s_addr);
        } else {
          f[D][0] = lds_read_b128<0>(r_addr[0]);
          f[D][1] = lds_read_b128<16 * 128>(r_addr[0]);
          f[D][2] = lds_read_b128<0>(r_addr[1]);
          f[D][3] = lds_read_b128<16 * 128>(r_addr[1]);
        }
      };
      rd(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
      static_for<9>([&](auto grp_c) {
        constexpr int G = decltype(grp_c)::value;
        constexpr int cur = G & 1, nxt = cur ^ 1;
        if constexpr (G + 1 < 9) {
          rd(std::integral_constant<int, G + 1>{}, std::integral_constant<int, nxt>{});
          lgkm_wait<4>(f[cur][0], f[cur][1], f[cur][2], f[cur][3]);
        } else {
          lgkm_wait<0>(f[cur][0], f[cur][1], f[cur][2], f[cur][3]);
        }
        sacc[0] = mfma16(f[cur][0], qf[2 * G], sacc[0]);
        sacc[1] = mfma16(f[cur][1], qf[2 * G], sacc[1]);
        sacc[0] = mfma16(f[cur][2], qf[2 * G + 1], sacc[0]);
        sacc[1] = mfma16(f[cur][3], qf[2 * G + 1], sacc[1]);
      });
    }
    // ---- online softmax over the 8 scores this lane holds (tokens 16*i + 4*q4 + v)
    const int limit = vis_q - (t0 + tile * 32);
    float s8[8];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int v = 0; v < 4; v++) {
        const float x = sacc[i][v];
        s8[4 * i + v] = (limit < 32 && 16 * i + 4 * q4 + v >= limit) ? -INFINITY : x;
      }
    float mx = s8[0];
#pragma unroll
    for (int e = 1; e < 8; e++) mx = fmaxf(mx, s8[e]);
    mx = max_quads(mx) * a.c;
    const float m_new = (mx > m + RESCALE_TAU) ? mx : m;   // lazy reference, see softmax_block
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {
      const float alpha = fast_exp2(m - m_use);
      l *= alpha;
      // the accumulators live in accumulation registers, which the vector ALU cannot address;
      // routing them through these statements keeps their copies inside the rare branch
      // (otherwise the copies are hoisted and run for every tile)
#pragma unroll
      for (int mb = 0; mb < 32; mb++) {
        asm volatile("" : "+a"(o[mb]));
#pragma unroll
        for (int v = 0; v < 4; v++) o[mb][v] *= alpha;
        asm volatile("" : "+a"(o[mb]));
      }
    }
    m = m_new;
    bf16x8 p;
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const float pe = fast_exp2(__builtin_fmaf(s8[e], a.c, -m_use));
      sum += pe;
      p[e] = (__bf16)pe;
    }
    l += sum;
    // ---- P V: 32 latent blocks of 16, one k-step of 32 tokens; groups of 4 blocks
    {
      short4v lo[2][4], hi[2][4];
      auto rdv = [&](auto gsel, auto dsts) {
        constexpr int G = decltype(gsel)::value;
        constexpr int D = decltype(dsts)::value;
        static_for<4>([&](auto j) {
          constexpr int mb = 4 * G + decltype(j)::value;
          lo[D][decltype(j)::value] = lds_read_tr16_b64<32 * mb>(v_addr);
          hi[D][decltype(j)::value] = lds_read_tr16_b64<32 * mb + 16 * A16_ROW_BYTES>(v_addr);
        });
      };
      rdv(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
      static_for<8>([&](auto grp_c) {
        constexpr int G = decltype(grp_c)::value;
        constexpr int cur = G & 1, nxt = cur ^ 1;
        if constexpr (G + 1 < 8) {
          rdv(std::integral_constant<int, G + 1>{}, std::integral_constant<int, nxt>{});
          lgkm_wait<8>(lo[cur][0], lo[cur][1], lo[cur][2], lo[cur][3]);
          lgkm_wait<8>(hi[cur][0], hi[cur][1], hi[cur][2], hi[cur][3]);
        } else {
          lgkm_wait<0>(lo[cur][0], lo[cur][1], lo[cur][2], lo[cur][3]);
          lgkm_wait<0>(hi[cur][0], hi[cur][1], hi[cur][2], hi[cur][3]);
        }
        static_for<4>([&](auto j) {
          constexpr int mb = 4 * G + decltype(j)::value;
          o[mb] = mfma16(join_tr(lo[cur][decltype(j)::value], hi[cur][decltype(j)::value]), p,
                         o[mb]);
        });
      });
    }
    // every LDS read of the tile has been consumed: the slot can be refilled
    if (tile + 1 < ntile) issue(tile + 1);
  }

  const float lt = sum_quads(l);
  if (!q_valid) return;
  if (lt > 0.f) {
    const float inv = 1.f / lt;
#pragma unroll
    for (int mb = 0; mb < 32; mb++) {
      bf16x4 w;
#pragma unroll
      for (int e = 0; e < 4; e++) w[e] = (__bf16)(o[mb][e] * inv);
      *(bf16x4*)(o_dst + 16 * mb) = w;
    }
    if (q4 == 0) *l_dst = (m + fast_log2(lt)) * LN2;
  } else if (q4 == 0) {
    *l_dst = -INFINITY;
  }
}

int mfma_absorb16_attention(const Plan& p, const DecodeArgs& d) {
  if (p.n_lat <= 0 || p.rows == 0) return TMLA_OK;
  Absorb16Args a;
  a.qabs = (const __bf16*)(d.ws + p.off_qabs);
  a.pc = (const __bf16*)d.prefix_ckv;
  a.pr = (const __bf16*)d.prefix_krope;
  a.pool = (const __bf16*)d.suffix_pool;
  a.block_table = d.block_table;
  a.lens = d.suffix_lens;
  a.lat_o = (__bf16*)(d.ws + p.off_lat_o);
  a.lat_lse = (float*)(d.ws + p.off_lat_lse);
  a.Sq = p.Sq; a.H = p.H; a.R = p.Sq * p.H; a.Ls = p.Ls;
  a.ap_chunks = p.ap_chunks; a.ap_chunk = p.ap_chunk;
  a.as_chunks = p.as_chunks; a.as_chunk = p.as_chunk;
  a.ap_groups = (p.ap_chunks + 3) / 4;
  a.max_blocks = d.max_blocks; a.block_size = d.block_size;
  a.rows = p.rows;
  a.c = d.sm_scale * LOG2E;
  static LdsOptIn lds;
  if (lds.ensure((const void*)absorb16_kernel, A16_LDS_BYTES) != hipSuccess) return TMLA_ERR_HIP;
  dim3 grid(a.ap_groups + (p.as_chunks + 3) / 4, p.B);
  a.order = suffix_request_order(p, d, (long long)grid.x * grid.y);
  hipLaunchKernelGGL(absorb16_kernel, grid, dim3(256), A16_LDS_BYTES, d.stream, a);
  return TMLA_OK;
}

}  // namespace tmla
