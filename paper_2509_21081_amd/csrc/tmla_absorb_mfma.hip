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
//   NQB = 4: four wavefronts own 4 x 32 query rows and all 512 latent columns each  (H >= 128)
//   NQB = 2: 2 x 32 query rows, two wavefronts per block own 256 latent columns each
//   NQB = 1: 32 query rows (H = 16 with S_q <= 2), four wavefronts own 128 latent columns each;
//            the scores are recomputed per wavefront, which the HBM-bound small-H case affords.
#include <cstdlib>

#include "tmla_common.hpp"
#include "tmla_mfma.hpp"

namespace tmla {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;

struct AbsorbArgs {
  const __bf16* qabs;        // [rows, 576]
  const __bf16* pc;          // prefix latent [Ls, 512]  (absorb_only)
  const __bf16* pr;          // prefix rope   [Ls, 64]
  const __bf16* pool;        // [num_blocks, block_size, 576]
  const int32_t* block_table;
  const int32_t* lens;
  float* lat_o;              // [n_lat, rows, 512]
  float* lat_lse;            // [n_lat, rows]
  int Sq, H, R, Ls, ap_chunks, ap_chunk, as_chunk, max_blocks, block_size;
  int64_t rows;
  float c;                   // sm_scale * log2(e)
};

constexpr int AB_ROW_BYTES = 1184;                 // 1152 + 32: see bank notes below
constexpr int AB_TILE_BYTES = 32 * AB_ROW_BYTES;   // 37888
constexpr int AB_LDS_BYTES = 2 * AB_TILE_BYTES;    // double buffer
constexpr int AB_CHUNKS = 72;                      // 16-byte chunks per cache row
// LDS tile: row r (token) at r * 1184; its 16-byte chunk c is stored at chunk slot
// c ^ ((r >> 2) & 1).  The 32-byte row skew keeps the transposing reads (4 rows x 32 B per
// 16 lanes) on distinct banks, the chunk swizzle separates rows r and r + 4 for the 16-byte reads.

template <int NQB>
__global__ void __launch_bounds__(256, 1) absorb_attn_kernel(AbsorbArgs a) {
  constexpr int NLP = 4 / NQB;
  constexpr int MBW = 16 / NLP;  // 32-latent blocks owned by a wavefront
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int item = blockIdx.x, qg = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int qb = wave % NQB, lp = wave / NQB;
  const int r_local = (qg * NQB + qb) * 32 + n;   // this lane's query row within the request
  const bool q_valid = r_local < a.R;
  const int64_t row = (int64_t)b * a.R + r_local; // global output row (b, s, h)

  // ---- which tokens
  int t0, t1, vis_q;
  const bool is_prefix = item < a.ap_chunks;
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
  float* o_dst = a.lat_o + ((size_t)item * a.rows + row) * D_L;
  float* l_dst = a.lat_lse + (size_t)item * a.rows + row;
  if (t1 <= t0) {   // empty chunk (workgroup-uniform)
    if (q_valid && lp == 0 && g == 0) *l_dst = -INFINITY;
    return;
  }
  const int ntile = (t1 - t0 + 31) / 32;

  // ---- absorbed query fragments (B operand): 36 k-steps of 16
  bf16x8 qf[36];
  {
    const __bf16* qp = a.qabs + row * D_ROW + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 36; ks++) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[ks] = q_valid ? *(const bf16x8*)(qp + 16 * ks) : z;
    }
  }

  // ---- tile loader: 32 rows x 72 chunks = 2304 chunks, 9 per thread
  bf16x8 stg[9];
  const int32_t* bt = a.block_table + (size_t)b * a.max_blocks;
  auto issue_loads = [&](int tile) {
    const int tok0 = t0 + tile * 32;
    const __bf16* page = nullptr;
    if (!is_prefix) {
      const int blk = bt[tok0 / a.block_size];
      page = a.pool + ((size_t)blk * a.block_size + tok0 % a.block_size) * D_ROW;
    }
#pragma unroll
    for (int i = 0; i < 9; i++) {
      const int cidx = tid + 256 * i;
      const int r = cidx / AB_CHUNKS, ch = cidx - r * AB_CHUNKS;
      const int tok = tok0 + r;
      bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (tok < t1) {
        const __bf16* src;
        if (is_prefix)
          src = (ch < 64) ? a.pc + (size_t)tok * D_L + ch * 8 : a.pr + (size_t)tok * D_R + (ch - 64) * 8;
        else
          src = page + (size_t)r * D_ROW + ch * 8;
        v = *(const bf16x8*)src;
      }
      stg[i] = v;
    }
  };
  auto store_lds = [&](int tile) {
    char* buf = smem + (tile & 1) * AB_TILE_BYTES;
#pragma unroll
    for (int i = 0; i < 9; i++) {
      const int cidx = tid + 256 * i;
      const int r = cidx / AB_CHUNKS, ch = cidx - r * AB_CHUNKS;
      *(bf16x8*)(buf + r * AB_ROW_BYTES + ((ch ^ ((r >> 2) & 1)) << 4)) = stg[i];
    }
  };

  // per-lane LDS offsets
  //   S phase: row n, chunk 2*ks + g  ->  n*1184 + ((g ^ sw_n) * 16) + 32*ks
  const int s_off = n * AB_ROW_BYTES + ((g ^ ((n >> 2) & 1)) << 4);
  //   P V phase (transposing read, 16-lane groups j = lane/16, r = lane%16):
  //     token row 16*kk + 8*half + 4*g + r/4, latent 32*mb + 16*(j%2) + 4*(r%4)
  const int j16 = lane >> 4, r16 = lane & 15;
  const int v_off = (4 * g + (r16 >> 2)) * AB_ROW_BYTES +
                    ((2 * (j16 & 1) + (((r16 & 3) >> 1) ^ g)) << 4) + 8 * (r16 & 1);

  f32x16 o[MBW];
#pragma unroll
  for (int mb = 0; mb < MBW; mb++)
#pragma unroll
    for (int v = 0; v < 16; v++) o[mb][v] = 0.f;
  float m = -INFINITY, l = 0.f;

  issue_loads(0);
  store_lds(0);
  __syncthreads();
  for (int tile = 0; tile < ntile; tile++) {
    if (tile + 1 < ntile) issue_loads(tile + 1);
    const char* buf = smem + (tile & 1) * AB_TILE_BYTES;
    f32x16 sacc;
#pragma unroll
    for (int v = 0; v < 16; v++) sacc[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 36; ks++) {
      const bf16x8 cf = *(const bf16x8*)(buf + s_off + 32 * ks);
      sacc = mfma32(cf, qf[ks], sacc);
    }
    const int limit = min(32, vis_q - (t0 + tile * 32));
    bf16x8 p[2];
    bool rescale;
    const float alpha = softmax_block(sacc, m, l, a.c, limit, g, p[0], p[1], rescale);
    if (rescale) {
#pragma unroll
      for (int mb = 0; mb < MBW; mb++)
#pragma unroll
        for (int v = 0; v < 16; v++) o[mb][v] *= alpha;
    }
#pragma unroll
    for (int mb = 0; mb < MBW; mb++) {
#pragma unroll
      for (int kk = 0; kk < 2; kk++) {
        const char* src = buf + v_off + (16 * kk) * AB_ROW_BYTES + 64 * (lp * MBW + mb);
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(src));
        const short4v hi =
            __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(src + 8 * AB_ROW_BYTES));
        typedef short short8v __attribute__((ext_vector_type(8)));
        const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        o[mb] = mfma32(__builtin_bit_cast(bf16x8, both), p[kk], o[mb]);
      }
    }
    if (tile + 1 < ntile) store_lds(tile + 1);
    __syncthreads();
  }

  const float lt = sum_halves(l);
  if (!q_valid) return;
  if (lt > 0.f) {
    const float inv = 1.f / lt;
#pragma unroll
    for (int mb = 0; mb < MBW; mb++)
#pragma unroll
      for (int v4 = 0; v4 < 4; v4++) {
        float4 w = make_float4(o[mb][4 * v4] * inv, o[mb][4 * v4 + 1] * inv,
                               o[mb][4 * v4 + 2] * inv, o[mb][4 * v4 + 3] * inv);
        *(float4*)(o_dst + 32 * (lp * MBW + mb) + 8 * v4 + 4 * g) = w;
      }
    if (lp == 0 && g == 0) *l_dst = (m + fast_log2(lt)) * LN2;
  } else if (lp == 0 && g == 0) {
    *l_dst = -INFINITY;   // causal mask hid every token of this chunk from this query
  }
}

int mfma_absorb_attention(const Plan& p, const DecodeArgs& d) {
  if (p.n_lat <= 0 || p.rows == 0) return TMLA_OK;
  AbsorbArgs a;
  a.qabs = (const __bf16*)(d.ws + p.off_qabs);
  a.pc = (const __bf16*)d.prefix_ckv;
  a.pr = (const __bf16*)d.prefix_krope;
  a.pool = (const __bf16*)d.suffix_pool;
  a.block_table = d.block_table;
  a.lens = d.suffix_lens;
  a.lat_o = (float*)(d.ws + p.off_lat_o);
  a.lat_lse = (float*)(d.ws + p.off_lat_lse);
  a.Sq = p.Sq; a.H = p.H; a.R = p.Sq * p.H; a.Ls = p.Ls;
  a.ap_chunks = p.ap_chunks; a.ap_chunk = p.ap_chunk; a.as_chunk = p.as_chunk;
  a.max_blocks = d.max_blocks; a.block_size = d.block_size;
  a.rows = p.rows;
  a.c = d.sm_scale * LOG2E;
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)absorb_attn_kernel<4>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, AB_LDS_BYTES) != hipSuccess ||
        hipFuncSetAttribute((const void*)absorb_attn_kernel<2>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, AB_LDS_BYTES) != hipSuccess ||
        hipFuncSetAttribute((const void*)absorb_attn_kernel<1>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, AB_LDS_BYTES) != hipSuccess)
      return TMLA_ERR_HIP;
    attr_set = true;
  }
  const int R = a.R;
  static const int force_nqb4 = getenv("TMLA_ABSORB_NQB4") ? atoi(getenv("TMLA_ABSORB_NQB4")) : 0;
  if (R > 64 && force_nqb4) {
    dim3 grid(p.n_lat, (R + 127) / 128, p.B);
    hipLaunchKernelGGL(absorb_attn_kernel<4>, grid, dim3(256), AB_LDS_BYTES, d.stream, a);
  } else if (R > 32) {
    dim3 grid(p.n_lat, (R + 63) / 64, p.B);
    hipLaunchKernelGGL(absorb_attn_kernel<2>, grid, dim3(256), AB_LDS_BYTES, d.stream, a);
  } else {
    dim3 grid(p.n_lat, 1, p.B);
    hipLaunchKernelGGL(absorb_attn_kernel<1>, grid, dim3(256), AB_LDS_BYTES, d.stream, a);
  }
  return TMLA_OK;
}

}  // namespace tmla
