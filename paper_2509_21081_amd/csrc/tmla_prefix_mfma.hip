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
constexpr int QS_BLOCK_BYTES = (K_BLK_ELEMS + V_BLK_ELEMS) * 2;  // 20480
constexpr int QS_STAGE_BLOCKS = 2;
constexpr int QS_LDS_BYTES = 2 * QS_STAGE_BLOCKS * QS_BLOCK_BYTES;  // 81920

__global__ void __launch_bounds__(256, 1) prefix_attn_query_split_kernel(PrefixArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int h = blockIdx.x, mb = blockIdx.y, sp = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int q0 = mb * 256 + wave * 64;
  const bool active = q0 < a.M;

  bf16x8 qf[2][12];
  load_q_frags(a, h, q0, n, g, qf);

  const int tb0 = sp * a.blocks_per_split;
  const int tb1 = min(a.ntb, tb0 + a.blocks_per_split);
  const int nblk = tb1 - tb0;
  const int nstage = (nblk + QS_STAGE_BLOCKS - 1) / QS_STAGE_BLOCKS;
  const __bf16* kbase = a.pk + ((size_t)h * a.ntb) * K_BLK_ELEMS;
  const __bf16* vbase = a.pv + ((size_t)h * a.ntb) * V_BLK_ELEMS;

  // one block = 1280 chunks of 16 B: 768 of K then 512 of V; 5 chunks per thread
  bf16x8 stg[QS_STAGE_BLOCKS][5];
  auto issue_loads = [&](int s) {
#pragma unroll
    for (int j = 0; j < QS_STAGE_BLOCKS; j++) {
      const int tb = tb0 + s * QS_STAGE_BLOCKS + j;
      if (tb < tb1) {
        const __bf16* kb = kbase + (size_t)tb * K_BLK_ELEMS;
        const __bf16* vb = vbase + (size_t)tb * V_BLK_ELEMS;
#pragma unroll
        for (int i = 0; i < 3; i++) stg[j][i] = *(const bf16x8*)(kb + (tid + 256 * i) * 8);
#pragma unroll
        for (int i = 3; i < 5; i++) stg[j][i] = *(const bf16x8*)(vb + (tid + 256 * (i - 3)) * 8);
      }
    }
  };
  auto store_lds = [&](int s) {
    char* buf = smem + (s & 1) * (QS_STAGE_BLOCKS * QS_BLOCK_BYTES);
#pragma unroll
    for (int j = 0; j < QS_STAGE_BLOCKS; j++) {
      if (tb0 + s * QS_STAGE_BLOCKS + j < tb1) {
#pragma unroll
        for (int i = 0; i < 5; i++)
          *(bf16x8*)(buf + j * QS_BLOCK_BYTES + (tid + 256 * i) * 16) = stg[j][i];
      }
    }
  };

  f32x16 o[4][2];
#pragma unroll
  for (int db = 0; db < 4; db++)
#pragma unroll
    for (int nb = 0; nb < 2; nb++)
#pragma unroll
      for (int v = 0; v < 16; v++) o[db][nb][v] = 0.f;
  float m[2] = {-INFINITY, -INFINITY}, l[2] = {0.f, 0.f};

  if (nstage > 0) {
    issue_loads(0);
    store_lds(0);
  }
  __syncthreads();
  for (int s = 0; s < nstage; s++) {
    if (s + 1 < nstage) issue_loads(s + 1);
    if (active) {
      const char* buf = smem + (s & 1) * (QS_STAGE_BLOCKS * QS_BLOCK_BYTES);
#pragma unroll
      for (int j = 0; j < QS_STAGE_BLOCKS; j++) {
        const int tb = tb0 + s * QS_STAGE_BLOCKS + j;
        if (tb < tb1) {
          const char* kb = buf + j * QS_BLOCK_BYTES + lane * 16;
          const char* vb = kb + K_BLK_ELEMS * 2;
          f32x16 sacc[2];
#pragma unroll
          for (int nb = 0; nb < 2; nb++)
#pragma unroll
            for (int v = 0; v < 16; v++) sacc[nb][v] = 0.f;
#pragma unroll
          for (int ks = 0; ks < 12; ks++) {
            const bf16x8 kf = *(const bf16x8*)(kb + ks * 1024);
            sacc[0] = mfma32(kf, qf[0][ks], sacc[0]);
            sacc[1] = mfma32(kf, qf[1][ks], sacc[1]);
          }
          const int limit = min(32, a.Ls - tb * TOK_BLK);
          bf16x8 p[2][2];
#pragma unroll
          for (int nb = 0; nb < 2; nb++) {
            bool rescale;
            const float alpha = softmax_block(sacc[nb], m[nb], l[nb], a.c, limit, g, p[nb][0],
                                              p[nb][1], rescale);
            if (rescale) {
#pragma unroll
              for (int db = 0; db < 4; db++)
#pragma unroll
                for (int v = 0; v < 16; v++) o[db][nb][v] *= alpha;
            }
          }
#pragma unroll
          for (int kk = 0; kk < 2; kk++)
#pragma unroll
            for (int db = 0; db < 4; db++) {
              const bf16x8 vf = *(const bf16x8*)(vb + (kk * 4 + db) * 1024);
              o[db][0] = mfma32(vf, p[0][kk], o[db][0]);
              o[db][1] = mfma32(vf, p[1][kk], o[db][1]);
            }
        }
      }
    }
    if (s + 1 < nstage) store_lds(s + 1);
    __syncthreads();
  }

  if (!active) return;
#pragma unroll
  for (int nb = 0; nb < 2; nb++) {
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

// ------------------------------------------------------------------ token-split workgroup
constexpr int TS_ROW_FLOATS = 132;  // 128 + 4 padding: conflict-free 16-byte LDS accesses
constexpr int TS_LDS_BYTES = 4 * 64 * TS_ROW_FLOATS * 4 + 2 * 4 * 64 * 4;  // O regions + m, l

__global__ void __launch_bounds__(256, 1) prefix_attn_token_split_kernel(PrefixArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int h = blockIdx.x, mb = blockIdx.y, sp = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int q0 = mb * 64;

  bf16x8 qf[2][12];
  load_q_frags(a, h, q0, n, g, qf);

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

  // wavefront w takes blocks tb0 + w, tb0 + w + 4, ...; K of the next block is fetched while the
  // current block's P V product runs, V of the current block while its scores are computed
  bf16x8 kf[12], vf[8];
  int tb = tb0 + wave;
  if (tb < tb1) {
#pragma unroll
    for (int ks = 0; ks < 12; ks++)
      kf[ks] = *(const bf16x8*)(kbase + (size_t)tb * K_BLK_ELEMS + ks * 512);
  }
  for (; tb < tb1; tb += 4) {
#pragma unroll
    for (int f = 0; f < 8; f++)
      vf[f] = *(const bf16x8*)(vbase + (size_t)tb * V_BLK_ELEMS + f * 512);
    f32x16 sacc[2];
#pragma unroll
    for (int nb = 0; nb < 2; nb++)
#pragma unroll
      for (int v = 0; v < 16; v++) sacc[nb][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 12; ks++) {
      sacc[0] = mfma32(kf[ks], qf[0][ks], sacc[0]);
      sacc[1] = mfma32(kf[ks], qf[1][ks], sacc[1]);
    }
    if (tb + 4 < tb1) {
#pragma unroll
      for (int ks = 0; ks < 12; ks++)
        kf[ks] = *(const bf16x8*)(kbase + (size_t)(tb + 4) * K_BLK_ELEMS + ks * 512);
    }
    const int limit = min(32, a.Ls - tb * TOK_BLK);
    bf16x8 p[2][2];
#pragma unroll
    for (int nb = 0; nb < 2; nb++) {
      bool rescale;
      const float alpha =
          softmax_block(sacc[nb], m[nb], l[nb], a.c, limit, g, p[nb][0], p[nb][1], rescale);
      if (rescale) {
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
          for (int v = 0; v < 16; v++) o[db][nb][v] *= alpha;
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
    dim3 grid(p.H, (a.M + 255) / 256, p.np_split);
    hipLaunchKernelGGL(prefix_attn_query_split_kernel, grid, dim3(256), QS_LDS_BYTES, d.stream, a);
  } else {
    dim3 grid(p.H, (a.M + 63) / 64, p.np_split);
    hipLaunchKernelGGL(prefix_attn_token_split_kernel, grid, dim3(256), TS_LDS_BYTES, d.stream, a);
  }
  return TMLA_OK;
}

}  // namespace tmla
