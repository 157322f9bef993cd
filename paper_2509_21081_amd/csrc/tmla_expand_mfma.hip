// Prefix (and pool) expansion on the matrix cores (paper Section 3.1 "Prefill": the shared part of
// the latent caches is expanded through the up-projection into per-head K and V):
//     K[h, t, 0:128] = W_UK[h] c_t,   K[h, t, 128:192] = r_t,   V[h, t, :] = W_UV[h] c_t
// i.e. one GEMM [tokens x 512] x [512 x 256 H] whose epilogue writes the matrix-core operand
// order the decode kernels read (see typhoon_mla.h).
//
// LDS-tiled GEMM, workgroup tile 128 tokens x 128 outputs (one head's K-nope or V), k = 512 in
// steps of 64, four wavefronts of 64 x 64 (2 x 2 MFMA blocks, each LDS fragment used twice).
// Both operands are k-contiguous in memory (rows of c_KV, rows of W), so either can be the MFMA
// row operand: the K half computes W c^T (lanes own tokens, 4 consecutive d per register group ->
// 8-byte stores into the K fragment order), the V half computes c W^T (lanes own d, 8 consecutive
// accumulators are exactly one 16-byte V fragment chunk).
#include "tmla_common.hpp"
#include "tmla_mfma.hpp"

namespace tmla {

constexpr int EX_TILE = 128;          // rows per operand tile
constexpr int EX_KSTEP = 64;          // k elements per LDS stage
constexpr int EX_ROW_BYTES = 144;     // 128 B of data + 16 B pad: conflict-free 16-byte reads
constexpr int EX_TILE_BYTES = EX_TILE * EX_ROW_BYTES;   // 18432

struct ExpandArgs {
  const __bf16* c; int64_t c_stride;      // latent rows [ntok, 512] (element stride between rows)
  const __bf16* r; int64_t r_stride;      // rope rows   [ntok, 64]
  const __bf16* w_uk; const __bf16* w_uv; // [H, 128, 512]
  __bf16* k_out; __bf16* v_out;
  int64_t ntok, ntb;
  int H;
};

__global__ void __launch_bounds__(256) expand_gemm_kernel(ExpandArgs a) {
  __shared__ __attribute__((aligned(16))) char lds[2][2][EX_TILE_BYTES];  // [stage][tok|w]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int64_t t_base = (int64_t)blockIdx.x * EX_TILE;
  const int h = blockIdx.y >> 1;
  const bool is_v = blockIdx.y & 1;
  const __bf16* w = (is_v ? a.w_uv : a.w_uk) + (size_t)h * 128 * D_L;

  // global -> registers -> LDS: each tile stage is 128 rows x 8 chunks of 16 B, 4 per thread
  bf16x8 st_c[4], st_w[4];
  auto load_stage = [&](int kt) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int cidx = tid + 256 * i;
      const int row = cidx >> 3, ch = cidx & 7;
      const int64_t t = t_base + row;
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      st_c[i] = (t < a.ntok) ? *(const bf16x8*)(a.c + t * a.c_stride + kt * EX_KSTEP + ch * 8) : z;
      st_w[i] = *(const bf16x8*)(w + (size_t)row * D_L + kt * EX_KSTEP + ch * 8);
    }
  };
  auto store_stage = [&](int s) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int cidx = tid + 256 * i;
      const int row = cidx >> 3, ch = cidx & 7;
      *(bf16x8*)(lds[s & 1][0] + row * EX_ROW_BYTES + ch * 16) = st_c[i];
      *(bf16x8*)(lds[s & 1][1] + row * EX_ROW_BYTES + ch * 16) = st_w[i];
    }
  };

  // wavefront sub-tile: row-operand rows [64*wm, +64), column-operand rows [64*wn, +64)
  const int wm = wave >> 1, wn = wave & 1;
  const int row_op = is_v ? 0 : 1;   // V: rows = tokens (c), cols = d (W);  K: rows = d, cols = tokens
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  load_stage(0);
  store_stage(0);
  __syncthreads();
  constexpr int NKT = D_L / EX_KSTEP;   // 8
  for (int kt = 0; kt < NKT; kt++) {
    if (kt + 1 < NKT) load_stage(kt + 1);
    const char* ta = lds[kt & 1][row_op] + (64 * wm + n) * EX_ROW_BYTES + g * 16;
    const char* tb = lds[kt & 1][row_op ^ 1] + (64 * wn + n) * EX_ROW_BYTES + g * 16;
#pragma unroll
    for (int ks = 0; ks < EX_KSTEP / 16; ks++) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; i++) {
        fa[i] = *(const bf16x8*)(ta + i * 32 * EX_ROW_BYTES + ks * 32);
        fb[i] = *(const bf16x8*)(tb + i * 32 * EX_ROW_BYTES + ks * 32);
      }
#pragma unroll
      for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++) acc[i][j] = mfma32(fa[i], fb[j], acc[i][j]);
    }
    if (kt + 1 < NKT) store_stage(kt + 1);
    __syncthreads();
  }

  if (is_v) {
    // block (i, j): tokens t_base + 64*wm + 32*i + acc_row, d = 64*wn + 32*j + n
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const int64_t tb32 = (t_base + 64 * wm + 32 * i) / TOK_BLK;
      if (tb32 >= a.ntb) continue;
#pragma unroll
      for (int j = 0; j < 2; j++) {
        const int db = 2 * wn + j;
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
          bf16x8 o;
#pragma unroll
          for (int e = 0; e < 8; e++) o[e] = (__bf16)acc[i][j][8 * kk + e];
          *(bf16x8*)(a.v_out + (((((size_t)h * a.ntb + tb32) * 2 + kk) * 4 + db) * 64 + lane) * 8) = o;
        }
      }
    }
  } else {
    // block (i, j): d = 64*wm + 32*i + acc_row, tokens t_base + 64*wn + 32*j + n
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int64_t tb32 = (t_base + 64 * wn + 32 * j) / TOK_BLK;
      if (tb32 >= a.ntb) continue;
#pragma unroll
      for (int i = 0; i < 2; i++) {
#pragma unroll
        for (int q = 0; q < 4; q++) {   // d = 64*wm + 32*i + 8*q + 4*g + (0..3)
          const int d0 = 64 * wm + 32 * i + 8 * q;
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; e++) o[e] = (__bf16)acc[i][j][4 * q + e];
          *(bf16x4*)(a.k_out + ((((size_t)h * a.ntb + tb32) * 12 + d0 / 16) * 64 + n +
                                32 * ((d0 % 16) / 8)) * 8 + 4 * g) = o;
        }
      }
    }
    // rope part of K: verbatim copy, 128 tokens x 8 chunks of 16 B
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int cidx = tid + 256 * i;
      const int row = cidx >> 3, q = cidx & 7;
      const int64_t t = t_base + row;
      const int64_t tb32 = t / TOK_BLK;
      if (tb32 >= a.ntb) continue;
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      const bf16x8 val = (t < a.ntok) ? *(const bf16x8*)(a.r + t * a.r_stride + q * 8) : z;
      *(bf16x8*)(a.k_out + ((((size_t)h * a.ntb + tb32) * 12 + 8 + q / 2) * 64 + (int)(t % TOK_BLK) +
                            32 * (q % 2)) * 8) = val;
    }
  }
}

int mfma_expand(int H, int64_t ntok, const void* c, int64_t c_stride, const void* r,
                int64_t r_stride, const void* w_uk, const void* w_uv, void* k_out, void* v_out,
                hipStream_t stream) {
  if (ntok <= 0) return TMLA_OK;
  ExpandArgs a;
  a.c = (const __bf16*)c; a.c_stride = c_stride; a.r = (const __bf16*)r; a.r_stride = r_stride;
  a.w_uk = (const __bf16*)w_uk; a.w_uv = (const __bf16*)w_uv;
  a.k_out = (__bf16*)k_out; a.v_out = (__bf16*)v_out;
  a.ntok = ntok; a.ntb = (ntok + TOK_BLK - 1) / TOK_BLK; a.H = H;
  const int64_t tiles = (ntok + EX_TILE - 1) / EX_TILE;
  if (tiles > 0x7fffffff) return TMLA_ERR_UNSUPPORTED;
  dim3 grid((unsigned)tiles, 2 * H);
  hipLaunchKernelGGL(expand_gemm_kernel, grid, dim3(256), 0, stream, a);
  return TMLA_OK;
}

}  // namespace tmla
