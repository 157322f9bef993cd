// Prefix (and pool) expansion on the matrix cores (paper Section 3.1 "Prefill": the shared part of
// the latent caches is expanded through the up-projection into per-head K and V):
//     K[h, t, 0:128] = W_UK[h] c_t,   K[h, t, 128:192] = r_t,   V[h, t, :] = W_UV[h] c_t
// i.e. one GEMM [tokens x 512] x [512 x 256 H] whose epilogue writes the matrix-core operand
// order the decode kernels read (see typhoon_mla.h).
//
// Workgroup tile: 256 tokens x one head's 256 outputs (128 K-nope + 128 V), k = 512 in 16 stages
// of 32.  Four wavefronts of 128 x 128 (4 x 4 MFMA blocks of 32 x 32): every fragment read from
// LDS feeds four MFMAs, so the LDS runs at half its rate when the matrix cores are busy.  Both
// operands are k-contiguous in memory (rows of c_KV, rows of W), so either can be the MFMA row
// operand: the K wavefronts compute W c^T (lanes own tokens, 4 consecutive d per register group
// -> 8-byte stores into the K fragment order), the V wavefronts compute c W^T (lanes own d,
// 8 consecutive accumulators are exactly one 16-byte V fragment chunk).
// Stages stream global -> LDS (global_load_lds) through a ring of four, three in flight.
#include <type_traits>

#include "tmla_common.hpp"
#include "tmla_lds_asm.hpp"
#include "tmla_mfma.hpp"

namespace tmla {

constexpr int EX_TOK = 256;           // tokens per workgroup tile
constexpr int EX_KSTAGE = 32;         // k elements per stage: 64 B per row = 4 chunks of 16 B
constexpr int EX_NSTAGE = D_L / EX_KSTAGE;                 // 16
constexpr int EX_OPER_BYTES = 256 * 64;                    // one operand tile of a stage: 16 KiB
constexpr int EX_STAGE_BYTES = 2 * EX_OPER_BYTES;          // tokens, then weights
constexpr int EX_RING = 4;
constexpr int EX_LDS_BYTES = EX_RING * EX_STAGE_BYTES;     // 128 KiB
constexpr int EX_DMA_PER_WAVE = 8;                         // 32 transfers of 1 KiB per stage

struct ExpandArgs {
  const __bf16* c; int64_t c_stride;      // latent rows [ntok, 512] (element stride between rows)
  const __bf16* r; int64_t r_stride;      // rope rows   [ntok, 64]
  const __bf16* w_uk; const __bf16* w_uv; // [H, 128, 512]
  __bf16* k_out; __bf16* v_out;
  int64_t ntok, ntb, tiles;
  int H;
};

// LDS operand tile of a stage: row i at i * 64, its 16-byte chunk c (k = 8c .. 8c+7) in slot
// c ^ ((i >> 2) & 3): rows 64 B apart would put rows i and i + 4 on the same banks for the
// 16-byte fragment reads (lane n reads row n); the slot swizzle spreads 16 consecutive rows over
// all 16 sixteen-byte bank groups.  A 1 KiB transfer covers 16 rows (lane l: row l / 4, slot l % 4).
__global__ void __launch_bounds__(256, 1) expand_gemm_kernel(ExpandArgs a) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t t_base = (int64_t)(blockIdx.x % a.tiles) * EX_TOK;
  const int h = (int)(blockIdx.x / a.tiles);
  const int wm = wave >> 1;          // token half of the tile: tokens [128 wm, 128 wm + 128)
  const bool is_v = wave & 1;        // K-nope or V outputs

  // ---- transfers: wavefront w moves token rows [64 w, 64 w + 64) and weight rows
  // [64 w, 64 w + 64) (rows 0..127 = W_UK[h], 128..255 = W_UV[h]) of every stage, 4 + 4 transfers
  // (base pointers are wave-uniform; the per-lane parts are 32-bit offsets)
  const int dr = lane >> 2;                          // row inside a 16-row transfer
  const int chunk16 = ((lane & 3) ^ ((dr >> 2) & 3)) << 4;   // 64 w + 16 i does not change the swizzle
  const char* c_base = (const char*)(a.c + t_base * a.c_stride);
  const int last_rel = (int)min((int64_t)EX_TOK - 1, a.ntok - 1 - t_base);   // rows past the end
  int c_off[4];                                                               // repeat the last one
#pragma unroll
  for (int i = 0; i < 4; i++)
    c_off[i] = min(64 * wave + 16 * i + dr, last_rel) * (int)(a.c_stride * 2) + chunk16;
  const char* w_base = (const char*)((wave < 2 ? a.w_uk : a.w_uv) +
                                     ((size_t)h * 128 + 64 * (wave & 1)) * D_L);
  const int w_lane = dr * (D_L * 2) + chunk16;
  auto issue = [&](int st) __attribute__((always_inline)) {
    char* dst = smem + (st % EX_RING) * EX_STAGE_BYTES + (64 * wave) * 64;
    const char* cs = c_base + st * (EX_KSTAGE * 2);
    const char* ws = w_base + st * (EX_KSTAGE * 2) + w_lane;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      dma16(cs + c_off[i], dst + i * 1024);
      dma16(ws + i * 16 * (D_L * 2), dst + EX_OPER_BYTES + i * 1024);
    }
  };

  // ---- fragment addresses: row operand rows [ra, ra + 128), column operand rows [rb, rb + 128)
  //   K wavefronts: rows = d (W_UK, weight tile rows 0..127), columns = tokens
  //   V wavefronts: rows = tokens, columns = d (W_UV, weight tile rows 128..255)
  const uint32_t base = lds_addr(smem);
  const uint32_t tok_off = (128 * wm + n) * 64;
  const uint32_t w_off = EX_OPER_BYTES + ((is_v ? 128 : 0) + n) * 64;
  const uint32_t a_off = is_v ? tok_off : w_off;
  const uint32_t b_off = is_v ? w_off : tok_off;
  // chunk 2*ks + g of row n + 32 i: slot (2 ks + g) ^ ((n >> 2) & 3)  (32 i does not change it)
  const uint32_t sw = (n >> 2) & 3;
  const uint32_t sl0 = ((0 + g) ^ sw) << 4, sl1 = ((2 + g) ^ sw) << 4;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

#pragma unroll
  for (int st = 0; st < EX_RING - 1; st++) issue(st);

  // Software pipeline over the two k-steps of a stage: while the 16 MFMAs of one k-step run, the
  // fragments of the next one (possibly of the next stage) come in from LDS, the barrier for
  // the next stage is passed and this wavefront's 8 transfers of the stage three ahead are
  // issued between the MFMAs (a transfer holds the issuing wavefront for some tens of cycles).
  bf16x8 fa[2][4], fb[2][4];
  auto read_frags = [&](int st, auto ks_) __attribute__((always_inline)) {
    constexpr int ks = decltype(ks_)::value;
    const uint32_t sb = base + (st % EX_RING) * EX_STAGE_BYTES;
    const uint32_t sl = ks ? sl1 : sl0;
    static_for<4>([&](auto i_) {
      constexpr int i = decltype(i_)::value;
      fa[ks][i] = lds_read_b128<i * 32 * 64>(sb + a_off + sl);
      fb[ks][i] = lds_read_b128<i * 32 * 64>(sb + b_off + sl);
    });
  };
  auto mma = [&](auto ks_, int pf_stage) __attribute__((always_inline)) {
    constexpr int ks = decltype(ks_)::value;
    // pf_stage >= 0: issue half of that stage's transfers (4 of 8) between the MFMAs
    char* dst = smem + (pf_stage % EX_RING) * EX_STAGE_BYTES + (64 * wave) * 64;
    const char* cs = c_base + pf_stage * (EX_KSTAGE * 2);
    const char* ws = w_base + pf_stage * (EX_KSTAGE * 2) + w_lane;
    static_for<4>([&](auto i_) {
      constexpr int i = decltype(i_)::value;
#pragma unroll
      for (int j = 0; j < 4; j++) acc[i][j] = mfma32(fa[ks][i], fb[ks][j], acc[i][j]);
      if (pf_stage >= 0) {
        if constexpr (ks == 0) dma16(cs + c_off[i], dst + i * 1024);
        else dma16(ws + i * 16 * (D_L * 2), dst + EX_OPER_BYTES + i * 1024);
      }
    });
  };
  constexpr std::integral_constant<int, 0> K0{};
  constexpr std::integral_constant<int, 1> K1{};

  vm_wait<2 * EX_DMA_PER_WAVE>();   // stage 0 (EX_NSTAGE > EX_RING: three stages are in flight)
  raw_barrier();
  read_frags(0, K0);
  read_frags(0, K1);
  for (int st = 0; st < EX_NSTAGE; st++) {
    // the transfers of stage st + 3 go into the slot of stage st - 1, which everyone has left:
    // each wavefront read its last fragments of it before the barrier of the previous iteration
    const int pf = st + EX_RING - 1 < EX_NSTAGE ? st + EX_RING - 1 : -1;
    lgkm_wait<8>(fa[0][0], fa[0][1], fa[0][2], fa[0][3]);
    lgkm_wait<8>(fb[0][0], fb[0][1], fb[0][2], fb[0][3]);
    mma(K0, pf);
    lgkm_wait<0>(fa[1][0], fa[1][1], fa[1][2], fa[1][3]);
    lgkm_wait<0>(fb[1][0], fb[1][1], fb[1][2], fb[1][3]);
    if (st + 1 < EX_NSTAGE) {
      // stage st + 1 must have landed for everyone before its fragments are read.  In flight
      // behind it: stage st + 2 (8 transfers) and the first half of stage st + 3 (4)
      const int ahead = EX_NSTAGE - 2 - st;           // stages issued after st + 1
      if (ahead >= 2) vm_wait<EX_DMA_PER_WAVE + 4>();
      else if (ahead == 1) vm_wait<EX_DMA_PER_WAVE>();
      else vm_wait<0>();
      raw_barrier();
      read_frags(st + 1, K0);
    }
    mma(K1, pf);
    if (st + 1 < EX_NSTAGE) read_frags(st + 1, K1);
  }

  // ---- epilogue: bf16, fragment order; tokens past the end are stored as zeros (the padding of
  // the last 32-token block must be finite for the decode kernels and is specified as zero).
  // The lane indices pass through an opaque statement so that the store addresses are computed
  // here and not hoisted above the main loop, where they would push its registers into scratch
  // (a scratch reload inside the loop waits for every transfer in flight).
  int en = n, eg = g, elane = lane, etid = tid;
  asm volatile("" : "+v"(en), "+v"(eg), "+v"(elane), "+v"(etid));
  // likewise the accumulators: they stay in accumulation registers until here, their copies to
  // vector registers (for the conversion) must not be spread over the loop
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) asm volatile("" : "+a"(acc[i][j]));
  if (is_v) {
    // block (i, j): tokens t_base + 128 wm + 32 i + acc_row, d = 32 j + n
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int64_t tok0 = t_base + 128 * wm + 32 * i;
      const int64_t tb32 = tok0 / TOK_BLK;
      if (tb32 >= a.ntb) continue;
#pragma unroll
      for (int j = 0; j < 4; j++) {
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
          bf16x8 o;
#pragma unroll
          for (int e = 0; e < 8; e++) {
            const int v = 8 * kk + e;
            o[e] = (tok0 + acc_row(v, eg) < a.ntok) ? (__bf16)acc[i][j][v] : (__bf16)0.f;
          }
          *(bf16x8*)(a.v_out + (((((size_t)h * a.ntb + tb32) * 2 + kk) * 4 + j) * 64 + elane) * 8) = o;
        }
      }
    }
  } else {
    // block (i, j): d = 32 i + acc_row, tokens t_base + 128 wm + 32 j + n
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int64_t tok0 = t_base + 128 * wm + 32 * j;
      const int64_t tb32 = tok0 / TOK_BLK;
      if (tb32 >= a.ntb) continue;
      const bool real = tok0 + en < a.ntok;
#pragma unroll
      for (int i = 0; i < 4; i++) {
#pragma unroll
        for (int q = 0; q < 4; q++) {   // d = 32 i + 8 q + 4 g + (0..3)
          const int d0 = 32 * i + 8 * q;
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; e++) o[e] = real ? (__bf16)acc[i][j][4 * q + e] : (__bf16)0.f;
          *(bf16x4*)(a.k_out + ((((size_t)h * a.ntb + tb32) * 12 + d0 / 16) * 64 + en +
                                32 * ((d0 % 16) / 8)) * 8 + 4 * eg) = o;
        }
      }
    }
  }
  // rope part of K: verbatim copy, 256 tokens x 8 chunks of 16 B
#pragma unroll
  for (int i = 0; i < 8; i++) {
    const int cidx = etid + 256 * i;
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

int mfma_expand(int H, int64_t ntok, const void* c, int64_t c_stride, const void* r,
                int64_t r_stride, const void* w_uk, const void* w_uv, void* k_out, void* v_out,
                hipStream_t stream) {
  if (ntok <= 0) return TMLA_OK;
  ExpandArgs a;
  a.c = (const __bf16*)c; a.c_stride = c_stride; a.r = (const __bf16*)r; a.r_stride = r_stride;
  a.w_uk = (const __bf16*)w_uk; a.w_uv = (const __bf16*)w_uv;
  a.k_out = (__bf16*)k_out; a.v_out = (__bf16*)v_out;
  a.ntok = ntok; a.ntb = (ntok + TOK_BLK - 1) / TOK_BLK; a.H = H;
  a.tiles = (ntok + EX_TOK - 1) / EX_TOK;
  if (a.tiles * H > 0x7fffffff) return TMLA_ERR_UNSUPPORTED;
  static LdsOptIn lds;
  if (lds.ensure((const void*)expand_gemm_kernel, EX_LDS_BYTES) != hipSuccess) return TMLA_ERR_HIP;
  hipLaunchKernelGGL(expand_gemm_kernel, dim3((unsigned)(a.tiles * H)), dim3(256), EX_LDS_BYTES,
                     stream, a);
  return TMLA_OK;
}

}  // namespace tmla
