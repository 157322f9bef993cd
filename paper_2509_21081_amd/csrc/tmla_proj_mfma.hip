// The two absorb projections on the matrix cores, each fused with its neighbour step:
//   * query absorption  Q_abs = Q_nope W_UK  (paper Algorithm 1 step 5), plus the copy of the
//     RoPE part, producing the 576-wide absorbed query rows the latent attention consumes;
//   * up-projection O_A = O_lat W_UV^T (step 7) fused with the LSE combine (step 8): the latent
//     split partials are merged on the fly while they are loaded as the MFMA operand, projected,
//     then merged with the 128-wide naive partials and stored.
// Both are per-head GEMMs with the queries on the MFMA column axis (transposed products, see
// tmla_mfma.hpp), so all per-query softmax weights are per-lane scalars.
#include "tmla_common.hpp"
#include "tmla_lds_asm.hpp"
#include "tmla_mfma.hpp"

namespace tmla {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;

// ------------------------------------------------------------------ step 5
// grid (H, 4 latent quarters, ceil(M/128)); 4 wavefronts x 32 queries.  W_UK[h] is [128, 512]
// with the contraction index (noPE dim) as the row, i.e. k-major: a [128 x 128] slice is staged
// in LDS and read through the transposing LDS load to form the A operand (rows = latent columns).
constexpr int QA_ROW_BYTES = 320;  // 256 + 64: 16 banks on per row, so the 4 rows x 64 B of a transposing read (32 lanes) cover the 64 banks once

// QBK: blocks of 128 queries a workgroup takes in turn with its weight slice staged once (large
// batches: the slice would otherwise be fetched again for every 128 queries).  The fragments of
// the next block are requested right behind the MFMAs of the current one and arrive while its
// rows are turned around and stored.
template <int QBK>
__global__ void __launch_bounds__(256) qabs_kernel(const __bf16* __restrict__ q,
                                                   const __bf16* __restrict__ w_uk,
                                                   __bf16* __restrict__ qabs, int M, int H) {
  constexpr int ST_ROW = 272;   // row of the store staging: 256 + 16 B, rows stay 16-byte aligned
  __shared__ __attribute__((aligned(16))) char wt[128 * QA_ROW_BYTES];   // 40 KiB weight slice
  // store staging: its own region when the slice must survive for the next block, else the slice
  __shared__ __attribute__((aligned(16))) char st_own[QBK > 1 ? 4 * 32 * ST_ROW : 16];
  const int h = blockIdx.x, lq = blockIdx.y, qs0 = blockIdx.z * QBK;
  const int nqs = (M + 127) / 128;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, g = lane >> 5;
  // stage W_UK[h][0:128][lq*128 : lq*128+128]: 128 rows x 16 chunks of 16 B
  {
    const __bf16* src = w_uk + ((size_t)h * D_N) * D_L + lq * 128;
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const int cidx = tid + 256 * i;
      const int r = cidx >> 4, ch = cidx & 15;
      *(bf16x8*)(wt + r * QA_ROW_BYTES + ch * 16) = *(const bf16x8*)(src + (size_t)r * D_L + ch * 8);
    }
  }
  bf16x8 qf[8];
  auto load_q = [&](int qsb) __attribute__((always_inline)) {
    const int qi = (qsb * 4 + wave) * 32 + n;
    const size_t row = (size_t)(qi < M ? qi : 0) * H + h;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
      bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[ks] = qi < M ? *(const bf16x8*)(q + row * D_QK + 16 * ks + 8 * g) : z;
    }
  };
  load_q(qs0);
  __syncthreads();
  const int j16 = lane >> 4, r16 = lane & 15;
  // transposing read: contraction row 16*ks + 8*g + 4*half + r/4, latent 32*mb + 16*(j%2) + 4*(r%4)
  const int a_off = (8 * g + (r16 >> 2)) * QA_ROW_BYTES + (16 * (j16 & 1) + 4 * (r16 & 3)) * 2;
  for (int it = 0; it < QBK; it++) {
    const int qsb = qs0 + it;
    if (qsb >= nqs) break;                    // workgroup-uniform
    f32x16 acc[4];
#pragma unroll
    for (int mb = 0; mb < 4; mb++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[mb][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
#pragma unroll
      for (int mb = 0; mb < 4; mb++) {
        const char* src = wt + a_off + (16 * ks) * QA_ROW_BYTES + 64 * mb;
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(src));
        const short4v hi =
            __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(src + 4 * QA_ROW_BYTES));
        const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        acc[mb] = mfma32(__builtin_bit_cast(bf16x8, both), qf[ks], acc[mb]);
      }
    }
    if (QBK > 1 && it + 1 < QBK && qsb + 1 < nqs) load_q(qsb + 1);
    // Store through LDS: a lane holds 8-byte pieces of its query's row, 16 bytes apart from its
    // neighbour's; turned around in LDS, sixteen lanes write one query's 256 bytes of this latent
    // quarter in one piece.  With a single block the weight slice is free once everybody has
    // its fragments and serves as the staging buffer.
    if (QBK == 1) __syncthreads();
    {
      char* mine = (QBK > 1 ? st_own : wt) + wave * (32 * ST_ROW);
#pragma unroll
      for (int mb = 0; mb < 4; mb++)
#pragma unroll
        for (int v4 = 0; v4 < 4; v4++) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; e++) w[e] = (__bf16)acc[mb][4 * v4 + e];
          *(bf16x4*)(mine + n * ST_ROW + (32 * mb + 8 * v4 + 4 * g) * 2) = w;
        }
      // (each wavefront reads back only what it wrote itself: no barrier)
      const int rr = lane >> 4, ch = lane & 15;
#pragma unroll
      for (int i = 0; i < 8; i++) {
        const int r = 4 * i + rr;
        const bf16x8 w = *(const bf16x8*)(mine + r * ST_ROW + ch * 16);
        const int qq = (qsb * 4 + wave) * 32 + r;
        if (qq < M) *(bf16x8*)(qabs + ((size_t)qq * H + h) * D_ROW + lq * 128 + ch * 8) = w;
      }
    }
    if (lq == 0) {  // RoPE part: verbatim copy, 128 queries x 8 chunks
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int cidx = tid + 256 * i;
        const int qq = qsb * 128 + (cidx >> 3), ch = cidx & 7;
        if (qq < M) {
          const size_t rr = (size_t)qq * H + h;
          *(bf16x8*)(qabs + rr * D_ROW + D_L + ch * 8) = *(const bf16x8*)(q + rr * D_QK + D_N + ch * 8);
        }
      }
    }
  }
}

int mfma_query_absorb(const Plan& p, const DecodeArgs& d) {
  if (p.n_lat <= 0 || p.rows == 0) return TMLA_OK;
  const int M = p.B * p.Sq;
  const int nqs = (M + 127) / 128;
  // Four blocks of 128 queries per workgroup for large batches (measured: -13 % at 1024 queries
  // per head, nothing to gain at 256 and below), as long as the grid still covers the chip twice
  const int qbk = (nqs >= 8 && p.H * 4 * ((nqs + 3) / 4) >= 2 * NUM_CU) ? 4 : 1;
  dim3 grid(p.H, 4, (nqs + qbk - 1) / qbk);
  const __bf16* q = (const __bf16*)d.q;
  const __bf16* w = (const __bf16*)d.w_uk;
  __bf16* out = (__bf16*)(d.ws + p.off_qabs);
  if (qbk == 4) hipLaunchKernelGGL(qabs_kernel<4>, grid, dim3(256), 0, d.stream, q, w, out, M, p.H);
  else hipLaunchKernelGGL(qabs_kernel<1>, grid, dim3(256), 0, d.stream, q, w, out, M, p.H);
  return TMLA_OK;
}

// ------------------------------------------------------------------ steps 7 + 8
// grid (H, ceil(M/32)); the four wavefronts of a workgroup share 32 queries of one head and split
// the 512-wide contraction of the up-projection in four; their partial products are summed
// through LDS, after which wavefront w finishes value columns [32w, 32w+32): merge with the naive
// partials, normalise, store.
constexpr int FIN_MAX_LAT = 64;  // latent partials per row supported by the weight table in LDS
constexpr int MERGE_MAX_LAT = 128;   // ... by the separate merge pass (two per lane)
static_assert(2 * MAX_CHUNKS <= MERGE_MAX_LAT, "latent prefix + suffix chunks per request");

struct FinalizeArgs {
  const float* naive_o; const float* naive_lse; const __bf16* lat_o; const float* lat_lse;
  const __bf16* w_uv; __bf16* out; float* lse_out;
  int M, H, n_naive, n_lat;
  int64_t rows;
};

// The naive partials of a row for this lane (value columns 32 wave + 8 v4 + 4 g .. + 3), loaded
// ahead of the projection so that the epilogue does not pay a memory round trip of its own.
template <int NN>
struct NaivePrefetch {
  float lse[NN];
  f32x4 o[NN][4];
};
template <int NN>
__device__ inline void prefetch_naive(const FinalizeArgs& a, size_t row, int wave, int g,
                                      NaivePrefetch<NN>& pre) {
#pragma unroll
  for (int i = 0; i < NN; i++) {
    pre.lse[i] = a.naive_lse[(size_t)i * a.rows + row];
    const float* src = a.naive_o + ((size_t)i * a.rows + row) * D_V + 32 * wave + 4 * g;
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) pre.o[i][v4] = *(const f32x4*)(src + 8 * v4);
  }
}
// merge O_A (LSE l_a) with NN prefetched naive partials, normalise, store
template <int NN>
__device__ inline void finalize_tail_prefetched(const FinalizeArgs& a, size_t row, int wave, int g,
                                                float l_a, float (&oa)[16],
                                                const NaivePrefetch<NN>& pre) {
  float m2 = l_a;
#pragma unroll
  for (int i = 0; i < NN; i++) m2 = fmaxf(m2, pre.lse[i]);
  __bf16* dst = a.out + row * D_V + 32 * wave + 4 * g;
  if (m2 == -INFINITY) {
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      bf16x4 w = {0, 0, 0, 0};
      *(bf16x4*)(dst + 8 * v4) = w;
    }
    if (a.lse_out && wave == 0 && g == 0) a.lse_out[row] = -INFINITY;
    return;
  }
  const float w_a = (l_a > -INFINITY) ? __expf(l_a - m2) : 0.f;
  float z2 = w_a;
#pragma unroll
  for (int v = 0; v < 16; v++) oa[v] *= w_a;
#pragma unroll
  for (int i = 0; i < NN; i++) {
    // (a partial with LSE = -inf was never written: it is skipped, not multiplied by zero)
    if (pre.lse[i] == -INFINITY) continue;
    const float w = __expf(pre.lse[i] - m2);
    z2 += w;
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      const f32x4 x = pre.o[i][v4];
      oa[4 * v4] += w * x[0]; oa[4 * v4 + 1] += w * x[1];
      oa[4 * v4 + 2] += w * x[2]; oa[4 * v4 + 3] += w * x[3];
    }
  }
  const float inv2 = 1.f / z2;
#pragma unroll
  for (int v4 = 0; v4 < 4; v4++) {
    bf16x4 w;
#pragma unroll
    for (int e = 0; e < 4; e++) w[e] = (__bf16)(oa[4 * v4 + e] * inv2);
    *(bf16x4*)(dst + 8 * v4) = w;
  }
  if (a.lse_out && wave == 0 && g == 0) a.lse_out[row] = m2 + __logf(z2);
}

// Workgroup id -> (head, block of 32 queries).  The query blocks of a head read the same W_UV[h]:
// they get ids 8 apart and consecutive in that stride, so they run at the same time on one XCD
// (hardware deals consecutive ids round-robin over the 8 XCDs) and the weights come from HBM
// once.
__device__ inline bool finalize_item(const FinalizeArgs& a, int& h, int& qb) {
  const int nqb = (a.M + 31) / 32;
  const int id = blockIdx.x, x = id & 7, sl = id >> 3;
  qb = sl % nqb;
  h = (sl / nqb) * 8 + x;
  return h < a.H;
}

// Steps shared by both finalize kernels: merge O_A (LSE l_a, this wavefront's 32 value columns
// in oa) with the naive partials, normalise, store.
__device__ inline void finalize_tail(const FinalizeArgs& a, size_t row, int wave, int g, float l_a,
                                     float (&oa)[16]) {
  // merge O_A (LSE l_a) with the naive partials; this wavefront owns value block `wave`
  float m2 = l_a;
  for (int i = 0; i < a.n_naive; i++) m2 = fmaxf(m2, a.naive_lse[(size_t)i * a.rows + row]);
  __bf16* dst = a.out + row * D_V + 32 * wave + 4 * g;
  if (m2 == -INFINITY) {
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      bf16x4 w = {0, 0, 0, 0};
      *(bf16x4*)(dst + 8 * v4) = w;
    }
    if (a.lse_out && wave == 0 && g == 0) a.lse_out[row] = -INFINITY;
    return;
  }
  const float w_a = (l_a > -INFINITY) ? __expf(l_a - m2) : 0.f;
  float z2 = w_a;
#pragma unroll
  for (int v = 0; v < 16; v++) oa[v] *= w_a;
  for (int i = 0; i < a.n_naive; i++) {
    const float li = a.naive_lse[(size_t)i * a.rows + row];
    if (li == -INFINITY) continue;
    const float w = __expf(li - m2);
    z2 += w;
    const float* src = a.naive_o + ((size_t)i * a.rows + row) * D_V + 32 * wave + 4 * g;
#pragma unroll
    for (int v4 = 0; v4 < 4; v4++) {
      const float4 x = *(const float4*)(src + 8 * v4);
      oa[4 * v4] += w * x.x; oa[4 * v4 + 1] += w * x.y;
      oa[4 * v4 + 2] += w * x.z; oa[4 * v4 + 3] += w * x.w;
    }
  }
  const float inv2 = 1.f / z2;
#pragma unroll
  for (int v4 = 0; v4 < 4; v4++) {
    bf16x4 w;
#pragma unroll
    for (int e = 0; e < 4; e++) w[e] = (__bf16)(oa[4 * v4 + e] * inv2);
    *(bf16x4*)(dst + 8 * v4) = w;
  }
  if (a.lse_out && wave == 0 && g == 0) a.lse_out[row] = m2 + __logf(z2);
}

__global__ void __launch_bounds__(256) finalize_kernel(FinalizeArgs a) {
  __shared__ float wtab[FIN_MAX_LAT][32];    // normalised merge weight of each latent partial
  __shared__ float red[4][4][16][64];        // [wavefront][value block][acc register][lane]
  int h, qb;
  if (!finalize_item(a, h, qb)) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int qi = qb * 32 + n;
  const bool valid = qi < a.M;
  const size_t row = valid ? (size_t)qi * a.H + h : 0;

  float l_a = -INFINITY;
  float oa[16];   // this wavefront's 32 value columns of O_A after the cross-wavefront sum
#pragma unroll
  for (int v = 0; v < 16; v++) oa[v] = 0.f;
  if (a.n_lat > 0) {
    float mx = -INFINITY;
    for (int i = 0; i < a.n_lat; i++) mx = fmaxf(mx, a.lat_lse[(size_t)i * a.rows + row]);
    float z = 0.f;
    if (mx > -INFINITY)
      for (int i = 0; i < a.n_lat; i++) z += __expf(a.lat_lse[(size_t)i * a.rows + row] - mx);
    const float inv = (z > 0.f && valid) ? 1.f / z : 0.f;
    // every wavefront computes the same weights; wavefront 0 publishes them
    if (wave == 0 && g == 0)
      for (int i = 0; i < a.n_lat; i++)
        wtab[i][n] = (inv > 0.f) ? __expf(a.lat_lse[(size_t)i * a.rows + row] - mx) * inv : 0.f;
    if (z > 0.f && valid) l_a = mx + __logf(z);
    __syncthreads();

    f32x16 acc[4];
#pragma unroll
    for (int mb = 0; mb < 4; mb++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[mb][v] = 0.f;
    const __bf16* wp = a.w_uv + ((size_t)h * D_V + n) * D_L + 8 * g + 128 * wave;
    const __bf16* lp = a.lat_o + row * D_L + 8 * g + 128 * wave;
    for (int ks = 0; ks < 8; ks++) {
      float m8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int i = 0; i < a.n_lat; i++) {
        const float w = wtab[i][n];
        if (w > 0.f) {
          const bf16x8 x = *(const bf16x8*)(lp + (size_t)i * a.rows * D_L + 16 * ks);
#pragma unroll
          for (int e = 0; e < 8; e++) m8[e] += w * (float)x[e];
        }
      }
      bf16x8 bfrag;
#pragma unroll
      for (int e = 0; e < 8; e++) bfrag[e] = (__bf16)m8[e];
#pragma unroll
      for (int mb = 0; mb < 4; mb++) {
        const bf16x8 afrag = *(const bf16x8*)(wp + (size_t)(32 * mb) * D_L + 16 * ks);
        acc[mb] = mfma32(afrag, bfrag, acc[mb]);
      }
    }
#pragma unroll
    for (int mb = 0; mb < 4; mb++)
#pragma unroll
      for (int v = 0; v < 16; v++) red[wave][mb][v][lane] = acc[mb][v];
    __syncthreads();
#pragma unroll
    for (int v = 0; v < 16; v++)
      oa[v] = red[0][wave][v][lane] + red[1][wave][v][lane] + red[2][wave][v][lane] +
              red[3][wave][v][lane];
  }
  if (!valid) return;
  finalize_tail(a, row, wave, g, l_a, oa);
}

// Same computation for a compile-time number NL <= 4 of latent partials (the common case: the
// suffix is rarely split more).  Nothing depends on anything but the loads, so all of them --
// partial LSEs, weight fragments, latent partials -- are issued back to back and the kernel pays
// one memory round trip instead of one per k-step; the merge weights live in registers.
// NN > 0: the number of naive partials is NN and they are loaded up front with everything else
// (0: any number, loaded in the epilogue).
template <int NL, int NN>
__global__ void __launch_bounds__(256) finalize_few_kernel(FinalizeArgs a) {
  __shared__ float red[4][4][16][64];        // [wavefront][value block][acc register][lane]
  int h, qb;
  if (!finalize_item(a, h, qb)) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int qi = qb * 32 + n;
  const bool valid = qi < a.M;
  const size_t row = valid ? (size_t)qi * a.H + h : 0;

  float ll[NL];
#pragma unroll
  for (int i = 0; i < NL; i++) ll[i] = a.lat_lse[(size_t)i * a.rows + row];
  const __bf16* wp = a.w_uv + ((size_t)h * D_V + n) * D_L + 8 * g + 128 * wave;
  const __bf16* lp = a.lat_o + row * D_L + 8 * g + 128 * wave;
  bf16x8 wf[8][4];
#pragma unroll
  for (int ks = 0; ks < 8; ks++)
#pragma unroll
    for (int mb = 0; mb < 4; mb++)
      wf[ks][mb] = *(const bf16x8*)(wp + (size_t)(32 * mb) * D_L + 16 * ks);
  bf16x8 x[NL][8];
#pragma unroll
  for (int i = 0; i < NL; i++)
#pragma unroll
    for (int ks = 0; ks < 8; ks++)
      x[i][ks] = *(const bf16x8*)(lp + (size_t)i * a.rows * D_L + 16 * ks);
  NaivePrefetch<(NN > 0 ? NN : 1)> pre;
  if constexpr (NN > 0) {
    prefetch_naive(a, row, wave, g, pre);
#pragma unroll
    for (int i = 0; i < NN; i++)
      asm volatile("" : "+v"(pre.lse[i]), "+v"(pre.o[i][0]), "+v"(pre.o[i][1]), "+v"(pre.o[i][2]),
                        "+v"(pre.o[i][3]));
  }

  // pin every load above this point: without it the scheduler sinks the loads next to their
  // uses to save registers, and each k-step waits for its own round trip
#pragma unroll
  for (int ks = 0; ks < 8; ks++) {
    asm volatile("" : "+v"(wf[ks][0]), "+v"(wf[ks][1]), "+v"(wf[ks][2]), "+v"(wf[ks][3]));
#pragma unroll
    for (int i = 0; i < NL; i++) asm volatile("" : "+v"(x[i][ks]));
  }

  // merge weights of the latent partials (a partial with LSE = -inf was never written)
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < NL; i++) mx = fmaxf(mx, ll[i]);
  float w[NL], z = 0.f;
#pragma unroll
  for (int i = 0; i < NL; i++) {
    w[i] = (ll[i] > -INFINITY) ? __expf(ll[i] - mx) : 0.f;
    z += w[i];
  }
  const bool any = z > 0.f && valid;
  const float inv = any ? 1.f / z : 0.f;
  const float l_a = any ? mx + __logf(z) : -INFINITY;
#pragma unroll
  for (int i = 0; i < NL; i++) w[i] *= inv;

  f32x16 acc[4];
#pragma unroll
  for (int mb = 0; mb < 4; mb++)
#pragma unroll
    for (int v = 0; v < 16; v++) acc[mb][v] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 8; ks++) {
    bf16x8 bfrag;
    if constexpr (NL == 1) {
      // a single partial is already the merged latent output (weight 1, or 0 if it saw nothing)
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
      bfrag = w[0] > 0.f ? x[0][ks] : zero;
    } else {
      float m8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < NL; i++) {
        const bool use = w[i] > 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) m8[e] += use ? w[i] * (float)x[i][ks][e] : 0.f;
      }
#pragma unroll
      for (int e = 0; e < 8; e++) bfrag[e] = (__bf16)m8[e];
    }
#pragma unroll
    for (int mb = 0; mb < 4; mb++) acc[mb] = mfma32(wf[ks][mb], bfrag, acc[mb]);
  }
#pragma unroll
  for (int mb = 0; mb < 4; mb++)
#pragma unroll
    for (int v = 0; v < 16; v++) red[wave][mb][v][lane] = acc[mb][v];
  __syncthreads();
  float oa[16];
#pragma unroll
  for (int v = 0; v < 16; v++)
    oa[v] = red[0][wave][v][lane] + red[1][wave][v][lane] + red[2][wave][v][lane] +
            red[3][wave][v][lane];
  if (!valid) return;
  if constexpr (NN > 0) finalize_tail_prefetched(a, row, wave, g, l_a, oa, pre);
  else finalize_tail(a, row, wave, g, l_a, oa);
}

// One latent partial (the suffix is in one chunk -- every large batch) and many queries per head:
// a workgroup takes a run of consecutive blocks of 32 queries of its head with its share of
// W_UV[h] resident in registers, and the partials of a block -- 32 latent rows of 1 KiB and the
// 32 x 512 B of each naive partial -- stream through an LDS ring of whole blocks, one or two
// blocks ahead of their use.  Wavefront w owns value columns [32 w, 32 w + 32) over the whole
// contraction, so nothing is summed across wavefronts; the latent rows in LDS are shared by all
// four.  A compute unit takes in data at a limited rate and every request here is a full
// contiguous row (the per-lane fragment loads of the other kernels fetch 32 bytes per row and
// instruction), which is what this kernel is about: it is bound by memory, not by its 32 MFMAs
// per block and wavefront.
//   LDS slot: latent row r at r * 1024, its 16-byte chunk c in place c ^ (r & 15) (the reads of
//   a k-step take one chunk from each of 16 rows: the swizzle spreads them over the banks);
//   behind it naive partial i, row r at r * 512, chunk c (of 32) in place c ^ (r & 15).
// vmcnt bookkeeping: a block's transfers are the youngest memory operations but for the
// transfers of the blocks behind it, so "at most TPW * (FS_NSLOT - 2) in flight" means it landed
// (stores in between only make the wait stricter).
constexpr int FS_X_BYTES = 32 * 1024;
constexpr int FS_N_BYTES = 32 * 512;
template <int NN>
struct FsLayout {
  static constexpr int NSLOT = NN == 1 ? 3 : 2;
  static constexpr int SLOT = FS_X_BYTES + NN * FS_N_BYTES;
  static constexpr int BYTES = NSLOT * SLOT;     // 144 KiB (one naive partial), 128 KiB (two)
  static constexpr int TPW = 8 + 4 * NN;         // transfers per wavefront and block
};

template <int NN>
__global__ void __launch_bounds__(256, 1) finalize_stream_kernel(FinalizeArgs a, int qbk) {
  using L = FsLayout<NN>;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int nqb = (a.M + 31) / 32, ngrp = (nqb + qbk - 1) / qbk;
  const int id = blockIdx.x, sl = id >> 3;
  const int qg = sl % ngrp, h = (sl / ngrp) * 8 + (id & 7);   // groups of a head: same XCD
  if (h >= a.H) return;
  const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qb0 = qg * qbk, nblk = min(qbk, nqb - qb0);

  auto row_of = [&](int qb, int r) {
    const int qi = qb * 32 + r;
    return qi < a.M ? (size_t)qi * a.H + h : (size_t)h;
  };
  // the transfers of block qb into ring slot `slot` issued by this wavefront: latent rows
  // wave, wave + 4, ...; pairs of naive rows 2 t, 2 t + 1 for t = wave, wave + 4, ...
  auto issue_block = [&](int qb, int slot) __attribute__((always_inline)) {
    char* dst = smem + slot * L::SLOT;
#pragma unroll
    for (int k = 0; k < 8; k++) {
      const int r = wave + 4 * k;
      const char* src = (const char*)(a.lat_o + row_of(qb, r) * D_L);
      dma16(src + ((lane ^ (r & 15)) << 4), dst + r * 1024);
    }
#pragma unroll
    for (int i = 0; i < NN; i++)
#pragma unroll
      for (int k = 0; k < 4; k++) {
        const int t = wave + 4 * k, r = 2 * t + g;
        const char* src = (const char*)(a.naive_o + ((size_t)i * a.rows + row_of(qb, r)) * D_V);
        dma16(src + ((n ^ (r & 15)) << 4), dst + FS_X_BYTES + i * FS_N_BYTES + t * 1024);
      }
  };
  struct Lse { float lat, naive[NN]; };
  auto load_lse = [&](int qb, Lse& l) __attribute__((always_inline)) {
    const size_t row = row_of(qb, n);
    l.lat = a.lat_lse[row];
#pragma unroll
    for (int i = 0; i < NN; i++) l.naive[i] = a.naive_lse[(size_t)i * a.rows + row];
  };

  // W_UV[h][32 wave + n][16 ks + 8 g ..]: the A fragments of all 32 k-steps
  bf16x8 wf[32];
  {
    const __bf16* wp = a.w_uv + ((size_t)h * D_V + 32 * wave + n) * D_L + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 32; ks++) wf[ks] = *(const bf16x8*)(wp + 16 * ks);
  }
  Lse lse_cur, lse_next;
  load_lse(qb0, lse_cur);
  lse_next = lse_cur;
#pragma unroll
  for (int j = 0; j < L::NSLOT - 1; j++)
    if (j < nblk) issue_block(qb0 + j, j);

  const uint32_t smem_base = lds_addr(smem);
  const uint32_t x_lane = n * 1024 + ((g ^ (n & 15)) << 4);
  const uint32_t n_lane = FS_X_BYTES + n * 512;
  int slot = 0;
  for (int it = 0; it < nblk; it++) {
    const int qb = qb0 + it;
    // block `it` has landed when only the transfers of the blocks behind it are in flight
    if (L::NSLOT == 3 && it + 1 < nblk) vm_wait<L::TPW>();
    else vm_wait<0>();
    raw_barrier();   // everybody's part of the block is there; everybody is done with block it - 1
    if (it + 1 < nblk) load_lse(qb + 1, lse_next);
    if (it + L::NSLOT - 1 < nblk) {
      int fill = slot - 1;
      if (fill < 0) fill += L::NSLOT;
      issue_block(qb + L::NSLOT - 1, fill);
    }
    const uint32_t sb = smem_base + slot * L::SLOT;
    const bool valid = qb * 32 + n < a.M;
    // a single partial is already the merged latent output (weight 1, or 0 if it saw nothing:
    // then its row was never written and is replaced by zeros)
    const bool any = lse_cur.lat > -INFINITY && valid;
    const float l_a = any ? lse_cur.lat : -INFINITY;

    // ---- up-projection: fragments through a ring of eight registers, eight reads ahead
    uint32_t xa[8];
#pragma unroll
    for (int j = 0; j < 8; j++) xa[j] = (sb + x_lane) ^ (j << 5);
    bf16x8 fr[8];
    static_for<8>([&](auto j_) {
      constexpr int j = decltype(j_)::value;
      fr[j] = lds_read_b128<0>(xa[j]);
    });
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; v++) acc[v] = 0.f;
    static_for<32>([&](auto ks_) {
      constexpr int ks = decltype(ks_)::value;
      constexpr int later = 31 - ks < 7 ? 31 - ks : 7;
      lgkm_wait<later>(fr[ks % 8]);
      const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
      const bf16x8 bfrag = any ? fr[ks % 8] : zero;
      acc = mfma32(wf[ks], bfrag, acc);
      if constexpr (ks + 8 < 32) fr[ks % 8] = lds_read_b128<256 * ((ks + 8) >> 3)>(xa[ks % 8]);
    });

    // ---- the naive partials of this lane's value columns, then merge, normalise, store
    NaivePrefetch<NN> pre;
#pragma unroll
    for (int i = 0; i < NN; i++) {
      pre.lse[i] = lse_cur.naive[i];
#pragma unroll
      for (int v4 = 0; v4 < 4; v4++) {
        const int c = 8 * wave + 2 * v4 + g;
        pre.o[i][v4] = lds_read_f32x4(sb + n_lane + i * FS_N_BYTES + ((c ^ (n & 15)) << 4));
      }
    }
    float oa[16];
#pragma unroll
    for (int v = 0; v < 16; v++) oa[v] = acc[v];
#pragma unroll
    for (int i = 0; i < NN; i++)
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(pre.o[i][0]), "+v"(pre.o[i][1]), "+v"(pre.o[i][2]), "+v"(pre.o[i][3])
                   :: "memory");
    if (valid) finalize_tail_prefetched(a, row_of(qb, n), wave, g, l_a, oa, pre);
    lse_cur = lse_next;
    slot = slot + 1 == L::NSLOT ? 0 : slot + 1;
  }
}

template <int NN>
static int launch_finalize_stream(const FinalizeArgs& a, int heads8, int nqb, int qbk,
                                  hipStream_t stream) {
  static LdsOptIn lds;
  if (lds.ensure((const void*)finalize_stream_kernel<NN>, FsLayout<NN>::BYTES) != hipSuccess)
    return TMLA_ERR_HIP;
  dim3 grid(heads8 * ((nqb + qbk - 1) / qbk));
  hipLaunchKernelGGL(finalize_stream_kernel<NN>, grid, dim3(256), FsLayout<NN>::BYTES, stream, a,
                     qbk);
  return TMLA_OK;
}

template <int NL>
static void launch_finalize_few(const FinalizeArgs& a, dim3 grid, hipStream_t stream) {
  // The prefetch costs 34 registers, which halves the wavefronts per SIMD: it pays only where a
  // compute unit gets so few workgroups that latency, not occupancy, sets the time.
  const bool few_wgs = grid.x <= 2 * NUM_CU;
  switch (few_wgs ? a.n_naive : 0) {
    case 1: hipLaunchKernelGGL((finalize_few_kernel<NL, 1>), grid, dim3(256), 0, stream, a); break;
    case 2: hipLaunchKernelGGL((finalize_few_kernel<NL, 2>), grid, dim3(256), 0, stream, a); break;
    default: hipLaunchKernelGGL((finalize_few_kernel<NL, 0>), grid, dim3(256), 0, stream, a);
  }
}

// More than four latent partials per row -- a small batch whose long prefix (absorb_only) or
// suffix is cut into many chunks so that the pass fills the chip -- are merged by a pass of its
// own into partial 0, after which the up-projection sees a single partial.  Merging inside the
// projection kernel walks the partials one dependent load after the other, for 32 query
// columns of which a small batch fills one or two: 53-110 us at batch 1-8 against 4-8 us here.
// One workgroup per row: the partials are dealt out to the four wavefronts (i = w, w + 4, ...),
// a wavefront reads a partial row as one contiguous KiB (lane = 16-byte chunk) eight at a time,
// the four sums meet in LDS.  Lane i holds the LSEs and the weights of partials i and i + 64 (at
// most MERGE_MAX_LAT = 128 partials).  A partial with LSE = -inf was never written and is skipped.
__global__ void __launch_bounds__(256) merge_latent_kernel(__bf16* lat_o, float* lat_lse,
                                                           int n_lat, int64_t rows) {
  __shared__ float part[4][64][8];
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  float li[2], e[2], wgt[2];
#pragma unroll
  for (int k = 0; k < 2; k++)
    li[k] = lane + 64 * k < n_lat ? lat_lse[(size_t)(lane + 64 * k) * rows + row] : -INFINITY;
  float mx = fmaxf(li[0], li[1]);
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) mx = fmaxf(mx, __shfl_xor(mx, s));
#pragma unroll
  for (int k = 0; k < 2; k++) e[k] = mx > -INFINITY && li[k] > -INFINITY ? __expf(li[k] - mx) : 0.f;
  float z = e[0] + e[1];
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) z += __shfl_xor(z, s);
#pragma unroll
  for (int k = 0; k < 2; k++) wgt[k] = z > 0.f ? e[k] / z : 0.f;   // normalised weights
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const __bf16* src = lat_o + (size_t)row * D_L + lane * 8;
  for (int i0 = wave; i0 < n_lat; i0 += 32) {
    bf16x8 x[8];
    float w[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
      const int i = i0 + 4 * j;
      w[j] = i < n_lat ? __shfl(i < 64 ? wgt[0] : wgt[1], i & 63) : 0.f;   // wave-uniform
      if (w[j] > 0.f) x[j] = *(const bf16x8*)(src + (size_t)i * rows * D_L);
    }
#pragma unroll
    for (int j = 0; j < 8; j++)
      if (w[j] > 0.f) {
#pragma unroll
        for (int k = 0; k < 8; k++) acc[k] += w[j] * (float)x[j][k];
      }
  }
#pragma unroll
  for (int k = 0; k < 8; k++) part[wave][lane][k] = acc[k];
  __syncthreads();   // every wavefront has read what it needs of partial 0 as well
  if (wave == 0) {
    bf16x8 o;
#pragma unroll
    for (int k = 0; k < 8; k++)
      o[k] = (__bf16)(part[0][lane][k] + part[1][lane][k] + part[2][lane][k] + part[3][lane][k]);
    *(bf16x8*)(lat_o + (size_t)row * D_L + lane * 8) = o;
    if (lane == 0) lat_lse[row] = z > 0.f ? mx + __logf(z) : -INFINITY;
  }
}

int mfma_finalize(const Plan& p, const DecodeArgs& d) {
  if (p.rows == 0) return TMLA_OK;
  const bool merge_inside = (debug_flags() & 0x10000) != 0;   // debug: no separate merge pass
  if (p.n_lat > (merge_inside ? FIN_MAX_LAT : MERGE_MAX_LAT)) return TMLA_ERR_UNSUPPORTED;
  FinalizeArgs a;
  a.naive_o = (const float*)(d.ws + p.off_naive_o);
  a.naive_lse = (const float*)(d.ws + p.off_naive_lse);
  a.lat_o = (const __bf16*)(d.ws + p.off_lat_o);
  a.lat_lse = (const float*)(d.ws + p.off_lat_lse);
  a.w_uv = (const __bf16*)d.w_uv;
  a.out = (__bf16*)d.out;
  a.lse_out = d.lse_out;
  a.M = p.B * p.Sq; a.H = p.H; a.n_naive = p.n_naive; a.n_lat = p.n_lat; a.rows = p.rows;
  if (a.n_lat > 4 && !merge_inside) {
    hipLaunchKernelGGL(merge_latent_kernel, dim3((unsigned)p.rows), dim3(256), 0, d.stream,
                       (__bf16*)(d.ws + p.off_lat_o), (float*)(d.ws + p.off_lat_lse), a.n_lat,
                       (int64_t)p.rows);
    a.n_lat = 1;
  }
  // one latent partial, one or two naive partials, and at least two blocks of 32 queries per
  // compute unit: runs of up to eight blocks per workgroup, so that the grid still covers the chip
  if (a.n_lat == 1 && (p.n_naive == 1 || p.n_naive == 2)) {
    const int nqb = (a.M + 31) / 32;
    const int heads8 = (p.H + 7) / 8 * 8;
    const long long per_cu = (long long)heads8 * nqb / NUM_CU;
    const int qbk = (int)(per_cu > 8 ? 8 : per_cu);
    if (qbk >= 2)
      return p.n_naive == 1 ? launch_finalize_stream<1>(a, heads8, nqb, qbk, d.stream)
                            : launch_finalize_stream<2>(a, heads8, nqb, qbk, d.stream);
  }
  dim3 grid(8 * ((a.M + 31) / 32) * ((p.H + 7) / 8));
  switch (a.n_lat) {
    case 1: launch_finalize_few<1>(a, grid, d.stream); break;
    case 2: launch_finalize_few<2>(a, grid, d.stream); break;
    case 3: launch_finalize_few<3>(a, grid, d.stream); break;
    case 4: launch_finalize_few<4>(a, grid, d.stream); break;
    default: hipLaunchKernelGGL(finalize_kernel, grid, dim3(256), 0, d.stream, a);
  }
  return TMLA_OK;
}

}  // namespace tmla
