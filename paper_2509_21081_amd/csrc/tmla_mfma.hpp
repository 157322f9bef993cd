// Matrix-core (MFMA) building blocks shared by the gfx950 kernels.
//
// v_mfma_f32_32x32x16_bf16 operand layout (64-lane wavefront, lane = n + 32*g, n in [0,32)):
//   A (32 x 16): lane holds row n,    k = 8*g + e, e in [0,8)
//   B (16 x 32): lane holds column n, k = 8*g + e
//   D (32 x 32): lane holds column n, rows 8*(v/4) + 4*g + v%4 for v in [0,16)
// The attention kernels compute transposed products (tokens on the MFMA row axis, queries on the
// column axis): S^T = K Q^T and O^T = V^T P^T.  Each lane then owns one query column, so the
// softmax statistics are per-lane scalars, and the D layout of S^T regrouped as k = 8*g + e is
// directly a B operand of the second product once the V^T operand uses the same token order.
#pragma once
#include <hip/hip_runtime.h>

namespace tmla {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float RESCALE_TAU = 8.f;   // softmax_block_fast assumes 2^(RESCALE_TAU + 4) = 4096

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// value held by the lane 32 positions away (lane ^ 32)
__device__ inline float other_half(float x) {
  const int xi = __float_as_int(x);
  auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  // r[0] = {x.lo, x.lo}, r[1] = {x.hi, x.hi} over the two 32-lane halves
  return __int_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ inline float max_halves(float x) {
  const int xi = __float_as_int(x);
  auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
}
__device__ inline float sum_halves(float x) {
  const int xi = __float_as_int(x);
  auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return __int_as_float(r[0]) + __int_as_float(r[1]);
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// row (token) index inside a 32-row MFMA result held in accumulator register v by lane-half g
__device__ inline int acc_row(int v, int g) { return 8 * (v >> 2) + 4 * g + (v & 3); }

// Online-softmax update for one 32-token block and one 32-query column block.
//   s      : S^T accumulator (raw dot products); on return holds nothing useful
//   m, l   : exponent reference (log2 domain, scaled; >= running max - RESCALE_TAU) and this
//            lane's partial denominator relative to it
//   c      : sm_scale * log2(e)
//   limit  : rows with acc_row >= limit are masked out (pass 32 for a full block); with
//            MASK = false the block is known to be full and no masking code is emitted
//   p0, p1 : the probabilities as bf16 B operands for the two 16-token k-steps
// Returns the factor by which the caller must rescale its output accumulators (1 if unchanged);
// `rescale` is wave-uniform and tells whether any lane needs it.
template <bool MASK = true>
__device__ __forceinline__ float softmax_block(f32x16& s, float& m, float& l, float c, int limit, int g,
                                      bf16x8& p0, bf16x8& p1, bool& rescale) {
  if (MASK && limit < 32) {
#pragma unroll
    for (int v = 0; v < 16; v++)
      if (acc_row(v, g) >= limit) s[v] = -INFINITY;
  }
  float mx = s[0];
#pragma unroll
  for (int v = 1; v < 16; v++) mx = fmaxf(mx, s[v]);
  mx = max_halves(mx) * c;
  // Lazy reference update: `m` is the exponent reference, not necessarily the running maximum.
  // It only moves when the block maximum exceeds it by more than RESCALE_TAU (log2 units), so
  // probabilities stay below 2^RESCALE_TAU and the costly rescale of the output accumulators
  // becomes rare.  The result is unchanged: numerator and denominator share the reference.
  const float m_new = (mx > m + RESCALE_TAU) ? mx : m;
  const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
  float alpha = 1.f;
  rescale = __builtin_amdgcn_ballot_w64(m_new > m) != 0;
  if (rescale) {
    alpha = fast_exp2(m - m_use);   // m = -inf -> 0
    l *= alpha;
  }
  m = m_new;
  float sum = 0.f;
#pragma unroll
  for (int v = 0; v < 8; v++) {
    const float p = fast_exp2(__builtin_fmaf(s[v], c, -m_use));
    sum += p;
    p0[v] = (__bf16)p;
  }
#pragma unroll
  for (int v = 0; v < 8; v++) {
    const float p = fast_exp2(__builtin_fmaf(s[8 + v], c, -m_use));
    sum += p;
    p1[v] = (__bf16)p;
  }
  l += sum;
  return alpha;
}

// Same contract as softmax_block, for blocks known to be full (no masking), with a shortcut for
// the common case that the exponent reference is still good: the probabilities are formed
// against the current reference straight away, and their per-lane sum doubles as the range
// check: no probability can exceed a sum that stays below 2^(RESCALE_TAU + 4).  Then neither the
// block maximum nor the exchange between the lane halves is needed.  Otherwise (first block, or
// a score far above the reference) the scores are still intact and the full update runs.  The
// sum is taken over the unrounded exponentials: the bf16 rounding of a dominant probability
// (relative 2^-9) would otherwise go straight into the denominator and the LSE.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ inline float softmax_block_fast(f32x16& s, float& m, float& l, float c, int g,
                                           bf16x8& p0, bf16x8& p1, bool& rescale) {
  bf16x8 q0, q1;
  float sum = 0.f;
#pragma unroll
  for (int v = 0; v < 8; v++) {
    const float e0 = fast_exp2(__builtin_fmaf(s[v], c, -m));       // m = -inf gives inf: falls through
    const float e1 = fast_exp2(__builtin_fmaf(s[8 + v], c, -m));
    sum += e0 + e1;
    q0[v] = (__bf16)e0;
    q1[v] = (__bf16)e1;
  }
  const bool good = sum <= 16.f * 256.f;   // 2^(RESCALE_TAU + 4); false for inf and NaN
  if (__builtin_amdgcn_ballot_w64(!good) == 0) {
    l += sum;
    p0 = q0;
    p1 = q1;
    rescale = false;
    return 1.f;
  }
  return softmax_block<false>(s, m, l, c, 32, g, p0, p1, rescale);
}

}  // namespace tmla
