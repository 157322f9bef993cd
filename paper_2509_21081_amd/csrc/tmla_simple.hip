// Scalar (non matrix-core) HIP kernels for every step of the decode path.  They are the fp32
// implementation and a second, independent GPU implementation of the bf16 path used to bring up
// and cross-check the matrix-core kernels.  fp32 accumulation everywhere.
//
// Steps (paper Algorithm 1): prefix expansion (Section 3.1 "Prefill"), naive attention over
// expanded K/V (step 4), query absorption q_nope W_UK (step 5), absorb attention over latent
// rows (step 6), up-projection by W_UV (step 7) and the LSE combine (step 8).
#include "tmla_common.hpp"

namespace tmla {

constexpr int NT = 128;  // threads per block in the attention kernels

__device__ inline float block_reduce_max(float v, float* red) {
  const int tid = threadIdx.x;
  red[tid] = v;
  __syncthreads();
  for (int s = NT / 2; s > 0; s >>= 1) {
    if (tid < s) red[tid] = fmaxf(red[tid], red[tid + s]);
    __syncthreads();
  }
  const float r = red[0];
  __syncthreads();
  return r;
}
__device__ inline float block_reduce_sum(float v, float* red) {
  const int tid = threadIdx.x;
  red[tid] = v;
  __syncthreads();
  for (int s = NT / 2; s > 0; s >>= 1) {
    if (tid < s) red[tid] += red[tid + s];
    __syncthreads();
  }
  const float r = red[0];
  __syncthreads();
  return r;
}

// One softmax-attention pass of a single query vector (in LDS, fp32) over tokens [t0, t1).
// kf(t, i): key element i of token t; vf(t, d): value element d.  Writes the normalised partial
// output (DV values of type OT) and its natural-log LSE; an empty range writes LSE = -inf only.
template <int DK, int DV, typename OT, typename KF, typename VF>
__device__ void attend_range(const float* q_lds, int t0, int t1, float scale, KF kf, VF vf,
                             OT* o_out, float* lse_out) {
  __shared__ float p_lds[NT];
  __shared__ float red[NT];
  constexpr int VPT = DV / NT;
  const int tid = threadIdx.x;
  float acc[VPT];
  for (int c = 0; c < VPT; c++) acc[c] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  for (int base = t0; base < t1; base += NT) {
    const int t = base + tid;
    float s = -INFINITY;
    if (t < t1) {
      float dot = 0.f;
      for (int i = 0; i < DK; i++) dot += q_lds[i] * kf(t, i);
      s = dot * scale;
    }
    const float m_tile = block_reduce_max(s, red);
    const float m_new = fmaxf(m_run, m_tile);
    const float p = (t < t1) ? expf(s - m_new) : 0.f;
    const float alpha = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
    p_lds[tid] = p;
    const float l_tile = block_reduce_sum(p, red);  // also publishes p_lds
    l_run = l_run * alpha + l_tile;
    const int n = min(NT, t1 - base);
    for (int c = 0; c < VPT; c++) {
      const int d = tid + c * NT;
      float a = acc[c] * alpha;
      for (int j = 0; j < n; j++) a += p_lds[j] * vf(base + j, d);
      acc[c] = a;
    }
    m_run = m_new;
    __syncthreads();
  }
  if (t1 > t0) {
    const float inv = 1.f / l_run;
    for (int c = 0; c < VPT; c++) o_out[tid + c * NT] = from_float<OT>(acc[c] * inv);
    if (tid == 0) *lse_out = m_run + logf(l_run);
  } else if (tid == 0) {
    *lse_out = -INFINITY;
  }
}

__device__ inline int visible_suffix(int len_b, int q_len, int s) {
  return max(0, min(len_b, len_b - q_len + s + 1));
}

// ---------------------------------------------------------------- prefix / pool expansion
template <typename T>
__global__ void __launch_bounds__(256)
simple_expand_kernel(int H, int64_t ntok, const T* __restrict__ c, int64_t c_stride,
                     const T* __restrict__ r, int64_t r_stride, const T* __restrict__ w_uk,
                     const T* __restrict__ w_uv, T* __restrict__ k_out, T* __restrict__ v_out) {
  __shared__ float c_lds[D_L];
  const int64_t t = blockIdx.x;
  const int h = blockIdx.y;
  const int tid = threadIdx.x;
  for (int i = tid; i < D_L; i += 256) c_lds[i] = to_float(c[t * c_stride + i]);
  __syncthreads();
  const T* w = (tid < D_N) ? w_uk + ((size_t)h * D_N + tid) * D_L
                           : w_uv + ((size_t)h * D_V + (tid - D_N)) * D_L;
  float acc = 0.f;
  for (int l = 0; l < D_L; l++) acc += to_float(w[l]) * c_lds[l];
  if (tid < D_N) k_out[ExpLayout<T>::k(h, ntok, t, tid)] = from_float<T>(acc);
  else v_out[ExpLayout<T>::v(h, ntok, t, tid - D_N)] = from_float<T>(acc);
  if (tid < D_R) k_out[ExpLayout<T>::k(h, ntok, t, D_N + tid)] = r[t * r_stride + tid];
}

// zero the padding tokens [ntok, roundup(ntok, 32)) of the bf16 tiled layout
__global__ void expand_pad_kernel(int H, int64_t ntok, bf16_t* k_out, bf16_t* v_out) {
  const int64_t ntb = (ntok + TOK_BLK - 1) / TOK_BLK;
  const int h = blockIdx.x;
  bf16_t z; z.x = 0;
  for (int64_t t = ntok; t < ntb * TOK_BLK; t++) {
    // ExpLayout formulas only use t / 32 and t % 32, so padded token indices address correctly
    for (int d = threadIdx.x; d < D_QK; d += blockDim.x)
      k_out[ExpLayout<bf16_t>::k(h, ntb * TOK_BLK, t, d)] = z;
    for (int d = threadIdx.x; d < D_V; d += blockDim.x)
      v_out[ExpLayout<bf16_t>::v(h, ntb * TOK_BLK, t, d)] = z;
  }
}

template <typename T>
void simple_expand(int H, int64_t ntok, const T* c, int64_t c_stride, const T* r, int64_t r_stride,
                   const T* w_uk, const T* w_uv, T* k_out, T* v_out, hipStream_t stream) {
  if (ntok <= 0) return;
  // grid.x is limited to 2^31-1 blocks; token counts here are far below that
  dim3 grid((unsigned)ntok, (unsigned)H);
  hipLaunchKernelGGL(simple_expand_kernel<T>, grid, dim3(256), 0, stream, H, ntok, c, c_stride, r,
                     r_stride, w_uk, w_uv, k_out, v_out);
  if constexpr (sizeof(T) == 2) {
    if (ntok % TOK_BLK)
      hipLaunchKernelGGL(expand_pad_kernel, dim3(H), dim3(64), 0, stream, H, ntok,
                         (bf16_t*)k_out, (bf16_t*)v_out);
  }
}
template void simple_expand<float>(int, int64_t, const float*, int64_t, const float*, int64_t,
                                   const float*, const float*, float*, float*, hipStream_t);
template void simple_expand<bf16_t>(int, int64_t, const bf16_t*, int64_t, const bf16_t*, int64_t,
                                    const bf16_t*, const bf16_t*, bf16_t*, bf16_t*, hipStream_t);

// ---------------------------------------------------------------- step 5: q_abs = q_nope W_UK
template <typename T>
__global__ void __launch_bounds__(256)
simple_qabs_kernel(int H, const T* __restrict__ q, const T* __restrict__ w_uk,
                   T* __restrict__ qabs) {
  __shared__ float qn[D_N];
  const int64_t row = blockIdx.x;
  const int h = (int)(row % H);
  const int tid = threadIdx.x;
  if (tid < D_N) qn[tid] = to_float(q[row * D_QK + tid]);
  __syncthreads();
  for (int l = tid; l < D_L; l += 256) {
    float acc = 0.f;
    for (int i = 0; i < D_N; i++) acc += qn[i] * to_float(w_uk[((size_t)h * D_N + i) * D_L + l]);
    qabs[row * D_ROW + l] = from_float<T>(acc);
  }
  if (tid < D_R) qabs[row * D_ROW + D_L + tid] = q[row * D_QK + D_N + tid];
}

// ---------------------------------------------------------------- step 4: naive attention
// grid (rows, chunks).  Chunks [0, np_split) cover the shared prefix; chunks beyond (naive_only)
// cover the request's own expanded paged suffix.
template <typename T>
__global__ void __launch_bounds__(NT)
simple_naive_kernel(Plan p, const T* __restrict__ q, const T* __restrict__ pk,
                    const T* __restrict__ pv, const T* __restrict__ sk, const T* __restrict__ sv,
                    const int32_t* __restrict__ block_table, const int32_t* __restrict__ lens,
                    int max_blocks, int block_size, int64_t pool_tokens, float scale,
                    float* __restrict__ naive_o, float* __restrict__ naive_lse, int first_chunk) {
  __shared__ float q_lds[D_QK];
  const int64_t row = blockIdx.x;
  const int chunk = first_chunk + blockIdx.y;
  const int h = (int)(row % p.H);
  const int s = (int)((row / p.H) % p.Sq);
  const int b = (int)(row / ((int64_t)p.H * p.Sq));
  for (int i = threadIdx.x; i < D_QK; i += NT) q_lds[i] = to_float(q[row * D_QK + i]);
  __syncthreads();
  float* o_out = naive_o + ((size_t)chunk * p.rows + row) * D_V;
  float* l_out = naive_lse + (size_t)chunk * p.rows + row;
  if (chunk < p.np_split) {
    const int t0 = chunk * p.p_chunk, t1 = min(p.Ls, t0 + p.p_chunk);
    const int64_t ntok = p.Ls;
    attend_range<D_QK, D_V, float>(
        q_lds, t0, t1, scale,
        [=](int t, int i) { return to_float(pk[ExpLayout<T>::k(h, ntok, t, i)]); },
        [=](int t, int d) { return to_float(pv[ExpLayout<T>::v(h, ntok, t, d)]); }, o_out, l_out);
  } else {
    const int c = chunk - p.np_split;
    const int vis = visible_suffix(lens[b], p.Sq, s);
    const int t0 = min(vis, c * p.ns_chunk), t1 = min(vis, t0 + p.ns_chunk);
    const int32_t* bt = block_table + (size_t)b * max_blocks;
    auto phys = [=](int j) { return (int64_t)bt[j / block_size] * block_size + j % block_size; };
    attend_range<D_QK, D_V, float>(
        q_lds, t0, t1, scale,
        [=](int j, int i) { return to_float(sk[ExpLayout<T>::k(h, pool_tokens, phys(j), i)]); },
        [=](int j, int d) { return to_float(sv[ExpLayout<T>::v(h, pool_tokens, phys(j), d)]); },
        o_out, l_out);
  }
}

// ---------------------------------------------------------------- step 6: absorb attention
// grid (rows, n_lat).  Items [0, ap_chunks) run over the latent prefix (absorb_only), the rest
// over the request's paged suffix rows.
template <typename T>
__global__ void __launch_bounds__(NT)
simple_absorb_kernel(Plan p, const T* __restrict__ qabs, const T* __restrict__ pc,
                     const T* __restrict__ pr, const T* __restrict__ pool,
                     const int32_t* __restrict__ block_table, const int32_t* __restrict__ lens,
                     int max_blocks, int block_size, float scale, T* __restrict__ lat_o,
                     float* __restrict__ lat_lse) {
  __shared__ float q_lds[D_ROW];
  const int64_t row = blockIdx.x;
  const int item = blockIdx.y;
  const int s = (int)((row / p.H) % p.Sq);
  const int b = (int)(row / ((int64_t)p.H * p.Sq));
  for (int i = threadIdx.x; i < D_ROW; i += NT) q_lds[i] = to_float(qabs[row * D_ROW + i]);
  __syncthreads();
  T* o_out = lat_o + ((size_t)item * p.rows + row) * D_L;
  float* l_out = lat_lse + (size_t)item * p.rows + row;
  if (item < p.ap_chunks) {
    const int t0 = min(p.Ls, item * p.ap_chunk), t1 = min(p.Ls, t0 + p.ap_chunk);
    attend_range<D_ROW, D_L, T>(
        q_lds, t0, t1, scale,
        [=](int t, int i) {
          return i < D_L ? to_float(pc[(size_t)t * D_L + i]) : to_float(pr[(size_t)t * D_R + i - D_L]);
        },
        [=](int t, int d) { return to_float(pc[(size_t)t * D_L + d]); }, o_out, l_out);
  } else {
    const int c = item - p.ap_chunks;
    const int vis = visible_suffix(lens[b], p.Sq, s);
    const int t0 = min(vis, c * p.as_chunk), t1 = min(vis, t0 + p.as_chunk);
    const int32_t* bt = block_table + (size_t)b * max_blocks;
    auto rowp = [=](int j) {
      return pool + ((size_t)bt[j / block_size] * block_size + j % block_size) * D_ROW;
    };
    attend_range<D_ROW, D_L, T>(
        q_lds, t0, t1, scale, [=](int j, int i) { return to_float(rowp(j)[i]); },
        [=](int j, int d) { return to_float(rowp(j)[d]); }, o_out, l_out);
  }
}

// ---------------------------------------------------------------- steps 7 + 8
// Per output row: merge the latent partials, up-project through W_UV[h], then merge with the
// 128-wide naive partials and store.
template <typename T>
__global__ void __launch_bounds__(NT)
simple_finalize_kernel(Plan p, const float* __restrict__ naive_o,
                       const float* __restrict__ naive_lse, const T* __restrict__ lat_o,
                       const float* __restrict__ lat_lse, const T* __restrict__ w_uv,
                       T* __restrict__ out, float* __restrict__ lse_out) {
  __shared__ float lat[D_L];
  const int64_t row = blockIdx.x;
  const int h = (int)(row % p.H);
  const int tid = threadIdx.x;
  float l_a = -INFINITY, o_a = 0.f;
  if (p.n_lat > 0) {
    float m = -INFINITY;
    for (int i = 0; i < p.n_lat; i++) m = fmaxf(m, lat_lse[(size_t)i * p.rows + row]);
    if (m > -INFINITY) {
      float z = 0.f, acc[D_L / NT] = {0.f, 0.f, 0.f, 0.f};
      for (int i = 0; i < p.n_lat; i++) {
        const float li = lat_lse[(size_t)i * p.rows + row];
        if (li == -INFINITY) continue;
        const float w = expf(li - m);
        z += w;
        const T* src = lat_o + ((size_t)i * p.rows + row) * D_L;
        for (int c = 0; c < D_L / NT; c++) acc[c] += w * to_float(src[tid + c * NT]);
      }
      const float inv = 1.f / z;
      // the latent output passes through the I/O dtype before the up-projection, as it does
      // when the absorb output is materialised between Algorithm 1 steps 6 and 7
      for (int c = 0; c < D_L / NT; c++)
        lat[tid + c * NT] = to_float(from_float<T>(acc[c] * inv));
      l_a = m + logf(z);
      __syncthreads();
      const T* w = w_uv + ((size_t)h * D_V + tid) * D_L;
      float a = 0.f;
      for (int l = 0; l < D_L; l++) a += to_float(w[l]) * lat[l];
      o_a = a;
    }
  }
  float m = l_a;
  for (int i = 0; i < p.n_naive; i++) m = fmaxf(m, naive_lse[(size_t)i * p.rows + row]);
  if (m == -INFINITY) {
    out[row * D_V + tid] = from_float<T>(0.f);
    if (lse_out && tid == 0) lse_out[row] = -INFINITY;
    return;
  }
  float z = 0.f, num = 0.f;
  if (l_a > -INFINITY) { const float w = expf(l_a - m); z += w; num += w * o_a; }
  for (int i = 0; i < p.n_naive; i++) {
    const float li = naive_lse[(size_t)i * p.rows + row];
    if (li == -INFINITY) continue;
    const float w = expf(li - m);
    z += w;
    num += w * naive_o[((size_t)i * p.rows + row) * D_V + tid];
  }
  out[row * D_V + tid] = from_float<T>(num / z);
  if (lse_out && tid == 0) lse_out[row] = m + logf(z);
}

__global__ void fill_f32_kernel(float* p, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
void launch_fill_f32(float* p, int64_t n, float v, hipStream_t stream) {
  if (n <= 0) return;
  hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n, v);
}

// `grid_rows` < 0: all p.rows rows; otherwise only the first grid_rows rows behind the (already
// offset) query and partial pointers, p.rows staying the stride between chunks
template <typename T>
void simple_stage_naive(const Plan& p, const DecodeArgs& a, int first_chunk, int n_chunks,
                        int64_t grid_rows) {
  if (grid_rows < 0) grid_rows = p.rows;
  if (grid_rows == 0 || n_chunks <= 0) return;
  const int64_t pool_tokens = (int64_t)a.num_blocks * a.block_size;
  hipLaunchKernelGGL(simple_naive_kernel<T>, dim3((unsigned)grid_rows, n_chunks), dim3(NT), 0,
                     a.stream, p, (const T*)a.q, (const T*)a.prefix_k, (const T*)a.prefix_v,
                     (const T*)a.suffix_k_pool, (const T*)a.suffix_v_pool, a.block_table,
                     a.suffix_lens, a.max_blocks, a.block_size, pool_tokens, a.sm_scale,
                     (float*)(a.ws + p.off_naive_o), (float*)(a.ws + p.off_naive_lse), first_chunk);
}
template <typename T>
void simple_stage_qabs(const Plan& p, const DecodeArgs& a) {
  if (p.rows == 0 || p.n_lat <= 0) return;
  hipLaunchKernelGGL(simple_qabs_kernel<T>, dim3((unsigned)p.rows), dim3(256), 0, a.stream, p.H,
                     (const T*)a.q, (const T*)a.w_uk, (T*)(a.ws + p.off_qabs));
}
template <typename T>
void simple_stage_absorb(const Plan& p, const DecodeArgs& a) {
  if (p.rows == 0 || p.n_lat <= 0) return;
  hipLaunchKernelGGL(simple_absorb_kernel<T>, dim3((unsigned)p.rows, p.n_lat), dim3(NT), 0,
                     a.stream, p, (const T*)(a.ws + p.off_qabs), (const T*)a.prefix_ckv,
                     (const T*)a.prefix_krope, (const T*)a.suffix_pool, a.block_table,
                     a.suffix_lens, a.max_blocks, a.block_size, a.sm_scale,
                     (T*)(a.ws + p.off_lat_o), (float*)(a.ws + p.off_lat_lse));
}
template <typename T>
void simple_stage_finalize(const Plan& p, const DecodeArgs& a) {
  if (p.rows == 0) return;
  hipLaunchKernelGGL(simple_finalize_kernel<T>, dim3((unsigned)p.rows), dim3(NT), 0, a.stream, p,
                     (const float*)(a.ws + p.off_naive_o), (const float*)(a.ws + p.off_naive_lse),
                     (const T*)(a.ws + p.off_lat_o), (const float*)(a.ws + p.off_lat_lse),
                     (const T*)a.w_uv, (T*)a.out, a.lse_out);
}
#define TMLA_INSTANTIATE(T)                                                        \
  template void simple_stage_naive<T>(const Plan&, const DecodeArgs&, int, int, int64_t);   \
  template void simple_stage_qabs<T>(const Plan&, const DecodeArgs&);              \
  template void simple_stage_absorb<T>(const Plan&, const DecodeArgs&);            \
  template void simple_stage_finalize<T>(const Plan&, const DecodeArgs&);
TMLA_INSTANTIATE(float)
TMLA_INSTANTIATE(bf16_t)
#undef TMLA_INSTANTIATE

// ---------------------------------------------------------------- stand-alone CombineLSE
// One wavefront per row: lanes stride over the width, the max / sum over partials are per-lane
// loops (every lane reads the same few LSE values), so no cross-lane traffic is needed.
template <typename T>
__global__ void __launch_bounds__(256)
combine_lse_kernel(int n, int64_t rows, int width, const float* __restrict__ po,
                   const float* __restrict__ pl, T* __restrict__ out, float* __restrict__ lse_out) {
  const int lane = threadIdx.x % 64;
  const int64_t row = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
  if (row >= rows) return;
  float m = -INFINITY;
  for (int i = 0; i < n; i++) m = fmaxf(m, pl[(size_t)i * rows + row]);
  if (m == -INFINITY) {
    for (int d = lane; d < width; d += 64) out[row * width + d] = from_float<T>(0.f);
    if (lse_out && lane == 0) lse_out[row] = -INFINITY;
    return;
  }
  float z = 0.f;
  for (int i = 0; i < n; i++) {
    const float li = pl[(size_t)i * rows + row];
    if (li > -INFINITY) z += expf(li - m);
  }
  const float inv = 1.f / z;
  for (int d = lane * 4; d < width; d += 256) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = 0; i < n; i++) {
      const float li = pl[(size_t)i * rows + row];
      if (li == -INFINITY) continue;
      const float w = expf(li - m);
      const float4 v = *(const float4*)(po + ((size_t)i * rows + row) * width + d);
      acc.x += w * v.x; acc.y += w * v.y; acc.z += w * v.z; acc.w += w * v.w;
    }
    T* o = out + row * width + d;
    o[0] = from_float<T>(acc.x * inv); o[1] = from_float<T>(acc.y * inv);
    o[2] = from_float<T>(acc.z * inv); o[3] = from_float<T>(acc.w * inv);
  }
  if (lse_out && lane == 0) lse_out[row] = m + logf(z);
}

void launch_combine_lse(int n, int64_t rows, int width, const float* po, const float* pl,
                        void* out, int out_dtype, float* lse_out, hipStream_t stream) {
  if (rows <= 0) return;
  const unsigned grid = (unsigned)((rows + 3) / 4);
  if (out_dtype == TMLA_FP32)
    hipLaunchKernelGGL(combine_lse_kernel<float>, dim3(grid), dim3(256), 0, stream, n, rows, width,
                       po, pl, (float*)out, lse_out);
  else
    hipLaunchKernelGGL(combine_lse_kernel<bf16_t>, dim3(grid), dim3(256), 0, stream, n, rows,
                       width, po, pl, (bf16_t*)out, lse_out);
}

}  // namespace tmla
