// Shared declarations of the TyphoonMLA decode library: fixed MLA dimensions, the expanded-cache
// element addressing, the host-side launch plan / workspace layout and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/typhoon_mla.h"

namespace tmla {

constexpr int NUM_CU = 256;  // MI355X compute units; work is cut to a small multiple of this

// DeepSeek-v3 / Kimi K2 MLA dimensions (paper Table 1).
constexpr int D_L = 512;          // KV LoRA rank (latent width)
constexpr int D_N = 128;          // noPE head dim
constexpr int D_R = 64;           // RoPE head dim
constexpr int D_V = 128;          // value head dim
constexpr int D_QK = D_N + D_R;   // 192
constexpr int D_ROW = D_L + D_R;  // 576: one latent cache row (c_KV ++ k_rope)
constexpr int TOK_BLK = 32;       // token granularity of the bf16 expanded layout
constexpr int K_BLK_ELEMS = TOK_BLK * D_QK;  // 6144
constexpr int V_BLK_ELEMS = TOK_BLK * D_V;   // 4096

struct bf16_t { uint16_t x; };

__host__ __device__ inline float bf16_to_float(bf16_t v) {
  union { uint32_t u; float f; } c; c.u = (uint32_t)v.x << 16; return c.f;
}
__host__ __device__ inline bf16_t float_to_bf16(float f) {
  union { uint32_t u; float f; } c; c.f = f;
  uint32_t u = c.u;
  bf16_t r;
  if ((u & 0x7fffffffu) > 0x7f800000u) { r.x = (uint16_t)((u >> 16) | 0x40u); return r; }
  u += 0x7fffu + ((u >> 16) & 1u);
  r.x = (uint16_t)(u >> 16);
  return r;
}
__host__ __device__ inline float to_float(float v) { return v; }
__host__ __device__ inline float to_float(bf16_t v) { return bf16_to_float(v); }
template <typename T> __host__ __device__ inline T from_float(float f);
template <> __host__ __device__ inline float from_float<float>(float f) { return f; }
template <> __host__ __device__ inline bf16_t from_float<bf16_t>(float f) { return float_to_bf16(f); }

// Expanded-cache element offsets (see the layout description in typhoon_mla.h).
template <typename T> struct ExpLayout;
template <> struct ExpLayout<float> {
  __host__ __device__ static size_t k(int h, int64_t ntok, int64_t t, int d) {
    return ((size_t)h * ntok + t) * D_QK + d;
  }
  __host__ __device__ static size_t v(int h, int64_t ntok, int64_t t, int d) {
    return ((size_t)h * ntok + t) * D_V + d;
  }
};
template <> struct ExpLayout<bf16_t> {
  __host__ __device__ static size_t k(int h, int64_t ntok, int64_t t, int d) {
    const int64_t ntb = (ntok + TOK_BLK - 1) / TOK_BLK;
    const int tt = (int)(t % TOK_BLK);
    return ((((size_t)h * ntb + t / TOK_BLK) * 12 + d / 16) * 64 + tt + 32 * ((d % 16) / 8)) * 8 +
           d % 8;
  }
  __host__ __device__ static size_t v(int h, int64_t ntok, int64_t t, int d) {
    const int64_t ntb = (ntok + TOK_BLK - 1) / TOK_BLK;
    const int tt = (int)(t % TOK_BLK);
    const int u = tt % 16;
    return (((((size_t)h * ntb + t / TOK_BLK) * 2 + tt / 16) * 4 + d / 32) * 64 + (d % 32) +
            32 * ((u / 4) % 2)) * 8 + 4 * (u / 8) + u % 4;
  }
};

// Launch plan: how a decode call is cut into work items, and where each intermediate lives in
// the caller's workspace.  A pure function of the host-visible sizes.
struct Plan {
  int B, Sq, H, Ls, max_suffix, mode, dtype;
  int64_t rows;        // B*Sq*H output rows, row = (b*Sq + s)*H + h
  int np_split;        // naive prefix: number of token splits (0: no naive prefix pass)
  int p_chunk;         //   tokens per split (multiple of 32)
  int ns_chunks;       // naive suffix (naive_only): chunks per request
  int ns_chunk;        //   tokens per chunk (multiple of block_size)
  int ap_chunks;       // absorb over the latent prefix (absorb_only): chunks per request
  int ap_chunk;        //   tokens per chunk (multiple of 32)
  int as_chunks;       // absorb over the paged suffix: chunks per request
  int as_chunk;        //   tokens per chunk (multiple of block_size)
  int n_naive;         // = np_split + ns_chunks   (128-wide partials per row)
  int n_lat;           // = ap_chunks + as_chunks  (512-wide latent partials per row)
  size_t off_qabs, off_naive_o, off_naive_lse, off_lat_o, off_lat_lse, off_order, total;
};

int debug_flags();   // current typhoon_mla_set_debug_flags value

// A kernel's opt-in to more dynamic LDS than the default limit, made once per device.  The
// attribute call is idempotent, so two host threads racing here only repeat it.
struct LdsOptIn {
  std::atomic<uint64_t> done{0};
  hipError_t ensure(const void* fn, int bytes) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
    const uint64_t bit = (dev >= 0 && dev < 64) ? 1ull << dev : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
  }
};

// Reports the errors of the launches made while it is alive and nothing else: an error that was
// already pending in the calling thread when the library was entered is the caller's and stays
// where it is (the library neither clears nor reports it).
struct LaunchCheck {
  hipError_t before;
  LaunchCheck() : before(hipPeekAtLastError()) {}
  int status() const {
    const hipError_t after = hipPeekAtLastError();
    if (after == hipSuccess || after == before) return TMLA_OK;
    if (before == hipSuccess) (void)hipGetLastError();   // ours: consumed here
    return TMLA_ERR_HIP;
  }
};

int make_plan(const tmla_dims* dims, int mode, int batch, int q_len, int prefix_len,
              int max_suffix_len, int block_size, Plan* plan);

struct DecodeArgs {
  const void *q, *prefix_k, *prefix_v, *prefix_ckv, *prefix_krope, *suffix_pool;
  const int32_t *block_table, *suffix_lens;
  const void *suffix_k_pool, *suffix_v_pool, *w_uk, *w_uv;
  void* out; float* lse_out; char* ws;
  int num_blocks, block_size, max_blocks;
  float sm_scale;
  hipStream_t stream;
};

// Scalar reference kernels (any dtype; the only path for fp32).
template <typename T>
void simple_expand(int H, int64_t ntok, const T* c, int64_t c_stride, const T* r, int64_t r_stride,
                   const T* w_uk, const T* w_uv, T* k_out, T* v_out, hipStream_t stream);
template <typename T> void simple_stage_naive(const Plan& p, const DecodeArgs& a, int first_chunk,
                                              int n_chunks, int64_t grid_rows = -1);
void launch_fill_f32(float* p, int64_t n, float v, hipStream_t stream);
template <typename T> void simple_stage_qabs(const Plan& p, const DecodeArgs& a);
template <typename T> void simple_stage_absorb(const Plan& p, const DecodeArgs& a);
template <typename T> void simple_stage_finalize(const Plan& p, const DecodeArgs& a);

// Matrix-core kernels (bf16).  Each returns a tmla_status.
int mfma_expand(int H, int64_t ntok, const void* c, int64_t c_stride, const void* r,
                int64_t r_stride, const void* w_uk, const void* w_uv, void* k_out, void* v_out,
                hipStream_t stream);
int mfma_prefix_attention(const Plan& p, const DecodeArgs& a);
int mfma_naive_suffix_attention(const Plan& p, const DecodeArgs& a);
int mfma_query_absorb(const Plan& p, const DecodeArgs& a);
int mfma_absorb_attention(const Plan& p, const DecodeArgs& a);
// Requests sorted by suffix length, longest first (written to the workspace by a small kernel
// on the call's stream), for a pass that launches `wgs` workgroups; nullptr = keep the order
// of the batch.
const int32_t* suffix_request_order(const Plan& p, const DecodeArgs& a, long long wgs);
int mfma_absorb16_attention(const Plan& p, const DecodeArgs& a);   // S_q * H <= 16
int mfma_finalize(const Plan& p, const DecodeArgs& a);
// more queries per head than this: the software-pipelined prefix kernel (256 queries per
// workgroup); up to this many: the token-split kernel (64 queries per workgroup, the query groups
// of a head sharing its cache through L2).  Measured with the bound at 64: equal at 4096-token
// prefixes, 7 % less kernel time at 32768 tokens but a longer step (more partials to combine).
constexpr int PIPELINED_MIN_M = 128;
constexpr int MAX_CHUNKS = 64;  // per-request chunk bound for each of the latent prefix / suffix
void launch_combine_lse(int num_partials, int64_t rows, int width, const float* po,
                        const float* pl, void* out, int out_dtype, float* lse_out,
                        hipStream_t stream);

}  // namespace tmla
