// C ABI of the TyphoonMLA decode library: host-side argument validation, launch planning /
// workspace layout, and dispatch to the kernels.  No HIP call is made before validation passes.
#include <algorithm>
#include <cmath>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "tmla_common.hpp"

namespace tmla {

// The only state the library keeps: debug flags and tuning overrides, both process-wide, both
// set through their own entry points (see typhoon_mla.h).
static std::atomic<int> g_debug_flags{0};
int debug_flags() { return g_debug_flags.load(std::memory_order_relaxed); }

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline int round_up(int a, int b) { return ceil_div(a, b) * b; }

// Tuning overrides; 0 = the library's own choice.  The environment gives the initial values and
// is read once, when the first call needs them.
struct Tuning {
  std::atomic<int> v[TMLA_TUNE_COUNT];
  double auto_threshold;   // < 0: closed form
  Tuning() {
    static const char* const names[TMLA_TUNE_COUNT] = {
        "TMLA_PREFIX_SPLITS", "TMLA_SUFFIX_CHUNK", "TMLA_ABSORB_PREFIX_CHUNK",
        "TMLA_NAIVE_SUFFIX_CHUNK"};
    for (int i = 0; i < TMLA_TUNE_COUNT; i++) {
      const char* s = getenv(names[i]);
      v[i].store((s && *s) ? atoi(s) : 0);
    }
    const char* e = getenv("TMLA_AUTO_BATCH_THRESHOLD");
    auto_threshold = (e && *e) ? atof(e) : -1.0;
  }
};
static Tuning& tuning() {
  static Tuning t;
  return t;
}
static int tune(int key) { return tuning().v[key].load(std::memory_order_relaxed); }

static int check_dims(const tmla_dims* d) {
  if (!d) return TMLA_ERR_INVALID_ARG;
  if (d->num_heads <= 0) return TMLA_ERR_INVALID_ARG;
  if (d->dtype != TMLA_BF16 && d->dtype != TMLA_FP32) return TMLA_ERR_UNSUPPORTED;
  if (d->kv_lora_rank != D_L || d->qk_nope_dim != D_N || d->qk_rope_dim != D_R ||
      d->v_head_dim != D_V)
    return TMLA_ERR_UNSUPPORTED;
  if (d->num_heads % 16 != 0) return TMLA_ERR_UNSUPPORTED;
  if (!(d->sm_scale > 0.f) || !(d->sm_scale < 1e30f)) return TMLA_ERR_INVALID_ARG;
  return TMLA_OK;
}

static inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }


// Token splits of a naive pass over Ls shared tokens for M queries per head.
static void plan_prefix_splits(int H, int M, int Ls, int* p_chunk, int* np_split) {
  const int wgs = std::max(1, H * (M > PIPELINED_MIN_M ? ceil_div(M, 256) : ceil_div(M, 64)));
  int splits = tune(TMLA_TUNE_PREFIX_SPLITS);
  if (splits <= 0) splits = std::max(1, NUM_CU / wgs);
  splits = std::max(1, std::min(splits, ceil_div(Ls, 128)));
  *p_chunk = round_up(ceil_div(Ls, splits), TOK_BLK);
  *np_split = ceil_div(Ls, *p_chunk);
}

void layout_workspace(Plan* p);

// Token chunk of the absorb pass for a grid with fewer (request, row group) pairs than compute
// units, where the chunk count alone decides how the pass fills the chip: 264 workgroups take two
// rounds on 256 units, 240 take one.  Every chunk length (in 64-token steps) is priced with a
// small model of the 64- and 128-row kernels -- rounds x (start-up + steps x step time) plus the
// merge of the partials -- and the cheapest is taken.  The constants are measured on MI355X
// (start-up 15 us, 3.3 / 4.1 us per step, partials merged at 3 TB/s); they only have to rank the
// candidates.  Ls = latent prefix tokens walked in absorb form (0 in mixed mode).
static int plan_small_grid_chunk(int B, int R, int Ls, int Ln, int block_size) {
  const int g64 = ceil_div(R, 64);
  const int longest = std::max(Ls, Ln);
  double best = 1e300;
  int best_T = 0;
  // candidates: the longer part cut into n = 1 ... MAX_CHUNKS equal chunks of whole 64-token steps
  // (chunks under 256 tokens are not worth a partial)
  for (int n = 1; n <= MAX_CHUNKS; n++) {
    const int T = (int)((((int64_t)longest + n - 1) / n + 63) / 64 * 64);
    if (n > 1 && T < 256) break;
    const int Ts = round_up(T, block_size);
    const int ap = Ls > 0 ? ceil_div(Ls, T) : 0, as = Ln > 0 ? ceil_div(Ln, Ts) : 0;
    if (ap > MAX_CHUNKS || as > MAX_CHUNKS) continue;
    const int n_lat = ap + as;
    const bool rows128 = R % 128 == 0 && (long long)n_lat * B * (R / 128) >= NUM_CU;
    const long long wgs = (long long)n_lat * B * (rows128 ? R / 128 : g64);
    const int steps = ceil_div(std::max(std::min(T, Ls), std::min(Ts, Ln)), 64);
    const double rounds = (double)((wgs + NUM_CU - 1) / NUM_CU);
    double t = rounds * (15.0 + steps * (rows128 ? 4.1 : 3.3));
    if (n_lat > 4) t += 3.0 + (double)n_lat * B * R * 1024.0 / 3e6;
    else t += 1.5 * (n_lat - 1);
    if (t < best) { best = t; best_T = T; }   // ties: the longer chunk
  }
  return best_T ? best_T : round_up(std::max(longest, 64), 64);
}

// Cuts the call into work items (token chunks) and lays the intermediates out in the workspace.
// Chunk counts per request are bounds derived from host-visible sizes only; a chunk that turns
// out empty on the device reports LSE = -inf and is skipped by the combine step.
int make_plan(const tmla_dims* dims, int mode, int B, int Sq, int Ls, int max_suffix,
              int block_size, Plan* p) {
  memset(p, 0, sizeof(*p));
  p->B = B; p->Sq = Sq; p->H = dims->num_heads; p->Ls = Ls; p->max_suffix = max_suffix;
  p->mode = mode; p->dtype = dims->dtype;
  p->rows = (int64_t)B * Sq * dims->num_heads;
  const int H = dims->num_heads;
  const int M = B * Sq;
  const int target = 2 * NUM_CU;

  if (Ls > 0 && mode != TMLA_MODE_ABSORB_ONLY) {
    // naive prefix pass: one workgroup owns a head and a block of up to 256 queries
    // (64 when the batch is small and the token-split kernel runs); one workgroup fits per
    // compute unit, so the prefix is split until the grid covers the chip once
    plan_prefix_splits(H, M, Ls, &p->p_chunk, &p->np_split);
  }
  if (mode == TMLA_MODE_NAIVE_ONLY && max_suffix > 0) {
    int chunk = tune(TMLA_TUNE_NAIVE_SUFFIX_CHUNK);
    if (chunk <= 0) chunk = 1024;
    p->ns_chunk = round_up(std::min(chunk, round_up(max_suffix, block_size)), block_size);
    p->ns_chunks = ceil_div(max_suffix, p->ns_chunk);
  }
  if (mode != TMLA_MODE_NAIVE_ONLY) {
    // absorb pass: one workgroup owns a request, one token chunk and up to 64 of its S_q*H query
    // rows (with at most 16 rows: four consecutive chunks, one per wavefront).  Chunks are kept
    // as long as the grid still covers the chip about twice: every extra chunk costs a
    // 512-wide partial per row and a workgroup start-up.
    const int R = Sq * H;
    const int per_wg = R <= 16 ? 4 : 1;
    const int wgs = std::max(1, B * ceil_div(R, 64));
    const int want = std::max(1, ceil_div(2 * NUM_CU, wgs)) * per_wg;   // chunks per request
    const int Ls_abs = mode == TMLA_MODE_ABSORB_ONLY ? Ls : 0;
    // small grids of the 64- / 128-row kernels: chunk from the model above
    const int modelled = (R > 32 && wgs < NUM_CU && (Ls_abs > 0 || max_suffix > 0))
                             ? plan_small_grid_chunk(B, R, Ls_abs, max_suffix, block_size) : 0;
    if (mode == TMLA_MODE_ABSORB_ONLY && Ls > 0) {
      int chunk = tune(TMLA_TUNE_ABSORB_PREFIX_CHUNK);
      if (chunk <= 0) chunk = modelled ? modelled : std::max(256, ceil_div(Ls, want));
      chunk = std::max(chunk, ceil_div(Ls, MAX_CHUNKS));
      p->ap_chunk = round_up(std::min(chunk, round_up(Ls, TOK_BLK)), TOK_BLK);
      p->ap_chunks = ceil_div(Ls, p->ap_chunk);
    }
    if (max_suffix > 0) {
      int chunk = tune(TMLA_TUNE_SUFFIX_CHUNK);
      if (chunk <= 0) chunk = modelled ? modelled : std::max(256, ceil_div(max_suffix, want));
      chunk = std::max(chunk, ceil_div(max_suffix, MAX_CHUNKS));
      p->as_chunk = round_up(std::min(chunk, round_up(max_suffix, block_size)), block_size);
      p->as_chunks = ceil_div(max_suffix, p->as_chunk);
    }
  }
  p->n_naive = p->np_split + p->ns_chunks;
  p->n_lat = p->ap_chunks + p->as_chunks;

  layout_workspace(p);
  return TMLA_OK;
}

void layout_workspace(Plan* p) {
  const size_t esz = p->dtype == TMLA_BF16 ? 2 : 4;
  size_t off = 0;
  p->off_qabs = off;      off = align_up(off + (p->n_lat ? (size_t)p->rows * D_ROW * esz : 0), 256);
  p->off_naive_o = off;   off = align_up(off + (size_t)p->n_naive * p->rows * D_V * 4, 256);
  p->off_naive_lse = off; off = align_up(off + (size_t)p->n_naive * p->rows * 4, 256);
  p->off_lat_o = off;     off = align_up(off + (size_t)p->n_lat * p->rows * D_L * esz, 256);
  p->off_lat_lse = off;   off = align_up(off + (size_t)p->n_lat * p->rows * 4, 256);
  p->off_order = off;     off = align_up(off + (p->n_lat ? (size_t)p->B * 4 : 0), 256);
  p->total = off + 256;
}

static int64_t padded_tokens(const tmla_dims* dims, int64_t n) {
  return dims->dtype == TMLA_BF16 ? (n + TOK_BLK - 1) / TOK_BLK * TOK_BLK : n;
}

}  // namespace tmla

using namespace tmla;

extern "C" {

const char* typhoon_mla_status_string(int status) {
  switch (status) {
    case TMLA_OK: return "ok";
    case TMLA_ERR_INVALID_ARG: return "invalid argument";
    case TMLA_ERR_UNSUPPORTED: return "unsupported dimensions, head count, block size or dtype";
    case TMLA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case TMLA_ERR_HIP: return "HIP launch error";
    case TMLA_ERR_SCRATCH_LIMIT:
      return "the call needs more scratch memory than the library's static buffer holds";
    default: return "unknown status";
  }
}

int typhoon_mla_set_debug_flags(int flags) { return g_debug_flags.exchange(flags); }

int typhoon_mla_set_tuning(int key, int value) {
  if (key < 0 || key >= TMLA_TUNE_COUNT || value < 0) return -1;
  return tuning().v[key].exchange(value);
}

size_t typhoon_mla_expanded_k_bytes(const tmla_dims* dims, int64_t num_tokens) {
  if (check_dims(dims) != TMLA_OK || num_tokens < 0) return 0;
  const size_t esz = dims->dtype == TMLA_BF16 ? 2 : 4;
  return (size_t)dims->num_heads * padded_tokens(dims, num_tokens) * D_QK * esz;
}
size_t typhoon_mla_expanded_v_bytes(const tmla_dims* dims, int64_t num_tokens) {
  if (check_dims(dims) != TMLA_OK || num_tokens < 0) return 0;
  const size_t esz = dims->dtype == TMLA_BF16 ? 2 : 4;
  return (size_t)dims->num_heads * padded_tokens(dims, num_tokens) * D_V * esz;
}

static int expand_common(const tmla_dims* dims, int64_t ntok, const void* c, int64_t c_stride,
                         const void* r, int64_t r_stride, const void* w_uk, const void* w_uv,
                         void* k_out, void* v_out, void* stream) {
  if (ntok == 0) return TMLA_OK;
  if (!c || !r || !w_uk || !w_uv || !k_out || !v_out) return TMLA_ERR_INVALID_ARG;
  if (misaligned(c, 16) || misaligned(r, 16) || misaligned(w_uk, 16) || misaligned(w_uv, 16) ||
      misaligned(k_out, 16) || misaligned(v_out, 16))
    return TMLA_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  const LaunchCheck launches;
  if (dims->dtype == TMLA_FP32) {
    simple_expand<float>(dims->num_heads, ntok, (const float*)c, c_stride, (const float*)r,
                         r_stride, (const float*)w_uk, (const float*)w_uv, (float*)k_out,
                         (float*)v_out, st);
  } else if (debug_flags() & 1) {
    simple_expand<bf16_t>(dims->num_heads, ntok, (const bf16_t*)c, c_stride, (const bf16_t*)r,
                          r_stride, (const bf16_t*)w_uk, (const bf16_t*)w_uv, (bf16_t*)k_out,
                          (bf16_t*)v_out, st);
  } else {
    const int rc = mfma_expand(dims->num_heads, ntok, c, c_stride, r, r_stride, w_uk, w_uv, k_out,
                               v_out, st);
    if (rc != TMLA_OK) return rc;
  }
  return launches.status();
}

int typhoon_mla_expand_prefix(const tmla_dims* dims, int32_t prefix_len, const void* prefix_ckv,
                              const void* prefix_krope, const void* w_uk, const void* w_uv,
                              void* prefix_k, void* prefix_v, void* stream) {
  const int st = check_dims(dims);
  if (st != TMLA_OK) return st;
  if (prefix_len < 0) return TMLA_ERR_INVALID_ARG;
  return expand_common(dims, prefix_len, prefix_ckv, D_L, prefix_krope, D_R, w_uk, w_uv, prefix_k,
                       prefix_v, stream);
}

int typhoon_mla_expand_pool(const tmla_dims* dims, int32_t num_blocks, int32_t block_size,
                            const void* suffix_pool, const void* w_uk, const void* w_uv,
                            void* suffix_k_pool, void* suffix_v_pool, void* stream) {
  const int st = check_dims(dims);
  if (st != TMLA_OK) return st;
  if (num_blocks < 0) return TMLA_ERR_INVALID_ARG;
  if (block_size != 64 && block_size != 128) return TMLA_ERR_UNSUPPORTED;
  const size_t esz = dims->dtype == TMLA_BF16 ? 2 : 4;
  const char* rope = suffix_pool ? (const char*)suffix_pool + D_L * esz : nullptr;
  return expand_common(dims, (int64_t)num_blocks * block_size, suffix_pool, D_ROW, rope, D_ROW,
                       w_uk, w_uv, suffix_k_pool, suffix_v_pool, stream);
}

static int check_decode_sizes(const tmla_dims* dims, int mode, int batch, int q_len,
                              int prefix_len, int max_suffix_len) {
  const int st = check_dims(dims);
  if (st != TMLA_OK) return st;
  if (mode != TMLA_MODE_MIXED && mode != TMLA_MODE_NAIVE_ONLY && mode != TMLA_MODE_ABSORB_ONLY &&
      mode != TMLA_MODE_AUTO)
    return TMLA_ERR_INVALID_ARG;
  if (batch < 0 || q_len <= 0 || prefix_len < 0 || max_suffix_len < 0) return TMLA_ERR_INVALID_ARG;
  if (q_len > 8) return TMLA_ERR_UNSUPPORTED;
  if ((int64_t)batch * q_len * dims->num_heads > (int64_t)1 << 30) return TMLA_ERR_UNSUPPORTED;
  // (token counts are rounded up to blocks and chunks in 32-bit arithmetic)
  if (prefix_len > 1 << 30 || max_suffix_len > 1 << 30) return TMLA_ERR_UNSUPPORTED;
  return TMLA_OK;
}

// Section 3.2's break-even batch is B_theta = (D_qk + D_v) / (S_q (2 D_l + D_r)) * T / M with the
// absorb throughput T and the memory bandwidth M as constants (with T ~ 300 TFLOP/s for a small
// batch and M ~ 5.5 TB/s it gives 16).  Near the cross-over neither side is that simple on this
// GPU: in absorb form a small batch is cut into chunks until it fills the chip and its partials
// are merged afterwards, the naive pass streams L_s (H (D_n + D_v) + D_r) elements whatever the
// batch, and a short step is mostly launch latency.  So the library interpolates its own
// measured cross-overs (bench.py --sweep, S_q = 1, suffix 512: the batch at which mixed
// overtakes absorb_only) in log2(heads) x log2(prefix length), clamped at the table's edges.
// (The dips at 32 heads are real: 32 query rows per request run the small shared-tile kernel.)
static double fitted_batch_threshold(int heads, int prefix_len) {
  static const double cross[4][4] = {
      //  16     32     64    128 heads
      {220.0, 64.0, 128.0, 70.0},   // prefix 1024: short steps, the modes differ little
      {60.0, 16.0, 52.0, 45.0},     // prefix 4096
      {19.0, 11.0, 35.0, 40.0},     // prefix 16384
      {11.0, 12.0, 32.0, 40.0},     // prefix 65536
  };
  const double x = std::min(3.0, std::max(0.0, std::log2(std::max(1, heads) / 16.0)));
  const double y = std::min(3.0, std::max(0.0, std::log2(std::max(1, prefix_len) / 1024.0) / 2.0));
  const int x0 = std::min(2, (int)x), y0 = std::min(2, (int)y);
  const double fx = x - x0, fy = y - y0;
  auto lg = [&](int r, int c) { return std::log2(cross[r][c]); };
  const double v = (1 - fy) * ((1 - fx) * lg(y0, x0) + fx * lg(y0, x0 + 1)) +
                   fy * ((1 - fx) * lg(y0 + 1, x0) + fx * lg(y0 + 1, x0 + 1));
  return std::exp2(v);
}

double typhoon_mla_auto_batch_threshold(const tmla_dims* dims, int32_t q_len, int32_t prefix_len) {
  if (check_dims(dims) != TMLA_OK || prefix_len < 0) return -1.0;
  if (tuning().auto_threshold >= 0.0) return tuning().auto_threshold;
  if (q_len <= 0) q_len = 1;
  return fitted_batch_threshold(dims->num_heads, prefix_len) / q_len;
}

static int resolve_auto(const tmla_dims* dims, int mode, int batch, int q_len, int prefix_len) {
  if (mode != TMLA_MODE_AUTO) return mode;
  if (prefix_len == 0) return TMLA_MODE_MIXED;   // nothing to choose: both run the absorb suffix
  return batch >= typhoon_mla_auto_batch_threshold(dims, q_len, prefix_len) ? TMLA_MODE_MIXED
                                                                           : TMLA_MODE_ABSORB_ONLY;
}

size_t typhoon_mla_decode_workspace_bytes(const tmla_dims* dims, int32_t mode, int32_t batch,
                                          int32_t q_len, int32_t prefix_len,
                                          int32_t max_suffix_len) {
  if (check_decode_sizes(dims, mode, batch, q_len, prefix_len, max_suffix_len) != TMLA_OK) return 0;
  mode = resolve_auto(dims, mode, batch, q_len, prefix_len);
  Plan p;
  // the plan rounds suffix chunks to the paged block size; 128 covers both supported sizes
  make_plan(dims, mode, batch, q_len, prefix_len, max_suffix_len, 128, &p);
  size_t a = p.total;
  make_plan(dims, mode, batch, q_len, prefix_len, max_suffix_len, 64, &p);
  return std::max(a, p.total);
}

// Where the scratch memory of a decode call comes from: the caller's workspace, or the library's
// static device array (then `get` is called after validation, with the bytes the plan needs).
struct ScratchSource {
  void* workspace;
  size_t workspace_bytes;
  int (*get)(size_t need, void** ptr);   // nullptr: use workspace / workspace_bytes
};

static int decode_impl(const tmla_dims* dims, int32_t mode, int32_t batch, int32_t q_len,
                       const void* q, int32_t prefix_len, const void* prefix_k,
                       const void* prefix_v, const void* prefix_ckv, const void* prefix_krope,
                       const void* suffix_pool, int32_t num_blocks, int32_t block_size,
                       const int32_t* block_table, int32_t max_blocks, const int32_t* suffix_lens,
                       int32_t max_suffix_len, const void* suffix_k_pool,
                       const void* suffix_v_pool, const void* w_uk, const void* w_uv, void* out,
                       float* lse_out, const ScratchSource& scratch_src, void* stream) {
  int st = check_decode_sizes(dims, mode, batch, q_len, prefix_len, max_suffix_len);
  if (st != TMLA_OK) return st;
  if (block_size != 64 && block_size != 128) return TMLA_ERR_UNSUPPORTED;
  if (num_blocks < 0 || max_blocks < 0) return TMLA_ERR_INVALID_ARG;
  if ((int64_t)max_blocks * block_size < max_suffix_len) return TMLA_ERR_INVALID_ARG;
  if (batch == 0) return TMLA_OK;
  if (!q || !out || !suffix_lens) return TMLA_ERR_INVALID_ARG;
  if (mode == TMLA_MODE_AUTO) {
    if (prefix_len > 0 && (!prefix_k || !prefix_v || !prefix_ckv || !prefix_krope))
      return TMLA_ERR_INVALID_ARG;
    mode = resolve_auto(dims, mode, batch, q_len, prefix_len);
  }
  const bool need_naive_prefix = prefix_len > 0 && mode != TMLA_MODE_ABSORB_ONLY;
  const bool need_latent_prefix = prefix_len > 0 && mode == TMLA_MODE_ABSORB_ONLY;
  const bool need_latent_suffix = max_suffix_len > 0 && mode != TMLA_MODE_NAIVE_ONLY;
  const bool need_naive_suffix = max_suffix_len > 0 && mode == TMLA_MODE_NAIVE_ONLY;
  if (need_naive_prefix && (!prefix_k || !prefix_v)) return TMLA_ERR_INVALID_ARG;
  if (need_latent_prefix && (!prefix_ckv || !prefix_krope)) return TMLA_ERR_INVALID_ARG;
  if (need_latent_suffix && (!suffix_pool || !block_table || num_blocks == 0))
    return TMLA_ERR_INVALID_ARG;
  if (need_naive_suffix && (!suffix_k_pool || !suffix_v_pool || !block_table || num_blocks == 0))
    return TMLA_ERR_INVALID_ARG;
  if ((need_latent_prefix || need_latent_suffix) && (!w_uk || !w_uv)) return TMLA_ERR_INVALID_ARG;
  const void* ptrs[] = {q, out, prefix_k, prefix_v, prefix_ckv, prefix_krope, suffix_pool,
                        suffix_k_pool, suffix_v_pool, w_uk, w_uv};
  for (const void* ptr : ptrs)
    if (ptr && misaligned(ptr, 16)) return TMLA_ERR_INVALID_ARG;
  if (misaligned(block_table, 4) || misaligned(suffix_lens, 4) || misaligned(lse_out, 4))
    return TMLA_ERR_INVALID_ARG;

  Plan p;
  make_plan(dims, mode, batch, q_len, prefix_len, max_suffix_len, block_size, &p);
  void* workspace = scratch_src.workspace;
  if (scratch_src.get) {
    if ((st = scratch_src.get(p.total, &workspace)) != TMLA_OK) return st;
  } else {
    if (!workspace || misaligned(workspace, 256)) return TMLA_ERR_INVALID_ARG;
    if (scratch_src.workspace_bytes < p.total) return TMLA_ERR_WORKSPACE_TOO_SMALL;
  }

  DecodeArgs a;
  a.q = q; a.prefix_k = prefix_k; a.prefix_v = prefix_v; a.prefix_ckv = prefix_ckv;
  a.prefix_krope = prefix_krope; a.suffix_pool = suffix_pool; a.block_table = block_table;
  a.suffix_lens = suffix_lens; a.suffix_k_pool = suffix_k_pool; a.suffix_v_pool = suffix_v_pool;
  a.w_uk = w_uk; a.w_uv = w_uv; a.out = out; a.lse_out = lse_out; a.ws = (char*)workspace;
  a.num_blocks = num_blocks; a.block_size = block_size; a.max_blocks = max_blocks;
  a.sm_scale = dims->sm_scale; a.stream = (hipStream_t)stream;

  const LaunchCheck launches;
  if (dims->dtype == TMLA_FP32) {
    simple_stage_naive<float>(p, a, 0, p.n_naive);
    simple_stage_qabs<float>(p, a);
    simple_stage_absorb<float>(p, a);
    simple_stage_finalize<float>(p, a);
  } else if (debug_flags() & 1) {
    simple_stage_naive<bf16_t>(p, a, 0, p.n_naive);
    simple_stage_qabs<bf16_t>(p, a);
    simple_stage_absorb<bf16_t>(p, a);
    simple_stage_finalize<bf16_t>(p, a);
  } else {
    // bits 4..8 of the debug flags restrict the call to single stages (for per-kernel timing)
    const int only = debug_flags() & 0x1f0;
    if (!only || (only & 0x10)) {
      st = mfma_prefix_attention(p, a);
      if (st != TMLA_OK) return st;
    }
    if (!only || (only & 0x20)) {
      // (bit 9 of the debug flags keeps the scalar kernel for this stage)
      if ((debug_flags() & 0x200) || p.Sq > 64)
        simple_stage_naive<bf16_t>(p, a, p.np_split, p.ns_chunks);
      else if ((st = mfma_naive_suffix_attention(p, a)) != TMLA_OK) return st;
    }
    if (!only || (only & 0x40)) {
      if (debug_flags() & 2) simple_stage_qabs<bf16_t>(p, a);
      else if ((st = mfma_query_absorb(p, a)) != TMLA_OK) return st;
    }
    if (!only || (only & 0x80)) {
      if (debug_flags() & 4) simple_stage_absorb<bf16_t>(p, a);
      else if ((st = mfma_absorb_attention(p, a)) != TMLA_OK) return st;
    }
    if (!only || (only & 0x100)) {
      if (debug_flags() & 8) simple_stage_finalize<bf16_t>(p, a);
      else if ((st = mfma_finalize(p, a)) != TMLA_OK) return st;
    }
  }
  return launches.status();
}

int typhoon_mla_decode(const tmla_dims* dims, int32_t mode, int32_t batch, int32_t q_len,
                       const void* q, int32_t prefix_len, const void* prefix_k,
                       const void* prefix_v, const void* prefix_ckv, const void* prefix_krope,
                       const void* suffix_pool, int32_t num_blocks, int32_t block_size,
                       const int32_t* block_table, int32_t max_blocks, const int32_t* suffix_lens,
                       int32_t max_suffix_len, const void* suffix_k_pool,
                       const void* suffix_v_pool, const void* w_uk, const void* w_uv, void* out,
                       float* lse_out, void* workspace, size_t workspace_bytes, void* stream) {
  const ScratchSource src = {workspace, workspace_bytes, nullptr};
  return decode_impl(dims, mode, batch, q_len, q, prefix_len, prefix_k, prefix_v, prefix_ckv,
                     prefix_krope, suffix_pool, num_blocks, block_size, block_table, max_blocks,
                     suffix_lens, max_suffix_len, suffix_k_pool, suffix_v_pool, w_uk, w_uv, out,
                     lse_out, src, stream);
}

// ---- decode on the library's own static scratch (for callers that cannot allocate) -----------
// One array per GPU the library's code is loaded on, held until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; the device address it yields (per
// device) is what the kernels get.
static __device__ __align__(256) unsigned char scratch[TMLA_STATIC_SCRATCH_BYTES];

static constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[MAX_DEVICES] = {};

static int static_scratch(size_t need, void** ptr) {
  if (need > (size_t)TMLA_STATIC_SCRATCH_BYTES) return TMLA_ERR_SCRATCH_LIMIT;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return TMLA_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TMLA_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return TMLA_OK;
}

int typhoon_mla_decode_static_scratch(
    const tmla_dims* dims, int32_t mode, int32_t batch, int32_t q_len, const void* q,
    int32_t prefix_len, const void* prefix_k, const void* prefix_v, const void* prefix_ckv,
    const void* prefix_krope, const void* suffix_pool, int32_t num_blocks, int32_t block_size,
    const int32_t* block_table, int32_t max_blocks, const int32_t* suffix_lens,
    int32_t max_suffix_len, const void* suffix_k_pool, const void* suffix_v_pool, const void* w_uk,
    const void* w_uv, void* out, float* lse_out, void* stream) {
  const ScratchSource src = {nullptr, 0, static_scratch};
  return decode_impl(dims, mode, batch, q_len, q, prefix_len, prefix_k, prefix_v, prefix_ckv,
                     prefix_krope, suffix_pool, num_blocks, block_size, block_table, max_blocks,
                     suffix_lens, max_suffix_len, suffix_k_pool, suffix_v_pool, w_uk, w_uv, out,
                     lse_out, src, stream);
}

// ---- tree-shaped shared prefixes -----------------------------------------------------------
constexpr int TREE_MAX_LEVELS = 8;

struct TreePlan {
  Plan p;                            // suffix plan + workspace layout; n_naive = all level slots
  int level_slot0[TREE_MAX_LEVELS];  // first partial slot of a level
  std::vector<int> chunk, splits;    // per node
};

// Validates the nodes and fixes the partial slots: a level owns as many slots as its most split
// node; rows of a level that no node covers keep the LSE = -inf the slots are initialised with.
static int make_tree_plan(const tmla_dims* dims, int batch, int q_len, const tmla_prefix_node* nodes,
                          int num_nodes, int max_suffix_len, int block_size, TreePlan* tp) {
  int st = check_decode_sizes(dims, TMLA_MODE_MIXED, batch, q_len, 0, max_suffix_len);
  if (st != TMLA_OK) return st;
  if (num_nodes < 0 || (num_nodes > 0 && !nodes)) return TMLA_ERR_INVALID_ARG;
  make_plan(dims, TMLA_MODE_MIXED, batch, q_len, 0, max_suffix_len, block_size, &tp->p);
  int level_slots[TREE_MAX_LEVELS] = {0};
  tp->chunk.assign(num_nodes, 0);
  tp->splits.assign(num_nodes, 0);
  for (int i = 0; i < num_nodes; i++) {
    const tmla_prefix_node& nd = nodes[i];
    if (nd.len < 0 || nd.level < 0 || nd.level >= TREE_MAX_LEVELS || nd.batch_begin < 0 ||
        nd.batch_count < 0 || (int64_t)nd.batch_begin + nd.batch_count > batch)
      return TMLA_ERR_INVALID_ARG;
    if (nd.len == 0 || nd.batch_count == 0) continue;
    for (int j = 0; j < i; j++) {
      const tmla_prefix_node& o = nodes[j];
      if (o.level != nd.level || o.len == 0 || o.batch_count == 0) continue;
      if (nd.batch_begin < o.batch_begin + o.batch_count && o.batch_begin < nd.batch_begin + nd.batch_count)
        return TMLA_ERR_INVALID_ARG;
    }
    plan_prefix_splits(dims->num_heads, nd.batch_count * q_len, nd.len, &tp->chunk[i],
                       &tp->splits[i]);
    level_slots[nd.level] = std::max(level_slots[nd.level], tp->splits[i]);
  }
  int slots = 0;
  for (int l = 0; l < TREE_MAX_LEVELS; l++) {
    tp->level_slot0[l] = slots;
    slots += level_slots[l];
  }
  tp->p.np_split = 0;
  tp->p.n_naive = slots;
  layout_workspace(&tp->p);
  return TMLA_OK;
}

size_t typhoon_mla_decode_tree_workspace_bytes(const tmla_dims* dims, int32_t batch, int32_t q_len,
                                               const tmla_prefix_node* nodes, int32_t num_nodes,
                                               int32_t max_suffix_len) {
  TreePlan tp;
  if (make_tree_plan(dims, batch, q_len, nodes, num_nodes, max_suffix_len, 128, &tp) != TMLA_OK)
    return 0;
  const size_t a = tp.p.total;
  make_tree_plan(dims, batch, q_len, nodes, num_nodes, max_suffix_len, 64, &tp);
  return std::max(a, tp.p.total);
}

int typhoon_mla_decode_tree(const tmla_dims* dims, int32_t batch, int32_t q_len, const void* q,
                            const tmla_prefix_node* nodes, int32_t num_nodes,
                            const void* suffix_pool, int32_t num_blocks, int32_t block_size,
                            const int32_t* block_table, int32_t max_blocks,
                            const int32_t* suffix_lens, int32_t max_suffix_len, const void* w_uk,
                            const void* w_uv, void* out, float* lse_out, void* workspace,
                            size_t workspace_bytes, void* stream) {
  if (block_size != 64 && block_size != 128) {
    const int st0 = check_dims(dims);
    return st0 != TMLA_OK ? st0 : TMLA_ERR_UNSUPPORTED;
  }
  TreePlan tp;
  int st = make_tree_plan(dims, batch, q_len, nodes, num_nodes, max_suffix_len, block_size, &tp);
  if (st != TMLA_OK) return st;
  if (num_blocks < 0 || max_blocks < 0) return TMLA_ERR_INVALID_ARG;
  if ((int64_t)max_blocks * block_size < max_suffix_len) return TMLA_ERR_INVALID_ARG;
  if (batch == 0) return TMLA_OK;
  if (!q || !out || !suffix_lens) return TMLA_ERR_INVALID_ARG;
  const bool need_suffix = max_suffix_len > 0;
  if (need_suffix && (!suffix_pool || !block_table || num_blocks == 0 || !w_uk || !w_uv))
    return TMLA_ERR_INVALID_ARG;
  const void* ptrs[] = {q, out, suffix_pool, w_uk, w_uv};
  for (const void* ptr : ptrs)
    if (ptr && misaligned(ptr, 16)) return TMLA_ERR_INVALID_ARG;
  if (misaligned(block_table, 4) || misaligned(suffix_lens, 4) || misaligned(lse_out, 4))
    return TMLA_ERR_INVALID_ARG;
  for (int i = 0; i < num_nodes; i++)
    if (tp.splits[i] > 0 && (!nodes[i].k || !nodes[i].v || misaligned(nodes[i].k, 16) ||
                             misaligned(nodes[i].v, 16)))
      return TMLA_ERR_INVALID_ARG;
  const Plan& p = tp.p;
  if (!workspace || misaligned(workspace, 256)) return TMLA_ERR_INVALID_ARG;
  if (workspace_bytes < p.total) return TMLA_ERR_WORKSPACE_TOO_SMALL;

  DecodeArgs a;
  memset(&a, 0, sizeof(a));
  a.q = q; a.suffix_pool = suffix_pool; a.block_table = block_table; a.suffix_lens = suffix_lens;
  a.w_uk = w_uk; a.w_uv = w_uv; a.out = out; a.lse_out = lse_out; a.ws = (char*)workspace;
  a.num_blocks = num_blocks; a.block_size = block_size; a.max_blocks = max_blocks;
  a.sm_scale = dims->sm_scale; a.stream = (hipStream_t)stream;
  const bool bf16 = dims->dtype == TMLA_BF16;
  const size_t esz = bf16 ? 2 : 4;

  const LaunchCheck launches;
  // every level slot starts empty; a node's pass fills the rows of its own requests
  launch_fill_f32((float*)(a.ws + p.off_naive_lse), (int64_t)p.n_naive * p.rows, -INFINITY, a.stream);
  for (int i = 0; i < num_nodes; i++) {
    if (tp.splits[i] == 0) continue;
    const tmla_prefix_node& nd = nodes[i];
    const int64_t row0 = (int64_t)nd.batch_begin * q_len * dims->num_heads;
    const int64_t slot_row0 = (int64_t)tp.level_slot0[nd.level] * p.rows + row0;
    Plan pn = p;                       // rows stays the stride between splits
    pn.B = nd.batch_count; pn.Ls = nd.len; pn.p_chunk = tp.chunk[i]; pn.np_split = tp.splits[i];
    pn.off_naive_o = p.off_naive_o + (size_t)slot_row0 * D_V * 4;
    pn.off_naive_lse = p.off_naive_lse + (size_t)slot_row0 * 4;
    DecodeArgs an = a;
    an.q = (const char*)q + (size_t)row0 * D_QK * esz;
    an.prefix_k = nd.k; an.prefix_v = nd.v;
    if (bf16 && !(debug_flags() & 1)) {
      if ((st = mfma_prefix_attention(pn, an)) != TMLA_OK) return st;
    } else if (bf16) {
      simple_stage_naive<bf16_t>(pn, an, 0, pn.np_split, (int64_t)nd.batch_count * q_len * dims->num_heads);
    } else {
      simple_stage_naive<float>(pn, an, 0, pn.np_split, (int64_t)nd.batch_count * q_len * dims->num_heads);
    }
  }
  if (!bf16) {
    simple_stage_qabs<float>(p, a);
    simple_stage_absorb<float>(p, a);
    simple_stage_finalize<float>(p, a);
  } else if (debug_flags() & 1) {
    simple_stage_qabs<bf16_t>(p, a);
    simple_stage_absorb<bf16_t>(p, a);
    simple_stage_finalize<bf16_t>(p, a);
  } else {
    if ((st = mfma_query_absorb(p, a)) != TMLA_OK) return st;
    if ((st = mfma_absorb_attention(p, a)) != TMLA_OK) return st;
    if ((st = mfma_finalize(p, a)) != TMLA_OK) return st;
  }
  return launches.status();
}

int typhoon_mla_combine_lse(int32_t num_partials, int64_t rows, int32_t width,
                            const float* partial_out, const float* partial_lse, void* out,
                            int32_t out_dtype, float* lse_out, void* stream) {
  if (num_partials <= 0 || rows < 0 || width <= 0) return TMLA_ERR_INVALID_ARG;
  if (width % 4 != 0 || width > 512) return TMLA_ERR_UNSUPPORTED;
  if (out_dtype != TMLA_BF16 && out_dtype != TMLA_FP32) return TMLA_ERR_UNSUPPORTED;
  if (rows == 0) return TMLA_OK;
  if (!partial_out || !partial_lse || !out) return TMLA_ERR_INVALID_ARG;
  if (misaligned(partial_out, 16) || misaligned(out, 8) || misaligned(partial_lse, 4) ||
      misaligned(lse_out, 4))
    return TMLA_ERR_INVALID_ARG;
  const LaunchCheck launches;
  launch_combine_lse(num_partials, rows, width, partial_out, partial_lse, out, out_dtype, lse_out,
                     (hipStream_t)stream);
  return launches.status();
}

}  // extern "C"
