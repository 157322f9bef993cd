/*
 * typhoon_mla.h -- C ABI of the MI355X (gfx950) TyphoonMLA decode library.
 *
 * One multi-head latent attention (MLA) decode step over a batch whose KV cache is a prefix
 * shared by every request plus a per-request paged suffix (paper: Section 3.1, Algorithm 1).
 * The shared prefix is attended in the naive formulation over per-head K/V expanded once from
 * the latent cache (Algorithm 1 step 4), the suffix in the absorb formulation over the raw
 * 576-wide latent rows (steps 5-7), and the partial softmaxes are merged exactly with their
 * log-sum-exps (step 8).  `mode` also selects the two single-formulation baselines of Table 1.
 *
 * Conventions for every entry point
 *   - Every data pointer is CALLER-OWNED DEVICE MEMORY, 16-byte aligned, dense in the stated
 *     layout.  The library allocates nothing, never synchronises the host and enqueues work only
 *     on `stream` (a hipStream_t passed as void*, NULL = the default stream).  Results are ready
 *     when the stream reaches the end of the enqueued work.
 *   - State: none between calls, with two documented exceptions, both process-wide and both
 *     changed only through their own entry points -- typhoon_mla_set_debug_flags and
 *     typhoon_mla_set_tuning (development switches; a production caller touches neither).  The
 *     first launch of a kernel on a device also raises that kernel's dynamic-LDS limit, once per
 *     device.  Entry points may be called from several host threads.
 *   - Return value: a tmla_status.  Arguments are validated on the host before anything is
 *     launched, so argument errors are reported without touching the GPU.  TMLA_ERR_HIP reports a
 *     failure of the library's own launches only: a HIP error already pending in the calling
 *     thread at entry is neither cleared nor reported.
 *   - Supported dimensions: kv_lora_rank 512, qk_nope_dim 128, qk_rope_dim 64, v_head_dim 128
 *     (DeepSeek-v3 / Kimi K2, Table 1), num_heads a multiple of 16, paged block_size 64 or 128.
 *   - dtype TMLA_BF16: bf16 storage, fp32 accumulation and softmax.  TMLA_FP32: fp32 throughout.
 *   - RoPE is applied by the caller: q[..., 128:192] and every cached rope part arrive rotated
 *     (the inputs of Algorithm 1 are the query after its up-projection and rotation).
 *
 * Expanded ("naive") cache layout -- what typhoon_mla_expand_* writes and decode reads.
 *   TMLA_FP32: K [H, L, 192], V [H, L, 128], row-major.
 *   TMLA_BF16: matrix-core operand order, so a tile is copied to LDS or registers verbatim.
 *     Tokens are grouped in blocks of 32 (the last block zero-padded), NTB = ceil(L / 32).
 *     K element (h, t, d), d in [0,192):
 *        (((h*NTB + t/32)*12 + d/16)*64 + (t%32) + 32*((d%16)/8))*8 + d%8
 *     V element (h, t, d), d in [0,128), with u = t%16:
 *        ((((h*NTB + t/32)*2 + (t%32)/16)*4 + d/32)*64 + (d%32) + 32*((u/4)%2))*8 + 4*(u/8) + u%4
 *     i.e. 6144 K elements and 4096 V elements per (head, 32-token block).
 *     The RoPE part of a key (d in [128,192)) is the same for every head (Algorithm 1: the
 *     RoPE cache has no head axis); the expansion writes it into every head's blocks, and the
 *     bf16 decode kernels read it from head 0's blocks for all heads, so that it comes from HBM
 *     once.  A buffer filled by other means must keep that part identical across heads.
 *   Use typhoon_mla_expanded_k_bytes / _v_bytes for the buffer sizes.
 */
#ifndef TYPHOON_MLA_H
#define TYPHOON_MLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TMLA_OK = 0,
  TMLA_ERR_INVALID_ARG = 1,        /* null / negative / misaligned / inconsistent argument   */
  TMLA_ERR_UNSUPPORTED = 2,        /* dimensions, head count, block size or dtype not built  */
  TMLA_ERR_WORKSPACE_TOO_SMALL = 3,
  TMLA_ERR_HIP = 4,                /* one of the library's own launches failed                 */
  TMLA_ERR_SCRATCH_LIMIT = 5       /* typhoon_mla_decode_static_scratch: the call needs more
                                      than TMLA_STATIC_SCRATCH_BYTES of scratch memory       */
} tmla_status;

typedef enum {
  TMLA_MODE_MIXED = 0,       /* Algorithm 1: naive prefix + absorb suffix + LSE combine      */
  TMLA_MODE_NAIVE_ONLY = 1,  /* Table 1 "Naive": expanded K/V for prefix and suffix           */
  TMLA_MODE_ABSORB_ONLY = 2, /* Table 1 "Absorb": latent cache for prefix and suffix         */
  TMLA_MODE_AUTO = 3         /* Section 3.1 "Fall-back to Absorb": mixed when batch*q_len reaches
                                the break-even batch of Section 3.2, absorb_only below it       */
} tmla_mode;

typedef enum { TMLA_BF16 = 0, TMLA_FP32 = 1 } tmla_dtype;

typedef struct {
  int32_t num_heads;      /* H                                   */
  int32_t kv_lora_rank;   /* D_l = 512                           */
  int32_t qk_nope_dim;    /* D_n = 128                           */
  int32_t qk_rope_dim;    /* D_r = 64                            */
  int32_t v_head_dim;     /* D_v = 128                           */
  float sm_scale;         /* softmax scale on the full 192-wide score (e.g. 1/sqrt(192)) */
  int32_t dtype;          /* tmla_dtype                          */
} tmla_dims;

/* Static text for a tmla_status (never NULL). */
const char* typhoon_mla_status_string(int status);

/* Bytes of the expanded K (resp. V) buffer for `num_tokens` tokens; 0 on invalid arguments. */
size_t typhoon_mla_expanded_k_bytes(const tmla_dims* dims, int64_t num_tokens);
size_t typhoon_mla_expanded_v_bytes(const tmla_dims* dims, int64_t num_tokens);

/*
 * Prefix expansion (Section 3.1 "Prefill": the shared part of the latent caches is expanded
 * through the up-projection into per-head K and V):
 *   K[h,t,:] = [ W_UK[h] c_t (128) ; r_t (64) ],  V[h,t,:] = W_UV[h] c_t (128).
 *   prefix_ckv   in  [prefix_len, 512]     prefix_krope in  [prefix_len, 64]
 *   w_uk, w_uv   in  [H, 128, 512]         (W_KVb1, W_KVb2 of Algorithm 1)
 *   prefix_k / prefix_v  out, expanded layout above, typhoon_mla_expanded_{k,v}_bytes each.
 * prefix_len == 0 is legal and launches nothing.
 */
int typhoon_mla_expand_prefix(const tmla_dims* dims, int32_t prefix_len,
                              const void* prefix_ckv, const void* prefix_krope,
                              const void* w_uk, const void* w_uv,
                              void* prefix_k, void* prefix_v, void* stream);

/*
 * Same expansion applied to a whole paged pool of fused rows [num_blocks, block_size, 576]
 * (latent 512 ++ rope 64); pool slot (p, j) becomes expanded token p*block_size + j.  Only
 * TMLA_MODE_NAIVE_ONLY needs it (its Table 1 row reads expanded K/V for the suffix too).
 * Slots holding garbage expand to garbage; decode never reads slots beyond a request's length.
 */
int typhoon_mla_expand_pool(const tmla_dims* dims, int32_t num_blocks, int32_t block_size,
                            const void* suffix_pool, const void* w_uk, const void* w_uv,
                            void* suffix_k_pool, void* suffix_v_pool, void* stream);

/*
 * Break-even batch size of Section 3.2 ("Fall-back to Absorb" in Section 3.1): TMLA_MODE_AUTO
 * runs mixed when batch >= this value and absorb_only below it.  The paper's closed form,
 * B_theta = (D_qk + D_v) / (q_len (2 D_l + D_r)) * T / M, takes the absorb throughput T and the
 * bandwidth M as constants; near the cross-over neither is one on MI355X (a small batch is cut
 * into chunks to fill the chip, short steps are mostly launch latency), so the library
 * interpolates its own measured cross-overs (q_len = 1) in log2(heads) x log2(prefix_len),
 * clamped at the edges:
 *     prefix_len   16 heads   32    64   128
 *        1024        220      64   128    70
 *        4096         60      16    52    45
 *       16384         19      11    35    40
 *       65536         11      12    32    40
 * and divides by q_len.
 * The environment variable TMLA_AUTO_BATCH_THRESHOLD, read once per process, overrides it.
 * Returns -1 on invalid arguments.
 */
double typhoon_mla_auto_batch_threshold(const tmla_dims* dims, int32_t q_len, int32_t prefix_len);

/* Scratch bytes typhoon_mla_decode needs for this problem size (a pure host function). */
size_t typhoon_mla_decode_workspace_bytes(const tmla_dims* dims, int32_t mode, int32_t batch,
                                          int32_t q_len, int32_t prefix_len,
                                          int32_t max_suffix_len);

/*
 * One decode step (Algorithm 1; Section 3.1 "Decode").
 *   q            in  [B, q_len, H, 192]  noPE 128 ++ RoPE 64
 *   prefix_k/_v  in  expanded prefix (mixed, naive_only; may be NULL otherwise or if prefix_len==0)
 *   prefix_ckv   in  [prefix_len, 512], prefix_krope [prefix_len, 64] (absorb_only; else may be NULL)
 *                    TMLA_MODE_AUTO needs both forms of the prefix
 *   suffix_pool  in  [num_blocks, block_size, 576] latent rows (mixed, absorb_only)
 *   block_table  in  [B, max_blocks] int32 physical block of each logical suffix block;
 *                    entries beyond ceil(suffix_lens[b]/block_size) are never read
 *   suffix_lens  in  [B] int32 (device); 0 <= suffix_lens[b] <= max_suffix_len, which is a host
 *                    upper bound with ceil(max_suffix_len/block_size) <= max_blocks
 *   suffix_k_pool/_v_pool in expanded pool from typhoon_mla_expand_pool (naive_only; else NULL)
 *   w_uk, w_uv   in  [H, 128, 512] (mixed, absorb_only)
 *   out          out [B, q_len, H, 128] in dims->dtype
 *   lse_out      out [B, q_len, H] fp32 natural-log LSE of the scaled scores, or NULL
 *   workspace    scratch of at least typhoon_mla_decode_workspace_bytes(...), 256-byte aligned
 * Visibility: every query sees the whole prefix; query position s of request b sees suffix
 * tokens j <= suffix_lens[b] - q_len + s (the suffix already holds the q_len new tokens).
 * A query that sees no token yields zeros and LSE = -inf.
 * Limits (TMLA_ERR_UNSUPPORTED beyond them): q_len <= 8, batch * q_len * H <= 2^30,
 * prefix_len and max_suffix_len <= 2^30.
 */
int typhoon_mla_decode(const tmla_dims* dims, int32_t mode, int32_t batch, int32_t q_len,
                       const void* q, int32_t prefix_len,
                       const void* prefix_k, const void* prefix_v,
                       const void* prefix_ckv, const void* prefix_krope,
                       const void* suffix_pool, int32_t num_blocks, int32_t block_size,
                       const int32_t* block_table, int32_t max_blocks,
                       const int32_t* suffix_lens, int32_t max_suffix_len,
                       const void* suffix_k_pool, const void* suffix_v_pool,
                       const void* w_uk, const void* w_uv,
                       void* out, float* lse_out,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * typhoon_mla_decode for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and kernels as typhoon_mla_decode, without `workspace`: the
 * intermediates (absorbed queries, split partials, the request order) live in a static device
 * array of TMLA_STATIC_SCRATCH_BYTES inside the library, one per GPU the library runs on, held
 * until the process ends.  The call allocates nothing and frees nothing.
 *   - A problem whose typhoon_mla_decode_workspace_bytes exceeds TMLA_STATIC_SCRATCH_BYTES is
 *     rejected with TMLA_ERR_SCRATCH_LIMIT before anything is launched (128 MiB covers batch 256
 *     at 128 heads, batch 128 with q_len 2, and batch 512 at 16 heads with suffixes up to 4096).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two host threads) race on it; serialise them.  Nothing in it has to start at
 *     zero -- every call writes what it reads -- so a call may follow any other.
 *   - The first call on a device looks the array's address up; make that call outside graph
 *     capture.
 */
#define TMLA_STATIC_SCRATCH_BYTES (128u << 20)
int typhoon_mla_decode_static_scratch(const tmla_dims* dims, int32_t mode, int32_t batch,
                                      int32_t q_len, const void* q, int32_t prefix_len,
                                      const void* prefix_k, const void* prefix_v,
                                      const void* prefix_ckv, const void* prefix_krope,
                                      const void* suffix_pool, int32_t num_blocks,
                                      int32_t block_size, const int32_t* block_table,
                                      int32_t max_blocks, const int32_t* suffix_lens,
                                      int32_t max_suffix_len, const void* suffix_k_pool,
                                      const void* suffix_v_pool, const void* w_uk,
                                      const void* w_uv, void* out, float* lse_out, void* stream);

/*
 * Multi-level (tree-shaped) shared prefixes.  Section 3.1 ("Prefill") speaks of a tree-like query
 * structure formed from the requests and their shared prefix, and the related-work discussion of
 * prefix sharing says that the handling of tree-structured caches applies to the naive and the
 * absorb part alike.  Here a request's context is the concatenation of the nodes on its path (e.g. a system prompt shared by all requests, then a per-tenant prompt shared by a
 * group) followed by its own suffix.  Each node is attended in the naive formulation over its
 * own expanded K/V (typhoon_mla_expand_prefix per node) by exactly the requests that share it,
 * the suffixes in the absorb formulation, and all partials are merged with CombineLSE -- the
 * merge of Algorithm 1 step 8 with one more partial per level.
 *
 * A node covers the contiguous request range [batch_begin, batch_begin + batch_count) and sits on
 * `level` (0 = root side).  Nodes of one level must not overlap; a request may skip a level.
 * The array of nodes lives in HOST memory and is only read during the call; k/v are device
 * pointers in the expanded layout for `len` tokens.  Attention is over a set, so the order of the
 * levels has no effect on the result.
 */
typedef struct {
  const void* k;        /* expanded K of the node's tokens (device) */
  const void* v;        /* expanded V (device)                      */
  int32_t len;          /* tokens in the node, >= 0                 */
  int32_t level;        /* 0 <= level < 8                           */
  int32_t batch_begin;  /* first request sharing the node           */
  int32_t batch_count;  /* number of requests sharing it, >= 0      */
} tmla_prefix_node;

/* Scratch bytes typhoon_mla_decode_tree needs (a pure host function; 0 on invalid arguments). */
size_t typhoon_mla_decode_tree_workspace_bytes(const tmla_dims* dims, int32_t batch, int32_t q_len,
                                               const tmla_prefix_node* nodes, int32_t num_nodes,
                                               int32_t max_suffix_len);

/*
 * One decode step over tree-shaped shared prefixes (mixed formulation).  Arguments as for
 * typhoon_mla_decode, with `nodes` in place of the single prefix; num_nodes == 0 is the
 * suffix-only case.  Errors: TMLA_ERR_INVALID_ARG also for a node range outside the batch, a
 * level outside [0, 8) or two overlapping nodes of one level.
 */
int typhoon_mla_decode_tree(const tmla_dims* dims, int32_t batch, int32_t q_len, const void* q,
                            const tmla_prefix_node* nodes, int32_t num_nodes,
                            const void* suffix_pool, int32_t num_blocks, int32_t block_size,
                            const int32_t* block_table, int32_t max_blocks,
                            const int32_t* suffix_lens, int32_t max_suffix_len, const void* w_uk,
                            const void* w_uv, void* out, float* lse_out, void* workspace,
                            size_t workspace_bytes, void* stream);

/*
 * CombineLSE alone (Algorithm 1 step 8; Section 3.2): exact merge of `num_partials` normalised
 * partial outputs with their natural-log LSEs.
 *   partial_out in [num_partials, rows, width] fp32,  partial_lse in [num_partials, rows] fp32
 *   out         out [rows, width] in `out_dtype`,     lse_out out [rows] fp32 or NULL
 * A partial with LSE = -inf contributes nothing (its values are ignored, NaN included).
 * width must be a multiple of 4 and at most 512.
 */
int typhoon_mla_combine_lse(int32_t num_partials, int64_t rows, int32_t width,
                            const float* partial_out, const float* partial_lse,
                            void* out, int32_t out_dtype, float* lse_out, void* stream);

/*
 * Debug switches (process-wide; default 0; the switch itself is atomic, but a call that runs
 * while another thread changes it may see either value).
 *   bit 0: run the scalar reference kernels instead of the matrix-core kernels for bf16.
 *   bits 1..3: scalar kernel for one stage only -- 2 query absorption, 4 absorb attention,
 *     8 up-projection + combine (the other stages stay on the matrix cores).
 *   bits 4..8 (bf16 matrix-core path only): when any is set, decode launches only the selected
 *     stages, for per-kernel timing -- 0x10 naive prefix attention, 0x20 naive suffix attention,
 *     0x40 query absorption, 0x80 absorb attention, 0x100 up-projection + combine.  The output
 *     is then meaningless unless the workspace still holds the other stages' results.
 *   bit 9 (0x200): scalar kernel for the naive suffix attention of naive_only mode.
 *   bit 10 (0x400): naive prefix attention with more than 128 queries per head runs on the
 *     8-wavefront kernel (moving exponent references) instead of the software-pipelined one.
 *   bit 11 (0x800): the absorb attention kernel for more than 32 query rows per request walks
 *     every chunk with moving exponent references (otherwise only chunks in which its first walk,
 *     with references fixed at the chunk's first tokens, overflowed).
 *   bit 12 (0x1000): requests with a multiple of 128 query rows keep the absorb kernel that
 *     gives a workgroup 64 rows; bit 13 (0x2000): they take the 128-row kernel even when its
 *     grid does not cover the chip (by default it is chosen only when it does).
 *   bit 14 (0x4000): the absorb attention kernels start the requests with the longest suffix
 *     first whatever the grid size (by default only when a pass has more workgroups than the
 *     chip has compute units, and the batch has at most 4096 requests); bit 15 (0x8000): never.
 * Returns the previous value.
 */
int typhoon_mla_set_debug_flags(int flags);

/*
 * Tuning overrides of the launch plan (process-wide; 0 = the library's own choice, the default).
 * The initial value of each key is read once from the environment variable of the same name
 * with the prefix TMLA_ (TMLA_PREFIX_SPLITS, ...), when the first call needs it.  The workspace
 * size depends on them: set them before typhoon_mla_decode_workspace_bytes, not between it and
 * the decode call.  Returns the previous value, or -1 for an unknown key or a negative value.
 */
typedef enum {
  TMLA_TUNE_PREFIX_SPLITS = 0,        /* token splits of the naive prefix pass                   */
  TMLA_TUNE_SUFFIX_CHUNK = 1,         /* tokens per chunk of the absorb pass over the suffix     */
  TMLA_TUNE_ABSORB_PREFIX_CHUNK = 2,  /* tokens per chunk of the absorb pass over the prefix     */
  TMLA_TUNE_NAIVE_SUFFIX_CHUNK = 3,   /* tokens per chunk of the naive pass over the suffix      */
  TMLA_TUNE_COUNT = 4
} tmla_tuning_key;
int typhoon_mla_set_tuning(int key, int value);

#ifdef __cplusplus
}
#endif
#endif /* TYPHOON_MLA_H */
