"""fp64 CPU oracle for one MLA decode step over a shared prefix plus per-request paged suffixes.

THIS IS TEST INFRASTRUCTURE.  Only the test-suite, the smoke check and the benchmark's
CPU-baseline leg may import it; the library itself never does, and nothing here imports the
library.  It is deliberately plain and slow so it can be checked against the paper by eye.

What it computes (paper: Section 2.1 "Naive", Algorithm 1, Section 3.1 "Decode"):
for every request b, query position s and head h, textbook softmax attention of the 192-wide
query against the per-head keys and values obtained by up-projecting every visible latent cache
token -- i.e. the *naive definition* evaluated over the concatenation prefix ++ suffix_b.  The
mixed method of Algorithm 1 (naive on the prefix, absorb on the suffix, LSE combine) is stated
by the paper to be mathematically equivalent to this, so the definition is the oracle; it never
forms an absorbed query, never splits a softmax and never merges partial results.

A second, separately written routine (`mla_decode_absorb_form`) evaluates the *absorb*
formulation (Section 2.1 "Absorb"; Algorithm 1 steps 5-7 applied to the whole cache).  It is
pinned to the definition by the naive == absorb invariant in the CPU tests and is used where the
definition is too expensive (its cost per token-head is 1088 MACs instead of 131072).

`mla_decode_absorb_all_heads` is the same absorb formulation written the way Algorithm 1 prints
it -- whole tensors, all heads of a request at once (steps 5, 6, 7 as three matrix products) --
so that it is cheap enough to cover every output row of the full-size configurations.  It is
pinned to the definition by the same invariant and by the scalar brute force.

`combine_lse` is the LSE merge of Algorithm 1 step 8 written from its definition; it is used
only to pin that "merge of split softmaxes == one softmax" and to check the GPU merge kernel.

Readings of the paper taken here (the paper is silent or inconsistent on these points):
  * softmax scale: explicit `sm_scale`, applied to the sum of the noPE and RoPE score parts
    (Algorithm 1 prints no scale);
  * the shared K/V cache has one copy with a head axis (Algorithm 1 prints a batch axis, Table 1's
    HBM term `L_s H (D_qk + D_v)` has none);
  * RoPE is applied upstream: q[..., 128:192] and the cached rope part arrive rotated;
  * LSE is the natural-log log-sum-exp of the scaled scores;
  * S_q > 1: causal mask inside the suffix only, aligned to the end of the suffix (the suffix
    length already counts the S_q new tokens); the prefix is always fully visible;
  * a query that sees no token at all returns zeros and LSE = -inf.

Parity pins (tests/test_oracle_pins.py): naive == absorb, split/merge == full softmax, rows of
softmax sum to one and outputs lie in the value hull, scalar brute force on tiny inputs, closed
forms (L = 1, q = 0, identical tokens, logit shift, token / block-table permutation, zero
weights), and agreement with a library fp64 scaled-dot-product attention on expanded K/V.
"""
import numpy as np

D_LATENT = 512  # D_l, KV LoRA rank
D_NOPE = 128    # D_n
D_ROPE = 64     # D_r
D_V = 128       # D_v
D_QK = D_NOPE + D_ROPE


def gather_suffix_rows(pool, block_table_row, length):
    """Rows of request's suffix, token j at pool[block_table_row[j // bs], j % bs] (576 wide)."""
    bs = pool.shape[1]
    rows = np.empty((length, pool.shape[2]), dtype=np.float64)
    for j in range(length):
        rows[j] = pool[block_table_row[j // bs], j % bs]
    return rows


def expand_tokens(c_lat, k_rope, w_uk_h, w_uv_h):
    """Per-head key/value of latent tokens (Section 2.1 "Naive"; prefill expansion, Section 3.1).

    k_t = [W_UK[h] c_t ; r_t] (192), v_t = W_UV[h] c_t (128).
    """
    k = np.concatenate([c_lat @ w_uk_h.T, k_rope], axis=1)
    v = c_lat @ w_uv_h.T
    return k, v


def softmax_attend(x, v):
    """One softmax row: returns (sum_t p_t v_t, LSE).  x: [L] scaled scores, v: [L, D]."""
    if x.shape[0] == 0:
        return np.zeros(v.shape[1]), -np.inf
    m = np.max(x)
    e = np.exp(x - m)
    z = np.sum(e)
    return (e / z) @ v, m + np.log(z)


def _visible_suffix(len_b, s_q, s):
    """Number of suffix tokens query position s may see (end-aligned causal mask)."""
    return max(0, min(len_b, len_b - s_q + s + 1))


def mla_decode_definition(q, prefix_ckv, prefix_krope, pool, block_table, suffix_lens,
                          w_uk, w_uv, sm_scale, pairs=None):
    """Naive-definition MLA decode in fp64.

    q            [B, S_q, H, 192]   (noPE 128 ++ RoPE 64, RoPE already applied)
    prefix_ckv   [L_s, 512], prefix_krope [L_s, 64]     shared prefix, latent form
    pool         [n_blocks, block, 576]   paged suffix rows (latent 512 ++ rope 64)
    block_table  [B, max_blocks] int,  suffix_lens [B] int
    w_uk, w_uv   [H, 128, 512]
    pairs        optional iterable of (b, h); only those are computed, the rest are NaN.
    Returns O [B, S_q, H, 128], LSE [B, S_q, H] (float64).
    """
    q = np.asarray(q, dtype=np.float64)
    B, S_q, H, _ = q.shape
    L_s = prefix_ckv.shape[0]
    out = np.full((B, S_q, H, D_V), np.nan)
    lse = np.full((B, S_q, H), np.nan)
    if pairs is None:
        pairs = [(b, h) for b in range(B) for h in range(H)]
    by_request = {}
    for b, h in pairs:
        by_request.setdefault(int(b), []).append(int(h))
    prefix_kv = {}  # memo: the prefix expansion of a head is the same for every request
    for b in sorted(by_request):
        len_b = int(suffix_lens[b])
        rows = gather_suffix_rows(pool, block_table[b], len_b)
        suf_c, suf_r = rows[:, :D_LATENT], rows[:, D_LATENT:]
        for h in by_request[b]:
            if h not in prefix_kv:
                prefix_kv[h] = expand_tokens(prefix_ckv, prefix_krope, w_uk[h], w_uv[h])
            k_p, v_p = prefix_kv[h]
            k_s, v_s = expand_tokens(suf_c, suf_r, w_uk[h], w_uv[h])
            k = np.concatenate([k_p, k_s], axis=0)
            v = np.concatenate([v_p, v_s], axis=0)
            for s in range(S_q):
                n_vis = L_s + _visible_suffix(len_b, S_q, s)
                x = sm_scale * (k[:n_vis] @ q[b, s, h])
                out[b, s, h], lse[b, s, h] = softmax_attend(x, v[:n_vis])
    return out, lse


def mla_decode_absorb_form(q, prefix_ckv, prefix_krope, pool, block_table, suffix_lens,
                           w_uk, w_uv, sm_scale, pairs=None):
    """Absorb-formulation MLA decode in fp64 (Algorithm 1 steps 5-7 over the whole cache).

    q_A = W_UK[h]^T q_nope (512); x_t = sm_scale (<q_A, c_t> + <q_rope, r_t>);
    o = W_UV[h] (sum_t p_t c_t).  Same arguments and results as `mla_decode_definition`.
    """
    q = np.asarray(q, dtype=np.float64)
    B, S_q, H, _ = q.shape
    L_s = prefix_ckv.shape[0]
    out = np.full((B, S_q, H, D_V), np.nan)
    lse = np.full((B, S_q, H), np.nan)
    if pairs is None:
        pairs = [(b, h) for b in range(B) for h in range(H)]
    by_request = {}
    for b, h in pairs:
        by_request.setdefault(int(b), []).append(int(h))
    for b in sorted(by_request):
        len_b = int(suffix_lens[b])
        rows = gather_suffix_rows(pool, block_table[b], len_b)
        c_all = np.concatenate([prefix_ckv, rows[:, :D_LATENT]], axis=0)
        r_all = np.concatenate([prefix_krope, rows[:, D_LATENT:]], axis=0)
        for h in by_request[b]:
            for s in range(S_q):
                n_vis = L_s + _visible_suffix(len_b, S_q, s)
                q_nope, q_rope = q[b, s, h, :D_NOPE], q[b, s, h, D_NOPE:]
                q_a = w_uk[h].T @ q_nope
                x = sm_scale * (c_all[:n_vis] @ q_a + r_all[:n_vis] @ q_rope)
                o_lat, lse[b, s, h] = softmax_attend(x, c_all[:n_vis])
                out[b, s, h] = w_uv[h] @ o_lat
    return out, lse


def mla_decode_absorb_all_heads(q, prefix_ckv, prefix_krope, pool, block_table, suffix_lens,
                                w_uk, w_uv, sm_scale, requests=None):
    """Absorb formulation in Algorithm 1's tensor form, one request at a time, all heads at once.

    For request b and query position s, with C_N / C_R the visible latent and rope rows:
      step 5   Q_A = Q_N W_KVb1              [H, 512]   (per head: q_nope W_UK[h])
      step 6   P   = softmax(sm_scale (Q_A C_N^T + Q_R C_R^T))   [H, n_visible]
               O_lat = P C_N                 [H, 512]
      step 7   O   = O_lat W_KVb2^T          [H, 128]   (per head: W_UV[h] o_lat)
    requests: optional iterable of b; other requests stay NaN.  Returns (O, LSE) like
    `mla_decode_definition`.
    """
    q = np.asarray(q, dtype=np.float64)
    B, S_q, H, _ = q.shape
    L_s = prefix_ckv.shape[0]
    out = np.full((B, S_q, H, D_V), np.nan)
    lse = np.full((B, S_q, H), np.nan)
    for b in (range(B) if requests is None else requests):
        len_b = int(suffix_lens[b])
        rows = gather_suffix_rows(pool, block_table[b], len_b)
        c_all = np.concatenate([prefix_ckv, rows[:, :D_LATENT]], axis=0)
        r_all = np.concatenate([prefix_krope, rows[:, D_LATENT:]], axis=0)
        for s in range(S_q):
            n_vis = L_s + _visible_suffix(len_b, S_q, s)
            if n_vis == 0:
                out[b, s] = 0.0
                lse[b, s] = -np.inf
                continue
            q_n, q_r = q[b, s, :, :D_NOPE], q[b, s, :, D_NOPE:]
            q_a = np.einsum("hn,hnl->hl", q_n, w_uk)                       # step 5
            x = sm_scale * (q_a @ c_all[:n_vis].T + q_r @ r_all[:n_vis].T)  # [H, n_vis]
            m = np.max(x, axis=1)
            e = np.exp(x - m[:, None])
            z = np.sum(e, axis=1)
            o_lat = (e / z[:, None]) @ c_all[:n_vis]                       # step 6
            out[b, s] = np.einsum("hl,hvl->hv", o_lat, w_uv)               # step 7
            lse[b, s] = m + np.log(z)
    return out, lse


def combine_lse(outs, lses):
    """Exact merge of partial softmax results (Algorithm 1 step 8; Section 3.2 "CombineLSE").

    outs [P, ..., D]: each partial's normalised output; lses [P, ...]: its natural-log LSE
    (-inf for an empty partial, whose output is ignored).  Returns (O [..., D], LSE [...]).
    """
    outs = np.asarray(outs, dtype=np.float64)
    lses = np.asarray(lses, dtype=np.float64)
    m = np.max(lses, axis=0)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    w = np.exp(lses - m_safe)            # exp(-inf) = 0 for empty partials
    z = np.sum(w, axis=0)
    num = np.sum(w[..., None] * np.where(w[..., None] > 0, outs, 0.0), axis=0)
    z_safe = np.where(z > 0, z, 1.0)
    o = num / z_safe[..., None]
    lse = np.where(z > 0, m_safe + np.log(z_safe), -np.inf)
    return o, lse


def expand_prefix_definition(prefix_ckv, prefix_krope, w_uk, w_uv):
    """Expanded shared cache in logical layout: K [H, L_s, 192], V [H, L_s, 128] (fp64)."""
    H = w_uk.shape[0]
    L = prefix_ckv.shape[0]
    k = np.empty((H, L, D_QK))
    v = np.empty((H, L, D_V))
    for h in range(H):
        k[h], v[h] = expand_tokens(prefix_ckv, prefix_krope, w_uk[h], w_uv[h])
    return k, v
