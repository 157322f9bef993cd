"""Shared test utilities: run a workload through the C-ABI library, compare with the oracle."""
import numpy as np
import torch

from paper_2509_21081_amd import binding as T

# Tolerances: bf16 I/O with fp32 accumulation -> max-abs 1e-2 + max-rel 2e-2 element-wise, plus a
# row-wise relative L2 bound and an LSE bound so that small outputs cannot hide an error;
# fp32 mode -> 1e-4 for all three.
#
# Peaked softmax rows (queries scaled by a gain g, or one part of the keys scaled up): bf16
# storage alone -- the expanded keys of the prefix and the absorbed query of the suffix, both
# mandated by bf16 I/O -- perturbs a logit by sigma_x = 3.9e-4 g (relative rounding 2^-9 / sqrt 3 on
# each of 128 products q_i k_i).  In a near-uniform softmax these errors average out (LSE error
# 1.1e-5 simulated at g = 1); in a peaked row the LSE moves by the error of the top logit and the
# output by |do| <= dx * sum_t p_t |v_t - o|.  Simulated in fp64 with only those two roundings
# on the B = 64, H = 128 configuration at g = 8: LSE error sigma 3.1e-3, maximum 1.6e-2 = 5.1
# sigma over 2048 rows; the per-row sigma varies with the query's size, so over the 10^4 .. 10^5
# rows of a full configuration the maximum reaches 6 sigma.  Bounds for peaked rows:
#   LSE      8 sigma_x                         = 3.2e-3 g
#   output   8 sigma_x * 0.8 (sum p |v - o| <= 1.8 sigma_v, sigma_v = 0.45), never below the
#            unscaled bound                    = max(1e-2, 2.5e-3 g) absolute, + 2e-2 relative
#   row L2   the same error against a row norm of about |v_top| = sigma_v sqrt(128):
#            max(2e-2, 5e-3 g)
TOL = {"bf16": dict(atol=1e-2, rtol=2e-2, row_l2=2e-2, lse=2e-3),
       "fp32": dict(atol=1e-4, rtol=1e-4, row_l2=1e-4, lse=1e-4)}


def _worker_count():
    import os
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def _merge_nan(parts, like):
    out = np.full_like(like[0], np.nan), np.full_like(like[1], np.nan)
    for o, l in parts:
        m = ~np.isnan(l)
        out[0][m] = o[m]
        out[1][m] = l[m]
    return out


def oracle_definition_parallel(O, a, pairs, workers=None):
    """O.mla_decode_definition on `pairs`, the heads dealt out to a pool of threads (numpy's
    kernels release the interpreter lock).  A head stays within one thread, so its prefix
    expansion is still formed once.  The oracle itself is called as it stands."""
    from concurrent.futures import ThreadPoolExecutor
    from threadpoolctl import threadpool_limits
    workers = workers or _worker_count()
    heads = sorted({h for _, h in pairs})
    groups = [[p for p in pairs if p[1] in set(heads[w::workers])] for w in range(workers)]
    groups = [g for g in groups if g]
    with threadpool_limits(limits=1):
        with ThreadPoolExecutor(len(groups)) as ex:
            parts = list(ex.map(lambda g: O.mla_decode_definition(**a, pairs=g), groups))
    return _merge_nan(parts, parts[0])


def oracle_absorb_all_heads_parallel(O, a, requests=None, workers=None):
    """O.mla_decode_absorb_all_heads over `requests` (default: all), the requests dealt out to a
    pool of threads."""
    from concurrent.futures import ThreadPoolExecutor
    from threadpoolctl import threadpool_limits
    workers = workers or _worker_count()
    reqs = list(range(a["q"].shape[0])) if requests is None else list(requests)
    groups = [reqs[w::workers] for w in range(workers)]
    groups = [g for g in groups if g]
    with threadpool_limits(limits=1):
        with ThreadPoolExecutor(len(groups)) as ex:
            parts = list(ex.map(lambda g: O.mla_decode_absorb_all_heads(**a, requests=g), groups))
    return _merge_nan(parts, parts[0])


def dims_of(wl):
    return T.make_dims(wl.spec.heads, wl.sm_scale, wl.spec.dtype)


def run_library(wl, mode, device, expanded=None, flags=0):
    """wl: CPU Workload.  Returns (out, lse) as float64 numpy arrays."""
    d = wl.to(device)
    dims = dims_of(wl)
    old = T.typhoon_mla_set_debug_flags(flags)
    try:
        pk = pv = sk = sv = None
        L_s = wl.spec.prefix_len
        if mode in ("mixed", "naive_only", "auto") and L_s > 0:
            pk, pv = T.typhoon_mla_expand_prefix(dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv)
        if mode == "naive_only":
            sk, sv = T.typhoon_mla_expand_pool(dims, d.pool, d.w_uk, d.w_uv)
        out, lse = T.typhoon_mla_decode(
            dims, mode, d.q, L_s, prefix_k=pk, prefix_v=pv, prefix_ckv=d.prefix_ckv,
            prefix_krope=d.prefix_krope, suffix_pool=d.pool, block_table=d.block_table,
            suffix_lens=d.suffix_lens, max_suffix_len=wl.max_suffix_len, suffix_k_pool=sk,
            suffix_v_pool=sv, w_uk=d.w_uk, w_uv=d.w_uv)
        torch.cuda.synchronize(device)
    finally:
        T.typhoon_mla_set_debug_flags(old)
    return out.double().cpu().numpy(), lse.double().cpu().numpy()


def assert_parity(got, got_lse, ref, ref_lse, dtype, what="", logit_gain=1.0, peaked=None):
    """Element-wise, row-wise and LSE comparison wherever the reference was computed (not NaN).

    `logit_gain`: factor by which the queries (hence the logits) were scaled up; `peaked`: the
    softmax rows are dominated by few tokens (default: logit_gain > 1).  For peaked rows the
    bounds follow the rounding of the stored operands as derived at the top of this file."""
    tol = dict(TOL[dtype])
    if peaked is None:
        peaked = logit_gain > 1.0
    if dtype == "bf16" and peaked:
        g = max(1.0, logit_gain)
        tol["lse"] = 3.2e-3 * g
        tol["atol"] = max(tol["atol"], 2.5e-3 * g)
        tol["row_l2"] = max(tol["row_l2"], 5e-3 * g)
    mask = ~np.isnan(ref_lse)
    assert mask.any(), "reference is empty"
    g, r = got[mask], ref[mask]
    assert not np.isnan(g).any(), f"{what}: NaN in output"
    err = np.abs(g - r)
    bound = tol["atol"] + tol["rtol"] * np.abs(r)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert np.all(err <= bound), (
        f"{what}: element-wise |g-r|={err[worst]:.3e} > {bound[worst]:.3e} at {worst}; "
        f"max abs err {err.max():.3e}")
    norm = np.linalg.norm(r, axis=-1)
    rel = np.linalg.norm(g - r, axis=-1) / np.maximum(norm, 1e-30)
    nz = norm > 0
    assert np.all(rel[nz] <= tol["row_l2"]), (
        f"{what}: row relative L2 {rel[nz].max():.3e} > {tol['row_l2']:.1e}")
    assert np.all(g[~nz] == 0), f"{what}: rows that see no token must be exactly zero"
    gl, rl = got_lse[mask], ref_lse[mask]
    fin = np.isfinite(rl)
    assert np.array_equal(np.isneginf(gl), np.isneginf(rl)), f"{what}: -inf LSE pattern differs"
    if fin.any():
        dl = np.abs(gl[fin] - rl[fin]).max()
        assert dl <= tol["lse"], f"{what}: LSE error {dl:.3e} > {tol['lse']:.1e}"
    return dict(max_abs=float(err.max()), row_l2=float(rel[nz].max()) if nz.any() else 0.0)


def k_offset(h, ntok, t, d, dtype):
    """Expanded-K element offset, restated from the layout text in include/typhoon_mla.h."""
    if dtype == "fp32":
        return (h * ntok + t) * 192 + d
    ntb = (ntok + 31) // 32
    return ((((h * ntb + t // 32) * 12 + d // 16) * 64 + (t % 32) + 32 * ((d % 16) // 8)) * 8
            + d % 8)


def v_offset(h, ntok, t, d, dtype):
    if dtype == "fp32":
        return (h * ntok + t) * 128 + d
    ntb = (ntok + 31) // 32
    u = t % 16
    return (((((h * ntb + t // 32) * 2 + (t % 32) // 16) * 4 + d // 32) * 64 + (d % 32)
             + 32 * ((u // 4) % 2)) * 8 + 4 * (u // 8) + u % 4)


def unpack_expanded(k_bytes, v_bytes, H, ntok, dtype):
    """Opaque expanded buffers -> logical K [H, L, 192], V [H, L, 128] float64 numpy."""
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    k = k_bytes.view(td).double().cpu().numpy()
    v = v_bytes.view(td).double().cpu().numpy()
    hh, tt, dd = np.meshgrid(np.arange(H), np.arange(ntok), np.arange(192), indexing="ij")
    K = k[k_offset(hh, ntok, tt, dd, dtype)]
    hh, tt, dd = np.meshgrid(np.arange(H), np.arange(ntok), np.arange(128), indexing="ij")
    V = v[v_offset(hh, ntok, tt, dd, dtype)]
    return K, V
