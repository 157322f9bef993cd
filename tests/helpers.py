"""Shared test utilities: run a workload through the C-ABI library, compare with the oracle."""
import numpy as np
import torch

from paper_2509_21081_amd import binding as T

# Tolerances: bf16 I/O with fp32 accumulation -> max-abs 1e-2 + max-rel 2e-2 element-wise, plus a
# row-wise relative L2 bound and an LSE bound so that small outputs cannot hide an error;
# fp32 mode -> 1e-4 for all three.
TOL = {"bf16": dict(atol=1e-2, rtol=2e-2, row_l2=2e-2, lse=2e-3),
       "fp32": dict(atol=1e-4, rtol=1e-4, row_l2=1e-4, lse=1e-4)}


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


def assert_parity(got, got_lse, ref, ref_lse, dtype, what="", logit_gain=1.0):
    """Element-wise, row-wise and LSE comparison wherever the reference was computed (not NaN).

    `logit_gain`: factor by which the queries (hence the logits) were scaled up; the bf16
    rounding of the expanded keys and of the absorbed query perturbs a logit in proportion to
    its magnitude, so the LSE bound scales with it (the output bounds do not)."""
    tol = dict(TOL[dtype])
    if dtype == "bf16":
        tol["lse"] *= max(1.0, logit_gain)
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
