"""Pins for the fp64 oracle: it is checked against what the paper and the mathematics fix, not
against itself.  (CPU only.)

  I1 naive == absorb                       (paper Section 1/2.1: the two forms are equivalent)
  I2 LSE merge of any token partition == one softmax   (Algorithm 1 step 8, Section 3.2)
  I3 softmax rows sum to 1; outputs inside the hull of the values
  I4 scalar triple-loop brute force on tiny inputs
  I5 closed forms and symmetries
  I6 the naive form is textbook multi-head attention -> library fp64 SDPA on expanded K/V
"""
import math

import numpy as np
import pytest
import torch

from oracle import mla_oracle as O
from paper_2509_21081_amd import workloads as W


def _wl(**kw):
    kw.setdefault("dtype", "fp32")
    spec = W.small_spec(**kw)
    return W.make_workload(spec, poison=True)


def _args(wl):
    return wl.as_float64()


# ---------------------------------------------------------------- I4: brute force
def _brute_force(a, b, s, h):
    """No matrix code at all: python loops straight from the definition."""
    q = a["q"][b, s, h]
    L_s = a["prefix_ckv"].shape[0]
    bs = a["pool"].shape[1]
    S_q = a["q"].shape[1]
    n_suf = int(a["suffix_lens"][b])
    toks = []
    for t in range(L_s):
        toks.append((a["prefix_ckv"][t], a["prefix_krope"][t]))
    vis = max(0, min(n_suf, n_suf - S_q + s + 1))
    for j in range(vis):
        row = a["pool"][a["block_table"][b][j // bs]][j % bs]
        toks.append((row[:512], row[512:]))
    if not toks:
        return [0.0] * 128, -math.inf
    xs, vs = [], []
    for c, r in toks:
        dot = 0.0
        for i in range(128):
            kn = 0.0
            for l in range(512):
                kn += a["w_uk"][h][i][l] * c[l]
            dot += q[i] * kn
        for i in range(64):
            dot += q[128 + i] * r[i]
        xs.append(a["sm_scale"] * dot)
        v = []
        for i in range(128):
            acc = 0.0
            for l in range(512):
                acc += a["w_uv"][h][i][l] * c[l]
            v.append(acc)
        vs.append(v)
    m = max(xs)
    es = [math.exp(x - m) for x in xs]
    z = sum(es)
    out = [sum(es[t] / z * vs[t][i] for t in range(len(xs))) for i in range(128)]
    return out, m + math.log(z)


def test_I4_brute_force_tiny():
    wl = _wl(batch=2, heads=2, q_len=2, prefix_len=3, suffix_min=1, suffix_max=4, block_size=2,
             seed=5)
    a = _args(wl)
    out, lse = O.mla_decode_definition(**a)
    for b in range(2):
        for s in range(2):
            for h in range(2):
                o_bf, l_bf = _brute_force(a, b, s, h)
                np.testing.assert_allclose(out[b, s, h], o_bf, rtol=1e-11, atol=1e-13)
                assert abs(lse[b, s, h] - l_bf) < 1e-11


# ---------------------------------------------------------------- I1: naive == absorb
@pytest.mark.parametrize("q_len,prefix_len", [(1, 37), (2, 20), (3, 0)])
def test_I1_naive_equals_absorb(q_len, prefix_len):
    wl = _wl(batch=3, heads=4, q_len=q_len, prefix_len=prefix_len, suffix_min=0, suffix_max=70,
             block_size=16, seed=7 + q_len)
    a = _args(wl)
    o_n, l_n = O.mla_decode_definition(**a)
    o_a, l_a = O.mla_decode_absorb_form(**a)
    assert np.all(np.isfinite(o_n))
    np.testing.assert_allclose(o_a, o_n, rtol=1e-10, atol=1e-13)
    fin = np.isfinite(l_n)
    np.testing.assert_allclose(l_a[fin], l_n[fin], rtol=0, atol=1e-11)
    assert np.array_equal(np.isfinite(l_a), fin)


@pytest.mark.parametrize("q_len,prefix_len", [(1, 37), (2, 20), (3, 0)])
def test_I1_all_heads_absorb_form_equals_definition(q_len, prefix_len):
    """The tensor-form absorb checker (all heads of a request at once) against the naive
    definition, on the same ragged inputs as the per-row absorb form: empty suffixes, queries
    that see nothing, poisoned storage behind every request's last token."""
    wl = _wl(batch=3, heads=4, q_len=q_len, prefix_len=prefix_len, suffix_min=0, suffix_max=70,
             block_size=16, seed=7 + q_len)
    a = _args(wl)
    o_n, l_n = O.mla_decode_definition(**a)
    o_a, l_a = O.mla_decode_absorb_all_heads(**a)
    np.testing.assert_allclose(o_a, o_n, rtol=1e-10, atol=1e-13)
    fin = np.isfinite(l_n)
    np.testing.assert_allclose(l_a[fin], l_n[fin], rtol=0, atol=1e-11)
    assert np.array_equal(np.isneginf(l_a), np.isneginf(l_n)) and not np.isnan(o_a).any()
    # a subset of requests leaves the others untouched
    o_s, l_s = O.mla_decode_absorb_all_heads(**a, requests=[2])
    np.testing.assert_array_equal(o_s[2], o_a[2])
    assert np.isnan(o_s[:2]).all() and np.isnan(l_s[:2]).all()


def test_I4_all_heads_absorb_form_against_brute_force():
    wl = _wl(batch=2, heads=2, q_len=2, prefix_len=3, suffix_min=1, suffix_max=4, block_size=2,
             seed=5)
    a = _args(wl)
    out, lse = O.mla_decode_absorb_all_heads(**a)
    for b in range(2):
        for s in range(2):
            for h in range(2):
                o_bf, l_bf = _brute_force(a, b, s, h)
                np.testing.assert_allclose(out[b, s, h], o_bf, rtol=1e-10, atol=1e-13)
                assert abs(lse[b, s, h] - l_bf) < 1e-11


def test_I5_all_heads_absorb_form_causal_rows():
    # S_q = 3, suffix lengths 5, 2, 0 and no prefix (see test_I5_causal_mask_and_empty_rows)
    a = _tiny(0, [5, 2, 0], S_q=3, seed=8)
    out, lse = O.mla_decode_absorb_all_heads(**a)
    assert np.all(out[1, 0] == 0) and np.all(np.isneginf(lse[1, 0]))
    row0 = a["pool"][a["block_table"][1, 0], 0]
    np.testing.assert_allclose(out[1, 1, 0], a["w_uv"][0] @ row0[:512], rtol=1e-12)
    assert np.all(out[2] == 0) and np.all(np.isneginf(lse[2])) and not np.any(np.isnan(out))


# ---------------------------------------------------------------- I2: split + merge == full
def _partial(a, b, s, h, idx_tokens):
    """softmax restricted to a subset of the visible tokens, via the oracle's own pieces."""
    L_s = a["prefix_ckv"].shape[0]
    n = int(a["suffix_lens"][b])
    rows = O.gather_suffix_rows(a["pool"], a["block_table"][b], n)
    c = np.concatenate([a["prefix_ckv"], rows[:, :512]])
    r = np.concatenate([a["prefix_krope"], rows[:, 512:]])
    k, v = O.expand_tokens(c, r, a["w_uk"][h], a["w_uv"][h])
    x = a["sm_scale"] * (k[idx_tokens] @ a["q"][b, s, h])
    return O.softmax_attend(x, v[idx_tokens])


@pytest.mark.parametrize("cuts", [[40], [0], [90], [1, 2, 50, 50, 89], [13, 40, 77]])
def test_I2_merge_of_partition_equals_full(cuts):
    wl = _wl(batch=1, heads=2, q_len=1, prefix_len=40, suffix_min=50, suffix_max=50, seed=3)
    a = _args(wl)
    full_o, full_l = O.mla_decode_definition(**a)
    total = 90
    edges = [0] + list(cuts) + [total]
    for h in range(2):
        outs, lses = [], []
        for lo, hi in zip(edges[:-1], edges[1:]):
            o, l = _partial(a, 0, 0, h, np.arange(lo, hi))
            outs.append(o); lses.append(l)
        o, l = O.combine_lse(np.stack(outs), np.array(lses))
        np.testing.assert_allclose(o, full_o[0, 0, h], rtol=1e-11, atol=1e-14)
        assert abs(l - full_l[0, 0, h]) < 1e-12


def test_I2_merge_is_associative_and_ignores_empty():
    rng = np.random.default_rng(0)
    outs = rng.normal(size=(4, 5, 8))
    lses = rng.normal(size=(4, 5)) * 3
    o_all, l_all = O.combine_lse(outs, lses)
    o01, l01 = O.combine_lse(outs[:2], lses[:2])
    o23, l23 = O.combine_lse(outs[2:], lses[2:])
    o_n, l_n = O.combine_lse(np.stack([o01, o23]), np.stack([l01, l23]))
    np.testing.assert_allclose(o_n, o_all, rtol=1e-12)
    np.testing.assert_allclose(l_n, l_all, rtol=1e-12)
    # an empty partial (LSE = -inf, garbage output) changes nothing
    outs_e = np.concatenate([outs, np.full((1, 5, 8), np.nan)])
    lses_e = np.concatenate([lses, np.full((1, 5), -np.inf)])
    o_e, l_e = O.combine_lse(outs_e, lses_e)
    np.testing.assert_allclose(o_e, o_all, rtol=1e-12)
    np.testing.assert_allclose(l_e, l_all, rtol=1e-12)
    # all empty -> zeros and -inf
    o_z, l_z = O.combine_lse(np.full((2, 3, 4), np.nan), np.full((2, 3), -np.inf))
    assert np.all(o_z == 0) and np.all(np.isneginf(l_z))


def test_I2_merge_two_way_closed_form():
    # two partials with weights e^{l1}, e^{l2}: o = (e^{l1} o1 + e^{l2} o2)/(e^{l1}+e^{l2})
    o1, o2 = np.array([1.0, -2.0]), np.array([3.0, 5.0])
    l1, l2 = math.log(3.0), math.log(1.0)
    o, l = O.combine_lse(np.stack([o1, o2]), np.array([l1, l2]))
    np.testing.assert_allclose(o, (3 * o1 + o2) / 4, rtol=1e-14)
    assert abs(l - math.log(4.0)) < 1e-14


# ---------------------------------------------------------------- I3: softmax invariants
def test_I3_softmax_rows_and_hull():
    rng = np.random.default_rng(1)
    x = rng.normal(size=33) * 4
    v = np.eye(33)               # values = unit vectors: the output IS the probability row
    p, lse = O.softmax_attend(x, v)
    assert abs(p.sum() - 1) < 1e-14 and np.all(p >= 0)
    np.testing.assert_allclose(p, np.exp(x - lse), rtol=1e-13)
    wl = _wl(batch=2, heads=3, prefix_len=17, suffix_min=5, suffix_max=30, seed=9)
    a = _args(wl)
    out, _ = O.mla_decode_definition(**a)
    k, v = O.expand_prefix_definition(a["prefix_ckv"], a["prefix_krope"], a["w_uk"], a["w_uv"])
    for b in range(2):
        rows = O.gather_suffix_rows(a["pool"], a["block_table"][b], int(a["suffix_lens"][b]))
        for h in range(3):
            vs = np.concatenate([v[h], rows[:, :512] @ a["w_uv"][h].T])
            assert np.all(out[b, 0, h] <= vs.max(axis=0) + 1e-12)
            assert np.all(out[b, 0, h] >= vs.min(axis=0) - 1e-12)


# ---------------------------------------------------------------- I5: closed forms
def _tiny(L_s, lens, H=2, S_q=1, bs=4, seed=0, poison=True):
    rng = np.random.default_rng(seed)
    B = len(lens)
    nb = [max(1, -(-n // bs)) for n in lens]
    pool = np.full((sum(nb) + 1, bs, 576), np.nan if poison else 0.0)
    bt = np.full((B, max(nb)), -1, dtype=np.int64)
    order = rng.permutation(sum(nb) + 1)
    p = 0
    for b, n in enumerate(lens):
        for i in range(-(-n // bs)):
            bt[b, i] = order[p]; p += 1
            m = min(bs, n - i * bs)
            pool[bt[b, i], :m] = rng.normal(size=(m, 576))
    return dict(q=rng.normal(size=(B, S_q, H, 192)), prefix_ckv=rng.normal(size=(L_s, 512)),
                prefix_krope=rng.normal(size=(L_s, 64)), pool=pool, block_table=bt,
                suffix_lens=np.array(lens), w_uk=rng.normal(size=(H, 128, 512)) * 0.05,
                w_uv=rng.normal(size=(H, 128, 512)) * 0.05, sm_scale=0.11)


def test_I5_single_token():
    a = _tiny(1, [0])
    out, lse = O.mla_decode_definition(**a)
    for h in range(2):
        v0 = a["w_uv"][h] @ a["prefix_ckv"][0]
        k0 = np.concatenate([a["w_uk"][h] @ a["prefix_ckv"][0], a["prefix_krope"][0]])
        np.testing.assert_allclose(out[0, 0, h], v0, rtol=1e-13)
        assert abs(lse[0, 0, h] - a["sm_scale"] * (k0 @ a["q"][0, 0, h])) < 1e-13
    # same with the single token living in the paged suffix
    a = _tiny(0, [1])
    out, lse = O.mla_decode_definition(**a)
    row = a["pool"][a["block_table"][0, 0], 0]
    np.testing.assert_allclose(out[0, 0, 1], a["w_uv"][1] @ row[:512], rtol=1e-13)


def test_I5_zero_query_gives_uniform_mean():
    a = _tiny(5, [6, 0])
    a["q"][:] = 0
    out, lse = O.mla_decode_definition(**a)
    rows = O.gather_suffix_rows(a["pool"], a["block_table"][0], 6)
    c = np.concatenate([a["prefix_ckv"], rows[:, :512]])
    np.testing.assert_allclose(out[0, 0, 0], (c @ a["w_uv"][0].T).mean(axis=0), rtol=1e-12)
    np.testing.assert_allclose(lse[0, 0], math.log(11), rtol=1e-14)
    np.testing.assert_allclose(lse[1, 0], math.log(5), rtol=1e-14)


def test_I5_identical_tokens_and_logit_shift():
    a = _tiny(4, [4])
    a["prefix_ckv"][:] = a["prefix_ckv"][0]
    a["prefix_krope"][:] = a["prefix_krope"][0]
    for j in range(4):
        a["pool"][a["block_table"][0, 0], j, :512] = a["prefix_ckv"][0]
        a["pool"][a["block_table"][0, 0], j, 512:] = a["prefix_krope"][0]
    out, lse = O.mla_decode_definition(**a)
    np.testing.assert_allclose(out[0, 0, 1], a["w_uv"][1] @ a["prefix_ckv"][0], rtol=1e-12)
    # adding delta * q_rope/|q_rope|^2 to every rope key shifts every logit of that head by
    # sm_scale * delta: output unchanged, LSE shifted.
    b = _tiny(6, [5], seed=3)
    out0, lse0 = O.mla_decode_definition(**b)
    h, delta = 0, 2.5
    qr = b["q"][0, 0, h, 128:]
    shift = delta * qr / (qr @ qr)
    b["prefix_krope"] += shift
    blk = b["block_table"][0]
    for j in range(5):
        b["pool"][blk[j // 4], j % 4, 512:] += shift
    out1, lse1 = O.mla_decode_definition(**b)
    np.testing.assert_allclose(out1[0, 0, h], out0[0, 0, h], rtol=1e-10, atol=1e-13)
    assert abs((lse1[0, 0, h] - lse0[0, 0, h]) - b["sm_scale"] * delta) < 1e-11


def test_I5_permutations_leave_result_unchanged():
    a = _tiny(7, [9, 3], seed=4)
    out0, lse0 = O.mla_decode_definition(**a)
    # permute prefix tokens (S_q = 1: order is irrelevant)
    perm = np.random.default_rng(0).permutation(7)
    b = dict(a); b["prefix_ckv"] = a["prefix_ckv"][perm]; b["prefix_krope"] = a["prefix_krope"][perm]
    out1, lse1 = O.mla_decode_definition(**b)
    np.testing.assert_allclose(out1, out0, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(lse1, lse0, rtol=1e-13)
    # relocate the physical blocks (new pool order + matching block table)
    nblk = a["pool"].shape[0]
    p2 = np.random.default_rng(1).permutation(nblk)         # new_pool[p2[i]] = pool[i]
    c = dict(a); new_pool = np.empty_like(a["pool"]); new_pool[p2] = a["pool"]
    c["pool"] = new_pool
    c["block_table"] = np.where(a["block_table"] >= 0, p2[np.maximum(a["block_table"], 0)], -1)
    out2, lse2 = O.mla_decode_definition(**c)
    np.testing.assert_array_equal(out2, out0)
    np.testing.assert_array_equal(lse2, lse0)


def test_I5_zero_weights():
    a = _tiny(5, [5], seed=6)
    z = dict(a); z["w_uv"] = np.zeros_like(a["w_uv"])
    out, _ = O.mla_decode_definition(**z)
    assert np.all(out == 0)
    z = dict(a); z["w_uk"] = np.zeros_like(a["w_uk"])
    _, lse = O.mla_decode_definition(**z)
    rows = O.gather_suffix_rows(a["pool"], a["block_table"][0], 5)
    r = np.concatenate([a["prefix_krope"], rows[:, 512:]])
    x = a["sm_scale"] * (r @ a["q"][0, 0, 1, 128:])
    assert abs(lse[0, 0, 1] - (x.max() + math.log(np.exp(x - x.max()).sum()))) < 1e-12


def test_I5_causal_mask_and_empty_rows():
    # S_q = 3, suffix lengths 5, 2, 0 and no prefix: query s sees suffix tokens j <= L - 3 + s.
    a = _tiny(0, [5, 2, 0], S_q=3, seed=8)
    out, lse = O.mla_decode_definition(**a)
    # request 1 (L = 2): s = 0 sees nothing, s = 1 sees token 0, s = 2 sees tokens 0, 1
    assert np.all(out[1, 0] == 0) and np.all(np.isneginf(lse[1, 0]))
    row0 = a["pool"][a["block_table"][1, 0], 0]
    np.testing.assert_allclose(out[1, 1, 0], a["w_uv"][0] @ row0[:512], rtol=1e-12)
    assert np.all(np.isfinite(out[1, 2]))
    # request 2 sees nothing at any position; no NaN leaks from poisoned storage
    assert np.all(out[2] == 0) and np.all(np.isneginf(lse[2]))
    assert not np.any(np.isnan(out))
    # request 0, last query position == unmasked attention over all 5 tokens
    b = dict(a); b["q"] = a["q"][:, 2:3]
    out_last, lse_last = O.mla_decode_definition(**b)
    np.testing.assert_allclose(out[0, 2], out_last[0, 0], rtol=1e-13)
    # and position 0 == attention over the first 3 tokens only
    c = dict(a); c["q"] = a["q"][:, 0:1]; c["suffix_lens"] = np.array([3, 0, 0])
    out_first, _ = O.mla_decode_definition(**c)
    np.testing.assert_allclose(out[0, 0], out_first[0, 0], rtol=1e-13)


# ---------------------------------------------------------------- I6: library SDPA
def test_I6_matches_library_sdpa_on_expanded_cache():
    wl = _wl(batch=2, heads=4, q_len=1, prefix_len=29, suffix_min=21, suffix_max=21, block_size=8,
             seed=12)
    a = _args(wl)
    out, _ = O.mla_decode_definition(**a)
    k_p, v_p = O.expand_prefix_definition(a["prefix_ckv"], a["prefix_krope"], a["w_uk"], a["w_uv"])
    for b in range(2):
        rows = O.gather_suffix_rows(a["pool"], a["block_table"][b], 21)
        k_s, v_s = O.expand_prefix_definition(rows[:, :512], rows[:, 512:], a["w_uk"], a["w_uv"])
        k = torch.from_numpy(np.concatenate([k_p, k_s], axis=1))[None]      # [1, H, L, 192]
        v = torch.from_numpy(np.concatenate([v_p, v_s], axis=1))[None]
        qq = torch.from_numpy(a["q"][b].transpose(1, 0, 2))[None]           # [1, H, S_q, 192]
        ref = torch.nn.functional.scaled_dot_product_attention(qq, k, v, scale=a["sm_scale"])
        np.testing.assert_allclose(out[b, 0], ref[0, :, 0].numpy(), rtol=1e-10, atol=1e-13)


def test_pairs_subset_matches_full():
    wl = _wl(batch=3, heads=4, prefix_len=10, suffix_min=3, suffix_max=20, seed=2)
    a = _args(wl)
    full, lfull = O.mla_decode_definition(**a)
    sub, lsub = O.mla_decode_definition(**a, pairs=[(2, 1), (0, 3)])
    np.testing.assert_array_equal(sub[2, :, 1], full[2, :, 1])
    np.testing.assert_array_equal(lsub[0, :, 3], lfull[0, :, 3])
    assert np.isnan(sub[1]).all()
