"""GPU parity of the tree-shaped shared-prefix decode (typhoon_mla_decode_tree) against the fp64
oracle: the oracle has no notion of a tree, it is simply called once per group of requests with
the concatenation of the nodes on their path as the shared prefix."""
import numpy as np
import pytest
import torch

from oracle import mla_oracle as O
from paper_2509_21081_amd import binding as T
from paper_2509_21081_amd import workloads as W
from tests import helpers as Hh

pytestmark = pytest.mark.gpu


def _latents(n, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    td = W.torch_dtype(dtype)
    return (torch.randn((n, 512), generator=g).to(td), torch.randn((n, 64), generator=g).to(td))


# (level, batch_begin, batch_count, len) on top of the root, which every request shares
TREES = {
    "two_levels": [(1, 0, 2, 45), (1, 3, 3, 70), (2, 4, 1, 33)],
    "root_only": [],
    "empty_nodes": [(1, 0, 3, 0), (1, 3, 0, 50), (2, 1, 4, 129)],
}
# batch 160: a node shared by 150 requests runs the query-split prefix kernel on a sub-batch that
# does not start at request 0, its neighbour (10 requests) the token-split kernel
BIG_TREE = [(1, 0, 10, 300), (1, 10, 150, 260), (2, 100, 60, 64)]


@pytest.mark.parametrize("flags", [0, 1], ids=["mfma", "scalar"])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("heads,q_len", [(16, 1), (64, 2)])
@pytest.mark.parametrize("tree", list(TREES) + ["big"])
def test_tree_decode_matches_oracle(tree, heads, q_len, dtype, flags, gpu_device):
    if dtype == "fp32" and flags == 1:
        pytest.skip("fp32 always runs the scalar kernels")
    if tree == "big" and (heads != 16 or dtype != "bf16"):
        pytest.skip("the large batch runs once per kernel family")
    B = 160 if tree == "big" else 6
    wl = W.make_workload(W.small_spec(name=f"tree_{tree}", dtype=dtype, batch=B, heads=heads,
                                      q_len=q_len, prefix_len=90, suffix_min=0,
                                      suffix_max=40 if tree == "big" else 140,
                                      seed=50 + heads + q_len))
    extra = [(lv, b0, bc, ln) + _latents(ln, dtype, 700 + i)
             for i, (lv, b0, bc, ln) in enumerate(BIG_TREE if tree == "big" else TREES[tree])]
    a = wl.as_float64()
    f64 = lambda t: t.double().numpy()

    # ---- oracle: one call per request with its path's tokens as the shared prefix
    ref = np.zeros((B, q_len, heads, 128))
    ref_lse = np.zeros((B, q_len, heads))
    for b in range(B):
        ckv, kr = [a["prefix_ckv"]], [a["prefix_krope"]]
        for lv, b0, bc, ln, c, r in sorted(extra, key=lambda e: e[0]):
            if b0 <= b < b0 + bc and ln > 0:
                ckv.append(f64(c))
                kr.append(f64(r))
        o, l = O.mla_decode_definition(
            q=a["q"][b:b + 1], prefix_ckv=np.concatenate(ckv), prefix_krope=np.concatenate(kr),
            pool=a["pool"], block_table=a["block_table"][b:b + 1],
            suffix_lens=a["suffix_lens"][b:b + 1], w_uk=a["w_uk"], w_uv=a["w_uv"],
            sm_scale=a["sm_scale"])
        ref[b], ref_lse[b] = o[0], l[0]

    # ---- library
    d = wl.to(gpu_device)
    dims = Hh.dims_of(wl)
    print(f"tree={tree} heads={heads} q_len={q_len} dtype={dtype} flags={flags}", flush=True)
    old = T.typhoon_mla_set_debug_flags(flags)
    try:
        keep = []
        nodes = []
        pk, pv = T.typhoon_mla_expand_prefix(dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv)
        keep.append((pk, pv))
        nodes.append((pk, pv, wl.spec.prefix_len, 0, 0, B))
        for lv, b0, bc, ln, c, r in extra:
            if ln > 0:
                k, v = T.typhoon_mla_expand_prefix(dims, c.to(gpu_device), r.to(gpu_device),
                                                   d.w_uk, d.w_uv)
                keep.append((k, v))
            else:
                k = v = None
            nodes.append((k, v, ln, lv, b0, bc))
        out, lse = T.typhoon_mla_decode_tree(
            dims, d.q, nodes, suffix_pool=d.pool, block_table=d.block_table,
            suffix_lens=d.suffix_lens, max_suffix_len=wl.max_suffix_len, w_uk=d.w_uk, w_uv=d.w_uv)
        torch.cuda.synchronize(gpu_device)
    finally:
        T.typhoon_mla_set_debug_flags(old)
    Hh.assert_parity(out.double().cpu().numpy(), lse.double().cpu().numpy(), ref, ref_lse, dtype,
                     f"tree/{tree}/{dtype}")


def test_tree_with_one_root_equals_plain_decode(gpu_device):
    """A tree that is just the root must reproduce typhoon_mla_decode(mixed) bit for bit."""
    wl = W.make_workload(W.small_spec(name="tree_plain", batch=5, heads=64, prefix_len=200,
                                      suffix_min=5, suffix_max=150, seed=61))
    d = wl.to(gpu_device)
    dims = Hh.dims_of(wl)
    pk, pv = T.typhoon_mla_expand_prefix(dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv)
    o1, l1 = T.typhoon_mla_decode(dims, "mixed", d.q, wl.spec.prefix_len, prefix_k=pk, prefix_v=pv,
                                  suffix_pool=d.pool, block_table=d.block_table,
                                  suffix_lens=d.suffix_lens, max_suffix_len=wl.max_suffix_len,
                                  w_uk=d.w_uk, w_uv=d.w_uv)
    o2, l2 = T.typhoon_mla_decode_tree(dims, d.q, [(pk, pv, wl.spec.prefix_len, 0, 0, 5)],
                                       suffix_pool=d.pool, block_table=d.block_table,
                                       suffix_lens=d.suffix_lens,
                                       max_suffix_len=wl.max_suffix_len, w_uk=d.w_uk, w_uv=d.w_uv)
    torch.cuda.synchronize(gpu_device)
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
