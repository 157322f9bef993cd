"""The seeded input generators (CPU only): determinism, the poisoning that makes stray reads
visible, the full-size sample and the peaked variant used by the full-size parity tests."""
import dataclasses

import numpy as np
import torch

from paper_2509_21081_amd import workloads as W


def _small(**kw):
    base = dict(batch=7, heads=16, q_len=2, prefix_len=40, suffix_min=0, suffix_max=150, seed=3)
    base.update(kw)
    return W.small_spec(**base)


def test_same_seed_same_bits_and_poisoned_storage():
    a = W.make_workload(_small())
    b = W.make_workload(_small())
    for name in ("q", "prefix_ckv", "prefix_krope", "w_uk", "w_uv", "block_table", "suffix_lens"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    assert torch.equal(torch.isnan(a.pool), torch.isnan(b.pool))
    bs = a.spec.block_size
    used = set()
    for r in range(a.spec.batch):
        n = int(a.suffix_lens[r])
        nb = (n + bs - 1) // bs
        assert (a.block_table[r, nb:] == -1).all()                # padding of the table
        for i in range(nb):
            blk = int(a.block_table[r, i])
            assert blk not in used                                # no block is shared
            used.add(blk)
            valid = min(bs, n - i * bs)
            assert not torch.isnan(a.pool[blk, :valid].float()).any()
            assert torch.isnan(a.pool[blk, valid:].float()).all()  # tail of the last block
    for blk in set(range(a.pool.shape[0])) - used:
        assert torch.isnan(a.pool[blk].float()).all()              # spare blocks
    assert a.max_suffix_len == int(a.suffix_lens.max())


def test_peaked_variant_is_the_same_draw_with_scaled_queries():
    base = W.make_workload(_small())
    peaked = W.make_workload(dataclasses.replace(_small(), q_gain=8.0))
    assert torch.equal(peaked.q, (base.q.float() * 8.0).to(base.q.dtype))
    for name in ("prefix_ckv", "prefix_krope", "w_uk", "w_uv", "block_table", "suffix_lens"):
        assert torch.equal(getattr(peaked, name), getattr(base, name)), name
    assert torch.equal(torch.nan_to_num(peaked.pool.float()), torch.nan_to_num(base.pool.float()))


def test_sample_pairs_covers_the_extremes_and_every_request():
    wl = W.make_workload(_small(batch=40, heads=32, q_len=1, suffix_min=1, suffix_max=300, seed=9))
    pairs = W.sample_pairs(wl)
    assert pairs == sorted(set(pairs))
    B, H = 40, 32
    by_req = {}
    for b, h in pairs:
        by_req.setdefault(b, set()).add(h)
    full = [b for b, hs in by_req.items() if len(hs) == H]
    lens = wl.suffix_lens.numpy()
    assert len(full) >= 8
    for must in (0, B - 1, int(np.argmin(lens)), int(np.argmax(lens))):
        assert must in full
    assert set(by_req) == set(range(B))                           # every request appears
    common = set.intersection(*by_req.values())
    assert len(common) >= 2 and {0, H - 1} <= common              # for at least two heads
