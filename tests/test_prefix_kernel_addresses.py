"""Host-side walk of every global -> LDS transfer the software-pipelined prefix kernel issues
(CPU only).  The kernel's ring constants are read from its source; the schedule below restates
which transfer group is issued where (the fill before the first period, the pre-period, then one
group per period, unguarded only in the steady state) and checks, for splits that end in a short
or partial last chunk as well:
  * every transfer reads 1 KiB inside the expanded K / V buffers of typhoon_mla_expanded_*_bytes,
    also for the last head and the last split;
  * every transfer lands inside the kernel's LDS allocation;
  * a ring slot is refilled only after the barrier that follows the last period reading it;
  * every block read in a period has been issued, and the transfers the top-of-period wait
    leaves in flight do not include it."""
import os
import re

import pytest

from paper_2509_21081_amd import binding as T
from paper_2509_21081_amd import build as B

SRC = open(os.path.join(B.CSRC, "tmla_prefix_mfma.hip")).read()


def _const(name):
    m = re.search(r"constexpr int %s = ([^;]+);" % name, SRC)
    assert m, name
    expr = m.group(1).split("//")[0]
    for other in ("PL_AHEAD", "PL_NK", "PL_NV", "PL_K_BYTES", "PL_V_BYTES", "PL_V_BASE",
                  "K_BLK_ELEMS", "V_BLK_ELEMS"):
        if other in expr and other != name:
            expr = expr.replace(other, str(_const(other)) if other.startswith("PL_") else
                                {"K_BLK_ELEMS": "6144", "V_BLK_ELEMS": "4096"}[other])
    return int(eval(expr))


AHEAD, NK, NV = _const("PL_AHEAD"), _const("PL_NK"), _const("PL_NV")
KB, VB, VBASE, LDS = _const("PL_K_BYTES"), _const("PL_V_BYTES"), _const("PL_V_BASE"), \
    _const("PL_LDS_BYTES")


def _walk(H, Ls, np_split, p_chunk):
    """Yields (period_issued, kind, block, global_offset, lds_offset, guarded) for the worst
    head (the last one) of every split; period -2 = fill, -1 = pre-period."""
    ntb = (Ls + 31) // 32
    bps = p_chunk // 32
    for sp in range(np_split):
        tb0 = sp * bps
        tb1 = min(ntb, tb0 + bps)
        nblk = tb1 - tb0
        if nblk <= 0:
            continue
        has_tail = tb1 == ntb and Ls % 32 != 0
        nfull = nblk - 1 if has_tail else nblk
        kbase = ((H - 1) * ntb + tb0) * KB
        vbase = ((H - 1) * ntb + tb0) * VB
        rbase = tb0 * KB      # fragments 8 .. 11 (the RoPE part) come from head 0's blocks
        # steady periods: t = 2, 3, ... in pairs while t + 1 + AHEAD < nblk
        steady = set()
        t = 2
        while t + 1 + AHEAD < nblk:
            steady.update((t, t + 1))
            t += 2

        def group(k, when, guarded):
            out = []
            if (not guarded) or k < nblk:
                for f in range(3):
                    for w in range(4):
                        out.append((when, "K", k,
                                    (rbase if f == 2 else kbase) + k * KB + f * 4096 + w * 1024,
                                    (k % NK) * KB + f * 4096 + w * 1024, guarded))
            kv = k - 3
            if (not guarded) or 0 <= kv < nblk:
                for f in range(2):
                    for w in range(4):
                        out.append((when, "V", kv, vbase + kv * VB + f * 4096 + w * 1024,
                                    VBASE + (kv % NV) * VB + f * 4096 + w * 1024, guarded))
            return out
        for k in range(AHEAD - 1):
            yield from group(k, -2, True)
        yield from group(AHEAD - 1, -1, True)
        for t in range(0, nfull + 1):
            yield from group(t + AHEAD, t, t not in steady)
        yield ("end", nblk, nfull, ntb, sp, steady)


CASES = [  # (H, Ls, forced splits): long steady runs, short chunks, partial tails, odd chunk counts
    (128, 32768, 2), (128, 8192, 2), (16, 16384, 8), (16, 1100, 1), (16, 1024, 1), (16, 288, 1),
    (16, 40, 1), (16, 31, 1), (16, 4000, 3), (32, 33 * 32 + 5, 2), (16, 2 * 1024 + 7, 5),
]


@pytest.mark.parametrize("H,Ls,splits", CASES)
def test_every_transfer_stays_inside_its_buffers_and_ring_slots_are_free(H, Ls, splits):
    dims = T.make_dims(H, 0.07, "bf16")
    k_bytes = T.typhoon_mla_expanded_k_bytes(dims, Ls)
    v_bytes = T.typhoon_mla_expanded_v_bytes(dims, Ls)
    # the host plan: chunk = ceil(Ls / splits) rounded up to whole 32-token blocks
    p_chunk = ((Ls + splits - 1) // splits + 31) // 32 * 32
    np_split = (Ls + p_chunk - 1) // p_chunk
    issued_k, issued_v = {}, {}
    n = 0
    for rec in _walk(H, Ls, np_split, p_chunk):
        if rec[0] == "end":
            _, nblk, nfull, ntb, sp, steady = rec
            # K(b) is first read at the end of period b - 2 (the head of the block after next) and
            # V(b) in period b + 1; the wait at the top of a period can only cover transfers issued
            # in an earlier period (or before the first one)
            for b in range(nblk):
                assert issued_k[b] < max(b - 2, 0), (sp, b, issued_k[b])
                assert issued_v[b] < b + 1, (sp, b, issued_v[b])
            # ring slots: block b + NK reuses K(b)'s slot, issued in period b (after the barrier
            # that ends period b - 1, the last reader of K(b)); V(b + NV) is issued in period
            # b + NV + 3 - AHEAD >= b + 2, after the barrier ending period b + 1
            for b in range(nblk):
                if b + NK in issued_k:
                    assert issued_k[b + NK] >= b, (sp, b)
                if b + NV in issued_v:
                    assert issued_v[b + NV] >= b + 2, (sp, b)
            # unguarded (steady) periods touch only blocks that exist
            for t in steady:
                assert t + AHEAD < nblk and t + AHEAD - 3 >= 0
            issued_k, issued_v = {}, {}
            continue
        when, kind, blk, goff, loff, guarded = rec
        n += 1
        limit = k_bytes if kind == "K" else v_bytes
        assert 0 <= goff and goff + 1024 <= limit, (kind, blk, goff, limit)
        assert 0 <= loff and loff + 1024 <= LDS, (kind, blk, loff)
        if kind == "V":
            assert loff >= VBASE
        else:
            assert loff + 1024 <= VBASE
        (issued_k if kind == "K" else issued_v).setdefault(blk, when)
    assert n > 0


def test_ring_constants_fill_the_lds_exactly():
    assert NK & (NK - 1) == 0 and NV & (NV - 1) == 0
    assert VBASE == NK * KB and LDS == VBASE + NV * VB == 160 * 1024
    assert KB == 32 * 192 * 2 and VB == 32 * 128 * 2
