"""Seeded random decode shapes against the tensor-form absorb checker (every output row) and the
definition oracle (a few pairs): batch sizes, head counts, query lengths, prefix and suffix
lengths and block sizes that no hand-picked case names, so that every launch plan the host can
come up with for small and medium problems -- kernel choice by rows per request, token chunks,
number of partials, merge pass, projection kernel -- meets the oracle at least once."""
import numpy as np
import pytest

from oracle import mla_oracle as O
from paper_2509_21081_amd import workloads as W
from tests import helpers as Hh

pytestmark = pytest.mark.gpu


def _specs(count=48, seed=2024):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        heads = int(rng.choice([16, 32, 48, 64, 128]))
        q_len = int(rng.choice([1, 1, 1, 2, 3]))
        # keep the oracle's work bounded: rows x tokens
        batch = int(rng.integers(1, max(2, 2600 // (heads * q_len)) + 1))
        u, v = rng.random(), rng.random()
        prefix_len = 0 if u < 0.12 else int(rng.choice([1, 33])) if u < 0.2 else \
            int(rng.integers(64, 3000))
        suffix_max = 0 if v < 0.08 else 5 if v < 0.16 else int(rng.integers(q_len, 1800))
        suffix_min = int(rng.integers(0, suffix_max + 1))
        out.append(dict(name=f"random_{i}", dtype="bf16", batch=batch, heads=heads, q_len=q_len,
                        prefix_len=prefix_len, suffix_min=suffix_min, suffix_max=suffix_max,
                        block_size=int(rng.choice([64, 128])), seed=1000 + i))
    return out


def _wide_specs(count=10, seed=77):
    """Many requests, few tokens: the large-grid kernels (pipelined prefix pass, streaming
    up-projection, multi-block query absorption) with ragged query counts."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        heads = int(rng.choice([16, 32, 64, 128]))
        q_len = int(rng.choice([1, 1, 2]))
        batch = int(rng.integers(130, 40000 // (heads * q_len) + 131))
        prefix_len = int(rng.integers(129, 420))
        suffix_max = int(rng.integers(q_len, 48))
        out.append(dict(name=f"wide_{i}", dtype="bf16", batch=batch, heads=heads, q_len=q_len,
                        prefix_len=prefix_len, suffix_min=int(rng.integers(0, suffix_max + 1)),
                        suffix_max=suffix_max, block_size=int(rng.choice([64, 128])),
                        seed=2000 + i))
    return out


SPECS = _specs() + _wide_specs()


@pytest.mark.parametrize("idx", range(len(SPECS)))
def test_random_shape(idx, gpu_device):
    kw = SPECS[idx]
    wl = W.make_workload(W.small_spec(**kw))
    a = wl.as_float64()
    ref2, ref2_lse = Hh.oracle_absorb_all_heads_parallel(O, a)
    B, H = kw["batch"], kw["heads"]
    pairs = sorted({(0, 0), (B - 1, H - 1), (B // 2, H // 2)})
    ref, ref_lse = O.mla_decode_definition(**a, pairs=pairs)
    print(f"random shape {idx}: {kw}", flush=True)
    for mode in ("mixed", "absorb_only", "auto"):
        got, got_lse = Hh.run_library(wl, mode, gpu_device)
        Hh.assert_parity(got, got_lse, ref2, ref2_lse, "bf16", f"random_{idx}/{mode}/absorb-form")
        Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"random_{idx}/{mode}/definition")
