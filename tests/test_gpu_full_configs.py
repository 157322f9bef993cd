"""Full-size parity: the five benchmark configurations, in the launch configuration bench.py
times, compared with the fp64 oracle on sampled (request, head) outputs it can compute one by
one (definition oracle), plus wider coverage with the absorb-form fp64 checker (pinned to the
definition by the CPU tests) and cross-mode agreement over every output row."""
import numpy as np
import pytest
import torch

from oracle import mla_oracle as O
from paper_2509_21081_amd import binding as T
from paper_2509_21081_amd import workloads as W
from tests import helpers as Hh

pytestmark = pytest.mark.gpu

FULL = ["cfg2_dsv3_b64", "cfg3_long_prompt", "cfg4_mtp", "cfg5_tp_rank", "cfg5b_no_prefix"]


def _sample(wl, n_req, heads):
    B = wl.spec.batch
    lens = wl.suffix_lens
    reqs = [int(torch.argmin(lens)), int(torch.argmax(lens)), 0, B - 1, B // 2]
    uniq = []
    for b in reqs:
        if b not in uniq:
            uniq.append(b)
    return [(b, h) for b in uniq[:n_req] for h in heads]


@pytest.mark.parametrize("name", FULL)
def test_full_config(name, gpu_device):
    spec = W.CONFIGS[name]
    wl = W.make_workload(spec)
    a = wl.as_float64()
    H = spec.heads
    heads = sorted({0, H // 2 - 1, H - 1})
    pairs_def = _sample(wl, 3, heads)
    ref, ref_lse = O.mla_decode_definition(**a, pairs=pairs_def)
    # wider, cheaper sample with the absorb-form checker: all heads of two requests
    pairs_abs = _sample(wl, 2, list(range(H)))
    ref2, ref2_lse = O.mla_decode_absorb_form(**a, pairs=pairs_abs)
    outs = {}
    for mode in ["mixed", "absorb_only", "naive_only"]:
        print(f"full config {name} mode={mode}", flush=True)
        got, got_lse = Hh.run_library(wl, mode, gpu_device)
        Hh.assert_parity(got, got_lse, ref, ref_lse, spec.dtype, f"{name}/{mode}/definition")
        Hh.assert_parity(got, got_lse, ref2, ref2_lse, spec.dtype, f"{name}/{mode}/absorb-form")
        assert not np.isnan(got).any() and not np.isnan(got_lse).any()
        outs[mode] = (got, got_lse)
        torch.cuda.empty_cache()
    # every row: the three formulations agree with each other (independent code paths)
    for mode in ["absorb_only", "naive_only"]:
        d = np.abs(outs[mode][0] - outs["mixed"][0])
        bound = 1e-2 + 2e-2 * np.abs(outs["mixed"][0])
        assert np.all(d <= bound), f"{name}: {mode} vs mixed differ by {d.max():.3e}"
        assert np.abs(outs[mode][1] - outs["mixed"][1]).max() <= 4e-3
