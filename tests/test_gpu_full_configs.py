"""Full-size parity: the five benchmark configurations, in the launch configuration bench.py
times, against the fp64 oracle.

  * definition oracle on the deterministic sample of workloads.sample_pairs: every head of eight
    requests (first, last, shortest and longest suffix, four spread over the batch) and every
    request for three heads;
  * the tensor-form absorb checker (pinned to the definition by the CPU tests) on EVERY output
    row (b, s, h);
  * all three modes, which must also agree with each other on every row;
  * and the same again for the peaked variant of each configuration (queries scaled by 8: logits
    of std ~5.5, outputs of size 0.1-0.4, so that a dropped tile or a mask error cannot hide in
    a near-uniform softmax).
"""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import mla_oracle as O
from paper_2509_21081_amd import workloads as W
from tests import helpers as Hh

pytestmark = pytest.mark.gpu

FULL = ["cfg2_dsv3_b64", "cfg3_long_prompt", "cfg4_mtp", "cfg5_tp_rank", "cfg5b_no_prefix"]
PEAK_GAIN = 8.0

_held = {}   # one configuration's workload at a time (cfg5's fp64 copy is 5 GB)


def _base_workload(name):
    if _held.get("name") != name:
        _held.clear()
        wl = W.make_workload(W.CONFIGS[name])
        _held.update(name=name, wl=wl)
    return _held["wl"]


def _peaked(wl):
    """The workload make_workload gives for q_gain = 8: only the queries differ, and scaling by a
    power of two commutes with their rounding (checked against the generator in the CPU tests)."""
    spec = dataclasses.replace(wl.spec, q_gain=PEAK_GAIN)
    return dataclasses.replace(wl, spec=spec, q=(wl.q.float() * PEAK_GAIN).to(wl.q.dtype))


@pytest.mark.parametrize("variant", ["as_configured", "peaked"])
@pytest.mark.parametrize("name", FULL)
def test_full_config(name, variant, gpu_device):
    wl = _base_workload(name)
    if variant == "peaked":
        wl = _peaked(wl)
    spec = wl.spec
    a = wl.as_float64()
    pairs = W.sample_pairs(wl, n_full_requests=8 if variant == "as_configured" else 4,
                           n_full_heads=2 if variant == "as_configured" else 1)
    print(f"full config {name}/{variant}: definition oracle on {len(pairs)} (b, h) pairs", flush=True)
    ref, ref_lse = Hh.oracle_definition_parallel(O, a, pairs)
    print(f"full config {name}/{variant}: absorb-form checker on every row", flush=True)
    ref2, ref2_lse = Hh.oracle_absorb_all_heads_parallel(O, a)
    assert not np.isnan(ref2_lse).any()
    # the two references agree where both exist (fp64, different formulations)
    m = ~np.isnan(ref_lse)
    np.testing.assert_allclose(ref2[m], ref[m], rtol=1e-9, atol=1e-12)
    del a
    gain = spec.q_gain
    outs = {}
    for mode in ["mixed", "absorb_only", "naive_only"]:
        print(f"full config {name}/{variant} mode={mode}", flush=True)
        got, got_lse = Hh.run_library(wl, mode, gpu_device)
        assert not np.isnan(got).any() and not np.isnan(got_lse).any()
        Hh.assert_parity(got, got_lse, ref, ref_lse, spec.dtype, f"{name}/{variant}/{mode}/definition",
                         logit_gain=gain)
        Hh.assert_parity(got, got_lse, ref2, ref2_lse, spec.dtype,
                         f"{name}/{variant}/{mode}/absorb-form", logit_gain=gain)
        outs[mode] = (got, got_lse)
        torch.cuda.empty_cache()
    # every row: the three formulations agree with each other (independent code paths)
    for mode in ["absorb_only", "naive_only"]:
        d = np.abs(outs[mode][0] - outs["mixed"][0])
        if gain <= 1:
            bound = 1e-2 + 2e-2 * np.abs(outs["mixed"][0])
            lse_bound = 4e-3
        else:   # two results, each within the peaked-row bounds of helpers.assert_parity
            bound = 2 * max(1e-2, 2.5e-3 * gain) + 4e-2 * np.abs(outs["mixed"][0])
            lse_bound = 2 * 3.2e-3 * gain
        worst = np.unravel_index(np.argmax(d - bound), d.shape)
        assert np.all(d <= bound), (f"{name}: {mode} vs mixed differ by {d[worst]:.3e} > "
                                    f"{bound[worst]:.3e} at {worst}")
        assert np.abs(outs[mode][1] - outs["mixed"][1]).max() <= lse_bound
