"""The decode entry point that allocates nothing (static device scratch inside the library):
called through the C ABI twice in a row, the second time with a smaller input, and compared with
typhoon_mla_decode on a caller workspace -- same kernels, no atomics, so bit for bit -- and with
the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import mla_oracle as O
from paper_2509_21081_amd import binding as T
from paper_2509_21081_amd import workloads as W
from tests import helpers as Hh

pytestmark = pytest.mark.gpu

CALLS = [   # first a larger input, then a smaller one
    dict(batch=70, heads=128, q_len=1, prefix_len=300, suffix_min=40, suffix_max=330, seed=71),
    dict(batch=3, heads=16, q_len=2, prefix_len=100, suffix_min=0, suffix_max=150, seed=72),
]


def _run_both(wl, mode, dev):
    d = wl.to(dev)
    dims = Hh.dims_of(wl)
    spec = wl.spec
    pk, pv = T.typhoon_mla_expand_prefix(dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv)
    kw = dict(prefix_k=pk, prefix_v=pv, prefix_ckv=d.prefix_ckv, prefix_krope=d.prefix_krope,
              suffix_pool=d.pool, block_table=d.block_table, suffix_lens=d.suffix_lens,
              max_suffix_len=wl.max_suffix_len, w_uk=d.w_uk, w_uv=d.w_uv)
    shape = (spec.batch, spec.q_len, spec.heads)
    out = torch.full(shape + (128,), float("nan"), dtype=torch.bfloat16, device=dev)
    lse = torch.full(shape, float("nan"), dtype=torch.float32, device=dev)
    T.typhoon_mla_decode_static_scratch(dims, mode, d.q, spec.prefix_len, out, lse, **kw)
    ref_out, ref_lse = T.typhoon_mla_decode(dims, mode, d.q, spec.prefix_len, **kw)
    torch.cuda.synchronize(dev)
    return out, lse, ref_out, ref_lse


@pytest.mark.parametrize("mode", ["mixed", "absorb_only"])
def test_static_scratch_decode_matches_workspace_decode(mode, gpu_device):
    for i, kw in enumerate(CALLS):
        wl = W.make_workload(W.small_spec(name=f"static_scratch_{i}", dtype="bf16", **kw))
        print(f"static scratch call {i} mode={mode} {kw}", flush=True)
        out, lse, ref_out, ref_lse = _run_both(wl, mode, gpu_device)
        assert torch.equal(out, ref_out), f"call {i}: outputs differ from typhoon_mla_decode"
        assert torch.equal(lse, ref_lse), f"call {i}: LSEs differ from typhoon_mla_decode"
        want, want_lse = O.mla_decode_definition(**wl.as_float64())
        Hh.assert_parity(out.double().cpu().numpy(), lse.double().cpu().numpy(), want, want_lse,
                         "bf16", f"static scratch call {i}/{mode}")


def test_static_scratch_decode_rejects_what_does_not_fit(gpu_device):
    """Beyond the static array's size the call fails before anything is launched (the same check
    runs without a GPU in the host tests)."""
    dims = T.make_dims(128, 0.07, "bf16")
    need = T.typhoon_mla_decode_workspace_bytes(dims, T.MODE_MIXED, 2048, 1, 4096, 4096)
    assert need > T.STATIC_SCRATCH_BYTES
    q = torch.zeros((2048, 1, 128, 192), dtype=torch.bfloat16, device=gpu_device)
    out = torch.empty((2048, 1, 128, 128), dtype=torch.bfloat16, device=gpu_device)
    one = torch.zeros(4096, dtype=torch.bfloat16, device=gpu_device)
    lens = torch.zeros(2048, dtype=torch.int32, device=gpu_device)
    bt = torch.zeros((2048, 64), dtype=torch.int32, device=gpu_device)
    pool = torch.zeros((4, 64, 576), dtype=torch.bfloat16, device=gpu_device)
    with pytest.raises(T.TyphoonMLAError) as e:
        T.typhoon_mla_decode_static_scratch(dims, "mixed", q, 4096, out, None, prefix_k=one,
                                            prefix_v=one, suffix_pool=pool, block_table=bt,
                                            suffix_lens=lens, max_suffix_len=4096, w_uk=one,
                                            w_uv=one)
    assert e.value.status == T.TMLA_ERR_SCRATCH_LIMIT
