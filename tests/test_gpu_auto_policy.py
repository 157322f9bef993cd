"""TMLA_MODE_AUTO against the two fixed modes it chooses between (Section 3.1 "Fall-back to
Absorb", Section 3.2 break-even batch): on a grid of head counts, prefix lengths and batch sizes
around the measured cross-overs, the step time of auto stays close to the faster of mixed and
absorb_only.  Step times are medians of interleaved rounds (the clock moves with what ran just
before); the bound leaves room for that noise -- at a cross-over the two modes are equally fast
by definition, so a wrong choice there costs little, and away from it the choice is clear."""
import pytest
import torch

from paper_2509_21081_amd import binding as T
from paper_2509_21081_amd import workloads as W

pytestmark = pytest.mark.gpu

GRID = [(H, Ls, B) for H in (16, 64, 128) for Ls in (1024, 4096, 16384, 65536)
        for B in (1, 8, 32, 128)]


def _median_times(step, modes, rounds=5, steps=10):
    times = {m: [] for m in modes}
    for _ in range(rounds):
        for m in modes:
            step(m)
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                step(m)
            e1.record()
            e1.synchronize()
            times[m].append(e0.elapsed_time(e1) / steps)
    return {m: sorted(v)[len(v) // 2] for m, v in times.items()}


@pytest.mark.parametrize("H,Ls,B", GRID)
def test_auto_is_close_to_the_faster_fixed_mode(H, Ls, B, gpu_device):
    spec = W.WorkloadSpec(f"auto_{H}_{Ls}_{B}", "bf16", B, H, 1, Ls, 512, 512, seed=5)
    d = W.make_workload(spec, poison=False).to(gpu_device)
    dims = T.make_dims(H, 1.0 / 192 ** 0.5, "bf16")
    pk, pv = T.typhoon_mla_expand_prefix(dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv)
    out = torch.empty((B, 1, H, 128), dtype=torch.bfloat16, device=gpu_device)
    ws = {m: torch.empty(max(256, T.typhoon_mla_decode_workspace_bytes(dims, T.MODES[m], B, 1, Ls, 512)),
                         dtype=torch.uint8, device=gpu_device)
          for m in ("mixed", "absorb_only", "auto")}

    def step(mode):
        T.typhoon_mla_decode(dims, mode, d.q, Ls, prefix_k=pk, prefix_v=pv, prefix_ckv=d.prefix_ckv,
                             prefix_krope=d.prefix_krope, suffix_pool=d.pool,
                             block_table=d.block_table, suffix_lens=d.suffix_lens,
                             max_suffix_len=512, w_uk=d.w_uk, w_uv=d.w_uv, out=out, want_lse=False,
                             workspace=ws[mode])
    print(f"auto policy H={H} Ls={Ls} B={B}", flush=True)
    t = _median_times(step, ("mixed", "absorb_only", "auto"))
    best = min(t["mixed"], t["absorb_only"])
    thr = T.typhoon_mla_auto_batch_threshold(dims, 1, Ls)
    chosen = "mixed" if B >= thr else "absorb_only"
    print(f"  mixed {t['mixed'] * 1e3:.0f} us, absorb_only {t['absorb_only'] * 1e3:.0f} us, "
          f"auto {t['auto'] * 1e3:.0f} us, threshold {thr:.1f} -> {chosen}", flush=True)
    # The policy is judged by the fixed mode it resolves to (auto launches exactly that mode's
    # kernels -- the parity tests check the outputs are bit-identical -- and a second timing of the
    # same kernels differs by whatever ran in between: these steps are power-limited, a heavy
    # absorb_only round in front costs the next one up to 10 %).
    assert t[chosen] <= 1.08 * best, (
        f"auto resolves to {chosen}: {t[chosen] * 1e3:.0f} us, the faster fixed mode "
        f"{best * 1e3:.0f} us")
    assert t["auto"] <= 1.25 * t[chosen]
