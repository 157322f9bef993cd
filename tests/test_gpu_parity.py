"""GPU parity: the HIP library (through its C ABI) against the fp64 oracle, element by element, on
seeded inputs small enough for the oracle yet spanning several tiles and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import mla_oracle as O
from paper_2509_21081_amd import binding as T
from paper_2509_21081_amd import workloads as W
from tests import helpers as Hh

pytestmark = pytest.mark.gpu

MODES = ["mixed", "naive_only", "absorb_only"]

# (name, kwargs for small_spec)
SMALL_CASES = {
    "ragged_h16": dict(batch=3, heads=16, q_len=1, prefix_len=100, suffix_min=0, suffix_max=150),
    "mtp_h32": dict(batch=2, heads=32, q_len=2, prefix_len=70, suffix_min=1, suffix_max=200,
                    seed=21),
    "no_prefix": dict(batch=4, heads=16, q_len=1, prefix_len=0, suffix_min=1, suffix_max=130,
                      seed=22),
    "no_suffix": dict(batch=2, heads=16, q_len=1, prefix_len=97, suffix_min=0, suffix_max=0,
                      seed=23),
    "block128_qlen3": dict(batch=2, heads=16, q_len=3, prefix_len=33, suffix_min=0, suffix_max=260,
                           block_size=128, seed=24),
    "peaked": dict(batch=2, heads=16, q_len=1, prefix_len=150, suffix_min=20, suffix_max=90,
                   seed=25, q_gain=8.0),
    "h128_many_tiles": dict(batch=5, heads=128, q_len=1, prefix_len=300, suffix_min=40,
                            suffix_max=330, seed=26),
    "batch_300": dict(batch=300, heads=16, q_len=1, prefix_len=200, suffix_min=0, suffix_max=40,
                      seed=28),
    "nothing_visible": dict(batch=6, heads=16, q_len=3, prefix_len=0, suffix_min=0, suffix_max=4,
                            seed=29),
    "one_token_prefix": dict(batch=2, heads=16, q_len=1, prefix_len=1, suffix_min=0, suffix_max=1,
                             seed=30),
    "h64_kimi_like": dict(batch=3, heads=64, q_len=1, prefix_len=160, suffix_min=10, suffix_max=140,
                          seed=31),
    "wide_batch": dict(batch=70, heads=16, q_len=1, prefix_len=130, suffix_min=0, suffix_max=70,
                       seed=27),
    # 48 query rows per request: the second 32-row query block of a workgroup is half empty
    "h48_half_block": dict(batch=3, heads=48, q_len=1, prefix_len=90, suffix_min=30,
                           suffix_max=200, seed=32),
    # 96 rows: the second workgroup of a request holds one full and one empty query block;
    # q_len = 2 puts the causal edge inside a 64-token step
    "h48_mtp_empty_block": dict(batch=3, heads=48, q_len=2, prefix_len=65, suffix_min=60,
                                suffix_max=135, seed=33),
    # suffix lengths straddling the 32/64-token tile and step boundaries, causal over 3 queries
    "h32_step_edges": dict(batch=9, heads=32, q_len=3, prefix_len=64, suffix_min=61,
                           suffix_max=69, seed=34),
    # the largest supported query length: 8 positions x 16 heads = 128 rows per request (the
    # causal edge runs through one workgroup's rows), and x 32 heads = 256 rows
    "qlen8_h16": dict(batch=3, heads=16, q_len=8, prefix_len=70, suffix_min=3, suffix_max=200,
                      seed=35),
    "qlen8_h32": dict(batch=2, heads=32, q_len=8, prefix_len=40, suffix_min=8, suffix_max=150,
                      seed=36),
    # more requests than the device-side ranking of suffix lengths handles (4096): batch order
    "batch_5000": dict(batch=5000, heads=16, q_len=1, prefix_len=64, suffix_min=0, suffix_max=20,
                       seed=37),
    # one long suffix: the per-request chunk bound is reached and chunks grow instead
    "long_suffix": dict(batch=2, heads=16, q_len=1, prefix_len=40, suffix_min=9000,
                        suffix_max=9500, seed=38),
}

_cache = {}


def _workload_and_ref(case, dtype):
    key = (case, dtype)
    if key not in _cache:
        wl = W.make_workload(W.small_spec(name=case, dtype=dtype, **SMALL_CASES[case]))
        ref = O.mla_decode_definition(**wl.as_float64())
        _cache[key] = (wl, ref)
    return _cache[key]


@pytest.mark.parametrize("flags", [0, 1], ids=["mfma", "scalar"])
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("case", list(SMALL_CASES))
def test_small_cases(case, dtype, mode, flags, gpu_device):
    if dtype == "fp32" and flags == 1:
        pytest.skip("fp32 always runs the scalar kernels")
    wl, (ref, ref_lse) = _workload_and_ref(case, dtype)
    print(f"case={case} dtype={dtype} mode={mode} flags={flags}", flush=True)
    got, got_lse = Hh.run_library(wl, mode, gpu_device, flags=flags)
    Hh.assert_parity(got, got_lse, ref, ref_lse, dtype, f"{case}/{dtype}/{mode}",
                     logit_gain=wl.spec.q_gain)


@pytest.mark.parametrize("mode", ["mixed", "absorb_only"])
@pytest.mark.parametrize("case", ["h128_many_tiles", "mtp_h32", "h48_mtp_empty_block",
                                  "ragged_h16"])
def test_forced_small_chunks(case, mode, gpu_device, tune):
    """Token chunks of one 64-token step (32 tokens for the <= 16-row kernel's wavefront shares):
    every chunk boundary, empty chunks of short requests and the merge of many latent partials."""
    tune(T.TUNE_SUFFIX_CHUNK, 64)
    tune(T.TUNE_ABSORB_PREFIX_CHUNK, 64)
    wl, (ref, ref_lse) = _workload_and_ref(case, "bf16")
    print(f"forced chunks case={case} mode={mode}", flush=True)
    got, got_lse = Hh.run_library(wl, mode, gpu_device)
    Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"{case}/chunk64/{mode}",
                     logit_gain=wl.spec.q_gain)


@pytest.mark.parametrize("flags", [0, 0x10000], ids=["merge_pass", "merge_inside"])
@pytest.mark.parametrize("mode", ["mixed", "absorb_only"])
def test_many_latent_partials_small_batch(mode, flags, gpu_device):
    """One and three requests of 128 heads over a 5000-token prefix and suffixes of up to 3000
    tokens: the plan cuts the tokens into many chunks to fill the chip (tens of latent partials per
    row, some empty for the shorter suffix), which the separate merge pass folds into one before
    the up-projection -- or, with debug flag bit 16, the projection kernel merges itself."""
    for batch, seed in ((1, 61), (3, 62)):
        spec = W.small_spec(name=f"many_partials_b{batch}", dtype="bf16", batch=batch, heads=128,
                            q_len=1, prefix_len=5000, suffix_min=700, suffix_max=3000, seed=seed)
        wl = W.make_workload(spec)
        a = wl.as_float64()
        ref2, ref2_lse = Hh.oracle_absorb_all_heads_parallel(O, a)
        pairs = [(b, h) for b in range(batch) for h in (0, 77, 127)]
        ref, ref_lse = O.mla_decode_definition(**a, pairs=pairs)
        print(f"many partials batch={batch} mode={mode} flags={flags:#x}", flush=True)
        got, got_lse = Hh.run_library(wl, mode, gpu_device, flags=flags)
        Hh.assert_parity(got, got_lse, ref2, ref2_lse, "bf16", f"many_partials/{mode}/absorb-form")
        Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"many_partials/{mode}/definition")


@pytest.mark.parametrize("flags", [0, 0x400], ids=["pipelined", "8-wave"])
@pytest.mark.parametrize("prefix_len", [31, 32, 40, 288, 1024, 1100])
def test_pipelined_prefix_kernel_long_runs(prefix_len, flags, gpu_device, tune):
    """More than 128 queries per head select the software-pipelined prefix kernel; one split
    (forced) makes a single workgroup walk the whole prefix: a partial block only, one full
    block, full + partial, one block more than the transfer look-ahead, and long runs with and
    without a partial tail.  Also with the 8-wavefront kernel, its fallback, running alone."""
    tune(T.TUNE_PREFIX_SPLITS, 1)
    spec = W.small_spec(name=f"pipe_{prefix_len}", dtype="bf16", batch=200, heads=16, q_len=1,
                        prefix_len=prefix_len, suffix_min=0, suffix_max=40, seed=41 + prefix_len)
    wl = W.make_workload(spec)
    ref, ref_lse = O.mla_decode_definition(**wl.as_float64())
    print(f"pipelined prefix, prefix_len={prefix_len} flags={flags}", flush=True)
    got, got_lse = Hh.run_library(wl, "mixed", gpu_device, flags=flags)
    Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"pipe_{prefix_len}")


@pytest.mark.parametrize("gain,first", [(256.0, 64), (256.0, 1000), (16.0, 64), (1.0 / 64.0, 64)])
def test_prefix_scores_far_from_the_first_block(gain, first, gpu_device, tune):
    """The RoPE part of the keys from token `first` on is scaled by `gain` (a power of two, and
    that part of a key is stored as given, so the oracle sees exactly what the kernels see): the
    scores there lie far above (or below) those of the first block, whose maximum the pipelined
    kernel takes as its exponent reference.  With gain 256 its denominators overflow for every
    query: it must notice, form the exact maxima in a scores-only pass and walk the prefix
    again.  The 8-wavefront kernel (moving references; debug flag 0x400) is held against the
    oracle on the same inputs."""
    tune(T.TUNE_PREFIX_SPLITS, 1)
    spec = W.small_spec(name="growth", dtype="bf16", batch=150, heads=16, q_len=1,
                        prefix_len=1100, suffix_min=0, suffix_max=30, seed=77)
    wl = W.make_workload(spec)
    wl.prefix_krope[first:] *= gain
    ref, ref_lse = O.mla_decode_definition(**wl.as_float64())
    print(f"prefix score growth, gain={gain} from token {first}", flush=True)
    got, got_lse = Hh.run_library(wl, "mixed", gpu_device)
    alone, alone_lse = Hh.run_library(wl, "mixed", gpu_device, flags=0x400)
    # only the rope part of the keys was scaled, and it is stored exactly, so nothing grows with
    # the gain; but the rows are peaked, which exposes the rounding of the top logit's noPE part
    Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"growth_{gain}_{first}", peaked=True)
    Hh.assert_parity(alone, alone_lse, ref, ref_lse, "bf16", f"growth_{gain}_{first}/8-wave",
                     peaked=True)


@pytest.mark.parametrize("gain", [256.0, 16.0, 1.0 / 64.0])
def test_suffix_scores_far_from_the_first_step(gain, gpu_device, tune):
    """The same for the absorb pass over the suffix with more than 32 query rows per request: the
    64-row kernel first walks a chunk with exponent references fixed at its first 64 tokens and
    walks it again with moving references if its denominators overflowed.  The RoPE part of every
    cached suffix row behind the first block is scaled (stored as given, so exact for the
    oracle); one chunk per request (forced), so with gain 256 every workgroup overflows and the
    result is bit-identical to the walk with moving references alone (debug flag 0x800)."""
    tune(T.TUNE_SUFFIX_CHUNK, 4096)
    spec = W.small_spec(name="suffix_growth", dtype="bf16", batch=6, heads=128, q_len=1,
                        prefix_len=40, suffix_min=200, suffix_max=700, seed=91)
    wl = W.make_workload(spec)
    wl.pool[:, :, 512:] *= gain
    for b in range(spec.batch):
        wl.pool[int(wl.block_table[b, 0]), :, 512:] /= gain     # the first 64 tokens stay
    ref, ref_lse = O.mla_decode_definition(**wl.as_float64())
    print(f"suffix score growth, gain={gain}", flush=True)
    # (the scaled rope part is stored exactly: the bounds are those of peaked rows at gain 1)
    for mode in ["mixed", "absorb_only"]:
        got, got_lse = Hh.run_library(wl, mode, gpu_device)
        alone, alone_lse = Hh.run_library(wl, mode, gpu_device, flags=0x800)
        Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"suffix_growth_{gain}/{mode}",
                         peaked=True)
        Hh.assert_parity(alone, alone_lse, ref, ref_lse, "bf16",
                         f"suffix_growth_{gain}/{mode}/moving", peaked=True)
        if gain >= 256.0 and mode == "mixed":
            assert np.array_equal(got, alone) and np.array_equal(got_lse, alone_lse)


# requests with whole blocks of 128 query rows: (name, kwargs for small_spec)
ROWS128_CASES = {
    "h128": dict(batch=5, heads=128, q_len=1, prefix_len=300, suffix_min=40, suffix_max=330,
                 seed=26),
    # 256 rows = two workgroups per request; the causal edge runs through the rows
    "h128_mtp": dict(batch=3, heads=128, q_len=2, prefix_len=70, suffix_min=1, suffix_max=200,
                     seed=41),
    # two query positions inside one workgroup's 128 rows, long enough for an odd number of steps
    "h64_qlen2": dict(batch=4, heads=64, q_len=2, prefix_len=130, suffix_min=60, suffix_max=450,
                      seed=42),
    "h128_block128": dict(batch=2, heads=128, q_len=1, prefix_len=33, suffix_min=0,
                          suffix_max=260, block_size=128, seed=43),
}


@pytest.mark.parametrize("chunk", [0, 64], ids=["auto_chunks", "chunk64"])
@pytest.mark.parametrize("mode", ["mixed", "absorb_only"])
@pytest.mark.parametrize("case", list(ROWS128_CASES))
def test_absorb_kernel_with_128_rows_per_workgroup(case, mode, chunk, gpu_device, tune):
    """The absorb kernel that gives a workgroup 128 query rows is chosen only for grids that cover
    the chip; debug flag 0x2000 takes it at any size.  Parity with the oracle, and agreement with
    the 64-row kernel (flag 0x1000) to the same tolerance."""
    if chunk:
        tune(T.TUNE_SUFFIX_CHUNK, chunk)
        tune(T.TUNE_ABSORB_PREFIX_CHUNK, chunk)
    wl = W.make_workload(W.small_spec(name=case, dtype="bf16", **ROWS128_CASES[case]))
    ref, ref_lse = O.mla_decode_definition(**wl.as_float64())
    print(f"128-row absorb kernel case={case} mode={mode} chunk={chunk}", flush=True)
    got, got_lse = Hh.run_library(wl, mode, gpu_device, flags=0x2000)
    Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"{case}/rows128/{mode}")
    other, other_lse = Hh.run_library(wl, mode, gpu_device, flags=0x1000)
    Hh.assert_parity(other, other_lse, ref, ref_lse, "bf16", f"{case}/rows64/{mode}")


ORDER_CASES = {
    # one per absorb kernel: <= 16, <= 32, 64 and 128 query rows per workgroup
    "h16": (dict(batch=9, heads=16, q_len=1, prefix_len=70, suffix_min=0, suffix_max=300,
                 seed=61), 0),
    "h32": (dict(batch=7, heads=32, q_len=1, prefix_len=40, suffix_min=1, suffix_max=200,
                 seed=62), 0),
    "h64_sq2": (dict(batch=6, heads=64, q_len=2, prefix_len=33, suffix_min=2, suffix_max=260,
                     seed=63), 0x1000),
    "h128": (dict(batch=5, heads=128, q_len=1, prefix_len=64, suffix_min=0, suffix_max=200,
                  seed=64), 0x2000),
}


@pytest.mark.parametrize("mode", ["mixed", "absorb_only"])
@pytest.mark.parametrize("case", list(ORDER_CASES))
def test_longest_suffix_first_order_changes_nothing(case, mode, gpu_device):
    """Grids with more workgroups than compute units start the requests with the longest suffix
    first (a small kernel ranks them); debug flag 0x4000 does so at any grid size, 0x8000 never.
    A request's result does not depend on when its workgroups run: parity with the oracle, and
    bit-identical to the run in batch order."""
    kw, kernel_flag = ORDER_CASES[case]
    wl = W.make_workload(W.small_spec(name="order_" + case, dtype="bf16", **kw))
    assert len(set(int(x) for x in wl.suffix_lens)) > 2     # ragged, with ties possible
    ref, ref_lse = O.mla_decode_definition(**wl.as_float64())
    print(f"longest-first order case={case} mode={mode}", flush=True)
    got, got_lse = Hh.run_library(wl, mode, gpu_device, flags=0x4000 | kernel_flag)
    Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"{case}/ordered/{mode}")
    plain, plain_lse = Hh.run_library(wl, mode, gpu_device, flags=0x8000 | kernel_flag)
    assert np.array_equal(got, plain, equal_nan=True)
    assert np.array_equal(got_lse, plain_lse, equal_nan=True)


@pytest.mark.parametrize("gain", [256.0, 16.0, 1.0 / 64.0])
def test_suffix_scores_far_from_the_first_step_128_rows(gain, gpu_device, tune):
    """test_suffix_scores_far_from_the_first_step for the 128-row absorb kernel, whose second
    walk takes exact maxima from a scores-only pass."""
    tune(T.TUNE_SUFFIX_CHUNK, 4096)
    spec = W.small_spec(name="suffix_growth_128", dtype="bf16", batch=4, heads=128, q_len=2,
                        prefix_len=40, suffix_min=200, suffix_max=700, seed=92)
    wl = W.make_workload(spec)
    wl.pool[:, :, 512:] *= gain
    for b in range(spec.batch):
        wl.pool[int(wl.block_table[b, 0]), :, 512:] /= gain     # the first 64 tokens stay
    ref, ref_lse = O.mla_decode_definition(**wl.as_float64())
    print(f"suffix score growth, 128-row kernel, gain={gain}", flush=True)
    for mode in ["mixed", "absorb_only"]:
        got, got_lse = Hh.run_library(wl, mode, gpu_device, flags=0x2000)
        Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"suffix_growth_128_{gain}/{mode}",
                         peaked=True)


@pytest.mark.parametrize("flags", [0, 1], ids=["mfma", "scalar"])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("ntok", [1, 31, 64, 100, 300])
def test_expand_prefix_matches_definition(dtype, ntok, flags, gpu_device):
    if dtype == "fp32" and flags == 1:
        pytest.skip("fp32 always runs the scalar kernels")
    wl = W.make_workload(W.small_spec(dtype=dtype, batch=1, heads=16, prefix_len=ntok,
                                      suffix_min=1, suffix_max=1, seed=40 + ntok))
    a = wl.as_float64()
    k_ref, v_ref = O.expand_prefix_definition(a["prefix_ckv"], a["prefix_krope"], a["w_uk"],
                                              a["w_uv"])
    d = wl.to(gpu_device)
    dims = Hh.dims_of(wl)
    print(f"expand dtype={dtype} ntok={ntok} flags={flags}", flush=True)
    old = T.typhoon_mla_set_debug_flags(flags)
    try:
        pk, pv = T.typhoon_mla_expand_prefix(dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv)
        torch.cuda.synchronize()
    finally:
        T.typhoon_mla_set_debug_flags(old)
    K, V = Hh.unpack_expanded(pk, pv, 16, ntok, dtype)
    rt = 2.0 ** -8 if dtype == "bf16" else 1e-5      # one bf16 rounding of an fp32 accumulation
    np.testing.assert_allclose(K, k_ref, rtol=rt, atol=1e-3 if dtype == "bf16" else 1e-6)
    np.testing.assert_allclose(V, v_ref, rtol=rt, atol=1e-3 if dtype == "bf16" else 1e-6)
    # the rope part is a verbatim copy
    np.testing.assert_array_equal(K[:, :, 128:], np.broadcast_to(a["prefix_krope"], (16, ntok, 64)))
    if dtype == "bf16" and ntok % 32:
        # padding tokens of the last 32-token block are zero
        kraw = pk.view(torch.bfloat16).double().cpu().numpy()
        hh, dd = np.meshgrid(np.arange(16), np.arange(192), indexing="ij")
        ntb32 = (ntok + 31) // 32 * 32
        for t in range(ntok, ntb32):
            assert np.all(kraw[Hh.k_offset(hh, ntb32, t, dd, dtype)] == 0)


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,rows,width", [(1, 5, 128), (3, 130, 128), (7, 33, 512), (2, 1, 4)])
def test_combine_lse_matches_definition(n, rows, width, out_dtype, gpu_device):
    g = torch.Generator().manual_seed(n * 1000 + rows)
    po = torch.randn((n, rows, width), generator=g)
    pl = torch.randn((n, rows), generator=g) * 4
    # sprinkle empty partials (LSE = -inf with NaN payload) and one fully empty row
    pl[0, ::3] = float("-inf")
    po[0, ::3] = float("nan")
    if rows > 1:
        pl[:, 1] = float("-inf")
    ref_o, ref_l = O.combine_lse(po.double().numpy(), pl.double().numpy())
    print(f"combine n={n} rows={rows} width={width} {out_dtype}", flush=True)
    out, lse = T.typhoon_mla_combine_lse(po.to(gpu_device), pl.to(gpu_device), out_dtype)
    torch.cuda.synchronize()
    tol = 1e-5 if out_dtype == torch.float32 else 2.0 ** -8
    np.testing.assert_allclose(out.double().cpu().numpy(), ref_o, rtol=tol, atol=1e-6)
    got_l = lse.double().cpu().numpy()
    assert np.array_equal(np.isneginf(got_l), np.isneginf(ref_l))
    fin = np.isfinite(ref_l)
    np.testing.assert_allclose(got_l[fin], ref_l[fin], atol=1e-5, rtol=1e-6)


@pytest.mark.parametrize("mode", ["mixed", "absorb_only"])
def test_large_batch_projection_kernels(mode, gpu_device):
    """More than 1024 queries per head at 64 heads: the query absorption stages a weight slice once
    for four blocks of 128 queries, and the up-projection streams runs of eight blocks of 32
    through its LDS ring (three slots, one naive partial) -- both with a ragged last group
    (1100 = 8 x 128 + 76 = 34 x 32 + 12 queries: runs of 8, 8, 8, 8 and 3 blocks).  Every row
    against the tensor-form absorb checker, a sample against the definition."""
    spec = W.small_spec(name="large_batch_h64", dtype="bf16", batch=1100, heads=64, q_len=1,
                        prefix_len=64, suffix_min=0, suffix_max=24, seed=55)
    wl = W.make_workload(spec)
    a = wl.as_float64()
    ref2, ref2_lse = Hh.oracle_absorb_all_heads_parallel(O, a)
    pairs = [(b, h) for b in (0, 1, 511, 1023, 1024, 1099) for h in (0, 31, 63)]
    ref, ref_lse = O.mla_decode_definition(**a, pairs=pairs)
    print(f"large batch projections mode={mode}", flush=True)
    got, got_lse = Hh.run_library(wl, mode, gpu_device)
    Hh.assert_parity(got, got_lse, ref2, ref2_lse, "bf16", f"large_batch/{mode}/absorb-form")
    Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"large_batch/{mode}/definition")


def test_streaming_upprojection_two_naive_partials(gpu_device):
    """200 requests x 128 heads: the prefix pass splits its tokens in two (two naive partials per
    row), and the up-projection takes runs of 3, 3 and 1 blocks of 32 queries through its
    two-slot ring, the last block with 8 valid rows.  Some requests have no suffix at all (their
    latent partial is never written and must count as zeros)."""
    spec = W.small_spec(name="two_naive_partials_h128", dtype="bf16", batch=200, heads=128, q_len=1,
                        prefix_len=160, suffix_min=0, suffix_max=20, seed=77)
    wl = W.make_workload(spec)
    a = wl.as_float64()
    ref2, ref2_lse = Hh.oracle_absorb_all_heads_parallel(O, a)
    pairs = [(b, h) for b in (0, 95, 96, 191, 192, 199) for h in (0, 64, 127)]
    ref, ref_lse = O.mla_decode_definition(**a, pairs=pairs)
    print("streaming up-projection, two naive partials", flush=True)
    got, got_lse = Hh.run_library(wl, "mixed", gpu_device)
    Hh.assert_parity(got, got_lse, ref2, ref2_lse, "bf16", "two_naive/absorb-form")
    Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", "two_naive/definition")


@pytest.mark.parametrize("mode", MODES)
def test_bitwise_repeatable(mode, gpu_device):
    wl, _ = _workload_and_ref("ragged_h16", "bf16")
    a = Hh.run_library(wl, mode, gpu_device)
    b = Hh.run_library(wl, mode, gpu_device)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.parametrize("mode", MODES)
def test_cfg1_tiny_fp32_full(mode, gpu_device):
    wl = W.make_workload(W.CONFIGS["cfg1_tiny_fp32"])
    ref, ref_lse = O.mla_decode_definition(**wl.as_float64())
    print(f"cfg1 mode={mode}", flush=True)
    got, got_lse = Hh.run_library(wl, mode, gpu_device)
    Hh.assert_parity(got, got_lse, ref, ref_lse, "fp32", f"cfg1/{mode}")


def test_modes_agree_with_each_other(gpu_device):
    wl, _ = _workload_and_ref("mtp_h32", "bf16")
    outs = {m: Hh.run_library(wl, m, gpu_device) for m in MODES}
    for m in MODES[1:]:
        np.testing.assert_allclose(outs[m][0], outs["mixed"][0], atol=1e-2, rtol=2e-2)
        fin = np.isfinite(outs["mixed"][1])
        np.testing.assert_allclose(outs[m][1][fin], outs["mixed"][1][fin], atol=2e-3)


AUTO_CASES = {
    # below the break-even batch of 128 heads and a 2048-token prefix (56): absorb_only runs
    "below_break_even": dict(batch=2, heads=128, q_len=1, prefix_len=2048, suffix_min=10,
                             suffix_max=120, seed=51),
    # above that of 32 heads (32): mixed runs
    "above_break_even": dict(batch=40, heads=32, q_len=1, prefix_len=2048, suffix_min=0,
                             suffix_max=60, seed=52),
    # two query positions per request halve it (16)
    "above_with_two_queries": dict(batch=20, heads=32, q_len=2, prefix_len=2048, suffix_min=2,
                                   suffix_max=60, seed=53),
}


@pytest.mark.parametrize("case", list(AUTO_CASES))
def test_auto_mode_matches_oracle(case, gpu_device):
    wl = W.make_workload(W.small_spec(name=case, dtype="bf16", **AUTO_CASES[case]))
    spec = wl.spec
    thr = T.typhoon_mla_auto_batch_threshold(Hh.dims_of(wl), spec.q_len, spec.prefix_len)
    assert (spec.batch < thr) == (case == "below_break_even")
    ref, ref_lse = O.mla_decode_definition(**wl.as_float64())
    print(f"auto mode case={case} threshold={thr:.2f}", flush=True)
    got, got_lse = Hh.run_library(wl, "auto", gpu_device)
    Hh.assert_parity(got, got_lse, ref, ref_lse, "bf16", f"{case}/auto")
    # auto is exactly the mode it resolves to
    same, same_lse = Hh.run_library(wl, "absorb_only" if spec.batch < thr else "mixed", gpu_device)
    assert np.array_equal(got, same) and np.array_equal(got_lse, same_lse)


@pytest.mark.parametrize("case,flags", [("h128_many_tiles", 0), ("ragged_h16", 0),
                                        ("h128_many_tiles", 0x2000)],
                         ids=["h128", "h16", "h128_rows128"])
def test_decode_replays_from_a_hip_graph(case, flags, gpu_device):
    """The library only enqueues kernels on the caller's stream (no allocation, no host
    synchronisation, no memset nodes), so a decode step can be captured into a HIP graph.  Every
    replay, with eager work and synchronisations in between, must reproduce the eager result bit
    for bit, also after the inputs have changed in place."""
    wl, (ref, ref_lse) = _workload_and_ref(case, "bf16")
    d = wl.to(gpu_device)
    dims = Hh.dims_of(wl)
    L_s = wl.spec.prefix_len
    pk, pv = T.typhoon_mla_expand_prefix(dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv)
    B, S, H = wl.spec.batch, wl.spec.q_len, wl.spec.heads
    out = torch.empty((B, S, H, 128), dtype=torch.bfloat16, device=gpu_device)
    lse = torch.empty((B, S, H), dtype=torch.float32, device=gpu_device)
    nbytes = T.typhoon_mla_decode_workspace_bytes(dims, T.MODE_MIXED, B, S, L_s, wl.max_suffix_len)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=gpu_device)
    q = d.q.clone()

    def step():
        T.typhoon_mla_decode(dims, "mixed", q, L_s, prefix_k=pk, prefix_v=pv,
                             suffix_pool=d.pool, block_table=d.block_table,
                             suffix_lens=d.suffix_lens, max_suffix_len=wl.max_suffix_len,
                             w_uk=d.w_uk, w_uv=d.w_uv, out=out, lse_out=lse, workspace=ws)

    print(f"graph capture case={case} flags={flags:#x}", flush=True)
    old_flags = T.typhoon_mla_set_debug_flags(flags)   # 0x2000: the 128-row absorb kernel
    try:
        step()                                   # eager: also performs the one-time kernel set-up
        torch.cuda.synchronize(gpu_device)
        eager = (out.clone(), lse.clone())
        Hh.assert_parity(out.double().cpu().numpy(), lse.double().cpu().numpy(), ref, ref_lse, "bf16",
                         f"{case}/eager")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for rep in range(3):
            out.fill_(float("nan"))              # eager work between replays
            lse.fill_(float("nan"))
            torch.cuda.synchronize(gpu_device)
            graph.replay()
            torch.cuda.synchronize(gpu_device)
            assert torch.equal(out, eager[0]) and torch.equal(lse, eager[1]), f"replay {rep} differs"
        # new queries written in place are picked up by the next replay
        q.copy_(torch.flip(d.q, dims=[0]))
        graph.replay()
        torch.cuda.synchronize(gpu_device)
        flipped = (out.clone(), lse.clone())
        step()
        torch.cuda.synchronize(gpu_device)
        assert torch.equal(out, flipped[0]) and torch.equal(lse, flipped[1])
    finally:
        T.typhoon_mla_set_debug_flags(old_flags)
