#!/usr/bin/env python3
"""Benchmark of the TyphoonMLA decode hot path on one MI355X.

A "step" is one pass of the whole hot path -- typhoon_mla_decode in mixed mode: naive prefix
attention, query absorption, absorb suffix attention, up-projection and LSE combine -- over one
batch of seeded synthetic input already resident in HBM.  The one-off prefix expansion is timed
separately.  Prints ONE JSON line: metric, value (tokens/s over the whole batch), ms_per_step,
config.workload, per-kernel times, `roofline` for the dominant kernel, `cpu_baseline` (the fp64
oracle timed on the host cores) and, under `all_configs`, the same measurements (all three modes,
speed-ups, cold-cache time, per-kernel times and roofline fractions, parity on an oracle sample)
for every benchmark configuration.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3_long_prompt]
                  [--configs all|headline|name,name,...] [--modes mixed,absorb_only,naive_only]
                  [--no-cpu-baseline] [--no-stages]
  python bench.py --sweep      batch-size sweep at L_s = 4096, L_n = 512 for 128 and 64 heads
                               (one JSON line per point, then a table)
  --workload also takes an ad-hoc shape "B=128,H=64,Ls=4096,Ln=512[,Lmax=..][,Sq=1][,seed=7]"
  or "tree:B=64,H=128,L0=4096,G=4,L1=1024,Ln=512" (tree-shaped shared prefixes).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # B/s, MI355X published
MFMA_BF16_PEAK = 2.5e15    # FLOP/s dense bf16, MI355X published

# single-stage masks of typhoon_mla_set_debug_flags, in the order the library launches the stages
STAGES = [("prefix_attention", 0x10), ("query_absorb", 0x40), ("absorb_attention", 0x80),
          ("upproj_combine", 0x100)]
HEADLINE = "cfg3_long_prompt"
BENCH_CONFIGS = ["cfg2_dsv3_b64", "cfg3_long_prompt", "cfg4_mtp", "cfg5_tp_rank", "cfg5b_no_prefix"]
DATA = "synthetic (seeded N(0,1) latents and queries, N(0,0.02) up-projections)"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--configs", default="all",
                    help="which other benchmark configurations are measured beside the workload: "
                         "all, headline (none), or a comma-separated list")
    ap.add_argument("--modes", default="mixed,absorb_only,naive_only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stages", action="store_true")
    ap.add_argument("--sweep", action="store_true")
    ap.add_argument("--sweep-heads", default="128,64")
    ap.add_argument("--sweep-batches", default="1,2,4,8,16,32,64,128,256,512,1024")
    ap.add_argument("--sweep-prefix", type=int, default=4096)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for HBM counters)")
    ap.add_argument("--cpu-sample-requests", type=int, default=0,
                    help="requests (all heads each) in the oracle sample; 0 = auto")
    return ap.parse_args()


def host_workers():
    """Threads for the CPU legs: the cores this process may run on, at most 16 (a one-GPU machine's
    share whatever the machine shows)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def time_steps(fn, steps, warmup, torch):
    """Wall-clock ms per call over `steps` calls, synchronised on both sides."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def event_time(fn, steps, warmup, torch):
    """Average device time per call (HIP events on the stream the kernels run on)."""
    for _ in range(warmup):
        fn()
    stream = torch.cuda.current_stream()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(steps):
        fn()
    e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) / steps


def cold_time(fn, iters, torch, dev):
    """Average device time per call when every call starts with cold caches: a 512 MiB fill (twice
    the 256 MB last-level cache) runs before each call, outside the event pair that times it."""
    flush = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    pairs = []
    for i in range(iters):
        flush.fill_(i & 0xFF)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn()
        e1.record(stream)
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    del flush
    return sum(a.elapsed_time(b) for a, b in pairs) / iters


def stage_times_in_step(step_mixed, T, torch, samples, L_s, lead_in=2):
    """Device time of each kernel stage INSIDE a running sequence of steps.  A sample is a few
    untimed full steps (`lead_in`: they keep the stream busy while the host queues what follows
    -- about a millisecond's worth, so that no stage waits for the host -- and leave the caches
    as a step finds them in steady state) and then the four stages of one more step, launched
    one by one through the library's single-stage switch, in the library's own order, each
    between its own pair of HIP events on the launch stream."""
    stream = torch.cuda.current_stream()
    stages = [(n, bit) for n, bit in STAGES if not (n == "prefix_attention" and L_s == 0)]
    acc = {n: 0.0 for n, _ in stages}
    for _ in range(samples):
        for _ in range(lead_in):
            step_mixed()
        evs = []
        try:
            for name, bit in stages:
                T.typhoon_mla_set_debug_flags(bit)
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                step_mixed()
                e1.record(stream)
                evs.append((name, e0, e1))
        finally:
            T.typhoon_mla_set_debug_flags(0)
        torch.cuda.synchronize()
        for name, e0, e1 in evs:
            acc[name] += e0.elapsed_time(e1)
    return {n: v / samples for n, v in acc.items()}


def read_traffic(workload, kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc and stored in profiles/hbm_traffic.txt
    (NOT measured by this run), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 3 and f[0] == workload and f[1] == kernel:
            try:
                return float(f[2])
            except ValueError:
                return None
    return None


def spec_of(name, W):
    if name in W.CONFIGS:
        return W.CONFIGS[name]
    # ad-hoc shape: "B=128,H=64,Ls=4096,Ln=512[,Lmax=..][,Sq=1][,seed=7]" (bf16, 64-token blocks)
    kv = dict(item.split("=") for item in name.split(","))
    ln = int(kv.get("Ln", 512))
    return W.WorkloadSpec(name, "bf16", int(kv["B"]), int(kv.get("H", 128)), int(kv.get("Sq", 1)),
                          int(kv.get("Ls", 4096)), ln, int(kv.get("Lmax", ln)),
                          seed=int(kv.get("seed", 7)))


class Case:
    """One workload resident on the GPU, with everything a decode call needs."""

    def __init__(self, spec, modes, torch, T, C, W, dev):
        self.spec, self.torch, self.T = spec, torch, T
        t0 = time.perf_counter()
        self.wl = W.make_workload(spec, poison=True)
        self.gen_s = time.perf_counter() - t0
        self.d = d = self.wl.to(dev)
        self.dims = T.make_dims(spec.heads, self.wl.sm_scale, spec.dtype)
        B, S, H, L_s = spec.batch, spec.q_len, spec.heads, spec.prefix_len
        self.sum_ln = int(self.wl.suffix_lens.sum())
        self.shape = C.Shape(B, S, H, L_s, self.sum_ln, 2 if spec.dtype == "bf16" else 4)
        self.modes = modes
        # one-off prefix expansion (prefill-time cost, Section 3.1), timed separately
        self.pk = self.pv = None
        self.expand_ms = None
        if L_s > 0:
            self.pk, self.pv = T.typhoon_mla_expand_prefix(self.dims, d.prefix_ckv, d.prefix_krope,
                                                           d.w_uk, d.w_uv)
            self.expand_ms = event_time(lambda: T.typhoon_mla_expand_prefix(
                self.dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv, self.pk, self.pv), 3, 1,
                torch)
        self.sk = self.sv = None
        if "naive_only" in modes:
            self.sk, self.sv = T.typhoon_mla_expand_pool(self.dims, d.pool, d.w_uk, d.w_uv)
        self.out = torch.empty((B, S, H, 128), dtype=d.q.dtype, device=dev)
        self.lse = torch.empty((B, S, H), dtype=torch.float32, device=dev)
        self.ws = {}
        for m in modes:
            nbytes = T.typhoon_mla_decode_workspace_bytes(self.dims, T.MODES[m], B, S, L_s,
                                                          self.wl.max_suffix_len)
            self.ws[m] = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)

    def step(self, mode):
        d = self.d
        self.T.typhoon_mla_decode(
            self.dims, mode, d.q, self.spec.prefix_len, prefix_k=self.pk, prefix_v=self.pv,
            prefix_ckv=d.prefix_ckv, prefix_krope=d.prefix_krope, suffix_pool=d.pool,
            block_table=d.block_table, suffix_lens=d.suffix_lens,
            max_suffix_len=self.wl.max_suffix_len, suffix_k_pool=self.sk, suffix_v_pool=self.sv,
            w_uk=d.w_uk, w_uv=d.w_uv, out=self.out, lse_out=self.lse, workspace=self.ws[mode])

    def config(self):
        s = self.spec
        return {"workload": s.name, "batch": s.batch, "q_len": s.q_len, "heads": s.heads,
                "prefix_len": s.prefix_len, "suffix_tokens_total": self.sum_ln,
                "suffix_len_range": [s.suffix_min, s.suffix_max], "block_size": s.block_size,
                "seed": s.seed}


def kernel_rooflines(case, stage_ms, C):
    """Every attention kernel against both ceilings, and the dominant stage's `roofline` object."""
    shape, L_s = case.shape, case.spec.prefix_len
    work = {"prefix_attention": C.prefix_kernel_work(shape, 1) if L_s else None,
            "absorb_attention": C.suffix_kernel_work(shape, 0)}
    per_kernel = {}
    for name, w in work.items():
        if w is None or name not in stage_ms:
            continue
        t = stage_ms[name] * 1e-3
        per_kernel[name] = {"ms": stage_ms[name], "GB/s": w["bytes"] / t / 1e9,
                            "hbm_frac": w["bytes"] / t / HBM_PEAK,
                            "TFLOP/s": w["flops"] / t / 1e12,
                            "mfma_frac": w["flops"] / t / MFMA_BF16_PEAK}
    roofline = None
    if stage_ms:
        dom = max(stage_ms, key=stage_ms.get)
        w = work.get(dom)
        if w is not None:
            t = stage_ms[dom] * 1e-3
            if w["flops"] / w["bytes"] < MFMA_BF16_PEAK / HBM_PEAK:
                roofline = {"kernel": dom, "bound": "hbm", "achieved": w["bytes"] / t / 1e9,
                            "peak": HBM_PEAK / 1e9, "unit": "GB/s"}
            else:
                roofline = {"kernel": dom, "bound": "mfma", "achieved": w["flops"] / t / 1e12,
                            "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s"}
            roofline["frac"] = roofline["achieved"] / roofline["peak"]
            roofline["traffic"] = read_traffic(case.spec.name, dom)
            roofline["traffic_source"] = ("profiles/hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / "
                                          "WRITE_SIZE runs of this workload, not this run)"
                                          if roofline["traffic"] is not None else None)
            roofline["algorithmic_bytes"] = w["bytes"]
            if "bytes_table1" in w:      # the paper's Table 1 accounting of the same pass
                roofline["algorithmic_bytes_table1"] = w["bytes_table1"]
            roofline["algorithmic_flops"] = w["flops"]
            roofline["kernel_ms"] = stage_ms[dom]
            roofline["mfma_frac"] = w["flops"] / t / MFMA_BF16_PEAK
            roofline["hbm_frac"] = w["bytes"] / t / HBM_PEAK
    return per_kernel, roofline


def measure(case, steps, warmup, args, torch, T, C, dev):
    """Times one workload: mixed (the timed region proper), the other modes, the cold-cache step
    and the per-kernel stages.  Returns the measurements and the mixed-mode outputs."""
    ms = {"mixed": time_steps(lambda: case.step("mixed"), steps, warmup, torch)}
    got = case.out.double().cpu().numpy()
    got_lse = case.lse.double().cpu().numpy()
    for m in case.modes:
        if m != "mixed":
            ms[m] = time_steps(lambda: case.step(m), max(3, steps // 5), max(1, warmup // 5), torch)
    # the same step with the caches flushed before every call (the timed region above runs the
    # steps back to back, so whatever fits the last-level cache -- weights, queries, partials,
    # a short prefix -- stays there between steps: `value` is a cache-warm number)
    ms_cold = cold_time(lambda: case.step("mixed"), 10, torch, dev)
    stage_ms = {}
    if not args.no_stages and case.spec.dtype == "bf16":
        stage_ms = stage_times_in_step(lambda: case.step("mixed"), T, torch,
                                       max(5, min(20, steps // 2)), case.spec.prefix_len,
                                       lead_in=max(2, min(12, int(1.0 / ms["mixed"]) + 1)))
    per_kernel, roofline = kernel_rooflines(case, stage_ms, C)
    B, S = case.spec.batch, case.spec.q_len
    flops = 2 * C.table1_macs(case.shape, "mixed") + 2 * C.projection_macs(case.shape)
    res = {
        "ms_per_step": ms["mixed"],
        "tokens_per_s": B * S / (ms["mixed"] * 1e-3),
        "tflops": flops / (ms["mixed"] * 1e-3) / 1e12,
        "ms_per_step_by_mode": ms,
        "ms_per_step_cold_cache": ms_cold,
        "speedup_vs_absorb_only": (ms["absorb_only"] / ms["mixed"]) if "absorb_only" in ms else None,
        "speedup_vs_naive_only": (ms["naive_only"] / ms["mixed"]) if "naive_only" in ms else None,
        "prefix_expand_ms": case.expand_ms,
        "expanded_prefix_bytes": C.expanded_prefix_bytes(case.shape),
        "latent_prefix_bytes": C.latent_prefix_bytes(case.shape),
        "kernel_ms": stage_ms,
        "kernel_rooflines": per_kernel,
        "roofline": roofline,
    }
    return res, got, got_lse


def oracle_on_pairs(O, a, pairs, workers):
    """The definition oracle as it stands on `pairs`, the heads dealt out to `workers` threads
    (numpy's kernels release the interpreter lock; BLAS is held to one thread per worker).  A
    head stays in one thread, so its prefix expansion is formed once, as in a single call."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    heads = sorted({h for _, h in pairs})
    groups = [[p for p in pairs if p[1] in set(heads[w::workers])] for w in range(workers)]
    groups = [g for g in groups if g]
    try:
        from threadpoolctl import threadpool_limits
        limit = threadpool_limits(limits=1)
    except Exception:
        limit = None
    try:
        with ThreadPoolExecutor(len(groups)) as ex:
            parts = list(ex.map(lambda g: O.mla_decode_definition(**a, pairs=g), groups))
    finally:
        if limit is not None:
            limit.restore_original_limits()
    out, lse = np.full_like(parts[0][0], np.nan), np.full_like(parts[0][1], np.nan)
    for o, l in parts:
        m = ~np.isnan(l)
        out[m] = o[m]
        lse[m] = l[m]
    return out, lse, len(groups)


def oracle_leg(case, got, got_lse, n_req, budget_macs):
    """Times the fp64 oracle on a bounded sample of the workload (whole requests: all heads, whole
    prefix + suffix) and compares the benchmark's own output with it."""
    import numpy as np
    from oracle import mla_oracle as O
    spec = case.spec
    B, S, H, L_s = spec.batch, spec.q_len, spec.heads, spec.prefix_len
    workers = host_workers()
    a = case.wl.as_float64()
    if n_req <= 0:
        # the cost is dominated by up-projecting every visible token once per head: the prefix
        # once per head, the suffix per request
        per_req = (case.sum_ln / max(1, B)) * H * 131072.0
        n_req = int(max(2, min(B, (budget_macs - L_s * H * 131072.0) / max(per_req, 1.0))))
    reqs = sorted({0, B - 1} | set(range(0, B, max(1, B // n_req))))[:max(n_req, 1)]
    reqs = [b for b in reqs if b < B]
    pairs = [(b, h) for b in reqs for h in range(H)]
    t0 = time.perf_counter()
    ref, ref_lse, used = oracle_on_pairs(O, a, pairs, workers)
    cpu_s = time.perf_counter() - t0
    mask = ~np.isnan(ref_lse)
    err = np.abs(got[mask] - ref[mask])
    rn = np.linalg.norm(ref[mask], axis=-1)
    rel = np.linalg.norm(got[mask] - ref[mask], axis=-1) / np.maximum(rn, 1e-30)
    fin = np.isfinite(ref_lse[mask])
    full = len(reqs) == B
    baseline = {
        "value": len(reqs) * S / cpu_s, "unit": "tokens/s", "cores": int(used), "kind": "oracle",
        "sample": "%d of %d requests (all %d heads, whole prefix + suffix; the prefix is "
                  "up-projected once per head, as it would be for the whole batch), fp64 "
                  "definition oracle, heads dealt out to %d threads, %.1f s%s" % (
                      len(reqs), B, H, used, cpu_s,
                      "" if full else "; tokens/s of the sample, the full batch is extrapolated "
                                      "from it"),
        "rows_per_s": len(pairs) * S / cpu_s, "extrapolated": not full}
    parity = {
        "rows": int(mask.sum()), "max_abs_err": float(err.max()),
        "max_row_rel_l2": float(rel[rn > 0].max()) if (rn > 0).any() else 0.0,
        "max_lse_err": float(np.abs(got_lse[mask][fin] - ref_lse[mask][fin]).max())
        if fin.any() else 0.0}
    return baseline, parity


def bench_tree(args, torch, T, C, W, dev):
    """--workload "tree:B=64,H=128,L0=4096,G=4,L1=1024,Ln=512": a root prefix of L0 tokens shared by
    all B requests, G groups of B/G requests sharing L1 more tokens each, Ln private suffix
    tokens.  Timed: typhoon_mla_decode_tree, and beside it the flat alternative that shares only
    the root and carries the group prefix in every request's suffix (typhoon_mla_decode, mixed)."""
    kv = dict(item.split("=") for item in args.workload[5:].split(","))
    B, H = int(kv["B"]), int(kv.get("H", 128))
    L0, G, L1, Ln = int(kv.get("L0", 4096)), int(kv.get("G", 4)), int(kv.get("L1", 1024)), \
        int(kv.get("Ln", 512))
    assert B % G == 0
    spec = W.WorkloadSpec(args.workload, "bf16", B, H, 1, L0, Ln, Ln, seed=9)
    wl = W.make_workload(spec, poison=True)
    d = wl.to(dev)
    dims = T.make_dims(H, wl.sm_scale, "bf16")
    pk, pv = T.typhoon_mla_expand_prefix(dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv)
    nodes, keep = [(pk, pv, L0, 0, 0, B)], []
    gen = torch.Generator().manual_seed(10)
    for gi in range(G):
        c = torch.randn((L1, 512), generator=gen).to(torch.bfloat16).to(dev)
        r = torch.randn((L1, 64), generator=gen).to(torch.bfloat16).to(dev)
        k, v = T.typhoon_mla_expand_prefix(dims, c, r, d.w_uk, d.w_uv)
        keep.append((k, v))
        nodes.append((k, v, L1, 1, gi * (B // G), B // G))
    out = torch.empty((B, 1, H, 128), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((B, 1, H), dtype=torch.float32, device=dev)
    ws = torch.empty(T.typhoon_mla_decode_tree_workspace_bytes(dims, B, 1, nodes, Ln),
                     dtype=torch.uint8, device=dev)

    def step_tree():
        T.typhoon_mla_decode_tree(dims, d.q, nodes, suffix_pool=d.pool, block_table=d.block_table,
                                  suffix_lens=d.suffix_lens, max_suffix_len=Ln, w_uk=d.w_uk,
                                  w_uv=d.w_uv, out=out, lse_out=lse, workspace=ws)
    ms_tree = time_steps(step_tree, args.steps, args.warmup, torch)
    # flat alternative: same token counts, group prefix inside each request's suffix
    flat = W.make_workload(W.WorkloadSpec("flat", "bf16", B, H, 1, L0, L1 + Ln, L1 + Ln, seed=9),
                           poison=False).to(dev)
    ws2 = torch.empty(T.typhoon_mla_decode_workspace_bytes(dims, T.MODE_MIXED, B, 1, L0, L1 + Ln),
                      dtype=torch.uint8, device=dev)

    def step_flat():
        T.typhoon_mla_decode(dims, "mixed", flat.q, L0, prefix_k=pk, prefix_v=pv,
                             suffix_pool=flat.pool, block_table=flat.block_table,
                             suffix_lens=flat.suffix_lens, max_suffix_len=L1 + Ln, w_uk=d.w_uk,
                             w_uv=d.w_uv, out=out, lse_out=lse, workspace=ws2)
    ms_flat = time_steps(step_flat, max(3, args.steps // 2), max(1, args.warmup // 2), torch)
    elem = 2
    alg_bytes = ((L0 + G * L1) * H * 320 * elem + B * Ln * 576 * elem + B * H * (192 + 576) * elem
                 + 2 * H * 128 * 512 * elem)
    flops = 2 * B * H * ((L0 + L1) * 320 + Ln * 1088) + 4 * B * H * 128 * 512
    t = ms_tree * 1e-3
    print(json.dumps({
        "metric": "MLA decode tokens/s (tree-shaped shared prefixes: naive per node + absorb "
                  "suffix, one layer)",
        "value": B / t, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_tree, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": DATA,
        "config": {"workload": args.workload, "batch": B, "heads": H, "root_len": L0,
                   "groups": G, "group_prefix_len": L1, "suffix_len": Ln},
        "tflops": flops / t / 1e12,
        "ms_flat_root_only_sharing": ms_flat, "speedup_vs_flat": ms_flat / ms_tree,
        "roofline": {"kernel": "whole step", "bound": "hbm", "achieved": alg_bytes / t / 1e9,
                     "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": alg_bytes / t / HBM_PEAK,
                     "traffic": None, "algorithmic_bytes": alg_bytes},
        "cpu_baseline": None}))


def bench_sweep(args, torch, T, C, W, dev):
    """Batch-size sensitivity at L_s = 4096, L_n = 512 (the shape of the paper's latency-breakdown
    and batch-sweep experiments: Section 4 "Latency Breakdown", appendix batch-sensitivity
    figure) for DeepSeek-v3 (128 heads) and Kimi K2 (64 heads): mixed / absorb_only / auto step
    times and the per-kernel breakdown of the mixed step."""
    rows = []
    Ls = args.sweep_prefix
    for H in [int(x) for x in args.sweep_heads.split(",")]:
        for B in [int(x) for x in args.sweep_batches.split(",")]:
            name = "B=%d,H=%d,Ls=%d,Ln=512" % (B, H, Ls)
            case = Case(spec_of(name, W), ["mixed", "absorb_only", "auto"], torch, T, C, W, dev)
            steps = 20 if B <= 256 else 10
            # the clock moves with what ran just before: the modes take turns and the median of
            # the rounds is kept
            rounds = {m: [] for m in ("mixed", "absorb_only", "auto")}
            for _ in range(5):
                for m in rounds:
                    rounds[m].append(event_time(lambda: case.step(m), steps, 2, torch))
            ms = {m: sorted(v)[len(v) // 2] for m, v in rounds.items()}
            st = stage_times_in_step(lambda: case.step("mixed"), T, torch, 5, Ls,
                                     lead_in=max(2, min(12, int(1.0 / ms["mixed"]) + 1)))
            row = {"heads": H, "batch": B, "prefix_len": Ls, "ms_mixed": ms["mixed"], "ms_absorb_only": ms["absorb_only"],
                   "ms_auto": ms["auto"], "speedup_vs_absorb_only": ms["absorb_only"] / ms["mixed"],
                   "auto_vs_best": ms["auto"] / min(ms["mixed"], ms["absorb_only"]),
                   "auto_threshold": T.typhoon_mla_auto_batch_threshold(case.dims, 1, Ls), "kernel_ms": st}
            rows.append(row)
            print(json.dumps(row), flush=True)
            del case
            torch.cuda.empty_cache()
    print("| H | B | mixed us | absorb_only us | auto us | mixed speed-up | auto / best | "
          "stage 1 (naive prefix) | B1-proj (q absorb) | stage 2 (absorb suffix) | "
          "B2-proj + CombineLSE |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for r in rows:
        k = r["kernel_ms"]
        print("| %d | %d | %.0f | %.0f | %.0f | %.2f | %.2f | %.0f | %.0f | %.0f | %.0f |" % (
            r["heads"], r["batch"], r["ms_mixed"] * 1e3, r["ms_absorb_only"] * 1e3,
            r["ms_auto"] * 1e3, r["speedup_vs_absorb_only"], r["auto_vs_best"],
            k["prefix_attention"] * 1e3, k["query_absorb"] * 1e3, k["absorb_attention"] * 1e3,
            k["upproj_combine"] * 1e3))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives are part of "
              "it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2509_21081_amd import binding as T
    from paper_2509_21081_amd import cost_model as C
    from paper_2509_21081_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    T.lib()  # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    if args.sweep:
        return bench_sweep(args, torch, T, C, W, dev)
    if args.workload.startswith("tree:"):
        return bench_tree(args, torch, T, C, W, dev)
    modes = [m for m in args.modes.split(",") if m]
    if "mixed" not in modes:
        modes = ["mixed"] + modes

    case = Case(spec_of(args.workload, W), modes, torch, T, C, W, dev)
    spec = case.spec
    if args.calibrate_copy:
        # a plain copy of known size: rocprofv3's FETCH_SIZE / WRITE_SIZE for this kernel give the
        # scale factor of the HBM traffic counters
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region: exactly K steps of the whole hot path, inputs resident in HBM
    res, got, got_lse = measure(case, args.steps, args.warmup, args, torch, T, C, dev)
    result = {
        "metric": "MLA decode tokens/s (mixed naive-prefix + absorb-suffix attention, one layer)",
        "value": res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": spec.dtype, "data": DATA, "config": case.config(),
    }
    for k in ("tflops", "ms_per_step_by_mode", "ms_per_step_cold_cache", "speedup_vs_absorb_only",
              "speedup_vs_naive_only", "prefix_expand_ms", "expanded_prefix_bytes",
              "latent_prefix_bytes", "kernel_ms", "roofline", "kernel_rooflines"):
        result[k] = res[k]
    result["batch_threshold_nominal"] = C.batch_threshold(MFMA_BF16_PEAK, HBM_PEAK, spec.q_len)

    # ---- CPU baseline: the fp64 oracle as it stands, on a bounded sample of the same workload,
    # which also serves as a parity check of the timed output
    if not args.no_cpu_baseline:
        result["cpu_baseline"], result["parity_on_sample"] = oracle_leg(
            case, got, got_lse, args.cpu_sample_requests, 1.0e12)
    else:
        result["cpu_baseline"] = None
    result["input_generation_s"] = case.gen_s

    # ---- every other benchmark configuration, same protocol with fewer steps
    others = []
    if args.configs == "all":
        others = [c for c in BENCH_CONFIGS if c != spec.name]
    elif args.configs != "headline":
        others = [c for c in args.configs.split(",") if c and c != spec.name]
    if others:
        summary = {spec.name: dict(res, config=case.config(),
                                   parity_on_sample=result.get("parity_on_sample"))}
        del case, got, got_lse
        torch.cuda.empty_cache()
        for name in others:
            c = Case(spec_of(name, W), modes, torch, T, C, W, dev)
            r, g, gl = measure(c, max(10, args.steps // 2), max(3, args.warmup // 2), args, torch,
                               T, C, dev)
            r["config"] = c.config()
            if not args.no_cpu_baseline:
                # two whole requests against the oracle: a check of this run's output, not a timing
                _, r["parity_on_sample"] = oracle_leg(c, g, gl, 2, 0.0)
            summary[name] = r
            del c, g, gl
            torch.cuda.empty_cache()
        result["all_configs"] = summary
    print(json.dumps(result))


if __name__ == "__main__":
    main()
