#!/usr/bin/env python3
"""Benchmark of the TyphoonMLA decode hot path on one MI355X.

A "step" is one pass of the whole hot path -- typhoon_mla_decode in mixed mode: naive prefix
attention, query absorption, absorb suffix attention, up-projection and LSE combine -- over one
batch of seeded synthetic input already resident in HBM.  The one-off prefix expansion is timed
separately.  Prints ONE JSON line: metric, value (tokens/s over the whole batch), ms_per_step,
config.workload, the per-kernel times, `roofline` for the dominant kernel and `cpu_baseline` (the
fp64 oracle timed on the host).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2_dsv3_b64]
                  [--modes mixed,absorb_only,naive_only] [--no-cpu-baseline] [--no-stages]
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

STAGES = {"prefix_attention": 0x10, "naive_suffix_attention": 0x20, "query_absorb": 0x40,
          "absorb_attention": 0x80, "upproj_combine": 0x100}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2_dsv3_b64")
    ap.add_argument("--modes", default="mixed,absorb_only,naive_only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stages", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for HBM counters)")
    ap.add_argument("--cpu-sample-requests", type=int, default=0,
                    help="requests (all heads each) in the oracle sample; 0 = auto")
    return ap.parse_args()


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


def read_traffic(workload, kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc (profiles/hbm_traffic.txt), or None."""
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
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic (seeded N(0,1) latents and queries, N(0,0.02) up-projections)",
        "config": {"workload": args.workload, "batch": B, "heads": H, "root_len": L0,
                   "groups": G, "group_prefix_len": L1, "suffix_len": Ln},
        "tflops": flops / t / 1e12,
        "ms_flat_root_only_sharing": ms_flat, "speedup_vs_flat": ms_flat / ms_tree,
        "roofline": {"kernel": "whole step", "bound": "hbm", "achieved": alg_bytes / t / 1e9,
                     "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": alg_bytes / t / HBM_PEAK,
                     "traffic": None, "algorithmic_bytes": alg_bytes},
        "cpu_baseline": None}))


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
    if args.workload.startswith("tree:"):
        return bench_tree(args, torch, T, C, W, dev)
    if args.workload in W.CONFIGS:
        spec = W.CONFIGS[args.workload]
    else:
        # ad-hoc shape: "B=128,H=64,Ls=4096,Ln=512[,Lmax=..][,Sq=1][,seed=7]" (bf16, 64-token blocks)
        kv = dict(item.split("=") for item in args.workload.split(","))
        ln = int(kv.get("Ln", 512))
        spec = W.WorkloadSpec(args.workload, "bf16", int(kv["B"]), int(kv.get("H", 128)),
                              int(kv.get("Sq", 1)), int(kv.get("Ls", 4096)), ln,
                              int(kv.get("Lmax", ln)), seed=int(kv.get("seed", 7)))
    t0 = time.perf_counter()
    wl = W.make_workload(spec, poison=True)
    gen_s = time.perf_counter() - t0
    d = wl.to(dev)
    dims = T.make_dims(spec.heads, wl.sm_scale, spec.dtype)
    B, S, H, L_s = spec.batch, spec.q_len, spec.heads, spec.prefix_len
    sum_ln = int(wl.suffix_lens.sum())
    shape = C.Shape(B, S, H, L_s, sum_ln, 2 if spec.dtype == "bf16" else 4)
    modes = [m for m in args.modes.split(",") if m]
    if "mixed" not in modes:
        modes = ["mixed"] + modes

    # one-off prefix expansion (prefill-time cost, Section 3.1), timed separately
    pk = pv = None
    expand_ms = None
    if L_s > 0:
        pk, pv = T.typhoon_mla_expand_prefix(dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv)
        expand_ms = event_time(lambda: T.typhoon_mla_expand_prefix(
            dims, d.prefix_ckv, d.prefix_krope, d.w_uk, d.w_uv, pk, pv), 3, 1, torch)
    sk = sv = None
    if "naive_only" in modes:
        sk, sv = T.typhoon_mla_expand_pool(dims, d.pool, d.w_uk, d.w_uv)

    out = torch.empty((B, S, H, 128), dtype=d.q.dtype, device=dev)
    lse = torch.empty((B, S, H), dtype=torch.float32, device=dev)
    ws = {}
    for m in modes:
        nbytes = T.typhoon_mla_decode_workspace_bytes(dims, T.MODES[m], B, S, L_s,
                                                      wl.max_suffix_len)
        ws[m] = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)

    def step(mode):
        T.typhoon_mla_decode(dims, mode, d.q, L_s, prefix_k=pk, prefix_v=pv,
                             prefix_ckv=d.prefix_ckv, prefix_krope=d.prefix_krope,
                             suffix_pool=d.pool, block_table=d.block_table,
                             suffix_lens=d.suffix_lens, max_suffix_len=wl.max_suffix_len,
                             suffix_k_pool=sk, suffix_v_pool=sv, w_uk=d.w_uk, w_uv=d.w_uv,
                             out=out, lse_out=lse, workspace=ws[mode])

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
    ms = {}
    ms["mixed"] = time_steps(lambda: step("mixed"), args.steps, args.warmup, torch)
    got = out.double().cpu().numpy()
    got_lse = lse.double().cpu().numpy()
    for m in modes:
        if m != "mixed":
            k = max(3, args.steps // 5)
            ms[m] = time_steps(lambda: step(m), k, max(1, args.warmup // 5), torch)

    # the same step with the caches flushed before every call (the timed region above runs the
    # steps back to back, so whatever fits the last-level cache -- weights, queries, partials,
    # a short prefix -- stays there between steps: `value` is a cache-warm number)
    ms_cold = cold_time(lambda: step("mixed"), 10, torch, dev)

    # ---- per-kernel device time (mixed mode), for the roofline of the dominant kernel
    stage_ms = {}
    if not args.no_stages and spec.dtype == "bf16":
        step("mixed")
        for name, bit in STAGES.items():
            if name == "naive_suffix_attention":
                continue
            if name == "prefix_attention" and L_s == 0:
                continue
            T.typhoon_mla_set_debug_flags(bit)
            try:
                stage_ms[name] = event_time(lambda: step("mixed"), args.steps, 3, torch)
            finally:
                T.typhoon_mla_set_debug_flags(0)
    tokens = B * S
    flops_mixed = 2 * C.table1_macs(shape, "mixed") + 2 * C.projection_macs(shape)
    result = {
        "metric": "MLA decode tokens/s (mixed naive-prefix + absorb-suffix attention, one layer)",
        "value": tokens / (ms["mixed"] * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms["mixed"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": spec.dtype, "data": "synthetic (seeded N(0,1) latents and queries, "
                                     "N(0,0.02) up-projections)",
        "config": {"workload": spec.name, "batch": B, "q_len": S, "heads": H, "prefix_len": L_s,
                   "suffix_tokens_total": sum_ln, "suffix_len_range": [spec.suffix_min,
                                                                       spec.suffix_max],
                   "block_size": spec.block_size, "seed": spec.seed},
        "tflops": flops_mixed / (ms["mixed"] * 1e-3) / 1e12,
        "ms_per_step_by_mode": ms,
        "ms_per_step_cold_cache": ms_cold,
        "speedup_vs_absorb_only": (ms["absorb_only"] / ms["mixed"]) if "absorb_only" in ms else None,
        "speedup_vs_naive_only": (ms["naive_only"] / ms["mixed"]) if "naive_only" in ms else None,
        "prefix_expand_ms": expand_ms,
        "expanded_prefix_bytes": C.expanded_prefix_bytes(shape),
        "latent_prefix_bytes": C.latent_prefix_bytes(shape),
        "kernel_ms": stage_ms,
        "batch_threshold_nominal": C.batch_threshold(MFMA_BF16_PEAK, HBM_PEAK, S),
    }

    # ---- roofline of the dominant kernel
    roofline = None
    if stage_ms:
        dom = max(stage_ms, key=stage_ms.get)
        t = stage_ms[dom] * 1e-3
        if dom == "prefix_attention":
            # number of prefix splits actually planned is not visible here; the partial-output
            # traffic is small, count one split
            w = C.prefix_kernel_work(shape, 1)
        elif dom == "absorb_attention":
            w = C.suffix_kernel_work(shape, 0)
        else:
            w = None
        if w is not None:
            intensity = w["flops"] / w["bytes"]
            ridge = MFMA_BF16_PEAK / HBM_PEAK
            if intensity < ridge:
                roofline = {"kernel": dom, "bound": "hbm", "achieved": w["bytes"] / t / 1e9,
                            "peak": HBM_PEAK / 1e9, "unit": "GB/s"}
            else:
                roofline = {"kernel": dom, "bound": "mfma", "achieved": w["flops"] / t / 1e12,
                            "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s"}
            roofline["frac"] = roofline["achieved"] / roofline["peak"]
            roofline["traffic"] = read_traffic(spec.name, dom)
            roofline["algorithmic_bytes"] = w["bytes"]
            roofline["algorithmic_flops"] = w["flops"]
            roofline["kernel_ms"] = stage_ms[dom]
            roofline["mfma_frac"] = w["flops"] / t / MFMA_BF16_PEAK
            roofline["hbm_frac"] = w["bytes"] / t / HBM_PEAK
    result["roofline"] = roofline
    # every attention kernel against both ceilings (the dominant one is in "roofline")
    per_kernel = {}
    for name, w in (("prefix_attention", C.prefix_kernel_work(shape, 1) if L_s else None),
                    ("absorb_attention", C.suffix_kernel_work(shape, 0))):
        if w is None or name not in stage_ms:
            continue
        t = stage_ms[name] * 1e-3
        per_kernel[name] = {"ms": stage_ms[name], "GB/s": w["bytes"] / t / 1e9,
                            "hbm_frac": w["bytes"] / t / HBM_PEAK,
                            "TFLOP/s": w["flops"] / t / 1e12,
                            "mfma_frac": w["flops"] / t / MFMA_BF16_PEAK}
    result["kernel_rooflines"] = per_kernel

    # ---- CPU baseline: the fp64 oracle as it stands, on a bounded sample of the same workload,
    # which also serves as a parity check of the timed output
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import mla_oracle as O
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            threads = os.cpu_count()
        a = wl.as_float64()
        n_req = args.cpu_sample_requests
        if n_req <= 0:
            # the cost is dominated by up-projecting every visible token once per head; the
            # small configurations run in full, the large ones on a few requests, which keeps
            # this leg to roughly 10-30 s of CPU work
            per_req = (sum_ln / max(1, B)) * H * 131072.0
            budget = 1.5e12 - L_s * H * 131072.0          # MACs, at ~1e11 fp64 MAC/s
            n_req = int(max(2, min(B, budget / max(per_req, 1.0))))
        reqs = sorted({0, B - 1} | set(range(0, B, max(1, B // n_req))))[:max(n_req, 1)]
        reqs = [b for b in reqs if b < B]
        pairs = [(b, h) for b in reqs for h in range(H)]
        t0 = time.perf_counter()
        ref, ref_lse = O.mla_decode_definition(**a, pairs=pairs)
        cpu_s = time.perf_counter() - t0
        mask = ~np.isnan(ref_lse)
        err = np.abs(got[mask] - ref[mask])
        rn = np.linalg.norm(ref[mask], axis=-1)
        rel = np.linalg.norm(got[mask] - ref[mask], axis=-1) / np.maximum(rn, 1e-30)
        fin = np.isfinite(ref_lse[mask])
        result["cpu_baseline"] = {
            "value": len(reqs) * S / cpu_s, "unit": "tokens/s", "cores": int(threads),
            "kind": "oracle",
            "sample": "%d of %d requests (all %d heads, whole prefix + suffix), fp64 definition "
                      "oracle, %.1f s" % (len(reqs), B, H, cpu_s)}
        result["parity_on_sample"] = {
            "rows": int(mask.sum()), "max_abs_err": float(err.max()),
            "max_row_rel_l2": float(rel[rn > 0].max()) if (rn > 0).any() else 0.0,
            "max_lse_err": float(np.abs(got_lse[mask][fin] - ref_lse[mask][fin]).max())
            if fin.any() else 0.0}
    result["input_generation_s"] = gen_s
    print(json.dumps(result))


if __name__ == "__main__":
    main()
