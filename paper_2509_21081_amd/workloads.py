"""Seeded synthetic MLA-decode workloads (inputs only: no attention arithmetic lives here).

The paper measures on question datasets behind three long system prompts under continuous
batching (Section 4, "Experiments on NPUs", Table 2).  Only lengths and batch sizes reach the
attention kernel, so these generators stand in for those workloads: DeepSeek-v3 head dimensions
(Table 1), a shared prefix of 256 ... 32768 tokens and a paged, variable-length suffix.

Draw order is fixed (CPU `torch.Generator`, so every consumer sees identical bits):
  q, prefix_ckv, prefix_krope, suffix_lens, suffix rows per request, W_UK, W_UV,
  block-table permutation.
Values: q, c_KV, k_rope ~ N(0, 1); W ~ N(0, std 0.02); each rounded once (RNE) to the I/O dtype.
Unused pool blocks, the tail slots of each request's last block and the padding of the block
table can be poisoned (NaN rows / index -1) so that any read outside the visible cache shows up.
"""
import math
from dataclasses import dataclass, field

import torch

D_LATENT, D_NOPE, D_ROPE, D_V = 512, 128, 64, 128
D_QK = D_NOPE + D_ROPE
D_ROW = D_LATENT + D_ROPE


@dataclass
class WorkloadSpec:
    name: str
    dtype: str            # "bf16" | "fp32"
    batch: int
    heads: int
    q_len: int
    prefix_len: int
    suffix_min: int
    suffix_max: int       # inclusive; == suffix_min for fixed-length configs
    block_size: int = 64
    shuffle_blocks: bool = False
    seed: int = 0
    q_gain: float = 1.0   # >1 gives a peaked softmax (larger logits) for bug-revealing variants


# The five benchmark configurations (batch, heads, lengths, paging and seeds as specified for
# this build; dimensions are DeepSeek-v3's, Table 1).
CONFIGS = {
    "cfg1_tiny_fp32": WorkloadSpec("cfg1_tiny_fp32", "fp32", 4, 16, 1, 256, 64, 64, seed=0),
    "cfg2_dsv3_b64": WorkloadSpec("cfg2_dsv3_b64", "bf16", 64, 128, 1, 4096, 512, 512, seed=1),
    "cfg3_long_prompt": WorkloadSpec("cfg3_long_prompt", "bf16", 256, 128, 1, 32768, 256, 2048,
                                     shuffle_blocks=True, seed=2),
    "cfg4_mtp": WorkloadSpec("cfg4_mtp", "bf16", 128, 128, 2, 8192, 1024, 1024, seed=3),
    "cfg5_tp_rank": WorkloadSpec("cfg5_tp_rank", "bf16", 512, 16, 1, 16384, 512, 4096, seed=4),
    "cfg5b_no_prefix": WorkloadSpec("cfg5b_no_prefix", "bf16", 512, 16, 1, 0, 512, 4096, seed=4),
}


@dataclass
class Workload:
    spec: WorkloadSpec
    sm_scale: float
    q: torch.Tensor             # [B, S_q, H, 192]
    prefix_ckv: torch.Tensor    # [L_s, 512]
    prefix_krope: torch.Tensor  # [L_s, 64]
    pool: torch.Tensor          # [n_blocks, block, 576]
    block_table: torch.Tensor   # [B, max_blocks] int32
    suffix_lens: torch.Tensor   # [B] int32
    w_uk: torch.Tensor          # [H, 128, 512]
    w_uv: torch.Tensor          # [H, 128, 512]
    max_suffix_len: int = 0
    extras: dict = field(default_factory=dict)

    def to(self, device):
        moved = {}
        for name in ("q", "prefix_ckv", "prefix_krope", "pool", "block_table", "suffix_lens",
                     "w_uk", "w_uv"):
            moved[name] = getattr(self, name).to(device)
        return Workload(self.spec, self.sm_scale, max_suffix_len=self.max_suffix_len,
                        extras=dict(self.extras), **moved)

    def as_float64(self):
        """Exact promotion of the stored (already rounded) inputs, as numpy arrays."""
        f = lambda t: t.detach().cpu().to(torch.float64).numpy()
        return dict(q=f(self.q), prefix_ckv=f(self.prefix_ckv), prefix_krope=f(self.prefix_krope),
                    pool=f(self.pool), block_table=self.block_table.cpu().numpy(),
                    suffix_lens=self.suffix_lens.cpu().numpy(), w_uk=f(self.w_uk),
                    w_uv=f(self.w_uv), sm_scale=self.sm_scale)


def torch_dtype(name):
    return {"bf16": torch.bfloat16, "fp32": torch.float32}[name]


def _randn(gen, shape, std, dtype, chunk_rows=1 << 16):
    """N(0, std) drawn in fp32 on the CPU generator, rounded once to `dtype`."""
    out = torch.empty(shape, dtype=dtype)
    flat = out.view(-1, shape[-1]) if len(shape) > 1 else out.view(1, -1)
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        x = torch.randn((r1 - r0, flat.shape[1]), generator=gen, dtype=torch.float32)
        if std != 1.0:
            x.mul_(std)
        flat[r0:r1] = x.to(dtype)
    return out


def make_workload(spec, poison=True, spare_blocks=3):
    dt = torch_dtype(spec.dtype)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(spec.seed)
    B, S, H, bs = spec.batch, spec.q_len, spec.heads, spec.block_size

    q = _randn(gen, (B, S, H, D_QK), 1.0, torch.float32)
    if spec.q_gain != 1.0:
        q = q * spec.q_gain
    q = q.to(dt)
    prefix_ckv = _randn(gen, (spec.prefix_len, D_LATENT), 1.0, dt) if spec.prefix_len else \
        torch.empty((0, D_LATENT), dtype=dt)
    prefix_krope = _randn(gen, (spec.prefix_len, D_ROPE), 1.0, dt) if spec.prefix_len else \
        torch.empty((0, D_ROPE), dtype=dt)
    if spec.suffix_max > spec.suffix_min:
        lens = torch.randint(spec.suffix_min, spec.suffix_max + 1, (B,), generator=gen)
    else:
        lens = torch.full((B,), spec.suffix_min, dtype=torch.int64)
    blocks_per_req = [(int(n) + bs - 1) // bs for n in lens]
    used = sum(blocks_per_req)
    n_blocks = used + spare_blocks
    max_blocks = max(1, max(blocks_per_req) if blocks_per_req else 1)

    pool = torch.empty((n_blocks, bs, D_ROW), dtype=dt)
    if poison:
        pool.fill_(float("nan"))
    else:
        pool.zero_()
    # suffix rows are drawn request by request into a staging area in logical order
    staged = []
    for b in range(B):
        n = int(lens[b])
        staged.append(_randn(gen, (n, D_ROW), 1.0, dt) if n else torch.empty((0, D_ROW), dtype=dt))
    w_uk = _randn(gen, (H, D_NOPE, D_LATENT), 0.02, dt)
    w_uv = _randn(gen, (H, D_V, D_LATENT), 0.02, dt)
    if spec.shuffle_blocks:
        perm = torch.randperm(n_blocks, generator=gen)
    else:
        perm = torch.arange(n_blocks)

    block_table = torch.full((B, max_blocks), -1 if poison else 0, dtype=torch.int32)
    nxt = 0
    for b in range(B):
        n = int(lens[b])
        for i in range(blocks_per_req[b]):
            phys = int(perm[nxt]); nxt += 1
            block_table[b, i] = phys
            lo, hi = i * bs, min(n, (i + 1) * bs)
            pool[phys, : hi - lo] = staged[b][lo:hi]
    staged = None
    max_suffix_len = int(lens.max()) if B else 0
    return Workload(spec, 1.0 / math.sqrt(D_QK), q, prefix_ckv, prefix_krope, pool, block_table,
                    lens.to(torch.int32), w_uk, w_uv, max_suffix_len=max_suffix_len)


def small_spec(name="small", dtype="bf16", batch=3, heads=16, q_len=1, prefix_len=100,
               suffix_min=0, suffix_max=150, block_size=64, shuffle_blocks=True, seed=11,
               q_gain=1.0):
    """Test-sized spec: spans several tiles with ragged tails, still seconds for the oracle."""
    return WorkloadSpec(name, dtype, batch, heads, q_len, prefix_len, suffix_min, suffix_max,
                        block_size, shuffle_blocks, seed, q_gain)


def sample_pairs(workload, n_full_requests=8, n_full_heads=2):
    """Deterministic (b, h) sample for full-size parity: every head of a few requests (the
    shortest and longest suffix, the first and last index, then evenly spaced ones) plus every
    request for a few heads."""
    B, H = workload.spec.batch, workload.spec.heads
    lens = workload.suffix_lens.cpu()
    chosen = [0, B - 1, int(torch.argmin(lens)), int(torch.argmax(lens))]
    step = max(1, B // max(1, n_full_requests))
    chosen += list(range(step // 2, B, step))
    reqs = []
    for b in chosen:
        if b not in reqs:
            reqs.append(b)
    reqs = reqs[:max(n_full_requests, 4)]
    heads = sorted({0, H - 1} | {(H // max(1, n_full_heads)) * i for i in range(n_full_heads)})
    pairs = {(b, h) for b in reqs for h in range(H)} | {(b, h) for b in range(B) for h in heads}
    return sorted(pairs)
