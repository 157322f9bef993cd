"""Analytic work model of MLA decode attention (paper Table 1 and Section 3.2).

MAC and HBM-element counts of the naive, absorb and mixed (TyphoonMLA) formulations, the batch
threshold B_theta of the break-even equation, and the per-kernel algorithmic bytes / flops that
the benchmark divides by measured kernel time.  Table 1 counts elements ("words"); bytes are
elements x element size and FLOPs are 2 x MACs.
"""
from dataclasses import dataclass

D_L, D_N, D_R, D_V = 512, 128, 64, 128
D_QK = D_N + D_R


@dataclass
class Shape:
    B: int
    S_q: int
    H: int
    L_s: int
    sum_L_n: int          # total suffix tokens over the batch (B * L_n for fixed lengths)
    elem_bytes: int = 2


def macs_naive_per_token_head():      # D_qk + D_v            (Table 1, "Naive" MAC row)
    return D_QK + D_V


def macs_absorb_per_token_head():     # 2 D_l + D_r           (Table 1, "Absorb" MAC row)
    return 2 * D_L + D_R


def table1_macs(sh, mode):
    """MACs of the attention itself (projections excluded), Table 1 upper half."""
    shared = sh.B * sh.S_q * sh.L_s * sh.H
    own = sh.S_q * sh.sum_L_n * sh.H
    n, a = macs_naive_per_token_head(), macs_absorb_per_token_head()
    return {"naive_only": shared * n + own * n,
            "absorb_only": shared * a + own * a,
            "mixed": shared * n + own * a}[mode]


def table1_hbm_elements(sh, mode):
    """Cache elements read from HBM, Table 1 lower half."""
    exp = sh.H * (D_QK + D_V)
    lat = D_L + D_R
    return {"naive_only": sh.L_s * exp + sh.sum_L_n * exp,
            "absorb_only": sh.L_s * lat + sh.sum_L_n * lat,
            "mixed": sh.L_s * exp + sh.sum_L_n * lat}[mode]


def projection_macs(sh):
    """q_nope W_UK and O_lat W_UV^T (Algorithm 1 steps 5 and 7): 2 x rows x 128 x 512."""
    return 2 * sh.B * sh.S_q * sh.H * D_N * D_L


def batch_threshold(T_ops, M_bytes, S_q=1):
    """B_theta = (D_qk + D_v) / (S_q (2 D_l + D_r)) * T / M  (Section 3.2 break-even equation)."""
    return (D_QK + D_V) / (S_q * (2 * D_L + D_R)) * T_ops / M_bytes


def combine_elements(sh):
    """CombineLSE reads 2 B S_q H D_v elements (Section 3.2)."""
    return 2 * sh.B * sh.S_q * sh.H * D_V


# ---- per-kernel algorithmic work (what the method itself must move / compute) ----------------
def prefix_kernel_work(sh, n_split=1):
    """Naive shared-prefix pass: expanded K/V once, queries once, partial outputs written.

    The RoPE part of a key is the same for every head; the kernels fetch it from one head's
    blocks, so per token the pass must move H x (D_n + D_v) + D_r elements, not the
    H x (D_qk + D_v) of Table 1 (kept as `bytes_table1` for comparison)."""
    rows = sh.B * sh.S_q * sh.H
    other = rows * D_QK * sh.elem_bytes + n_split * rows * (D_V + 1) * 4
    bytes_ = sh.L_s * (sh.H * (D_N + D_V) + D_R) * sh.elem_bytes + other
    table1 = sh.L_s * sh.H * (D_QK + D_V) * sh.elem_bytes + other
    flops = 2 * sh.B * sh.S_q * sh.L_s * sh.H * (D_QK + D_V)
    return dict(bytes=bytes_, flops=flops, bytes_table1=table1)


def suffix_kernel_work(sh, n_partials_rows=0):
    """Absorb suffix pass: latent rows once, absorbed queries once, latent partials written.
    n_partials_rows = number of (row, chunk) partials actually written."""
    rows = sh.B * sh.S_q * sh.H
    bytes_ = (sh.sum_L_n * (D_L + D_R) * sh.elem_bytes + rows * (D_L + D_R) * sh.elem_bytes
              + n_partials_rows * (D_L * sh.elem_bytes + 4))
    flops = 2 * sh.S_q * sh.sum_L_n * sh.H * (2 * D_L + D_R)
    return dict(bytes=bytes_, flops=flops)


def expanded_prefix_bytes(sh):
    return sh.L_s * sh.H * (D_QK + D_V) * sh.elem_bytes


def latent_prefix_bytes(sh):
    return sh.L_s * (D_L + D_R) * sh.elem_bytes
