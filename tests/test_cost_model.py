"""The analytic work model against the numbers the paper prints (Table 1, Section 3.2)."""
import json
import os

from paper_2509_21081_amd import cost_model as C

G = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "table1_deepseek_v3.json")))


def test_table1_deepseek_constants():
    H = G["heads"]
    assert H * C.macs_naive_per_token_head() / 1024 == G["naive_macs_per_BL_x1024"]
    assert H * C.macs_absorb_per_token_head() / 1024 == G["absorb_macs_per_BL_x1024"]
    sh = C.Shape(B=7, S_q=1, H=H, L_s=1000, sum_L_n=0)
    assert C.table1_macs(sh, "naive_only") == 7 * 1000 * 40 * 1024
    assert C.table1_macs(sh, "absorb_only") == 7 * 1000 * 136 * 1024
    assert C.table1_macs(sh, "mixed") == 7 * 1000 * 40 * 1024
    assert C.table1_hbm_elements(sh, "naive_only") == 1000 * 40 * 1024       # no batch factor
    assert round(C.table1_hbm_elements(sh, "absorb_only") / 1000 / 1024, 2) == \
        G["absorb_hbm_per_L_x1024_rounded_2dp"]
    own = C.Shape(B=7, S_q=1, H=H, L_s=0, sum_L_n=7 * 300)
    assert C.table1_macs(own, "mixed") == C.table1_macs(own, "absorb_only") == 7 * 300 * 136 * 1024
    assert C.table1_hbm_elements(own, "mixed") == C.table1_hbm_elements(own, "absorb_only")
    ratio = C.table1_hbm_elements(own, "naive_only") / C.table1_hbm_elements(own, "mixed")
    assert abs(ratio - G["nonshared_hbm_ratio_naive_over_absorb_approx"]) < 2      # "approx. 70x"
    assert round(C.macs_absorb_per_token_head() / C.macs_naive_per_token_head(), 1) == \
        G["shared_mac_ratio_absorb_over_naive"]


def test_batch_threshold_worked_number():
    bt = G["batch_threshold"]
    b = C.batch_threshold(bt["T_tops"] * 1e12, bt["M_tbps"] * 1e12)
    assert int(b) == bt["B_theta_printed"]
    # halves with two query tokens per request
    assert abs(C.batch_threshold(376e12, 1.8e12, S_q=2) - b / 2) < 1e-9


def test_measured_breakdown_matches_predicted_ratio():
    lb = G["latency_breakdown"]
    measured = (lb["absorb_only_ms"] - lb["absorb_stage_ms"]) / lb["naive_stage_ms"]
    assert round(measured, 1) == lb["shared_ratio_printed"]
    assert abs(measured - C.macs_absorb_per_token_head() / C.macs_naive_per_token_head()) < 0.15


def test_combine_cost():
    sh = C.Shape(B=3, S_q=2, H=16, L_s=5, sum_L_n=9)
    assert C.combine_elements(sh) == 2 * 3 * 2 * 16 * 128
