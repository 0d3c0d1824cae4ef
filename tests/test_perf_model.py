"""Pins for the analytical performance model (CPU only): the entries of the paper's Table 3 on round
numbers worked out by hand, the two printed forms of the maximal batch size, the scaling statements of
Appendix A.3, and the paper's two observations (section 3.1) on hardware of the class it measures on."""
import math

import pytest

from paper_2503_06433_amd import perf_model as pm

TOY = pm.Model(W=1e9, L=10, h_q=10, h_kv=5, d=100)
HW = pm.Hardware(hbm_bw=1e11, flops=1e12, link_bw=1e10, mem_bytes=1e11)


def test_table3_entries_on_round_numbers():
    p = pm.components(TOY, HW, "prefill", b=1, s=1000, tp=1)
    assert p["dm_lin"] == pytest.approx(0.02)                 # 2 W / B
    assert p["comp_lin"] == pytest.approx(2.0)                # 2 b W s / F
    assert p["dm_attn"] == pytest.approx(4e-5)                # 2 b s (h_q + 2 h_kv) d / B = 2*1000*20*100/1e11
    assert p["comp_attn"] == pytest.approx(2e-3)              # 2 b h_q s^2 d / F
    assert p["nw"] == 0.0
    d = pm.components(TOY, HW, "decode", b=8, s=1000, tp=2)
    assert d["dm_lin"] == pytest.approx(0.02)
    assert d["comp_lin"] == pytest.approx(0.016)              # 2 b W / F
    assert d["dm_attn"] == pytest.approx(1.6e-4)              # 4 b s h_kv d / B = 4*8*1000*5*100/1e11
    assert d["nw"] == pytest.approx(4 * 8 * 10 * 100 / 1e10)  # B_ar(2) = link_bw
    assert pm.layer_time(d) == pytest.approx(0.02 + d["comp_attn"] if d["comp_attn"] > d["dm_attn"] else 0.02 + 1.6e-4 + d["nw"])


def test_max_batch_two_printed_forms_agree():
    for tp, pp, dp in ((1, 1, 1), (2, 1, 1), (2, 2, 2), (1, 4, 2)):
        m_kv = HW.mem_bytes - 2 * TOY.L * TOY.W / (tp * pp)
        first = dp * m_kv * tp * pp / (4 * TOY.L * TOY.h_kv * TOY.d * 2000)
        assert pm.max_batch(TOY, HW, 2000, tp, pp, dp) == pytest.approx(first)
    # TP and PP scale the batch more than linearly, DP linearly
    b1 = pm.max_batch(TOY, HW, 2000)
    assert pm.max_batch(TOY, HW, 2000, tp=2) > 2 * b1 and pm.max_batch(TOY, HW, 2000, pp=2) > 2 * b1
    assert pm.max_batch(TOY, HW, 2000, dp=2) == pytest.approx(2 * b1)


def test_scaling_statements():
    free = pm.Hardware(hbm_bw=1e11, flops=1e12, link_bw=math.inf, mem_bytes=1e11)
    b, s = 4, 500
    base = pm.inv_throughput(TOY, free, "decode", b, s)
    # weight-bound decode: tensor parallelism divides the weight term, pipeline parallelism does not
    assert pm.inv_throughput(TOY, free, "decode", b, s, tp=4) < 0.3 * base
    assert pm.inv_throughput(TOY, free, "decode", b, s, pp=4) > 0.9 * base
    # compute-bound prefill with free links: both divide the work by the number of GPUs
    pb = pm.inv_throughput(TOY, free, "prefill", b, s)
    assert pm.inv_throughput(TOY, free, "prefill", b, s, tp=4) == pytest.approx(pb / 4, rel=1e-2)
    assert pm.inv_throughput(TOY, free, "prefill", b, s, pp=4) == pytest.approx(pb / 4, rel=1e-2)
    # ... and with real links the all-reduce term is charged to tensor parallelism only
    assert pm.inv_throughput(TOY, HW, "prefill", b, s, tp=4) > pm.inv_throughput(TOY, HW, "prefill", b, s, pp=4)


def test_the_two_observations_on_pcie_class_hardware():
    # a 24 GB, 125 TFLOP/s, 600 GB/s GPU with PCIe-class links (the class of the paper's A10 testbed)
    a10 = pm.Hardware(hbm_bw=600e9, flops=125e12, link_bw=8e9, mem_bytes=24e9)
    m = pm.LLAMA2_13B
    tp, pp, _ = pm.best_strategy(m, a10, "prefill", 8, 1000, 4)
    assert (tp, pp) == (1, 4)                                  # observation 1: prefill wants pipeline parallelism
    b = pm.max_batch(m, a10, 1200, tp=4)
    tp, pp, _ = pm.best_strategy(m, a10, "decode", b, 1200, 4)
    assert tp == 4                                             # observation 2: decode wants tensor parallelism


def test_report_runs():
    text = pm.report()
    assert "LLaMA-3-70B" in text and "measured kernel rates" in text


def test_efficiencies_follow_a_bench_record(tmp_path):
    rec = {"rooflines": {"c5.prefill_gemms": {"frac": 0.45}, "c5.prefill_attention": {"frac": 0.25},
                         "c4.decode_gemms": {"frac": 0.08}, "c4.decode_attention": {"frac": 0.58},
                         "c2.decode_gemms": {"frac": 0.2}}}
    hw = pm.hardware_from_bench(rec, "LLaMA-3-70B")
    assert (hw.eff_linear_prefill, hw.eff_attn_prefill, hw.eff_linear_decode, hw.eff_attn_decode) == (0.45, 0.25, 0.08, 0.58)
    assert hw.hbm_bw == pm.MI355X_PEAK.hbm_bw
    hw7 = pm.hardware_from_bench(rec, "LLaMA-2-7B")            # classes the record lacks keep the fallback
    assert hw7.eff_linear_decode == 0.2 and hw7.eff_linear_prefill == pm.MI355X_MEASURED.eff_linear_prefill
    import json
    path = tmp_path / "BENCH.json"
    path.write_text(json.dumps({"parsed": rec}))               # the driver's record form
    assert pm.hardware_from_bench(str(path), "LLaMA-3-70B").eff_attn_decode == 0.58
    # a slower decode GEMM makes the modelled decode step slower, nothing else
    slow = pm.hardware_from_bench({"rooflines": {"c4.decode_gemms": {"frac": 0.04}}}, "LLaMA-3-70B")
    a = pm.components(pm.LLAMA3_70B, hw, "decode", 64, 2000)["dm_lin"]
    b = pm.components(pm.LLAMA3_70B, slow, "decode", 64, 2000)["dm_lin"]
    assert b == pytest.approx(2 * a)


def test_link_sweep_resharding_never_loses_and_pays_on_slow_links():
    # A10-class hardware (the paper's testbed class): re-sharding can always keep one strategy, so it never loses
    # by more than its (upper-bound) movement charge, and with PCIe-class links it wins (sections 6.2, 6.5)
    a10 = pm.Hardware(hbm_bw=600e9, flops=125e12, link_bw=8e9, mem_bytes=24e9)
    rows = pm.link_sweep(pm.LLAMA2_13B, a10, 4, s_in=1000, s_out=200, host_bw=8e9)
    gains = [r[6] for r in rows]
    assert all(g >= 0.999 for g in gains)
    switched = [r for r in rows if r[3] != r[4]]
    assert switched and all(r[3] < r[4] and r[6] > 1.03 for r in switched)   # pipeline-heavier prefill, tensor-heavier decode
    assert rows[0][3] == rows[0][4] == 1                       # links ten times slower: pipeline parallelism throughout
    assert rows[-1][3] == rows[-1][4] == 4                     # links fifty times faster: tensor parallelism throughout
    # request_time is the sum of its parts: no outputs -> the prefill term alone
    t = pm.request_time(pm.LLAMA2_13B, a10, 4, 1000, 0, 1, 1)
    assert t == pytest.approx(pm.inv_throughput(pm.LLAMA2_13B, a10, "prefill", 16, 1000, tp=1, pp=4))
