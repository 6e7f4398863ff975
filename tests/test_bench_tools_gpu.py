"""bench.py's measurement modes keep their contract: one JSON line each, with the fields the profiles are built
from, and figures that make sense (run as subprocesses, the way the profiles' commands run them)."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + list(args), stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True, timeout=280)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, res.stdout[-2000:]
    return json.loads(lines[0])


def test_bench_line_of_a_short_config_and_comparison_with_the_same_library():
    lib = os.path.join(ROOT, "paper_2512_18134_amd", "libmi355attn.so")
    d = run_bench("--config", "2", "--steps", "10", "--warmup", "5", "--compare-lib", lib)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "compare"):
        assert key in d, key
    assert d["config"]["workload"].startswith("config2_") and d["n_gpus"] == 1 and d["steps"] == 10
    assert d["roofline"]["bound"] == "mfma" and 0.0 < d["roofline"]["frac"] < 1.0
    assert abs(d["roofline"]["frac"] - d["roofline"]["achieved"] / d["roofline"]["peak"]) < 1e-9
    # a 25 us kernel: timed between one pair of events, which cannot come out above the per-launch pairs by much
    assert d["config"]["kernel_ms_avg"] <= 1.2 * d["config"]["kernel_ms_events_around_each_launch"]
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["cores"] >= 1
    # the library against itself: same bits, about the same time
    assert d["compare"]["same_bits"] is True
    assert 0.8 < d["compare"]["other_over_this"] < 1.25


def test_timeline_accounts_for_every_tile():
    d = run_bench("--timeline", "--config", "3")
    # config 3: B2 H16 S4096 D128 causal = 32 heads x 16 query tiles of 256 rows, two per CU slot
    assert d["workgroups"] == 512 and d["cus_used"] == 256
    assert d["workgroups_per_cu_min_mean_max"] == [2, 2.0, 2]
    ph = d["phase_us_mean_max"]
    assert set(ph) == {"take_up_to_loads_issued", "loads_issued_to_k0_q_landed", "s0_and_setup", "loop",
                       "loop_end_to_o_staged", "store_o"}
    assert all(v[0] >= 0.0 and v[1] >= v[0] for v in ph.values())
    assert 0.5 < d["loop_share_of_cu_time"] < 1.0
    assert 0.5 * d["span_us"] < 1e3 * d["event_ms"] < 3.0 * d["span_us"]
    assert len(d["last_end_per_xcd_us_mean_min_max"]) == 8


def test_mfma_probe_reports_the_ceiling_and_what_it_depends_on():
    d = run_bench("--probe-mfma", "--steps", "3")
    res, pat = d["results"], d["random_operand_patterns"]
    assert set(res) == {"%d_waves_per_simd_%s" % (w, k) for w in (1, 2) for k in ("random", "constant", "zero")}
    assert set(pat) == {"both_operands_change", "a_shared_by_pairs", "a_fixed_b_changes", "both_fixed",
                        "16x16x32_both_change", "f16_both_change"}
    for v in list(res.values()) + list(pat.values()):
        assert 0.3 < v["frac_of_peak"] < 1.02, v
    # operands that are all zero cost the matrix pipe no power: nothing runs faster than that
    assert res["1_waves_per_simd_zero"]["frac_of_peak"] > 0.9
    assert all(v["frac_of_peak"] <= res["1_waves_per_simd_zero"]["frac_of_peak"] + 0.02 for v in pat.values())


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True, timeout=120)
    assert res.returncode != 0 and "ONE GPU" in res.stderr
