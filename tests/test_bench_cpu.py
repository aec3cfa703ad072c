"""Host-side checks of bench.py that need no GPU: the single-GPU contract, the fixed headline choices, and the
roofline arithmetic on a made-up timing."""
import os
import subprocess
import sys
import types

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode == 2 and "single-GPU" in res.stderr and res.stdout.strip() == ""


def test_headline_is_the_largest_config_in_one_fixed_form():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.HEADLINE_CONFIG == 5 and bench.CONFIG_TEXT[5].startswith("configs[4]")
    # one fixed form per configuration (never the best of several): one fused launch for the single-layer
    # configurations, one persistent launch per pass for the 53-layer stacks
    assert bench.HEADLINE_FORM == {1: "fused", 2: "fused", 3: "fused", 4: "fused", 5: "fused_chain"}
    assert all(f in bench.POLICY_TEXT for f in bench.HEADLINE_FORM.values())
    # a step of the fused policy lasts at least several milliseconds at the measured pass times
    measured_us = {1: 5.5, 2: 8.8, 3: 14.4, 4: 49.4, 5: 451.0}
    for cfg, passes in bench.PASSES_PER_STEP.items():
        assert passes * measured_us[cfg] >= 10e3


def test_roofline_arithmetic():
    sys.path.insert(0, ROOT)
    import bench
    # config-5-like numbers: 49 launches, HBM-bound
    wl = types.SimpleNamespace(cfg=5, flops=65394180096, bytes=723700736, launches={"fused": 49, "fused_chain": 1},
                               launch_work=[(65394180096 // 49, 723700736 // 49)] * 49)
    r = bench.roofline(wl, "fused", {"event_us_per_pass_median": 490.0})
    assert r["bound"] == "hbm" and r["launches_per_pass"] == 49
    assert abs(r["avg_launch_us"] - 10.0) < 1e-9
    assert abs(r["achieved"] - 723700736 / 49 / 10e-6 / 1e9) < 1e-6 and abs(r["frac"] - r["achieved"] / 8000.0) < 1e-12
    assert abs(r["bound_us_per_pass"] - 723700736 / 8e12 * 1e6) < 0.05      # every launch is HBM-bound here
    assert abs(r["frac_of_own_bound"] - r["bound_us_per_pass"] / 490.0) < 1e-12
    c = bench.roofline(wl, "fused_chain", {"event_us_per_pass_median": 700.0})
    assert c["launches_per_pass"] == 1 and abs(c["avg_launch_us"] - 700.0) < 1e-9 and c["kernel"] == "st_chain_kernel"
    # a compute-bound workload is priced against the MFMA peak of its dtype
    wm = types.SimpleNamespace(cfg=4, flops=10 ** 12, bytes=10 ** 8, launches={"fused": 1}, launch_work=[(10 ** 12, 10 ** 8)])
    m = bench.roofline(wm, "fused", {"event_us_per_pass_median": 1000.0})
    assert m["bound"] == "mfma" and m["unit"] == "TFLOP/s" and abs(m["achieved"] - 1000.0) < 1e-9 and m["peak"] == 2516.6
