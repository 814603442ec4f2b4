"""CPU checks of the benchmark's bookkeeping: the algorithmic work per kernel, the compulsory bytes it sums into the
HBM floor, and the HBM traffic it reads from the committed rocprofv3 summaries (no GPU, nothing is timed)."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_work_per_kernel_adds_up():
    from paper_2508_02317_amd.inputs import CONFIGS
    B = _bench()
    cfg = CONFIGS["a3b_8k"]
    P = cfg.T * cfg.k
    work = B.kernel_work(cfg, P, gather=True, save_gu=True)
    products = ("ffn_gate_up", "ffn_down", "ffn_dact", "ffn_dx", "wgrad_down", "wgrad_gate_up")
    assert sum(work[n][1] for n in products) == 18.0 * P * cfg.d * cfg.f          # routed flops of one step
    assert all(work[n][0] == "mfma" for n in products)
    floor = sum(work[n][2] for n in products)
    s = 2
    Pd, Pf, Edf, Td = P * cfg.d * s, P * cfg.f * s, cfg.E * cfg.d * cfg.f * s, cfg.T * cfg.d * s
    # every weight read three times (forward, input gradient, as the other operand's gradient is written once), x and dy by token
    assert floor == (Td + 2 * Edf + 3 * Pf) + (Pf + Edf + Pd) + (Td + Edf + 4 * Pf) + (2 * Pf + 2 * Edf + Pd) + (Td + Pf + Edf) + (2 * Pf + Td + 2 * Edf)
    late = B.kernel_work(cfg, P, gather=True, save_gu=True, late_weight=True)
    assert late["ffn_dact"][2] - work["ffn_dact"][2] == Pf                         # w * act written by the backward
    movers = B.kernel_work(cfg, P, gather=False, save_gu=True)
    assert movers["combine_fwd"] == ("hbm", (P + cfg.T) * cfg.d * s + P * 8, None)
    f32 = B.kernel_work(CONFIGS["tiny"], 512, gather=True, save_gu=True)
    assert f32["f32_gate_up"][0] == "alu"


def test_traffic_comes_from_the_committed_profiles():
    B = _bench()
    for workload, gather in (("a3b_8k", True), ("a3b_8k", False), ("a3b_long", True), ("a3b_ep_skew", True), ("small", True)):
        traffic, source = B.measured_traffic(workload, gather)
        assert source == os.path.join("profiles", workload + ("" if gather else "_no_gather") + ".md")
        for name in ("ffn_gate_up", "ffn_down", "ffn_dact", "ffn_dx", "wgrad_down", "wgrad_gate_up", "combine_fwd"):
            assert traffic[name] > 1e6, (workload, name)
    traffic, source = B.measured_traffic("no_such_workload", True)
    assert traffic == {} and source is None


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "single-GPU" in res.stderr
