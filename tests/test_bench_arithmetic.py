"""The work the bench credits: algorithmic FLOPs of the StreamBP step (Sec. 3.2) - host arithmetic only."""
import importlib.util
import os

from paper_2506_03077_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
bench = importlib.util.module_from_spec(spec)
spec.loader.exec_module(bench)


def test_headline_workload_flops():
    cfg = synth.CONFIGS["7b"]
    T = 32768
    fl = bench.algorithmic_flops(cfg, T, T - T // 4)
    # 6 * P_lin per token with P_lin = d*Hq*dh + 2*d*Hkv*dh + Hq*dh*d + 3*d*F = 233,046,016
    p_lin = 3584 * 28 * 128 * 2 + 2 * 3584 * 4 * 128 + 3 * 3584 * 18944
    assert p_lin == 233_046_016
    assert fl["linear"] == 6.0 * p_lin * T
    assert abs(fl["linear"] / 1e12 - 45.82) < 0.01
    # 14 * dh per visible (query, key) pair per query head: 4 forward + 10 backward; exact causal pairs T(T+1)/2
    assert abs(fl["attention"] / 1e12 - 26.94) < 0.01
    # chunked causal attention visits (1 + D) / (2 D) of the square (Sec. 3.2.2): an upper allowance, never credited
    D = T // 2048
    assert fl["attention"] <= 14.0 * 128 * 28 * (1 + D) * T * T / (2 * D)
    assert abs(fl["head_all_rows"] / 1e12 - 107.15) < 0.01
    assert abs(fl["head_active_rows"] / 1e12 - 80.36) < 0.01
    assert fl["total"] == fl["linear"] + fl["attention"] + fl["head_active_rows"]
    assert abs(fl["total_all_rows"] / 1e12 - 179.9) < 0.05


def test_other_workloads_flops():
    ll = synth.CONFIGS["llama_layer"]
    fl = bench.algorithmic_flops(ll, 8192, 0, batch=1, has_layer=True, has_head=False)
    assert abs(fl["linear"] / 1e12 - 10.72) < 0.01 and abs(fl["attention"] / 1e12 - 1.92) < 0.01 and fl["head_all_rows"] == 0
    g = synth.CONFIGS["grpo"]
    fl = bench.algorithmic_flops(g, 16384, 8 * 12288, batch=8)
    assert abs(fl["linear"] / 1e12 - 8 * 22.91) < 0.05 and abs(fl["attention"] / 1e12 - 8 * 6.73) < 0.05
    assert abs(fl["head_active_rows"] / 1e12 - 321.5) < 0.1 and abs(fl["head_all_rows"] / 1e12 - 428.6) < 0.1


def test_more_than_one_gpu_is_refused():
    import subprocess
    import sys
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0 and "ONE GPU" in p.stderr


def test_whole_stack_flops():
    # 28 layers + head on all 32768 positions: 28 * (45.82 + 26.94) + 107.15 TF = 2.144 PF
    cfg = synth.CONFIGS["7b"]
    fl = bench.algorithmic_flops(cfg, 32768, 32768, n_layers=28)
    assert abs(fl["total"] / 1e15 - 2.144) < 0.002
    one = bench.algorithmic_flops(cfg, 32768, 32768)
    assert abs(one["total"] / 1e12 - 179.9) < 0.05 and one["total"] == one["total_all_rows"]
