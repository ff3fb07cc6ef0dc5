"""Host-side pieces of bench.py that need no GPU: the resumable sweep log and the byte / flop counts the
roofline figures are built from."""
import dataclasses

import bench
from paper_2505_19645_amd.synth import PRESETS


def test_sweep_log_resumes(tmp_path):
    path = str(tmp_path / "sweep.csv")
    log = bench.SweepLog(path)
    assert log.get("qwen", 1, 0) is None
    row = {"B": 16, "gamma": 3, "T": 64, "us": 194.5, "n_active": 58, "N_model": 59.27, "Texp_model": 4.32,
           "layer_hbm_frac": 0.69, "roofline_us": 134.2, "roofline_frac": 0.69}
    log.put("qwen", row)
    log.put("qwen/skew1.5", dict(row, us=150.0))
    again = bench.SweepLog(path)                       # a later run finds both points and nothing else
    assert again.get("qwen", 16, 3) == row and again.get("qwen/skew1.5", 16, 3)["us"] == 150.0
    assert again.get("qwen", 16, 0) is None
    assert open(path).read().count("\n") == 3          # header + two points, not rewritten on reopening


def test_algorithmic_bytes_and_flops():
    s = PRESETS["deepseek-v3"]
    n, T = 214, 64
    per_expert = 3 * 7168 * 2048 * 2
    assert s.expert_bytes == per_expert and s.shared_bytes == per_expert and s.router_bytes == 256 * 7168 * 2
    assert bench.layer_bytes(s, n, T) == n * per_expert + per_expert + 256 * 7168 * 2 + 2 * T * 7168 * 2
    assert bench.gate_up_bytes(s, n, T) + bench.down_bytes(s, n, T) == \
        (n + 1) * per_expert + T * 7168 * 2 + 2 * (T * 8 * 2048 + T * 2048) * 2 + (T * 8 * 7168 + T * 7168) * 4
    assert bench.layer_flops(s, T) == 6 * T * 8 * 7168 * 2048 + 6 * T * 7168 * 2048 + 2 * T * 256 * 7168
    q = dataclasses.replace(s, weight_format=1)        # one byte per weight plus one fp32 scale per weight row
    assert q.expert_bytes == 3 * 7168 * 2048 + (2 * 2048 + 7168) * 4
    assert bench.gate_up_bytes(q, n, T) - bench.gate_up_bytes(q, n - 1, T) == 2 * 7168 * 2048 + 2 * 2048 * 4
