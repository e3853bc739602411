"""CPU: the host logic of bench.py - the byte counts the fractions are made of, the
statistics, the one-GPU rule and the parsing of the driver's clock / power files."""
import os
import subprocess
import sys
import types

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402
from paper_2511_05589_amd import workloads as W  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0
    assert "--gpus 2 is not supported" in res.stderr and res.stdout.strip() == ""


def test_algorithmic_bytes_are_the_per_unit_figures_times_the_units():
    # 2 * Hkv * D * sizeof per context token (2048 B at the 7B shape), 4 B per block-table entry
    # used, q in and out; W once + hidden + 12 B per row; 17 B per token of the ratio batch
    cfg = W.DECODE_CONFIGS[2]
    ctx = np.array([1, 16, 17, 4000], dtype=np.int32)
    small = types.SimpleNamespace(**{k: getattr(cfg, k) for k in ("Hq", "Hkv", "D", "H", "V", "page_size", "elem_bytes")},
                                  C=4)
    ab = bench.algorithmic_bytes(small, {"ctx_len": ctx}, {"N": 1000})
    assert 2 * cfg.Hkv * cfg.D * cfg.elem_bytes == 2048
    assert ab["kv"] == 2048 * int(ctx.sum())
    assert ab["attn"] == ab["kv"] + 4 * (1 + 1 + 2 + 250) + 2 * 4 * 28 * 128 * 2
    assert ab["lm"] == 151936 * 3584 * 2 + 4 * 3584 * 2 + 12 * 4
    assert ab["is"] == 17000
    assert bench.algorithmic_bytes(small, {"ctx_len": ctx}, None)["is"] == 0


def test_dist_reports_median_and_percentiles():
    d = bench.dist([5.0, 1.0, 2.0, 3.0, 4.0, 6.0, 7.0, 8.0, 9.0, 10.0, 11.0])
    assert d["median"] == 6.0 and d["p10"] == 2.0 and d["p90"] == 10.0 and d["mean"] == 6.0 and d["n"] == 11


def test_clock_and_power_files_are_parsed(tmp_path):
    sclk = tmp_path / "pp_dpm_sclk"
    sclk.write_text("0: 132Mhz\n1: 1687Mhz *\n2: 2400Mhz\n")
    power = tmp_path / "power1_input"
    power.write_text("1399000000\n")
    (tmp_path / "power1_cap").write_text("1400000000\n")
    cs = bench.ClockSampler()
    cs.path, cs.power_path = str(sclk), str(power)
    assert cs._read() == 1687.0
    assert cs._read_power() == 1399.0
    assert cs.power_cap_w() == 1400.0
    cs.path = str(tmp_path / "missing")
    assert cs._read() is None
