"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT,
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = run_bench("--gpus", "2")
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_unknown_workload_is_an_argument_error():
    p = run_bench("--config", "C9")
    assert p.returncode != 0 and "C9" in p.stderr


def test_algorithmic_bytes_follow_the_stated_formulas():
    """2.5 bytes per channel plus 16 per token for rotate+quant (bf16 in, half a byte of codes and one record out),
    plus three quarters of a byte per channel for the fp6 copy; group records scale with K / group."""
    sys.path.insert(0, ROOT)
    import bench
    M, K, N = 4096, 8192, 28672
    assert bench.algorithmic_bytes_rotate_quant(M, K, False, 0) == M * (2 * K + K // 2 + 16)
    assert bench.algorithmic_bytes_rotate_quant(M, K, True, 0) == M * (2 * K + K // 2 + 16) + M * K * 3 // 4
    assert bench.algorithmic_bytes_rotate_quant(M, K, False, 128) == M * (2 * K + K // 2 + 16 * (K // 128))
    # decode-sized product: the weights once, their three vectors, the codes, records and the output
    assert bench.algorithmic_bytes_gemm(16, 4096, 4096, False) == 4096 * 2048 + 4096 * 12 + 16 * (2048 + 16) + 2 * 16 * 4096


import json

import pytest


@pytest.mark.gpu
@pytest.mark.parametrize("args", [["--config", "C1"], ["--config", "C3_M4"], ["--config", "C1", "--group-size", "128"],
                                  ["--config", "C1", "--group-size", "128", "--matrix-path", "int8"],
                                  ["--config", "C1", "--only", "rotate_quant", "--rot-size", "128", "--group-size", "128"],
                                  ["--config", "C3_M1", "--graph"]])
def test_bench_prints_one_json_line_with_the_contract_fields(args):
    p = run_bench("--steps", "3", "--warmup", "1", "--no-cpu-baseline", *args)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["data"] == "synthetic" and "workload" in d["config"]
    r = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in r, key
    assert r["bound"] in ("hbm", "mfma") and 0.0 < r["frac"] < 1.0 and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
