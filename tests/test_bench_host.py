"""Host-side checks of the benchmark's bookkeeping (no GPU): the algorithmic bytes it
prices the kernels with, and its refusal of more than one GPU."""
import subprocess
import sys
import os

import pytest

import bench
from workloads import PRESETS, budget_to_groups

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("name,mb", [("c2", 30.94), ("c3", 246.6), ("c4", 810.4), ("c5", 192.9)])
def test_algorithmic_bytes_per_layer_match_the_workload_table(name, mb):
    # K_lr read + selected K and V read + q read twice + out written + A read + group scores
    # written and read + idx written and read
    ab = bench.algorithmic_bytes(PRESETS[name])
    assert ab["step"] == ab["predict"] + ab["topk"] + ab["attn"]
    assert abs(ab["step"] / 1e6 - mb) / mb < 2e-3


def test_algorithmic_bytes_by_hand_for_c2():
    c = PRESETS["c2"]
    ab = bench.algorithmic_bytes(c)
    q = 32 * 128 * 2
    assert ab["predict"] == 8 * 32768 * 32 * 2 + q + 8 * 128 * 32 * 4 + 8 * 8192 * 4
    assert ab["topk"] == 8 * 8192 * 4 + 8 * 820 * 4
    assert ab["attn"] == 8 * 820 * 4 + 2 * 8 * 820 * 4 * 128 * 2 + 2 * q
    # joint-head design: one metadata row and one selection per sequence; 8-bit metadata halves the stream
    j = bench.algorithmic_bytes(PRESETS["c2j"])
    assert j["predict"] == 32768 * 32 * 2 + q + 8 * 128 * 32 * 4 + 8192 * 4
    assert j["attn"] == 820 * 4 + 2 * 8 * 820 * 4 * 128 * 2 + 2 * q
    f = bench.algorithmic_bytes(c, meta_bytes=1)
    assert ab["predict"] - f["predict"] == 8 * 32768 * 32


def test_budget_rounding_of_the_workload_table():
    assert budget_to_groups(0.10, 8192) == 820
    assert [budget_to_groups(x, 4096) for x in (0.02, 0.05, 0.10, 0.25, 1.0)] == [82, 205, 410, 1024, 4096]


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
