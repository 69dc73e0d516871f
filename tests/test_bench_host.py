"""Host logic of bench.py that needs no GPU: algorithmic bytes per node-parameter of every workload,
the counter summaries it reads from profiles/, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import bench
from paper_1811_10792_amd import synthetic as syn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_bytes_per_update():
    want = {"c1_n4_d1k": 16.0,                                   # x, g read; x, z written
            "c2_n8_d1m": 24.0, "c3_n16_resnet50": 24.0, "c4_n32_resnet50": 24.0,   # + u read and written
            "c5_n16_transformer_2peer_overlap": 32.0,            # + messages read and written
            "x1_n16_transformer_2peer_tau2": 28.0,               # messages at every second iteration
            "x2_n32_resnet50_complete": 24.0,
            "x3_n16_transformer_2peer_overlap_adam": 40.0,       # + second moment read and written
            "x4_n32_resnet50_2peer": 24.0, "x5_n16_resnet50_2peer": 24.0}
    assert set(want) == set(syn.WORKLOADS)
    for name, b in want.items():
        assert bench.algorithmic_bytes_per_update(syn.WORKLOADS[name]) == b, name


def test_committed_counter_summaries_match_the_algorithmic_traffic():
    for name in ("c3_n16_resnet50", "c4_n32_resnet50", "c5_n16_transformer_2peer_overlap",
                 "x2_n32_resnet50_complete"):
        wl = syn.WORKLOADS[name]
        measured = bench.read_traffic(name)
        algorithmic = bench.algorithmic_bytes_per_update(wl) * wl.n * wl.d
        assert measured is not None and abs(measured / algorithmic - 1.0) < 0.002, name
    assert bench.read_traffic("no_such_workload") is None


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_padded_row_stride():
    assert syn.padded_ld(25_557_032) == 25_557_248 and syn.padded_ld(1024) == 1024
    assert syn.padded_ld(213_000_000) % 256 == 0
