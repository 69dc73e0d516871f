"""Host logic of bench.py that needs no GPU: algorithmic bytes per node-parameter of every workload,
the counter summaries it reads from profiles/, and the refusal of more than one GPU."""
import glob
import os
import re
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
            "x4_n32_resnet50_2peer": 24.0, "x5_n16_resnet50_2peer": 24.0, "x6_n24_resnet50_stats": 24.0,
            "x7_n32_resnet50_overlap_stats": 32.0,            # + message read and written
            "h1_n32_resnet50_bf16_gz": 20.0, "h2_n32_resnet50_bf16_guz": 16.0}   # storage experiment
    assert set(want) == set(syn.WORKLOADS)
    for name, b in want.items():
        assert bench.algorithmic_bytes_per_update(syn.WORKLOADS[name]) == b, name


def _fields(path):
    out = {}
    for line in open(path):
        m = re.match(r"^(\w+):\s*(\S+)", line)
        if m:
            out[m.group(1)] = m.group(2)
    return out


def test_committed_counter_summaries_match_the_algorithmic_traffic():
    """Every committed counter summary names its kernel and shape, its traffic is the algorithmic
    one to within 0.2 %, and bench.read_traffic hands it out only for that kernel and shape."""
    seen = 0
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "step_kernel_*_pmc.txt"))):
        f = _fields(path)
        name = f["workload"]
        wl = syn.WORKLOADS[name]
        ld = syn.padded_ld(wl.d)
        assert (int(f["n"]), int(f["d"]), int(f["ld"])) == (wl.n, wl.d, ld), path
        measured, source = bench.read_traffic(name, f["kernel"], wl.n, wl.d, ld)
        algorithmic = bench.algorithmic_bytes_per_update(wl) * wl.n * wl.d
        assert measured is not None and abs(measured / algorithmic - 1.0) < 0.002, name
        assert source == os.path.join("profiles", os.path.basename(path))
        assert bench.read_traffic(name, "k_other", wl.n, wl.d, ld) == (None, None)      # another kernel ran
        assert bench.read_traffic(name, f["kernel"], wl.n, wl.d, ld + 256) == (None, None)
        seen += 1
    assert seen >= 1 and os.path.exists(os.path.join(ROOT, "profiles", "step_kernel_c4_n32_resnet50_pmc.txt"))
    assert bench.read_traffic("no_such_workload", "k", 1, 1, 1) == (None, None)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_padded_row_stride():
    assert syn.padded_ld(25_557_032) == 25_557_248 and syn.padded_ld(1024) == 1024
    assert syn.padded_ld(213_000_000) % 256 == 0
