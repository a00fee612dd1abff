"""Host-side checks of bench.py that need no GPU: the one-GPU rule and the FLOP count the throughput is quoted on."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_executed_flops_counts_valid_tokens_only():
    """4 d per (row, attended valid key): rows of each query block x (valid persistent tokens + valid tokens of the
    selected blocks), checked against a count written out by hand for a tiny case."""
    torch = pytest.importorskip("torch")
    sys.path.insert(0, ROOT)
    import bench
    d = 64
    # one head, two query blocks of 64 and 8 rows; slots of 64, 17 and 0 tokens; local blocks of 64, 64, 8 tokens
    p_len = torch.tensor([[64, 17, 0]], dtype=torch.int32)
    l_len = torch.tensor([64, 64, 8], dtype=torch.int32)
    rows = torch.tensor([64, 8], dtype=torch.int32)
    sel = torch.tensor([[[0, 2], [1, -1]]], dtype=torch.int32)        # block 0 selects 0 and 2, block 1 selects 1 only
    want = 4 * d * (64 * (81 + 64 + 8) + 8 * (81 + 64))
    assert float(bench.executed_flops(sel, p_len, l_len, rows, d)) == want


def test_traffic_figure_comes_from_the_committed_profile():
    """roofline.traffic is read from the summary of the counter runs under profiles/ (FETCH_SIZE and WRITE_SIZE in KiB,
    each with its copy-calibration factor), so it cannot drift from what is committed; a workload without a summary
    reports none."""
    sys.path.insert(0, ROOT)
    import bench
    import re
    text = open(os.path.join(ROOT, "profiles", "attention_cfg5_hbm_counters.txt")).read()
    m = re.search(r"->\s*([\d,]+) KiB \* ([\d.]+) \+ ([\d,]+) KiB \* ([\d.]+) = ([\d,]+) KiB", text)
    assert m, "the summary states the figure in the form the benchmark reads"
    f, a, w, b, total = (float(x.replace(",", "")) for x in m.groups())
    assert abs(f * a + w * b - total) <= 1.0
    got = bench.hbm_traffic_bytes("cfg5")
    assert got == int((f * a + w * b) * 1024) and 3e8 < got < 6e8
    assert bench.hbm_traffic_bytes("no_such_workload") is None
