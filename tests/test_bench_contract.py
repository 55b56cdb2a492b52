"""Host-side checks of bench.py's contract (no GPU): the refusal of more than one GPU, and that the traffic
figures it reports belong to the kernel sources in the tree."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode == 2
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_traffic_figures_were_read_on_the_kernel_sources_in_the_tree():
    # roofline.traffic is reported only while this holds; after a change to one of the files the counters are read
    # again (bench.py --probe-traffic under rocprofv3 --pmc) and the figures and the digest are updated together
    import bench
    assert bench.kernel_sources_digest() == bench.MEASURED_TRAFFIC_7B["sources"]
    for name in bench.TRAFFIC_SOURCES:
        assert os.path.exists(os.path.join(ROOT, "paper_2403_03507_amd", "csrc", name)), name
    b = bench.MEASURED_TRAFFIC_7B["bytes"]
    # algorithmic bytes of the weight-update launch of one 7B layer set (W read and written in bf16, P and N read once)
    shapes = [(4096, 4096)] * 4 + [(4096, 11008)] * 2 + [(11008, 4096)]
    algorithmic = sum(2 * 2 * m * n + 2 * 1024 * (m + n) for m, n in shapes)
    assert algorithmic <= b["back"] <= 2.0 * algorithmic
