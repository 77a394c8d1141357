"""Host-side behaviour of the benchmark's command line (no GPU needed)."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          cwd=ROOT, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    """This build is single-GPU: --gpus N with N > 1 exits at once, says so, and prints no result line."""
    r = _bench("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode != 0
    assert "single-GPU" in r.stderr and "--gpus 2" in r.stderr
    assert r.stdout.strip() == ""


def test_unknown_layout_or_weight_type_is_refused_by_the_parser():
    for bad in (("--layout", "blocked"), ("--weights", "int4")):
        r = _bench(*bad)
        assert r.returncode == 2 and "invalid choice" in r.stderr and r.stdout.strip() == ""


def test_traffic_figure_comes_from_the_committed_counter_summaries():
    """roofline.traffic is read from profiles/: the files must be there, carry the line bench.py parses, and agree
    with the algorithmic bytes they quote to within a few percent (no wasted re-reads)."""
    for name in ("gateup_kernel_mixtral_hbm_traffic.txt", "gateup_kernel_mixtral_fp8_hbm_traffic.txt",
                 "gateup_kernel_olmoe_hbm_traffic.txt", "gateup_kernel_deepseek_hbm_traffic.txt"):
        text = open(os.path.join(ROOT, "profiles", name)).read()
        traffic = [int(l.split()[-1]) for l in text.splitlines() if l.startswith("traffic_bytes_per_launch gateup_kernel")]
        alg = [int(l.split("=")[-1]) for l in text.splitlines() if l.startswith("algorithmic bytes per launch")]
        assert len(traffic) == 1 and len(alg) == 1
        assert 0.99 <= traffic[0] / alg[0] <= 1.03
        assert "rocprofv3 --pmc FETCH_SIZE" in text and "rocprofv3 --pmc WRITE_SIZE" in text
