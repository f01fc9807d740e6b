"""bench.py's contract that can be checked without a GPU: one GPU only, and HBM-traffic figures that are taken from
the committed profile summaries only while those summaries belong to the library as it is built now."""
import os
import subprocess
import sys

import paper_2601_21444_amd as apbv
from paper_2601_21444_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_figures_belong_to_the_library_version_that_is_built():
    v = apbv.apbv_version()
    att, src = bench.measured_traffic(f"profiles/host_attention_{wl.HEADLINE}_pmc.txt", v)
    assert att is not None and src.endswith("_pmc.txt"), "regenerate profiles/ after changing the library version"
    assert 150e6 < att < 2e9                      # at least the compulsory bytes of the headline attention launch
    comp, _ = bench.measured_traffic(f"profiles/compress_{wl.HEADLINE}_batch96_pmc.txt", v)
    assert comp is not None and comp >= 96 * wl.CONFIGS[wl.HEADLINE].compress_bytes
    # another version, workload or batch: nothing is reported
    assert bench.measured_traffic(f"profiles/host_attention_{wl.HEADLINE}_pmc.txt", v + 1) == (None, None)
    assert bench.measured_traffic("profiles/host_attention_3b-8k_pmc.txt", v) == (None, None)
    assert bench.measured_traffic(f"profiles/compress_{wl.HEADLINE}_batch7_pmc.txt", v) == (None, None)
