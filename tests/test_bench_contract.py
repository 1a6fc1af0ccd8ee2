"""bench.py's contract that can be checked without a GPU: more than one GPU is refused with a message, and the
profiled counters it may print were taken on the kernel sources now in the tree."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_profiled_counters_belong_to_the_sources_in_the_tree():
    sys.path.insert(0, ROOT)
    import bench
    now = bench.csrc_sha16()
    for key, prof in bench.PROFILED.items():
        assert prof["csrc_sha16"] == now, (key, "re-take %s or its figures print as null" % prof["source"])
        text = open(os.path.join(ROOT, prof["source"])).read()
        assert now in text, prof["source"]
