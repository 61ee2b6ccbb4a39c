"""Host-side checks of bench.py that need no GPU: the one-GPU rule and the parser of the recorded traffic figures."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_module():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""  # no JSON line for a run that did not happen


def test_recorded_traffic_comes_from_the_profile_summary():
    bench = _bench_module()
    rec = bench.recorded_traffic()
    assert set(rec) >= {"score_mode0", "score_mode1", "select_scaled"}
    # a scoring pass moves the 2 GiB key cache once (plus the partial score vectors in the second pass)
    k_bytes = 8 * 1048576 * 128 * 2
    assert k_bytes <= rec["score_mode0"] < 1.05 * k_bytes
    assert k_bytes <= rec["score_mode1"] < 1.08 * k_bytes
    # the scaled selection reads its 2^27 scores once
    assert 4 * 2 ** 27 <= rec["select_scaled"] < 1.1 * 4 * 2 ** 27
    with open(bench.TRAFFIC_PROFILE) as f:
        assert sum(line.startswith("traffic_bytes_per_launch:") for line in f) == 1
