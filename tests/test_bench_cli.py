"""Host-side checks of bench.py's contract that need no GPU: more than one GPU is refused with a message,
and the accounting constants agree with the byte counts of the workloads they describe."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True, timeout=120)
    assert res.returncode == 2
    assert res.stdout.strip() == ""                       # no JSON line is printed
    assert "one GPU" in res.stderr and "--gpus" in res.stderr


def test_a_multi_rank_launch_is_refused_too():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0", LOCAL_RANK="0")
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                         text=True, env=env, timeout=120)
    assert res.returncode == 2 and res.stdout.strip() == ""


def test_accounting_constants():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.HBM_PEAK_GBS == 8000.0
    assert bench.Q_BYTES_PER_SEQ == 64 * 256 * 2 and bench.OUT_BYTES_PER_SEQ == 64 * 256 * 4
    # algorithmic bytes of the default workload: 64 x 4096 tokens x 1024 B + 64 x (Q + out)
    assert 64 * 4096 * 1024 + 64 * (bench.Q_BYTES_PER_SEQ + bench.OUT_BYTES_PER_SEQ) == 274726912
    # profiled traffic may exceed the algorithmic bytes by partial results and query re-reads, not by a re-read of
    # the cache; every figure names the file under profiles/ it was taken from, and that file exists
    assert 1.0 <= bench.PROFILED_TRAFFIC["cfg2"][0] / 274726912 <= 1.15
    for _, source in bench.PROFILED_TRAFFIC.values():
        assert os.path.exists(os.path.join(ROOT, source))
    assert bench.EVENT_SAMPLES >= 50
