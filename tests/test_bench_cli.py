"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       cwd=ROOT)
    assert r.returncode != 0
    assert "one-GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, cwd=ROOT,
                       env=env)
    assert r.returncode != 0 and "one-GPU" in r.stderr


def test_the_paper_grid_table_is_complete():
    sys.path.insert(0, ROOT)
    import bench
    keys = set(bench.PAPER_TABLE2)
    assert keys == {(n, v) for n in (1024, 4096, 8192, 16384, 32768) for v in (32768, 65536, 131072, 262144)}
    for canon_ms, prop_ms, canon_mb, prop_mb in bench.PAPER_TABLE2.values():
        assert prop_ms <= canon_ms and prop_mb < canon_mb        # the paper's kernel wins every cell of its Table 2
