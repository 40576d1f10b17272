"""Host-side checks of bench.py's command-line contract (nothing here touches a GPU)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_world_size_above_one_is_refused_too():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0", LOCAL_RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, timeout=120,
                       env=env)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_roofline_traffic_comes_from_the_counter_summary():
    """bench.py holds no traffic figure of its own: it reads the line stored beside the rocprofv3 counter summary."""
    sys.path.insert(0, ROOT)
    import bench
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert not __import__("re").search(r"\b5\d\d\.\de6\b", src)
    v = bench.stored_traffic("c2.attn_proj")
    text = open(os.path.join(ROOT, "profiles", "c2_attn_proj_counters.md")).read()
    assert v is not None and f"traffic_bytes_per_launch[c2.attn_proj] = {v / 1e6:.1f}e6" in text
    assert 2.2e8 < v < 2e9      # above the algorithmic 220.2 MB, below ten times it
    assert bench.stored_traffic("no.such.workload") is None


def test_gpu_test_of_the_entry_point_that_allocates_nothing_is_collected_last():
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests"), "--collect-only", "-q", "-m", "gpu"],
                       capture_output=True, text=True, timeout=300, cwd=ROOT)
    ids = [l for l in r.stdout.splitlines() if "::" in l]
    assert ids and ids[-1].startswith("tests/test_zz_no_alloc.py::"), ids[-3:]
