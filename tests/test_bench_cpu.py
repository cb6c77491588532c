"""Host-side checks of bench.py that need no GPU: the traffic figure of the roofline object is read from the
rocprofv3 counter summary that measured it, so the summary must be there and carry the line the parser wants;
a multi-GPU request is refused with a message."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_traffic_is_read_from_the_committed_counter_summary():
    sys.path.insert(0, ROOT)
    import bench
    text = open(bench.TRAFFIC_PROFILE).read()
    assert "rocprofv3 --pmc FETCH_SIZE" in text and "rocprofv3 --pmc WRITE_SIZE" in text      # the commands that made it
    v = bench.traffic_from_profile()
    assert isinstance(v, int)
    # between the algorithmic bytes of the gate|up launch at 8192 rows (0.47 GB) and ten times that
    assert 0.4e9 < v < 5e9
    m = re.search(r"(\d+(?:\.\d+)?) MB read \+ (\d+(?:\.\d+)?) MB written per launch", text)
    assert m and abs((float(m.group(1)) + float(m.group(2))) * 1e6 - v) < 0.01 * v        # the line agrees with the table above it


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
