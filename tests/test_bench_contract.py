"""Host-side checks of bench.py's bookkeeping: the HBM-traffic figures it reports are copies of the rocprofv3
summaries under profiles/ and must not drift from them; more than one GPU is refused with a message."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


@pytest.mark.parametrize("cid", sorted(bench.MEASURED_TRAFFIC_BYTES))
def test_reported_traffic_is_the_profiles_figure(cid):
    value, path = bench.MEASURED_TRAFFIC_BYTES[cid]
    text = open(os.path.join(ROOT, path)).read()
    # the dominant (tile) kernel's line: "`<kernel>`: fetch + write = 1.2034e+09 B per launch (...)"
    lines = re.findall(r"^`([^`]*)`: fetch \+ write = ([0-9.e+]+) B per launch", text, flags=re.M)
    assert lines, path
    tile = [float(v) for k, v in lines if "mfma_kernel" in k]
    assert len(tile) == 1, (path, lines)
    assert abs(value - tile[0]) <= 1e-3 * tile[0], (cid, value, tile[0])
    # the summary is of the workload the constant is used for, and says how it was made
    assert f"bench.py --config {cid} " in text and "rocprofv3 --pmc FETCH_SIZE" in text


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "one GPU" in res.stderr
